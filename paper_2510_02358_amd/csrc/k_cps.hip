// Causal-consistency path search: left-to-right beam search over the pruned token lattice.
//
// One wavefront per sequence.  The search is a chain of K dependent steps, each tiny
// (B live hypotheses x C candidates <= 16 x 17 expansions), so it is latency-bound: the wavefront
// keeps the beam in registers (lane b holds hypothesis b), scores one expansion per lane slot,
// selects the B best with wavefront arg-max reductions over a 64-bit (score, order) key, and
// records (parent, token) back-pointers in LDS for the final back-track.
//
// Arithmetic is float32 with explicitly unfused multiply/add in the order
//   term = (lambda * l_dlm) + ((1 - lambda) * l_ng);  score = score + term
// so that the kept hypotheses are bit-for-bit those of a plain float32 evaluation.
#include <limits.h>
#include <math.h>

#include "ds_common.h"

namespace ds {
namespace {

constexpr int kMaxCand = DS_MAX_TOPM + 1;                          // + retained EOS
constexpr int kMaxExp = DS_MAX_BEAM * kMaxCand;                    // 272 expansions
constexpr int kSlots = (kMaxExp + kWave - 1) / kWave;              // 5 per lane

__device__ __forceinline__ uint32_t ngram_slot(uint32_t u, uint32_t v, uint32_t w, uint32_t mask) {
  uint32_t x = u * 0x9E3779B1u;
  x ^= x >> 15;
  x = (x + v) * 0x85EBCA77u;
  x ^= x >> 13;
  x = (x + w) * 0xC2B2AE3Du;
  x ^= x >> 16;
  return x & mask;
}

// Monotone map float -> uint32 (larger float, larger integer).
__device__ __forceinline__ uint32_t ordered_bits(float f) {
  uint32_t u = __float_as_uint(f);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

__device__ __forceinline__ unsigned long long wave_max_u64(unsigned long long k) {
#pragma unroll
  for (int off = kWave / 2; off > 0; off >>= 1) {
    unsigned long long o = __shfl_xor(k, off);
    k = o > k ? o : k;
  }
  return k;
}

__global__ __launch_bounds__(kWave) void cps_kernel(const int32_t* __restrict__ cand_id,
                                                    const float* __restrict__ cand_logp,
                                                    const int32_t* __restrict__ cand_cnt,
                                                    const float* __restrict__ eos_logp, int K, int m_max, int B,
                                                    float lambda, const float* __restrict__ table,
                                                    uint32_t table_mask, const int32_t* __restrict__ ctx,
                                                    int32_t eos_id, int32_t* __restrict__ path,
                                                    int32_t* __restrict__ path_len,
                                                    float* __restrict__ path_score) {
  extern __shared__ int32_t smem[];
  int32_t* bp_tok = smem;                                                  // [K][B]
  uint8_t* bp_par = reinterpret_cast<uint8_t*>(smem + (size_t)K * B);      // [K][B]
  const int seq = blockIdx.x, lane = threadIdx.x;
  const size_t row0 = (size_t)seq * K;
  const float one_minus = __fsub_rn(1.0f, lambda);

  // beam: lane b < n_live holds hypothesis b
  int n_live = 1;
  float h_score = 0.f;
  int h_u = ctx[seq * 2 + 0], h_v = ctx[seq * 2 + 1];

  int out_len = K, out_slot = 0;
  float out_score = 0.f;
  bool finished = false;

  for (int i = 0; i < K && !finished; ++i) {
    // candidates of this position: lane c < n_cand
    int cnt = cand_cnt[row0 + i];
    cnt = cnt < 1 ? 1 : (cnt > m_max ? m_max : cnt);
    int c_tok = 0;
    float c_lp = 0.f;
    if (lane < cnt) {
      c_tok = cand_id[(row0 + i) * m_max + lane];
      c_lp = cand_logp[(row0 + i) * m_max + lane];
    }
    int n_cand = cnt;
    if (eos_id >= 0) {
      bool has = __ballot(lane < cnt && c_tok == eos_id) != 0ull;
      if (!has) {
        if (lane == cnt) {
          c_tok = eos_id;
          c_lp = eos_logp[row0 + i];
        }
        n_cand = cnt + 1;
      }
    }
    const int n_exp = n_live * n_cand;

    // score the expansions: slot j of lane l is expansion e = l + 64 j = parent * n_cand + cand
    float e_score[kSlots];
    unsigned taken = 0;
#pragma unroll
    for (int j = 0; j < kSlots; ++j) {
      const int e = lane + j * kWave;
      const int b = e / n_cand, c = e - b * n_cand;
      const int src_b = b < kWave ? b : 0, src_c = c;
      float ps = __shfl(h_score, src_b);
      int pu = __shfl(h_u, src_b), pv = __shfl(h_v, src_b);
      int w = __shfl(c_tok, src_c);
      float ld = __shfl(c_lp, src_c);
      float lng = 0.f;
      if (e < n_exp && table) lng = table[ngram_slot((uint32_t)pu, (uint32_t)pv, (uint32_t)w, table_mask)];
      float term = __fadd_rn(__fmul_rn(lambda, ld), __fmul_rn(one_minus, lng));
      e_score[j] = __fadd_rn(ps, term);
      if (e >= n_exp) taken |= 1u << j;
    }

    // keep the best B by (score descending, expansion index ascending)
    const int n_keep = n_exp < B ? n_exp : B;
    float k_score = 0.f;   // lane r < n_keep: r-th kept expansion
    int k_exp = 0;
    for (int r = 0; r < n_keep; ++r) {
      unsigned long long best = 0ull;
#pragma unroll
      for (int j = 0; j < kSlots; ++j) {
        if (!(taken & (1u << j))) {
          unsigned long long key = ((unsigned long long)ordered_bits(e_score[j]) << 32) |
                                   (unsigned long long)(0xFFFFFFFFu - (uint32_t)(lane + j * kWave));
          best = key > best ? key : best;
        }
      }
      best = wave_max_u64(best);
      const int e = (int)(0xFFFFFFFFu - (uint32_t)(best & 0xFFFFFFFFull));
      const int owner = e & (kWave - 1), slot = e / kWave;
      float sc = 0.f;
#pragma unroll
      for (int j = 0; j < kSlots; ++j)
        if (j == slot) sc = e_score[j];
      sc = __shfl(sc, owner);
      if (lane == owner) taken |= 1u << slot;
      if (lane == r) {
        k_score = sc;
        k_exp = e;
      }
    }

    // kept lane r: parent, token
    const int k_par = k_exp / n_cand, k_c = k_exp - k_par * n_cand;
    const int k_tok = __shfl(c_tok, k_c);
    const int k_v = __shfl(h_v, k_par < kWave ? k_par : 0);
    const bool k_valid = lane < n_keep;
    const bool k_eos = k_valid && eos_id >= 0 && k_tok == eos_id;

    // the best kept hypothesis ends in EOS: it is the result
    const bool best_eos = __shfl((int)k_eos, 0) != 0;
    // survivors: kept hypotheses that do not end in EOS, order preserved
    unsigned long long live_mask = __ballot(k_valid && !k_eos);
    const int new_slot = __popcll(live_mask & ((1ull << lane) - 1ull));
    if (best_eos) {
      if (lane == 0) {
        bp_tok[i * B + 0] = k_tok;
        bp_par[i * B + 0] = (uint8_t)k_par;
      }
      out_len = i + 1;
      out_slot = 0;
      out_score = __shfl(k_score, 0);
      finished = true;
    } else {
      if (k_valid && !k_eos) {
        bp_tok[i * B + new_slot] = k_tok;
        bp_par[i * B + new_slot] = (uint8_t)k_par;
      }
      // compact the survivors into lanes 0 .. n_live-1
      n_live = __popcll(live_mask);
      // lane t takes the t-th set bit of live_mask
      int src = 0;
      {
        unsigned long long m = live_mask;
        for (int t = 0; t < lane && m; ++t) m &= m - 1;
        src = m ? (__ffsll((long long)m) - 1) : 0;
      }
      float ns = __shfl(k_score, src);
      int nu = __shfl(k_v, src), nv = __shfl(k_tok, src);
      if (lane < n_live) {
        h_score = ns;
        h_u = nu;
        h_v = nv;
      }
      if (i == K - 1) {
        out_len = K;
        out_slot = 0;
        out_score = __shfl(h_score, 0);
      }
    }
    __syncthreads();  // back-pointers of this depth visible (single wavefront: orders LDS traffic)
  }

  // back-track
  if (lane == 0) {
    int slot = out_slot;
    for (int i = out_len - 1; i >= 0; --i) {
      path[row0 + i] = bp_tok[i * B + slot];
      slot = bp_par[i * B + slot];
    }
    path_len[seq] = out_len;
    path_score[seq] = out_score;
  }
  for (int i = out_len + lane; i < K; i += kWave) path[row0 + i] = -1;
}

}  // namespace

int launch_cps(const int32_t* cand_id, const float* cand_logp, const int32_t* cand_cnt,
               const float* eos_logp, int batch, int K, int m_max, int B, float lambda,
               const float* table, int log2_size, const int32_t* ctx, int32_t eos_id, int32_t* path,
               int32_t* path_len, float* path_score, hipStream_t st) {
  size_t lds = (size_t)K * B * sizeof(int32_t) + align_up((size_t)K * B, 4);
  uint32_t mask = table ? ((1u << log2_size) - 1u) : 0u;
  hipLaunchKernelGGL(cps_kernel, dim3(batch), dim3(kWave), lds, st, cand_id, cand_logp, cand_cnt, eos_logp, K,
                     m_max, B, lambda, table, mask, ctx, eos_id, path, path_len, path_score);
  DS_LAUNCH_CHECK("cps_kernel");
  return DS_OK;
}

}  // namespace ds
