// Causal-consistency path search: left-to-right beam search over the pruned token lattice.
//
// One workgroup per sequence.  The search itself is a chain of K dependent steps, each tiny
// (B live hypotheses x C candidates <= 16 x 17 expansions), so it is latency-bound and runs in ONE
// wavefront: the beam lives in registers (lane b holds hypothesis b), every expansion gets a lane slot,
// the B best are picked by wavefront arg-max reductions, and (parent, token) back-pointers go to LDS
// for the final back-track.
//
// What dominates a step is the dependent gather of the causal-proxy score T[hash(u, v, w)] from a 16 MB
// table.  The lattice fixes in advance which tokens can occupy each position, so when K * C^3 scores fit
// in LDS the whole workgroup first gathers the proxy score of EVERY (u in C[i-2], v in C[i-1], w in C[i])
// combination in parallel; the sequential search then only touches LDS.  Larger lattices gather on
// demand inside the step.
//
// Arithmetic is float32 with explicitly unfused multiply/add in the order
//   term = (lambda * l_dlm) + ((1 - lambda) * l_ng);  score = score + term
// so that the kept hypotheses are bit-for-bit those of a plain float32 evaluation.
#include <limits.h>
#include <math.h>

#include "ds_common.h"
#include "ds_wave.h"

// The score arithmetic must stay unfused (see above).  It is written with plain operators under this pragma: the
// __fmul_rn / __fadd_rn helpers are ordinary * and + compiled in their own header, where contraction is allowed, so
// after inlining the compiler may still fuse them into a multiply-add (whether it does depends on scheduling).
#pragma clang fp contract(off)

namespace ds {
namespace {

constexpr int kMaxCand = DS_MAX_TOPM + 1;                          // + retained EOS
constexpr int kMaxExp = DS_MAX_BEAM * kMaxCand;                    // 272 expansions
constexpr int kMaxSlots = (kMaxExp + kWave - 1) / kWave;           // 5 lane slots cover every case
constexpr size_t kLdsBudget = 120 * 1024;                          // bytes this kernel may use

__device__ __forceinline__ uint32_t ngram_slot(uint32_t u, uint32_t v, uint32_t w, uint32_t mask) {
  uint32_t x = u * 0x9E3779B1u;
  x ^= x >> 15;
  x = (x + v) * 0x85EBCA77u;
  x ^= x >> 13;
  x = (x + w) * 0xC2B2AE3Du;
  x ^= x >> 16;
  return x & mask;
}

struct Lds {
  int4* meta;         // [K] {n_cand, eos_rank (-1: none), ceil(65536 / n_cand), 0}
  int4* beam;         // [2][B] {score bits, u, v, rank_u | rank_v << 8}
  int32_t* cand_tok;  // [K][CM]
  float* cand_lp;     // [K][CM]
  int32_t* bp_tok;    // [K][B]
  uint8_t* bp_par;    // [K][B]
  float* ng;          // [K][CM][CM][CM] or nullptr
};

__host__ __device__ inline size_t lds_fixed_bytes(int K, int CM, int B) {
  return (size_t)K * 16 + (size_t)2 * B * 16 + (size_t)K * CM * 8 + (size_t)K * B * 4 +
         ((size_t)K * B + 15) / 16 * 16;
}

// Candidate list of one lattice position (first cand_cnt entries, EOS appended if absent): token ids only.
__device__ __forceinline__ int position_tokens(const int32_t* __restrict__ cand_id, const int32_t* __restrict__ cand_cnt,
                                               size_t row, int m_max, int32_t eos_id, int32_t* tok) {
  int cnt = cand_cnt[row];
  cnt = cnt < 1 ? 1 : (cnt > m_max ? m_max : cnt);
  bool has_eos = false;
  for (int c = 0; c < cnt; ++c) {
    tok[c] = cand_id[row * m_max + c];
    has_eos |= (tok[c] == eos_id);
  }
  if (eos_id >= 0 && !has_eos) tok[cnt++] = eos_id;
  return cnt;
}

// Proxy scores of every (u in C[i-2], v in C[i-1], w in C[i]) for one position i of one sequence, spread
// over the chip (grid = positions x sequences) and written to g[seq][i][a][b][c]; the search kernel then
// copies its sequence's block into LDS with plain coalesced loads.
__global__ __launch_bounds__(256) void cps_gather_kernel(const int32_t* __restrict__ cand_id,
                                                         const int32_t* __restrict__ cand_cnt, int K, int m_max,
                                                         const float* __restrict__ table, uint32_t table_mask,
                                                         const int32_t* __restrict__ ctx, int32_t eos_id,
                                                         float* __restrict__ g) {
  __shared__ int32_t tok[3][kMaxCand];
  __shared__ int n[3];
  const int i = blockIdx.x, seq = blockIdx.y, CM = m_max + 1;
  if (threadIdx.x < 3) {
    const int t = threadIdx.x, pos = i - 2 + t;  // t = 0: position i-2, 1: i-1, 2: i
    if (pos >= 0) {
      n[t] = position_tokens(cand_id, cand_cnt, (size_t)seq * K + pos, m_max, eos_id, tok[t]);
    } else {  // before the block: the context token (pos -2 -> older, -1 -> newer)
      tok[t][0] = ctx[seq * 2 + (pos + 2)];
      n[t] = 1;
    }
  }
  __syncthreads();
  const int cube = CM * CM * CM;
  float* out = g + ((size_t)seq * K + i) * cube;
  for (int idx = threadIdx.x; idx < cube; idx += blockDim.x) {
    const int a = idx / (CM * CM), rem = idx - a * (CM * CM), b = rem / CM, c = rem - b * CM;
    if (a < n[0] && b < n[1] && c < n[2])
      out[idx] = table[ngram_slot((uint32_t)tok[0][a], (uint32_t)tok[1][b], (uint32_t)tok[2][c], table_mask)];
  }
}

// PRE: proxy scores pre-gathered into LDS.  kSlots: expansions per lane (B * (M_max + 1) <= 64 * kSlots).
template <bool PRE, int kSlots>
__global__ __launch_bounds__(1024) void cps_kernel(const int32_t* __restrict__ cand_id,
                                                   const float* __restrict__ cand_logp,
                                                   const int32_t* __restrict__ cand_cnt,
                                                   const float* __restrict__ eos_logp, int K, int m_max, int B,
                                                   float lambda, const float* __restrict__ table,
                                                   uint32_t table_mask, const int32_t* __restrict__ ctx,
                                                   int32_t eos_id, const float* __restrict__ g,
                                                   int32_t* __restrict__ path, int32_t* __restrict__ path_len,
                                                   float* __restrict__ path_score, int32_t* __restrict__ mirror) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  const int CM = m_max + 1;
  Lds L;
  {
    unsigned char* p = smem;
    L.meta = reinterpret_cast<int4*>(p);        p += (size_t)K * 16;
    L.beam = reinterpret_cast<int4*>(p);        p += (size_t)2 * B * 16;
    L.cand_tok = reinterpret_cast<int32_t*>(p); p += (size_t)K * CM * 4;
    L.cand_lp = reinterpret_cast<float*>(p);    p += (size_t)K * CM * 4;
    L.bp_tok = reinterpret_cast<int32_t*>(p);   p += (size_t)K * B * 4;
    L.bp_par = p;                               p += ((size_t)K * B + 15) / 16 * 16;
    L.ng = PRE ? reinterpret_cast<float*>(p) : nullptr;
  }
  const int seq = blockIdx.x, tid = threadIdx.x, lane = tid & (kWave - 1), n_thr = blockDim.x;
  const size_t row0 = (size_t)seq * K;
  const int ctx_u = ctx[seq * 2 + 0], ctx_v = ctx[seq * 2 + 1];

  // ---- phase A (whole workgroup): candidate lists of every position, EOS retained ------------------
  for (int i = tid; i < K; i += n_thr) {
    int cnt = cand_cnt[row0 + i];
    cnt = cnt < 1 ? 1 : (cnt > m_max ? m_max : cnt);
    int eos_rank = -1;
    for (int c = 0; c < cnt; ++c) {
      const int t = cand_id[(row0 + i) * m_max + c];
      L.cand_tok[i * CM + c] = t;
      L.cand_lp[i * CM + c] = cand_logp[(row0 + i) * m_max + c];
      if (eos_id >= 0 && t == eos_id && eos_rank < 0) eos_rank = c;
    }
    if (eos_id >= 0 && eos_rank < 0) {
      L.cand_tok[i * CM + cnt] = eos_id;
      L.cand_lp[i * CM + cnt] = eos_logp[row0 + i];
      eos_rank = cnt;
      ++cnt;
    }
    L.meta[i] = make_int4(cnt, eos_rank, (65536 + cnt - 1) / cnt, 0);
  }
  __syncthreads();

  if (PRE && g) {  // scores were gathered by cps_gather_kernel: plain copy into LDS
    const int total = K * CM * CM * CM;
    const float* src = g + (size_t)seq * total;
    if ((total & 3) == 0 && (((uintptr_t)src | (uintptr_t)L.ng) & 15) == 0) {  // 16 bytes per load, several in flight
      const float4* src4 = reinterpret_cast<const float4*>(src);
      float4* dst4 = reinterpret_cast<float4*>(L.ng);
#pragma unroll 4
      for (int idx = tid; idx < total / 4; idx += n_thr) dst4[idx] = src4[idx];
    } else {
      for (int idx = tid; idx < total; idx += n_thr) L.ng[idx] = src[idx];
    }
  } else if (PRE) {  // gather here: proxy score of every (u, v, w) the search can ask for
    const int pairs = K * CM * CM;
    for (int p = tid; p < pairs; p += n_thr) {
      const int i = p / (CM * CM), rem = p - i * (CM * CM);
      const int a = rem / CM, b = rem - a * CM;
      const int na = i >= 2 ? L.meta[i - 2].x : 1, nb = i >= 1 ? L.meta[i - 1].x : 1;
      if (a >= na || b >= nb) continue;
      const uint32_t u = (uint32_t)(i >= 2 ? L.cand_tok[(i - 2) * CM + a] : (i == 1 ? ctx_v : ctx_u));
      const uint32_t v = (uint32_t)(i >= 1 ? L.cand_tok[(i - 1) * CM + b] : ctx_v);
      const int nc = L.meta[i].x;
      float vals[kMaxCand];
#pragma unroll
      for (int c = 0; c < kMaxCand; ++c)
        vals[c] = c < nc ? table[ngram_slot(u, v, (uint32_t)L.cand_tok[i * CM + c], table_mask)] : 0.f;
#pragma unroll
      for (int c = 0; c < kMaxCand; ++c)
        if (c < nc) L.ng[(size_t)p * CM + c] = vals[c];
    }
  }
  if (tid == 0) L.beam[0] = make_int4((int)__float_as_uint(0.f), ctx_u, ctx_v, 0);
  __syncthreads();
  if (tid >= kWave) return;  // the search runs in the first wavefront

  // ---- phase B: the beam lives in LDS (beam[depth parity][slot]); lanes hold expansions --------------
  const float one_minus = 1.0f - lambda;
  int n_live = 1;
  int out_len = K;
  float out_score = 0.f;
  bool finished = false;

  int4 mt_next = L.meta[0];  // the next step's meta is read one step ahead, off the dependent chain
  for (int i = 0; i < K && !finished; ++i) {
    const int4 mt = mt_next;
    mt_next = L.meta[i + 1 < K ? i + 1 : i];
    const int n_cand = __builtin_amdgcn_readfirstlane(mt.x), eos_rank = __builtin_amdgcn_readfirstlane(mt.y);
    const uint32_t inv = (uint32_t)__builtin_amdgcn_readfirstlane(mt.z);
    const int n_exp = n_live * n_cand;
    const int4* cur = L.beam + (i & 1) * B;
    int4* nxt = L.beam + ((i + 1) & 1) * B;

    // score the expansions: slot j of lane l is expansion e = l + 64 j = parent * n_cand + cand
    uint32_t e_bits[kSlots];   // ordered score bits, 0 = no open expansion in this slot
    float e_score[kSlots];
    int e_v[kSlots], e_tok[kSlots], e_rank[kSlots];
#pragma unroll
    for (int j = 0; j < kSlots; ++j) {
      const int e = lane + j * kWave;
      e_bits[j] = 0u;
      e_score[j] = 0.f;
      e_v[j] = e_tok[j] = e_rank[j] = 0;
      if (j * kWave >= n_exp) continue;  // wavefront-uniform
      if (e < n_exp) {
        const int b = (int)(((uint32_t)e * inv) >> 16), c = e - b * n_cand;
        const int4 st = cur[b];
        const float ld = L.cand_lp[i * CM + c];
        const int tok = L.cand_tok[i * CM + c];
        const int ra = st.w & 0xFF, rb = (st.w >> 8) & 0xFF;
        float lng = 0.f;
        if (PRE) {
          lng = L.ng[(((size_t)i * CM + ra) * CM + rb) * CM + c];
        } else if (table) {
          lng = table[ngram_slot((uint32_t)st.y, (uint32_t)st.z, (uint32_t)tok, table_mask)];
        }
        const float dlm_part = lambda * ld, ng_part = one_minus * lng;  // two roundings, then two more below
        const float term = dlm_part + ng_part;
        e_score[j] = __uint_as_float((uint32_t)st.x) + term;
        e_bits[j] = ordered_bits(e_score[j]);
        e_v[j] = st.z;
        e_tok[j] = tok;
        e_rank[j] = rb | (c << 8);  // (rank of the previous token, rank of this token)
      }
    }

    // keep the best B by (score descending, expansion index ascending).  Each selection round only marks its
    // winner (the owning lane notes the beam slot it will fill, or that it ended in EOS and is dropped); the
    // survivors are written to the next beam in one go after the last round, so a round is a short branch-free
    // chain: wavefront maximum, first lane at the maximum, a few scalar operations.
    const int n_keep = n_exp < B ? n_exp : B;
    int e_par[kSlots], e_dst[kSlots];  // parent of this expansion; beam slot it won (-1: none)
#pragma unroll
    for (int j = 0; j < kSlots; ++j) {
      e_par[j] = (int)(((uint32_t)(lane + j * kWave) * inv) >> 16);
      e_dst[j] = -1;
    }
    int live = 0;
    for (int r = 0; r < n_keep; ++r) {
      uint32_t best_bits = 0;
      int best_slot = 0;
#pragma unroll
      for (int j = kSlots - 1; j >= 0; --j) {
        if (e_bits[j] != 0u && e_bits[j] >= best_bits) {
          best_bits = e_bits[j];
          best_slot = j;
        }
      }
      const uint32_t top = wave_max_u32(best_bits);
      int e;
      if (kSlots == 1) {
        e = __ffsll((long long)__ballot(best_bits == top)) - 1;
      } else {
        const uint32_t my_e = best_bits == top ? (uint32_t)(lane + best_slot * kWave) : 0xFFFFFFFFu;
        e = (int)(0xFFFFFFFFu - wave_max_u32(0xFFFFFFFFu - my_e));
      }
      e = __builtin_amdgcn_readfirstlane(e);
      const int owner = e & (kWave - 1), slot = e >> 6;
      const int par = (int)(((uint32_t)e * inv) >> 16), c = e - par * n_cand;
      const bool is_eos = (c == eos_rank);
      if (r == 0 && is_eos) {  // the best kept hypothesis ends in EOS: it is the result
        if (lane == owner) {
#pragma unroll
          for (int j = 0; j < kSlots; ++j)
            if (j == slot) {
              L.bp_tok[i * B] = e_tok[j];
              L.bp_par[i * B] = (uint8_t)par;
            }
        }
        out_len = i + 1;
        out_score = __uint_as_float(top & 0x80000000u ? (top & 0x7FFFFFFFu) : ~top);
        finished = true;
        break;
      }
#pragma unroll
      for (int j = 0; j < kSlots; ++j) {
        const bool mine = lane == owner && j == slot;
        e_bits[j] = mine ? 0u : e_bits[j];                     // taken
        e_dst[j] = (mine && !is_eos) ? live : e_dst[j];
      }
      live += is_eos ? 0 : 1;
    }
    if (finished) break;
#pragma unroll
    for (int j = 0; j < kSlots; ++j)
      if (e_dst[j] >= 0) {
        nxt[e_dst[j]] = make_int4((int)__float_as_uint(e_score[j]), e_v[j], e_tok[j], e_rank[j]);
        L.bp_tok[i * B + e_dst[j]] = e_tok[j];
        L.bp_par[i * B + e_dst[j]] = (uint8_t)e_par[j];
      }
    n_live = live;
  }
  // the search ran to the end: the result is the best live hypothesis of the last step
  if (!finished && n_live > 0) out_score = __uint_as_float((uint32_t)L.beam[(K & 1) * B].x);

  // back-track: lane 0 walks the parents (it reads what other lanes of this wavefront wrote: the LDS operations of a
  // wavefront complete in order) and leaves the path's token of depth i in slot 0 of that depth, which the walk no
  // longer needs; then all lanes store the path.
  // mirror (optional, device-visible host memory): per sequence the path, its length and the raw draft (the top
  // candidate of every position), so that a host loop needs no copy of its own to see them.
  int32_t* mine = mirror ? mirror + (size_t)seq * (2 * K + 1) : nullptr;
  if (lane == 0) {
    int slot = 0;
    for (int i = out_len - 1; i >= 0; --i) {
      const int32_t t = L.bp_tok[i * B + slot];
      slot = L.bp_par[i * B + slot];
      L.bp_tok[i * B] = t;
    }
    path_len[seq] = out_len;
    path_score[seq] = out_score;
    if (mine) mine[K] = out_len;
  }
  __builtin_amdgcn_wave_barrier();
  for (int i = lane; i < K; i += kWave) {
    const int32_t t = i < out_len ? L.bp_tok[i * B] : -1;
    path[row0 + i] = t;
    if (mine) {
      mine[i] = t;
      mine[K + 1 + i] = L.cand_tok[i * CM];
    }
  }
}

}  // namespace

size_t cps_ws_bytes(int batch, int K, int m_max) {
  const size_t CM = (size_t)m_max + 1;
  return align_up((size_t)batch * K * CM * CM * CM * sizeof(float), 256);
}

int launch_cps(const int32_t* cand_id, const float* cand_logp, const int32_t* cand_cnt,
               const float* eos_logp, int batch, int K, int m_max, int B, float lambda,
               const float* table, int log2_size, const int32_t* ctx, int32_t eos_id, int32_t* path,
               int32_t* path_len, float* path_score, int32_t* mirror, void* ws, size_t ws_bytes, hipStream_t st) {
  const int CM = m_max + 1;
  const size_t fixed = align_up(lds_fixed_bytes(K, CM, B), 16);
  const size_t pre = (size_t)K * CM * CM * CM * sizeof(float);
  const bool use_pre = table != nullptr && fixed + pre <= kLdsBudget;
  const uint32_t mask = table ? ((1u << log2_size) - 1u) : 0u;
  const int slots = ceil_div(B * CM, kWave);  // 1 .. kMaxSlots
#define DS_CPS_LAUNCH(PRE_, SLOTS_, THREADS_, LDS_)                                                          \
  hipLaunchKernelGGL((cps_kernel<PRE_, SLOTS_>), dim3(batch), dim3(THREADS_), LDS_, st, cand_id, cand_logp,   \
                     cand_cnt, eos_logp, K, m_max, B, lambda, table, mask, ctx, eos_id, g, path, path_len,   \
                     path_score, mirror)
  const float* g = nullptr;
  if (use_pre && ws && ws_bytes >= cps_ws_bytes(batch, K, m_max)) {
    float* gw = static_cast<float*>(ws);
    hipLaunchKernelGGL(cps_gather_kernel, dim3(K, batch), dim3(256), 0, st, cand_id, cand_cnt, K, m_max, table, mask,
                       ctx, eos_id, gw);
    DS_LAUNCH_CHECK("cps_gather_kernel");
    g = gw;
  }
  if (use_pre) {
    const size_t lds = fixed + pre;
    if (lds > 48 * 1024) {
      static thread_local bool granted[3] = {false, false, false};
      const int which = slots == 1 ? 0 : (slots <= 3 ? 1 : 2);
      if (!granted[which]) {
        const void* fn = which == 0   ? reinterpret_cast<const void*>(&cps_kernel<true, 1>)
                         : which == 1 ? reinterpret_cast<const void*>(&cps_kernel<true, 3>)
                                      : reinterpret_cast<const void*>(&cps_kernel<true, kMaxSlots>);
        DS_HIP_CHECK(hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLdsBudget));
        granted[which] = true;
      }
    }
    if (slots == 1) DS_CPS_LAUNCH(true, 1, 1024, lds);
    else if (slots <= 3) DS_CPS_LAUNCH(true, 3, 1024, lds);
    else DS_CPS_LAUNCH(true, kMaxSlots, 1024, lds);
  } else {
    if (slots == 1) DS_CPS_LAUNCH(false, 1, kWave, fixed);
    else if (slots <= 3) DS_CPS_LAUNCH(false, 3, kWave, fixed);
    else DS_CPS_LAUNCH(false, kMaxSlots, kWave, fixed);
  }
#undef DS_CPS_LAUNCH
  DS_LAUNCH_CHECK("cps_kernel");
  return DS_OK;
}

}  // namespace ds
