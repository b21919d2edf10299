// Causal-consistency path search with a tiny causal LM as the causal proxy (Sec. 3.2, "Scoring and search").
//
// The search is the depth-synchronous beam search of k_cps.hip; what differs is where the proxy score comes from.
// With an LM proxy the score of a hypothesis' next token is log softmax(z)[token], z being the proxy's logits after
// the committed tokens and the hypothesis' own tokens, so the proxy has to take one step per depth for every live
// hypothesis.  The host side (ds_cps_path_lm) therefore enqueues, per depth, one proxy forward of one row per beam
// slot (each slot a sequence with its own KV cache) and three small kernels of this file:
//   lm_score_kernel      per slot and vocabulary segment: the segment's largest logit and its sum of
//                        exp(x - largest), the pieces of the row's log-sum-exp;
//   lm_beam_step_kernel  one wavefront: joins the pieces, scores every (live hypothesis, candidate) expansion with
//                        log softmax = logit - lse, keeps the best B by (score descending, expansion index
//                        ascending), applies the EOS rule, and leaves the next step's tokens, each new slot's parent
//                        and the back-pointers in device memory;
//   kv_copy_kernel       gives every new slot the block-region keys / values of its parent (the beam reorders).
// Nothing returns to the host between the steps; after an EOS ends the search the remaining steps' kernels see the
// `finished` flag and do nothing.  Score arithmetic is the unfused float32 order of k_cps.hip.
#include <limits.h>
#include <math.h>

#include "ds_common.h"
#include "ds_wave.h"

#pragma clang fp contract(off)

namespace ds {
namespace {

constexpr int kMaxCand = DS_MAX_TOPM + 1;  // + retained EOS
constexpr int kSlots = (kLmBeam * kMaxCand + kWave - 1) / kWave;  // expansions per lane

__global__ __launch_bounds__(64) void lm_init_kernel(LmSearchState* st) {
  const int t = threadIdx.x;
  if (t < kLmBeam) {
    st->tok[0][t] = st->tok[1][t] = 0;
    st->score[0][t] = st->score[1][t] = 0.f;
    st->par[t] = 0;
  }
  if (t == 0) {
    st->n_live = 1;
    st->finished = 0;
    st->out_len = 0;
    st->out_score = 0.f;
  }
}

// Workgroup (s, g): segment g of logits row s -> (largest value, sum of exp(x - largest)), float32, fixed order.
__global__ __launch_bounds__(256) void lm_score_kernel(const float* __restrict__ logits, int vocab,
                                                      LmSearchState* st) {
  __shared__ float red[4];
  const int s = blockIdx.x, g = blockIdx.y, tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
  if (st->finished || s >= st->n_live) return;  // uniform over the workgroup
  const int seg = ((vocab + kLmParts - 1) / kLmParts + 3) & ~3;
  const int lo = g * seg, hi = lo + seg < vocab ? lo + seg : vocab;
  const float* z = logits + (size_t)s * vocab;
  // a thread keeps the values it reads (at most kPer float4) so that the row is read once
  constexpr int kPer = 8;
  const bool vec = (vocab & 3) == 0 && seg <= kPer * 256 * 4;
  float4 v[kPer];
  float mx = -INFINITY;
  if (vec) {
#pragma unroll
    for (int j = 0; j < kPer; ++j) {
      const int c = lo + (j * 256 + tid) * 4;
      v[j] = c < hi ? *reinterpret_cast<const float4*>(z + c) : make_float4(-INFINITY, -INFINITY, -INFINITY, -INFINITY);
      mx = fmaxf(fmaxf(mx, fmaxf(v[j].x, v[j].y)), fmaxf(v[j].z, v[j].w));
    }
  } else {
    for (int c = lo + tid; c < hi; c += 256) mx = fmaxf(mx, z[c]);
  }
#pragma unroll
  for (int off = kWave / 2; off > 0; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off));
  if (lane == 0) red[wave] = mx;
  __syncthreads();
  mx = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
  __syncthreads();
  float sum = 0.f;
  if (mx > -INFINITY) {
    if (vec) {
#pragma unroll
      for (int j = 0; j < kPer; ++j)
        sum += (expf(v[j].x - mx) + expf(v[j].y - mx)) + (expf(v[j].z - mx) + expf(v[j].w - mx));
    } else {
      for (int c = lo + tid; c < hi; c += 256) sum += expf(z[c] - mx);
    }
  }
#pragma unroll
  for (int off = kWave / 2; off > 0; off >>= 1) sum += __shfl_xor(sum, off);
  if (lane == 0) red[wave] = sum;
  __syncthreads();
  if (tid == 0) st->part[s][g] = make_float2(mx, (red[0] + red[1]) + (red[2] + red[3]));
}

// Depth i of the search, one wavefront.  Reads the beam of parity i & 1, writes the beam of parity (i + 1) & 1.
__global__ __launch_bounds__(64) void lm_beam_step_kernel(LmSearchState* st, const float* __restrict__ logits,
                                                         int vocab, const int32_t* __restrict__ cand_id,
                                                         const float* __restrict__ cand_logp,
                                                         const int32_t* __restrict__ cand_cnt,
                                                         const float* __restrict__ eos_logp, int i, int K, int m_max,
                                                         int B, float lambda, int32_t eos_id) {
  __shared__ int32_t c_tok[kMaxCand];
  __shared__ float c_lp[kMaxCand];
  __shared__ float s_lse[kLmBeam];
  if (st->finished) return;
  const int lane = threadIdx.x;
  // candidates of lattice row i, one per lane: the first cand_cnt entries, EOS appended if it is not among them
  int n_cand = cand_cnt[i];
  n_cand = n_cand < 1 ? 1 : (n_cand > m_max ? m_max : n_cand);
  int my_tok = -1;
  float my_lp = 0.f;
  if (lane < n_cand) {
    my_tok = cand_id[(size_t)i * m_max + lane];
    my_lp = cand_logp[(size_t)i * m_max + lane];
  }
  const unsigned long long at_eos = __ballot(lane < n_cand && eos_id >= 0 && my_tok == eos_id);
  int eos_rank = at_eos ? __ffsll((long long)at_eos) - 1 : -1;
  if (eos_id >= 0 && eos_rank < 0) {
    if (lane == n_cand) {
      my_tok = eos_id;
      my_lp = eos_logp[i];
    }
    eos_rank = n_cand;
    ++n_cand;
  }
  if (lane < n_cand) {
    c_tok[lane] = my_tok;
    c_lp[lane] = my_lp;
  }
  __syncthreads();
  const int n_live = st->n_live;
  // log-sum-exp of every live row from its segments (fixed order: the same bits whatever else runs)
  for (int b = 0; b < n_live; ++b) {
    const float2 pc = lane < kLmParts ? st->part[b][lane] : make_float2(-INFINITY, 0.f);
    float mx = pc.x;
#pragma unroll
    for (int off = kWave / 2; off > 0; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off));
    float sum = pc.y > 0.f ? pc.y * expf(pc.x - mx) : 0.f;
#pragma unroll
    for (int off = kWave / 2; off > 0; off >>= 1) sum += __shfl_xor(sum, off);
    if (lane == 0) s_lse[b] = mx + logf(sum);
  }
  __syncthreads();
  const int n_exp = n_live * n_cand;
  const float one_minus = 1.0f - lambda;
  const int cur = i & 1, nxt = cur ^ 1;

  uint32_t e_bits[kSlots];
  float e_score[kSlots];
  int e_tok[kSlots], e_par[kSlots], e_dst[kSlots];
#pragma unroll
  for (int j = 0; j < kSlots; ++j) {
    const int e = lane + j * kWave;
    e_bits[j] = 0u;
    e_score[j] = 0.f;
    e_tok[j] = e_par[j] = 0;
    e_dst[j] = -1;
    if (e < n_exp) {
      const int b = e / n_cand, c = e - b * n_cand;
      int t = c_tok[c];
      t = (t < 0 || t >= vocab) ? 0 : t;
      const float lng = logits[(size_t)b * vocab + t] - s_lse[b];
      const float dlm_part = lambda * c_lp[c], ng_part = one_minus * lng;
      const float term = dlm_part + ng_part;
      e_score[j] = st->score[cur][b] + term;
      e_bits[j] = ordered_bits(e_score[j]);
      e_tok[j] = c_tok[c];
      e_par[j] = b;
    }
  }

  const int n_keep = n_exp < B ? n_exp : B;
  int live = 0;
  bool finished = false;
  for (int r = 0; r < n_keep; ++r) {
    // this lane's best open expansion: largest score, lowest expansion index among equals
    uint32_t best_bits = 0;
    int best_slot = 0;
#pragma unroll
    for (int j = kSlots - 1; j >= 0; --j)
      if (e_bits[j] != 0u && e_bits[j] >= best_bits) {
        best_bits = e_bits[j];
        best_slot = j;
      }
    const uint32_t top = wave_max_u32(best_bits);
    const uint32_t my_e = (best_bits == top && best_bits != 0u) ? (uint32_t)(lane + best_slot * kWave) : 0xFFFFFFFFu;
    const int e = __builtin_amdgcn_readfirstlane((int)(0xFFFFFFFFu - wave_max_u32(0xFFFFFFFFu - my_e)));
    const int owner = e & (kWave - 1), slot = e >> 6;
    const int par = e / n_cand, c = e - par * n_cand;
    const bool is_eos = (c == eos_rank);
    if (r == 0 && is_eos) {  // the best kept hypothesis ends in EOS: it is the result
      if (lane == owner) {
        st->bp_tok[i][0] = eos_id;
        st->bp_par[i][0] = par;
        st->out_len = i + 1;
        st->out_score = __uint_as_float(top & 0x80000000u ? (top & 0x7FFFFFFFu) : ~top);
        st->finished = 1;
      }
      finished = true;
      break;
    }
#pragma unroll
    for (int j = 0; j < kSlots; ++j) {
      const bool mine = lane == owner && j == slot;
      e_bits[j] = mine ? 0u : e_bits[j];
      e_dst[j] = (mine && !is_eos) ? live : e_dst[j];
    }
    live += is_eos ? 0 : 1;
  }
  if (finished) return;
#pragma unroll
  for (int j = 0; j < kSlots; ++j)
    if (e_dst[j] >= 0) {
      const int d = e_dst[j];
      st->tok[nxt][d] = e_tok[j];
      st->score[nxt][d] = e_score[j];
      st->par[d] = e_par[j];
      st->bp_tok[i][d] = e_tok[j];
      st->bp_par[i][d] = e_par[j];
      if (d == 0 && i + 1 == K) {  // ran to the end: the best live hypothesis of the last step
        st->out_len = K;
        st->out_score = e_score[j];
      }
    }
  if (lane == 0) st->n_live = live;
}

__global__ __launch_bounds__(64) void lm_backtrack_kernel(const LmSearchState* st, int K, int32_t* __restrict__ path,
                                                         int32_t* __restrict__ path_len,
                                                         float* __restrict__ path_score) {
  const int lane = threadIdx.x;
  const int out_len = st->out_len;
  if (lane == 0) {
    int slot = 0;
    for (int i = out_len - 1; i >= 0; --i) {
      path[i] = st->bp_tok[i][slot];
      slot = st->bp_par[i][slot];
    }
    path_len[0] = out_len;
    path_score[0] = st->out_score;
  }
  for (int i = out_len + lane; i < K; i += kWave) path[i] = -1;
}

// Destination cache d receives bytes [lo, hi) of every (layer, head) segment of its source cache: source
// src_of[d], or the cache of slot par[d] if par is given (then slots >= n_live, and everything once the search
// has finished, are skipped).
__global__ __launch_bounds__(256) void kv_copy_kernel(KvCopyPlan p, const int32_t* __restrict__ par,
                                                     const LmSearchState* st, size_t head_bytes, size_t lo,
                                                     size_t hi) {
  const int d = blockIdx.y >> 1, is_v = blockIdx.y & 1;
  if (st && (st->finished || d >= st->n_live)) return;
  int src = par ? par[d] : p.src_of[d];
  src = src < 0 ? 0 : (src >= p.n_src ? p.n_src - 1 : src);
  const char* s = static_cast<const char*>(is_v ? p.src_v[src] : p.src_k[src]) + (size_t)blockIdx.x * head_bytes;
  char* t = static_cast<char*>(is_v ? p.dst_v[d] : p.dst_k[d]) + (size_t)blockIdx.x * head_bytes;
  if (s == t) return;
  if (((lo | hi) & 15) == 0) {
    for (size_t off = lo + (size_t)threadIdx.x * 16; off < hi; off += 256 * 16)
      *reinterpret_cast<uint4*>(t + off) = *reinterpret_cast<const uint4*>(s + off);
  } else {  // float32 caches of narrow heads: 4-byte words
    for (size_t off = lo + (size_t)threadIdx.x * 4; off < hi; off += 256 * 4)
      *reinterpret_cast<uint32_t*>(t + off) = *reinterpret_cast<const uint32_t*>(s + off);
  }
}

}  // namespace

int launch_lm_init(LmSearchState* st, hipStream_t s) {
  hipLaunchKernelGGL(lm_init_kernel, dim3(1), dim3(64), 0, s, st);
  DS_LAUNCH_CHECK("lm_init_kernel");
  return DS_OK;
}

int launch_lm_score(const float* logits, int n_rows, int vocab, LmSearchState* st, hipStream_t s) {
  hipLaunchKernelGGL(lm_score_kernel, dim3(n_rows, kLmParts), dim3(256), 0, s, logits, vocab, st);
  DS_LAUNCH_CHECK("lm_score_kernel");
  return DS_OK;
}

int launch_lm_beam_step(LmSearchState* st, const float* logits, int vocab, const int32_t* cand_id,
                        const float* cand_logp, const int32_t* cand_cnt, const float* eos_logp, int i, int K,
                        int m_max, int B, float lambda, int32_t eos_id, hipStream_t s) {
  hipLaunchKernelGGL(lm_beam_step_kernel, dim3(1), dim3(64), 0, s, st, logits, vocab, cand_id, cand_logp, cand_cnt,
                     eos_logp, i, K, m_max, B, lambda, eos_id);
  DS_LAUNCH_CHECK("lm_beam_step_kernel");
  return DS_OK;
}

int launch_lm_backtrack(const LmSearchState* st, int K, int32_t* path, int32_t* path_len, float* path_score,
                        hipStream_t s) {
  hipLaunchKernelGGL(lm_backtrack_kernel, dim3(1), dim3(64), 0, s, st, K, path, path_len, path_score);
  DS_LAUNCH_CHECK("lm_backtrack_kernel");
  return DS_OK;
}

int launch_kv_copy(const KvCopyPlan& plan, const int32_t* par, const LmSearchState* st, int n_segments,
                   size_t head_bytes, size_t lo, size_t hi, hipStream_t s) {
  if (plan.n_dst <= 0 || hi <= lo) return DS_OK;
  DS_REQUIRE(plan.n_dst <= 2 * kMaxSeq && plan.n_src >= 1 && plan.n_src <= kMaxSeq && hi <= head_bytes &&
                 (lo & 3) == 0 && (hi & 3) == 0,
             DS_E_INVALID, "kv copy: bad plan");
  hipLaunchKernelGGL(kv_copy_kernel, dim3(n_segments, plan.n_dst * 2), dim3(256), 0, s, plan, par, st, head_bytes, lo,
                     hi);
  DS_LAUNCH_CHECK("kv_copy_kernel");
  return DS_OK;
}

}  // namespace ds
