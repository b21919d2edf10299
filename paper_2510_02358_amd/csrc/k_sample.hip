// Two small pieces beyond the greedy single-pass round:
//
//  * stochastic block verification (Sec. 2, "Parallel verification": accept draft token i with
//    probability min(1, p / q), replace the first rejected token by a draw from the residual
//    max(p - q, 0), draw a bonus token from p after full acceptance).  The uniforms are inputs, so the
//    kernels hold no random-number generator; the draw is an inverse-CDF walk in vocabulary order.
//  * the update step of multi-pass refinement (Sec. 2, refinement update equation): fix the most
//    confident still-masked positions to their arg-max token and freeze their lattice rows.
//
// Both are latency-sized (a few rows of the vocabulary, at most 256 block positions): plain ALU code,
// float32 arithmetic, every sum taken in a fixed order.
#include <limits.h>
#include <math.h>

#include "ds_common.h"

namespace ds {
namespace {

constexpr int kStatThreads = 1024;

// max then sum of one workgroup (same value in every thread)
__device__ __forceinline__ float block_max(float v, float* red) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v = fmaxf(v, __shfl_xor(v, off));
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  __syncthreads();
  if (lane == 0) red[wave] = v;
  __syncthreads();
  float m = red[0];
  for (int w = 1; w < (int)(blockDim.x >> 6); ++w) m = fmaxf(m, red[w]);
  return m;
}
__device__ __forceinline__ float block_sum(float v, float* red) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off);
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  __syncthreads();
  if (lane == 0) red[wave] = v;
  __syncthreads();
  float s = 0.f;
  for (int w = 0; w < (int)(blockDim.x >> 6); ++w) s += red[w];
  return s;
}

// Log-sum-exp of the logits rows, in two steps so that a handful of rows still fills the chip: every row is cut
// into kLseSeg equal segments of whole float4 groups (the last one also takes the tail); workgroup (b, g) leaves
// (max, sum of exp(x - max)) of segment g of row b in part[b][g]; the acceptance kernel combines the kLseSeg pairs
// of a row in segment order.  Row b < n_p is verifier row b, the others drafter row b - n_p.
constexpr int kLseSeg = 8;
constexpr int kLseThreads = 256;

__global__ __launch_bounds__(kLseThreads) void row_lse_kernel(const float* __restrict__ p_logits, int n_p,
                                                             const float* __restrict__ q_logits, int vocab,
                                                             float2* __restrict__ part) {
  __shared__ float red[kLseThreads / 64];
  const int b = blockIdx.x, g = blockIdx.y;
  const float* row = b < n_p ? p_logits + (size_t)b * vocab : q_logits + (size_t)(b - n_p) * vocab;
  const bool vec = (vocab & 3) == 0 && (((uintptr_t)row) & 15) == 0;
  // segment bounds in elements: multiples of 4 except the end of the last segment
  const int per = ((vocab / kLseSeg) + 3) & ~3;
  int lo = g * per, hi = (g == kLseSeg - 1) ? vocab : lo + per;
  lo = lo < vocab ? lo : vocab;
  hi = hi < vocab ? hi : vocab;
  const int n4 = vec ? (hi - lo) >> 2 : 0;
  typedef float vec4 __attribute__((ext_vector_type(4)));
  const vec4* row4 = reinterpret_cast<const vec4*>(row + lo);
  // one pass: each thread keeps a running (max, sum) over batches of kLseBatch independent 16-byte loads
  constexpr int kLseBatch = 8;
  float tm = -INFINITY, ts = 0.f;
  for (int i0 = threadIdx.x; i0 < n4; i0 += kLseThreads * kLseBatch) {
    vec4 v[kLseBatch];
#pragma unroll
    for (int k = 0; k < kLseBatch; ++k) {
      const int i = i0 + k * kLseThreads;
      // ordinary loads on purpose: the acceptance kernel reads one of these rows again right afterwards
      v[k] = i < n4 ? row4[i] : vec4{-INFINITY, -INFINITY, -INFINITY, -INFINITY};
    }
    float bm = -INFINITY;
#pragma unroll
    for (int k = 0; k < kLseBatch; ++k) bm = fmaxf(bm, fmaxf(fmaxf(v[k][0], v[k][1]), fmaxf(v[k][2], v[k][3])));
    if (bm > tm) {
      ts *= __expf(tm - bm);  // tm = -inf: 0 * 0
      tm = bm;
    }
    if (tm > -INFINITY) {
      float acc = 0.f;
#pragma unroll
      for (int k = 0; k < kLseBatch; ++k)
        acc += (__expf(v[k][0] - tm) + __expf(v[k][1] - tm)) + (__expf(v[k][2] - tm) + __expf(v[k][3] - tm));
      ts += acc;
    }
  }
  for (int v = lo + n4 * 4 + threadIdx.x; v < hi; v += kLseThreads) {
    const float x = row[v];
    if (x > tm) {
      ts *= __expf(tm - x);
      tm = x;
    }
    if (tm > -INFINITY) ts += __expf(x - tm);
  }
  const float mx = block_max(tm, red);
  float s = (tm > -INFINITY) ? ts * __expf(tm - mx) : 0.f;
  s = block_sum(s, red);
  if (threadIdx.x == 0) part[(size_t)b * kLseSeg + g] = make_float2(mx, s);
}

// lse of row b from its segment pairs (fixed order).
__device__ __forceinline__ float combine_lse(const float2* __restrict__ part, int b) {
  float mx = -INFINITY;
#pragma unroll
  for (int g = 0; g < kLseSeg; ++g) mx = fmaxf(mx, part[(size_t)b * kLseSeg + g].x);
  float s = 0.f;
#pragma unroll
  for (int g = 0; g < kLseSeg; ++g) {
    const float2 q = part[(size_t)b * kLseSeg + g];
    if (q.x > -INFINITY) s += q.y * __expf(q.x - mx);
  }
  return mx + __logf(s);
}

// Stochastic acceptance in two kernels.
//
// sample_decide_kernel (one workgroup): log-sum-exp of every row from its segment pairs, the acceptance
// probabilities alpha, the accepted prefix length L (first i with u[i] >= alpha_i) and whether an accepted token is
// EOS.  Leaves {L, eos flag, effective path length, arrival counter = 0} in ctl and the lse values in lse.
//
// sample_draw_kernel (one workgroup per segment of kSeg = 4096 consecutive tokens): the inverse-CDF draw on verifier
// row L, in vocabulary order, hierarchically and with coalesced loads; inside a segment thread t owns the 4
// consecutive tokens 4 t .. 4 t + 3.
//   pass 1: every workgroup sums the weights of its segment (per-wavefront sums in lane order, the 16 wavefront
//   sums in order) and leaves the total in seg_tot; the workgroup that arrives last goes on alone (nobody waits):
//   it finds the segment whose cumulative total first exceeds the target by walking the <= 64 totals in order;
//   pass 2: inside that segment, an inclusive scan of the 1024 four-token sums finds the owning thread, which
//   walks its 4 tokens.  Every sum has a fixed order, so the drawn token is reproducible bit for bit.
//   If the residual max(p - q, 0) is empty (p == q up to rounding) the last workgroup redoes pass 1 on p alone, by
//   itself: rare, and then slower.
constexpr int kSeg = 4 * kStatThreads;
constexpr int kMaxSeg = 64;  // vocabularies up to 262144 tokens

__global__ __launch_bounds__(256) void sample_decide_kernel(
    const float* __restrict__ p_logits, const float* __restrict__ q_logits, int m, int vocab,
    const float2* __restrict__ lse_part, const int32_t* __restrict__ block, const int32_t* __restrict__ path_len,
    const float* __restrict__ u, int32_t eos_id, float* __restrict__ lse, int32_t* __restrict__ ctl,
    float* __restrict__ alpha_out) {
  __shared__ int s_first, s_eos;
  const int t = threadIdx.x;
  int m_eff = m;
  if (path_len) {
    const int pl = *path_len;
    m_eff = pl < m ? (pl < 0 ? 0 : pl) : m;
  }
  if (t == 0) {
    s_first = m_eff;
    s_eos = 0;
  }
  for (int b = t; b < 2 * m + 1; b += blockDim.x) lse[b] = combine_lse(lse_part, b);
  __syncthreads();  // also orders this workgroup's lse stores before its own loads below
  for (int i = t; i < m; i += blockDim.x) {
    const int tok = block[i + 1];
    float a = 0.f;
    if (tok >= 0 && tok < vocab) {
      const float lp = p_logits[(size_t)i * vocab + tok] - combine_lse(lse_part, i);
      const float lq = q_logits[(size_t)i * vocab + tok] - combine_lse(lse_part, m + 1 + i);
      a = lq <= lp ? 1.0f : __expf(lp - lq);
    }
    alpha_out[i] = a;
    if (i < m_eff && !(u[i] < a)) atomicMin(&s_first, i);
  }
  __syncthreads();
  const int L = s_first;  // accepted prefix length; the draw uses verifier row L
  for (int i = t; i < L; i += blockDim.x)
    if (eos_id >= 0 && block[i + 1] == eos_id) atomicOr(&s_eos, 1);
  __syncthreads();
  if (t == 0) {
    ctl[0] = L;
    ctl[1] = s_eos;
    ctl[2] = m_eff;
    ctl[3] = 0;  // arrival counter of the draw kernel
  }
}

__global__ __launch_bounds__(kStatThreads) void sample_draw_kernel(
    const float* __restrict__ p_logits, const float* __restrict__ q_logits, int m, int vocab,
    const float* __restrict__ lse, int32_t* __restrict__ ctl, float* seg_tot, const float* __restrict__ u,
    int32_t eos_id, int32_t* __restrict__ n_accept, int32_t* __restrict__ next_token,
    int32_t* __restrict__ eos_accepted) {
  __shared__ float wave_sum[kStatThreads / 64];
  __shared__ float seg_total[kMaxSeg];
  __shared__ float part[2][kStatThreads];
  __shared__ float s_before, s_target, s_total;
  __shared__ int s_seg, s_thread, s_last;
  __shared__ bool s_is_last;
  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  const int L = ctl[0], acc_eos = ctl[1], m_eff = ctl[2];

  const float* prow = p_logits + (size_t)L * vocab;
  const float* qrow = L < m ? q_logits + (size_t)L * vocab : nullptr;
  const float lse_p = lse[L], lse_q = L < m ? lse[m + 1 + L] : 0.f;
  const int n_seg = (vocab + kSeg - 1) / kSeg;
  bool residual = L < m_eff;
  const bool vec = (vocab & 3) == 0 && (((uintptr_t)prow) & 15) == 0 && (!qrow || (((uintptr_t)qrow) & 15) == 0);

  // the four weights thread t owns in segment seg (0 beyond the vocabulary)
  auto weights4 = [&](int seg, float w[4]) {
    const int v0 = seg * kSeg + 4 * t;
    float pv[4], qv[4];
    if (vec && v0 + 3 < vocab) {
      const float4 a = *reinterpret_cast<const float4*>(prow + v0);
      pv[0] = a.x; pv[1] = a.y; pv[2] = a.z; pv[3] = a.w;
      if (residual) {
        const float4 c = *reinterpret_cast<const float4*>(qrow + v0);
        qv[0] = c.x; qv[1] = c.y; qv[2] = c.z; qv[3] = c.w;
      }
    } else {
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        pv[e] = v0 + e < vocab ? prow[v0 + e] : -INFINITY;
        qv[e] = (residual && v0 + e < vocab) ? qrow[v0 + e] : -INFINITY;
      }
    }
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      float x = __expf(pv[e] - lse_p);  // exp(-inf) = 0 beyond the vocabulary
      if (residual) x = fmaxf(x - __expf(qv[e] - lse_q), 0.f);
      w[e] = x;
    }
  };
  // total weight of one segment: wavefront sums in lane order, then the wavefront sums in order (every thread
  // of the workgroup calls this; the value is valid in thread 0)
  auto segment_total = [&](int seg) {
    float w[4];
    weights4(seg, w);
    float s = (w[0] + w[1]) + (w[2] + w[3]);
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) s += __shfl_xor(s, off);
    __syncthreads();
    if (lane == 0) wave_sum[wave] = s;
    __syncthreads();
    float ss = 0.f;
    if (t == 0)
      for (int w2 = 0; w2 < kStatThreads / 64; ++w2) ss += wave_sum[w2];
    return ss;
  };

  // pass 1, this workgroup's segment; the last workgroup to arrive continues
  {
    const float ss = segment_total((int)blockIdx.x);
    if (t == 0) {
      __hip_atomic_store(&seg_tot[blockIdx.x], ss, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      __threadfence();
      const int seen = __hip_atomic_fetch_add(&ctl[3], 1, __ATOMIC_ACQ_REL, __HIP_MEMORY_SCOPE_AGENT);
      s_is_last = seen == n_seg - 1;
    }
    __syncthreads();
    if (!s_is_last) return;
    __threadfence();
    if (t < n_seg) seg_total[t] = __hip_atomic_load(&seg_tot[t], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __syncthreads();
  }

  for (int attempt = 0; attempt < 2; ++attempt) {
    if (t == 0) {
      float total = 0.f;
      for (int seg = 0; seg < n_seg; ++seg) total += seg_total[seg];
      const float target = u[m] * total;
      float c = 0.f;
      int pick = -1, last_pos = -1;
      for (int seg = 0; seg < n_seg; ++seg) {
        const float ss = seg_total[seg];
        if (ss > 0.f) {
          last_pos = seg;
          if (c + ss > target) {
            pick = seg;
            break;
          }
        }
        c += ss;
      }
      if (pick < 0) {  // rounding left the target past the mass: the last segment that has any
        pick = last_pos;
        c = 0.f;
        for (int seg = 0; seg < pick; ++seg) c += seg_total[seg];
      }
      s_total = total;
      s_target = target;
      s_before = c;
      s_seg = pick;
    }
    __syncthreads();
    if (!(residual && !(s_total > 0.f))) break;
    residual = false;  // p == q up to rounding: the residual is empty, draw from p instead
    for (int seg = 0; seg < n_seg; ++seg) {
      const float ss = segment_total(seg);
      if (t == 0) seg_total[seg] = ss;
    }
    __syncthreads();
  }

  // pass 2: inside the chosen segment
  const int seg = s_seg;
  float w[4] = {0.f, 0.f, 0.f, 0.f};
  if (seg >= 0) weights4(seg, w);
  const float s4 = (w[0] + w[1]) + (w[2] + w[3]);
  int cur = 0;
  part[0][t] = s4;
  if (t == 0) {
    s_thread = INT_MAX;
    s_last = -1;
  }
  __syncthreads();
  for (int off = 1; off < kStatThreads; off <<= 1) {
    const float x = part[cur][t] + (t >= off ? part[cur][t - off] : 0.f);
    part[cur ^ 1][t] = x;
    cur ^= 1;
    __syncthreads();
  }
  const float incl = s_before + part[cur][t];
  const float excl = s_before + (t > 0 ? part[cur][t - 1] : 0.f);
  if (s4 > 0.f) {
    atomicMax(&s_last, t);
    if (incl > s_target) atomicMin(&s_thread, t);
  }
  __syncthreads();
  const int pick_t = s_thread != INT_MAX ? s_thread : s_last;
  if (pick_t < 0 && t == 0) {  // no positive weight anywhere (NaN logits are a caller error): defined outputs
    *n_accept = L;
    *next_token = 0;
    __threadfence_system();
    *eos_accepted = acc_eos;
  }
  if (t == pick_t) {
    float c = excl;
    int chosen = -1, last_pos = -1;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      c += w[e];
      if (w[e] > 0.f) {
        last_pos = e;
        if (chosen < 0 && c > s_target) chosen = e;
      }
    }
    if (chosen < 0) chosen = last_pos;
    const int tok = seg * kSeg + 4 * t + chosen;
    *n_accept = L;
    *next_token = tok;
    __threadfence_system();  // eos_accepted last, as in the greedy kernels
    *eos_accepted = (acc_eos || (eos_id >= 0 && tok == eos_id)) ? 1 : 0;
  }
}

// Refinement update: among positions whose block token is still mask_id, the n_update with the largest
// top-1 log-probability (ties: lower position) take their arg-max token, and their lattice rows are
// copied to the output lattice.  One workgroup, one thread per position.
__global__ __launch_bounds__(256) void refine_select_kernel(
    const int32_t* __restrict__ cand_id, const float* __restrict__ cand_logp, const int32_t* __restrict__ cand_cnt,
    const float* __restrict__ eos_logp, const float* __restrict__ lse, int K, int m_max, int n_update,
    int32_t mask_id, int32_t* __restrict__ block_tokens, int32_t* __restrict__ o_id, float* __restrict__ o_logp,
    int32_t* __restrict__ o_cnt, float* __restrict__ o_eos, float* __restrict__ o_lse) {
  __shared__ float conf[256];
  __shared__ int masked[256];
  const int i = threadIdx.x;
  if (i < K) {
    masked[i] = block_tokens[i] == mask_id;
    conf[i] = cand_logp[(size_t)i * m_max];
  }
  __syncthreads();
  if (i >= K || !masked[i]) return;
  int rank = 0;
  const float mine = conf[i];
  for (int j = 0; j < K; ++j)
    if (masked[j] && (conf[j] > mine || (conf[j] == mine && j < i))) ++rank;
  if (rank >= n_update) return;
  block_tokens[i] = cand_id[(size_t)i * m_max];
  for (int c = 0; c < m_max; ++c) {
    o_id[(size_t)i * m_max + c] = cand_id[(size_t)i * m_max + c];
    o_logp[(size_t)i * m_max + c] = cand_logp[(size_t)i * m_max + c];
  }
  o_cnt[i] = cand_cnt[i];
  o_eos[i] = eos_logp[i];
  o_lse[i] = lse[i];
}

}  // namespace

// workspace: segment pairs of the row log-sum-exps, the log-sum-exps, the control words, the segment totals
size_t sample_ws_bytes(int m) {
  return align_up((size_t)(2 * m + 1) * kLseSeg * sizeof(float2), 256) + align_up((size_t)(2 * m + 1) * sizeof(float), 256) +
         256 + align_up(kMaxSeg * sizeof(float), 256);
}

int launch_sample_accept(const float* p_logits, const float* q_logits, int m, int vocab, const int32_t* block,
                         const int32_t* path_len, const float* u, int32_t eos_id, int32_t* n_accept,
                         int32_t* next_token, int32_t* eos_accepted, float* alpha, void* ws, size_t ws_bytes,
                         hipStream_t st) {
  DS_REQUIRE(ws_bytes >= sample_ws_bytes(m), DS_E_CAPACITY, "sampling workspace: need %zu bytes, got %zu",
             sample_ws_bytes(m), ws_bytes);
  DS_REQUIRE(vocab <= kSeg * kMaxSeg, DS_E_UNSUPPORTED, "stochastic acceptance: vocab %d exceeds %d", vocab,
             kSeg * kMaxSeg);
  char* base = static_cast<char*>(ws);
  float2* lse_part = reinterpret_cast<float2*>(base);  // per-segment (max, sum) pairs
  base += align_up((size_t)(2 * m + 1) * kLseSeg * sizeof(float2), 256);
  float* lse = reinterpret_cast<float*>(base);
  base += align_up((size_t)(2 * m + 1) * sizeof(float), 256);
  int32_t* ctl = reinterpret_cast<int32_t*>(base);
  float* seg_tot = reinterpret_cast<float*>(base + 256);
  hipLaunchKernelGGL(row_lse_kernel, dim3(2 * m + 1, kLseSeg), dim3(kLseThreads), 0, st, p_logits, m + 1, q_logits,
                     vocab, lse_part);
  DS_LAUNCH_CHECK("row_lse_kernel");
  hipLaunchKernelGGL(sample_decide_kernel, dim3(1), dim3(256), 0, st, p_logits, q_logits, m, vocab, lse_part, block,
                     path_len, u, eos_id, lse, ctl, alpha);
  DS_LAUNCH_CHECK("sample_decide_kernel");
  const int n_seg = ceil_div(vocab, kSeg);
  hipLaunchKernelGGL(sample_draw_kernel, dim3(n_seg), dim3(kStatThreads), 0, st, p_logits, q_logits, m, vocab, lse, ctl,
                     seg_tot, u, eos_id, n_accept, next_token, eos_accepted);
  DS_LAUNCH_CHECK("sample_draw_kernel");
  return DS_OK;
}

int launch_refine_select(const int32_t* cand_id, const float* cand_logp, const int32_t* cand_cnt,
                         const float* eos_logp, const float* lse, int K, int m_max, int n_update, int32_t mask_id,
                         int32_t* block_tokens, int32_t* o_id, float* o_logp, int32_t* o_cnt, float* o_eos,
                         float* o_lse, hipStream_t st) {
  hipLaunchKernelGGL(refine_select_kernel, dim3(1), dim3(256), 0, st, cand_id, cand_logp, cand_cnt, eos_logp, lse, K,
                     m_max, n_update, mask_id, block_tokens, o_id, o_logp, o_cnt, o_eos, o_lse);
  DS_LAUNCH_CHECK("refine_select_kernel");
  return DS_OK;
}

}  // namespace ds
