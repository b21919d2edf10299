// Grouped-query attention of a few query rows against the KV cache (cached prefix + the rows of the
// current call), split over the key axis ("flash-decoding" style) with an exact log-sum-exp merge.
//
// Visibility: row r (absolute position pos0 + r) sees key p iff p < n_keys and
//   r >= n_causal (a [MASK] row of the draft block: sees everything)  or  p <= pos0 + r (causal).
//
// Half-precision kernel (bf16 models, head_dim 128; q, K, V and probabilities are IEEE half): the
// query rows of all heads that share a KV head are packed together, so one pass over that head's
// keys/values serves group x rows query rows; both products run on the 16x16x32 f16 matrix cores.
// Scores are computed transposed, S^T = K Q^T, because the accumulator layout of S^T (lane = query
// row, 4 consecutive keys per register quad) is already the operand layout the second product P V
// needs: probabilities never leave registers.
//
// Cache layout (private to the library): per KV head the cache is a sequence of 64-key chunks, and a
// chunk of K (and of V) is stored as the 16 matrix-core operand tiles the kernel multiplies with
// (kv_k_offset / kv_v_offset in ds_act.h).  Staging a chunk is therefore a straight, fully coalesced
// 16 KB + 16 KB copy into LDS; two LDS buffers alternate, so the copy of chunk c + 1 (global ->
// registers before the math, registers -> LDS after it) overlaps the math of chunk c with one barrier
// per chunk.
//
// f32 kernel: plain ALU version for the float32 parity mode (any head_dim <= 128, row-major cache).
#include <math.h>

#include "ds_act.h"
#include "ds_common.h"

namespace ds {

typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

namespace {

constexpr int kChunk = 64;  // keys per staged chunk
constexpr int kHd = 128;    // head_dim of the half-precision kernel
constexpr int kChunkElems = kChunk * kHd;  // halfs per chunk of K (and of V): 16 tiles x 512

union Pack8 {
  f16x8 v;
  uint16_t h[8];
  u32x2 half[2];
  u32x4 q;
};

template <int QB>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2))) void attn_f16_kernel(const uint16_t* __restrict__ q,
                                                        const uint16_t* __restrict__ kc,
                                                        const uint16_t* __restrict__ vc, int rows, int rows_pad,
                                                        int rows_stride, int n_causal, int pos0, int n_keys, int n_q,
                                                        int n_kv, int cap, int chunks_per_split, float scale_log2,
                                                        float* __restrict__ part_o, float* __restrict__ part_ml) {
  // rows / rows_pad: the rows of ONE sequence (q, part_o and part_ml already point at its first row);
  // rows_stride: padded rows of the whole call (stride between heads and between splits)
  __shared__ __attribute__((aligned(16))) uint16_t ks_lds[2][kChunkElems];
  __shared__ __attribute__((aligned(16))) uint16_t vs_lds[2][kChunkElems];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int j = lane & 15, g = lane >> 4;
  const int split = blockIdx.x, kvh = blockIdx.y;
  const int group = n_q / n_kv, rb_count = rows_pad >> 4, n_qb = group * rb_count;
  const int n_chunks = (n_keys + kChunk - 1) / kChunk;
  const int c_begin = split * chunks_per_split;
  int c_end = c_begin + chunks_per_split;
  if (c_end > n_chunks) c_end = n_chunks;

  int head[QB], rb[QB], lim_min[QB], limit[QB];
  bool valid[QB];
  f16x8 bq[QB][4];
  f32x4 o[QB][8];
  float m_run[QB], l_run[QB];  // running maximum in log2 units, running sum
#pragma unroll
  for (int t = 0; t < QB; ++t) {
    const int qb = (blockIdx.z * 4 + wave) * QB + t;
    valid[t] = qb < n_qb;
    const int qbc = valid[t] ? qb : 0;
    head[t] = kvh * group + qbc / rb_count;
    rb[t] = qbc % rb_count;
    const uint16_t* qh = q + (size_t)head[t] * rows_stride * kHd + (size_t)rb[t] * 4 * 512;
#pragma unroll
    for (int s = 0; s < 4; ++s) bq[t][s] = *reinterpret_cast<const f16x8*>(qh + s * 512 + lane * 8);
#pragma unroll
    for (int d = 0; d < 8; ++d) o[t][d] = f32x4{0.f, 0.f, 0.f, 0.f};
    m_run[t] = -INFINITY;
    l_run[t] = 0.f;
    const int r = rb[t] * 16 + j;
    limit[t] = (r >= n_causal) ? n_keys - 1 : pos0 + r;                       // last key this lane's row sees
    lim_min[t] = (rb[t] * 16 >= n_causal) ? n_keys - 1 : pos0 + rb[t] * 16;   // smallest limit in the row block
  }

  const uint16_t* kbase = kc + (size_t)kvh * cap * kHd;
  const uint16_t* vbase = vc + (size_t)kvh * cap * kHd;

  // Staging: a chunk is 2 x 1024 pieces of 16 bytes, already in operand order; thread t moves pieces
  // t, t + 256, t + 512, t + 768 of K and of V.
  u32x4 kreg[4], vreg[4];
  auto load_chunk = [&](int c) {
    const uint16_t* ksrc = kbase + (size_t)c * kChunkElems + threadIdx.x * 8;
    const uint16_t* vsrc = vbase + (size_t)c * kChunkElems + threadIdx.x * 8;
#pragma unroll
    for (int p = 0; p < 4; ++p) {
      kreg[p] = *reinterpret_cast<const u32x4*>(ksrc + p * 2048);
      vreg[p] = *reinterpret_cast<const u32x4*>(vsrc + p * 2048);
    }
  };
  auto store_chunk = [&](int c, int buf) {
    const int c0 = c * kChunk;
#pragma unroll
    for (int p = 0; p < 4; ++p) {
      *reinterpret_cast<u32x4*>(&ks_lds[buf][(threadIdx.x + p * 256) * 8]) = kreg[p];
      Pack8 pk;
      pk.q = vreg[p];
      if (c0 + kChunk > n_keys) {  // tail chunk: slots past the last key may hold anything -> zero
        const int t2 = (wave + 4 * p) & 1;  // tile index of this piece = wave + 4 p (V tile = db * 2 + t2)
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const int key = c0 + 32 * t2 + 4 * g + (e & 3) + ((e >> 2) << 4);
          if (key >= n_keys) pk.h[e] = 0;
        }
      }
      *reinterpret_cast<u32x4*>(&vs_lds[buf][(threadIdx.x + p * 256) * 8]) = pk.q;
    }
  };

  if (c_begin < c_end) {
    load_chunk(c_begin);
    store_chunk(c_begin, 0);
  }
  __syncthreads();
  int buf = 0;
  for (int c = c_begin; c < c_end; ++c, buf ^= 1) {
    const int c0 = c * kChunk;
    const int c_next = c + 1 < c_end ? c + 1 : c;  // clamped: the last iteration reloads its own chunk
    load_chunk(c_next);
    __builtin_amdgcn_sched_barrier(0);

    // scores: every K tile is read once and used for all QB query blocks; consecutive products go to
    // different accumulators
    f32x4 s4[QB][4];
#pragma unroll
    for (int t = 0; t < QB; ++t)
#pragma unroll
      for (int kb = 0; kb < 4; ++kb) s4[t][kb] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int s = 0; s < 4; ++s)
#pragma unroll
      for (int kb = 0; kb < 4; ++kb) {
        const f16x8 a = *reinterpret_cast<const f16x8*>(&ks_lds[buf][((kb * 4 + s) * 64 + lane) * 8]);
#pragma unroll
        for (int t = 0; t < QB; ++t)
          s4[t][kb] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a, bq[t][s], s4[t][kb], 0, 0, 0);
      }
    // s4[t][kb][e] = score of key c0 + 16 kb + 4 g + e for query row 16 rb + j
    Pack8 pb[QB][2];
#pragma unroll
    for (int t = 0; t < QB; ++t) {
      const bool need_mask = c0 + kChunk - 1 > lim_min[t];  // same for the whole wavefront
      float mx = -INFINITY;
#pragma unroll
      for (int kb = 0; kb < 4; ++kb)
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          float sv = s4[t][kb][e] * scale_log2;
          if (need_mask && c0 + kb * 16 + 4 * g + e > limit[t]) sv = -INFINITY;
          s4[t][kb][e] = sv;
          mx = fmaxf(mx, sv);
        }
      mx = fmaxf(mx, __shfl_xor(mx, 16));
      mx = fmaxf(mx, __shfl_xor(mx, 32));
      const float m_new = fmaxf(m_run[t], mx);
      const float m_use = (m_new == -INFINITY) ? 0.f : m_new;
      const float alpha = __builtin_amdgcn_exp2f(m_run[t] - m_use);
      float psum = 0.f;
#pragma unroll
      for (int kb = 0; kb < 4; ++kb)
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const float p = __builtin_amdgcn_exp2f(s4[t][kb][e] - m_use);
          psum += p;
          pb[t][kb >> 1].h[(kb & 1) * 4 + e] = float_to_half_bits(p);
        }
      l_run[t] = l_run[t] * alpha + psum;
      m_run[t] = m_new;
      if (__builtin_amdgcn_ballot_w64(alpha != 1.0f)) {  // the running maximum moved somewhere in the wavefront
#pragma unroll
        for (int d = 0; d < 8; ++d) o[t][d] *= alpha;
      }
    }
#pragma unroll
    for (int t2 = 0; t2 < 2; ++t2)
#pragma unroll
      for (int d = 0; d < 8; ++d) {
        const f16x8 a = *reinterpret_cast<const f16x8*>(&vs_lds[buf][((d * 2 + t2) * 64 + lane) * 8]);
#pragma unroll
        for (int t = 0; t < QB; ++t)
          o[t][d] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a, pb[t][t2].v, o[t][d], 0, 0, 0);
      }
    __builtin_amdgcn_sched_barrier(0);
    store_chunk(c_next, buf ^ 1);  // the other buffer: nobody reads it until the barrier below
    __syncthreads();
  }

#pragma unroll
  for (int t = 0; t < QB; ++t) {
    float l = l_run[t];
    l += __shfl_xor(l, 16);
    l += __shfl_xor(l, 32);
    const int r = rb[t] * 16 + j;
    if (!valid[t] || r >= rows) continue;  // padding rows are never merged
    const size_t row = ((size_t)split * n_q + head[t]) * rows_stride + r;
#pragma unroll
    for (int d = 0; d < 8; ++d)
      *reinterpret_cast<float4*>(part_o + row * kHd + d * 16 + 4 * g) =
          make_float4(o[t][d][0], o[t][d][1], o[t][d][2], o[t][d][3]);
    // the merge works in natural-log units
    if (g == 0) *reinterpret_cast<float2*>(part_ml + row * 2) = make_float2(m_run[t] * 0.6931471805599453f, l);
  }
}

// float32 parity mode.  grid (n_split, n_q); each wavefront walks rows r = wave, wave + 4, ...
__global__ __launch_bounds__(256) void attn_f32_kernel(const float* __restrict__ q, const float* __restrict__ kc,
                                                       const float* __restrict__ vc, int rows, int rows_stride,
                                                       int n_causal, int pos0, int n_keys, int n_q, int n_kv,
                                                       int hd, int cap, int chunks_per_split, float scale,
                                                       float* __restrict__ part_o, float* __restrict__ part_ml) {
  __shared__ float qbuf[4][128];
  __shared__ float pbuf[4][kChunk];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int split = blockIdx.x, head = blockIdx.y;
  const int kvh = head / (n_q / n_kv);
  const int n_chunks = (n_keys + kChunk - 1) / kChunk;
  const int c_begin = split * chunks_per_split;
  int c_end = c_begin + chunks_per_split;
  if (c_end > n_chunks) c_end = n_chunks;
  const float* kh = kc + (size_t)kvh * cap * hd;
  const float* vh = vc + (size_t)kvh * cap * hd;

  for (int r = wave; r < rows; r += 4) {
    const float* qr = q + ((size_t)head * rows_stride + r) * hd;
    for (int d = lane; d < hd; d += 64) qbuf[wave][d] = qr[d];
    __builtin_amdgcn_wave_barrier();
    const int limit = (r >= n_causal) ? n_keys - 1 : pos0 + r;
    float m_run = -INFINITY, l_run = 0.f, o0 = 0.f, o1 = 0.f;
    for (int c = c_begin; c < c_end; ++c) {
      const int key = c * kChunk + lane;
      float s = -INFINITY;
      if (key < n_keys && key <= limit) {
        const float* kr = kh + (size_t)key * hd;
        float acc = 0.f;
        for (int d = 0; d < hd; ++d) acc = fmaf(qbuf[wave][d], kr[d], acc);
        s = acc * scale;
      }
      float mx = s;
#pragma unroll
      for (int off = 32; off > 0; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off));
      const float m_new = fmaxf(m_run, mx);
      const float m_use = (m_new == -INFINITY) ? 0.f : m_new;
      const float alpha = expf(m_run - m_use);
      const float p = expf(s - m_use);
      float ps = p;
#pragma unroll
      for (int off = 32; off > 0; off >>= 1) ps += __shfl_xor(ps, off);
      l_run = l_run * alpha + ps;
      m_run = m_new;
      pbuf[wave][lane] = p;
      __builtin_amdgcn_wave_barrier();
      o0 *= alpha;
      o1 *= alpha;
      const int kmax = min(kChunk, n_keys - c * kChunk);
      for (int jj = 0; jj < kmax; ++jj) {
        const float pj = pbuf[wave][jj];
        const float* vr = vh + (size_t)(c * kChunk + jj) * hd;
        if (lane < hd) o0 = fmaf(pj, vr[lane], o0);
        if (lane + 64 < hd) o1 = fmaf(pj, vr[lane + 64], o1);
      }
      __builtin_amdgcn_wave_barrier();
    }
    const size_t row = ((size_t)split * n_q + head) * rows_stride + r;
    if (lane < hd) part_o[row * hd + lane] = o0;
    if (lane + 64 < hd) part_o[row * hd + lane + 64] = o1;
    if (lane == 0) {
      part_ml[row * 2 + 0] = m_run;
      part_ml[row * 2 + 1] = l_run;
    }
  }
}

// Exact merge of the per-split partial results: out = sum_s o_s e^(m_s - M) / sum_s l_s e^(m_s - M).
// One workgroup per (row, head), one thread per output column; loops are unrolled so that the loads of
// several splits are in flight together.
template <typename T>
__global__ void attn_merge_kernel(SeqTable tab, const float* __restrict__ part_o, const float* __restrict__ part_ml,
                                  int n_split, int n_q, int rows_pad, int hd, T* __restrict__ att,
                                  uint32_t* __restrict__ ovf) {
  // att: GEMM input [rows_pad, n_q * hd] of the output projection.  n_split: the largest split count among the
  // call's sequences (a sequence with fewer keys has left empty partials, weight zero, in the others).
  const int r = blockIdx.x, head = blockIdx.y, d = threadIdx.x;
  if (d >= hd) return;
  if (seq_of_row(tab, r) < 0) {  // padding row between two sequences: no partials exist; keep the row finite
    Act<T>::put(att, r, head * hd + d, n_q * hd, 0.f, nullptr);
    return;
  }
  const size_t stride = (size_t)n_q * rows_pad;           // rows between consecutive splits
  const size_t row0 = (size_t)head * rows_pad + r;
  float mx = -INFINITY;
#pragma unroll 8
  for (int s = 0; s < n_split; ++s) mx = fmaxf(mx, part_ml[(row0 + s * stride) * 2]);
  float num = 0.f, den = 0.f;
#pragma unroll 8
  for (int s = 0; s < n_split; ++s) {
    const size_t row = row0 + s * stride;
    const float m = part_ml[row * 2], l = part_ml[row * 2 + 1];
    const float o = part_o[row * hd + d];
    const float w = (m == -INFINITY) ? 0.f : expf(m - mx);
    num += o * w;
    den += l * w;
  }
  Act<T>::put(att, r, head * hd + d, n_q * hd, num / den, ovf);
}

}  // namespace

// Split plan over the key axis.  The split boundaries depend on the cache CAPACITY only (split s always
// covers the same absolute key positions), never on how many keys or query rows a call has.  Masked keys
// contribute exact zeros, empty splits merge with weight zero, and every other kernel of the forward works
// row by row in a fixed order, so the result of a query row is bit-identical whether the row is computed
// alone (one-token decoding) or inside a block (parallel verification): greedy verification then
// reproduces the target's own greedy stream exactly, not just up to rounding.
// Half-precision kernel: at most 32 splits over the capacity, at least two 64-key chunks per split.
// float32 kernel: at most 16 splits.
constexpr int kMaxSplitsF16 = 32, kMaxSplitsF32 = 16;

// Rows-equivalents of partial results the workspace holds for a call with rows_pad padded rows.
int attn_partial_rows(int rows_pad) { return kMaxSplitsF16 * rows_pad; }

AttnPlan attn_plan(int dtype, int cap, int n_keys) {
  const int cap_chunks = ceil_div(cap, kChunk), n_chunks = ceil_div(n_keys, kChunk);
  AttnPlan p;
  if (dtype == DS_BF16) {
    p.chunks_per_split = ceil_div(cap_chunks, kMaxSplitsF16);
    if (p.chunks_per_split < 2) p.chunks_per_split = 2;
  } else {
    p.chunks_per_split = ceil_div(cap_chunks, kMaxSplitsF32);
  }
  p.n_split = ceil_div(n_chunks, p.chunks_per_split);
  return p;
}

int launch_attention(int dtype, const SeqTable& tab, const void* q, int rows, int rows_pad, int n_q, int n_kv, int hd,
                     int cap, float* part_o, float* part_ml, void* att_out, uint32_t* ovf, hipStream_t st) {
  const float scale = 1.0f / sqrtf((float)hd);
  DS_REQUIRE(tab.n_seq >= 1 && tab.n_seq <= kMaxSeq, DS_E_SHAPE, "attention: %d sequences outside [1, %d]", tab.n_seq,
             kMaxSeq);
  if (dtype == DS_BF16) {
    DS_REQUIRE(hd == kHd, DS_E_UNSUPPORTED, "bf16 attention needs head_dim 128 (got %d)", hd);
    DS_REQUIRE(cap % kChunk == 0, DS_E_SHAPE, "bf16 attention needs a cache capacity that is a multiple of %d", kChunk);
  } else {
    DS_REQUIRE(hd <= 128 && (hd & 1) == 0, DS_E_UNSUPPORTED, "f32 attention needs even head_dim <= 128 (got %d)", hd);
  }
  // every sequence runs the split plan of its own key count; the merge walks the largest split count, so each
  // sequence's launch covers that many splits (the ones past its keys leave empty partials)
  int n_split_max = 1;
  for (int s = 0; s < tab.n_seq; ++s) {
    const int n_keys = tab.pos0[s] + tab.n_rows[s];
    DS_REQUIRE(tab.n_rows[s] >= 1 && (tab.row0[s] & 15) == 0 && tab.row0[s] + tab.n_rows[s] <= rows, DS_E_SHAPE,
               "attention: sequence %d has a bad row range", s);
    DS_REQUIRE(n_keys >= 1 && n_keys <= cap, DS_E_CAPACITY, "attention: %d keys exceed the cache capacity %d", n_keys, cap);
    const AttnPlan plan = attn_plan(dtype, cap, n_keys);
    n_split_max = plan.n_split > n_split_max ? plan.n_split : n_split_max;
  }
  DS_REQUIRE(n_split_max * rows_pad <= attn_partial_rows(rows_pad), DS_E_CAPACITY,
             "attention partials: %d splits x %d rows exceed the workspace", n_split_max, rows_pad);
  for (int s = 0; s < tab.n_seq; ++s) {
    const int n_keys = tab.pos0[s] + tab.n_rows[s], r0 = tab.row0[s], sr = tab.n_rows[s];
    const int srp = ceil_div(sr, 16) * 16;
    const AttnPlan plan = attn_plan(dtype, cap, n_keys);
    if (dtype == DS_BF16) {
      const int n_qb = (n_q / n_kv) * (srp >> 4);
      constexpr int QB = 2;
      dim3 grid(n_split_max, n_kv, ceil_div(n_qb, 4 * QB));
      hipLaunchKernelGGL((attn_f16_kernel<QB>), grid, dim3(256), 0, st,
                         static_cast<const uint16_t*>(q) + (size_t)(r0 >> 4) * 4 * 512,
                         static_cast<const uint16_t*>(tab.kc[s]), static_cast<const uint16_t*>(tab.vc[s]), sr, srp,
                         rows_pad, tab.n_causal[s], tab.pos0[s], n_keys, n_q, n_kv, cap, plan.chunks_per_split,
                         scale * 1.4426950408889634f, part_o + (size_t)r0 * kHd, part_ml + (size_t)r0 * 2);
      DS_LAUNCH_CHECK("attn_f16_kernel");
    } else {
      hipLaunchKernelGGL(attn_f32_kernel, dim3(n_split_max, n_q), dim3(256), 0, st,
                         static_cast<const float*>(q) + (size_t)r0 * hd, static_cast<const float*>(tab.kc[s]),
                         static_cast<const float*>(tab.vc[s]), sr, rows_pad, tab.n_causal[s], tab.pos0[s], n_keys, n_q,
                         n_kv, hd, cap, plan.chunks_per_split, scale, part_o + (size_t)r0 * hd,
                         part_ml + (size_t)r0 * 2);
      DS_LAUNCH_CHECK("attn_f32_kernel");
    }
  }
  if (dtype == DS_BF16)
    hipLaunchKernelGGL((attn_merge_kernel<bf16_t>), dim3(rows, n_q), dim3(hd), 0, st, tab, part_o, part_ml, n_split_max,
                       n_q, rows_pad, hd, static_cast<bf16_t*>(att_out), ovf);
  else
    hipLaunchKernelGGL((attn_merge_kernel<float>), dim3(rows, n_q), dim3(hd), 0, st, tab, part_o, part_ml, n_split_max,
                       n_q, rows_pad, hd, static_cast<float*>(att_out), ovf);
  DS_LAUNCH_CHECK("attn_merge_kernel");
  return DS_OK;
}

}  // namespace ds
