// Row-wise kernels between the GEMMs: token gather, RMSNorm, split-K reduction with residual add,
// rotary embedding with KV-cache append, SwiGLU.  Each one also performs the deterministic
// (fixed-order) sum of the GEMM's split-K partial planes, so no separate reduction pass exists.
//
// The residual stream x stays float32 [rows, d_model].  Activations that feed a GEMM are written in
// the model's storage form: IEEE half in tile order, or float32 row-major.
#include <math.h>

#include "ds_act.h"
#include "ds_common.h"

namespace ds {
namespace {

// Sum over the workgroup (THREADS / 64 wavefronts), same value and same summation order in every thread.
template <int THREADS>
__device__ __forceinline__ float block_sum(float v, float* red) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off);
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  __syncthreads();
  if (lane == 0) red[wave] = v;
  __syncthreads();
  float s = 0.f;
#pragma unroll
  for (int w = 0; w < THREADS / 64; ++w) s += red[w];
  return s;
}

constexpr int kMaxPlanes = 10;  // split-K planes summed per element (gemm_bf16_splits never exceeds it)

// Token and rotary arguments of the first kernel of a forward (FROM_EMBED).  Row i of sequence s reads its token
// from tok_a[off_a[s] + i] if i < n_a[s], else from tok_b[off_b[s] + i - n_a[s]] (or is `fill` if tok_b is NULL); ids
// outside [0, vocab) read as 0, and so do the padding rows between sequences (position 0).
struct Prologue {
  const int32_t* tok_a;
  const int32_t* tok_b;
  int vocab;
  int32_t fill;
  int half;            // rotary table: cs[r][i] = (cos, sin)(position(r) * base^(-i / half)), i < half
  double log2_base;
  float2* cs;
};

// x[r] = E[tok[r]] or x[r] + sum of split-K planes ; h[r] = rmsnorm(x[r]) * gain, written as GEMM input.
// FROM_EMBED: start from the embedding row (and fill this row of the rotary table, angles in double so
// that long contexts stay exact), else from the float32 residual x plus `n_part` planes.
// rm_out (optional): row-major float32 copy of the rows each sequence hands on (the boundary's hidden_out: rows
// tail0 .. of every sequence, compacted in sequence order); h_tail (optional): the same rows once more as a GEMM
// input (what the LM head multiplies).
// One workgroup per row (1024 threads for wide models so that every load of the row is issued at once),
// four consecutive columns per thread and step (d_model % 4 == 0); the planes
// are summed in index order, all loads of a step issued before the first add.
template <typename T, bool FROM_EMBED, int THREADS>
__global__ __launch_bounds__(THREADS) void norm_kernel(Prologue pro, SeqTable tab, const T* __restrict__ embed,
                                                   float* __restrict__ x, const float* __restrict__ part,
                                                   int n_part, int rows, int rows_pad, int d,
                                                   const float* __restrict__ gain, float eps, T* __restrict__ h,
                                                   float* __restrict__ rm_out, T* __restrict__ h_tail,
                                                   uint32_t* __restrict__ ovf) {
  constexpr int kMaxVec = 8192 / (4 * THREADS);  // float4 groups per thread (d_model <= 8192)
  __shared__ float red[THREADS / 64];
  const int r = blockIdx.x;
  const int sq = seq_of_row(tab, r);
  const int ri = sq >= 0 ? r - tab.row0[sq] : 0;  // row within its sequence
  int token = 0;
  if (FROM_EMBED) {
    int pos = 0;
    if (sq >= 0) {
      pos = tab.pos0[sq] + ri;
      token = ri < tab.n_a[sq] ? pro.tok_a[tab.off_a[sq] + ri]
                               : (pro.tok_b ? pro.tok_b[tab.off_b[sq] + ri - tab.n_a[sq]] : pro.fill);
      token = (token < 0 || token >= pro.vocab) ? 0 : token;
    }
    if ((int)threadIdx.x < pro.half) {
      const double theta = exp2(-((double)threadIdx.x / (double)pro.half) * pro.log2_base);
      double sn, cs;
      sincos((double)pos * theta, &sn, &cs);
      pro.cs[r * pro.half + threadIdx.x] = make_float2((float)cs, (float)sn);
    }
  }
  // rows handed on (rm_out / h_tail): rows ri >= tail0 of each sequence, compacted to tail_base + (ri - tail0)
  const bool is_tail = sq >= 0 && ri >= tab.tail0[sq];
  const int tail_row = is_tail ? tab.tail_base[sq] + ri - tab.tail0[sq] : 0;
  float4 v[kMaxVec];
  float ss = 0.f;
#pragma unroll
  for (int i = 0; i < kMaxVec; ++i) {
    const int c = (threadIdx.x + i * THREADS) * 4;
    v[i] = make_float4(0.f, 0.f, 0.f, 0.f);
    if (c < d) {
      float4 a;
      if (FROM_EMBED) {
        const T* e = embed + (size_t)token * d + c;
        a = make_float4(Act<T>::weight(e[0]), Act<T>::weight(e[1]), Act<T>::weight(e[2]), Act<T>::weight(e[3]));
      } else {
        a = *reinterpret_cast<const float4*>(x + (size_t)r * d + c);
        float4 p[kMaxPlanes];
#pragma unroll
        for (int s = 0; s < kMaxPlanes; ++s)
          p[s] = s < n_part ? *reinterpret_cast<const float4*>(part + ((size_t)s * rows + r) * d + c)
                            : make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
        for (int s = 0; s < kMaxPlanes; ++s) {
          a.x += p[s].x; a.y += p[s].y; a.z += p[s].z; a.w += p[s].w;
        }
      }
      *reinterpret_cast<float4*>(x + (size_t)r * d + c) = a;
      v[i] = a;
      ss += (a.x * a.x + a.y * a.y) + (a.z * a.z + a.w * a.w);
    }
  }
  ss = block_sum<THREADS>(ss, red);
  const float inv = 1.0f / sqrtf(ss / (float)d + eps);
#pragma unroll
  for (int i = 0; i < kMaxVec; ++i) {
    const int c = (threadIdx.x + i * THREADS) * 4;
    if (c < d) {
      const float4 gn = *reinterpret_cast<const float4*>(gain + c);
      const float4 y = make_float4(v[i].x * inv * gn.x, v[i].y * inv * gn.y, v[i].z * inv * gn.z, v[i].w * inv * gn.w);
      Act<T>::put4(h, r, c, d, y, ovf);
      if (rm_out && is_tail) *reinterpret_cast<float4*>(rm_out + (size_t)tail_row * d + c) = y;
      if (h_tail && is_tail) Act<T>::put4(h_tail, tail_row, c, d, y, nullptr);
    }
  }
}

// Row-major float32 hidden states [rows, d] -> GEMM input order.
template <typename T>
__global__ void to_gemm_input_kernel(const float* __restrict__ src, int rows_pad, int d, T* __restrict__ dst,
                                     uint32_t* __restrict__ ovf) {
  const int r = blockIdx.x;
  for (int c = threadIdx.x * 4; c < d; c += blockDim.x * 4)
    Act<T>::put4(dst, r, c, d, *reinterpret_cast<const float4*>(src + (size_t)r * d + c), ovf);
}

// One wavefront per (row, head slot): sums the QKV partial planes, rotates q and k, writes q in the
// attention kernel's order and appends k, v to the cache at position pos0 + row.
// Head slots: [0, n_q) queries, [n_q, n_q + n_kv) keys, then values.
template <typename T>
__global__ void qkv_rope_kernel(const float* __restrict__ part, int n_part, int rows, int rows_pad, int n_q,
                                int n_kv, int hd, const float2* __restrict__ cs, SeqTable tab, int cap, float q_scale,
                                typename Act<T>::kv_t* __restrict__ q, uint32_t* __restrict__ ovf) {
  using KV = typename Act<T>::kv_t;
  const int r = blockIdx.x, slot = blockIdx.y, i = threadIdx.x, half = hd >> 1;
  if (i >= half) return;
  const int sq = seq_of_row(tab, r);
  if (sq < 0 && slot >= n_q) return;  // a padding row has no place in any cache (its q stays finite and unused)
  KV* kc = sq >= 0 ? static_cast<KV*>(tab.kc[sq]) : nullptr;
  KV* vc = sq >= 0 ? static_cast<KV*>(tab.vc[sq]) : nullptr;
  const int pos0 = sq >= 0 ? tab.pos0[sq] - tab.row0[sq] : 0;  // position of row r = pos0 + r
  const int n_tot = (n_q + 2 * n_kv) * hd;
  // all planes' loads are issued before the first add (one memory round trip instead of n_part); the sum keeps
  // the plane order
  float pa[kMaxPlanes], pb[kMaxPlanes];
#pragma unroll
  for (int s = 0; s < kMaxPlanes; ++s) {
    pa[s] = pb[s] = 0.f;
    if (s < n_part) {
      const float* p = part + ((size_t)s * rows + r) * n_tot + (size_t)slot * hd;
      pa[s] = p[i];
      pb[s] = p[i + half];
    }
  }
  float a = 0.f, b = 0.f;
#pragma unroll
  for (int s = 0; s < kMaxPlanes; ++s)
    if (s < n_part) {
      a += pa[s];
      b += pb[s];
    }
  if (slot < n_q + n_kv) {
    const float2 t = cs[r * half + i];
    const float ra = a * t.x - b * t.y;
    const float rb = b * t.x + a * t.y;
    a = ra;
    b = rb;
  }
  const int pos = pos0 + r;
  if (slot < n_q) {
    KV* qh = q + (size_t)slot * rows_pad * hd;
    // the attention kernel's score scale goes into the queries before their one rounding
    qh[Act<T>::q_off(r, i, hd)] = Act<T>::to_kv(a * q_scale, ovf);
    qh[Act<T>::q_off(r, i + half, hd)] = Act<T>::to_kv(b * q_scale, ovf);
  } else if (slot < n_q + n_kv) {
    if (Act<T>::kTiledKV) {
      KV* kh = kc + (size_t)(slot - n_q) * cap * hd;
      kh[kv_k_offset(pos, i)] = Act<T>::to_kv(a, ovf);
      kh[kv_k_offset(pos, i + half)] = Act<T>::to_kv(b, ovf);
    } else {
      KV* kh = kc + ((size_t)(slot - n_q) * cap + pos) * hd;
      kh[i] = Act<T>::to_kv(a, ovf);
      kh[i + half] = Act<T>::to_kv(b, ovf);
    }
  } else {
    const int kvh = slot - n_q - n_kv;
    if (Act<T>::kTiledKV) {
      KV* vh = vc + (size_t)kvh * cap * hd;
      vh[kv_v_offset(pos, i)] = Act<T>::to_kv(a, ovf);
      vh[kv_v_offset(pos, i + half)] = Act<T>::to_kv(b, ovf);
    } else {
      KV* vh = vc + ((size_t)kvh * cap + pos) * hd;
      vh[i] = Act<T>::to_kv(a, ovf);
      vh[i + half] = Act<T>::to_kv(b, ovf);
    }
  }
}

// act[r][f] = silu(gate) * up with gate = sum_s part[s][r][f], up = sum_s part[s][r][F + f]; four
// consecutive f per thread (F % 4 == 0).
template <typename T>
__global__ void swiglu_kernel(const float* __restrict__ part, int n_part, int rows, int rows_pad, int F,
                              T* __restrict__ act, uint32_t* __restrict__ ovf) {
  const int r = blockIdx.y;
  const int f = (blockIdx.x * blockDim.x + threadIdx.x) * 4;
  if (f >= F) return;
  // all planes' loads first, then the sums in plane order
  float4 pg[kMaxPlanes], pu[kMaxPlanes];
#pragma unroll
  for (int s = 0; s < kMaxPlanes; ++s) {
    pg[s] = pu[s] = make_float4(0.f, 0.f, 0.f, 0.f);
    if (s < n_part) {
      const float* p = part + ((size_t)s * rows + r) * (2 * (size_t)F);
      pg[s] = *reinterpret_cast<const float4*>(p + f);
      pu[s] = *reinterpret_cast<const float4*>(p + F + f);
    }
  }
  float4 g = make_float4(0.f, 0.f, 0.f, 0.f), u = g;
#pragma unroll
  for (int s = 0; s < kMaxPlanes; ++s)
    if (s < n_part) {
      g.x += pg[s].x; g.y += pg[s].y; g.z += pg[s].z; g.w += pg[s].w;
      u.x += pu[s].x; u.y += pu[s].y; u.z += pu[s].z; u.w += pu[s].w;
    }
  const float4 y = make_float4(g.x / (1.0f + expf(-g.x)) * u.x, g.y / (1.0f + expf(-g.y)) * u.y,
                               g.z / (1.0f + expf(-g.z)) * u.z, g.w / (1.0f + expf(-g.w)) * u.w);
  Act<T>::put4(act, r, f, F, y, ovf);
}

// The same for a product whose columns alternate between 16 of gate and 16 of up (the weights were packed as a pair):
// gate f sits at column 32 (f / 16) + f % 16, up f sixteen further.  A thread sums four consecutive columns of the
// product (a wavefront reads 1 KB in one piece); the four lanes of a gate group take their up values from the four
// lanes after them (F % 128 == 0: a group of 32 columns never straddles the end of the row).
template <typename T>
__global__ void swiglu_paired_kernel(const float* __restrict__ part, int n_part, int rows, int rows_pad, int F,
                                     T* __restrict__ act, uint32_t* __restrict__ ovf) {
  const int r = blockIdx.y;
  const int col = (blockIdx.x * blockDim.x + threadIdx.x) * 4;
  const bool inside = col < 2 * F;  // whole groups of 32 columns are inside or outside together
  float4 pv[kMaxPlanes];
#pragma unroll
  for (int s = 0; s < kMaxPlanes; ++s) {
    pv[s] = make_float4(0.f, 0.f, 0.f, 0.f);
    if (s < n_part && inside)
      pv[s] = *reinterpret_cast<const float4*>(part + ((size_t)s * rows + r) * (2 * (size_t)F) + col);
  }
  float4 x = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
  for (int s = 0; s < kMaxPlanes; ++s)
    if (s < n_part) {
      x.x += pv[s].x; x.y += pv[s].y; x.z += pv[s].z; x.w += pv[s].w;
    }
  const float4 u = make_float4(__shfl_down(x.x, 4), __shfl_down(x.y, 4), __shfl_down(x.z, 4), __shfl_down(x.w, 4));
  if (inside && (col & 16) == 0) {
    const int f = ((col >> 5) << 4) + (col & 15);
    const float4 y = make_float4(x.x / (1.0f + expf(-x.x)) * u.x, x.y / (1.0f + expf(-x.y)) * u.y,
                                 x.z / (1.0f + expf(-x.z)) * u.z, x.w / (1.0f + expf(-x.w)) * u.w);
    Act<T>::put4(act, r, f, F, y, ovf);
  }
}

}  // namespace

template <typename T>
int launch_embed_norm(const SeqTable& tab, const int32_t* tok_a, const int32_t* tok_b, int32_t fill, int vocab, int hd,
                      double rope_base, float2* cs, const void* embed, float* x, int rows, int rows_pad, int d,
                      const float* gain, float eps, void* h, uint32_t* ovf, hipStream_t st) {
  Prologue pro{tok_a, tok_b, vocab, fill, hd / 2, log2(rope_base), cs};
  if (d >= 2048)
    hipLaunchKernelGGL((norm_kernel<T, true, 1024>), dim3(rows), dim3(1024), 0, st, pro, tab,
                       static_cast<const T*>(embed), x, (const float*)nullptr, 0, rows, rows_pad, d, gain, eps,
                       static_cast<T*>(h), (float*)nullptr, (T*)nullptr, ovf);
  else
    hipLaunchKernelGGL((norm_kernel<T, true, 256>), dim3(rows), dim3(256), 0, st, pro, tab,
                       static_cast<const T*>(embed), x, (const float*)nullptr, 0, rows, rows_pad, d, gain, eps,
                       static_cast<T*>(h), (float*)nullptr, (T*)nullptr, ovf);
  DS_LAUNCH_CHECK("norm_kernel<embed>");
  return DS_OK;
}

template <typename T>
int launch_add_norm(const SeqTable& tab, float* x, const float* part, int n_part, int rows, int rows_pad, int d,
                    const float* gain, float eps, void* h, float* rm_out, void* h_tail, uint32_t* ovf,
                    hipStream_t st) {
  DS_REQUIRE(n_part >= 0 && n_part <= kMaxPlanes, DS_E_SHAPE, "norm: %d partial planes, at most %d", n_part, kMaxPlanes);
  if (d >= 2048)
    hipLaunchKernelGGL((norm_kernel<T, false, 1024>), dim3(rows), dim3(1024), 0, st, Prologue{}, tab,
                       (const T*)nullptr, x, part, n_part, rows, rows_pad, d, gain, eps, static_cast<T*>(h), rm_out,
                       static_cast<T*>(h_tail), ovf);
  else
    hipLaunchKernelGGL((norm_kernel<T, false, 256>), dim3(rows), dim3(256), 0, st, Prologue{}, tab,
                       (const T*)nullptr, x, part, n_part, rows, rows_pad, d, gain, eps, static_cast<T*>(h), rm_out,
                       static_cast<T*>(h_tail), ovf);
  DS_LAUNCH_CHECK("norm_kernel<add>");
  return DS_OK;
}

template <typename T>
int launch_to_gemm_input(const float* src, int rows, int rows_pad, int d, void* dst, uint32_t* ovf, hipStream_t st) {
  hipLaunchKernelGGL((to_gemm_input_kernel<T>), dim3(rows), dim3(256), 0, st, src, rows_pad, d,
                     static_cast<T*>(dst), ovf);
  DS_LAUNCH_CHECK("to_gemm_input_kernel");
  return DS_OK;
}

template <typename T>
int launch_qkv_rope(const SeqTable& tab, const float* part, int n_part, int rows, int rows_pad, int n_q, int n_kv,
                    int hd, const float2* cs, int cap, float q_scale, void* q, uint32_t* ovf, hipStream_t st) {
  DS_REQUIRE(n_part >= 1 && n_part <= kMaxPlanes, DS_E_SHAPE, "rope: %d partial planes, at most %d", n_part, kMaxPlanes);
  hipLaunchKernelGGL((qkv_rope_kernel<T>), dim3(rows, n_q + 2 * n_kv), dim3(hd / 2), 0, st, part, n_part, rows,
                     rows_pad, n_q, n_kv, hd, cs, tab, cap, q_scale, static_cast<typename Act<T>::kv_t*>(q), ovf);
  DS_LAUNCH_CHECK("qkv_rope_kernel");
  return DS_OK;
}

template <typename T>
int launch_swiglu(const float* part, int n_part, int rows, int rows_pad, int F, bool paired, void* act, uint32_t* ovf,
                  hipStream_t st) {
  DS_REQUIRE(n_part >= 1 && n_part <= kMaxPlanes, DS_E_SHAPE, "SwiGLU: %d partial planes, at most %d", n_part, kMaxPlanes);
  if (paired) {
    DS_REQUIRE((F & 127) == 0, DS_E_SHAPE, "SwiGLU: a paired product needs F %% 128 == 0");
    hipLaunchKernelGGL((swiglu_paired_kernel<T>), dim3(ceil_div(2 * F, 1024), rows), dim3(256), 0, st, part, n_part,
                       rows, rows_pad, F, static_cast<T*>(act), ovf);
    DS_LAUNCH_CHECK("swiglu_paired_kernel");
    return DS_OK;
  }
  hipLaunchKernelGGL((swiglu_kernel<T>), dim3(ceil_div(F, 1024), rows), dim3(256), 0, st, part, n_part, rows,
                     rows_pad, F, static_cast<T*>(act), ovf);
  DS_LAUNCH_CHECK("swiglu_kernel");
  return DS_OK;
}

#define DS_INSTANTIATE(T)                                                                                          \
  template int launch_embed_norm<T>(const SeqTable&, const int32_t*, const int32_t*, int32_t, int, int, double,    \
                                    float2*, const void*, float*, int, int, int, const float*, float, void*,       \
                                    uint32_t*, hipStream_t);                                                       \
  template int launch_add_norm<T>(const SeqTable&, float*, const float*, int, int, int, int, const float*, float, \
                                  void*, float*, void*, uint32_t*, hipStream_t);                                   \
  template int launch_to_gemm_input<T>(const float*, int, int, int, void*, uint32_t*, hipStream_t);                \
  template int launch_qkv_rope<T>(const SeqTable&, const float*, int, int, int, int, int, int, const float2*, int, float, \
                                  void*, uint32_t*, hipStream_t);                                                  \
  template int launch_swiglu<T>(const float*, int, int, int, int, bool, void*, uint32_t*, hipStream_t);
DS_INSTANTIATE(float)
DS_INSTANTIATE(bf16_t)

}  // namespace ds
