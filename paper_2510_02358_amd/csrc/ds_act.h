// Storage-type traits.
//
// DS_F32 (parity mode): everything float32, row-major.
// DS_BF16: weights bf16.  An activation that feeds a GEMM is kept as a PAIR of bf16 planes
//   hi = bf16(x), lo = bf16(x - hi), both in tile order (xt_offset); the GEMM multiplies the bf16
//   weights with both planes and accumulates in float32, so the activation keeps ~16 mantissa bits
//   while every matrix-core product is still bf16 x bf16.  Queries, keys, values and attention
//   probabilities are IEEE half (11 mantissa bits, 2 bytes like bf16): with N(0, 0.02) random-init
//   weights the residual stream is ~0.03 rms, the RMSNorm after attention amplifies any error of
//   the attention output ~30x, and a bf16 KV cache alone would consume the whole 2e-2 logit budget.
#pragma once

#include "ds_common.h"

namespace ds {

struct bf16_t {
  uint16_t bits;
};

__device__ __forceinline__ float bf16_bits_to_float(uint16_t b) { return __uint_as_float((uint32_t)b << 16); }

// round to nearest, ties to even (NaN kept quiet)
__device__ __forceinline__ uint16_t float_to_bf16_bits(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (uint16_t)((u >> 16) | 0x40u);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}

__device__ __forceinline__ uint16_t float_to_half_bits(float f) {
  _Float16 h = (_Float16)f;  // round to nearest even
  return __builtin_bit_cast(uint16_t, h);
}

template <typename T>
struct Act;

template <>
struct Act<float> {
  using kv_t = float;                         // element type of q / K cache / V cache
  static constexpr bool kTransposedV = false;
  static constexpr int kPlanes = 1;
  // GEMM-input store: element (m, k) of a [rows_pad, K] activation
  __device__ static __forceinline__ void put(float* base, int m, int k, int K, size_t /*plane*/, float v) {
    base[(size_t)m * K + k] = v;
  }
  // four consecutive columns k .. k+3 (k % 4 == 0)
  __device__ static __forceinline__ void put4(float* base, int m, int k, int K, size_t /*plane*/, float4 v) {
    *reinterpret_cast<float4*>(base + (size_t)m * K + k) = v;
  }
  __device__ static __forceinline__ size_t q_off(int m, int k, int K) { return (size_t)m * K + k; }
  __device__ static __forceinline__ float to_kv(float v) { return v; }
  __device__ static __forceinline__ float weight(float v) { return v; }
};

template <>
struct Act<bf16_t> {
  using kv_t = uint16_t;                      // IEEE half bits
  static constexpr bool kTransposedV = true;  // V cache kept as [head_dim][capacity] per head
  static constexpr int kPlanes = 2;
  __device__ static __forceinline__ void put(bf16_t* base, int m, int k, int K, size_t plane, float v) {
    const size_t off = xt_offset(m, k, K);
    const uint16_t hi = float_to_bf16_bits(v);
    base[off].bits = hi;
    base[plane + off].bits = float_to_bf16_bits(v - bf16_bits_to_float(hi));
  }
  // four consecutive columns k .. k+3 (k % 4 == 0) are adjacent in tile order: one 8-byte store per plane
  __device__ static __forceinline__ void put4(bf16_t* base, int m, int k, int K, size_t plane, float4 v) {
    const size_t off = xt_offset(m, k, K);
    const float f[4] = {v.x, v.y, v.z, v.w};
    uint16_t hi[4], lo[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      hi[i] = float_to_bf16_bits(f[i]);
      lo[i] = float_to_bf16_bits(f[i] - bf16_bits_to_float(hi[i]));
    }
    *reinterpret_cast<uint2*>(base + off) = make_uint2(hi[0] | ((uint32_t)hi[1] << 16), hi[2] | ((uint32_t)hi[3] << 16));
    *reinterpret_cast<uint2*>(base + plane + off) =
        make_uint2(lo[0] | ((uint32_t)lo[1] << 16), lo[2] | ((uint32_t)lo[3] << 16));
  }
  __device__ static __forceinline__ size_t q_off(int m, int k, int K) { return xt_offset(m, k, K); }
  __device__ static __forceinline__ uint16_t to_kv(float v) { return float_to_half_bits(v); }
  __device__ static __forceinline__ float weight(bf16_t v) { return bf16_bits_to_float(v.bits); }
};

// ---- launchers implemented in k_elem.hip / k_gemm.hip / k_attn.hip --------------------------------
// First kernel of a forward: token gather (rows past n_real are `fill`), rotary table, embedding, RMSNorm.
template <typename T>
int launch_embed_norm(const int32_t* src, int n_real, int32_t fill, int vocab, int pos0, int hd, double rope_base,
                      float2* cs, const void* embed, float* x, int rows, int rows_pad, int d, const float* gain,
                      float eps, void* h, hipStream_t st);
template <typename T>
int launch_add_norm(float* x, const float* part, int n_part, int rows, int rows_pad, int d, const float* gain,
                    float eps, void* h, float* rm_out, int rm_row0, hipStream_t st);
template <typename T>
int launch_to_gemm_input(const float* src, int rows, int rows_pad, int d, void* dst, hipStream_t st);
template <typename T>
int launch_qkv_rope(const float* part, int n_part, int rows, int rows_pad, int n_q, int n_kv, int hd,
                    const float2* cs, int pos0, int cap, void* q, void* kc, void* vc, hipStream_t st);
template <typename T>
int launch_swiglu(const float* part, int n_part, int rows, int rows_pad, int F, void* act, hipStream_t st);

int launch_pack_weight(const void* w, int N, int K, void* dst, hipStream_t st);
int gemm_bf16_splits(int N, int K, int nbw);
int launch_gemm_bf16(const void* wp, const void* xt, int M, int N, int K, int nbw, int n_split, float* out,
                     hipStream_t st);
int launch_gemm_f32(const float* x, const float* w, int M, int N, int K, float* out, int ldc, hipStream_t st);

// Attention over keys [0, n_keys) of one layer's cache for `rows` query rows at positions pos0 + r.
// Row r sees key p iff r >= n_causal (a [MASK] row) or p <= pos0 + r.
int attn_splits(int dtype, int n_keys);
int attn_max_splits(int dtype, int capacity);
int launch_attention(int dtype, const void* q, const void* kc, const void* vc, int rows, int rows_pad, int n_causal,
                     int pos0, int n_keys, int n_q, int n_kv, int hd, int cap, int n_split, float* part_o,
                     float* part_ml, void* att_out, hipStream_t st);

}  // namespace ds
