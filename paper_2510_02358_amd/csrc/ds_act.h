// Storage-type traits for activations, weights and the KV cache: float32 (parity mode, row-major)
// or bf16 (bit patterns in uint16; GEMM inputs in tile order).
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

template <typename T>
struct Act;

template <>
struct Act<float> {
  static constexpr bool kTransposedV = false;
  __device__ static __forceinline__ size_t off(int m, int k, int K) { return (size_t)m * K + k; }
  __device__ static __forceinline__ float to_float(float v) { return v; }
  __device__ static __forceinline__ float from_float(float v) { return v; }
};

template <>
struct Act<bf16_t> {
  static constexpr bool kTransposedV = true;  // V cache kept as [head_dim][capacity] per head
  __device__ static __forceinline__ size_t off(int m, int k, int K) { return xt_offset(m, k, K); }
  __device__ static __forceinline__ float to_float(bf16_t v) { return bf16_bits_to_float(v.bits); }
  __device__ static __forceinline__ bf16_t from_float(float v) { return bf16_t{float_to_bf16_bits(v)}; }
};

// ---- launchers implemented in k_elem.hip / k_gemm.hip / k_attn.hip --------------------------------
int launch_tokens(const int32_t* src, int n_real, int rows, int32_t fill, int vocab, int32_t* tok, hipStream_t st);
int launch_rope_table(int pos0, int rows, int hd, double base, float2* cs, hipStream_t st);
template <typename T>
int launch_embed_norm(const int32_t* tok, const void* embed, float* x, int rows, int d, const float* gain, float eps,
                      void* h, hipStream_t st);
template <typename T>
int launch_add_norm(float* x, const float* part, int n_part, int rows, int d, const float* gain, float eps, void* h,
                    void* rm_out, int rm_row0, hipStream_t st);
template <typename T>
int launch_to_gemm_input(const void* src, int rows, int d, void* dst, hipStream_t st);
template <typename T>
int launch_qkv_rope(const float* part, int n_part, int rows, int rows_pad, int n_q, int n_kv, int hd,
                    const float2* cs, int pos0, int cap, void* q, void* kc, void* vc, hipStream_t st);
template <typename T>
int launch_swiglu(const float* part, int n_part, int rows, int F, void* act, hipStream_t st);

int launch_pack_weight(const void* w, int N, int K, void* dst, hipStream_t st);
int gemm_bf16_splits(int N, int K, int nbw);
int launch_gemm_bf16(const void* wp, const void* xt, int M, int N, int K, int nbw, int n_split, float* out,
                     hipStream_t st);
int launch_gemm_f32(const float* x, const float* w, int M, int N, int K, float* out, int ldc, hipStream_t st);

// Attention over keys [0, n_keys) of one layer's cache for `rows` query rows at positions pos0 + r.
// Row r sees key p iff r >= n_causal (a [MASK] row) or p <= pos0 + r.
int attn_splits(int dtype, int n_keys);
size_t attn_partial_floats(int n_split, int n_q, int rows_pad, int hd);
int launch_attention(int dtype, const void* q, const void* kc, const void* vc, int rows, int rows_pad, int n_causal,
                     int pos0, int n_keys, int n_q, int n_kv, int hd, int cap, int n_split, float* part_o,
                     float* part_ml, void* att_out, hipStream_t st);

}  // namespace ds
