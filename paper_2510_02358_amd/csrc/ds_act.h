// Storage-type traits.
//
// DS_F32 (parity mode): everything float32, row-major.
// DS_BF16: the caller's weights are bf16.  Every activation that meets a weight on the matrix cores
//   is IEEE half (11 mantissa bits, 2 bytes like bf16) in tile order (xt_offset), and the weight
//   copies the GEMM kernels stream are re-encoded from bf16 to half when they are packed: a bf16
//   value has 8 mantissa bits, so the re-encoding is exact for 2^-14 <= |w| <= 65504 (smaller values
//   land on the half subnormal grid, absolute error <= 2^-25; larger ones are refused).  One product
//   per element then carries ~8x less activation rounding than a bf16 activation would, at the same
//   matrix-core rate and with half the operand traffic of a two-term bf16 split.  Queries, keys,
//   values and attention probabilities are half as well: with N(0, 0.02) random-init weights the
//   residual stream is ~0.03 rms, the RMSNorm after attention amplifies any error of the attention
//   output ~30x, and a bf16 KV cache alone would consume the whole 2e-2 logit budget.
//   Accumulation, the residual stream, split-K partial sums and logits are float32.
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

// Half-precision KV cache of one head: 64-key chunks, each stored as the 16 matrix-core operand tiles
// (1 KB, 64 lanes x 8 halfs) the attention kernel multiplies with, so that staging a chunk is a linear copy.
//   K tile (kb, s), kb = key block of 16, s = 32-column step: lane (16 g + i) holds K[16 kb + i][32 s + 8 g .. + 7].
//   V tile (db, t2), db = 16 output columns, t2 = 32-key half: lane (16 g + i) holds column 16 db + i of the keys
//     32 t2 + 4 g + {0..3} and 32 t2 + 16 + 4 g + {0..3}  (the key order in which the transposed score
//     accumulator delivers the probabilities).
// Offsets are in elements from the head's base; pos = absolute key position, dim = column.
__host__ __device__ static inline size_t kv_k_offset(int pos, int dim) {
  const int c = pos >> 6, kb = (pos >> 4) & 3, i = pos & 15, s = dim >> 5, g = (dim >> 3) & 3, e = dim & 7;
  return ((size_t)c * 16 + kb * 4 + s) * 512 + (size_t)(g * 16 + i) * 8 + e;
}
__host__ __device__ static inline size_t kv_v_offset(int pos, int dim) {
  const int c = pos >> 6, t2 = (pos >> 5) & 1, r = pos & 31, g = (r & 15) >> 2, e = (r & 3) + ((r >> 4) << 2);
  const int db = dim >> 4, i = dim & 15;
  return ((size_t)c * 16 + db * 2 + t2) * 512 + (size_t)(g * 16 + i) * 8 + e;
}

template <typename T>
struct Act;

// `ovf` in the stores below: the model's activation-overflow counter ([dev] uint32, or NULL).  A half-precision
// model counts there every activation that did not fit the half range and was clamped to +-65504 (or was NaN), so
// that a caller can tell a clean forward from one whose logits the clamp has touched; float32 models never count.
template <>
struct Act<float> {
  using kv_t = float;                         // element type of q / K cache / V cache
  static constexpr bool kTiledKV = false;     // row-major [capacity][head_dim] per head
  // GEMM-input store: element (m, k) of a [rows_pad, K] activation
  __device__ static __forceinline__ void put(float* base, int m, int k, int K, float v, uint32_t*) {
    base[(size_t)m * K + k] = v;
  }
  // four consecutive columns k .. k+3 (k % 4 == 0)
  __device__ static __forceinline__ void put4(float* base, int m, int k, int K, float4 v, uint32_t*) {
    *reinterpret_cast<float4*>(base + (size_t)m * K + k) = v;
  }
  __device__ static __forceinline__ size_t q_off(int m, int k, int K) { return (size_t)m * K + k; }
  __device__ static __forceinline__ float to_kv(float v, uint32_t*) { return v; }
  __device__ static __forceinline__ float weight(float v) { return v; }
};

template <>
struct Act<bf16_t> {
  using kv_t = uint16_t;                      // IEEE half bits
  static constexpr bool kTiledKV = true;      // operand-tile order, see kv_k_offset / kv_v_offset
  // GEMM-input store: element (m, k) of a [rows_pad, K] half activation in tile order (values beyond the half
  // range saturate to +-65504 instead of becoming infinite)
  __device__ static __forceinline__ bool over(float v) { return !(fabsf(v) <= 65504.f); }  // also true for NaN
  __device__ static __forceinline__ uint16_t gemm_in(float v) {
    return float_to_half_bits(fminf(fmaxf(v, -65504.f), 65504.f));
  }
  __device__ static __forceinline__ void put(bf16_t* base, int m, int k, int K, float v, uint32_t* ovf) {
    base[xt_offset(m, k, K)].bits = gemm_in(v);
    if (ovf && over(v)) atomicAdd(ovf, 1u);
  }
  // four consecutive columns k .. k+3 (k % 4 == 0) are adjacent in tile order: one 8-byte store
  __device__ static __forceinline__ void put4(bf16_t* base, int m, int k, int K, float4 v, uint32_t* ovf) {
    const uint32_t h0 = gemm_in(v.x), h1 = gemm_in(v.y), h2 = gemm_in(v.z), h3 = gemm_in(v.w);
    *reinterpret_cast<uint2*>(base + xt_offset(m, k, K)) = make_uint2(h0 | (h1 << 16), h2 | (h3 << 16));
    const uint32_t n = (uint32_t)over(v.x) + (uint32_t)over(v.y) + (uint32_t)over(v.z) + (uint32_t)over(v.w);
    if (ovf && n) atomicAdd(ovf, n);
  }
  __device__ static __forceinline__ size_t q_off(int m, int k, int K) { return xt_offset(m, k, K); }
  // queries, keys and values: clamped like every other half activation, and counted
  __device__ static __forceinline__ uint16_t to_kv(float v, uint32_t* ovf) {
    if (ovf && over(v)) atomicAdd(ovf, 1u);
    return gemm_in(v);
  }
  __device__ static __forceinline__ float weight(bf16_t v) { return bf16_bits_to_float(v.bits); }
};

// ---- launchers implemented in k_elem.hip / k_gemm.hip / k_attn.hip --------------------------------
// First kernel of a forward: token gather (see SeqTable: tok_a / tok_b / fill), rotary table, embedding, RMSNorm.
template <typename T>
int launch_embed_norm(const SeqTable& tab, const int32_t* tok_a, const int32_t* tok_b, int32_t fill, int vocab, int hd,
                      double rope_base, float2* cs, const void* embed, float* x, int rows, int rows_pad, int d,
                      const float* gain, float eps, void* h, uint32_t* ovf, hipStream_t st);
// rm_out / h_tail (optional): the rows every sequence hands on (SeqTable::tail0 / tail_base), compacted.
template <typename T>
int launch_add_norm(const SeqTable& tab, float* x, const float* part, int n_part, int rows, int rows_pad, int d,
                    const float* gain, float eps, void* h, float* rm_out, void* h_tail, uint32_t* ovf,
                    hipStream_t st);
template <typename T>
int launch_to_gemm_input(const float* src, int rows, int rows_pad, int d, void* dst, uint32_t* ovf, hipStream_t st);
template <typename T>
int launch_qkv_rope(const SeqTable& tab, const float* part, int n_part, int rows, int rows_pad, int n_q, int n_kv,
                    int hd, const float2* cs, int cap, float q_scale, void* q, uint32_t* ovf, hipStream_t st);
template <typename T>
int launch_swiglu(const float* part, int n_part, int rows, int rows_pad, int F, bool paired, void* act, uint32_t* ovf,
                  hipStream_t st);

// bf16 -> half re-encoding into stream order; *range_flag [dev] is set to 1 if any |w| exceeds the half range
int launch_pack_weight(const void* w, int N, int K, void* dst, uint32_t* range_flag, hipStream_t st);
int gemm_bf16_splits(int N, int K, int nbw);
// What an unsplit product of full tiles (gemm_bf16_best_tile() > 0) leaves besides, or instead of, its output:
//   kBest  per tile of 64 * nbw columns and output row (padded to 16): the largest value and its column (int bits),
//          float2 [N / tile][rows_pad], then a 32-bit arrival counter for the consumer, which the product clears;
//          gemm_bf16_best_bytes in all;
//   kTop   per tile and row two float4: (v1, col1, v2, col2) the two largest values with their columns and
//          (v3, sum exp(x - v1), 0, 0) the third largest value and the tile's exponential sum; gemm_bf16_top_bytes;
//          export_out[row] (rows_pad floats, optional) receives the values of column export_col.
// With records the output pointer may be NULL.
struct GemmEpilogue {
  enum Kind { kNone = 0, kBest = 1, kTop = 2, kSwiGLU = 3 };
  Kind kind = kNone;
  void* records = nullptr;   // kBest / kTop: the per-tile records; kSwiGLU: the half-precision output [rows padded, N / 2]
  int export_col = -1;
  float* export_out = nullptr;
  uint32_t* ovf = nullptr;   // kSwiGLU: the model's saturation counter
};
// gate and up ([F, K] each) as one stream-order matrix with alternating 16-row blocks, for the kSwiGLU epilogue
int launch_pack_weight_pair(const void* w_a, const void* w_b, int F, int K, void* dst, uint32_t* range_flag,
                            hipStream_t st);
int gemm_bf16_best_tile(int N, int nbw, int n_split);
size_t gemm_bf16_best_bytes(int rows, int N, int tile);
size_t gemm_bf16_top_bytes(int rows, int N, int tile);
int launch_gemm_bf16(const void* wp, const void* xt, int M, int N, int K, int nbw, int n_split, float* out,
                     const GemmEpilogue& epi, hipStream_t st);
int launch_gemm_f32(const float* x, const float* w, int M, int N, int K, float* out, int ldc, hipStream_t st);

// Attention of every sequence of the call (SeqTable: rows, cache, position and causal boundary per sequence) over
// its own keys [0, pos0 + n_rows).  Row i of a sequence sees key p iff i >= n_causal (a [MASK] row) or p <= pos0 + i.
// rows / rows_pad: all rows of the call.  part_o / part_ml hold attn_partial_rows(rows_pad) * n_q rows of head_dim /
// 2 floats.
struct AttnPlan {
  int n_split, chunks_per_split;
};
AttnPlan attn_plan(int dtype, int cap, int n_keys);
float attn_q_scale(int dtype, int hd);  // factor the producer of q folds into the queries
int attn_partial_rows(int rows_pad);
int launch_attention(int dtype, const SeqTable& tab, const void* q, int rows, int rows_pad, int n_q, int n_kv, int hd,
                     int cap, float* part_o, float* part_ml, void* att_out, uint32_t* ovf, hipStream_t st);

}  // namespace ds
