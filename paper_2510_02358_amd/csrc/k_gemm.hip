// Skinny-M GEMMs: out[M, N] = X[M, K] * W[N, K]^T with M <= 144 rows.
//
// Every projection of the round (QKV, O, gate/up, down, LM head) has this shape, and with so few
// rows each one is a weight stream: every weight byte is read exactly once, so the kernel is bound
// by HBM bandwidth, not by the matrix cores.  MFMA is used because the work is a dense contraction
// and plain ALUs would become the limiter at M = 33..130.
//
// bf16 path (bf16 weights from the caller, half-precision products)
//   * W is kept in "stream order": tiles of 16 output rows x 32 inputs, 1 KB each, laid out
//     [N/16][K/32][64 lanes][8 half] so that lane (16 g + i) holds W[16 nb + i][32 ks + 8 g .. + 7].
//     That is exactly the register image of the 16x16x32 MFMA's first operand: a wavefront reads
//     one tile with one fully coalesced 16-byte-per-lane load and feeds it to the matrix core
//     with no LDS round trip.  A wavefront walks K for its NB row blocks, so its loads form NB
//     contiguous streams.  The packing kernel re-encodes each bf16 weight as IEEE half (exact for
//     2^-14 <= |w| <= 65504; smaller magnitudes round to the half subnormal grid, larger ones raise
//     a flag that fails model creation), so the activation operand can be half too.
//   * X arrives as IEEE half in tile order (see xt_offset): 11 mantissa bits per activation in a
//     single product per weight, float32 accumulation.  X is staged through LDS in chunks of 128
//     columns and shared by the 4 wavefronts of the workgroup; weight tiles for the next two chunks
//     are already in flight while the current chunk is multiplied.
//   * D[i][j] of the MFMA = out[16 mb + j][16 nb + i]: lane (16 g + j) ends with 4 consecutive
//     output columns of row j, stored as one float4.
//   * Split-K writes float32 partial planes out[s][M][N]; the consumer kernel sums them in a fixed
//     order (deterministic, no atomics).
//   * The weight loads are non-temporal: every weight byte is used once, and keeping the stream out of
//     the caches leaves them to the activation tiles that all workgroups re-read (measured: 6 % faster
//     on the LM head, 5-15 % on the layer projections).
//   * The unsplit LM-head product has three epilogues besides plain planes: logits stored non-temporally;
//     per-tile arg-max records (greedy verification); per-tile lattice records (two largest values with
//     their columns, third largest value, sum of exponentials).  With records the logits need not be
//     written at all: at 32 rows their 19.5 MB of writes cost as much as 100 MB of the read stream.
//
// f32 path: a plain wavefront-per-output-column kernel for the float32 parity mode.
#include <limits.h>
#include <math.h>
#include <type_traits>

#include "ds_act.h"
#include "ds_common.h"

namespace ds {

typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

namespace {

constexpr int kGemmThreads = 256;
constexpr int kGroup = 4;  // split-K granularity in k-steps of 32: 128 columns
constexpr int kKSC = 4;    // k-steps per LDS chunk: 128 columns (8 KB of X per row block and buffer pair)
// Register budget: two wavefronts per SIMD (<= 256 VGPRs) wherever the tile fits without spilling; the
// widest tiles keep one wavefront per SIMD and the full register file.
constexpr int min_waves_for(int MB, int NB) { return (NB == 2 && MB >= 6) ? 1 : 2; }

// Copy a canonical row-major bf16 matrix W[N, K] into stream order as IEEE half.  One thread per 16-byte piece.
// With a second matrix w2 (same shape [N / 2, K] each): the destination's 16-row blocks alternate between the two,
// block 2c = rows [16c, 16c + 16) of w, block 2c + 1 = the same rows of w2, so that a wavefront that multiplies two
// adjacent blocks holds column block c of both products.
__global__ void pack_weight_kernel(const uint16_t* __restrict__ w, const uint16_t* __restrict__ w2, int N, int K,
                                   uint16_t* __restrict__ dst, uint32_t* __restrict__ range_flag) {
  const size_t piece = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const size_t n_piece = (size_t)N * K / 8;
  if (piece >= n_piece) return;
  const int lane = piece & 63;
  const size_t tile = piece >> 6;
  const int ksteps = K >> 5;
  const int ks = (int)(tile % ksteps);
  const int nb = (int)(tile / ksteps);
  const int i = lane & 15, g = lane >> 4;
  const uint16_t* src = (w2 && (nb & 1)) ? w2 : w;
  const int sb = w2 ? nb >> 1 : nb;
  const uint4 v = *reinterpret_cast<const uint4*>(src + (size_t)(sb * 16 + i) * K + ks * 32 + g * 8);
  const uint32_t in[4] = {v.x, v.y, v.z, v.w};
  uint32_t o[4];
  bool bad = false;
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    const float lo = __uint_as_float(in[e] << 16), hi = __uint_as_float(in[e] & 0xFFFF0000u);
    bad |= !(fabsf(lo) <= 65504.f) || !(fabsf(hi) <= 65504.f);  // also true for NaN
    const _Float16 hl = (_Float16)lo, hh = (_Float16)hi;         // round to nearest even
    o[e] = (uint32_t)__builtin_bit_cast(uint16_t, hl) | ((uint32_t)__builtin_bit_cast(uint16_t, hh) << 16);
  }
  *reinterpret_cast<uint4*>(dst + piece * 8) = make_uint4(o[0], o[1], o[2], o[3]);
  if (bad) atomicOr(range_flag, 1u);
}

// EPI selects the epilogue at compile time, so that the split-K layer products carry none of the LM head's code:
//   kEpiPlanes  plain stores into this split's plane of `out`;
//   kEpiStream  unsplit product, non-temporal stores (logits are consumed once, later);
//   kEpiBest    unsplit product of full tiles: per-tile arg-max records into `rec`, and the non-temporal stores
//               only if `out` is not NULL;
//   kEpiTop     as kEpiBest, with per-tile lattice records instead: the two largest values with their columns,
//               the third largest value, the sum of exp(x - largest); and the values of one chosen column.
//   kEpiSwiGLU  unsplit product of a gate / up pair packed with alternating blocks (launch_pack_weight_pair): the
//               wavefront's two adjacent blocks are column block c of gate and of up, so silu(gate) * up is taken
//               in registers and stored as the next product's half-precision input; the float32 product never
//               reaches memory and no separate kernel runs.
//   kEpiSwiGLU2 the same for a pair whose product is split into TWO planes when it is not fused: wavefronts 0 and 1 of
//               a workgroup walk the first half of K, wavefronts 2 and 3 the second half of the same columns, the
//               second pair hands its sums over through LDS and the epilogue adds the halves in plane order, so the
//               fused result has the bits of the two-plane product followed by the SwiGLU kernel.
enum { kEpiPlanes = 0, kEpiStream = 1, kEpiBest = 2, kEpiTop = 3, kEpiSwiGLU = 4, kEpiSwiGLU2 = 5 };

// Running (largest, second largest, third largest) of a stream of values; the first two carry their columns and
// order equal values by column, the third is a value only.
struct Top3 {
  float v1 = -INFINITY, v2 = -INFINITY, v3 = -INFINITY;
  int i1 = INT_MAX, i2 = INT_MAX;
  __device__ __forceinline__ void offer(float x, int col) {
    if (x > v1 || (x == v1 && col < i1)) {
      v3 = v2;
      v2 = v1;
      i2 = i1;
      v1 = x;
      i1 = col;
    } else if (x > v2 || (x == v2 && col < i2)) {
      v3 = v2;
      v2 = x;
      i2 = col;
    } else {
      v3 = fmaxf(v3, x);
    }
  }
  __device__ __forceinline__ void merge(float ov1, int oi1, float ov2, int oi2, float ov3) {
    offer(ov1, oi1);
    offer(ov2, oi2);
    v3 = fmaxf(v3, ov3);
  }
};

// WAVES: wavefronts per workgroup, 4 or 8.  All of them share the staged X chunk, so eight wavefronts (one
// workgroup per CU instead of two) read X from L2 half as often per weight byte: with many rows the X loads, not the
// weight stream, are what slows the product down (a 65-row product without them runs at the one-row rate).  Every
// output element sees the same k order either way, so the choice does not change a single bit of the result.
template <int MB, int NB, int EPI, int WAVES = 4>
__global__ __launch_bounds__(WAVES * 64) __attribute__((amdgpu_waves_per_eu(min_waves_for(MB, NB))))
void gemm_bf16_kernel(const uint16_t* __restrict__ wp,
                                                                 const uint16_t* __restrict__ xt, int M, int N,
                                                                 int K, int groups_per_split, int n_big,
                                                                 float* __restrict__ out,
                                                                 void* __restrict__ rec, int export_col,
                                                                 float* __restrict__ export_out,
                                                                 uint32_t* __restrict__ ovf) {
  constexpr int kTiles = MB * kKSC;  // X tiles per chunk: row blocks x k-steps
  constexpr bool kTwo = EPI == kEpiSwiGLU2;  // two halves of K side by side in one workgroup
  constexpr int kHalves = kTwo ? 2 : 1;
  __shared__ __attribute__((aligned(16))) uint16_t xs[2][kHalves * kTiles * 512];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int n_blocks = N >> 4, ksteps = K >> 5, n_chunks = ksteps / kKSC;
  // kTwo: every step handles chunk c of the first half and chunk c_half + c of the second (the launcher has checked
  // that the halves are equal); the loop below runs over the first half's range.
  const int c_half = kTwo ? n_chunks / 2 : 0;
  const int my_half = kTwo ? wave >> 1 : 0;
  const int c_begin = kTwo ? 0 : blockIdx.y * groups_per_split * (kGroup / kKSC);
  int c_end = kTwo ? c_half : c_begin + groups_per_split * (kGroup / kKSC);
  if (c_end > n_chunks) c_end = n_chunks;

  static_assert(WAVES == 4 || EPI == kEpiPlanes || EPI == kEpiStream || EPI == kEpiSwiGLU,
                "the record epilogues reduce over four wavefronts");
  static_assert((EPI != kEpiSwiGLU && EPI != kEpiSwiGLU2) || NB == 2,
                "the fused epilogue pairs a wavefront's two column blocks");
  constexpr int kThreads = WAVES * 64;
  constexpr int kColWaves = WAVES / kHalves;  // wavefronts side by side over the columns
  // This workgroup's share of the output row blocks.  The first n_big workgroups take a full pass of
  // kColWaves * NB blocks each; a remainder goes to later workgroups in half-size pieces.
  const int full = kColWaves * NB, half = full / 2 > 0 ? full / 2 : 1;
  int nb_begin, nb_end;
  if ((int)blockIdx.x < n_big) {
    nb_begin = (int)blockIdx.x * full;
    nb_end = nb_begin + full;
  } else {
    nb_begin = n_big * full + ((int)blockIdx.x - n_big) * half;
    nb_end = nb_begin + half;
  }
  if (nb_end > n_blocks) nb_end = n_blocks;
  const int j_out = lane & 15, g_out = lane >> 4;
  float* out_plane = out + (size_t)blockIdx.y * M * N;

  for (int pass0 = nb_begin; pass0 < nb_end; pass0 += kColWaves * NB) {
  int nb[NB];
  const uint16_t* wrow[NB];
#pragma unroll
  for (int b = 0; b < NB; ++b) {
    nb[b] = pass0 + (kTwo ? wave & 1 : wave) * NB + b;  // a wavefront's blocks are adjacent
    const int nbc = nb[b] < nb_end ? nb[b] : nb_end - 1;  // clamp: loads stay in this workgroup's range
    wrow[b] = wp + ((size_t)nbc * ksteps + (size_t)my_half * c_half * kKSC) * 512 + lane * 8;
  }

  f32x4 acc[NB][MB];
#pragma unroll
  for (int b = 0; b < NB; ++b)
#pragma unroll
    for (int m = 0; m < MB; ++m) acc[b][m] = f32x4{0.f, 0.f, 0.f, 0.f};

  // 16-byte pieces of X per chunk, order [mb][s][lane]: kXPer per thread.  With four wavefronts the pieces split
  // evenly; with eight and an odd MB the last round is half full: those threads re-load the chunk's last piece
  // (no predicate on the loads, which therefore issue back to back) and skip the store.
  constexpr int kHalfPieces = kTiles * 64;
  constexpr int kPieces = kHalves * kHalfPieces;
  constexpr int kXPer = (kPieces + kThreads - 1) / kThreads;
  constexpr bool kXTail = (kPieces % kThreads) != 0;
  constexpr int kStages = 3;  // weight-tile register sets: two chunks are in flight while one is multiplied
  u32x4 xreg[kXPer];
  f16x8 areg[kStages][NB][kKSC];

  // Source offset of this thread's piece p within a chunk (halfs; the chunk offset is added per load).  A piece
  // holds 8 columns of one row (row = piece & 15 of its row block).  Rows past M are padding whose products are never
  // stored: their lanes read the block's last real row instead, which lands in the sectors the real rows fetch
  // anyway, so that a 33-row call moves 36 rows' worth of X through L2, not 48.  (Branch-free: the same loads issue.)
  size_t x_off[kXPer];
#pragma unroll
  for (int p = 0; p < kXPer; ++p) {
    int piece = threadIdx.x + p * kThreads;
    if (kXTail && piece >= kPieces) piece = kPieces - 1;
    const int x_half = kTwo ? piece / kHalfPieces : 0;  // the pieces of the second half's chunk follow the first's
    piece -= x_half * kHalfPieces;
    const int mb = piece / (kKSC * 64), rest = piece - mb * (kKSC * 64);
    const int j = rest & 15;
    int j_last = M - 1 - mb * 16;  // last real row of this block (>= 15: a full block)
    j_last = j_last < 0 ? 0 : j_last;
    const int jc = j < j_last ? j : j_last;
    x_off[p] = (size_t)mb * ksteps * 512 + (size_t)(rest - j + jc) * 8 + (size_t)x_half * c_half * kKSC * 512;
  }
  auto load_x = [&](int c) {
#pragma unroll
    for (int p = 0; p < kXPer; ++p)
      xreg[p] = *reinterpret_cast<const u32x4*>(xt + x_off[p] + (size_t)c * kKSC * 512);
  };
  auto store_x = [&](int buf) {
#pragma unroll
    for (int p = 0; p < kXPer; ++p)
      if (!kXTail || (int)threadIdx.x + p * kThreads < kPieces)
        *reinterpret_cast<u32x4*>(&xs[buf][(threadIdx.x + p * kThreads) * 8]) = xreg[p];
  };
  // Weights are read exactly once per product: non-temporal loads keep them from displacing the activations
  // (re-read by every workgroup) and the output lines in the caches.
  auto load_a = [&](auto set, int c) {
#pragma unroll
    for (int b = 0; b < NB; ++b)
#pragma unroll
      for (int s = 0; s < kKSC; ++s)
        areg[set][b][s] =
            __builtin_nontemporal_load(reinterpret_cast<const f16x8*>(wrow[b] + ((size_t)c * kKSC + s) * 512));
  };
  auto compute = [&](auto set, int buf) {
#pragma unroll
    for (int s = 0; s < kKSC; ++s) {
      f16x8 bx[MB];
#pragma unroll
      for (int m = 0; m < MB; ++m)
        bx[m] = *reinterpret_cast<const f16x8*>(&xs[buf][my_half * (kTiles * 512) + ((m * kKSC + s) * 64 + lane) * 8]);
#pragma unroll
      for (int b = 0; b < NB; ++b)
#pragma unroll
        for (int m = 0; m < MB; ++m)
          acc[b][m] = __builtin_amdgcn_mfma_f32_16x16x32_f16(areg[set][b][s], bx[m], acc[b][m], 0, 0, 0);
    }
  };
  // One pipeline step for chunk c (weights in register set SET, X in LDS buffer buf).  X(c + 1) was
  // loaded during the previous step and is published to the other LDS buffer first; then the X loads of
  // chunk c + 2 and the weight loads of chunk c + 2 are issued (X BEFORE the weights, so that waiting for
  // X next step leaves the younger weight loads in flight); then chunk c is multiplied.  Nothing that a
  // step waits for was issued less than one full step earlier.  Past the last chunk the loads are clamped
  // to it instead of predicated (branch-free body; the redundant tiles are never multiplied).
  const int c_last = c_end - 1;
  auto step = [&](auto set, int c, int buf) {
    constexpr int SET = decltype(set)::value;
    store_x(buf ^ 1);
    __builtin_amdgcn_sched_barrier(0);
    load_x(c + 2 < c_last ? c + 2 : c_last);
    __builtin_amdgcn_sched_barrier(0);  // keep the issue order: X loads, then weight loads, then math
    load_a(std::integral_constant<int, (SET + 2) % kStages>{}, c + 2 < c_last ? c + 2 : c_last);
    __builtin_amdgcn_sched_barrier(0);
    compute(set, buf);
    __syncthreads();
  };

  if (c_begin < c_end) {
    load_x(c_begin);
    load_a(std::integral_constant<int, 0>{}, c_begin);
    load_a(std::integral_constant<int, 1>{}, c_begin + 1 < c_last ? c_begin + 1 : c_last);
    store_x(0);
    load_x(c_begin + 1 < c_last ? c_begin + 1 : c_last);
    __syncthreads();
    // Main loop: groups of three chunks with no branch between the steps, so that the three steps form
    // one basic block and every prefetch stays where it is issued (two chunks ahead of its use).
    int buf = 0, c = c_begin;
    for (; c + kStages <= c_end; c += kStages) {
      step(std::integral_constant<int, 0>{}, c, buf);
      step(std::integral_constant<int, 1>{}, c + 1, buf ^ 1);
      step(std::integral_constant<int, 2>{}, c + 2, buf);
      buf ^= 1;
    }
    if (c < c_end) {  // one or two chunks left; c - c_begin is a multiple of three, so set 0 holds chunk c
      step(std::integral_constant<int, 0>{}, c, buf);
      if (c + 1 < c_end) step(std::integral_constant<int, 1>{}, c + 1, buf ^ 1);
    }
  }

  // D[i][j]: lane (16 g + j) holds rows i = 4 g .. 4 g + 3 of column j  ->  out[m = 16 mb + j][n = 16 nb + 4 g ..]
  if (kTwo) {
    // the second half's sums go to the wavefront of the first half that holds the same columns (the main loop is
    // past its last barrier: the X buffers are free); then plane order: the consumer of two planes starts from zero
    f32x4* red = reinterpret_cast<f32x4*>(&xs[0][0]);  // [2 wavefronts][NB][MB][64 lanes]
    static_assert(2 * NB * MB * 64 * sizeof(f32x4) <= sizeof(xs), "the exchange fits the X buffers");
    if (my_half == 1) {
#pragma unroll
      for (int b = 0; b < NB; ++b)
#pragma unroll
        for (int m = 0; m < MB; ++m) red[(((wave & 1) * NB + b) * MB + m) * 64 + lane] = acc[b][m];
    }
    __syncthreads();
    if (my_half == 0) {
#pragma unroll
      for (int b = 0; b < NB; ++b)
#pragma unroll
        for (int m = 0; m < MB; ++m) {
          const f32x4 other = red[(((wave & 1) * NB + b) * MB + m) * 64 + lane];
#pragma unroll
          for (int e = 0; e < 4; ++e) acc[b][m][e] = (0.f + acc[b][m][e]) + other[e];
        }
    }
  }
  if (EPI == kEpiSwiGLU || EPI == kEpiSwiGLU2) {
    // blocks 2c and 2c + 1 of the packed pair: gate and up of column block c.  rec: the half-precision GEMM input
    // [rows padded, N / 2] of the next product (tile order).
    bf16_t* act = static_cast<bf16_t*>(rec);
    if (nb[0] < nb_end && my_half == 0) {
      const int col = (nb[0] >> 1) * 16 + g_out * 4;
#pragma unroll
      for (int m = 0; m < MB; ++m) {
        const int row = m * 16 + j_out;
        if (row < M) {
          float4 y;
          y.x = acc[0][m][0] / (1.0f + expf(-acc[0][m][0])) * acc[NB - 1][m][0];
          y.y = acc[0][m][1] / (1.0f + expf(-acc[0][m][1])) * acc[NB - 1][m][1];
          y.z = acc[0][m][2] / (1.0f + expf(-acc[0][m][2])) * acc[NB - 1][m][2];
          y.w = acc[0][m][3] / (1.0f + expf(-acc[0][m][3])) * acc[NB - 1][m][3];
          Act<bf16_t>::put4(act, row, col, N >> 1, y, ovf);
        }
      }
    }
    if (kTwo) __syncthreads();  // a further pass reuses the X buffers
  } else if ((EPI != kEpiBest && EPI != kEpiTop) || out) {
#pragma unroll
    for (int b = 0; b < NB; ++b) {
      if (nb[b] >= nb_end) continue;
#pragma unroll
      for (int m = 0; m < MB; ++m) {
        const int row = m * 16 + j_out;
        if (row < M) {
          float* dst = out_plane + (size_t)row * N + nb[b] * 16 + g_out * 4;
          if (EPI != kEpiPlanes) {
#pragma unroll
            for (int e = 0; e < 4; ++e) __builtin_nontemporal_store(acc[b][m][e], dst + e);
          } else {
            *reinterpret_cast<float4*>(dst) = make_float4(acc[b][m][0], acc[b][m][1], acc[b][m][2], acc[b][m][3]);
          }
        }
      }
    }
  }
  // The largest value of every output row inside this workgroup's 64 * NB columns and its column (ties: lower
  // column): best[workgroup][row] = (value, column bits), MB * 16 rows per workgroup (padding rows included, so
  // that each workgroup writes one contiguous run of whole sectors).  A row's arg-max over all columns then needs
  // these pairs only, not the logits.  The word after the last record is the consumer's arrival counter, cleared
  // here.
  if (EPI == kEpiBest) {
    float2* best = static_cast<float2*>(rec);
    float2* red = reinterpret_cast<float2*>(&xs[0][0]);  // [4 waves][MB * 16 rows]; the main loop is past its last barrier
#pragma unroll
    for (int m = 0; m < MB; ++m) {
      float bv = -INFINITY;
      int bi = INT_MAX;
#pragma unroll
      for (int b = 0; b < NB; ++b)
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const int col = nb[b] * 16 + g_out * 4 + e;
          const float x = acc[b][m][e];
          if (x > bv || (x == bv && col < bi)) {
            bv = x;
            bi = col;
          }
        }
#pragma unroll
      for (int off = 16; off <= 32; off <<= 1) {
        const float ov = __shfl_xor(bv, off);
        const int oi = __shfl_xor(bi, off);
        if (ov > bv || (ov == bv && oi < bi)) {
          bv = ov;
          bi = oi;
        }
      }
      if (g_out == 0) red[(wave * MB + m) * 16 + j_out] = make_float2(bv, __int_as_float(bi));
    }
    __syncthreads();
    const int row = threadIdx.x;
    if (blockIdx.x == 0 && row == 0) *reinterpret_cast<uint32_t*>(best + (size_t)gridDim.x * MB * 16) = 0u;
    if (row < MB * 16) {
      float bv = -INFINITY;
      int bi = INT_MAX;
#pragma unroll
      for (int w = 0; w < 4; ++w) {
        const float2 q = red[w * MB * 16 + row];
        const int qi = __float_as_int(q.y);
        if (q.x > bv || (q.x == bv && qi < bi)) {
          bv = q.x;
          bi = qi;
        }
      }
      best[(size_t)blockIdx.x * MB * 16 + row] = make_float2(bv, __int_as_float(bi));
    }
  }
  // Lattice records of this workgroup's 128 columns, per output row: rec[workgroup][row] = two float4,
  // (v1, col1 bits, v2, col2 bits) and (v3, sum of exp(x - v1), 0, 0).  The log-sum-exp and the top-M of a row follow
  // from the records of all tiles unless some tile's third value could still enter the top-M, which the consumer
  // checks.  export_out[row] receives the value of column export_col (the EOS logit), if that column is here.
  if (EPI == kEpiTop) {
    constexpr float kLog2e = 1.4426950408889634f;
    float4* red_a = reinterpret_cast<float4*>(&xs[0][0]);        // [4 waves][MB * 16 rows]
    float2* red_b = reinterpret_cast<float2*>(red_a + 4 * MB * 16);
#pragma unroll
    for (int m = 0; m < MB; ++m) {
      Top3 t;
#pragma unroll
      for (int b = 0; b < NB; ++b)
#pragma unroll
        for (int e = 0; e < 4; ++e) t.offer(acc[b][m][e], nb[b] * 16 + g_out * 4 + e);
#pragma unroll
      for (int off = 16; off <= 32; off <<= 1) {
        const float ov1 = __shfl_xor(t.v1, off), ov2 = __shfl_xor(t.v2, off), ov3 = __shfl_xor(t.v3, off);
        const int oi1 = __shfl_xor(t.i1, off), oi2 = __shfl_xor(t.i2, off);
        t.merge(ov1, oi1, ov2, oi2, ov3);
      }
      const float nm = -t.v1 * kLog2e;
      float sum = 0.f;
#pragma unroll
      for (int b = 0; b < NB; ++b)
#pragma unroll
        for (int e = 0; e < 4; ++e) sum += __builtin_amdgcn_exp2f(fmaf(acc[b][m][e], kLog2e, nm));
      sum += __shfl_xor(sum, 16);
      sum += __shfl_xor(sum, 32);
      if (g_out == 0) {
        red_a[(wave * MB + m) * 16 + j_out] = make_float4(t.v1, __int_as_float(t.i1), t.v2, __int_as_float(t.i2));
        red_b[(wave * MB + m) * 16 + j_out] = make_float2(t.v3, sum);
      }
      if (export_out) {
#pragma unroll
        for (int b = 0; b < NB; ++b)
#pragma unroll
          for (int e = 0; e < 4; ++e)
            if (nb[b] * 16 + g_out * 4 + e == export_col) export_out[m * 16 + j_out] = acc[b][m][e];
      }
    }
    __syncthreads();
    const int row = threadIdx.x;
    if (row < MB * 16) {
      Top3 t;
      float vw[4], sw[4];
#pragma unroll
      for (int w = 0; w < 4; ++w) {
        const float4 a = red_a[w * MB * 16 + row];
        const float2 b = red_b[w * MB * 16 + row];
        vw[w] = a.x;
        sw[w] = b.y;
        t.merge(a.x, __float_as_int(a.y), a.z, __float_as_int(a.w), b.x);
      }
      float sum = 0.f;
#pragma unroll
      for (int w = 0; w < 4; ++w) sum += sw[w] * __builtin_amdgcn_exp2f((vw[w] - t.v1) * kLog2e);
      float4* dst = static_cast<float4*>(rec) + ((size_t)blockIdx.x * MB * 16 + row) * 2;
      dst[0] = make_float4(t.v1, __int_as_float(t.i1), t.v2, __int_as_float(t.i2));
      dst[1] = make_float4(t.v3, sum, 0.f, 0.f);
    }
  }
  __syncthreads();  // the next pass restages X into the same LDS buffers
  }  // passes
}

// float32 parity mode: one wavefront per output column n, lanes stride over k, rows in blocks of 8.
__global__ __launch_bounds__(256) void gemm_f32_kernel(const float* __restrict__ x, const float* __restrict__ w,
                                                       int M, int N, int K, float* __restrict__ out, int ldc) {
  const int lane = threadIdx.x & 63;
  const int n = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (n >= N) return;
  const float* wr = w + (size_t)n * K;
  for (int m0 = 0; m0 < M; m0 += 8) {
    float acc[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) acc[i] = 0.f;
    for (int k = lane; k < K; k += 64) {
      const float wv = wr[k];
#pragma unroll
      for (int i = 0; i < 8; ++i)
        if (m0 + i < M) acc[i] = fmaf(x[(size_t)(m0 + i) * K + k], wv, acc[i]);
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      float v = acc[i];
#pragma unroll
      for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off);
      if (lane == 0 && m0 + i < M) out[(size_t)(m0 + i) * ldc + n] = v;
    }
  }
}

template <int MB>
int launch_bf16_mb(const uint16_t* wp, const uint16_t* xt, int M, int N, int K, int nbw, int n_split, float* out,
                   const GemmEpilogue& epi, hipStream_t st) {
  const int n_groups = (K >> 5) / kGroup;
  const int gps = ceil_div(n_groups, n_split);
  // Eight wavefronts per workgroup from 65 rows up (measured: at 33 rows four are as fast or faster, at 65 rows the
  // 32B-shaped products gain 3 - 8 %, at 128 rows 20 %), where the row blocks divide into full passes, the
  // product writes planes or values, the tile fits two wavefronts per SIMD, and the workgroups - one per CU now -
  // fit the chip in one round; four otherwise.  Same bits either way.
  const int n_blocks = N >> 4;
  const bool plain = epi.kind == GemmEpilogue::kNone || epi.kind == GemmEpilogue::kSwiGLU;
  const bool wide = MB >= 5 && min_waves_for(MB, nbw) == 2 && plain &&
                    n_blocks % (8 * nbw) == 0 && (n_blocks / (8 * nbw)) * n_split <= 256;
  const int waves = wide ? 8 : 4;
  // A gate / up pair whose product takes two planes, fused: the workgroup's wavefronts pair up over the two halves of
  // K, so a workgroup covers half the columns (as many workgroups and wavefronts as the two-plane launch has).
  const bool two = epi.kind == GemmEpilogue::kSwiGLU && n_split == 2;
  // One workgroup per full pass of waves * nbw row blocks; a remainder goes to half-size workgroups at the end.
  const int full = (two ? waves / 2 : waves) * nbw, half = full / 2 > 0 ? full / 2 : 1;
  const int n_big = n_blocks / full;
  const int n_small = ceil_div(n_blocks - n_big * full, half);
  dim3 grid(n_big + n_small, two ? 1 : n_split);
  auto go = [&](auto kernel) {
    hipLaunchKernelGGL(kernel, grid, dim3(waves * 64), 0, st, wp, xt, M, N, K, gps, n_big, out, epi.records,
                       epi.export_col, epi.export_out, epi.ovf);
  };
  if (two) {
    if constexpr (MB <= 3) {
      go(gemm_bf16_kernel<MB, 2, kEpiSwiGLU2>);
      DS_LAUNCH_CHECK("gemm_bf16_kernel");
      return DS_OK;
    }
    return fail(DS_E_SHAPE, "GEMM: the fused two-plane gate / up product takes at most 48 rows");
  }
  if (wide) {
    if constexpr (MB >= 5) {
      if (epi.kind == GemmEpilogue::kSwiGLU) go(gemm_bf16_kernel<MB, 2, kEpiSwiGLU, 8>);
      else if (n_split == 1 && nbw == 2) go(gemm_bf16_kernel<MB, 2, kEpiStream, 8>);
      else if (n_split == 1) go(gemm_bf16_kernel<MB, 1, kEpiStream, 8>);
      else if (nbw == 2) go(gemm_bf16_kernel<MB, 2, kEpiPlanes, 8>);
      else go(gemm_bf16_kernel<MB, 1, kEpiPlanes, 8>);
      DS_LAUNCH_CHECK("gemm_bf16_kernel");
      return DS_OK;
    }
  }
  // records: the caller has checked nbw == 2 and n_split == 1
  if (epi.kind == GemmEpilogue::kBest) go(gemm_bf16_kernel<MB, 2, kEpiBest>);
  else if (epi.kind == GemmEpilogue::kTop) go(gemm_bf16_kernel<MB, 2, kEpiTop>);
  else if (epi.kind == GemmEpilogue::kSwiGLU) go(gemm_bf16_kernel<MB, 2, kEpiSwiGLU>);
  else if (n_split == 1 && nbw == 2) go(gemm_bf16_kernel<MB, 2, kEpiStream>);
  else if (n_split == 1) go(gemm_bf16_kernel<MB, 1, kEpiStream>);
  else if (nbw == 2) go(gemm_bf16_kernel<MB, 2, kEpiPlanes>);
  else go(gemm_bf16_kernel<MB, 1, kEpiPlanes>);
  DS_LAUNCH_CHECK("gemm_bf16_kernel");
  return DS_OK;
}

}  // namespace

int launch_pack_weight(const void* w, int N, int K, void* dst, uint32_t* range_flag, hipStream_t st) {
  DS_REQUIRE((N & 15) == 0 && (K & 127) == 0, DS_E_SHAPE,
             "bf16 matrix [%d, %d]: rows must be a multiple of 16 and columns of 128", N, K);
  const size_t n_piece = (size_t)N * K / 8;
  hipLaunchKernelGGL(pack_weight_kernel, dim3((unsigned)((n_piece + 255) / 256)), dim3(256), 0, st,
                     static_cast<const uint16_t*>(w), static_cast<const uint16_t*>(nullptr), N, K,
                     static_cast<uint16_t*>(dst), range_flag);
  DS_LAUNCH_CHECK("pack_weight_kernel");
  return DS_OK;
}

// Two matrices [F, K] packed as one [2 F, K] with their 16-row blocks alternating (see pack_weight_kernel).
int launch_pack_weight_pair(const void* w_a, const void* w_b, int F, int K, void* dst, uint32_t* range_flag,
                            hipStream_t st) {
  DS_REQUIRE((F & 15) == 0 && (K & 127) == 0, DS_E_SHAPE,
             "bf16 matrix [%d, %d]: rows must be a multiple of 16 and columns of 128", F, K);
  const size_t n_piece = (size_t)2 * F * K / 8;
  hipLaunchKernelGGL(pack_weight_kernel, dim3((unsigned)((n_piece + 255) / 256)), dim3(256), 0, st,
                     static_cast<const uint16_t*>(w_a), static_cast<const uint16_t*>(w_b), 2 * F, K,
                     static_cast<uint16_t*>(dst), range_flag);
  DS_LAUNCH_CHECK("pack_weight_kernel");
  return DS_OK;
}

// Number of float32 partial planes gemm_bf16 will write for this shape (the consumer sums them).
int gemm_bf16_splits(int N, int K, int nbw) {
  const int units = ceil_div(N >> 4, 4 * nbw);
  const int n_groups = (K >> 5) / kGroup;
  // two workgroups per compute unit are resident at once (512 on the chip): the largest split count that still
  // fits one residency round, one more if that would leave the chip visibly underfilled; at most 10 planes (the
  // consumers sum up to 10).  Depends on the weight shape only, never on the row count.
  int s = 512 / units;
  if (units * s < 416) ++s;
  if (s > 10) s = 10;
  if (s > n_groups) s = n_groups;
  if (s < 1) s = 1;
  const int gps = ceil_div(n_groups, s);
  return ceil_div(n_groups, gps);
}

// Width of the column tiles the per-tile arg-max epilogue reports, or 0 if this shape cannot use it (it needs one
// unsplit pass in which every workgroup owns a full tile).  The records take gemm_bf16_best_bytes.
int gemm_bf16_best_tile(int N, int nbw, int n_split) {
  const int w = 64 * nbw;
  return (nbw == 2 && n_split == 1 && N % w == 0) ? w : 0;
}

size_t gemm_bf16_best_bytes(int rows, int N, int tile) {
  return (size_t)(N / tile) * (ceil_div(rows, 16) * 16) * sizeof(float2) + 256;  // records, then the counter
}

size_t gemm_bf16_top_bytes(int rows, int N, int tile) {
  return (size_t)(N / tile) * (ceil_div(rows, 16) * 16) * 2 * sizeof(float4);
}

int launch_gemm_bf16(const void* wp, const void* xt, int M, int N, int K, int nbw, int n_split, float* out,
                     const GemmEpilogue& epi, hipStream_t st) {
  DS_REQUIRE(M >= 1 && M <= DS_MAX_ROWS, DS_E_SHAPE, "GEMM rows %d outside [1, %d]", M, DS_MAX_ROWS);
  DS_REQUIRE((N & 15) == 0 && (K & 127) == 0, DS_E_SHAPE, "GEMM [%d x %d]: N %% 16 and K %% 128 must be 0", N, K);
  if (epi.kind == GemmEpilogue::kSwiGLU)
    DS_REQUIRE(epi.records && nbw == 2 && (N >> 4) % 16 == 0 &&
                   (n_split == 1 || (n_split == 2 && M <= 48 && ((K >> 5) / kKSC) % 2 == 0 && kGroup == kKSC)),
               DS_E_SHAPE,
               "GEMM [%d x %d]: the fused gate / up epilogue needs whole pairs of blocks and one plane (or, up to 48 "
               "rows, two equal ones)", N, K);
  const bool records = epi.kind == GemmEpilogue::kBest || epi.kind == GemmEpilogue::kTop;
  DS_REQUIRE(out || records || epi.kind == GemmEpilogue::kSwiGLU, DS_E_INVALID,
             "GEMM: neither an output nor a per-tile record buffer");
  DS_REQUIRE(!records || (epi.records && gemm_bf16_best_tile(N, nbw, n_split) > 0), DS_E_SHAPE,
             "GEMM [%d x %d]: per-tile records need a buffer and an unsplit pass of full tiles", N, K);
  const uint16_t* w = static_cast<const uint16_t*>(wp);
  const uint16_t* x = static_cast<const uint16_t*>(xt);
  switch (ceil_div(M, 16)) {
    case 1: return launch_bf16_mb<1>(w, x, M, N, K, nbw, n_split, out, epi, st);
    case 2: return launch_bf16_mb<2>(w, x, M, N, K, nbw, n_split, out, epi, st);
    case 3: return launch_bf16_mb<3>(w, x, M, N, K, nbw, n_split, out, epi, st);
    case 4: return launch_bf16_mb<4>(w, x, M, N, K, nbw, n_split, out, epi, st);
    case 5: return launch_bf16_mb<5>(w, x, M, N, K, nbw, n_split, out, epi, st);
    case 6: return launch_bf16_mb<6>(w, x, M, N, K, nbw, n_split, out, epi, st);
    case 7: return launch_bf16_mb<7>(w, x, M, N, K, nbw, n_split, out, epi, st);
    case 8: return launch_bf16_mb<8>(w, x, M, N, K, nbw, n_split, out, epi, st);
    default: return launch_bf16_mb<9>(w, x, M, N, K, nbw, n_split, out, epi, st);
  }
}

int launch_gemm_f32(const float* x, const float* w, int M, int N, int K, float* out, int ldc, hipStream_t st) {
  hipLaunchKernelGGL(gemm_f32_kernel, dim3(ceil_div(N, 4)), dim3(256), 0, st, x, w, M, N, K, out, ldc);
  DS_LAUNCH_CHECK("gemm_f32_kernel");
  return DS_OK;
}

}  // namespace ds
