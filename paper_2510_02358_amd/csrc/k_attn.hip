// Grouped-query attention of a few query rows against the KV cache (cached prefix + the rows of the
// current call), split over the key axis ("flash-decoding" style) with an exact log-sum-exp merge.
//
// Visibility: row r (absolute position pos0 + r) sees key p iff p < n_keys and
//   r >= n_causal (a [MASK] row of the draft block: sees everything)  or  p <= pos0 + r (causal).
//
// Half-precision kernel (bf16 models, head_dim 128; q, K, V and probabilities are IEEE half): the
// query rows of all heads that share a KV head are packed densely into blocks of 16 (row v = head-in-group x
// rows + row; a block may span two heads), so one pass over that head's keys/values serves group x rows
// query rows with no padding between heads; both products run on the 16x16x32 f16 matrix cores.
// Scores are computed transposed, S^T = K Q^T, because the accumulator layout of S^T (lane = query
// row, 4 consecutive keys per register quad) is already the operand layout the second product P V
// needs: probabilities never leave registers.
//
// Cache layout (private to the library): per KV head the cache is a sequence of 64-key chunks, and a
// chunk of K (and of V) is stored as the 16 matrix-core operand tiles the kernel multiplies with
// (kv_k_offset / kv_v_offset in ds_act.h).  Staging a chunk is therefore a straight, fully coalesced
// 16 KB + 16 KB copy, issued as global -> LDS loads that pass through no registers; two LDS buffers
// alternate, so the copy of chunk c + 1 runs under the math of chunk c with one barrier per chunk.
//
// f32 kernel: plain ALU version for the float32 parity mode (any head_dim <= 128, row-major cache).
#include <math.h>

#include <type_traits>

#include "ds_act.h"
#include "ds_common.h"

namespace ds {

typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));

namespace {

constexpr int kChunk = 64;  // keys per staged chunk
constexpr int kHd = 128;    // head_dim of the half-precision kernel
constexpr int kChunkElems = kChunk * kHd;  // halfs per chunk of K (and of V): 16 tiles x 512

union Pack8 {
  f16x8 v;
  uint16_t h[8];
  uint32_t w[4];
  u32x2 half[2];
  u32x4 q;
};

// xor-reduction of a maximum over the four 16-lane rows of a wavefront (the lanes that hold one query row), with the
// row-swap instructions of the vector unit: no trip through the LDS crossbar.
__device__ __forceinline__ float max_over_lane_rows(float x) {
  // Written as assembly: through the compiler's builtins the maximum of a swap's two results is folded to the first
  // result, which drops the exchange.  The no-op covers the wait states a swap needs after a vector write of its
  // operands.
  float a = x, b = x;
  asm volatile("s_nop 1\n\tv_permlane32_swap_b32 %0, %1" : "+v"(a), "+v"(b));  // a = [lo, lo], b = [hi, hi] halves
  const float y = fmaxf(a, b);
  float c = y, d = y;
  asm volatile("s_nop 1\n\tv_permlane16_swap_b32 %0, %1" : "+v"(c), "+v"(d));  // even rows and odd rows
  return fmaxf(c, d);
}

// Scores arrive in log2 units (the queries are stored pre-multiplied by log2(e) / sqrt(head_dim)) and relative to a
// per-row reference m_ref: the score accumulators start at -m_ref instead of zero, so a probability is one exp2 of
// the accumulator, p = 2^(s - m_ref), with no further arithmetic per score.  m_ref follows the running maximum
// lazily: it moves only when a chunk's maximum exceeds it by more than kRefSlack (then o and l are rescaled), so
// p <= 2^kRefSlack, far inside the half range.  Row sums l come from the matrix core too (a product of P with an
// all-ones tile), summed from the same half-precision probabilities that weight V.
constexpr float kRefSlack = 8.0f;

// Matrix work of a chunk: o += V^T P and l += 1^T P for the probabilities in pb (has_pv), or s4 = K Q^T - m_ref
// (has_qk).  LDS reads run four tiles ahead of the products that consume them (the scheduling barriers pin that
// order), so the matrix core does not wait for every read.
template <int QB, bool has_pv, bool has_qk>
__device__ __forceinline__ void attn_matrix_phase(const uint16_t* __restrict__ vs, const uint16_t* __restrict__ ks,
                                                  int lane, const f16x8 (&bq)[QB][4],
                                                  const Pack8 (&pb)[QB][2], const f32x4 (&neg_m)[QB], f32x4 (&o)[QB][8],
                                                  f32x4 (&l_acc)[QB], f32x4 (&s4)[QB][4]) {
  constexpr int kAhead = 4;
  if (has_pv) {  // V tiles in the order (key half t2, column block d)
    f16x8 b[16];
#pragma unroll
    for (int i = 0; i < kAhead; ++i)
      b[i] = *reinterpret_cast<const f16x8*>(&vs[(((i & 7) * 2 + (i >> 3)) * 64 + lane) * 8]);
    Pack8 ones;
#pragma unroll
    for (int e = 0; e < 4; ++e) ones.w[e] = 0x3C003C00u;
#pragma unroll
    for (int t = 0; t < QB; ++t)
#pragma unroll
      for (int t2 = 0; t2 < 2; ++t2)
        l_acc[t] = __builtin_amdgcn_mfma_f32_16x16x32_f16(ones.v, pb[t][t2].v, l_acc[t], 0, 0, 0);
#pragma unroll
    for (int i = 0; i < 16; ++i) {
#pragma unroll
      for (int t = 0; t < QB; ++t)
        o[t][i & 7] = __builtin_amdgcn_mfma_f32_16x16x32_f16(b[i], pb[t][i >> 3].v, o[t][i & 7], 0, 0, 0);
      if (i + kAhead < 16) {
        const int n = i + kAhead;
        b[n] = *reinterpret_cast<const f16x8*>(&vs[(((n & 7) * 2 + (n >> 3)) * 64 + lane) * 8]);
      }
      __builtin_amdgcn_sched_barrier(0);
    }
  }
  if (has_qk) {  // K tiles in the order (column step s, key block kb): consecutive products go to different accumulators
    f16x8 a[16];
#pragma unroll
    for (int i = 0; i < kAhead; ++i)
      a[i] = *reinterpret_cast<const f16x8*>(&ks[(((i & 3) * 4 + (i >> 2)) * 64 + lane) * 8]);
#pragma unroll
    for (int i = 0; i < 16; ++i) {
#pragma unroll
      for (int t = 0; t < QB; ++t)
        s4[t][i & 3] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a[i], bq[t][i >> 2], i < 4 ? neg_m[t] : s4[t][i & 3], 0, 0, 0);
      if (i + kAhead < 16) {
        const int n = i + kAhead;
        a[n] = *reinterpret_cast<const f16x8*>(&ks[(((n & 3) * 4 + (n >> 2)) * 64 + lane) * 8]);
      }
      __builtin_amdgcn_sched_barrier(0);
    }
  }
}

// Softmax phase of the chunk starting at key c0: s4[t][kb][e] = score - m_ref of key c0 + 16 kb + 4 g + e for query
// row 16 rb + j.  Leaves the probabilities in pb (half, the P V operand).  Every decision is taken per row from that
// row's own values (the wavefront-wide test only skips work that would change nothing), so a row's result does not
// depend on which other rows share its wavefront.
template <int QB>
__device__ __forceinline__ void attn_softmax_phase(int g, int c0, const int (&lim_min)[QB], const int (&limit)[QB],
                                                   f32x4 (&s4)[QB][4], Pack8 (&pb)[QB][2], f32x4 (&o)[QB][8],
                                                   f32x4 (&l_acc)[QB], float (&m_ref)[QB], f32x4 (&neg_m)[QB]) {
#pragma unroll
  for (int t = 0; t < QB; ++t) {
    if (c0 + kChunk - 1 > lim_min[t]) {  // same for the whole wavefront: only the last chunks of a row block mask
      const int rel = limit[t] - c0 - 4 * g;
#pragma unroll
      for (int kb = 0; kb < 4; ++kb)
#pragma unroll
        for (int e = 0; e < 4; ++e)
          if (kb * 16 + e > rel) s4[t][kb][e] = -INFINITY;
    }
    float mx = fmaxf(s4[t][0][0], s4[t][0][1]);
#pragma unroll
    for (int kb = 0; kb < 4; ++kb)
#pragma unroll
      for (int e = (kb == 0 ? 2 : 0); e < 4; e += 2) mx = fmaxf(fmaxf(mx, s4[t][kb][e]), s4[t][kb][e + 1]);
    mx = max_over_lane_rows(mx);  // the chunk's maximum for this lane's query row, relative to m_ref
    const bool first = m_ref[t] == -INFINITY;  // nothing seen yet: the accumulators started at zero
    const float delta = first ? (mx == -INFINITY ? 0.f : mx) : (mx > kRefSlack ? mx : 0.f);
    if (__builtin_amdgcn_ballot_w64(delta != 0.f)) {  // some row of the wavefront moves its reference
      // The rare path updates its registers in place (assembly with tied operands): written as ordinary code, the
      // compiler gives the two sides of this branch different registers and copies all of o on the common side.
      const float alpha = first ? 1.0f : __builtin_amdgcn_exp2f(-delta);
#pragma unroll
      for (int kb = 0; kb < 4; ++kb)
#pragma unroll
        for (int e = 0; e < 4; ++e) asm volatile("v_sub_f32 %0, %0, %1" : "+v"(s4[t][kb][e]) : "v"(delta));
#pragma unroll
      for (int d = 0; d < 8; ++d)
#pragma unroll
        for (int e = 0; e < 4; ++e) asm volatile("v_mul_f32 %0, %0, %1" : "+v"(o[t][d][e]) : "v"(alpha));
#pragma unroll
      for (int e = 0; e < 4; ++e) asm volatile("v_mul_f32 %0, %0, %1" : "+v"(l_acc[t][e]) : "v"(alpha));
      m_ref[t] = first ? (mx == -INFINITY ? -INFINITY : mx) : m_ref[t] + delta;
      const float nm = (m_ref[t] == -INFINITY) ? 0.f : -m_ref[t];
      neg_m[t] = f32x4{nm, nm, nm, nm};
    }
#pragma unroll
    for (int kb = 0; kb < 4; ++kb)
#pragma unroll
      for (int e = 0; e < 4; e += 2) {
        const f32x2 pp = {__builtin_amdgcn_exp2f(s4[t][kb][e]), __builtin_amdgcn_exp2f(s4[t][kb][e + 1])};
        pb[t][kb >> 1].w[((kb & 1) * 4 + e) >> 1] = __builtin_bit_cast(uint32_t, __builtin_convertvector(pp, f16x2));
      }
  }
  // Passing the packed probabilities through an empty asm statement makes them exist here, in one run of vector
  // work; otherwise the compiler sinks each exponential down to the product that uses it, between the LDS reads
  // and matrix instructions whose order the P V loop pins.
#pragma unroll
  for (int t = 0; t < QB; ++t)
#pragma unroll
    for (int h = 0; h < 2; ++h)
#pragma unroll
      for (int k = 0; k < 4; ++k) asm volatile("" : "+v"(pb[t][h].w[k]));
}

// Barrier that closes a chunk: LDS traffic of this wavefront is complete (the tail patch writes LDS), then the
// workgroup barrier.  Unlike __syncthreads() it carries no wait for memory operations the compiler knows of.
__device__ __forceinline__ void phase_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

constexpr int kAttnThreads = 256;  // four wavefronts; two workgroups share a CU (64 KB of LDS each)
constexpr int kAttnQB = 2;         // query blocks of 16 rows per wavefront

// The chunk loop of one wavefront with NB live query blocks (NB = 0: a wavefront without query rows only copies and
// keeps the barriers).  i = chunk index within the split; chunk i uses LDS buffer i & 1.
template <int NB>
struct AttnWave {
  f16x8 bq[NB ? NB : 1][4];
  f32x4 o[NB ? NB : 1][8], s4[NB ? NB : 1][4], l_acc[NB ? NB : 1], neg_m[NB ? NB : 1];
  Pack8 pb[NB ? NB : 1][2];
  float m_ref[NB ? NB : 1];  // reference of the row's exponentials, log2 units (-inf until the row has seen a key)
  int lim_min[NB ? NB : 1], limit[NB ? NB : 1];
};

// The sequences of one attention launch: blockIdx.z = sequence * zdim + group of query blocks.  Each sequence has its
// own caches, row range (first row r0, a multiple of 16), key count and split plan; the launch covers the largest
// split count and the most query-block groups, and workgroups past a sequence's own extent leave empty partials
// or nothing.
struct AttnSeqs {
  const void* kc[kMaxSeq];
  const void* vc[kMaxSeq];
  int r0[kMaxSeq], rows[kMaxSeq], n_causal[kMaxSeq], pos0[kMaxSeq], n_keys[kMaxSeq], chunks_per_split[kMaxSeq];
  int zdim;
};

template <int QB>
__global__ __launch_bounds__(kAttnThreads) __attribute__((amdgpu_waves_per_eu(2))) void attn_f16_kernel(
    AttnSeqs sq, const uint16_t* __restrict__ q_all, int rows_stride, int n_q, int n_kv, int cap,
    float* __restrict__ part_o_all, float* __restrict__ part_ml_all) {
  // q: queries in log2 units (attn_q_scale folded in by the producer), per head [rows_stride rows] in tile order
  // rows: the rows of this workgroup's sequence (q, part_o and part_ml point at its first row, a multiple of 16);
  // rows_stride: padded rows of the whole call (stride between heads and between splits)
  __shared__ __attribute__((aligned(16))) uint16_t k_lds[2 * kChunkElems];
  __shared__ __attribute__((aligned(16))) uint16_t v_lds[2 * kChunkElems];
  const int seq = (int)blockIdx.z / sq.zdim, zq = (int)blockIdx.z - seq * sq.zdim;
  const uint16_t* __restrict__ q = q_all + (size_t)(sq.r0[seq] >> 4) * 4 * 512;
  const uint16_t* __restrict__ kc = static_cast<const uint16_t*>(sq.kc[seq]);
  const uint16_t* __restrict__ vc = static_cast<const uint16_t*>(sq.vc[seq]);
  const int rows = sq.rows[seq], n_causal = sq.n_causal[seq], pos0 = sq.pos0[seq], n_keys = sq.n_keys[seq];
  const int chunks_per_split = sq.chunks_per_split[seq];
  float* __restrict__ part_o = part_o_all + (size_t)sq.r0[seq] * kHd;
  float* __restrict__ part_ml = part_ml_all + (size_t)sq.r0[seq] * 2;
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int j = lane & 15, g = lane >> 4;
  const int split = blockIdx.x, kvh = blockIdx.y;
  const int group = n_q / n_kv, n_vrows = group * rows, n_qb = (n_vrows + 15) >> 4;
  const int n_chunks = (n_keys + kChunk - 1) / kChunk;
  const int c_begin = split * chunks_per_split;
  int c_end = c_begin + chunks_per_split;
  if (c_end > n_chunks) c_end = n_chunks;
  const int n = c_end > c_begin ? c_end - c_begin : 0;  // chunks of this split (same for the whole workgroup)
  const int qb0 = (zq * 4 + wave) * QB;                 // first query block of this wavefront
  const int nb = n_qb - qb0 >= QB ? QB : (n_qb > qb0 ? n_qb - qb0 : 0);  // its live blocks (a scalar)

  const uint16_t* kbase = kc + ((size_t)kvh * cap + (size_t)c_begin * kChunk) * kHd;
  const uint16_t* vbase = vc + ((size_t)kvh * cap + (size_t)c_begin * kChunk) * kHd;
  const uint32_t k_lds_addr = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) uint16_t*)k_lds;
  const uint32_t v_lds_addr = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) uint16_t*)v_lds;

  // Staging: a chunk is 2 x 1024 pieces of 16 bytes, already in operand order.  Each wavefront copies pieces
  // [64 wave + 256 p, + 64) of K and of V, p = 0..3, straight from global memory into LDS (16 bytes per lane, the
  // lanes of a wavefront land side by side from the wavefront's base address, which M0 carries).  Written as
  // assembly so that the compiler's wait-count bookkeeping does not put a wait for the copies in front of the LDS
  // reads of the chunk being computed (it cannot tell the two buffers apart); the wait that matters is explicit
  // (finish_chunk).  Nothing else in this kernel uses M0.
  auto issue_chunk = [&](int i) {
    const size_t off = (size_t)i * kChunkElems + threadIdx.x * 8;
    const uint32_t buf = (uint32_t)((i & 1) * kChunkElems * 2);
#pragma unroll
    for (int p = 0; p < 4; ++p) {
      const uint32_t dst = buf + (uint32_t)(wave * 64 + p * 256) * 16u;
      asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(k_lds_addr + dst),
                   "v"(kbase + off + p * 2048)
                   : "memory");
      asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(v_lds_addr + dst),
                   "v"(vbase + off + p * 2048)
                   : "memory");
    }
  };
  // After this wavefront's copies of chunk i have landed (and before the barrier that publishes them): in the tail
  // chunk the V slots past the last key may hold anything -> zero, so that probability 0 times that slot is 0.
  // Every thread patches the pieces its own lane copied.
  auto finish_chunk = [&](int i) {
    __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0)
    const int c0 = (c_begin + i) * kChunk;
    if (c0 + kChunk > n_keys) {
      uint16_t* vd = v_lds + (i & 1) * kChunkElems;
#pragma unroll
      for (int p = 0; p < 4; ++p) {
        Pack8 pk;
        pk.q = *reinterpret_cast<const u32x4*>(&vd[(threadIdx.x + p * 256) * 8]);
        const int t2 = (wave + 4 * p) & 1;  // tile index of this piece = wave + 4 p (V tile = db * 2 + t2)
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const int key = c0 + 32 * t2 + 4 * g + (e & 3) + ((e >> 2) << 4);
          if (key >= n_keys) pk.h[e] = 0;
        }
        *reinterpret_cast<u32x4*>(&vd[(threadIdx.x + p * 256) * 8]) = pk.q;
      }
    }
  };

  // The rows of block qb0 + t that this lane works for: virtual row v -> (head, row); lanes past the last virtual row
  // repeat it (they compute a copy that nobody stores).
  int head[QB], row[QB];
  bool live[QB];
#pragma unroll
  for (int t = 0; t < QB; ++t) {
    int v = (qb0 + t) * 16 + j;
    live[t] = v < n_vrows;
    if (v >= n_vrows) v = n_vrows - 1;
    head[t] = kvh * group + v / rows;
    row[t] = v % rows;
  }

  if (n == 0) {
    // An empty split (the whole workgroup takes this branch): a sequence of a batched call with fewer keys than
    // the longest one.  The merge walks every split, so leave partials of weight zero.
#pragma unroll
    for (int t = 0; t < QB; ++t) {
      if (!live[t]) continue;
      const size_t prow = ((size_t)split * n_q + head[t]) * rows_stride + row[t];
#pragma unroll
      for (int d = 0; d < 8; ++d)
        *reinterpret_cast<float4*>(part_o + prow * kHd + d * 16 + 4 * g) = make_float4(0.f, 0.f, 0.f, 0.f);
      if (g == 0) *reinterpret_cast<float2*>(part_ml + prow * 2) = make_float2(-INFINITY, 0.f);
    }
    return;
  }

  issue_chunk(0);
  auto run = [&](auto nb_tag) {
    constexpr int NB = decltype(nb_tag)::value;
    AttnWave<NB> w;
    if constexpr (NB > 0) {
#pragma unroll
      for (int t = 0; t < NB; ++t) {
        const uint16_t* qh = q + (size_t)head[t] * rows_stride * kHd + (size_t)(row[t] >> 4) * 4 * 512 + g * 128 +
                             (row[t] & 15) * 8;
#pragma unroll
        for (int s = 0; s < 4; ++s) w.bq[t][s] = *reinterpret_cast<const f16x8*>(qh + s * 512);
#pragma unroll
        for (int d = 0; d < 8; ++d) w.o[t][d] = f32x4{0.f, 0.f, 0.f, 0.f};
        w.l_acc[t] = f32x4{0.f, 0.f, 0.f, 0.f};
        w.neg_m[t] = f32x4{0.f, 0.f, 0.f, 0.f};
        w.m_ref[t] = -INFINITY;
        w.limit[t] = (row[t] >= n_causal) ? n_keys - 1 : pos0 + row[t];  // last key this lane's row sees
        int lm = w.limit[t];                                              // smallest limit in the block
#pragma unroll
        for (int off = 1; off < 16; off <<= 1) lm = min(lm, __shfl_xor(lm, off));
        w.lim_min[t] = lm;
      }
    }
    finish_chunk(0);
    __syncthreads();
    for (int i = 0; i < n; ++i) {
      if (i + 1 < n) issue_chunk(i + 1);
      if constexpr (NB > 0) {
        const uint16_t* ks = k_lds + (i & 1) * kChunkElems;
        const uint16_t* vs = v_lds + (i & 1) * kChunkElems;
        attn_matrix_phase<NB, false, true>(vs, ks, lane, w.bq, w.pb, w.neg_m, w.o, w.l_acc, w.s4);
        attn_softmax_phase<NB>(g, (c_begin + i) * kChunk, w.lim_min, w.limit, w.s4, w.pb, w.o, w.l_acc, w.m_ref, w.neg_m);
        attn_matrix_phase<NB, true, false>(vs, ks, lane, w.bq, w.pb, w.neg_m, w.o, w.l_acc, w.s4);
      }
      if (i + 1 < n) finish_chunk(i + 1);
      phase_barrier();
    }
    if constexpr (NB > 0) {
#pragma unroll
      for (int t = 0; t < NB; ++t) {
        if (!live[t]) continue;  // lanes past the last virtual row
        const size_t prow = ((size_t)split * n_q + head[t]) * rows_stride + row[t];
#pragma unroll
        for (int d = 0; d < 8; ++d)
          *reinterpret_cast<float4*>(part_o + prow * kHd + d * 16 + 4 * g) =
              make_float4(w.o[t][d][0], w.o[t][d][1], w.o[t][d][2], w.o[t][d][3]);
        // the merge works in natural-log units; every lane of a row holds the row's whole sum
        if (g == 0)
          *reinterpret_cast<float2*>(part_ml + prow * 2) =
              make_float2(w.m_ref[t] * 0.6931471805599453f, w.l_acc[t][0]);
      }
    }
  };
  if (nb == QB)
    run(std::integral_constant<int, QB>{});
  else if (nb == 1)
    run(std::integral_constant<int, 1>{});
  else
    run(std::integral_constant<int, 0>{});
}

// float32 parity mode.  grid (n_split, n_q); each wavefront walks rows r = wave, wave + 4, ...
__global__ __launch_bounds__(256) void attn_f32_kernel(AttnSeqs sq, const float* __restrict__ q_all, int rows_stride,
                                                       int n_q, int n_kv, int hd, int cap, float scale,
                                                       float* __restrict__ part_o_all,
                                                       float* __restrict__ part_ml_all) {
  __shared__ float qbuf[4][128];
  __shared__ float pbuf[4][kChunk];
  const int seq = blockIdx.z;
  const float* __restrict__ q = q_all + (size_t)sq.r0[seq] * hd;
  const float* __restrict__ kc = static_cast<const float*>(sq.kc[seq]);
  const float* __restrict__ vc = static_cast<const float*>(sq.vc[seq]);
  const int rows = sq.rows[seq], n_causal = sq.n_causal[seq], pos0 = sq.pos0[seq], n_keys = sq.n_keys[seq];
  const int chunks_per_split = sq.chunks_per_split[seq];
  float* __restrict__ part_o = part_o_all + (size_t)sq.r0[seq] * hd;
  float* __restrict__ part_ml = part_ml_all + (size_t)sq.r0[seq] * 2;
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
// Half-precision kernel: at most 21 splits over the capacity (at the long-context benchmark shape, 20 splits x 8 KV
// heads x 3 workgroups fill the 512 workgroup slots of the chip in one round), at least two 64-key chunks per split.
// float32 kernel: at most 16 splits.
constexpr int kMaxSplitsF16 = 21, kMaxSplitsF32 = 16;

// Rows-equivalents of partial results the workspace holds for a call with rows_pad padded rows.
int attn_partial_rows(int rows_pad) { return kMaxSplitsF16 * rows_pad; }

// What the producer of q multiplies the rotated queries by: the half-precision kernel takes them in log2 units.
float attn_q_scale(int dtype, int hd) { return dtype == DS_BF16 ? 1.4426950408889634f / sqrtf((float)hd) : 1.0f; }

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
  // one launch for all sequences (blockIdx.z carries the sequence)
  AttnSeqs sq{};
  int n_qb_max = 1;
  for (int s = 0; s < tab.n_seq; ++s) {
    const int n_keys = tab.pos0[s] + tab.n_rows[s];
    sq.kc[s] = tab.kc[s];
    sq.vc[s] = tab.vc[s];
    sq.r0[s] = tab.row0[s];
    sq.rows[s] = tab.n_rows[s];
    sq.n_causal[s] = tab.n_causal[s];
    sq.pos0[s] = tab.pos0[s];
    sq.n_keys[s] = n_keys;
    sq.chunks_per_split[s] = attn_plan(dtype, cap, n_keys).chunks_per_split;
    const int n_qb = ceil_div((n_q / n_kv) * tab.n_rows[s], 16);  // blocks of 16 densely packed (head, row) pairs
    n_qb_max = n_qb > n_qb_max ? n_qb : n_qb_max;
  }
  if (dtype == DS_BF16) {
    constexpr int QB = kAttnQB;
    sq.zdim = ceil_div(n_qb_max, 4 * QB);
    dim3 grid(n_split_max, n_kv, sq.zdim * tab.n_seq);
    hipLaunchKernelGGL((attn_f16_kernel<QB>), grid, dim3(kAttnThreads), 0, st, sq, static_cast<const uint16_t*>(q),
                       rows_pad, n_q, n_kv, cap, part_o, part_ml);
    DS_LAUNCH_CHECK("attn_f16_kernel");
  } else {
    sq.zdim = 1;
    hipLaunchKernelGGL(attn_f32_kernel, dim3(n_split_max, n_q, tab.n_seq), dim3(256), 0, st, sq,
                       static_cast<const float*>(q), rows_pad, n_q, n_kv, hd, cap, scale, part_o, part_ml);
    DS_LAUNCH_CHECK("attn_f32_kernel");
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
