// Internal declarations shared by the library's translation units (not part of the C ABI).
#pragma once

#include <hip/hip_runtime.h>
#include <hip/hip_bf16.h>
#include <stdint.h>
#include <stddef.h>

#include "ds.h"

namespace ds {

// ---- error reporting -------------------------------------------------------------------------
int fail(int code, const char* fmt, ...);  // records the thread's error text, returns code
void clear_error();

#define DS_REQUIRE(cond, code, ...) \
  do {                              \
    if (!(cond)) return ::ds::fail((code), __VA_ARGS__); \
  } while (0)

#define DS_HIP_CHECK(expr)                                                                  \
  do {                                                                                      \
    hipError_t e_ = (expr);                                                                 \
    if (e_ != hipSuccess) return ::ds::fail(DS_E_HIP, "%s: %s", #expr, hipGetErrorString(e_)); \
  } while (0)

#define DS_LAUNCH_CHECK(name)                                                                  \
  do {                                                                                         \
    hipError_t e_ = hipGetLastError();                                                         \
    if (e_ != hipSuccess) return ::ds::fail(DS_E_HIP, "launch %s: %s", name, hipGetErrorString(e_)); \
  } while (0)

static inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }
static inline int ceil_div(int a, int b) { return (a + b - 1) / b; }

constexpr int kWave = 64;

// ---- activation tile order (bf16 GEMM input) ---------------------------------------------------
// A bf16 activation matrix X[M, K] that feeds a GEMM is kept in "tile order": tiles of 16 rows x 32
// columns, tile (mb, ks) at ((mb * K/32) + ks) * 512 elements; inside a tile the 8 consecutive
// columns (8g .. 8g+7) of row j sit at lane (16g + j), i.e. element offset (16g + j) * 8.  This is
// the register image of the 16x16x32 bf16 MFMA's 16-wide operand, so a wave fetches one tile with a
// single coalesced 16-byte-per-lane load.  Rows are padded to a multiple of 16 (pad rows hold zeros
// or stale finite values; their products land in accumulator columns that are never stored).
__host__ __device__ static inline size_t xt_offset(int m, int k, int K) {
  int mb = m >> 4, j = m & 15, ks = k >> 5, g = (k >> 3) & 3, e = k & 7;
  return ((size_t)mb * (size_t)(K >> 5) + (size_t)ks) * 512 + (size_t)((g << 4) + j) * 8 + e;
}

// ---- sequences of one forward call ------------------------------------------------------------------
// A forward call carries the rows of up to kMaxSeq independent sequences through ONE pass over the weights
// (everything except attention and the cache append works row by row, so the rows of different sequences simply
// share the products).  Sequence s owns rows [row0[s], row0[s] + n_rows[s]); row0[s] is a multiple of 16 (the rows
// between two sequences are padding: finite, never stored anywhere that counts) and row0[n_seq] is the call's total
// row count.  Passed to kernels by value.
constexpr int kMaxSeq = 8;
struct SeqTable {
  int n_seq;
  int row0[kMaxSeq + 1];
  int n_rows[kMaxSeq];     // rows of the sequence in this call
  int n_a[kMaxSeq];        // the first n_a rows read their token from tok_a[off_a + i], the rest from tok_b[off_b + i - n_a]
  int off_a[kMaxSeq];      //   (or are `fill` if tok_b is NULL)
  int off_b[kMaxSeq];
  int pos0[kMaxSeq];       // absolute position of the sequence's first row = its committed cache length
  int n_causal[kMaxSeq];   // rows [0, n_causal) are causal real-token rows, the rest see every key
  int tail0[kMaxSeq];      // first row (within the sequence) whose final-normed state is handed on, and
  int tail_base[kMaxSeq];  //   the row it gets in the compact hand-on array
  void* kc[kMaxSeq];       // this layer's key / value cache of the sequence
  void* vc[kMaxSeq];
};
// The sequence a row belongs to, or -1 for a padding row.
__host__ __device__ static inline int seq_of_row(const SeqTable& t, int r) {
  int s = 0;
  while (s + 1 < t.n_seq && r >= t.row0[s + 1]) ++s;
  return (r - t.row0[s] < t.n_rows[s]) ? s : -1;
}

// Sequences of one verification call as the acceptance kernels see them: sequence s owns rows [row0[s], row0[s] +
// m[s] + 1) of the verifier pass; its path token n is path_tok[tok_off[s] + n]; its arg-max row i is written to
// argmax[out_off[s] + i] (rows of no sequence are written nowhere).
// carry (single-sequence calls; NULL: none): DS_MAX_ROWS + 2 words that receive what the next round reads from the
// device, namely the n_accept + 1 committed tokens right-aligned in carry[0, DS_MAX_ROWS), then the token before the
// last committed one and the last committed one.  first: the token of the sequence's row 0 (read before carry is
// written, so carry[DS_MAX_ROWS + 1] may be that very word).
struct AcceptSeqs {
  int n_seq;
  int row0[kMaxSeq], m[kMaxSeq], tok_off[kMaxSeq], out_off[kMaxSeq];
  const int32_t* first;
  int32_t* carry;
};
__host__ __device__ static inline int accept_out_index(const AcceptSeqs& q, int r) {
  for (int s = 0; s < q.n_seq; ++s)
    if (r >= q.row0[s] && r <= q.row0[s] + q.m[s]) return q.out_off[s] + r - q.row0[s];
  return -1;
}

// ---- lattice / acceptance kernels (k_lattice.hip) ----------------------------------------------
size_t lattice_ws_bytes(int rows, int vocab, int m_max);
int launch_lattice(const float* logits, int rows, int vocab, int m_max, float tau, int32_t eos_id,
                   int32_t* cand_id, float* cand_logp, int32_t* cand_cnt, float* eos_logp, float* lse,
                   void* ws, size_t ws_bytes, hipStream_t st);
size_t accept_ws_bytes(int rows, int vocab);
int launch_argmax_accept(const float* logits, int rows, int vocab, const AcceptSeqs& sq, const int32_t* path_tok,
                         const int32_t* path_len, int32_t eos_id, int32_t* n_accept, int32_t* next_token,
                         int32_t* argmax, int32_t* eos_accepted, void* ws, size_t ws_bytes, hipStream_t st);
// The same verdict from per-tile (largest logit, column) records written by the LM-head product's epilogue
// (layout and size: gemm_bf16_best_bytes, plus DS_MAX_ROWS words behind it).
int launch_tiles_accept(float2* tile_best, int rows, int n_tiles, const AcceptSeqs& sq, const int32_t* path_tok,
                        const int32_t* path_len, int32_t eos_id, int32_t* n_accept, int32_t* next_token,
                        int32_t* argmax, int32_t* eos_accepted, hipStream_t st);

// The lattice from the LM-head product's per-tile records (GemmEpilogue::kTop layout, tiles of 128 columns); wp / xt
// are the product's own operands (stream-order weights, tile-order activations), re-read for the rare tile whose
// records do not settle the top-M.  eos_logit: rows_pad floats written by the product (needed if eos_id >= 0).
bool lattice_tiles_supported(int n_tiles, int tile_cols);
int launch_lattice_tiles(const void* rec, int rows, int n_tiles, int m_max, float tau, int32_t eos_id,
                         const float* eos_logit, const void* wp, const void* xt, int K, int32_t* cand_id,
                         float* cand_logp, int32_t* cand_cnt, float* eos_logp, float* lse, hipStream_t st);

// ---- path search (k_cps.hip) --------------------------------------------------------------------
int launch_cps(const int32_t* cand_id, const float* cand_logp, const int32_t* cand_cnt,
               const float* eos_logp, int batch, int K, int m_max, int B, float lambda,
               const float* table, int log2_size, const int32_t* ctx, int32_t eos_id, int32_t* path,
               int32_t* path_len, float* path_score, int32_t* mirror, void* ws, size_t ws_bytes, hipStream_t st);
size_t cps_ws_bytes(int batch, int K, int m_max);

// ---- path search with a tiny causal LM as the proxy (k_cps_lm.hip) ------------------------------------
constexpr int kLmBeam = kMaxSeq;  // beam slots: each is one sequence of the proxy's forward call
constexpr int kLmMaxK = 256;
constexpr int kLmParts = 32;  // vocabulary segments the log-sum-exp of a proxy row is gathered from
// Device-resident state of one search (all written by the kernels; the host only passes the pointer on).
struct LmSearchState {
  int32_t tok[2][kLmBeam];   // [parity][slot] last token of each live hypothesis = input of the next proxy step
  float score[2][kLmBeam];
  int32_t par[kLmBeam];      // slot (of the previous depth) each new slot descends from
  int32_t n_live, finished, out_len;
  float out_score;
  float2 part[kLmBeam][kLmParts];       // per slot and vocabulary segment: (largest logit, sum of exp(x - largest))
  int32_t bp_tok[kLmMaxK][kLmBeam];     // back-pointers: token and parent slot of (depth, slot)
  int32_t bp_par[kLmMaxK][kLmBeam];
};
// One launch of the cache copy: destination d <- source src_of[d] (or the slot named by a device array).
struct KvCopyPlan {
  void* dst_k[2 * kMaxSeq];
  void* dst_v[2 * kMaxSeq];
  const void* src_k[kMaxSeq];
  const void* src_v[kMaxSeq];
  int src_of[2 * kMaxSeq];
  int n_dst, n_src;
};
int launch_lm_init(LmSearchState* st, hipStream_t s);
int launch_lm_score(const float* logits, int n_rows, int vocab, LmSearchState* st, hipStream_t s);
int launch_lm_beam_step(LmSearchState* st, const float* logits, int vocab, const int32_t* cand_id,
                        const float* cand_logp, const int32_t* cand_cnt, const float* eos_logp, int i, int K,
                        int m_max, int B, float lambda, int32_t eos_id, hipStream_t s);
int launch_lm_backtrack(const LmSearchState* st, int K, int32_t* path, int32_t* path_len, float* path_score,
                        hipStream_t s);
// Bytes [lo, hi) of each of the n_segments (layer, head) segments (head_bytes apart) of every destination cache.
int launch_kv_copy(const KvCopyPlan& plan, const int32_t* par, const LmSearchState* st, int n_segments,
                   size_t head_bytes, size_t lo, size_t hi, hipStream_t s);

// ---- stochastic acceptance and refinement update (k_sample.hip) -----------------------------------
size_t sample_ws_bytes(int m);
int launch_sample_accept(const float* p_logits, const float* q_logits, int m, int vocab, const int32_t* block,
                         const int32_t* path_len, const float* u, int32_t eos_id, int32_t* n_accept,
                         int32_t* next_token, int32_t* eos_accepted, float* alpha, void* ws, size_t ws_bytes,
                         hipStream_t st);
int launch_refine_select(const int32_t* cand_id, const float* cand_logp, const int32_t* cand_cnt,
                         const float* eos_logp, const float* lse, int K, int m_max, int n_update, int32_t mask_id,
                         int32_t* block_tokens, int32_t* o_id, float* o_logp, int32_t* o_cnt, float* o_eos,
                         float* o_lse, hipStream_t st);

}  // namespace ds
