// Token lattice (log-sum-exp + per-row top-M) and greedy acceptance (per-row arg-max, compare with the drafted
// path, longest accepted prefix), each in two forms.
//
// From logits in memory (any caller-supplied logits; float32 models): one pass over the float32 logits, 4 bytes per
// logit, HBM-bound.  A row is cut into segments so that even a few rows fill the chip; every wavefront keeps its
// running top-M as a sorted list spread over its lanes (lane i holds the i-th best) and only touches it when some
// lane's value beats the current M-th best, which becomes rare after the first few hundred values.  A second tiny
// kernel merges the per-wavefront partial results of each row.
//
// From the LM-head product's per-tile records (the round's path on bf16 models): the product's epilogue has already
// reduced every 128-column tile to a few numbers per row, so the logits are never written or read; see
// lattice_tiles_kernel and accept_tiles_kernel.
#include <limits.h>
#include <math.h>

#include "ds_common.h"
#include "ds_wave.h"

namespace ds {
namespace {

constexpr int kScanThreads = 256;
constexpr int kUnroll = 8;                                  // float4 loads in flight per thread
constexpr int kWaveChunk = kWave * 4 * kUnroll;             // 2048 logits per wavefront step
constexpr int kTile = kWaveChunk * (kScanThreads / kWave);  // 8192 logits per workgroup step

__device__ __forceinline__ bool beats(float v, int id, float w, int jd) {
  return v > w || (v == w && id < jd);
}

// Read lane `src` (wavefront-uniform) of a value into a scalar register.
__device__ __forceinline__ float lane_value(float v, int src) {
  return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), src));
}
__device__ __forceinline__ int lane_value(int v, int src) { return __builtin_amdgcn_readlane(v, src); }

// Insert the wavefront-uniform pair (x, xid) into the lane-distributed list sorted best-first: the
// entries it beats move one lane up (one DPP whole-wavefront shift), it lands in the gap.
__device__ __forceinline__ void list_insert(float& ev, int& eid, float x, int xid, int lane) {
  const int pos = __popcll(__ballot(beats(ev, eid, x, xid)));  // entries that stay ahead of x
  const float pv = __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(ev), 0x138, 0xF, 0xF, false));
  const int pid = __builtin_amdgcn_update_dpp(0, eid, 0x138, 0xF, 0xF, false);  // wave_shr:1
  if (lane == pos) {
    ev = x;
    eid = xid;
  } else if (lane > pos) {
    ev = pv;
    eid = pid;
  }
}

// Offer one value per lane to the list; only values beating the current m_max-th entry are inserted.
// Everything that crosses lanes here is a scalar read of one lane (no LDS-path permutes).
__device__ __forceinline__ void list_offer(float& ev, int& eid, float x, int xid, int m_max, int lane) {
  float thr = lane_value(ev, m_max - 1);
  int thrid = lane_value(eid, m_max - 1);
  unsigned long long mask = __ballot(beats(x, xid, thr, thrid));
  while (mask) {
    const int src = __ffsll((long long)mask) - 1;
    mask &= mask - 1;
    const float bx = lane_value(x, src);
    const int bid = lane_value(xid, src);
    if (!beats(bx, bid, thr, thrid)) continue;  // the bar moved up since the ballot
    list_insert(ev, eid, bx, bid, lane);
    thr = lane_value(ev, m_max - 1);
    thrid = lane_value(eid, m_max - 1);
  }
}

// Sort one (value, id) pair per lane across the wavefront, best first (bitonic network, 21 exchange steps).
// Used to start a list from 64 values at once instead of 64 sequential insertions.
__device__ __forceinline__ void wave_sort_best_first(float& v, int& id, int lane) {
#pragma unroll
  for (int k = 2; k <= kWave; k <<= 1) {
#pragma unroll
    for (int j = k >> 1; j > 0; j >>= 1) {
      const float ov = __shfl_xor(v, j);
      const int oid = __shfl_xor(id, j);
      const bool descending_block = (lane & k) == 0;     // k == 64: every lane
      const bool lower_lane = (lane & j) == 0;
      const bool want_better = lower_lane == descending_block;
      const bool take = want_better ? beats(ov, oid, v, id) : beats(v, id, ov, oid);
      if (take) {
        v = ov;
        id = oid;
      }
    }
  }
}

// Partial record of one wavefront for one row: { max, sum exp(v - max), m_max values, m_max ids }.
__host__ __device__ inline int rec_dwords(int m_max) { return 2 + 2 * m_max; }

// SOFTMAX = true: lattice scan (running max / sum of exp, top-m_max list).
// SOFTMAX = false: arg-max scan (m_max = 1): a plain per-lane running best, reduced once at the end.
template <bool SOFTMAX>
__global__ __launch_bounds__(kScanThreads) void scan_rows_kernel(const float* __restrict__ logits, int vocab,
                                                                 int m_max, int tiles_per_seg,
                                                                 uint32_t* __restrict__ partial) {
  const int row = blockIdx.y, seg = blockIdx.x, n_seg = gridDim.x;
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
  const float* rowp = logits + (size_t)row * (size_t)vocab;
  const bool vec = ((vocab & 3) == 0) && ((((uintptr_t)logits) & 15) == 0);

  float ev = -INFINITY;  // SOFTMAX: this lane's list entry; else: this lane's running best
  int eid = INT_MAX;
  float run_max = -INFINITY, run_sum = 0.f;
  bool list_empty = true;

  const int tile0 = seg * tiles_per_seg;
  for (int t = 0; t < tiles_per_seg; ++t) {
    const int base = (tile0 + t) * kTile + wave * kWaveChunk;
    if (base >= vocab) break;
    float v[kUnroll][4];
#pragma unroll
    for (int j = 0; j < kUnroll; ++j) {
      const int i0 = base + j * (kWave * 4) + lane * 4;
      if (vec && i0 + 3 < vocab) {
        typedef float vec4 __attribute__((ext_vector_type(4)));
        const vec4 q = __builtin_nontemporal_load(reinterpret_cast<const vec4*>(rowp + i0));  // read once
        v[j][0] = q.x; v[j][1] = q.y; v[j][2] = q.z; v[j][3] = q.w;
      } else {
#pragma unroll
        for (int c = 0; c < 4; ++c) v[j][c] = (i0 + c < vocab) ? rowp[i0 + c] : -INFINITY;
      }
    }
    if (!SOFTMAX) {
      // this lane's best of its 32 values (value descending, index ascending)
      float loc = -INFINITY;
      int loc_idx = INT_MAX;
#pragma unroll
      for (int j = 0; j < kUnroll; ++j)
#pragma unroll
        for (int c = 0; c < 4; ++c) {
          const int idx = base + j * (kWave * 4) + lane * 4 + c;
          if (idx < vocab && beats(v[j][c], idx, loc, loc_idx)) {
            loc = v[j][c];
            loc_idx = idx;
          }
        }
      if (beats(loc, loc_idx, ev, eid)) {
        ev = loc;
        eid = loc_idx;
      }
      continue;
    }
    // this lane's largest value (positions past the vocabulary were loaded as -inf)
    float lm = -INFINITY;
#pragma unroll
    for (int j = 0; j < kUnroll; ++j)
      lm = fmaxf(fmaxf(lm, fmaxf(v[j][0], v[j][1])), fmaxf(v[j][2], v[j][3]));
    if (lm > run_max) {
      run_sum *= __expf(run_max - lm);  // run_max = -inf gives 0 * 0
      run_max = lm;
    }
    if (run_max > -INFINITY) {
      // exp(v - run_max) as 2^(v * log2(e) - run_max * log2(e)): one fused multiply-add and one exp2 per value
      const float nm = -run_max * 1.4426950408889634f;
      float acc = 0.f;
#pragma unroll
      for (int j = 0; j < kUnroll; ++j)
#pragma unroll
        for (int c = 0; c < 4; ++c) acc += __builtin_amdgcn_exp2f(fmaf(v[j][c], 1.4426950408889634f, nm));
      run_sum += acc;
    }
    // top-M list.  `thr` is the value of the M-th entry (wavefront-uniform, only ever rises); nothing below
    // it can enter the list, so a step whose lane maxima all lie below it is done, and inside a step only the
    // values that reach it are offered (list_offer decides ties by index).
    int own = -1;  // index already in the list (skipped below)
    if (list_empty) {
      // start the list from the 64 per-lane bests in one sort; the bar is then already high
      float loc = -INFINITY;
      int loc_idx = INT_MAX;
#pragma unroll
      for (int j = 0; j < kUnroll; ++j)
#pragma unroll
        for (int c = 0; c < 4; ++c) {
          const int idx = base + j * (kWave * 4) + lane * 4 + c;
          if (idx < vocab && beats(v[j][c], idx, loc, loc_idx)) {
            loc = v[j][c];
            loc_idx = idx;
          }
        }
      ev = loc;
      eid = loc_idx;
      wave_sort_best_first(ev, eid, lane);
      own = loc_idx;
      list_empty = false;
    } else if (!__ballot(lm >= lane_value(ev, m_max - 1))) {
      continue;
    }
    float thr = lane_value(ev, m_max - 1);
#pragma unroll
    for (int j = 0; j < kUnroll; ++j)
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        const int idx = base + j * (kWave * 4) + lane * 4 + c;
        const bool ok = idx < vocab && idx != own && v[j][c] >= thr;
        if (__ballot(ok)) {
          list_offer(ev, eid, ok ? v[j][c] : -INFINITY, ok ? idx : INT_MAX, m_max, lane);
          thr = lane_value(ev, m_max - 1);
        }
      }
  }

  if (SOFTMAX) {  // wavefront reduction of (max, sum)
#pragma unroll
    for (int off = kWave / 2; off > 0; off >>= 1) {
      float om = __shfl_xor(run_max, off), os = __shfl_xor(run_sum, off);
      float nm = fmaxf(run_max, om);
      float a = (run_max > -INFINITY) ? run_sum * __expf(run_max - nm) : 0.f;
      float b = (om > -INFINITY) ? os * __expf(om - nm) : 0.f;
      run_max = nm;
      run_sum = a + b;
    }
  } else {  // wavefront reduction of the running best into lane 0
#pragma unroll
    for (int off = kWave / 2; off > 0; off >>= 1) {
      const float ov = __shfl_xor(ev, off);
      const int oid = __shfl_xor(eid, off);
      if (beats(ov, oid, ev, eid)) {
        ev = ov;
        eid = oid;
      }
    }
  }
  const int part = (row * n_seg + seg) * (kScanThreads / kWave) + wave;
  uint32_t* rec = partial + (size_t)part * rec_dwords(m_max);
  if (lane == 0) {
    rec[0] = __float_as_uint(run_max);
    rec[1] = __float_as_uint(run_sum);
  }
  if (lane < m_max) {
    rec[2 + lane] = __float_as_uint(ev);
    rec[2 + m_max + lane] = (uint32_t)eid;
  }
}

// Merge the partial top lists of one row; returns with lane i holding the i-th best overall.
// Entries are visited rank-major (all partials' best first), the first 64 sorted in one go.
__device__ __forceinline__ void merge_lists(const uint32_t* rec0, int n_part, int m_max, int lane, float& ev,
                                            int& eid) {
  ev = -INFINITY;
  eid = INT_MAX;
  const int total = n_part * m_max;
  for (int b = 0; b < total; b += kWave) {
    const int e = b + lane;
    float x = -INFINITY;
    int xid = INT_MAX;
    if (e < total) {
      const int rank = e / n_part, p = e - rank * n_part;
      const uint32_t* rec = rec0 + (size_t)p * rec_dwords(m_max);
      x = __uint_as_float(rec[2 + rank]);
      xid = (int)rec[2 + m_max + rank];
    }
    if (b == 0) {
      ev = x;
      eid = xid;
      wave_sort_best_first(ev, eid, lane);
    } else {
      list_offer(ev, eid, x, xid, m_max, lane);
    }
  }
}

__global__ __launch_bounds__(kWave) void lattice_merge_kernel(const float* __restrict__ logits, int vocab,
                                                              int m_max, float tau, int32_t eos_id,
                                                              int n_part, const uint32_t* __restrict__ partial,
                                                              int32_t* __restrict__ cand_id,
                                                              float* __restrict__ cand_logp,
                                                              int32_t* __restrict__ cand_cnt,
                                                              float* __restrict__ eos_logp,
                                                              float* __restrict__ lse_out) {
  const int row = blockIdx.x, lane = threadIdx.x;
  const uint32_t* rec0 = partial + (size_t)row * n_part * rec_dwords(m_max);
  float mx = -INFINITY;
  for (int p = lane; p < n_part; p += kWave)
    mx = fmaxf(mx, __uint_as_float(rec0[(size_t)p * rec_dwords(m_max)]));
#pragma unroll
  for (int off = kWave / 2; off > 0; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off));
  float sum = 0.f;
  for (int p = lane; p < n_part; p += kWave) {
    const uint32_t* rec = rec0 + (size_t)p * rec_dwords(m_max);
    float pm = __uint_as_float(rec[0]), ps = __uint_as_float(rec[1]);
    if (pm > -INFINITY) sum += ps * __expf(pm - mx);
  }
#pragma unroll
  for (int off = kWave / 2; off > 0; off >>= 1) sum += __shfl_xor(sum, off);
  const float lse = mx + logf(sum);

  float ev;
  int eid;
  merge_lists(rec0, n_part, m_max, lane, ev, eid);
  const float lp = ev - lse;
  if (lane < m_max) {
    cand_id[(size_t)row * m_max + lane] = eid;
    cand_logp[(size_t)row * m_max + lane] = lp;
  }
  // mass-adaptive pruning: smallest m with cumulative probability >= tau, float32 in candidate order
  int cnt = m_max;
  if (tau < 1.0f) {
    float cum = 0.f;
    bool done = false;
    for (int i = 0; i < m_max; ++i) {
      float p = expf(__shfl(lp, i));
      cum = __fadd_rn(cum, p);
      if (!done && cum >= tau) {
        cnt = i + 1;
        done = true;
      }
    }
  }
  if (lane == 0) {
    cand_cnt[row] = cnt;
    lse_out[row] = lse;
    eos_logp[row] = (eos_id >= 0) ? logits[(size_t)row * vocab + eos_id] - lse : 0.f;
  }
}

// The accepted-prefix rule for every sequence of the call, by one thread: am[row] holds every row's arg-max.
// Sequence s owns rows [row0[s], row0[s] + m[s] + 1); row i predicts the token after block row i, and path token n
// (0-based, = block row n + 1) is path_tok[tok_off[s] + n].  eos_accepted is stored last, after a system-scope
// fence: a host polling the last sequence's word in device-visible memory then sees every other output.
__device__ __forceinline__ void write_verdicts(const AcceptSeqs& sq, const int32_t* am, const int32_t* path_tok,
                                               const int32_t* path_len, int32_t eos_id, int32_t* n_accept,
                                               int32_t* next_token, int32_t* eos_accepted) {
  bool eos_flag[kMaxSeq];
  for (int s = 0; s < sq.n_seq; ++s) {
    int m = sq.m[s];
    if (path_len) {
      const int pl = path_len[s];
      m = pl < m ? (pl < 0 ? 0 : pl) : m;
    }
    const int32_t* a = am + sq.row0[s];
    const int32_t* tok = path_tok + sq.tok_off[s];
    int n = 0;
    bool eos = false;
    while (n < m && a[n] == tok[n]) {
      eos |= (eos_id >= 0 && tok[n] == eos_id);
      ++n;
    }
    const int nxt = a[n];
    eos |= (eos_id >= 0 && nxt == eos_id);
    n_accept[s] = n;
    next_token[s] = nxt;
    eos_flag[s] = eos;
    if (sq.carry && s == 0) {
      const int32_t before_last = n > 0 ? tok[n - 1] : sq.first[0];
      int32_t* c = sq.carry + DS_MAX_ROWS - 1 - n;
      for (int i = 0; i < n; ++i) c[i] = tok[i];
      c[n] = nxt;
      c[n + 1] = before_last;
      c[n + 2] = nxt;
    }
  }
  __threadfence_system();
  for (int s = 0; s < sq.n_seq; ++s) eos_accepted[s] = eos_flag[s] ? 1 : 0;
}

// One workgroup: arg-max of every row from the partial lists, then the accepted-prefix rule.
__global__ __launch_bounds__(1024) void accept_merge_kernel(int rows, int n_part,
                                                           const uint32_t* __restrict__ partial, AcceptSeqs sq,
                                                           const int32_t* __restrict__ path_tok,
                                                           const int32_t* __restrict__ path_len, int32_t eos_id,
                                                           int32_t* __restrict__ n_accept,
                                                           int32_t* __restrict__ next_token,
                                                           int32_t* __restrict__ argmax_out,
                                                           int32_t* __restrict__ eos_accepted) {
  __shared__ int32_t am[DS_MAX_ROWS];
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
  for (int r = wave; r < rows; r += (int)(blockDim.x / kWave)) {
    // arg-max over the per-wavefront winners of this row: plain (value, lower id) reduction
    const uint32_t* rec0 = partial + (size_t)r * n_part * rec_dwords(1);
    float ev = -INFINITY;
    int eid = INT_MAX;
    for (int p = lane; p < n_part; p += kWave) {
      const float x = __uint_as_float(rec0[(size_t)p * rec_dwords(1) + 2]);
      const int xid = (int)rec0[(size_t)p * rec_dwords(1) + 3];
      if (beats(x, xid, ev, eid)) {
        ev = x;
        eid = xid;
      }
    }
#pragma unroll
    for (int off = kWave / 2; off > 0; off >>= 1) {
      const float ov = __shfl_xor(ev, off);
      const int oid = __shfl_xor(eid, off);
      if (beats(ov, oid, ev, eid)) {
        ev = ov;
        eid = oid;
      }
    }
    if (lane == 0) {
      am[r] = eid;
      const int o = accept_out_index(sq, r);
      if (o >= 0) argmax_out[o] = eid;
    }
  }
  __syncthreads();
  if (threadIdx.x == 0) write_verdicts(sq, am, path_tok, path_len, eos_id, n_accept, next_token, eos_accepted);
}

// Same rule, fed by the LM-head product's own epilogue instead of a scan of the logits: tile_best[tile][row] is the
// largest logit of the row inside one tile of columns and its column (int bits in .y), tiles in column order,
// rows_pad rows per tile.  One workgroup per row reduces its records; the workgroup that arrives last (a counter
// behind the records, left at zero by the product) applies the accepted-prefix rule.  Every workgroup ends after
// one pass; nobody waits.
__global__ __launch_bounds__(256) void accept_tiles_kernel(int rows, int rows_pad, int n_tiles,
                                                          const float2* __restrict__ tile_best,
                                                          uint32_t* __restrict__ counter, int32_t* am,
                                                          AcceptSeqs sq, const int32_t* __restrict__ path_tok,
                                                          const int32_t* __restrict__ path_len, int32_t eos_id,
                                                          int32_t* __restrict__ n_accept,
                                                          int32_t* __restrict__ next_token,
                                                          int32_t* __restrict__ argmax_out,
                                                          int32_t* __restrict__ eos_accepted) {
  __shared__ float sv[4];
  __shared__ int si[4];
  __shared__ bool last;
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
  const int r = blockIdx.x;
  float ev = -INFINITY;
  int eid = INT_MAX;
#pragma unroll 8
  for (int t = threadIdx.x; t < n_tiles; t += (int)blockDim.x) {
    const float2 q = tile_best[(size_t)t * rows_pad + r];
    const int xid = __float_as_int(q.y);
    if (beats(q.x, xid, ev, eid)) {
      ev = q.x;
      eid = xid;
    }
  }
#pragma unroll
  for (int off = kWave / 2; off > 0; off >>= 1) {
    const float ov = __shfl_xor(ev, off);
    const int oid = __shfl_xor(eid, off);
    if (beats(ov, oid, ev, eid)) {
      ev = ov;
      eid = oid;
    }
  }
  if (lane == 0) {
    sv[wave] = ev;
    si[wave] = eid;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    for (int w = 1; w < (int)(blockDim.x / kWave); ++w)
      if (beats(sv[w], si[w], ev, eid)) {
        ev = sv[w];
        eid = si[w];
      }
    const int o = accept_out_index(sq, r);
    if (o >= 0) argmax_out[o] = eid;
    // The row's result goes out as a device-scope (write-through) store and has completed before the arrival is
    // counted; the last workgroup reads the results with device-scope loads.  No fence: a device-scope fence writes
    // back and invalidates a whole L2, which costs more than this kernel's work.
    __hip_atomic_store(&am[r], eid, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0)
    asm volatile("" ::: "memory");
    const uint32_t seen = __hip_atomic_fetch_add(counter, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    last = seen == (uint32_t)rows - 1u;
  }
  __syncthreads();
  if (!last) return;
  __shared__ int32_t ams[DS_MAX_ROWS];
  for (int i = threadIdx.x; i < rows; i += (int)blockDim.x)
    ams[i] = __hip_atomic_load(&am[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  __syncthreads();
  if (threadIdx.x == 0) {
    __hip_atomic_store(counter, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    write_verdicts(sq, ams, path_tok, path_len, eos_id, n_accept, next_token, eos_accepted);
  }
}

// ---- lattice straight from the LM-head product's per-tile records ---------------------------------------------
//
// The product leaves, per tile of 128 vocabulary columns and per row, the tile's two largest logits with their
// columns, its third largest value and its sum of exp(x - largest).  The log-sum-exp of a row follows from the
// records exactly as from the logits.  The top-M of the row is the top-M of all recorded pairs PROVIDED no tile hides
// a third value that could still enter it: a tile is "open" if its third value exceeds the M-th best found so far, or
// equals it while the tile's first column is lower than that entry's (equal logits rank by token id).  Open tiles
// are rare (three of a row's M best tokens within 128 consecutive ids); for each of them the workgroup recomputes the
// tile's 128 logits with the very MFMA sequence of the product (same operands, same order: the same bits) and offers
// them to the list, after which the result is exact.
typedef _Float16 lt_f16x8 __attribute__((ext_vector_type(8)));
typedef float lt_f32x4 __attribute__((ext_vector_type(4)));

constexpr int kTilesPerThread = 8;  // records held in registers per thread: at most 256 * 8 tiles per row
constexpr int kTileCols = 128;
constexpr int kOpenList = 64;

// The best (value descending, id ascending) of one pair per lane: its lane, wavefront-uniform; the pair in bv / bid.
__device__ __forceinline__ int wave_best(float v, int id, float& bv, int& bid) {
  const uint32_t key = ordered_bits(v);
  const uint32_t top = wave_max_u32(key);
  const unsigned long long at_top = __ballot(key == top);
  int src = __ffsll((long long)at_top) - 1;
  if (__popcll(at_top) > 1) {  // equal values: the lowest id among them
    const uint32_t idk = key == top ? 0xFFFFFFFFu - (uint32_t)id : 0u;
    const uint32_t low = wave_max_u32(idk);
    src = __ffsll((long long)__ballot(idk == low)) - 1;
  }
  bv = lane_value(v, src);
  bid = lane_value(id, src);
  return src;
}

// PER: tile records per thread (256 * PER >= tiles per row).
template <int PER>
__global__ __launch_bounds__(256) void lattice_tiles_kernel(const float4* __restrict__ rec, int rows_pad, int n_tiles,
                                                           int m_max, float tau, int32_t eos_id,
                                                           const float* __restrict__ eos_logit,
                                                           const uint16_t* __restrict__ wp,
                                                           const uint16_t* __restrict__ xt, int ksteps,
                                                           int32_t* __restrict__ cand_id,
                                                           float* __restrict__ cand_logp,
                                                           int32_t* __restrict__ cand_cnt,
                                                           float* __restrict__ eos_logp,
                                                           float* __restrict__ lse_out) {
  __shared__ float l_val[4][DS_MAX_TOPM];
  __shared__ int l_id[4][DS_MAX_TOPM];
  __shared__ float s_max[4], s_sum[4];
  __shared__ float thr_v;
  __shared__ int thr_i;
  __shared__ int n_open;
  __shared__ int open_tile[kOpenList];
  __shared__ float tile_vals[kTileCols];
  const int r = blockIdx.x, tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;

  float v1[PER], v2[PER], v3[PER], ss[PER];
  int i1[PER], i2[PER];
#pragma unroll
  for (int q = 0; q < PER; ++q) {
    const int t = q * 256 + tid;
    v1[q] = v2[q] = v3[q] = -INFINITY;
    ss[q] = 0.f;
    i1[q] = i2[q] = INT_MAX;
    if (t < n_tiles) {
      const float4 a = rec[((size_t)t * rows_pad + r) * 2], b = rec[((size_t)t * rows_pad + r) * 2 + 1];
      v1[q] = a.x;
      i1[q] = __float_as_int(a.y);
      v2[q] = a.z;
      i2[q] = __float_as_int(a.w);
      v3[q] = b.x;
      ss[q] = b.y;
    }
  }

  // log-sum-exp pieces of this wavefront
  float mx = -INFINITY;
#pragma unroll
  for (int q = 0; q < PER; ++q) mx = fmaxf(mx, v1[q]);
#pragma unroll
  for (int off = kWave / 2; off > 0; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off));
  float sum = 0.f;
#pragma unroll
  for (int q = 0; q < PER; ++q)
    if (v1[q] > -INFINITY) sum += ss[q] * __expf(v1[q] - mx);
#pragma unroll
  for (int off = kWave / 2; off > 0; off >>= 1) sum += __shfl_xor(sum, off);

  // this wavefront's best m_max of its recorded pairs: m_max rounds of arg-max over each lane's best open pair
  // (a tile's second value opens when its first has been taken)
  float cv[PER];
  int ci[PER];
#pragma unroll
  for (int q = 0; q < PER; ++q) {
    cv[q] = v1[q];
    ci[q] = i1[q];
  }
  uint32_t second = 0u;  // bit q: tile q already gave its first value
  auto lane_best = [&](float& lb, int& li, int& lq) {
    lb = -INFINITY;
    li = INT_MAX;
    lq = 0;
#pragma unroll
    for (int q = 0; q < PER; ++q)
      if (beats(cv[q], ci[q], lb, li)) {
        lb = cv[q];
        li = ci[q];
        lq = q;
      }
  };
  float lb;
  int li, lq;
  lane_best(lb, li, lq);
  float ev = -INFINITY;
  int eid = INT_MAX;
  for (int i = 0; i < m_max; ++i) {
    float bv;
    int bid;
    const int src = wave_best(lb, li, bv, bid);
    if (lane == i) {
      ev = bv;
      eid = bid;
    }
    if (lane == src) {
#pragma unroll
      for (int q = 0; q < PER; ++q)
        if (q == lq) {
          const bool was_second = (second >> q) & 1u;
          cv[q] = was_second ? -INFINITY : v2[q];
          ci[q] = was_second ? INT_MAX : i2[q];
          second |= 1u << q;
        }
      lane_best(lb, li, lq);
    }
  }
  if (lane < m_max) {
    l_val[wave][lane] = ev;
    l_id[wave][lane] = eid;
  }
  if (lane == 0) {
    s_max[wave] = mx;
    s_sum[wave] = sum;
  }
  __syncthreads();

  // wavefront 0 merges the four lists (one entry per lane) the same way; from here on it owns the list, lane i
  // holding the i-th best
  if (wave == 0) {
    float xv = -INFINITY;
    int xi = INT_MAX;
    if (lane < 4 * m_max) {
      xv = l_val[lane / m_max][lane % m_max];
      xi = l_id[lane / m_max][lane % m_max];
    }
    ev = -INFINITY;
    eid = INT_MAX;
    for (int i = 0; i < m_max; ++i) {
      float bv;
      int bid;
      const int src = wave_best(xv, xi, bv, bid);
      if (lane == i) {
        ev = bv;
        eid = bid;
      }
      if (lane == src) {
        xv = -INFINITY;
        xi = INT_MAX;
      }
    }
    if (lane == m_max - 1) {
      thr_v = ev;
      thr_i = eid;
    }
    if (lane == 0) n_open = 0;
  }
  __syncthreads();

  // open tiles: recompute and offer, until none is left (a tile is visited at most once)
  for (;;) {
    const float tv = thr_v;
    const int ti = thr_i;
#pragma unroll
    for (int q = 0; q < PER; ++q) {
      const int t = q * 256 + tid;
      if (t < n_tiles && (v3[q] > tv || (v3[q] == tv && t * kTileCols < ti))) {
        const int k = atomicAdd(&n_open, 1);
        if (k < kOpenList) {
          open_tile[k] = t;
          v3[q] = -INFINITY;  // visited
        }
      }
    }
    __syncthreads();
    const int n_now = n_open < kOpenList ? n_open : kOpenList;
    if (n_now == 0) break;
    for (int u = 0; u < n_now; ++u) {
      const int t = open_tile[u];
      // the product's arithmetic for this tile and this row's block of 16: wavefront w owns column blocks w and 4 + w
      const uint16_t* w0 = wp + ((size_t)(t * 8 + wave) * ksteps) * 512 + lane * 8;
      const uint16_t* w1 = wp + ((size_t)(t * 8 + 4 + wave) * ksteps) * 512 + lane * 8;
      const uint16_t* xb = xt + ((size_t)(r >> 4) * ksteps) * 512 + lane * 8;
      lt_f32x4 acc0 = {0.f, 0.f, 0.f, 0.f}, acc1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll 4
      for (int ks = 0; ks < ksteps; ++ks) {
        const lt_f16x8 a0 = *reinterpret_cast<const lt_f16x8*>(w0 + (size_t)ks * 512);
        const lt_f16x8 a1 = *reinterpret_cast<const lt_f16x8*>(w1 + (size_t)ks * 512);
        const lt_f16x8 bx = *reinterpret_cast<const lt_f16x8*>(xb + (size_t)ks * 512);
        acc0 = __builtin_amdgcn_mfma_f32_16x16x32_f16(a0, bx, acc0, 0, 0, 0);
        acc1 = __builtin_amdgcn_mfma_f32_16x16x32_f16(a1, bx, acc1, 0, 0, 0);
      }
      if ((lane & 15) == (r & 15)) {
        const int g = lane >> 4;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          tile_vals[wave * 16 + g * 4 + e] = acc0[e];
          tile_vals[(4 + wave) * 16 + g * 4 + e] = acc1[e];
        }
      }
      __syncthreads();
      if (wave == 0) {
        const float4 a = rec[((size_t)t * rows_pad + r) * 2];
        const int skip1 = __float_as_int(a.y), skip2 = __float_as_int(a.w);  // already in the list (or beaten)
#pragma unroll
        for (int h = 0; h < kTileCols / kWave; ++h) {
          const int id = t * kTileCols + h * kWave + lane;
          const bool ok = id != skip1 && id != skip2;
          list_offer(ev, eid, ok ? tile_vals[h * kWave + lane] : -INFINITY, ok ? id : INT_MAX, m_max, lane);
        }
      }
      __syncthreads();
    }
    if (wave == 0) {
      if (lane == m_max - 1) {
        thr_v = ev;
        thr_i = eid;
      }
      if (lane == 0) n_open = 0;
    }
    __syncthreads();
  }
  if (wave != 0) return;

  float all_max = fmaxf(fmaxf(s_max[0], s_max[1]), fmaxf(s_max[2], s_max[3]));
  float all_sum = 0.f;
#pragma unroll
  for (int w = 0; w < 4; ++w)
    if (s_max[w] > -INFINITY) all_sum += s_sum[w] * __expf(s_max[w] - all_max);
  const float lse = all_max + logf(all_sum);
  const float lp = ev - lse;
  if (lane < m_max) {
    cand_id[(size_t)r * m_max + lane] = eid;
    cand_logp[(size_t)r * m_max + lane] = lp;
  }
  int cnt = m_max;
  if (tau < 1.0f) {
    float cum = 0.f;
    bool done = false;
    for (int i = 0; i < m_max; ++i) {
      float p = expf(__shfl(lp, i));
      cum = __fadd_rn(cum, p);
      if (!done && cum >= tau) {
        cnt = i + 1;
        done = true;
      }
    }
  }
  if (lane == 0) {
    cand_cnt[r] = cnt;
    lse_out[r] = lse;
    eos_logp[r] = (eos_id >= 0) ? eos_logit[r] - lse : 0.f;
  }
}

struct ScanPlan {
  int n_seg, tiles_per_seg, n_part;
};

ScanPlan plan_scan(int rows, int vocab) {
  int tiles = ceil_div(vocab, kTile);
  // as many workgroups as are resident at once (7 wavefronts per SIMD: 1792 workgroups of 4), no second round
  int want = 1792 / rows;
  int n_seg = want < 1 ? 1 : (want > tiles ? tiles : want);
  int tps = ceil_div(tiles, n_seg);
  n_seg = ceil_div(tiles, tps);
  return {n_seg, tps, n_seg * (kScanThreads / kWave)};
}

}  // namespace

size_t lattice_ws_bytes(int rows, int vocab, int m_max) {
  ScanPlan p = plan_scan(rows, vocab);
  return align_up((size_t)rows * p.n_part * rec_dwords(m_max) * sizeof(uint32_t), 256);
}

int launch_lattice(const float* logits, int rows, int vocab, int m_max, float tau, int32_t eos_id,
                   int32_t* cand_id, float* cand_logp, int32_t* cand_cnt, float* eos_logp, float* lse,
                   void* ws, size_t ws_bytes, hipStream_t st) {
  DS_REQUIRE(ws_bytes >= lattice_ws_bytes(rows, vocab, m_max), DS_E_CAPACITY,
             "lattice workspace: need %zu bytes, got %zu", lattice_ws_bytes(rows, vocab, m_max), ws_bytes);
  ScanPlan p = plan_scan(rows, vocab);
  uint32_t* partial = static_cast<uint32_t*>(ws);
  hipLaunchKernelGGL(scan_rows_kernel<true>, dim3(p.n_seg, rows), dim3(kScanThreads), 0, st, logits, vocab,
                     m_max, p.tiles_per_seg, partial);
  DS_LAUNCH_CHECK("scan_rows_kernel<softmax>");
  hipLaunchKernelGGL(lattice_merge_kernel, dim3(rows), dim3(kWave), 0, st, logits, vocab, m_max, tau, eos_id,
                     p.n_part, partial, cand_id, cand_logp, cand_cnt, eos_logp, lse);
  DS_LAUNCH_CHECK("lattice_merge_kernel");
  return DS_OK;
}

size_t accept_ws_bytes(int rows, int vocab) { return lattice_ws_bytes(rows, vocab, 1); }

int launch_argmax_accept(const float* logits, int rows, int vocab, const AcceptSeqs& sq, const int32_t* path_tok,
                         const int32_t* path_len, int32_t eos_id, int32_t* n_accept, int32_t* next_token,
                         int32_t* argmax, int32_t* eos_accepted, void* ws, size_t ws_bytes, hipStream_t st) {
  DS_REQUIRE(ws_bytes >= accept_ws_bytes(rows, vocab), DS_E_CAPACITY,
             "acceptance workspace: need %zu bytes, got %zu", accept_ws_bytes(rows, vocab), ws_bytes);
  DS_REQUIRE(rows >= 1 && rows <= DS_MAX_ROWS, DS_E_SHAPE, "acceptance rows %d outside [1, %d]", rows,
             DS_MAX_ROWS);
  ScanPlan p = plan_scan(rows, vocab);
  uint32_t* partial = static_cast<uint32_t*>(ws);
  hipLaunchKernelGGL(scan_rows_kernel<false>, dim3(p.n_seg, rows), dim3(kScanThreads), 0, st, logits, vocab, 1,
                     p.tiles_per_seg, partial);
  DS_LAUNCH_CHECK("scan_rows_kernel<argmax>");
  hipLaunchKernelGGL(accept_merge_kernel, dim3(1), dim3(1024), 0, st, rows, p.n_part, partial, sq, path_tok, path_len,
                     eos_id, n_accept, next_token, argmax, eos_accepted);
  DS_LAUNCH_CHECK("accept_merge_kernel");
  return DS_OK;
}

bool lattice_tiles_supported(int n_tiles, int tile_cols) {
  return tile_cols == kTileCols && n_tiles >= 1 && n_tiles <= 256 * kTilesPerThread;
}

int launch_lattice_tiles(const void* rec, int rows, int n_tiles, int m_max, float tau, int32_t eos_id,
                         const float* eos_logit, const void* wp, const void* xt, int K, int32_t* cand_id,
                         float* cand_logp, int32_t* cand_cnt, float* eos_logp, float* lse, hipStream_t st) {
  DS_REQUIRE(rows >= 1 && rows <= DS_MAX_ROWS, DS_E_SHAPE, "lattice rows %d outside [1, %d]", rows, DS_MAX_ROWS);
  DS_REQUIRE(lattice_tiles_supported(n_tiles, kTileCols), DS_E_SHAPE, "lattice from tile records: %d tiles unsupported",
             n_tiles);
  DS_REQUIRE(m_max >= 1 && m_max <= DS_MAX_TOPM, DS_E_SHAPE, "M_max %d outside [1, %d]", m_max, DS_MAX_TOPM);
  DS_REQUIRE(rec && wp && xt && (K & 31) == 0 && (eos_id < 0 || eos_logit), DS_E_INVALID,
             "lattice from tile records: missing operand");
  const int per = ceil_div(n_tiles, 256);
  auto go = [&](auto kernel) {
    hipLaunchKernelGGL(kernel, dim3(rows), dim3(256), 0, st, static_cast<const float4*>(rec),
                       ceil_div(rows, 16) * 16, n_tiles, m_max, tau, eos_id, eos_logit,
                       static_cast<const uint16_t*>(wp), static_cast<const uint16_t*>(xt), K >> 5, cand_id, cand_logp,
                       cand_cnt, eos_logp, lse);
  };
  if (per <= 1) go(lattice_tiles_kernel<1>);
  else if (per <= 2) go(lattice_tiles_kernel<2>);
  else if (per <= 3) go(lattice_tiles_kernel<3>);
  else if (per <= 5) go(lattice_tiles_kernel<5>);
  else go(lattice_tiles_kernel<kTilesPerThread>);
  DS_LAUNCH_CHECK("lattice_tiles_kernel");
  return DS_OK;
}

int launch_tiles_accept(float2* tile_best, int rows, int n_tiles, const AcceptSeqs& sq, const int32_t* path_tok,
                        const int32_t* path_len, int32_t eos_id, int32_t* n_accept, int32_t* next_token,
                        int32_t* argmax, int32_t* eos_accepted, hipStream_t st) {
  DS_REQUIRE(rows >= 1 && rows <= DS_MAX_ROWS, DS_E_SHAPE, "acceptance rows %d outside [1, %d]", rows,
             DS_MAX_ROWS);
  DS_REQUIRE(tile_best && n_tiles >= 1, DS_E_INVALID, "acceptance from tiles: no tile records");
  const int rows_pad = ceil_div(rows, 16) * 16;
  // behind the records: the arrival counter (64 words reserved), then one arg-max word per row
  uint32_t* counter = reinterpret_cast<uint32_t*>(tile_best + (size_t)n_tiles * rows_pad);
  int32_t* am = reinterpret_cast<int32_t*>(counter + 64);
  hipLaunchKernelGGL(accept_tiles_kernel, dim3(rows), dim3(256), 0, st, rows, rows_pad, n_tiles, tile_best, counter,
                     am, sq, path_tok, path_len, eos_id, n_accept, next_token, argmax, eos_accepted);
  DS_LAUNCH_CHECK("accept_tiles_kernel");
  return DS_OK;
}

}  // namespace ds
