// Model handle and the forward passes behind ds_prefill / ds_draft_block / ds_lm_head / ds_lm_head_tiles /
// ds_lattice_from_tiles / ds_verify_block.  Host code only orchestrates: every arithmetic step runs in a kernel.
#include <math.h>
#include <string.h>

#include <new>
#include <vector>

#include "ds_act.h"
#include "ds_common.h"

using namespace ds;

namespace {

struct PackedLayer {
  const void *wqkv, *wo, *wgu, *wdown;  // bf16 stream order (wgu: see ds_model::fused_gu)
};

// Carve-up of the caller's workspace for a call with `rows` rows (all offsets 256-byte aligned).
struct Workspace {
  float* x;        // [rows, d] residual stream
  float2* cs;      // [rows, hd/2] rotary table
  void* h;         // GEMM input, d columns
  void* q;         // [n_q][rows_pad, hd]
  void* att;       // GEMM input, n_q*hd columns
  void* act;       // GEMM input, d_ffn columns
  void* y;         // GEMM input, d columns (final-normed rows)
  void* y_tail;    // GEMM input, d columns: the final-normed rows from hidden_row0 on, re-based to row 0
  float* gemm_out; // split-K planes of the widest projection
  float* att_o;    // attention partials
  float* att_ml;
  float* logits;   // [rows, vocab]
  void* scan;      // acceptance partials
  size_t scan_bytes;
  void* tile_rec;  // per LM-head column tile and row: arg-max records (greedy acceptance) or lattice records
  float* eos_col;  // [rows_pad] EOS logits exported by the LM-head product
  void* lat;       // lattice scan partials (unfused path)
  size_t lat_bytes;
  void* sample;    // stochastic acceptance: log-sum-exp of the verifier and drafter rows
  size_t sample_bytes;
  size_t total;
};

}  // namespace

// One sequence's KV cache of a model: the two caller buffers and the committed length.
struct ds_kv {
  ds_model* owner;
  void *k, *v;
  int len;
};

struct ds_model {
  ds_model_cfg cfg;
  const void* embed;
  std::vector<ds_layer_weights> canon;
  std::vector<PackedLayer> packed;
  const float* final_norm;
  const void* lm_head;  // bf16: stream order; f32: canonical
  ds_kv self;  // the cache given to ds_model_create (what the single-sequence calls use)
  size_t esize;
  uint32_t* ovf = nullptr;  // [dev] activation-overflow counter (bf16 models: a word of the packed buffer's tail)
  // bf16 models whose gate / up product takes one plane, or two equal ones (a function of its shape alone): gate
  // and up are packed as a pair with alternating 16-row blocks (pair_gu).  One plane (fused_gu): the product's
  // epilogue applies SwiGLU itself, always.  Two planes: up to kFuseTwoRows rows the workgroups walk both halves of K
  // and fuse (measured faster there), above that the two planes are written and the SwiGLU kernel reads the paired
  // columns; both ways produce the same bits.
  bool fused_gu = false, pair_gu = false;
  // what the last draft pass left behind for ds_lm_head(hidden = NULL): the block rows as a GEMM input
  const void* tail_ptr = nullptr;
  const void* tail_ws = nullptr;
  int tail_rows = 0;
  // what ds_lm_head_tiles left behind for ds_lattice_from_tiles: the product's activation operand (bf16 models,
  // records in the workspace) or the logits (float32 models)
  const void* rec_ws = nullptr;
  const void* rec_y = nullptr;
  const float* rec_logits = nullptr;
  int rec_rows = 0;
  int32_t rec_eos = -1;
};

namespace {

int n_qkv(const ds_model_cfg& c) { return (c.n_q + 2 * c.n_kv) * c.head_dim; }

int validate_cfg(const ds_model_cfg* c) {
  DS_REQUIRE(c, DS_E_INVALID, "cfg is NULL");
  DS_REQUIRE(c->dtype == DS_F32 || c->dtype == DS_BF16, DS_E_UNSUPPORTED, "dtype %d is neither DS_F32 nor DS_BF16",
             c->dtype);
  DS_REQUIRE(c->n_layers >= 1 && c->d_model >= 1 && c->n_q >= 1 && c->n_kv >= 1 && c->head_dim >= 2 &&
                 c->d_ffn >= 1 && c->vocab >= 2 && c->kv_capacity >= 1,
             DS_E_SHAPE, "model dimensions must be positive");
  DS_REQUIRE(c->n_q % c->n_kv == 0, DS_E_SHAPE, "n_q %d is not a multiple of n_kv %d", c->n_q, c->n_kv);
  DS_REQUIRE(c->d_model <= 8192 && c->d_model % 4 == 0, DS_E_SHAPE, "d_model %d: need a multiple of 4, at most 8192",
             c->d_model);
  DS_REQUIRE(c->d_ffn % 4 == 0, DS_E_SHAPE, "d_ffn %d: need a multiple of 4", c->d_ffn);
  DS_REQUIRE(c->head_dim % 2 == 0 && c->head_dim <= 128, DS_E_UNSUPPORTED, "head_dim %d: need even and <= 128",
             c->head_dim);
  DS_REQUIRE(c->rope_base > 1.f && c->rms_eps >= 0.f, DS_E_INVALID, "rope_base must exceed 1, rms_eps >= 0");
  if (c->dtype == DS_BF16) {
    DS_REQUIRE(c->head_dim == 128, DS_E_UNSUPPORTED, "bf16 path needs head_dim 128 (got %d)", c->head_dim);
    DS_REQUIRE(c->d_model % 128 == 0 && c->d_ffn % 128 == 0 && c->vocab % 16 == 0, DS_E_SHAPE,
               "bf16 path needs d_model %% 128 == 0, d_ffn %% 128 == 0, vocab %% 16 == 0");
    DS_REQUIRE(c->kv_capacity % 64 == 0, DS_E_SHAPE, "bf16 path needs kv_capacity %% 64 == 0 (got %d)",
               c->kv_capacity);
  }
  return DS_OK;
}

size_t esize_of(int dtype) { return dtype == DS_BF16 ? 2 : 4; }

constexpr int kFuseTwoRows = 48;  // a gate / up pair of two planes is fused up to this many rows
constexpr size_t kFlagBytes = 256;  // tail of the packed buffer: weight-range flag written by the packing kernels

size_t packed_bytes_of(const ds_model_cfg& c) {
  if (c.dtype != DS_BF16) return 0;
  const size_t d = c.d_model, f = c.d_ffn, qo = (size_t)c.n_q * c.head_dim;
  const size_t per_layer = ((size_t)n_qkv(c) * d + d * qo + 2 * f * d + d * f) * 2;
  return per_layer * c.n_layers + (size_t)c.vocab * d * 2 + kFlagBytes;
}

size_t kv_bytes_of(const ds_model_cfg& c) {
  return (size_t)c.n_layers * c.n_kv * c.kv_capacity * c.head_dim * esize_of(c.dtype);
}

int widest_split_floats(const ds_model_cfg& c, int rows, size_t* out) {
  // largest rows x N x splits over the four projections of a layer
  size_t best = 0;
  const int d = c.d_model, f = c.d_ffn, qo = c.n_q * c.head_dim;
  const int shapes[4][2] = {{n_qkv(c), d}, {d, qo}, {2 * f, d}, {d, f}};
  for (auto& s : shapes) {
    const int sp = c.dtype == DS_BF16 ? gemm_bf16_splits(s[0], s[1], &s == &shapes[2] ? 2 : 1) : 1;
    const size_t v = (size_t)rows * s[0] * sp;
    best = v > best ? v : best;
  }
  *out = best;
  return DS_OK;
}

Workspace carve(const ds_model_cfg& c, int rows, void* base) {
  Workspace w{};
  const size_t es = esize_of(c.dtype);
  const int rp = ceil_div(rows, 16) * 16;
  size_t off = 0;
  auto take = [&](size_t bytes) {
    void* p = base ? static_cast<char*>(base) + off : nullptr;
    off += align_up(bytes, 256);
    return p;
  };
  w.x = static_cast<float*>(take((size_t)rows * c.d_model * 4));
  w.cs = static_cast<float2*>(take((size_t)rows * (c.head_dim / 2) * 8));
  w.h = take((size_t)rp * c.d_model * es);  // GEMM inputs: half in tile order, or float32 row-major
  w.q = take((size_t)c.n_q * rp * c.head_dim * es);
  w.att = take((size_t)rp * c.n_q * c.head_dim * es);
  w.act = take((size_t)rp * c.d_ffn * es);
  w.y = take((size_t)rp * c.d_model * es);
  w.y_tail = take((size_t)rp * c.d_model * es);
  size_t gf = 0;
  widest_split_floats(c, rows, &gf);
  w.gemm_out = static_cast<float*>(take(gf * 4));
  const size_t part_rows = (size_t)attn_partial_rows(rp) * c.n_q;  // splits x heads x padded rows
  w.att_o = static_cast<float*>(take(part_rows * c.head_dim * 4));
  w.att_ml = static_cast<float*>(take(part_rows * 2 * 4));
  w.logits = static_cast<float*>(take((size_t)rows * c.vocab * 4));
  w.scan_bytes = accept_ws_bytes(rows, c.vocab);
  w.scan = take(w.scan_bytes);
  {
    // arg-max records + counter + per-row exchange words, or lattice records: whichever is larger
    const size_t best = gemm_bf16_best_bytes(rows, c.vocab, 128) + (size_t)DS_MAX_ROWS * sizeof(int32_t);
    const size_t top = gemm_bf16_top_bytes(rows, c.vocab, 128);
    w.tile_rec = take(best > top ? best : top);
  }
  w.eos_col = static_cast<float*>(take((size_t)rp * sizeof(float)));
  w.lat_bytes = lattice_ws_bytes(rows, c.vocab, DS_MAX_TOPM);
  w.lat = take(w.lat_bytes);
  w.sample_bytes = sample_ws_bytes(rows);
  w.sample = take(w.sample_bytes);
  w.total = off;
  return w;
}

template <typename T>
int gemm(const ds_model* m, int li, int which, const void* x_in, int rows, float* out, int* n_split,
         hipStream_t st, const GemmEpilogue& epi = GemmEpilogue{}) {
  // which: 0 qkv, 1 o, 2 gate/up, 3 down, 4 lm head
  const ds_model_cfg& c = m->cfg;
  const int d = c.d_model, f = c.d_ffn, qo = c.n_q * c.head_dim;
  int N = 0, K = 0;
  switch (which) {
    case 0: N = n_qkv(c); K = d; break;
    case 1: N = d; K = qo; break;
    case 2: N = 2 * f; K = d; break;
    case 3: N = d; K = f; break;
    default: N = c.vocab; K = d; break;
  }
  if (c.dtype == DS_BF16) {
    const void* w = nullptr;
    if (which == 4) w = m->lm_head;
    else {
      const PackedLayer& pl = m->packed[li];
      w = which == 0 ? pl.wqkv : which == 1 ? pl.wo : which == 2 ? pl.wgu : pl.wdown;
    }
    // two row blocks per wavefront where N is large (LM head, gate/up): half the X traffic per weight byte
    const int nbw = (which == 4 || which == 2) ? 2 : 1;
    *n_split = which == 4 ? 1 : gemm_bf16_splits(N, K, nbw);
    return launch_gemm_bf16(w, x_in, rows, N, K, nbw, *n_split, out, epi, st);
  }
  *n_split = 1;
  const float* x = static_cast<const float*>(x_in);
  if (which == 4) return launch_gemm_f32(x, static_cast<const float*>(m->lm_head), rows, N, K, out, N, st);
  const ds_layer_weights& lw = m->canon[li];
  int rc = DS_OK;
  switch (which) {
    case 0: {
      const int nq = c.n_q * c.head_dim, nk = c.n_kv * c.head_dim;
      rc = launch_gemm_f32(x, static_cast<const float*>(lw.wq), rows, nq, K, out, N, st);
      if (rc) return rc;
      rc = launch_gemm_f32(x, static_cast<const float*>(lw.wk), rows, nk, K, out + nq, N, st);
      if (rc) return rc;
      return launch_gemm_f32(x, static_cast<const float*>(lw.wv), rows, nk, K, out + nq + nk, N, st);
    }
    case 1: return launch_gemm_f32(x, static_cast<const float*>(lw.wo), rows, N, K, out, N, st);
    case 2:
      rc = launch_gemm_f32(x, static_cast<const float*>(lw.w_gate), rows, f, K, out, N, st);
      if (rc) return rc;
      return launch_gemm_f32(x, static_cast<const float*>(lw.w_up), rows, f, K, out + f, N, st);
    default: return launch_gemm_f32(x, static_cast<const float*>(lw.w_down), rows, N, K, out, N, st);
  }
}

// One forward call: up to kMaxSeq sequences, each with its own cache, share one pass over the weights.
struct FwdSeq {
  ds_kv* kv;
  int n_a;       // rows that read their token from tok_a (the rest read tok_b, or are `fill`)
  int n_rows;    // rows of the sequence in this call
  int n_causal;  // leading causal real-token rows; the rest see every key ([MASK] / block rows)
  int tail0;     // rows >= tail0 are handed on (hidden_out and the LM head's input); n_rows: none
};
struct FwdCall {
  int n_seq = 0;
  FwdSeq seq[kMaxSeq];
  const int32_t* tok_a = nullptr;
  const int32_t* tok_b = nullptr;
  int32_t fill = 0;
  float* hidden_out = nullptr;
};

// Row layout of a call (each sequence starts at a multiple of 16) and the host-side checks every forward needs.
int plan_call(const ds_model* m, const FwdCall& call, SeqTable* tab, int* rows_total, int* tail_rows) {
  DS_REQUIRE(call.n_seq >= 1 && call.n_seq <= kMaxSeq, DS_E_SHAPE, "%d sequences outside [1, %d]", call.n_seq, kMaxSeq);
  SeqTable t{};
  t.n_seq = call.n_seq;
  int row = 0, off_a = 0, off_b = 0, tail = 0;
  for (int s = 0; s < call.n_seq; ++s) {
    const FwdSeq& q = call.seq[s];
    DS_REQUIRE(q.kv && q.kv->owner == m, DS_E_INVALID, "sequence %d: KV handle is NULL or belongs to another model", s);
    for (int o = 0; o < s; ++o)
      DS_REQUIRE(call.seq[o].kv != q.kv, DS_E_INVALID, "sequences %d and %d share one KV handle", o, s);
    DS_REQUIRE(q.n_rows >= 1 && q.n_a >= 0 && q.n_a <= q.n_rows && q.n_causal >= 0 && q.n_causal <= q.n_rows &&
                   q.tail0 >= 0 && q.tail0 <= q.n_rows,
               DS_E_SHAPE, "sequence %d: bad row counts", s);
    DS_REQUIRE(q.kv->len + q.n_rows <= m->cfg.kv_capacity, DS_E_CAPACITY,
               "KV cache of sequence %d: %d + %d rows exceed capacity %d", s, q.kv->len, q.n_rows, m->cfg.kv_capacity);
    row = ceil_div(row, 16) * 16;
    t.row0[s] = row;
    t.n_rows[s] = q.n_rows;
    t.n_a[s] = q.n_a;
    t.off_a[s] = off_a;
    t.off_b[s] = off_b;
    t.pos0[s] = q.kv->len;
    t.n_causal[s] = q.n_causal;
    t.tail0[s] = q.tail0;
    t.tail_base[s] = tail;
    row += q.n_rows;
    off_a += q.n_a;
    off_b += q.n_rows - q.n_a;
    tail += q.n_rows - q.tail0;
  }
  t.row0[call.n_seq] = row;
  DS_REQUIRE(row <= DS_MAX_ROWS, DS_E_SHAPE,
             "%d rows (every sequence padded to a multiple of 16 but the last) exceed %d rows per call", row, DS_MAX_ROWS);
  DS_REQUIRE(call.tok_a || off_a == 0, DS_E_INVALID, "token pointer is NULL");
  *tab = t;
  *rows_total = row;
  *tail_rows = tail;
  return DS_OK;
}

// Forward of the call's rows, each sequence placed after its committed cache.  Leaves the final-normed states of all
// rows in ws.y (GEMM input order) and, for the rows every sequence hands on, a compact GEMM input in ws.y_tail and
// (if given) a row-major copy in call.hidden_out.
template <typename T>
int forward_rows(ds_model* m, const Workspace& w, const FwdCall& call, const SeqTable& tab, int rows, bool tail,
                 hipStream_t st) {
  const ds_model_cfg& c = m->cfg;
  const int rp = ceil_div(rows, 16) * 16;
  const int d = c.d_model, hd = c.head_dim;
  int rc;
  if ((rc = launch_embed_norm<T>(tab, call.tok_a, call.tok_b, call.fill, c.vocab, hd, (double)c.rope_base, w.cs, m->embed,
                                 w.x, rows, rp, d, m->canon[0].norm1, c.rms_eps, w.h, m->ovf, st)))
    return rc;
  for (int li = 0; li < c.n_layers; ++li) {
    const size_t layer_bytes = (size_t)c.n_kv * c.kv_capacity * hd * m->esize;
    SeqTable lt = tab;  // this layer's caches
    for (int s = 0; s < tab.n_seq; ++s) {
      lt.kc[s] = static_cast<char*>(call.seq[s].kv->k) + (size_t)li * layer_bytes;
      lt.vc[s] = static_cast<char*>(call.seq[s].kv->v) + (size_t)li * layer_bytes;
    }
    int sp = 1;
    if ((rc = gemm<T>(m, li, 0, w.h, rows, w.gemm_out, &sp, st))) return rc;
    if ((rc = launch_qkv_rope<T>(lt, w.gemm_out, sp, rows, rp, c.n_q, c.n_kv, hd, w.cs, c.kv_capacity,
                                 attn_q_scale(c.dtype, hd), w.q, m->ovf, st)))
      return rc;
    if ((rc = launch_attention(c.dtype, lt, w.q, rows, rp, c.n_q, c.n_kv, hd, c.kv_capacity, w.att_o, w.att_ml, w.att,
                               m->ovf, st)))
      return rc;
    if ((rc = gemm<T>(m, li, 1, w.att, rows, w.gemm_out, &sp, st))) return rc;
    if ((rc = launch_add_norm<T>(tab, w.x, w.gemm_out, sp, rows, rp, d, m->canon[li].norm2, c.rms_eps, w.h, nullptr,
                                 nullptr, m->ovf, st)))
      return rc;
    if (m->fused_gu || (m->pair_gu && rows <= kFuseTwoRows)) {  // SwiGLU in the product's epilogue
      GemmEpilogue epi;
      epi.kind = GemmEpilogue::kSwiGLU;
      epi.records = w.act;
      epi.ovf = m->ovf;
      if ((rc = gemm<T>(m, li, 2, w.h, rows, w.gemm_out, &sp, st, epi))) return rc;
    } else {
      if ((rc = gemm<T>(m, li, 2, w.h, rows, w.gemm_out, &sp, st))) return rc;
      if ((rc = launch_swiglu<T>(w.gemm_out, sp, rows, rp, c.d_ffn, m->pair_gu, w.act, m->ovf, st))) return rc;
    }
    if ((rc = gemm<T>(m, li, 3, w.act, rows, w.gemm_out, &sp, st))) return rc;
    const bool last = li + 1 == c.n_layers;
    const float* gain = last ? m->final_norm : m->canon[li + 1].norm1;
    if ((rc = launch_add_norm<T>(tab, w.x, w.gemm_out, sp, rows, rp, d, gain, c.rms_eps, last ? w.y : w.h,
                                 last ? call.hidden_out : nullptr, (last && tail) ? w.y_tail : nullptr, m->ovf, st)))
      return rc;
  }
  return DS_OK;
}

int forward_dispatch(ds_model* m, const Workspace& w, const FwdCall& call, const SeqTable& tab, int rows, bool tail,
                     hipStream_t st) {
  m->tail_ptr = nullptr;  // any forward overwrites the workspace
  m->rec_ws = nullptr;
  return m->cfg.dtype == DS_BF16 ? forward_rows<bf16_t>(m, w, call, tab, rows, tail, st)
                                 : forward_rows<float>(m, w, call, tab, rows, tail, st);
}

// epi (bf16 path with lm_head_tile() > 0 only): also leave per-tile records; logits may then be NULL.
int lm_head_rows(ds_model* m, const void* y_gemm_in, int rows, float* logits, hipStream_t st,
                 const GemmEpilogue& epi = GemmEpilogue{}) {
  int sp = 1;
  return m->cfg.dtype == DS_BF16 ? gemm<bf16_t>(m, 0, 4, y_gemm_in, rows, logits, &sp, st, epi)
                                 : gemm<float>(m, 0, 4, y_gemm_in, rows, logits, &sp, st);
}

// Columns per tile of the LM head's arg-max epilogue, 0 where the model cannot use it.
int lm_head_tile(const ds_model* m) {
  return m->cfg.dtype == DS_BF16 ? gemm_bf16_best_tile(m->cfg.vocab, 2, 1) : 0;
}

int check_ws(const ds_model* m, int rows, void* ws, size_t ws_bytes, Workspace* out) {
  DS_REQUIRE(ws, DS_E_INVALID, "workspace is NULL");
  DS_REQUIRE((((uintptr_t)ws) & 255) == 0, DS_E_INVALID, "workspace not 256-byte aligned");
  *out = carve(m->cfg, rows, ws);
  DS_REQUIRE(ws_bytes >= out->total, DS_E_CAPACITY, "workspace: %d rows need %zu bytes, got %zu", rows, out->total,
             ws_bytes);
  return DS_OK;
}

}  // namespace

extern "C" {

int ds_model_packed_bytes(const ds_model_cfg* cfg, size_t* bytes) {
  DS_REQUIRE(bytes, DS_E_INVALID, "bytes is NULL");
  int rc = validate_cfg(cfg);
  if (rc) return rc;
  *bytes = packed_bytes_of(*cfg);
  return DS_OK;
}

int ds_kv_bytes(const ds_model_cfg* cfg, size_t* bytes) {
  DS_REQUIRE(bytes, DS_E_INVALID, "bytes is NULL");
  int rc = validate_cfg(cfg);
  if (rc) return rc;
  *bytes = kv_bytes_of(*cfg);
  return DS_OK;
}

int ds_workspace_bytes(const ds_model_cfg* cfg, int max_rows, size_t* bytes) {
  DS_REQUIRE(bytes, DS_E_INVALID, "bytes is NULL");
  int rc = validate_cfg(cfg);
  if (rc) return rc;
  DS_REQUIRE(max_rows >= 1 && max_rows <= DS_MAX_ROWS, DS_E_SHAPE, "max_rows %d outside [1, %d]", max_rows,
             DS_MAX_ROWS);
  *bytes = carve(*cfg, max_rows, nullptr).total;
  return DS_OK;
}

int ds_model_create(const ds_model_cfg* cfg, const ds_weights* w, void* packed, size_t packed_bytes, void* kv_k,
                    void* kv_v, void* stream, ds_model** out) {
  DS_REQUIRE(out, DS_E_INVALID, "out is NULL");
  *out = nullptr;
  int rc = validate_cfg(cfg);
  if (rc) return rc;
  DS_REQUIRE(w && w->embed && w->layers && w->final_norm && w->lm_head, DS_E_INVALID, "weights: NULL pointer");
  DS_REQUIRE(kv_k && kv_v, DS_E_INVALID, "KV buffers: NULL pointer");
  DS_REQUIRE((((uintptr_t)kv_k | (uintptr_t)kv_v | (uintptr_t)w->embed | (uintptr_t)w->lm_head) & 15) == 0,
             DS_E_INVALID, "KV buffers and matrices must be 16-byte aligned");
  for (int l = 0; l < cfg->n_layers; ++l) {
    const ds_layer_weights& lw = w->layers[l];
    DS_REQUIRE(lw.wq && lw.wk && lw.wv && lw.wo && lw.w_gate && lw.w_up && lw.w_down && lw.norm1 && lw.norm2,
               DS_E_INVALID, "layer %d: NULL weight pointer", l);
  }
  const size_t need = packed_bytes_of(*cfg);
  if (need) {
    DS_REQUIRE(packed, DS_E_INVALID, "packed buffer is NULL");
    DS_REQUIRE((((uintptr_t)packed) & 255) == 0, DS_E_INVALID, "packed buffer not 256-byte aligned");
    DS_REQUIRE(packed_bytes >= need, DS_E_CAPACITY, "packed buffer: need %zu bytes, got %zu", need, packed_bytes);
  }
  ds_model* m = new (std::nothrow) ds_model();
  DS_REQUIRE(m, DS_E_INVALID, "out of host memory");
  m->cfg = *cfg;
  m->embed = w->embed;
  m->canon.assign(w->layers, w->layers + cfg->n_layers);
  m->final_norm = w->final_norm;
  m->self = ds_kv{m, kv_k, kv_v, 0};
  m->esize = esize_of(cfg->dtype);
  m->lm_head = w->lm_head;
  if (cfg->dtype == DS_BF16) {
    hipStream_t st = static_cast<hipStream_t>(stream);
    char* p = static_cast<char*>(packed);
    const int d = cfg->d_model, f = cfg->d_ffn, hd = cfg->head_dim, qo = cfg->n_q * hd, kvn = cfg->n_kv * hd;
    uint32_t* flag = reinterpret_cast<uint32_t*>(p + need - kFlagBytes);
    m->ovf = flag + 16;  // its own 64-byte line of the tail
    if (hipMemsetAsync(flag, 0, kFlagBytes, st) != hipSuccess) {
      delete m;
      return fail(DS_E_HIP, "hipMemsetAsync(weight-range flag) failed");
    }
    const int gu_planes = gemm_bf16_splits(2 * f, d, 2);
    m->fused_gu = gu_planes == 1 && (f % 128) == 0;
    m->pair_gu = (f % 128) == 0 && (gu_planes == 1 || (gu_planes == 2 && (d / 128) % 2 == 0));
    auto put = [&](const void* src, int N, int K) -> int {
      int r = launch_pack_weight(src, N, K, p, flag, st);
      p += (size_t)N * K * 2;
      return r;
    };
    for (int l = 0; l < cfg->n_layers && !rc; ++l) {
      const ds_layer_weights& lw = w->layers[l];
      PackedLayer pl{};
      pl.wqkv = p;
      if ((rc = put(lw.wq, qo, d)) || (rc = put(lw.wk, kvn, d)) || (rc = put(lw.wv, kvn, d))) break;
      pl.wo = p;
      if ((rc = put(lw.wo, d, qo))) break;
      pl.wgu = p;
      if (m->pair_gu) {
        if ((rc = launch_pack_weight_pair(lw.w_gate, lw.w_up, f, d, p, flag, st))) break;
        p += (size_t)2 * f * d * 2;
      } else if ((rc = put(lw.w_gate, f, d)) || (rc = put(lw.w_up, f, d))) {
        break;
      }
      pl.wdown = p;
      if ((rc = put(lw.w_down, d, f))) break;
      m->packed.push_back(pl);
    }
    if (!rc) {
      m->lm_head = p;
      rc = put(w->lm_head, cfg->vocab, d);
    }
    if (!rc) {  // the packed copies are half precision: refuse weights outside the half range
      uint32_t bad = 0;
      if (hipMemcpyAsync(&bad, flag, sizeof(bad), hipMemcpyDeviceToHost, st) != hipSuccess ||
          hipStreamSynchronize(st) != hipSuccess)
        rc = fail(DS_E_HIP, "reading the weight-range flag failed");
      else if (bad)
        rc = fail(DS_E_UNSUPPORTED, "a weight is NaN or exceeds the half-precision range (|w| > 65504)");
    }
    if (rc) {
      delete m;
      return rc;
    }
  }
  *out = m;
  return DS_OK;
}

void ds_model_destroy(ds_model* m) { delete m; }

int ds_model_overflow_count(ds_model* m, int reset, void* stream, uint32_t* count) {
  DS_REQUIRE(m && count, DS_E_INVALID, "ds_model_overflow_count: NULL pointer argument");
  *count = 0;
  if (!m->ovf) return DS_OK;  // float32 models have no half-precision rounding points
  hipStream_t st = static_cast<hipStream_t>(stream);
  DS_HIP_CHECK(hipMemcpyAsync(count, m->ovf, sizeof(uint32_t), hipMemcpyDeviceToHost, st));
  if (reset) DS_HIP_CHECK(hipMemsetAsync(m->ovf, 0, sizeof(uint32_t), st));
  DS_HIP_CHECK(hipStreamSynchronize(st));
  return DS_OK;
}

int ds_model_kv_len(const ds_model* m, int* len) {
  DS_REQUIRE(m && len, DS_E_INVALID, "ds_model_kv_len: NULL pointer argument");
  *len = m->self.len;
  return DS_OK;
}

int ds_model_kv_set_len(ds_model* m, int len) {
  DS_REQUIRE(m, DS_E_INVALID, "model is NULL");
  DS_REQUIRE(len >= 0 && len <= m->cfg.kv_capacity, DS_E_CAPACITY, "KV length %d outside [0, %d]", len,
             m->cfg.kv_capacity);
  m->self.len = len;
  return DS_OK;
}

int ds_kv_create(ds_model* m, void* kv_k, void* kv_v, ds_kv** out) {
  DS_REQUIRE(out, DS_E_INVALID, "out is NULL");
  *out = nullptr;
  DS_REQUIRE(m && kv_k && kv_v, DS_E_INVALID, "ds_kv_create: NULL pointer argument");
  DS_REQUIRE((((uintptr_t)kv_k | (uintptr_t)kv_v) & 15) == 0, DS_E_INVALID, "KV buffers must be 16-byte aligned");
  ds_kv* kv = new (std::nothrow) ds_kv{m, kv_k, kv_v, 0};
  DS_REQUIRE(kv, DS_E_INVALID, "out of host memory");
  *out = kv;
  return DS_OK;
}

void ds_kv_destroy(ds_kv* kv) { delete kv; }

int ds_kv_len(const ds_kv* kv, int* len) {
  DS_REQUIRE(kv && len, DS_E_INVALID, "ds_kv_len: NULL pointer argument");
  *len = kv->len;
  return DS_OK;
}

int ds_kv_set_len(ds_kv* kv, int len) {
  DS_REQUIRE(kv, DS_E_INVALID, "KV handle is NULL");
  DS_REQUIRE(len >= 0 && len <= kv->owner->cfg.kv_capacity, DS_E_CAPACITY, "KV length %d outside [0, %d]", len,
             kv->owner->cfg.kv_capacity);
  kv->len = len;
  return DS_OK;
}

}  // extern "C"

namespace {

int prefill_impl(ds_model* m, ds_kv* kv, const int32_t* tokens, int n, float* last_logits, void* ws, size_t ws_bytes,
                 void* stream) {
  DS_REQUIRE(m && kv && tokens, DS_E_INVALID, "prefill: NULL pointer argument");
  DS_REQUIRE(kv->owner == m, DS_E_INVALID, "prefill: the KV handle belongs to another model");
  DS_REQUIRE(n >= 1, DS_E_SHAPE, "n %d must be >= 1", n);
  DS_REQUIRE(kv->len + n <= m->cfg.kv_capacity, DS_E_CAPACITY, "KV cache: %d + %d tokens exceed capacity %d", kv->len,
             n, m->cfg.kv_capacity);
  // largest chunk the workspace can carry
  int chunk = n < DS_MAX_ROWS ? n : DS_MAX_ROWS;
  DS_REQUIRE(ws, DS_E_INVALID, "workspace is NULL");
  while (chunk > 1 && carve(m->cfg, chunk, nullptr).total > ws_bytes) chunk = chunk > 16 ? chunk - 16 : chunk - 1;
  Workspace w;
  int rc = check_ws(m, chunk, ws, ws_bytes, &w);
  if (rc) return rc;
  hipStream_t st = static_cast<hipStream_t>(stream);
  const int start_len = kv->len;
  for (int done = 0; done < n; done += chunk) {
    const int rows = n - done < chunk ? n - done : chunk;
    w = carve(m->cfg, rows, ws);
    FwdCall call;
    call.n_seq = 1;
    call.seq[0] = FwdSeq{kv, rows, rows, rows, rows};
    call.tok_a = tokens + done;
    SeqTable tab;
    int total = 0, tail = 0;
    if ((rc = plan_call(m, call, &tab, &total, &tail)) || (rc = forward_dispatch(m, w, call, tab, total, false, st))) {
      kv->len = start_len;
      return rc;
    }
    kv->len += rows;
    if (last_logits && done + rows == n) {
      // logits of all rows of the last chunk, then copy the last row out
      if ((rc = lm_head_rows(m, w.y, rows, w.logits, st)) ||
          (hipMemcpyAsync(last_logits, w.logits + (size_t)(rows - 1) * m->cfg.vocab, (size_t)m->cfg.vocab * 4,
                          hipMemcpyDeviceToDevice, st) != hipSuccess &&
           (rc = fail(DS_E_HIP, "prefill: copying the last row's logits failed")))) {
        kv->len = start_len;  // a failed call changes no state
        return rc;
      }
    }
  }
  return DS_OK;
}

// Drafter pass over n_seq sequences: n_pend[s] pending real tokens (causal) followed by K block rows each.
// block_tokens NULL: every block row is `mask_id`; else block row i of sequence s holds block_tokens[s * K + i].
int draft_impl(ds_model* m, ds_kv* const* kvs, int n_seq, const int32_t* pending, const int* n_pend, int K,
               const int32_t* block_tokens, int32_t mask_id, float* hidden_out, void* ws, size_t ws_bytes,
               void* stream) {
  DS_REQUIRE(m && hidden_out && kvs && n_pend, DS_E_INVALID, "draft pass: NULL pointer argument");
  DS_REQUIRE(n_seq >= 1 && n_seq <= kMaxSeq, DS_E_SHAPE, "%d sequences outside [1, %d]", n_seq, kMaxSeq);
  DS_REQUIRE(K >= 1, DS_E_SHAPE, "K %d must be >= 1", K);
  DS_REQUIRE(block_tokens || (mask_id >= 0 && mask_id < m->cfg.vocab), DS_E_INVALID, "mask_id %d outside the vocabulary",
             mask_id);
  FwdCall call;
  call.n_seq = n_seq;
  int n_pend_all = 0;
  for (int s = 0; s < n_seq; ++s) {
    DS_REQUIRE(n_pend[s] >= 0, DS_E_SHAPE, "sequence %d: n_pend %d is negative", s, n_pend[s]);
    DS_REQUIRE(n_pend[s] + K <= DS_MAX_ROWS, DS_E_SHAPE, "n_pend + K = %d exceeds %d rows", n_pend[s] + K, DS_MAX_ROWS);
    call.seq[s] = FwdSeq{kvs[s], n_pend[s], n_pend[s] + K, n_pend[s], n_pend[s]};
    n_pend_all += n_pend[s];
  }
  DS_REQUIRE(pending || n_pend_all == 0, DS_E_INVALID, "pending is NULL while n_pend > 0");
  call.tok_a = pending;
  call.tok_b = block_tokens;
  call.fill = mask_id;
  call.hidden_out = hidden_out;
  SeqTable tab;
  int rows = 0, tail = 0;
  int rc = plan_call(m, call, &tab, &rows, &tail);
  if (rc) return rc;
  Workspace w;
  if ((rc = check_ws(m, rows, ws, ws_bytes, &w))) return rc;
  hipStream_t st = static_cast<hipStream_t>(stream);
  if ((rc = forward_dispatch(m, w, call, tab, rows, true, st))) return rc;
  m->tail_ptr = w.y_tail;
  m->tail_ws = ws;
  m->tail_rows = tail;  // n_seq * K
  for (int s = 0; s < n_seq; ++s) kvs[s]->len += n_pend[s];  // block rows are never committed
  return DS_OK;
}

// Verifier pass + greedy acceptance over n_seq sequences of mlen + 1 causal rows each.  Row i of sequence s reads
// its token from first[s] (i == 0) or path[s * path_stride + i - 1]; the single-sequence entry point passes its
// block as first = block, path = block + 1.
int verify_impl(ds_model* m, ds_kv* const* kvs, int n_seq, const int32_t* first, const int32_t* path, int path_stride,
                int mlen, const int32_t* path_len, int32_t eos_id, int32_t* n_accept, int32_t* next_token,
                int32_t* argmax, int32_t* eos_accepted, float* logits_out, void* ws, size_t ws_bytes, void* stream,
                int32_t* carry = nullptr) {
  DS_REQUIRE(m && kvs && first && n_accept && next_token && argmax && eos_accepted, DS_E_INVALID,
             "verifier pass: NULL pointer argument");
  DS_REQUIRE(!carry || n_seq == 1, DS_E_INVALID, "carry is a single-sequence output");
  DS_REQUIRE(n_seq >= 1 && n_seq <= kMaxSeq, DS_E_SHAPE, "%d sequences outside [1, %d]", n_seq, kMaxSeq);
  DS_REQUIRE(mlen >= 0 && mlen + 1 <= DS_MAX_ROWS, DS_E_SHAPE, "m = %d: m + 1 rows outside [1, %d]", mlen, DS_MAX_ROWS);
  DS_REQUIRE(path || mlen == 0, DS_E_INVALID, "path is NULL while m > 0");
  DS_REQUIRE(eos_id < m->cfg.vocab, DS_E_INVALID, "eos_id %d >= vocab", eos_id);
  const int rows_s = mlen + 1;
  FwdCall call;
  call.n_seq = n_seq;
  AcceptSeqs aq{};
  aq.n_seq = n_seq;
  aq.first = first;
  aq.carry = carry;
  // token sources: tok_a = first (one per sequence), tok_b = path rows; the table's offsets advance by n_a and by
  // n_rows - n_a per sequence, so a dense path array needs path_stride == mlen (checked by the callers)
  for (int s = 0; s < n_seq; ++s) call.seq[s] = FwdSeq{kvs[s], 1, rows_s, rows_s, rows_s};
  call.tok_a = first;
  call.tok_b = path;
  SeqTable tab;
  int rows = 0, tail = 0;
  int rc = plan_call(m, call, &tab, &rows, &tail);
  if (rc) return rc;
  for (int s = 0; s < n_seq; ++s) {
    tab.off_a[s] = s;
    tab.off_b[s] = s * path_stride;
    aq.row0[s] = tab.row0[s];
    aq.m[s] = mlen;
    aq.tok_off[s] = s * path_stride;
    aq.out_off[s] = s * rows_s;
  }
  Workspace w;
  if ((rc = check_ws(m, rows, ws, ws_bytes, &w))) return rc;
  hipStream_t st = static_cast<hipStream_t>(stream);
  if ((rc = forward_dispatch(m, w, call, tab, rows, false, st))) return rc;
  if (const int tile = lm_head_tile(m)) {
    // The product's epilogue reports every tile's largest logit; the logits themselves are written only if asked for.
    GemmEpilogue epi;
    epi.kind = GemmEpilogue::kBest;
    epi.records = w.tile_rec;
    if ((rc = lm_head_rows(m, w.y, rows, logits_out, st, epi))) return rc;
    return launch_tiles_accept(static_cast<float2*>(w.tile_rec), rows, m->cfg.vocab / tile, aq, path, path_len, eos_id,
                               n_accept, next_token, argmax, eos_accepted, st);
  }
  float* logits = logits_out ? logits_out : w.logits;
  if ((rc = lm_head_rows(m, w.y, rows, logits, st))) return rc;
  return launch_argmax_accept(logits, rows, m->cfg.vocab, aq, path, path_len, eos_id, n_accept, next_token, argmax,
                              eos_accepted, w.scan, w.scan_bytes, st);
}

}  // namespace

extern "C" {

int ds_prefill(ds_model* m, const int32_t* tokens, int n, float* last_logits, void* ws, size_t ws_bytes,
               void* stream) {
  DS_REQUIRE(m, DS_E_INVALID, "ds_prefill: NULL model");
  return prefill_impl(m, &m->self, tokens, n, last_logits, ws, ws_bytes, stream);
}

int ds_prefill_seq(ds_model* m, ds_kv* kv, const int32_t* tokens, int n, float* last_logits, void* ws,
                   size_t ws_bytes, void* stream) {
  return prefill_impl(m, kv, tokens, n, last_logits, ws, ws_bytes, stream);
}

int ds_draft_block(ds_model* m, const int32_t* pending, int n_pend, int K, int32_t mask_id, float* hidden_out,
                   void* ws, size_t ws_bytes, void* stream) {
  DS_REQUIRE(m, DS_E_INVALID, "ds_draft_block: NULL model");
  ds_kv* kv = &m->self;
  return draft_impl(m, &kv, 1, pending, &n_pend, K, nullptr, mask_id, hidden_out, ws, ws_bytes, stream);
}

int ds_draft_block_batch(ds_model* m, ds_kv* const* seqs, int n_seq, const int32_t* pending, const int* n_pend, int K,
                         int32_t mask_id, float* hidden_out, void* ws, size_t ws_bytes, void* stream) {
  return draft_impl(m, seqs, n_seq, pending, n_pend, K, nullptr, mask_id, hidden_out, ws, ws_bytes, stream);
}

int ds_lm_head(ds_model* m, const float* hidden, int rows, float* logits, void* ws, size_t ws_bytes, void* stream) {
  DS_REQUIRE(m && logits, DS_E_INVALID, "ds_lm_head: NULL pointer argument");
  DS_REQUIRE(rows >= 1 && rows <= DS_MAX_ROWS, DS_E_SHAPE, "rows %d outside [1, %d]", rows, DS_MAX_ROWS);
  Workspace w;
  int rc = check_ws(m, rows, ws, ws_bytes, &w);
  if (rc) return rc;
  hipStream_t st = static_cast<hipStream_t>(stream);
  m->rec_ws = nullptr;
  if (!hidden) {  // the block rows of the last draft pass, still in the workspace as a GEMM input
    DS_REQUIRE(m->tail_ptr && m->tail_ws == ws && m->tail_rows == rows, DS_E_INVALID,
               "ds_lm_head(hidden = NULL) must directly follow a draft pass of %d block rows on this workspace", rows);
    return lm_head_rows(m, m->tail_ptr, rows, logits, st);
  }
  if (m->cfg.dtype == DS_BF16) {
    const int rp = ceil_div(rows, 16) * 16;
    if ((rc = launch_to_gemm_input<bf16_t>(hidden, rows, rp, m->cfg.d_model, w.y, m->ovf, st))) return rc;
    return lm_head_rows(m, w.y, rows, logits, st);
  }
  return lm_head_rows(m, hidden, rows, logits, st);
}

int ds_lm_head_tiles(ds_model* m, const float* hidden, int rows, int32_t eos_id, float* logits_out, void* ws,
                     size_t ws_bytes, void* stream) {
  DS_REQUIRE(m, DS_E_INVALID, "ds_lm_head_tiles: NULL model");
  DS_REQUIRE(rows >= 1 && rows <= DS_MAX_ROWS, DS_E_SHAPE, "rows %d outside [1, %d]", rows, DS_MAX_ROWS);
  const int vocab = m->cfg.vocab;
  DS_REQUIRE(eos_id < vocab, DS_E_INVALID, "eos_id %d >= vocab %d", eos_id, vocab);
  Workspace w;
  int rc = check_ws(m, rows, ws, ws_bytes, &w);
  if (rc) return rc;
  hipStream_t st = static_cast<hipStream_t>(stream);
  m->rec_ws = nullptr;
  const void* y = nullptr;
  if (!hidden) {  // the block rows of the last draft pass, still in the workspace as a GEMM input
    DS_REQUIRE(m->tail_ptr && m->tail_ws == ws && m->tail_rows == rows, DS_E_INVALID,
               "ds_lm_head_tiles(hidden = NULL) must directly follow a draft pass of %d block rows on this workspace",
               rows);
    y = m->tail_ptr;
  } else if (m->cfg.dtype == DS_BF16) {
    const int rp = ceil_div(rows, 16) * 16;
    if ((rc = launch_to_gemm_input<bf16_t>(hidden, rows, rp, m->cfg.d_model, w.y, m->ovf, st))) return rc;
    y = w.y;
  } else {
    y = hidden;
  }
  const int tile = lm_head_tile(m);
  if (tile > 0 && lattice_tiles_supported(vocab / tile, tile)) {
    GemmEpilogue epi;
    epi.kind = GemmEpilogue::kTop;
    epi.records = w.tile_rec;
    epi.export_col = eos_id;
    epi.export_out = eos_id >= 0 ? w.eos_col : nullptr;
    if ((rc = lm_head_rows(m, y, rows, logits_out, st, epi))) return rc;
    m->rec_logits = nullptr;
  } else {
    float* logits = logits_out ? logits_out : w.logits;
    if ((rc = lm_head_rows(m, y, rows, logits, st))) return rc;
    m->rec_logits = logits;
  }
  m->rec_ws = ws;
  m->rec_y = y;
  m->rec_rows = rows;
  m->rec_eos = eos_id;
  return DS_OK;
}

int ds_lattice_from_tiles(ds_model* m, int rows, int M_max, float tau, int32_t eos_id, int32_t* cand_id,
                          float* cand_logp, int32_t* cand_cnt, float* eos_logp, float* lse, void* ws,
                          size_t ws_bytes, void* stream) {
  DS_REQUIRE(m && cand_id && cand_logp && cand_cnt && eos_logp && lse, DS_E_INVALID,
             "ds_lattice_from_tiles: NULL pointer argument");
  DS_REQUIRE(rows >= 1 && rows <= DS_MAX_ROWS, DS_E_SHAPE, "rows %d outside [1, %d]", rows, DS_MAX_ROWS);
  const int vocab = m->cfg.vocab;
  DS_REQUIRE(M_max >= 1 && M_max <= DS_MAX_TOPM && M_max <= vocab, DS_E_SHAPE,
             "M_max %d outside [1, min(%d, vocab)]", M_max, DS_MAX_TOPM);
  DS_REQUIRE(!isnan(tau) && tau > 0.f, DS_E_INVALID, "tau must be positive");
  DS_REQUIRE(m->rec_ws && m->rec_ws == ws && m->rec_rows == rows && m->rec_eos == eos_id, DS_E_INVALID,
             "ds_lattice_from_tiles must directly follow ds_lm_head_tiles with the same rows (%d), eos_id and workspace",
             rows);
  Workspace w;
  int rc = check_ws(m, rows, ws, ws_bytes, &w);
  if (rc) return rc;
  hipStream_t st = static_cast<hipStream_t>(stream);
  if (m->rec_logits)
    return launch_lattice(m->rec_logits, rows, vocab, M_max, tau, eos_id, cand_id, cand_logp, cand_cnt, eos_logp, lse,
                          w.lat, w.lat_bytes, st);
  return launch_lattice_tiles(w.tile_rec, rows, vocab / lm_head_tile(m), M_max, tau, eos_id, w.eos_col, m->lm_head,
                              m->rec_y, m->cfg.d_model, cand_id, cand_logp, cand_cnt, eos_logp, lse, st);
}

int ds_draft_lattice(ds_model* m, const float* hidden, int rows, int M_max, float tau, int32_t eos_id,
                     int32_t* cand_id, float* cand_logp, int32_t* cand_cnt, float* eos_logp, float* lse,
                     float* logits_out, void* ws, size_t ws_bytes, void* stream) {
  DS_REQUIRE(m && cand_id && cand_logp && cand_cnt && eos_logp && lse, DS_E_INVALID,
             "ds_draft_lattice: NULL pointer argument");
  DS_REQUIRE(m->cfg.vocab >= M_max && M_max >= 1 && M_max <= DS_MAX_TOPM, DS_E_SHAPE,
             "M_max %d outside [1, min(%d, vocab)]", M_max, DS_MAX_TOPM);
  DS_REQUIRE(!isnan(tau) && tau > 0.f, DS_E_INVALID, "tau must be positive");
  int rc = ds_lm_head_tiles(m, hidden, rows, eos_id, logits_out, ws, ws_bytes, stream);
  if (rc) return rc;
  return ds_lattice_from_tiles(m, rows, M_max, tau, eos_id, cand_id, cand_logp, cand_cnt, eos_logp, lse, ws, ws_bytes,
                               stream);
}

int ds_verify_block(ds_model* m, const int32_t* block, int mlen, const int32_t* path_len, int32_t eos_id,
                    int32_t* n_accept, int32_t* next_token, int32_t* argmax, int32_t* eos_accepted,
                    float* logits_out, void* ws, size_t ws_bytes, void* stream) {
  DS_REQUIRE(m && block, DS_E_INVALID, "ds_verify_block: NULL pointer argument");
  ds_kv* kv = &m->self;
  return verify_impl(m, &kv, 1, block, block + 1, mlen, mlen, path_len, eos_id, n_accept, next_token, argmax,
                     eos_accepted, logits_out, ws, ws_bytes, stream);
}

int ds_verify_block_carry(ds_model* m, const int32_t* block, int mlen, const int32_t* path_len, int32_t eos_id,
                          int32_t* n_accept, int32_t* next_token, int32_t* argmax, int32_t* eos_accepted,
                          float* logits_out, int32_t* carry, void* ws, size_t ws_bytes, void* stream) {
  DS_REQUIRE(m && block && carry, DS_E_INVALID, "ds_verify_block_carry: NULL pointer argument");
  ds_kv* kv = &m->self;
  return verify_impl(m, &kv, 1, block, block + 1, mlen, mlen, path_len, eos_id, n_accept, next_token, argmax,
                     eos_accepted, logits_out, ws, ws_bytes, stream, carry);
}

int ds_verify_block_batch(ds_model* m, ds_kv* const* seqs, int n_seq, const int32_t* first, const int32_t* path,
                          int mlen, const int32_t* path_len, int32_t eos_id, int32_t* n_accept, int32_t* next_token,
                          int32_t* argmax, int32_t* eos_accepted, float* logits_out, void* ws, size_t ws_bytes,
                          void* stream) {
  return verify_impl(m, seqs, n_seq, first, path, mlen, mlen, path_len, eos_id, n_accept, next_token, argmax,
                     eos_accepted, logits_out, ws, ws_bytes, stream);
}

int ds_draft_block_tokens(ds_model* m, const int32_t* pending, int n_pend, const int32_t* block_tokens, int K,
                          float* hidden_out, void* ws, size_t ws_bytes, void* stream) {
  DS_REQUIRE(m && block_tokens, DS_E_INVALID, "ds_draft_block_tokens: NULL pointer argument");
  ds_kv* kv = &m->self;
  return draft_impl(m, &kv, 1, pending, &n_pend, K, block_tokens, 0, hidden_out, ws, ws_bytes, stream);
}

int ds_verify_block_stochastic(ds_model* m, const int32_t* block, int mlen, const int32_t* path_len,
                               const float* q_logits, const float* u, int32_t eos_id, int32_t* n_accept,
                               int32_t* next_token, int32_t* eos_accepted, float* alpha, float* logits_out, void* ws,
                               size_t ws_bytes, void* stream) {
  DS_REQUIRE(m && block && u && n_accept && next_token && eos_accepted, DS_E_INVALID,
             "ds_verify_block_stochastic: NULL pointer argument");
  DS_REQUIRE(mlen >= 0 && mlen + 1 <= DS_MAX_ROWS, DS_E_SHAPE, "m = %d: m + 1 rows outside [1, %d]", mlen,
             DS_MAX_ROWS);
  DS_REQUIRE(mlen == 0 || (q_logits && alpha), DS_E_INVALID, "q_logits / alpha is NULL while m > 0");
  DS_REQUIRE(eos_id < m->cfg.vocab, DS_E_INVALID, "eos_id %d >= vocab", eos_id);
  const int rows = mlen + 1;
  FwdCall call;
  call.n_seq = 1;
  call.seq[0] = FwdSeq{&m->self, rows, rows, rows, rows};
  call.tok_a = block;
  SeqTable tab;
  int total = 0, tail = 0;
  int rc = plan_call(m, call, &tab, &total, &tail);
  if (rc) return rc;
  Workspace w;
  if ((rc = check_ws(m, rows, ws, ws_bytes, &w))) return rc;
  hipStream_t st = static_cast<hipStream_t>(stream);
  if ((rc = forward_dispatch(m, w, call, tab, rows, false, st))) return rc;
  float* logits = logits_out ? logits_out : w.logits;
  if ((rc = lm_head_rows(m, w.y, rows, logits, st))) return rc;
  return launch_sample_accept(logits, q_logits, mlen, m->cfg.vocab, block, path_len, u, eos_id, n_accept, next_token,
                              eos_accepted, alpha, w.sample, w.sample_bytes, st);
}

}  // extern "C"

// ---- path search with a tiny causal LM as the causal proxy (Sec. 3.2, "Scoring and search") -----------------------
//
// The proxy is a ds_model; every beam slot is one sequence of its forward calls, with a KV cache of its own.  Two
// sets of `beam` caches alternate: the beam step names each new slot's parent, the block-region keys / values of the
// parent (in the set the last proxy step wrote) are copied into the slot's cache of the other set, and the next
// proxy step runs there.  All caches hold the same committed tokens; the state the search kernels keep between
// the steps lives behind them in the caller's buffer.
struct ds_lmproxy {
  ds_model* lm;
  int beam;
  ds_kv kv[2][kMaxSeq];
  LmSearchState* state;
  int len;  // committed tokens (every cache)
};

namespace {

size_t lmproxy_bytes_of(const ds_model_cfg& c, int beam) {
  return (size_t)4 * beam * align_up(kv_bytes_of(c), 256) + align_up(sizeof(LmSearchState), 256);
}

// Bytes of one (layer, head) cache segment that hold positions [p0, p1): whole 64-key chunks for the half layout
// (the other positions of a chunk are either committed, hence equal in every cache, or not yet written).
void kv_byte_range(const ds_model_cfg& c, int p0, int p1, size_t* lo, size_t* hi) {
  if (c.dtype == DS_BF16) {
    const size_t chunk = (size_t)64 * c.head_dim * 2;
    *lo = (size_t)(p0 >> 6) * chunk;
    *hi = (size_t)((p1 + 63) >> 6) * chunk;
  } else {
    *lo = (size_t)p0 * c.head_dim * 4;
    *hi = (size_t)p1 * c.head_dim * 4;
  }
}

int lmproxy_copy(ds_lmproxy* p, const KvCopyPlan& plan, const int32_t* par, const LmSearchState* st, int p0, int p1,
                 hipStream_t s) {
  if (p1 <= p0) return DS_OK;
  const ds_model_cfg& c = p->lm->cfg;
  size_t lo = 0, hi = 0;
  kv_byte_range(c, p0, p1, &lo, &hi);
  const size_t head_bytes = (size_t)c.kv_capacity * c.head_dim * p->lm->esize;
  return launch_kv_copy(plan, par, st, c.n_layers * c.n_kv, head_bytes, lo, hi, s);
}

// Positions [p0, p1) of cache (0, 0) into every other cache.
int lmproxy_broadcast(ds_lmproxy* p, int p0, int p1, hipStream_t s) {
  KvCopyPlan plan{};
  plan.n_src = 1;
  plan.src_k[0] = p->kv[0][0].k;
  plan.src_v[0] = p->kv[0][0].v;
  for (int set = 0; set < 2; ++set)
    for (int d = 0; d < p->beam; ++d) {
      if (set == 0 && d == 0) continue;
      plan.dst_k[plan.n_dst] = p->kv[set][d].k;
      plan.dst_v[plan.n_dst] = p->kv[set][d].v;
      plan.src_of[plan.n_dst] = 0;
      ++plan.n_dst;
    }
  return lmproxy_copy(p, plan, nullptr, nullptr, p0, p1, s);
}

}  // namespace

extern "C" {

int ds_lmproxy_bytes(const ds_model_cfg* cfg, int beam, size_t* bytes) {
  DS_REQUIRE(bytes, DS_E_INVALID, "bytes is NULL");
  int rc = validate_cfg(cfg);
  if (rc) return rc;
  DS_REQUIRE(beam >= 1 && beam <= kLmBeam, DS_E_SHAPE, "beam %d outside [1, %d]", beam, kLmBeam);
  *bytes = lmproxy_bytes_of(*cfg, beam);
  return DS_OK;
}

int ds_lmproxy_create(ds_model* lm, int beam, void* mem, size_t mem_bytes, ds_lmproxy** out) {
  DS_REQUIRE(out, DS_E_INVALID, "out is NULL");
  *out = nullptr;
  DS_REQUIRE(lm && mem, DS_E_INVALID, "ds_lmproxy_create: NULL pointer argument");
  DS_REQUIRE(beam >= 1 && beam <= kLmBeam, DS_E_SHAPE, "beam %d outside [1, %d]", beam, kLmBeam);
  DS_REQUIRE((((uintptr_t)mem) & 255) == 0, DS_E_INVALID, "proxy buffer not 256-byte aligned");
  const size_t need = lmproxy_bytes_of(lm->cfg, beam);
  DS_REQUIRE(mem_bytes >= need, DS_E_CAPACITY, "proxy buffer: need %zu bytes, got %zu", need, mem_bytes);
  ds_lmproxy* p = new (std::nothrow) ds_lmproxy{};
  DS_REQUIRE(p, DS_E_INVALID, "out of host memory");
  p->lm = lm;
  p->beam = beam;
  char* at = static_cast<char*>(mem);
  const size_t one = align_up(kv_bytes_of(lm->cfg), 256);
  for (int set = 0; set < 2; ++set)
    for (int d = 0; d < beam; ++d) {
      p->kv[set][d] = ds_kv{lm, at, at + one, 0};
      at += 2 * one;
    }
  p->state = reinterpret_cast<LmSearchState*>(at);
  p->len = 0;
  *out = p;
  return DS_OK;
}

void ds_lmproxy_destroy(ds_lmproxy* p) { delete p; }

int ds_lmproxy_len(const ds_lmproxy* p, int* len) {
  DS_REQUIRE(p && len, DS_E_INVALID, "ds_lmproxy_len: NULL pointer argument");
  *len = p->len;
  return DS_OK;
}

int ds_lmproxy_set_len(ds_lmproxy* p, int len) {
  DS_REQUIRE(p, DS_E_INVALID, "proxy handle is NULL");
  DS_REQUIRE(len >= 0 && len <= p->len, DS_E_CAPACITY, "proxy length %d outside [0, %d]: it can only be cut back", len,
             p->len);
  p->len = len;
  return DS_OK;
}

int ds_lmproxy_prefill(ds_lmproxy* p, const int32_t* tokens, int n, void* ws, size_t ws_bytes, void* stream) {
  DS_REQUIRE(p && tokens, DS_E_INVALID, "ds_lmproxy_prefill: NULL pointer argument");
  ds_kv* first = &p->kv[0][0];
  first->len = p->len;
  int rc = prefill_impl(p->lm, first, tokens, n, nullptr, ws, ws_bytes, stream);
  if (rc) return rc;
  if ((rc = lmproxy_broadcast(p, p->len, p->len + n, static_cast<hipStream_t>(stream)))) return rc;
  p->len += n;
  return DS_OK;
}

int ds_cps_path_lm(const int32_t* cand_id, const float* cand_logp, const int32_t* cand_cnt, const float* eos_logp,
                   int K, int M_max, int B, float lambda, ds_lmproxy* p, const int32_t* pending, int n_pend,
                   int32_t eos_id, int32_t* path, int32_t* path_len, float* path_score, void* ws, size_t ws_bytes,
                   void* stream) {
  DS_REQUIRE(cand_id && cand_logp && cand_cnt && p && pending && path && path_len && path_score, DS_E_INVALID,
             "ds_cps_path_lm: NULL pointer argument");
  DS_REQUIRE(eos_logp || eos_id < 0, DS_E_INVALID, "eos_logp is NULL while eos_id >= 0");
  DS_REQUIRE(K >= 1 && K <= kLmMaxK, DS_E_SHAPE, "K %d outside [1, %d]", K, kLmMaxK);
  DS_REQUIRE(M_max >= 1 && M_max <= DS_MAX_TOPM, DS_E_SHAPE, "M_max %d outside [1, %d]", M_max, DS_MAX_TOPM);
  DS_REQUIRE(B >= 1 && B <= p->beam, DS_E_SHAPE, "beam %d outside [1, %d] (the proxy's slot count)", B, p->beam);
  DS_REQUIRE(!isnan(lambda), DS_E_INVALID, "lambda is NaN");
  ds_model* m = p->lm;
  DS_REQUIRE(eos_id < m->cfg.vocab, DS_E_INVALID, "eos_id %d >= the proxy's vocabulary", eos_id);
  DS_REQUIRE(n_pend >= 1 && n_pend <= DS_MAX_ROWS, DS_E_SHAPE, "n_pend %d outside [1, %d]", n_pend, DS_MAX_ROWS);
  DS_REQUIRE(p->len + n_pend + K - 1 <= m->cfg.kv_capacity, DS_E_CAPACITY,
             "proxy KV cache: %d committed + %d pending + %d block tokens exceed capacity %d", p->len, n_pend, K - 1,
             m->cfg.kv_capacity);
  hipStream_t st = static_cast<hipStream_t>(stream);
  LmSearchState* state = p->state;
  int rc;
  // depth 0: the pending tokens (committed) go through cache (0, 0); the last row's logits are the root's
  {
    p->kv[0][0].len = p->len;
    FwdCall call;
    call.n_seq = 1;
    call.seq[0] = FwdSeq{&p->kv[0][0], n_pend, n_pend, n_pend, n_pend - 1};
    call.tok_a = pending;
    SeqTable tab;
    int rows = 0, tail = 0;
    if ((rc = plan_call(m, call, &tab, &rows, &tail))) return rc;
    Workspace w;
    if ((rc = check_ws(m, rows, ws, ws_bytes, &w))) return rc;
    // the widest later call must fit as well, before anything is enqueued
    Workspace w_all;
    if ((rc = check_ws(m, 16 * (B - 1) + 1, ws, ws_bytes, &w_all))) return rc;
    if ((rc = forward_dispatch(m, w, call, tab, rows, true, st))) return rc;
    if ((rc = lm_head_rows(m, w.y_tail, 1, w.logits, st))) return rc;
    if ((rc = lmproxy_broadcast(p, p->len, p->len + n_pend, st))) return rc;
    p->len += n_pend;
    if ((rc = launch_lm_init(state, st))) return rc;
    if ((rc = launch_lm_score(w.logits, 1, m->cfg.vocab, state, st))) return rc;
    if ((rc = launch_lm_beam_step(state, w.logits, m->cfg.vocab, cand_id, cand_logp, cand_cnt, eos_logp, 0, K, M_max,
                                  B, lambda, eos_id, st)))
      return rc;
  }
  const int base = p->len;
  int cur = 0;
  for (int i = 1; i < K; ++i) {
    if (i >= 2) {  // every new slot inherits its parent's block-region keys / values (depths 0 .. i - 2)
      KvCopyPlan plan{};
      plan.n_dst = plan.n_src = B;
      for (int d = 0; d < B; ++d) {
        plan.dst_k[d] = p->kv[cur ^ 1][d].k;
        plan.dst_v[d] = p->kv[cur ^ 1][d].v;
        plan.src_k[d] = p->kv[cur][d].k;
        plan.src_v[d] = p->kv[cur][d].v;
      }
      if ((rc = lmproxy_copy(p, plan, state->par, state, base, base + i - 1, st))) return rc;
      cur ^= 1;
    }
    FwdCall call;
    call.n_seq = B;
    for (int d = 0; d < B; ++d) {
      p->kv[cur][d].len = base + i - 1;
      call.seq[d] = FwdSeq{&p->kv[cur][d], 1, 1, 1, 0};
    }
    call.tok_a = state->tok[i & 1];
    SeqTable tab;
    int rows = 0, tail = 0;
    if ((rc = plan_call(m, call, &tab, &rows, &tail))) return rc;
    Workspace w;
    if ((rc = check_ws(m, rows, ws, ws_bytes, &w))) return rc;
    if ((rc = forward_dispatch(m, w, call, tab, rows, true, st))) return rc;
    if ((rc = lm_head_rows(m, w.y_tail, B, w.logits, st))) return rc;
    if ((rc = launch_lm_score(w.logits, B, m->cfg.vocab, state, st))) return rc;
    if ((rc = launch_lm_beam_step(state, w.logits, m->cfg.vocab, cand_id, cand_logp, cand_cnt, eos_logp, i, K, M_max,
                                  B, lambda, eos_id, st)))
      return rc;
  }
  for (int set = 0; set < 2; ++set)
    for (int d = 0; d < p->beam; ++d) p->kv[set][d].len = base;
  return launch_lm_backtrack(state, K, path, path_len, path_score, st);
}

}  // extern "C"
