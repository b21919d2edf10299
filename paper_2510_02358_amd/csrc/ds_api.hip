// C-ABI entry points that do not need a model handle: error text, lattice, path search, the causal
// proxy handle and the draft-length controller.  Every entry validates its arguments on the host
// before launching anything.
#include <math.h>
#include <stdarg.h>
#include <stdio.h>
#include <string.h>

#include <mutex>
#include <new>

#include "ds_common.h"

namespace ds {

static thread_local char g_err[512] = "";

int fail(int code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return code;
}

void clear_error() { g_err[0] = '\0'; }

}  // namespace ds

struct ds_ngram {
  const float* table;
  int log2_size;
};

struct ds_adl {
  int k_min, k_max;
  double delta, rho;
  double l_gen_ema, l_acc_ema;
};

using namespace ds;

// ---- library-owned scratch for callers that cannot allocate ------------------------------------------
// ds_build_lattice_static keeps the scan's per-wavefront partial records here instead of in a caller workspace.
// In host code `scratch` is only a stand-in for the symbol: the device address is looked up once per GPU (each GPU
// holds its own copy of the array) and from then on only that address is used.
constexpr size_t kStaticScratchBytes = (size_t)2 << 20;  // 2 MiB per GPU, held until the process ends
constexpr int kMaxDevices = 64;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
static void* g_scratch_ptr[kMaxDevices] = {};
static std::mutex g_scratch_mutex;

// Device address of `scratch` on the current GPU (looked up on the first call per GPU; allocates nothing).
static int static_scratch(void** out) {
  int dev = -1;
  DS_HIP_CHECK(hipGetDevice(&dev));
  DS_REQUIRE(dev >= 0 && dev < kMaxDevices, DS_E_UNSUPPORTED, "device index %d outside [0, %d)", dev, kMaxDevices);
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    DS_HIP_CHECK(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
    DS_REQUIRE(p && (((uintptr_t)p) & 255) == 0, DS_E_HIP, "static scratch: bad device address %p", p);
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return DS_OK;
}

extern "C" {

const char* ds_version(void) { return "diffuspec-mi355x 0.1 (gfx950)"; }

const char* ds_last_error(void) { return g_err; }

int ds_lattice_workspace_bytes(int rows, int vocab, int M_max, size_t* bytes) {
  DS_REQUIRE(bytes, DS_E_INVALID, "bytes is NULL");
  DS_REQUIRE(rows >= 1 && vocab >= 1, DS_E_SHAPE, "rows %d / vocab %d must be positive", rows, vocab);
  DS_REQUIRE(M_max >= 1 && M_max <= DS_MAX_TOPM, DS_E_SHAPE, "M_max %d outside [1, %d]", M_max, DS_MAX_TOPM);
  *bytes = lattice_ws_bytes(rows, vocab, M_max);
  return DS_OK;
}

int ds_build_lattice(const float* logits, int rows, int vocab, int M_max, float tau, int32_t eos_id,
                     int32_t* cand_id, float* cand_logp, int32_t* cand_cnt, float* eos_logp, float* lse,
                     void* ws, size_t ws_bytes, void* stream) {
  DS_REQUIRE(rows >= 0, DS_E_SHAPE, "rows %d is negative", rows);
  if (rows == 0) return DS_OK;  // empty block: nothing to do
  DS_REQUIRE(logits && cand_id && cand_logp && cand_cnt && eos_logp && lse && ws, DS_E_INVALID,
             "ds_build_lattice: NULL pointer argument");
  DS_REQUIRE(vocab >= 1 && (long long)rows * vocab < (1ll << 40), DS_E_SHAPE, "vocab %d not supported", vocab);
  DS_REQUIRE(M_max >= 1 && M_max <= DS_MAX_TOPM && M_max <= vocab, DS_E_SHAPE,
             "M_max %d outside [1, min(%d, vocab)]", M_max, DS_MAX_TOPM);
  DS_REQUIRE(eos_id < vocab, DS_E_INVALID, "eos_id %d >= vocab %d", eos_id, vocab);
  DS_REQUIRE(!isnan(tau) && tau > 0.f, DS_E_INVALID, "tau must be positive");
  DS_REQUIRE((((uintptr_t)logits) & 3) == 0, DS_E_INVALID, "logits not 4-byte aligned");
  return launch_lattice(logits, rows, vocab, M_max, tau, eos_id, cand_id, cand_logp, cand_cnt, eos_logp, lse, ws,
                        ws_bytes, static_cast<hipStream_t>(stream));
}

int ds_build_lattice_static(const float* logits, int rows, int vocab, int M_max, float tau, int32_t eos_id,
                            int32_t* cand_id, float* cand_logp, int32_t* cand_cnt, float* eos_logp, float* lse,
                            void* stream) {
  DS_REQUIRE(rows >= 0, DS_E_SHAPE, "rows %d is negative", rows);
  if (rows == 0) return DS_OK;
  DS_REQUIRE(logits && cand_id && cand_logp && cand_cnt && eos_logp && lse, DS_E_INVALID,
             "ds_build_lattice_static: NULL pointer argument");
  DS_REQUIRE(vocab >= 1 && (long long)rows * vocab < (1ll << 40), DS_E_SHAPE, "vocab %d not supported", vocab);
  DS_REQUIRE(M_max >= 1 && M_max <= DS_MAX_TOPM && M_max <= vocab, DS_E_SHAPE,
             "M_max %d outside [1, min(%d, vocab)]", M_max, DS_MAX_TOPM);
  DS_REQUIRE(eos_id < vocab, DS_E_INVALID, "eos_id %d >= vocab %d", eos_id, vocab);
  DS_REQUIRE(!isnan(tau) && tau > 0.f, DS_E_INVALID, "tau must be positive");
  DS_REQUIRE((((uintptr_t)logits) & 3) == 0, DS_E_INVALID, "logits not 4-byte aligned");
  const size_t need = lattice_ws_bytes(rows, vocab, M_max);
  DS_REQUIRE(need <= kStaticScratchBytes, DS_E_CAPACITY,
             "ds_build_lattice_static: %d rows x %d logits at M_max %d need %zu bytes of scratch, the library holds %zu "
             "(use ds_build_lattice with a caller workspace)",
             rows, vocab, M_max, need, kStaticScratchBytes);
  void* ws = nullptr;
  int rc = static_scratch(&ws);
  if (rc) return rc;
  return launch_lattice(logits, rows, vocab, M_max, tau, eos_id, cand_id, cand_logp, cand_cnt, eos_logp, lse, ws,
                        kStaticScratchBytes, static_cast<hipStream_t>(stream));
}

int ds_cps_workspace_bytes(int batch, int K, int M_max, size_t* bytes) {
  DS_REQUIRE(bytes, DS_E_INVALID, "bytes is NULL");
  DS_REQUIRE(batch >= 0 && K >= 1 && K <= 256, DS_E_SHAPE, "batch %d / K %d out of range", batch, K);
  DS_REQUIRE(M_max >= 1 && M_max <= DS_MAX_TOPM, DS_E_SHAPE, "M_max %d outside [1, %d]", M_max, DS_MAX_TOPM);
  *bytes = cps_ws_bytes(batch, K, M_max);
  return DS_OK;
}

int ds_ngram_create(const float* table, int log2_size, ds_ngram** out) {
  DS_REQUIRE(out, DS_E_INVALID, "out is NULL");
  *out = nullptr;
  DS_REQUIRE(table, DS_E_INVALID, "table is NULL");
  DS_REQUIRE(log2_size >= 1 && log2_size <= 30, DS_E_SHAPE, "log2_size %d outside [1, 30]", log2_size);
  ds_ngram* g = new (std::nothrow) ds_ngram{table, log2_size};
  DS_REQUIRE(g, DS_E_INVALID, "out of host memory");
  *out = g;
  return DS_OK;
}

void ds_ngram_destroy(ds_ngram* g) { delete g; }

int ds_cps_path(const int32_t* cand_id, const float* cand_logp, const int32_t* cand_cnt,
                const float* eos_logp, int batch, int K, int M_max, int B, float lambda,
                const ds_ngram* proxy, const int32_t* ctx, int32_t eos_id, int32_t* path,
                int32_t* path_len, float* path_score, int32_t* host_mirror, void* ws, size_t ws_bytes,
                void* stream) {
  DS_REQUIRE(batch >= 0, DS_E_SHAPE, "batch %d is negative", batch);
  if (batch == 0) return DS_OK;
  DS_REQUIRE(cand_id && cand_logp && cand_cnt && ctx && path && path_len && path_score, DS_E_INVALID,
             "ds_cps_path: NULL pointer argument");
  DS_REQUIRE(eos_id < 0 || eos_logp, DS_E_INVALID, "eos_logp is NULL while eos_id >= 0");
  DS_REQUIRE(K >= 1 && K <= 256, DS_E_SHAPE, "K %d outside [1, 256]", K);
  DS_REQUIRE(M_max >= 1 && M_max <= DS_MAX_TOPM, DS_E_SHAPE, "M_max %d outside [1, %d]", M_max, DS_MAX_TOPM);
  DS_REQUIRE(B >= 1 && B <= DS_MAX_BEAM, DS_E_SHAPE, "B %d outside [1, %d]", B, DS_MAX_BEAM);
  DS_REQUIRE(lambda >= 0.f && lambda <= 1.f, DS_E_INVALID, "lambda %g outside [0, 1]", (double)lambda);
  DS_REQUIRE(!ws || (((uintptr_t)ws) & 15) == 0, DS_E_INVALID, "workspace not 16-byte aligned");
  return launch_cps(cand_id, cand_logp, cand_cnt, eos_logp, batch, K, M_max, B, lambda,
                    proxy ? proxy->table : nullptr, proxy ? proxy->log2_size : 0, ctx, eos_id, path, path_len,
                    path_score, host_mirror, ws, ws_bytes, static_cast<hipStream_t>(stream));
}

int ds_sample_workspace_bytes(int m, size_t* bytes) {
  DS_REQUIRE(bytes, DS_E_INVALID, "bytes is NULL");
  DS_REQUIRE(m >= 0 && m < DS_MAX_ROWS, DS_E_SHAPE, "m %d outside [0, %d)", m, DS_MAX_ROWS);
  *bytes = sample_ws_bytes(m);
  return DS_OK;
}

int ds_accept_stochastic(const float* p_logits, const float* q_logits, int m, int vocab, const int32_t* block,
                         const int32_t* path_len, const float* u, int32_t eos_id, int32_t* n_accept,
                         int32_t* next_token, int32_t* eos_accepted, float* alpha, void* ws, size_t ws_bytes,
                         void* stream) {
  DS_REQUIRE(m >= 0 && m < DS_MAX_ROWS, DS_E_SHAPE, "m %d outside [0, %d)", m, DS_MAX_ROWS);
  DS_REQUIRE(vocab >= 1, DS_E_SHAPE, "vocab %d must be positive", vocab);
  DS_REQUIRE(p_logits && block && u && n_accept && next_token && eos_accepted && ws, DS_E_INVALID,
             "ds_accept_stochastic: NULL pointer argument");
  DS_REQUIRE(m == 0 || (q_logits && alpha), DS_E_INVALID, "q_logits / alpha is NULL while m > 0");
  DS_REQUIRE(eos_id < vocab, DS_E_INVALID, "eos_id %d >= vocab %d", eos_id, vocab);
  DS_REQUIRE((((uintptr_t)ws) & 3) == 0, DS_E_INVALID, "workspace not 4-byte aligned");
  return launch_sample_accept(p_logits, q_logits, m, vocab, block, path_len, u, eos_id, n_accept, next_token,
                              eos_accepted, alpha, ws, ws_bytes, static_cast<hipStream_t>(stream));
}

int ds_refine_select(const int32_t* cand_id, const float* cand_logp, const int32_t* cand_cnt,
                     const float* eos_logp, const float* lse, int K, int M_max, int n_update, int32_t mask_id,
                     int32_t* block_tokens, int32_t* out_cand_id, float* out_cand_logp, int32_t* out_cand_cnt,
                     float* out_eos_logp, float* out_lse, void* stream) {
  DS_REQUIRE(K >= 1 && K <= 256, DS_E_SHAPE, "K %d outside [1, 256]", K);
  DS_REQUIRE(M_max >= 1 && M_max <= DS_MAX_TOPM, DS_E_SHAPE, "M_max %d outside [1, %d]", M_max, DS_MAX_TOPM);
  DS_REQUIRE(n_update >= 0, DS_E_SHAPE, "n_update %d is negative", n_update);
  DS_REQUIRE(cand_id && cand_logp && cand_cnt && eos_logp && lse && block_tokens && out_cand_id && out_cand_logp &&
                 out_cand_cnt && out_eos_logp && out_lse,
             DS_E_INVALID, "ds_refine_select: NULL pointer argument");
  return launch_refine_select(cand_id, cand_logp, cand_cnt, eos_logp, lse, K, M_max, n_update, mask_id, block_tokens,
                              out_cand_id, out_cand_logp, out_cand_cnt, out_eos_logp, out_lse,
                              static_cast<hipStream_t>(stream));
}

int ds_refine_update_sizes(int K, int steps, int* sizes, int* n_sizes) {
  DS_REQUIRE(sizes && n_sizes, DS_E_INVALID, "ds_refine_update_sizes: NULL pointer argument");
  DS_REQUIRE(K >= 1 && K <= 256 && steps >= 1, DS_E_SHAPE, "need 1 <= K <= 256 and steps >= 1 (got %d, %d)", K, steps);
  int left = K, n = 0;
  for (int s = 1; s <= steps && left > 0; ++s) {
    const int share = steps - s + 1;
    const int u = (left + share - 1) / share;  // ceil(|M_{s-1}| / (S - s + 1))
    sizes[n++] = u;
    left -= u;
  }
  *n_sizes = n;
  return DS_OK;
}

int ds_adl_first_eos(const int32_t* raw_draft, int k, int stride, int32_t eos_id, int* first_eos) {
  DS_REQUIRE(raw_draft && first_eos, DS_E_INVALID, "ds_adl_first_eos: NULL pointer argument");
  DS_REQUIRE(k >= 0 && stride >= 1, DS_E_SHAPE, "need k >= 0 and stride >= 1 (got %d, %d)", k, stride);
  *first_eos = 0;
  if (eos_id < 0) return DS_OK;
  for (int i = 0; i < k; ++i)
    if (raw_draft[(size_t)i * stride] == eos_id) {
      *first_eos = i + 1;
      break;
    }
  return DS_OK;
}

int ds_adl_create(int k_min, int k_max, double delta, double rho, ds_adl** out) {
  DS_REQUIRE(out, DS_E_INVALID, "out is NULL");
  *out = nullptr;
  DS_REQUIRE(k_min >= 1 && k_max >= k_min, DS_E_INVALID, "need 1 <= k_min <= k_max (got %d, %d)", k_min, k_max);
  DS_REQUIRE(delta >= 0.0, DS_E_INVALID, "delta must be >= 0");
  DS_REQUIRE(rho > 0.0 && rho <= 1.0, DS_E_INVALID, "rho %g outside (0, 1]", rho);
  ds_adl* a = new (std::nothrow) ds_adl{k_min, k_max, delta, rho, 0.0, 0.0};
  DS_REQUIRE(a, DS_E_INVALID, "out of host memory");
  *out = a;
  return DS_OK;
}

void ds_adl_destroy(ds_adl* a) { delete a; }

int ds_adl_update(ds_adl* a, int k_t, int first_eos, int l_acc, int* k_next) {
  DS_REQUIRE(a && k_next, DS_E_INVALID, "ds_adl_update: NULL pointer argument");
  DS_REQUIRE(k_t >= 1 && first_eos >= 0 && l_acc >= 0, DS_E_INVALID,
             "need k_t >= 1, first_eos >= 0, l_acc >= 0 (got %d, %d, %d)", k_t, first_eos, l_acc);
  const int l_gen = (first_eos > 0 && first_eos - 1 < k_t) ? first_eos - 1 : k_t;
  a->l_gen_ema = (1.0 - a->rho) * a->l_gen_ema + a->rho * (double)l_gen;
  a->l_acc_ema = (1.0 - a->rho) * a->l_acc_ema + a->rho * (double)l_acc;
  const double z = ceil(a->l_gen_ema + (a->l_acc_ema >= a->l_gen_ema ? a->delta : 0.0));
  double k = z < (double)a->k_min ? (double)a->k_min : z;
  k = k > (double)a->k_max ? (double)a->k_max : k;
  *k_next = (int)k;
  return DS_OK;
}

int ds_adl_state(const ds_adl* a, double* l_gen_ema, double* l_acc_ema) {
  DS_REQUIRE(a && l_gen_ema && l_acc_ema, DS_E_INVALID, "ds_adl_state: NULL pointer argument");
  *l_gen_ema = a->l_gen_ema;
  *l_acc_ema = a->l_acc_ema;
  return DS_OK;
}

}  // extern "C"
