/*
 * libdiffuspec: one DiffuSpec speculative-decoding round on one MI355X (gfx950).
 *
 * The round (Alg. 1 of the paper, "DIFFUSPEC (4-stage)"):
 *   (1) the diffusion-LM drafter fills K [MASK] positions in a single pass      -> ds_draft_block
 *       and exposes a per-position top-M candidate lattice with log-scores       -> ds_build_lattice
 *   (2) causal-consistency path search picks one left-to-right path              -> ds_cps_path
 *   (3) the autoregressive target verifies the path in one parallel pass and
 *       keeps the longest accepted prefix (greedy verification)                  -> ds_verify_block
 *   (4) the adaptive draft-length controller sets the next K                     -> ds_adl_update
 *
 * Conventions
 *   - Plain C ABI.  Every function returns an int status (DS_OK = 0, negatives are errors);
 *     ds_last_error() gives the text of the calling thread's last error.
 *   - Arguments are validated on the host before anything is launched: a failed call enqueues
 *     no work and changes no state.
 *   - Ownership: the caller allocates and frees ALL device memory (weights, packed weights, KV
 *     caches, workspace, inputs, outputs) and passes raw device pointers.  The library only
 *     allocates small host structs behind the opaque handles, released by the *_destroy calls.
 *     Pointers marked [dev] are device memory (any memory the GPU can address: small outputs such as the
 *     acceptance verdict may also live in pinned, device-visible host memory), [host] host memory.
 *   - All device work is enqueued on `stream` (a hipStream_t passed as void*, NULL = default
 *     stream) and the call returns without synchronising.  Outputs are device memory; the caller
 *     synchronises the stream before reading them.
 *   - Determinism: the same inputs give bit-identical outputs (no floating-point atomics).
 *   - One GPU; calls that use the same handle or the same workspace must not overlap.
 */
#ifndef DS_H
#define DS_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define DS_OK 0
#define DS_E_INVALID (-1)     /* null pointer, bad alignment, value out of range */
#define DS_E_SHAPE (-2)       /* shape not supported by the kernels */
#define DS_E_CAPACITY (-3)    /* KV cache, workspace or packed-weight buffer too small */
#define DS_E_UNSUPPORTED (-4) /* dtype / head_dim / feature not implemented */
#define DS_E_HIP (-5)         /* a HIP runtime call failed */

#define DS_F32 0
#define DS_BF16 1

#define DS_MAX_ROWS 144 /* most rows one forward call may carry (pending + K, or m + 1) */
#define DS_MAX_TOPM 16  /* largest lattice width M_max */
#define DS_MAX_BEAM 16  /* largest beam width B */

#define DS_MAX_SEQ 8    /* most sequences one batched forward call may carry */

typedef struct ds_model ds_model;
typedef struct ds_kv ds_kv;
typedef struct ds_ngram ds_ngram;
typedef struct ds_adl ds_adl;

/* Shape of one pre-RMSNorm decoder with grouped-query attention, rotary embedding (rotate-half
 * pairing, absolute positions) and a SwiGLU MLP; no biases; untied embedding and LM head. */
typedef struct {
  int32_t n_layers, d_model, n_q, n_kv, head_dim, d_ffn, vocab;
  float rope_base, rms_eps;
  int32_t dtype;       /* DS_F32 or DS_BF16: storage type of the weights.  DS_BF16: bf16 weights (re-encoded
                          exactly as IEEE half inside the library), IEEE-half activations at every matrix
                          product and in the KV cache, float32 accumulation, residual stream and logits.
                          Half activations saturate at +-65504 instead of overflowing; every saturated value
                          is counted (ds_model_overflow_count).  DS_F32: everything float32. */
  int32_t kv_capacity; /* tokens each layer's KV buffer can hold (bf16: a multiple of 64) */
} ds_model_cfg;

/* Canonical weights: every matrix row-major [out_features, in_features] in cfg.dtype;
 * norm gains are float32 vectors of d_model. */
typedef struct {
  const void *wq, *wk, *wv, *wo, *w_gate, *w_up, *w_down; /* [dev] */
  const float *norm1, *norm2;                              /* [dev] */
} ds_layer_weights;

typedef struct {
  const void* embed;              /* [dev] [vocab, d_model] */
  const ds_layer_weights* layers; /* [host] array of n_layers */
  const float* final_norm;        /* [dev] */
  const void* lm_head;            /* [dev] [vocab, d_model] */
} ds_weights;

const char* ds_version(void);
const char* ds_last_error(void);

/* Bytes the caller must provide for kernel-order copies of the weights (0 for DS_F32) and for the
 * per-call workspace when at most max_rows rows go through one call. */
int ds_model_packed_bytes(const ds_model_cfg* cfg, size_t* bytes);
int ds_workspace_bytes(const ds_model_cfg* cfg, int max_rows, size_t* bytes);
/* Bytes of ONE of the two KV buffers (keys or values) for cfg. */
int ds_kv_bytes(const ds_model_cfg* cfg, size_t* bytes);

/* Bind a model.  For DS_BF16 this runs kernels that copy the matrices, re-encoded as IEEE half, into
 * the order the GEMM kernels stream them in (`packed`, ds_model_packed_bytes() bytes, 256-byte
 * aligned) and waits for them (this one call synchronises `stream`); afterwards the canonical matrices
 * other than `embed` are no longer read.  The re-encoding is exact for 2^-14 <= |w| <= 65504 (smaller
 * magnitudes round to multiples of 2^-24); a NaN or a weight beyond +-65504 fails the call with
 * DS_E_UNSUPPORTED.  For DS_F32 nothing is copied and the canonical matrices are read by every call.  kv_k / kv_v: ds_kv_bytes()
 * each; their internal layout is private to the library.  The committed KV length starts at 0. */
int ds_model_create(const ds_model_cfg* cfg, const ds_weights* w, void* packed, size_t packed_bytes,
                    void* kv_k, void* kv_v, void* stream, ds_model** out);
void ds_model_destroy(ds_model* m);

/* DS_BF16 models run every activation that meets a weight, and q / k / v, in IEEE half: a value beyond +-65504 (or a
 * NaN) is clamped to +-65504 instead of becoming infinite, and counted.  *count [host] receives the number of such
 * activation values since the model was created or the counter was last reset (reset != 0 clears it); 0 means no
 * forward of this model was touched by the half range.  Always 0 for DS_F32.  Synchronises `stream`. */
int ds_model_overflow_count(ds_model* m, int reset, void* stream, uint32_t* count);

/* Committed KV length: query, and set (truncate after a rejection / commit after verification). */
int ds_model_kv_len(const ds_model* m, int* len);
int ds_model_kv_set_len(ds_model* m, int len);

/* Causal forward of n real tokens (any n >= 1; processed in chunks), appended to the KV cache and
 * committed.  tokens [dev] int32[n].  last_logits [dev] float[vocab] or NULL: logits of the last
 * token.  Setup path: not part of the timed round. */
int ds_prefill(ds_model* m, const int32_t* tokens, int n, float* last_logits, void* ws, size_t ws_bytes,
               void* stream);

/* Step 1, drafter pass with S = 1 (Sec. 3.1 "Inference"; Alg. 1 step (1)).
 * Rows = n_pend real tokens (tokens committed since the drafter last ran; causal) followed by K
 * [MASK] tokens (each sees the whole cached prefix, the pending tokens and all K block positions).
 * Keys/values of the pending rows are appended and committed (length += n_pend); those of the mask
 * rows are scratch and never committed.  pending [dev] int32[n_pend] (may be NULL iff n_pend == 0).
 * hidden_out [dev] float[K, d_model]: final-normed hidden states of the mask rows; the state at block
 * position i gives the distribution of the token AT position i.
 * Requires 1 <= K, n_pend + K <= DS_MAX_ROWS, kv_len + n_pend + K <= kv_capacity. */
int ds_draft_block(ds_model* drafter, const int32_t* pending, int n_pend, int K, int32_t mask_id,
                   float* hidden_out, void* ws, size_t ws_bytes, void* stream);

/* logits[rows, vocab] = hidden[rows, d_model] times the LM head (all [dev] float32; DS_BF16 models round
 * each hidden value to IEEE half and accumulate the half x half products in float32).
 * hidden == NULL: multiply the block rows of the draft pass (ds_draft_block / ds_draft_block_tokens) that was the
 * last forward on this model and this workspace, rows == its K; the result is bit-identical to passing that
 * call's hidden_out, without converting it again.  Any other state fails with DS_E_INVALID. */
int ds_lm_head(ds_model* m, const float* hidden, int rows, float* logits, void* ws, size_t ws_bytes,
               void* stream);

/* Step 2, token lattice (Sec. 3.2 "Lattice and pruning").  Per row r of logits [dev] float[rows, vocab]:
 *   lse[r]           = log sum_v exp(logit)
 *   cand_id[r, :]    = the M_max largest logits' token ids (logit descending, ties: lower id)
 *   cand_logp[r, :]  = logit - lse  (the drafter log-score l_dlm of each candidate)
 *   cand_cnt[r]      = smallest m <= M_max whose cumulative probability >= tau (M_max if none;
 *                      tau >= 1 disables pruning)
 *   eos_logp[r]      = logit[eos_id] - lse (0 if eos_id < 0)
 * Outputs [dev]: cand_id int32[rows, M_max], cand_logp float[rows, M_max], cand_cnt int32[rows],
 * eos_logp float[rows], lse float[rows].  1 <= M_max <= DS_MAX_TOPM <= vocab.
 * ws: ds_lattice_workspace_bytes(rows, vocab, M_max) bytes.  NaN logits are a caller error. */
int ds_lattice_workspace_bytes(int rows, int vocab, int M_max, size_t* bytes);
int ds_build_lattice(const float* logits, int rows, int vocab, int M_max, float tau, int32_t eos_id,
                     int32_t* cand_id, float* cand_logp, int32_t* cand_cnt, float* eos_logp, float* lse,
                     void* ws, size_t ws_bytes, void* stream);

/* ds_build_lattice for callers that cannot allocate device memory or hand over a workspace (code under HIP graph
 * capture, tight serving loops, harnesses that forbid allocation): same inputs, outputs, rules and kernels, but the
 * scan's partial records live in a 2 MiB array inside the library's own device image (one copy per GPU, held until
 * the process ends).  The call allocates nothing.  Shapes whose ds_lattice_workspace_bytes() exceeds 2 MiB fail with
 * DS_E_CAPACITY (every rows <= 3855 fits at any vocab and M_max).  Nothing in the array needs clearing between
 * calls (each call overwrites what it reads), but all calls on one GPU share it: calls that overlap on one GPU
 * (different streams or threads) race and must be serialised by the caller. */
int ds_build_lattice_static(const float* logits, int rows, int vocab, int M_max, float tau, int32_t eos_id,
                            int32_t* cand_id, float* cand_logp, int32_t* cand_cnt, float* eos_logp, float* lse,
                            void* stream);

/* Steps 1b + 2 without the logits round trip (Sec. 3.2 "Lattice and pruning").
 * ds_lm_head_tiles: the LM head of ds_lm_head (hidden as there; NULL = the block rows of the preceding draft
 * pass), leaving in the workspace what the lattice needs.  On DS_BF16 models those are per-tile records written by
 * the product itself (per 128 token ids and row: the two largest logits with their ids, the third largest value,
 * the sum of exponentials) plus the logits of eos_id, so with logits_out == NULL the logits never reach memory;
 * logits_out [dev] float[rows, vocab] receives them if given.  DS_F32 models (and vocabularies the records do not
 * cover: not a multiple of 128, or above 262144) keep the logits, in logits_out or the workspace.
 * ds_lattice_from_tiles: the lattice of ds_build_lattice for those rows, same outputs, same rules (ties: lower id).
 * It must directly follow ds_lm_head_tiles on the same model and workspace with the same rows and eos_id
 * (DS_E_INVALID otherwise).  A tile whose third value could still enter the top-M_max is recomputed with the
 * product's own instruction sequence, so the candidates are exactly those of the logits ds_lm_head would write;
 * lse is summed tile by tile and may differ from ds_build_lattice's in the last bits.
 * ds_draft_lattice: both steps in one call. */
int ds_lm_head_tiles(ds_model* drafter, const float* hidden, int rows, int32_t eos_id, float* logits_out, void* ws,
                     size_t ws_bytes, void* stream);
int ds_lattice_from_tiles(ds_model* drafter, int rows, int M_max, float tau, int32_t eos_id, int32_t* cand_id,
                          float* cand_logp, int32_t* cand_cnt, float* eos_logp, float* lse, void* ws,
                          size_t ws_bytes, void* stream);
int ds_draft_lattice(ds_model* drafter, const float* hidden, int rows, int M_max, float tau, int32_t eos_id,
                     int32_t* cand_id, float* cand_logp, int32_t* cand_cnt, float* eos_logp, float* lse,
                     float* logits_out, void* ws, size_t ws_bytes, void* stream);

/* Causal proxy for the path search: a table of 2^log2_size float32 natural-log scores [dev]; the
 * 3-gram (u, v, w) reads slot hash(u, v, w) (fixed uint32 multiply / xor-shift mix). */
int ds_ngram_create(const float* table, int log2_size, ds_ngram** out);
void ds_ngram_destroy(ds_ngram* g);

/* Step 3, causal-consistency path search (Sec. 3.2 "Scoring and search"; Alg. 1 step (2)).
 * For each of `batch` independent sequences (lattice rows [s*K, (s+1)*K)): left-to-right beam search of
 * width B over the pruned lattice (EOS always a candidate, appended last if absent) maximising
 *   S(path) = sum_i [ lambda * l_dlm_i + (1 - lambda) * l_ng(path_i | two previous tokens) ],
 * float32 unfused, kept hypotheses ordered by (score desc, parent asc, candidate rank asc); returns at
 * the first depth whose best hypothesis ends in EOS (EOS included), else after K positions.
 * proxy NULL: l_ng = 0.  ctx [dev] int32[batch, 2]: the two tokens before each block (older first).
 * Outputs [dev]: path int32[batch, K] (tail beyond the length = -1), path_len int32[batch],
 * path_score float[batch].  1 <= B <= DS_MAX_BEAM, 1 <= M_max <= DS_MAX_TOPM, 1 <= K <= 256.
 * host_mirror, optional (NULL allowed) [host, pinned, device-visible] int32[batch, 2 K + 1]: the kernel also stores
 * there, per sequence, the path (K entries, tail -1), its length, and the raw draft (the top candidate of each of
 * the K positions: what the first-EOS index of Sec. 3.3 is taken from), so that a host loop reads them without a
 * copy of its own; they are complete once any later work of the stream is seen to have completed.
 * ws [dev], optional (NULL allowed): ds_cps_workspace_bytes() bytes of scratch that lets the proxy scores
 * be gathered by the whole chip before the search starts; results do not depend on it. */
int ds_cps_workspace_bytes(int batch, int K, int M_max, size_t* bytes);
int ds_cps_path(const int32_t* cand_id, const float* cand_logp, const int32_t* cand_cnt,
                const float* eos_logp, int batch, int K, int M_max, int B, float lambda,
                const ds_ngram* proxy, const int32_t* ctx, int32_t eos_id, int32_t* path,
                int32_t* path_len, float* path_score, int32_t* host_mirror, void* ws, size_t ws_bytes,
                void* stream);

/* Step 3 with the other causal proxy the paper names: a tiny causal LM instead of the n-gram table
 * (Sec. 3.2 "Scoring and search": the path score mixes the drafter's log-score with a small causal proxy,
 * an n-gram or a tiny causal LM).  Here l_ng of a hypothesis' next token w is log softmax(z)[w] (float32), z the
 * logits of the proxy model after the committed tokens followed by the hypothesis' tokens; the search itself
 * (candidates, EOS rule, ordering, float32 score arithmetic) is that of ds_cps_path.  One sequence per call.
 *
 * The proxy is any ds_model that shares the vocabulary (a small one: it takes one step per depth and beam slot).
 * ds_lmproxy_create binds it to `mem` [dev], ds_lmproxy_bytes(cfg of the model, beam) bytes, 256-byte aligned,
 * caller-owned: 2 * beam KV caches (every beam slot is a sequence of its own; the beam's reordering copies the
 * block region of a parent's cache) and the search state.  The model's own cache is not used.  `beam` (at most 8)
 * is the widest beam later calls may ask for.
 * ds_lmproxy_prefill appends n committed tokens [dev] to the proxy's history (chunked forward; setup path).
 * ds_lmproxy_len / _set_len: committed length; it can only be cut back (for a replay from an earlier point).
 * ds_cps_path_lm: pending [dev] int32[n_pend], n_pend >= 1: the tokens committed since the proxy's history was
 * last extended, the last committed token included (what ds_draft_block takes as `pending`); they are appended to
 * the history.  The lattice arguments, eos_id, B, lambda and the outputs path int32[K] (tail beyond the length
 * = -1), path_len int32[1], path_score float[1] [dev] are those of ds_cps_path with batch = 1.
 * 1 <= K <= 256, 1 <= B <= beam of the proxy, history + n_pend + K - 1 <= the model's kv_capacity.
 * ws [dev]: the proxy model's workspace, ds_workspace_bytes(cfg, DS_MAX_ROWS) bytes.
 * Everything is enqueued on `stream` (K proxy forwards, nothing returns to the host in between); after an
 * EOS has ended the search the remaining steps run without effect. */
typedef struct ds_lmproxy ds_lmproxy;
int ds_lmproxy_bytes(const ds_model_cfg* cfg, int beam, size_t* bytes);
int ds_lmproxy_create(ds_model* lm, int beam, void* mem, size_t mem_bytes, ds_lmproxy** out);
void ds_lmproxy_destroy(ds_lmproxy* proxy);
int ds_lmproxy_prefill(ds_lmproxy* proxy, const int32_t* tokens, int n, void* ws, size_t ws_bytes, void* stream);
int ds_lmproxy_len(const ds_lmproxy* proxy, int* len);
int ds_lmproxy_set_len(ds_lmproxy* proxy, int len);
int ds_cps_path_lm(const int32_t* cand_id, const float* cand_logp, const int32_t* cand_cnt,
                   const float* eos_logp, int K, int M_max, int B, float lambda, ds_lmproxy* proxy,
                   const int32_t* pending, int n_pend, int32_t eos_id, int32_t* path, int32_t* path_len,
                   float* path_score, void* ws, size_t ws_bytes, void* stream);

/* Step 4, parallel verification with greedy acceptance (Sec. 2 "Parallel verification" and
 * "Accepted prefix length"; Alg. 1 step (3); greedy verification as in Sec. 4).
 * block [dev] int32[m + 1] = last committed token followed by the path (ids outside [0, vocab) are
 * read as token 0; such rows lie past path_len and are ignored).  path_len [dev] int32 or NULL: if
 * given, only the first min(m, *path_len) path tokens take part in acceptance.
 * Causal forward of the m + 1 rows against the verifier's KV cache, LM head, per-row arg-max (ties:
 * lower id); n_accept = number of leading path tokens equal to the arg-max of the row before them;
 * next_token = argmax[n_accept]; eos_accepted = 1 if an accepted token or next_token is eos_id.
 * Keys/values of all rows are written at [len, len + m + 1) but the committed length is NOT advanced:
 * after reading n_accept the caller commits with ds_model_kv_set_len(len + 1 + n_accept).
 * Outputs [dev]: n_accept, next_token, eos_accepted int32[1]; argmax int32[m + 1];
 * logits_out float[m + 1, vocab] or NULL.  0 <= m, m + 1 <= DS_MAX_ROWS.
 * eos_accepted is stored last, after a system-scope fence: if the three scalars live in device-visible pinned
 * host memory, a host that sees eos_accepted change also sees n_accept and next_token (the round's one host
 * crossing can be a poll of that word instead of a stream synchronisation). */
int ds_verify_block(ds_model* verifier, const int32_t* block, int m, const int32_t* path_len,
                    int32_t eos_id, int32_t* n_accept, int32_t* next_token, int32_t* argmax,
                    int32_t* eos_accepted, float* logits_out, void* ws, size_t ws_bytes, void* stream);

/* ds_verify_block that also leaves on the device what the next round reads (Alg. 1: the accepted prefix and the
 * verifier's token are appended to the sequence; the next round drafts after them, scores its first positions
 * against the last two of them, and verifies a block that starts with the last one), so that a driver sends no
 * token to the device between rounds.  carry [dev] int32[DS_MAX_ROWS + 2], written by the acceptance kernel
 * before the verdict: the n_accept + 1 committed tokens (accepted path tokens, then next_token) right-aligned in
 * carry[0, DS_MAX_ROWS), i.e. at carry + DS_MAX_ROWS - (n_accept + 1) -- the next ds_draft_block's `pending`;
 * carry[DS_MAX_ROWS] = the token before the last committed one (block[0] if n_accept = 0) and
 * carry[DS_MAX_ROWS + 1] = next_token -- the next ds_cps_path's ctx, and the next block's first word.
 * carry may not overlap block, except that carry[DS_MAX_ROWS + 1] may be block[0] (read before it is written).
 * Everything else as ds_verify_block. */
int ds_verify_block_carry(ds_model* verifier, const int32_t* block, int m, const int32_t* path_len,
                          int32_t eos_id, int32_t* n_accept, int32_t* next_token, int32_t* argmax,
                          int32_t* eos_accepted, float* logits_out, int32_t* carry, void* ws, size_t ws_bytes,
                          void* stream);

/* Stochastic block verification (Sec. 2 "Parallel verification": acceptance probability
 * alpha_i = min(1, p(y_i) / q(y_i)), residual resampling; Sec. 2 left-to-right proxy q^L2R: with a single
 * drafter pass every in-block position is [MASK], so the drafter row of block position i IS the proxy).
 * Stand-alone form on given logits (all [dev]): p_logits float[m + 1, vocab] verifier rows (row r scores the
 * token after block[r]), q_logits float[m, vocab] drafter rows of the path positions, block int32[m + 1],
 * path_len int32 or NULL (as in ds_verify_block), u float[m + 1]: u[i] < alpha_i accepts draft token i + 1,
 * u[m] drives the one draw.  After the accepted prefix of length L the next token is drawn by inverse CDF in
 * vocabulary order (smallest v whose cumulative weight exceeds u[m] * total) from max(p_L - q_L, 0) after a
 * rejection, from p_L after full acceptance (also when the residual is empty).  float32 arithmetic, fixed
 * summation order; the caller owns the random stream.  Outputs [dev]: n_accept, next_token, eos_accepted
 * int32[1], alpha float[m].  ws: ds_sample_workspace_bytes(m) bytes.  0 <= m < DS_MAX_ROWS. */
int ds_sample_workspace_bytes(int m, size_t* bytes);
int ds_accept_stochastic(const float* p_logits, const float* q_logits, int m, int vocab, const int32_t* block,
                         const int32_t* path_len, const float* u, int32_t eos_id, int32_t* n_accept,
                         int32_t* next_token, int32_t* eos_accepted, float* alpha, void* ws, size_t ws_bytes,
                         void* stream);
/* The verifier pass of ds_verify_block followed by ds_accept_stochastic on its logits (same KV rules: nothing
 * is committed).  q_logits [dev] float[m, vocab]: the drafter's logits of block positions 1..m (what
 * ds_lm_head wrote for the draft block).  The model workspace `ws` also holds the sampling scratch. */
int ds_verify_block_stochastic(ds_model* verifier, const int32_t* block, int m, const int32_t* path_len,
                               const float* q_logits, const float* u, int32_t eos_id, int32_t* n_accept,
                               int32_t* next_token, int32_t* eos_accepted, float* alpha, float* logits_out,
                               void* ws, size_t ws_bytes, void* stream);

/* Multi-pass refinement of the draft block (Sec. 2 "Inference (iterative refinement)", refinement update
 * equation; S > 1 in Sec. 4).  ds_draft_block_tokens is ds_draft_block with explicit block contents:
 * block_tokens [dev] int32[K] holds the current draft (fixed tokens, mask_id where still masked); every block
 * row still sees the whole block.  ds_refine_select is the update: among the positions still holding mask_id,
 * the n_update with the largest top-1 log-probability cand_logp[i, 0] (ties: lower position) are fixed to
 * cand_id[i, 0] in block_tokens, and their rows of the pass lattice (cand_*, eos_logp, lse: as written by
 * ds_build_lattice for this pass) are copied to the out_* lattice, which after the last pass is the lattice the
 * path search runs on.  1 <= K <= 256, 1 <= M_max <= DS_MAX_TOPM, 0 <= n_update. */
int ds_draft_block_tokens(ds_model* drafter, const int32_t* pending, int n_pend, const int32_t* block_tokens,
                          int K, float* hidden_out, void* ws, size_t ws_bytes, void* stream);
int ds_refine_select(const int32_t* cand_id, const float* cand_logp, const int32_t* cand_cnt,
                     const float* eos_logp, const float* lse, int K, int M_max, int n_update, int32_t mask_id,
                     int32_t* block_tokens, int32_t* out_cand_id, float* out_cand_logp, int32_t* out_cand_cnt,
                     float* out_eos_logp, float* out_lse, void* stream);

/* The update schedule of the refinement (Sec. 2, refinement update equation; the paper leaves |U_s| open): pass s of
 * S fixes |U_s| = ceil(|M_{s-1}| / (S - s + 1)) of the still-masked positions, so a block of K positions is complete
 * after exactly min(S, K) passes.  Pure host code.  sizes [host] int[steps] receives |U_1|, |U_2|, ...; *n_sizes the
 * number of passes (<= steps). */
int ds_refine_update_sizes(int K, int steps, int* sizes, int* n_sizes);

/* Several sequences per call (batch > 1; Sec. 6 names batching as the way to better hardware use; every step of the
 * round is defined per sequence, so a batch is n_seq independent rounds that share one pass over the weights).
 * A ds_kv is one more sequence's KV cache of a model: kv_k / kv_v [dev] of ds_kv_bytes() each, owned by the caller;
 * its committed length starts at 0.  The cache passed to ds_model_create is the model's built-in sequence, used by
 * the single-sequence calls; the batched calls take explicit handles (distinct, all of the same model).
 * ds_prefill_seq: ds_prefill into the given sequence.
 * ds_draft_block_batch: ds_draft_block for n_seq <= DS_MAX_SEQ sequences.  pending [dev]: the pending tokens of all
 * sequences, concatenated in sequence order; n_pend [host] int[n_seq]; the same K for every sequence; hidden_out
 * [dev] float[n_seq * K, d_model], sequence-major.  Each sequence's rows are placed at a multiple of 16 inside the
 * call: sum over sequences of (n_pend[s] + K rounded up to 16; the last one not rounded) must not exceed DS_MAX_ROWS.
 * A following ds_draft_lattice(hidden = NULL, rows = n_seq * K) gives the lattice rows [s * K, (s + 1) * K) that
 * ds_cps_path(batch = n_seq) searches.
 * ds_verify_block_batch: ds_verify_block for n_seq sequences of m + 1 rows each: first [dev] int32[n_seq] (each
 * sequence's last committed token), path [dev] int32[n_seq, m] (what ds_cps_path wrote), path_len [dev] int32[n_seq]
 * or NULL.  Outputs [dev]: n_accept, next_token, eos_accepted int32[n_seq]; argmax int32[n_seq, m + 1]; logits_out
 * float[rows, vocab] or NULL, where sequence s occupies rows [s * R, s * R + m + 1) with R = m + 1 rounded up to 16.
 * The eos_accepted words are stored last, after a system-scope fence.  Committed lengths are not advanced: the caller
 * commits each sequence with ds_kv_set_len(len + 1 + n_accept[s]).
 * Every row's result is bit-identical to what the single-sequence call gives for that sequence alone. */
int ds_kv_create(ds_model* m, void* kv_k, void* kv_v, ds_kv** out);
void ds_kv_destroy(ds_kv* kv);
int ds_kv_len(const ds_kv* kv, int* len);
int ds_kv_set_len(ds_kv* kv, int len);
int ds_prefill_seq(ds_model* m, ds_kv* kv, const int32_t* tokens, int n, float* last_logits, void* ws,
                   size_t ws_bytes, void* stream);
int ds_draft_block_batch(ds_model* drafter, ds_kv* const* seqs, int n_seq, const int32_t* pending, const int* n_pend,
                         int K, int32_t mask_id, float* hidden_out, void* ws, size_t ws_bytes, void* stream);
int ds_verify_block_batch(ds_model* verifier, ds_kv* const* seqs, int n_seq, const int32_t* first,
                          const int32_t* path, int m, const int32_t* path_len, int32_t eos_id, int32_t* n_accept,
                          int32_t* next_token, int32_t* argmax, int32_t* eos_accepted, float* logits_out, void* ws,
                          size_t ws_bytes, void* stream);

/* Step 4 tail, adaptive draft length (Sec. 3.3: generation-length signal, moving averages,
 * controller).  Pure host code in double precision.  first_eos: 1-based index of the first EOS in the
 * raw draft (per-position top-1 before the search), 0 if none.  Averages start at 0 (Alg. 1 init). */
int ds_adl_create(int k_min, int k_max, double delta, double rho, ds_adl** out);
/* s_t of the generation-length signal (Sec. 3.3): the 1-based index of the first eos_id in the raw draft, 0 if
 * there is none or eos_id < 0.  raw_draft [host]: token i at raw_draft[i * stride], i < k (the top-1 column of the
 * candidate ids as the host read them back: stride = M_max).  Pure host code. */
int ds_adl_first_eos(const int32_t* raw_draft, int k, int stride, int32_t eos_id, int* first_eos);
void ds_adl_destroy(ds_adl* a);
int ds_adl_update(ds_adl* a, int k_t, int first_eos, int l_acc, int* k_next);
int ds_adl_state(const ds_adl* a, double* l_gen_ema, double* l_acc_ema);

/* The whole loop of Alg. 1 as one call: n_rounds rounds (draft -> lattice -> path search -> verification ->
 * draft-length update) driven from inside the library, one host crossing per round (the verdict, polled in pinned
 * memory) and no host -> device traffic between rounds (ds_verify_block_carry).  A client of the entry points above:
 * the same kernels, the same results as calling them one by one.  Greedy verification, single-pass draft, one
 * sequence, n-gram proxy (or none).
 *
 * ds_round_desc names every buffer; all caller-owned.  io [dev] int32[total of ds_round_io_layout(K_cap, M_max)]:
 *   io[0, DS_MAX_ROWS)                  pending tokens, right-aligned (the next ds_draft_block's `pending`)
 *   io[DS_MAX_ROWS], io[DS_MAX_ROWS+1]  the two tokens before the block; the second is also block[0]
 *   io[path_at, path_at + K_cap)        the searched path (path_at = DS_MAX_ROWS + 2), io[len_at] its length
 *   io[cand_at, + K_cap * M_max)        the lattice's candidate ids (cand_at a multiple of 4)
 * Before the first call the caller writes the pending tokens and the two context tokens there; afterwards the
 * acceptance kernel does.  host_out [host, pinned, device-visible] int32[2 K_cap + 1] is the path search's
 * host_mirror (path, length, raw draft of every round);
 * verdict [host, pinned, device-visible] int32[3] receives n_accept, next_token, eos_accepted.  drafter / verifier:
 * both caches committed to the same tokens but the *n_pend pending ones (drafter) / the last one (verifier).
 * ev_every > 0: rounds 0, ev_every, 2 ev_every, ... record the HIP events ev_start[j] / ev_end[j] (hipEvent_t handles,
 * j = round / ev_every) around the LM-head product alone, launched through the two-call form (same kernels).
 *
 * K: the first round's draft length (<= K_cap); follow_adl != 0: later rounds use the controller's proposal
 * (clipped to K_cap), else K stays.  stop_at_eos != 0: return after the round that accepted eos_id.
 * *n_pend in: the pending count of the first round; out: that of the next round (n_accept + 1 of the last one).
 * records [host] ds_round_record[n_rounds], *rounds_done, tokens_out [host] int32[tokens_cap] (the committed tokens
 * of all rounds in order, *n_tokens of them; DS_E_CAPACITY before a round that could overflow it).
 * A round that fails returns its error; the rounds before it stand (their outputs and counts are valid). */
typedef struct ds_round_desc {
  ds_model* drafter;
  ds_model* verifier;
  const ds_ngram* proxy; /* NULL: no proxy term */
  ds_adl* adl;
  int32_t K_cap, M_max, beam, eos_id, mask_id;
  float tau, lambda;
  float* hidden;       /* [dev] float[K_cap, drafter d_model] */
  float* cand_logp;    /* [dev] float[K_cap, M_max] */
  int32_t* cand_cnt;   /* [dev] int32[K_cap] */
  float* eos_logp;     /* [dev] float[K_cap] */
  float* lse;          /* [dev] float[K_cap] */
  int32_t* io;         /* [dev] see above */
  float* path_score;   /* [dev] float[1] */
  int32_t* argmax;     /* [dev] int32[K_cap + 1] */
  void* cps_ws;        /* [dev] ds_cps_workspace_bytes(1, K_cap, M_max), or NULL */
  size_t cps_ws_bytes;
  void* drafter_ws;    /* [dev] model workspaces */
  size_t drafter_ws_bytes;
  void* verifier_ws;
  size_t verifier_ws_bytes;
  int32_t* verdict;    /* [host, pinned] int32[3] */
  int32_t* host_out;   /* [host, pinned] int32[2 K_cap + 1] */
  int32_t ev_every;
  void* const* ev_start;
  void* const* ev_end;
} ds_round_desc;
typedef struct ds_round_record {
  int32_t k, path_len, n_accept, next_token, eos_accepted, first_eos, k_next;
} ds_round_record;
int ds_round_io_layout(int K_cap, int M_max, int* path_at, int* len_at, int* cand_at, int* total);
int ds_rounds_run(const ds_round_desc* d, int n_rounds, int K, int follow_adl, int stop_at_eos, int* n_pend,
                  ds_round_record* records, int* rounds_done, int32_t* tokens_out, int tokens_cap, int* n_tokens,
                  void* stream);

#ifdef __cplusplus
}
#endif
#endif /* DS_H */
