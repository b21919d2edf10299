// Host side of the speculative loop (Alg. 1, all four stages, round after round) as one C-ABI call.
//
// This file is a client of the library's own entry points: it holds no kernel and no arithmetic of the method.
// Per round it enqueues draft -> LM head / lattice -> path search (whose kernel also leaves the path, its length and
// the raw draft in pinned host memory) -> verification with the carry output, then waits for the verdict (a poll of the word
// the acceptance kernel stores last in device-visible pinned memory; bounded, with a stream synchronisation as the
// fallback), commits the verifier's cache length, takes the first-EOS index of the raw draft from the host copy,
// updates the draft-length controller and appends the committed tokens to the caller's host array.  Nothing is
// sent to the device between rounds: the acceptance kernel leaves the committed tokens where the next round reads
// them (ds_verify_block_carry).
#include <chrono>

#include "ds_common.h"

namespace {

constexpr int32_t kPending = -0x7EADBEEF;  // what the host leaves in the verdict's last word (eos_accepted is 0 or 1)

int wait_verdict(volatile int32_t* word, hipStream_t st) {
  uint64_t spins = 0;
  std::chrono::steady_clock::time_point t0;
  bool timing = false;
  while (*word == kPending) {
    if ((++spins & 0xFFFF) == 0) {
      const auto now = std::chrono::steady_clock::now();
      if (!timing) {
        t0 = now;
        timing = true;
      } else if (std::chrono::duration<double>(now - t0).count() > 10.0) {
        // surfaces a device error if there is one; a healthy stream has delivered the verdict by now
        if (hipStreamSynchronize(st) != hipSuccess) return ds::fail(DS_E_HIP, "the round's stream failed");
        if (*word == kPending) return ds::fail(DS_E_HIP, "no verdict from the acceptance kernel within 10 s");
      }
    }
  }
  return DS_OK;
}

}  // namespace

extern "C" {

int ds_round_io_layout(int K_cap, int M_max, int* path_at, int* len_at, int* cand_at, int* total) {
  DS_REQUIRE(K_cap >= 1 && K_cap < DS_MAX_ROWS && M_max >= 1 && M_max <= DS_MAX_TOPM, DS_E_SHAPE,
             "K_cap %d / M_max %d outside [1, %d) / [1, %d]", K_cap, M_max, DS_MAX_ROWS, DS_MAX_TOPM);
  const int p = DS_MAX_ROWS + 2, l = p + K_cap, c = (l + 1 + 3) / 4 * 4;
  if (path_at) *path_at = p;
  if (len_at) *len_at = l;
  if (cand_at) *cand_at = c;
  if (total) *total = c + K_cap * M_max;
  return DS_OK;
}

int ds_rounds_run(const ds_round_desc* d, int n_rounds, int K, int follow_adl, int stop_at_eos, int* n_pend,
                  ds_round_record* records, int* rounds_done, int32_t* tokens_out, int tokens_cap, int* n_tokens,
                  void* stream) {
  DS_REQUIRE(d && n_pend && records && rounds_done && tokens_out && n_tokens, DS_E_INVALID,
             "ds_rounds_run: NULL pointer argument");
  DS_REQUIRE(d->drafter && d->verifier && d->adl && d->hidden && d->cand_logp && d->cand_cnt && d->eos_logp &&
                 d->lse && d->io && d->path_score && d->argmax && d->verdict && d->host_out && d->drafter_ws &&
                 d->verifier_ws,
             DS_E_INVALID, "ds_rounds_run: NULL pointer in the descriptor");
  int path_at = 0, len_at = 0, cand_at = 0, total = 0;
  int rc = ds_round_io_layout(d->K_cap, d->M_max, &path_at, &len_at, &cand_at, &total);
  if (rc) return rc;
  DS_REQUIRE(n_rounds >= 0 && K >= 1 && K <= d->K_cap, DS_E_SHAPE, "K %d outside [1, K_cap = %d]", K, d->K_cap);
  DS_REQUIRE(*n_pend >= 1 && *n_pend + K <= DS_MAX_ROWS, DS_E_SHAPE, "n_pend %d: need 1 <= n_pend, n_pend + K <= %d",
             *n_pend, DS_MAX_ROWS);
  DS_REQUIRE(d->ev_every >= 0 && (d->ev_every == 0 || (d->ev_start && d->ev_end)), DS_E_INVALID,
             "ev_every without event arrays");
  hipStream_t st = static_cast<hipStream_t>(stream);
  const int P = DS_MAX_ROWS;
  int32_t* io = d->io;
  int32_t* cand_id = io + cand_at;
  volatile int32_t* verdict = d->verdict;
  int pend = *n_pend, used = 0;
  *n_tokens = 0;
  *rounds_done = 0;
  for (int t = 0; t < n_rounds; ++t) {
    DS_REQUIRE(pend + K <= DS_MAX_ROWS, DS_E_SHAPE, "round %d: %d pending + %d draft rows exceed %d", t, pend, K,
               DS_MAX_ROWS);
    DS_REQUIRE(used + K + 1 <= tokens_cap, DS_E_CAPACITY, "round %d: tokens_out holds %d tokens, %d + %d may be needed",
               t, tokens_cap, used, K + 1);
    int v_len = 0;
    if ((rc = ds_model_kv_len(d->verifier, &v_len))) return rc;
    verdict[2] = kPending;
    if ((rc = ds_draft_block(d->drafter, io + P - pend, pend, K, d->mask_id, d->hidden, d->drafter_ws,
                             d->drafter_ws_bytes, st)))
      return rc;
    const bool timed = d->ev_every > 0 && (t % d->ev_every) == 0;
    if (timed) {
      const int e = t / d->ev_every;
      DS_HIP_CHECK(hipEventRecord(static_cast<hipEvent_t>(d->ev_start[e]), st));
      if ((rc = ds_lm_head_tiles(d->drafter, nullptr, K, d->eos_id, nullptr, d->drafter_ws, d->drafter_ws_bytes, st)))
        return rc;
      DS_HIP_CHECK(hipEventRecord(static_cast<hipEvent_t>(d->ev_end[e]), st));
      if ((rc = ds_lattice_from_tiles(d->drafter, K, d->M_max, d->tau, d->eos_id, cand_id, d->cand_logp, d->cand_cnt,
                                      d->eos_logp, d->lse, d->drafter_ws, d->drafter_ws_bytes, st)))
        return rc;
    } else if ((rc = ds_draft_lattice(d->drafter, nullptr, K, d->M_max, d->tau, d->eos_id, cand_id, d->cand_logp,
                                      d->cand_cnt, d->eos_logp, d->lse, nullptr, d->drafter_ws, d->drafter_ws_bytes,
                                      st))) {
      return rc;
    }
    if ((rc = ds_cps_path(cand_id, d->cand_logp, d->cand_cnt, d->eos_logp, 1, K, d->M_max, d->beam, d->lambda,
                          d->proxy, io + P, d->eos_id, io + path_at, io + len_at, d->path_score, d->host_out,
                          d->cps_ws, d->cps_ws_bytes, st)))
      return rc;
    if ((rc = ds_verify_block_carry(d->verifier, io + P + 1, K, io + len_at, d->eos_id, d->verdict, d->verdict + 1,
                                    d->argmax, d->verdict + 2, nullptr, io, d->verifier_ws, d->verifier_ws_bytes,
                                    st)))
      return rc;
    if ((rc = wait_verdict(verdict + 2, st))) return rc;
    const int n_acc = verdict[0], nxt = verdict[1], eos = verdict[2];
    const int plen = d->host_out[K];  // the search's mirror: path [K], length, raw draft [K]
    DS_REQUIRE(n_acc >= 0 && n_acc <= K && plen >= 0 && plen <= K && n_acc <= plen, DS_E_HIP,
               "round %d: verdict out of range (n_accept %d, path_len %d)", t, n_acc, plen);
    if ((rc = ds_model_kv_set_len(d->verifier, v_len + 1 + n_acc))) return rc;
    int first_eos = 0, k_next = K;
    if ((rc = ds_adl_first_eos(d->host_out + K + 1, K, 1, d->eos_id, &first_eos))) return rc;
    if ((rc = ds_adl_update(d->adl, K, first_eos, n_acc, &k_next))) return rc;
    for (int i = 0; i < n_acc; ++i) tokens_out[used + i] = d->host_out[i];
    tokens_out[used + n_acc] = nxt;
    used += n_acc + 1;
    records[t] = ds_round_record{K, plen, n_acc, nxt, eos, first_eos, k_next};
    pend = n_acc + 1;
    *n_tokens = used;
    *n_pend = pend;
    *rounds_done = t + 1;
    if (follow_adl) K = k_next < d->K_cap ? k_next : d->K_cap;
    if (eos && stop_at_eos) break;
  }
  return DS_OK;
}

}  // extern "C"
