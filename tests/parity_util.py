"""Localised near-tie rules for end-to-end comparisons (no GPU code here).

End to end the GPU path and the oracle compute their own logits, which agree to the stated tolerance only.  An
integer decision may therefore differ where, and only where, the ORACLE's own margin for THAT decision is below
twice the tolerance:
(in whole rounds: twice the difference MEASURED between the two sides' logits in that round, which is far below the
bar the logits themselves are held to):
  * a lattice row: the gap between the oracle's values at the first differing rank and the next rank;
  * a verifier row: the gap between the oracle's largest and second largest logit of that row;
  * the path search: the smallest gap, at some depth, between neighbouring scores among the kept hypotheses and
    the best dropped one (the oracle's diagnostic margins), against the tolerance accumulated over that depth.
Every helper asserts the near-tie for the deviating item and returns what it flagged, so that a test can bound
and report the number of excused decisions.
"""
from __future__ import annotations

import numpy as np

from oracle import cps as o_cps
from oracle import round as o_round
from paper_2510_02358_amd import synth


def lattice_rows_flagged(gpu_ids: np.ndarray, ref_ids: np.ndarray, ref_logits: np.ndarray, tol: float) -> list:
    """Rows whose candidate ids differ; each must sit on a near-tie of the oracle's logits at the first differing
    rank (the token the GPU ranks there is within the tolerance of the oracle's, so the oracle's next value is)."""
    m_max = ref_ids.shape[1]
    flagged = []
    for r in np.nonzero(np.any(gpu_ids != ref_ids, axis=1))[0]:
        j = int(np.nonzero(gpu_ids[r] != ref_ids[r])[0][0])
        row = ref_logits[r].astype(np.float64)
        top = -np.sort(-np.partition(row, row.size - (m_max + 1))[-(m_max + 1):])  # m_max + 1 largest, descending
        gap = top[j] - top[j + 1]
        assert gap < 2 * tol, f"lattice row {r}: ids differ at rank {j} with a clear gap {gap:.3e}"
        # and the token the GPU put there is one of the two near-tied ones, not something else
        assert abs(row[gpu_ids[r, j]] - top[j]) < 2 * tol, f"lattice row {r}: rank {j} holds a token {2 * tol} away"
        flagged.append(int(r))
    return flagged


def argmax_rows_flagged(gpu_am: np.ndarray, ref_logits: np.ndarray, tol: float) -> list:
    """Verifier rows whose arg-max differs from the oracle's; each must have an oracle top-2 gap below 2 tol."""
    ref_am = np.argmax(ref_logits, axis=-1)
    flagged = []
    for r in np.nonzero(np.asarray(gpu_am) != ref_am)[0]:
        top2 = np.partition(ref_logits[r].astype(np.float64), -2)[-2:]
        gap = abs(top2[1] - top2[0])
        assert gap < 2 * tol, f"verifier row {r}: arg-max {gpu_am[r]} vs {ref_am[r]} with a clear gap {gap:.3e}"
        assert abs(ref_logits[r, gpu_am[r]] - top2.max()) < 2 * tol
        flagged.append(int(r))
    return flagged


def search_is_near_tied(ref_lat: dict, k: int, beam: int, lam: float, table, log2_size: int, ctx, eos_id: int,
                        tol: float) -> bool:
    """True iff the oracle's own search over its own lattice passes, at some depth i, a beam boundary whose score
    gap is below 4 tol (i + 1): a log-score is logit - lse, each of which differs by up to tol between the two
    sides, a score is a sum of i + 1 log-scores (weighted by lambda <= 1), and a gap compares two scores."""
    margins = []
    o_cps.cps_path(ref_lat, 0, k, beam, lam, table, log2_size, ctx, eos_id, margins=margins)
    return any(m < 4 * tol * (i + 1) for i, m in enumerate(margins))


def _snapshot(st):
    return (st.dcache.copy(), st.vcache.copy(), list(st.tokens), list(st.pending))


def _restore(st, snap):
    st.dcache, st.vcache, st.tokens, st.pending = snap[0].copy(), snap[1].copy(), list(snap[2]), list(snap[3])


def new_counts() -> dict:
    return {n: 0 for n in ("rounds", "lattice_rows", "lattice_rows_flagged", "paths", "paths_flagged",
                           "verifier_rows", "verifier_rows_flagged")}


def compare_round(dec, st, got, k, params, table, tol, counts, uniforms=None):
    """One GPU round (already run: `got`) against the oracle's round from the same state `st`, decision by
    decision.  A decision may differ only where the oracle's own margin for it is below twice the tolerance
    (tests/parity_util.py asserts that for the deviating item); what was excused is counted in `counts`.  When the
    searched paths differ, the oracle's round is repeated with the GPU's path forced so that verification can
    still be compared.  Returns the oracle's record, or None if the verdicts differ (then the two token streams
    part and the caller stops comparing).  With `uniforms` (stochastic verification) the verdict is left to the
    caller: the oracle's record is returned with the GPU's path verified."""
    m_max, tau, beam, lam = params.m_max, params.tau, params.beam, params.lam
    eos_id, ctx = st.dcfg.eos_id, list(st.tokens[-2:])
    snap = _snapshot(st)
    ref = o_round.spec_round(st, k, m_max, tau, beam, lam, table, synth.NGRAM_LOG2_SIZE, uniforms=uniforms)
    d_logits = dec.d_logits[:k].cpu().numpy()
    noise_d = float(np.max(np.abs(d_logits - ref["d_logits"])))
    assert noise_d <= tol
    counts["max_logit_err"] = max(counts.get("max_logit_err", 0.0), noise_d)
    # decisions are excused at the MEASURED difference of the two sides' logits in this round, not at the bar
    noise_d = max(noise_d, 1e-7)
    g_lat = {"cand_id": dec.cand_id[:k].cpu().numpy(), "cand_logp": dec.cand_logp[:k].cpu().numpy(),
             "cand_cnt": dec.cand_cnt[:k].cpu().numpy(), "eos_logp": dec.eos_logp[:k].cpu().numpy()}
    rows_f = lattice_rows_flagged(g_lat["cand_id"], ref["lattice"]["cand_id"], ref["d_logits"], noise_d)
    for r in np.nonzero(g_lat["cand_cnt"] != ref["lattice"]["cand_cnt"])[0]:
        if int(r) in rows_f:
            continue
        cum = np.cumsum(np.exp(ref["lattice"]["cand_logp"][r].astype(np.float64)))
        assert np.min(np.abs(cum - tau)) < 4 * noise_d, f"row {r}: pruned counts differ away from the threshold"
        rows_f.append(int(r))
    counts["lattice_rows"] += k
    counts["lattice_rows_flagged"] += len(rows_f)
    # the search itself is exact: on the GPU's own lattice the oracle search returns the GPU's path, bit for bit
    own, own_score, _ = o_cps.cps_path(g_lat, 0, k, beam, lam, table, synth.NGRAM_LOG2_SIZE, ctx, eos_id)
    assert list(got["path"]) == own
    assert np.float32(dec.path_score.cpu().numpy()[0]).view(np.uint32) == np.float32(own_score).view(np.uint32)
    counts["paths"] += 1
    if list(got["path"]) != ref["path"]:
        assert rows_f or search_is_near_tied(ref["lattice"], k, beam, lam, table, synth.NGRAM_LOG2_SIZE, ctx,
                                                eos_id, noise_d), "paths differ without a near-tie"
        counts["paths_flagged"] += 1
        _restore(st, snap)   # verify the GPU's path on the oracle too
        ref = o_round.spec_round(st, k, m_max, tau, beam, lam, table, synth.NGRAM_LOG2_SIZE,
                                 forced_path=list(got["path"]), uniforms=uniforms)
    if not rows_f:
        assert got["first_eos"] == ref["first_eos"]
    m = len(ref["path"])
    v_logits = dec.v_logits[:m + 1].cpu().numpy()
    noise_v = float(np.max(np.abs(v_logits - ref["v_logits"])))
    assert noise_v <= tol
    counts["max_logit_err"] = max(counts["max_logit_err"], noise_v)
    noise_v = max(noise_v, 1e-7)
    if uniforms is not None:   # the stochastic rule takes no arg-max
        return ref
    am_f = argmax_rows_flagged(dec.argmax[:m + 1].cpu().numpy(), ref["v_logits"], noise_v)
    counts["verifier_rows"] += m + 1
    counts["verifier_rows_flagged"] += len(am_f)
    same = (got["n_accept"], got["next_token"], got["eos_accepted"]) == (ref["n_accept"], ref["next_token"],
                                                                         ref["eos_accepted"])
    assert same or am_f, "verdicts differ although every verifier row agrees on its arg-max"
    return ref if same else None
