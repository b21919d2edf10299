"""Oracle token lattice (Sec. 3.2, "Lattice and pruning").  Test infrastructure only.

For every draft position the lattice keeps the top-M_max tokens of the drafter's
distribution with their log-probabilities l_dlm(v) = log q(v | ...), and the number of
candidates M_i that survive mass-adaptive pruning: the smallest m <= M_max whose
cumulative probability reaches tau (the pruning equation; if no m qualifies, M_i = M_max;
tau >= 1 switches pruning off).  The EOS log-probability is reported separately because
EOS is always retained by the search.

Order of candidates: logit descending, ties by lower token id.
Arithmetic: lse accumulated in float64 and rounded once to float32; log-prob =
float32(logit) - float32(lse); pruning mass accumulated in float32 in candidate order.
"""
from __future__ import annotations

import numpy as np


def log_sum_exp(row: np.ndarray) -> np.float32:
    r = row.astype(np.float64)
    mx = r.max()
    return np.float32(mx + np.log(np.sum(np.exp(r - mx))))


def top_m(row: np.ndarray, m_max: int) -> np.ndarray:
    """Token ids of the m_max largest logits; logit descending, then id ascending."""
    ids = np.arange(row.shape[0])
    order = np.lexsort((ids, -row.astype(np.float64)))  # last key is primary
    return order[:m_max].astype(np.int32)


def pruned_count(cand_logp: np.ndarray, tau: float) -> int:
    m_max = cand_logp.shape[0]
    if tau >= 1.0:
        return m_max
    cum = np.float32(0.0)
    for m in range(m_max):
        cum = np.float32(cum + np.exp(cand_logp[m], dtype=np.float32))
        if cum >= np.float32(tau):
            return m + 1
    return m_max


def build_lattice(logits: np.ndarray, m_max: int, tau: float, eos_id: int):
    """logits [rows, vocab] float32 -> dict of per-row lattice arrays.

    cand_id  int32 [rows, m_max], cand_logp float32 [rows, m_max], cand_cnt int32 [rows],
    eos_logp float32 [rows] (0 when eos_id < 0), lse float32 [rows].
    """
    logits = np.asarray(logits, dtype=np.float32)
    rows = logits.shape[0]
    cand_id = np.zeros((rows, m_max), dtype=np.int32)
    cand_logp = np.zeros((rows, m_max), dtype=np.float32)
    cand_cnt = np.zeros(rows, dtype=np.int32)
    eos_logp = np.zeros(rows, dtype=np.float32)
    lse = np.zeros(rows, dtype=np.float32)
    for r in range(rows):
        row = logits[r]
        lse[r] = log_sum_exp(row)
        cand_id[r] = top_m(row, m_max)
        cand_logp[r] = row[cand_id[r]] - lse[r]  # float32 - float32
        cand_cnt[r] = pruned_count(cand_logp[r], tau)
        if eos_id >= 0:
            eos_logp[r] = row[eos_id] - lse[r]
    return {"cand_id": cand_id, "cand_logp": cand_logp, "cand_cnt": cand_cnt,
            "eos_logp": eos_logp, "lse": lse}


def raw_draft(lat: dict) -> np.ndarray:
    """The drafter's own block: per-position arg-max (refinement update with S = 1)."""
    return lat["cand_id"][:, 0].copy()
