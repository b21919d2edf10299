"""Oracle stochastic block verification (Sec. 2, "Parallel verification": the standard acceptance rule
alpha = min(1, p / q) with residual resampling; Sec. 2, the left-to-right proxy q^L2R).  Test
infrastructure only.

Row r of the verifier's logits predicts the token after block[r] (block = [last committed token,
path_1 .. path_m]); row i-1 therefore scores draft token i.  The drafter probability of draft token i is
taken from the drafter's own row for block position i; with a single refinement pass every in-block
position is [MASK] in that pass, which is exactly the left-to-right proxy's input.

Draft token i is accepted iff u_i < alpha_i.  At the first rejection the replacement token is drawn from
the residual max(p - q, 0) (normalised); if every draft token is accepted a bonus token is drawn from the
verifier's next row.  Both draws use inverse-CDF sampling in vocabulary order with one uniform u_pick:
the smallest v whose cumulative weight exceeds u_pick * total.  The uniforms are inputs (the caller owns
the random stream).  Arithmetic: float64 softmax of the float32 logits, float64 cumulative sums.
"""
from __future__ import annotations

import numpy as np


def softmax64(row: np.ndarray) -> np.ndarray:
    r = np.asarray(row, dtype=np.float32).astype(np.float64)
    e = np.exp(r - r.max())
    return e / e.sum()


def inverse_cdf(weights: np.ndarray, u: float) -> int:
    """Smallest index whose cumulative weight exceeds u * total (u in [0, 1)); weights >= 0, total > 0."""
    total = float(np.sum(weights))
    target = u * total
    c = 0.0
    last_positive = -1
    for v, wv in enumerate(weights):
        if wv > 0.0:
            last_positive = v
        c += float(wv)
        if c > target and wv > 0.0:
            return v
    return last_positive  # rounding left the target at the very end of the mass


def acceptance_probability(p_row: np.ndarray, q_row: np.ndarray, token: int) -> float:
    p, q = softmax64(p_row)[token], softmax64(q_row)[token]
    return 1.0 if q <= p else p / q


def verify_stochastic(p_logits: np.ndarray, q_logits: np.ndarray, path: np.ndarray, u_accept: np.ndarray,
                      u_pick: float, eos_id: int):
    """p_logits [m + 1, V] verifier rows, q_logits [m, V] drafter rows of the path positions, path int [m].

    Returns (n_accept, next_token, eos_accepted, alpha float64 [m]); alpha beyond the first rejection is
    still reported (it is what the rule would have used) but plays no role.
    """
    path = np.asarray(path)
    m = path.shape[0]
    alpha = np.array([acceptance_probability(p_logits[i], q_logits[i], int(path[i])) for i in range(m)])
    n_accept = 0
    while n_accept < m and float(u_accept[n_accept]) < alpha[n_accept]:
        n_accept += 1
    p = softmax64(p_logits[n_accept])
    if n_accept < m:
        weights = np.maximum(p - softmax64(q_logits[n_accept]), 0.0)
        if not np.any(weights > 0.0):  # p == q up to rounding: the residual is empty, fall back to p
            weights = p
    else:
        weights = p
    next_token = inverse_cdf(weights, float(u_pick))
    eos = int(eos_id >= 0 and (next_token == eos_id or bool(np.any(path[:n_accept] == eos_id))))
    return n_accept, int(next_token), eos, alpha
