"""Oracle greedy block verification (Sec. 2, "Parallel verification" and "Accepted prefix
length", with greedy / temperature-0 verification as in Sec. 4).  Test infrastructure only.

Row r of the verifier's logits predicts the token that follows block[r], where
block = [last committed token, path_1 .. path_m].  Draft token i (1-based) is accepted iff
it equals the verifier's arg-max at row i-1 (ties: lower id).  The accepted length is the
longest all-accepted prefix; the round then also commits next = argmax[L_acc] (the correction
after a rejection, or a bonus token after full acceptance).
"""
from __future__ import annotations

import numpy as np


def greedy_argmax(logits: np.ndarray) -> np.ndarray:
    return np.argmax(np.asarray(logits, dtype=np.float32), axis=-1).astype(np.int32)


def accepted_length_max_form(a: np.ndarray) -> int:
    """max{ m : A_1 = ... = A_m = 1 }."""
    m = 0
    while m < len(a) and a[m] == 1:
        m += 1
    return m


def accepted_length_sum_form(a: np.ndarray) -> int:
    """sum_i prod_{r<=i} A_r."""
    return int(sum(int(np.prod(a[:i + 1])) for i in range(len(a))))


def verify_greedy(logits: np.ndarray, path: np.ndarray, eos_id: int):
    """logits [m+1, vocab]; path [m].  Returns (n_accept, next_token, argmax[m+1], eos_accepted)."""
    am = greedy_argmax(logits)
    m = len(path)
    a = np.array([1 if am[i] == path[i] else 0 for i in range(m)], dtype=np.int64)
    n_acc = accepted_length_max_form(a)
    nxt = int(am[n_acc])
    eos = 0
    if eos_id >= 0 and (nxt == eos_id or any(int(t) == eos_id for t in path[:n_acc])):
        eos = 1
    return n_acc, nxt, am, eos
