"""Oracle multi-step refinement of a draft block (Sec. 2, "Inference (iterative refinement)", the
refinement update equation; ablated as S > 1 in Sec. 4).  Test infrastructure only.

y^(0) = prefix o [MASK]^k with masked set M_0 = all k block positions.  Step s = 1..S: one drafter
pass on y^(s-1) gives the conditionals of the still-masked positions; an update subset U_s of M_{s-1}
is chosen by confidence and those positions are fixed to their arg-max token; M_s = M_{s-1} \\ U_s.

Readings (the paper leaves them open):
  * confidence of a position = probability of its arg-max token under the current pass, compared
    through the float32 log-probability the lattice reports (top-1 entry); ties go to the lower
    position;
  * |U_s| = ceil(|M_{s-1}| / (S - s + 1)): equal shares, so that M_S is empty after exactly
    min(S, k) passes (S = 1 fixes every position in the single pass, which is the default round);
  * the candidate lattice row of a position (top-M tokens, log-scores, pruned count, EOS score) is the
    one computed by the pass that fixes the position, i.e. the last pass in which it was still masked;
    no extra scoring pass is run after the block is complete.
"""
from __future__ import annotations

import numpy as np

from . import lattice as o_lattice
from . import model as o_model


def update_sizes(k: int, steps: int) -> list:
    """|U_1|, |U_2|, ... : equal shares of what is still masked, until nothing is."""
    sizes, left = [], k
    for s in range(1, steps + 1):
        if left == 0:
            break
        n = -(-left // (steps - s + 1))  # ceil
        sizes.append(n)
        left -= n
    return sizes


def select_update(conf: np.ndarray, masked: np.ndarray, n: int) -> np.ndarray:
    """Positions of the n most confident still-masked entries (ties: lower position), ascending."""
    pos = np.nonzero(masked)[0]
    order = sorted(pos, key=lambda i: (-np.float32(conf[i]), i))
    return np.sort(np.asarray(order[:n], dtype=np.int64))


def refine_block(cfg, w, cache: o_model.KVCache, pending, k: int, steps: int, m_max: int, tau: float,
                 eos_id: int):
    """Run the refinement and return (lattice dict, y^(S) int32 [k], fixed_at int32 [k]).

    fixed_at[i] = 1-based pass that fixed position i.  The pending tokens are committed by the first pass.
    """
    block = np.full(k, cfg.mask_id, dtype=np.int64)
    masked = np.ones(k, dtype=bool)
    fixed_at = np.zeros(k, dtype=np.int32)
    final = {"cand_id": np.zeros((k, m_max), np.int32), "cand_logp": np.zeros((k, m_max), np.float32),
             "cand_cnt": np.zeros(k, np.int32), "eos_logp": np.zeros(k, np.float32), "lse": np.zeros(k, np.float32)}
    for s, n in enumerate(update_sizes(k, steps), start=1):
        y = o_model.draft_block(cfg, w, cache, pending if s == 1 else [], k, block_tokens=block)
        lat = o_lattice.build_lattice(o_model.lm_head(w, y), m_max, tau, eos_id)
        upd = select_update(lat["cand_logp"][:, 0], masked, n)
        for i in upd:
            block[i] = lat["cand_id"][i, 0]
            for key in final:
                final[key][i] = lat[key][i]
            masked[i] = False
            fixed_at[i] = s
    assert not masked.any()
    return final, block.astype(np.int32), fixed_at
