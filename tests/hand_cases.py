"""Worked examples whose expected values were computed by hand (no oracle, no GPU): shared by the CPU pins of the
oracle and by the GPU tests, so that both sides meet the same hand-made numbers."""
import numpy as np


def narrow_beam_case(log2_size: int, slot_fn):
    """Path search, three positions, two candidates each, lambda = 1/2, context (1, 2); every number is a dyadic
    fraction, so the float32 sums are exact.  Proxy log-scores (all other 3-grams 0):
        (2,10,20) -2   (2,10,21) -4   (2,11,21) -6   (10,20,30) = (10,20,31) = (11,20,30) = (11,20,31) = -10
    Depth 0: [10] -0.5, [11] -1.0.
    Depth 1: [10,20] -0.5 + (-0.5 - 1) = -2.0   [10,21] -0.5 + (-0.5 - 2) = -3.0
             [11,20] -1.0 + (-0.5 + 0) = -1.5   [11,21] -1.0 + (-0.5 - 3) = -4.5
    Depth 2 adds (-0.5 + l_ng / 2) for token 30 and (-1.5 + l_ng / 2) for token 31.
      beam 4 (nothing pruned): best is [10,21,30] = -3.0 - 0.5 = -3.5
      beam 2: depth 1 keeps [11,20], [10,20] and drops [10,21], the prefix of the optimum;
              then [11,20,30] = -1.5 - 5.5 = -7.0 beats [10,20,30] = -7.5, [11,20,31] = -8.0, [10,20,31] = -8.5
      beam 1: [10] -> [10,20] -> [10,20,30] = -2.0 - 5.5 = -7.5
    slot_fn(u, v, w, log2_size): the table's slot function (the table is addressed through it, nothing else).
    Returns (lattice dict, table float32[2^log2_size], ctx, [(beam, path, score), ...])."""
    lat = {"cand_id": np.array([[10, 11], [20, 21], [30, 31]], np.int32),
           "cand_logp": np.array([[-1.0, -2.0], [-1.0, -1.0], [-1.0, -3.0]], np.float32),
           "cand_cnt": np.array([2, 2, 2], np.int32), "eos_logp": np.zeros(3, np.float32)}
    table = np.zeros(1 << log2_size, np.float32)
    entries = {(2, 10, 20): -2.0, (2, 10, 21): -4.0, (2, 11, 21): -6.0, (10, 20, 30): -10.0, (10, 20, 31): -10.0,
               (11, 20, 30): -10.0, (11, 20, 31): -10.0}
    every = [(1, 2, 10), (1, 2, 11), (2, 11, 20), (10, 21, 30), (10, 21, 31), (11, 21, 30), (11, 21, 31)] + list(entries)
    assert len({slot_fn(*t, log2_size) for t in every}) == len(every)          # no two of them share a slot
    for t, v in entries.items():
        table[slot_fn(*t, log2_size)] = v
    expected = [(4, [10, 21, 30], -3.5), (2, [11, 20, 30], -7.0), (1, [10, 20, 30], -7.5)]
    return lat, table, (1, 2), expected
