"""Pins for greedy acceptance and the draft-length controller (no GPU)."""
import itertools
import os

import numpy as np

from oracle import accept, adl

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "adl_traces.txt")


def test_both_forms_of_accepted_length_agree_on_every_pattern():
    for k in range(0, 9):
        for bits in itertools.product([0, 1], repeat=k):
            a = np.array(bits, dtype=np.int64)
            m = accept.accepted_length_max_form(a)
            assert m == accept.accepted_length_sum_form(a)
            assert all(a[:m] == 1) and (m == k or a[m] == 0)


def _one_hot_logits(tokens, vocab):
    lg = np.zeros((len(tokens), vocab), dtype=np.float32)
    lg[np.arange(len(tokens)), tokens] = 5.0
    return lg


def test_verify_greedy_prefix_cases():
    vocab, eos = 50, 48
    greedy = [7, 9, 11, 13, 15]          # verifier's own continuation after block[0]
    lg = _one_hot_logits(greedy, vocab)  # rows 0..4
    n, nxt, am, e = accept.verify_greedy(lg, np.array([7, 9, 11, 13]), eos)
    assert (n, nxt, e) == (4, 15, 0) and list(am) == greedy          # full acceptance + bonus
    n, nxt, _, _ = accept.verify_greedy(lg, np.array([8, 9, 11, 13]), eos)
    assert (n, nxt) == (0, 7)                                        # first token wrong -> correction
    n, nxt, _, _ = accept.verify_greedy(lg, np.array([7, 9, 12, 13]), eos)
    assert (n, nxt) == (2, 11)                                       # later matches do not count
    n, nxt, _, _ = accept.verify_greedy(lg[:1], np.array([], dtype=np.int64), eos)
    assert (n, nxt) == (0, 7)                                        # empty path


def test_verify_greedy_ties_and_eos():
    vocab, eos = 50, 48
    lg = np.zeros((2, vocab), dtype=np.float32)
    lg[0, [5, 3]] = 1.0                                               # tie -> lower id 3
    lg[1, eos] = 1.0
    n, nxt, am, e = accept.verify_greedy(lg, np.array([3]), eos)
    assert (n, nxt, e) == (1, eos, 1) and list(am) == [3, eos]
    n, nxt, am, e = accept.verify_greedy(lg, np.array([5]), eos)
    assert (n, nxt, e) == (0, 3, 0)
    lg = _one_hot_logits([eos, 4], vocab)
    n, nxt, _, e = accept.verify_greedy(lg, np.array([eos]), eos)     # accepted EOS inside the path
    assert (n, e) == (1, 1)
    n, nxt, _, e = accept.verify_greedy(lg, np.array([eos]), -1)      # EOS handling off
    assert (n, e) == (1, 0)


def _read_traces():
    out = []
    for line in open(GOLDEN):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        head, steps, ks = [p.strip() for p in line.split("|")]
        k_min, k_max, delta, rho, k1 = head.split()
        steps = [tuple(int(x) for x in s.split(":")) for s in steps.split()]
        out.append((int(k_min), int(k_max), float(delta), float(rho), int(k1), steps, [int(k) for k in ks.split()]))
    return out


def test_adl_hand_traces():
    traces = _read_traces()
    assert len(traces) >= 8
    for k_min, k_max, delta, rho, k1, steps, expect in traces:
        st = adl.AdlState(k_min, k_max, delta, rho)
        k = k1
        got = []
        for first_eos, l_acc in steps:
            k = adl.adl_update(st, k, first_eos, l_acc)
            got.append(k)
        assert got == expect, (k_min, k_max, delta, rho, k1, steps, got, expect)


def test_adl_fixed_points_and_bounds():
    st = adl.AdlState(4, 64, 10, 0.5)
    k = 16
    for _ in range(40):                 # full acceptance climbs to k_max and stays
        k = adl.adl_update(st, k, 0, k)
        assert 4 <= k <= 64
    assert k == 64
    for _ in range(40):                 # then nothing accepted: falls to the fixed point 8... of L_gen=k
        k = adl.adl_update(st, k, 0, 0)
    assert k == adl.adl_update(st, k, 0, 0)


def test_first_eos_index():
    assert adl.first_eos_index([3, 4, 9, 9], 9) == 3
    assert adl.first_eos_index([3, 4], 9) == 0
    assert adl.first_eos_index([9], -1) == 0
