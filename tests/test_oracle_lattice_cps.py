"""Pins for the oracle lattice and path search (no GPU).

Lattice: probability mass sums to one, top-M equals the head of a full stable sort, hand-made
rows for the mass-pruning rule, EOS retention.  Path search: exhaustive enumeration of every
lattice path (tiny K, M), a 3-gram Viterbi DP, the separable case lambda = 1, greedy case
B = 1, and the candidate-evaluation count of the complexity statement.
"""
import itertools

import numpy as np
import pytest

from oracle import cps, lattice, model
from paper_2510_02358_amd import synth

import hand_cases

f32 = np.float32
LOG2 = 12


def _table(seed=3):
    return synth.make_ngram_table(seed, LOG2)


def _random_lattice(rng, k, m_max, vocab, eos_id, cnt=None):
    logits = (rng.standard_normal((k, vocab)) * 2.0).astype(np.float32)
    lat = lattice.build_lattice(logits, m_max, 1.0, eos_id)
    if cnt is not None:
        lat["cand_cnt"][:] = cnt
    return lat, logits


# ------------------------------------------------------------------ lattice

def test_softmax_mass_is_one_and_topm_is_sorted_head():
    rng = np.random.default_rng(0)
    logits = (rng.standard_normal((5, 3000)) * 3).astype(np.float32)
    logits[2, 100] = logits[2, 7] = logits[2].max() + 1.0  # exact tie at the top: lower id first
    logits[3, :] = 0.25                                     # flat row: ids 0..M-1
    lat = lattice.build_lattice(logits, 6, 1.0, eos_id=2998)
    for r in range(5):
        mass = np.sum(np.exp(logits[r].astype(np.float64) - np.float64(lat["lse"][r])))
        assert abs(mass - 1.0) < 1e-6
        full = sorted(range(3000), key=lambda v: (-float(logits[r, v]), v))
        assert list(lat["cand_id"][r]) == full[:6]
        assert np.array_equal(lat["cand_logp"][r], logits[r, lat["cand_id"][r]] - lat["lse"][r])
        assert np.all(np.diff(lat["cand_logp"][r]) <= 0)
        assert lat["eos_logp"][r] == logits[r, 2998] - lat["lse"][r]
    assert list(lat["cand_id"][2][:2]) == [7, 100]
    assert list(lat["cand_id"][3]) == [0, 1, 2, 3, 4, 5]
    assert np.isclose(lat["lse"][3], 0.25 + np.log(3000.0), atol=1e-6)
    assert np.all(lat["cand_cnt"] == 6)  # tau >= 1: pruning off


def _row_from_probs(probs, vocab=64):
    """A logit row whose softmax has the given leading probabilities (rest spread evenly)."""
    p = np.full(vocab, (1.0 - sum(probs)) / (vocab - len(probs)))
    p[: len(probs)] = probs
    return np.log(p).astype(np.float32)


def test_mass_pruning_hand_rows():
    # 0.50 + 0.35 = 0.85 >= 0.8 -> two candidates survive
    lat = lattice.build_lattice(_row_from_probs([0.50, 0.35, 0.10])[None], 5, 0.8, -1)
    assert lat["cand_cnt"][0] == 2
    # peaky row: one candidate
    lat = lattice.build_lattice(_row_from_probs([0.93, 0.02])[None], 5, 0.8, -1)
    assert lat["cand_cnt"][0] == 1
    # 0.3,0.3,0.15,0.1 : cumulative 0.3, 0.6, 0.75, 0.85 -> four
    lat = lattice.build_lattice(_row_from_probs([0.3, 0.3, 0.15, 0.1])[None], 5, 0.8, -1)
    assert lat["cand_cnt"][0] == 4
    # flat row never reaches tau within M_max -> capped at M_max
    lat = lattice.build_lattice(np.zeros((1, 64), dtype=np.float32), 5, 0.8, -1)
    assert lat["cand_cnt"][0] == 5
    # threshold is reached with equality counted as reached (">=")
    assert lattice.pruned_count(np.log(np.array([0.5, 0.25, 0.25], dtype=np.float32)), 0.75) == 2
    # tau = 1 disables
    lat = lattice.build_lattice(_row_from_probs([0.93, 0.02])[None], 5, 1.0, -1)
    assert lat["cand_cnt"][0] == 5


def test_eos_is_retained_when_pruned_or_outside_topm():
    row = _row_from_probs([0.6, 0.3, 0.05])
    eos = 40
    lat = lattice.build_lattice(row[None], 3, 0.8, eos)
    cands = cps.position_candidates(lat, 0, eos)
    assert [t for t, _ in cands] == [0, 1, eos] and cands[-1][1] == lat["eos_logp"][0]
    # EOS inside the surviving set: not duplicated
    lat = lattice.build_lattice(row[None], 3, 0.8, 1)
    assert [t for t, _ in cps.position_candidates(lat, 0, 1)] == [0, 1]
    # EOS in the top-M but pruned away: appended again as the last candidate, same log-prob
    lat = lattice.build_lattice(row[None], 3, 0.8, 2)
    cands = cps.position_candidates(lat, 0, 2)
    assert [t for t, _ in cands] == [0, 1, 2] and cands[2][1] == lat["cand_logp"][0, 2]
    # EOS handling off
    assert [t for t, _ in cps.position_candidates(lat, 0, -1)] == [0, 1]


# ------------------------------------------------------------------ path search

def _path_score(lat, toks, ranks, lam, table, ctx):
    """Left-to-right float32 score of one path given candidate ranks per depth."""
    score = f32(0.0)
    u, v = int(ctx[0]), int(ctx[1])
    for i, w in enumerate(toks):
        l_dlm = ranks[i][1]
        l_ng = f32(table[cps.ngram_slot(u, v, w, LOG2)]) if table is not None else f32(0.0)
        one_minus = f32(f32(1.0) - f32(lam))
        score = f32(score + f32(f32(f32(lam) * l_dlm) + f32(one_minus * l_ng)))
        u, v = v, w
    return score


def _enumerate_best(lat, k, lam, table, ctx, eos_id):
    """Exhaustive search under the same termination rule, written independently of the beam code:
    depth by depth, all live (EOS-free) prefixes are extended by every candidate; if the best of all
    extensions ends in EOS it wins; otherwise EOS-ended ones are discarded."""
    live = [((), ())]  # (tokens, ((tok, l_dlm), ...))
    best = None
    for i in range(k):
        cands = cps.position_candidates(lat, i, eos_id)
        ext = []
        for toks, picks in live:
            for c, (w, l) in enumerate(cands):
                t2, p2 = toks + (w,), picks + ((w, l),)
                ext.append((_path_score(lat, t2, p2, lam, table, ctx), t2, p2))
        top = max(ext, key=lambda e: float(e[0]))
        best = top
        if eos_id >= 0 and top[1][-1] == eos_id:
            return list(top[1]), top[0]
        live = [(t, p) for _, t, p in ext if not (eos_id >= 0 and t[-1] == eos_id)]
    return list(best[1]), best[0]


@pytest.mark.parametrize("seed", range(6))
def test_wide_beam_equals_exhaustive_enumeration(seed):
    rng = np.random.default_rng(seed)
    k, m_max, vocab = int(rng.integers(2, 6)), int(rng.integers(2, 5)), 40
    eos = vocab - 2 if seed % 2 == 0 else -1
    lat, _ = _random_lattice(rng, k, m_max, vocab, eos)
    lat["cand_cnt"][:] = rng.integers(1, m_max + 1, size=k)
    if eos >= 0:  # make EOS competitive somewhere so the early stop is exercised
        lat["eos_logp"][:] = lat["cand_logp"][:, 0] - f32(0.05)
        lat["eos_logp"][k // 2] = lat["cand_logp"][k // 2, 0] + f32(0.5)
    table = _table()
    ctx = (3, 5)
    big = (m_max + 1) ** k
    toks, score, _ = cps.cps_path(lat, 0, k, big, 0.5, table, LOG2, ctx, eos)
    ref_toks, ref_score = _enumerate_best(lat, k, 0.5, table, ctx, eos)
    assert toks == ref_toks and score == ref_score


def test_eos_early_stop_returns_path_ending_in_eos():
    rng = np.random.default_rng(11)
    eos = 38
    lat, _ = _random_lattice(rng, 5, 3, 40, eos)
    lat["eos_logp"][:] = -30.0
    lat["eos_logp"][2] = 5.0   # EOS dominates at depth 3
    toks, _, _ = cps.cps_path(lat, 0, 5, 4, 1.0, None, LOG2, (0, 0), eos)
    assert len(toks) == 3 and toks[-1] == eos and eos not in toks[:-1]


def _viterbi(lat, k, lam, table, ctx):
    """Exact optimum without EOS: DP over (previous token, current token) states, float64."""
    lam = float(f32(lam))
    one_minus = float(f32(f32(1.0) - f32(lam)))
    states = {(int(ctx[0]), int(ctx[1])): (0.0, [])}
    for i in range(k):
        cands = cps.position_candidates(lat, i, -1)
        nxt = {}
        for (u, v), (sc, toks) in states.items():
            for w, l in cands:
                s = sc + lam * float(l) + one_minus * float(table[cps.ngram_slot(u, v, w, LOG2)])
                if (v, w) not in nxt or s > nxt[(v, w)][0]:
                    nxt[(v, w)] = (s, toks + [w])
        states = nxt
    return max(states.values(), key=lambda e: e[0])


@pytest.mark.parametrize("seed", range(4))
def test_wide_beam_equals_viterbi_without_eos(seed):
    rng = np.random.default_rng(100 + seed)
    k, m_max = 6, 3
    lat, _ = _random_lattice(rng, k, m_max, 30, -1)
    table = _table()
    toks, score, _ = cps.cps_path(lat, 0, k, m_max ** k, 0.5, table, LOG2, (1, 2), -1)
    v_score, v_toks = _viterbi(lat, k, 0.5, table, (1, 2))
    assert toks == v_toks and abs(float(score) - v_score) < 1e-4


@pytest.mark.parametrize("beam", [1, 2, 5])
def test_lambda_one_is_per_position_top1(beam):
    rng = np.random.default_rng(7)
    lat, _ = _random_lattice(rng, 9, 4, 50, -1)
    toks, score, _ = cps.cps_path(lat, 0, 9, beam, 1.0, _table(), LOG2, (4, 4), -1)
    assert toks == list(lat["cand_id"][:, 0])
    acc = f32(0.0)
    for i in range(9):
        acc = f32(acc + lat["cand_logp"][i, 0])
    assert score == acc
    # no proxy table at any lambda: ordering is by l_dlm alone
    toks2, _, _ = cps.cps_path(lat, 0, 9, beam, 0.3, None, LOG2, (4, 4), -1)
    assert toks2 == toks


def test_beam_one_is_greedy_left_to_right():
    rng = np.random.default_rng(8)
    lat, _ = _random_lattice(rng, 7, 4, 50, -1)
    table = _table()
    toks, _, _ = cps.cps_path(lat, 0, 7, 1, 0.5, table, LOG2, (9, 8), -1)
    u, v = 9, 8
    greedy = []
    for i in range(7):
        best = None
        for w, l in cps.position_candidates(lat, i, -1):
            s = cps.step_term(f32(0.5), l, f32(table[cps.ngram_slot(u, v, w, LOG2)]))
            if best is None or s > best[0]:
                best = (s, w)
        greedy.append(best[1])
        u, v = v, best[1]
    assert toks == greedy


def test_proxy_changes_the_path_and_context_matters():
    """With lambda < 1 the searched path differs from the raw draft somewhere and depends on ctx."""
    rng = np.random.default_rng(9)
    lat, _ = _random_lattice(rng, 12, 4, 60, -1)
    lat["cand_logp"][:] = lat["cand_logp"][:, :1] - np.arange(4, dtype=np.float32) * f32(0.01)
    table = _table()
    a, _, _ = cps.cps_path(lat, 0, 12, 4, 0.5, table, LOG2, (1, 2), -1)
    b, _, _ = cps.cps_path(lat, 0, 12, 4, 0.5, table, LOG2, (7, 3), -1)
    assert a != list(lat["cand_id"][:, 0])
    assert a != b


def test_candidate_evaluation_count_matches_complexity_statement():
    rng = np.random.default_rng(10)
    k, m_max, beam = 10, 5, 3
    lat, _ = _random_lattice(rng, k, m_max, 80, -1)
    lat["cand_cnt"][:] = rng.integers(1, m_max + 1, size=k)
    _, _, evals = cps.cps_path(lat, 0, k, beam, 0.5, _table(), LOG2, (1, 1), -1)
    live = 1
    expect = 0
    for i in range(k):
        c = int(lat["cand_cnt"][i])
        expect += live * c
        live = min(beam, live * c)
    assert evals == expect
    assert evals <= beam * (m_max + 1) * k


def test_beam_ordering_ties_parent_then_rank():
    """Equal scores: the lower parent index, then the lower candidate rank, is kept first."""
    k, m = 2, 2
    lat = {"cand_id": np.array([[10, 11], [20, 21]], dtype=np.int32),
           "cand_logp": np.array([[-1.0, -1.0], [-2.0, -2.0]], dtype=np.float32),
           "cand_cnt": np.array([2, 2], dtype=np.int32), "eos_logp": np.zeros(2, dtype=np.float32)}
    toks, _, _ = cps.cps_path(lat, 0, k, 2, 1.0, None, LOG2, (0, 0), -1)
    assert toks == [10, 20]


def test_ngram_slot_is_a_fixed_uint32_function():
    # worked by hand with Python integers (mod 2^32)
    def ref(u, v, w, bits):
        m = 0xFFFFFFFF
        x = (u * 0x9E3779B1) & m
        x ^= x >> 15
        x = ((x + v) * 0x85EBCA77) & m
        x ^= x >> 13
        x = ((x + w) * 0xC2B2AE3D) & m
        x ^= x >> 16
        return x & ((1 << bits) - 1)
    for u, v, w in [(0, 0, 0), (1, 2, 3), (152063, 152062, 7), (4095, 0, 4094)]:
        assert cps.ngram_slot(u, v, w, 22) == ref(u, v, w, 22)
    assert cps.ngram_slot(0, 0, 0, 22) == 0
    assert len({cps.ngram_slot(1, 2, w, 22) for w in range(1000)}) > 990


def test_search_margins_are_the_gaps_at_the_beam_boundary():
    """The diagnostic margins of the oracle search: per depth the smallest gap between neighbouring scores among the
    kept hypotheses and the best dropped one (hand-made two-position lattice, no proxy, lambda = 1)."""
    lat = {"cand_id": np.array([[1, 2, 3], [4, 5, 6]], np.int32),
           "cand_logp": np.array([[-1.0, -1.5, -4.0], [-0.25, -2.0, -2.125]], np.float32),
           "cand_cnt": np.array([3, 3], np.int32), "eos_logp": np.zeros(2, np.float32)}
    m = []
    toks, score, _ = cps.cps_path(lat, 0, 2, 2, 1.0, None, 0, [0, 0], -1, margins=m)
    assert toks == [1, 4] and score == f32(-1.25)
    # depth 0: kept -1.0, -1.5, dropped -4.0 -> gaps 0.5, 2.5; depth 1: scores -1.25, -1.75 kept, -3.0 dropped
    assert m == [0.5, 0.5]
    m = []
    cps.cps_path(lat, 0, 2, 3, 1.0, None, 0, [0, 0], -1, margins=m)
    # beam 3, depth 1: nine expansions -1.25 -1.75 -3.0 -3.125 -3.5 -3.625 ...: kept three, best dropped -3.125
    assert m == [0.5, 0.125]
    m = []
    cps.cps_path(lat, 0, 1, 4, 1.0, None, 0, [0, 0], -1, margins=m)
    assert m == [0.5]
    assert cps.cps_path(lat, 0, 2, 2, 1.0, None, 0, [0, 0], -1)[0] == [1, 4]   # unchanged without the list


def test_narrow_beams_on_a_hand_worked_lattice_where_pruning_loses_the_optimum():
    """The worked example of tests/hand_cases.py (all sums done by hand there): beams 4, 2 and 1 return three
    different paths, the narrower ones because the prefix of the optimum is pruned at depth 1."""
    lat, table, ctx, expected = hand_cases.narrow_beam_case(LOG2, cps.ngram_slot)
    for beam, want_toks, want_score in expected:
        toks, score, _ = cps.cps_path(lat, 0, 3, beam, 0.5, table, LOG2, ctx, -1)
        assert toks == want_toks and score == f32(want_score), beam
    m = []
    cps.cps_path(lat, 0, 3, 2, 0.5, table, LOG2, ctx, -1, margins=m)
    assert m == [0.5, 0.5, 0.5]      # -0.5 | -1.0;  -1.5 | -2.0 | -3.0;  -7.0 | -7.5 | -8.0


# ------------------------------------------------------------------ path search with a tiny causal LM as the proxy

PROXY = synth.ModelCfg(n_layers=1, d_model=32, n_q=2, n_kv=1, head_dim=16, d_ffn=48, vocab=40, rope_base=1.0e4,
                       dtype="f32")


def _proxy_setup(seed, n_committed=9, n_pending=2):
    pw = synth.make_weights(PROXY, 70 + seed)
    for name in ("embed", "lm_head"):            # a proxy with opinions: log-probabilities spread over several nats
        pw[name] = (pw[name] * 20.0).astype(np.float32)
    rng = np.random.default_rng(80 + seed)
    committed = [int(t) for t in rng.integers(0, 36, n_committed)]
    cache = model.KVCache(PROXY)
    if n_committed > n_pending:
        model.prefill(PROXY, pw, cache, committed[:-n_pending])
    return pw, committed, cache, committed[-n_pending:]


def _lm_path_score(lat, pw, committed, toks, picks, lam):
    """Left-to-right float32 score of one path; the proxy's distributions come from ONE causal pass over
    committed + path tokens from an empty cache (no incremental cache, no copies)."""
    seq = list(committed) + list(toks[:-1])
    y = model.full_sequence(PROXY, pw, np.asarray(seq), np.zeros(len(seq), dtype=bool))
    logits = model.lm_head(pw, y[len(committed) - 1:])
    score = f32(0.0)
    for i, w in enumerate(toks):
        l_ng = cps.proxy_log_probs(logits[i])[w]
        one_minus = f32(f32(1.0) - f32(lam))
        score = f32(score + f32(f32(f32(lam) * picks[i][1]) + f32(one_minus * l_ng)))
    return score


def _enumerate_best_lm(lat, k, lam, pw, committed, eos_id):
    live = [((), ())]
    best = None
    for i in range(k):
        cands = cps.position_candidates(lat, i, eos_id)
        ext = []
        for toks, picks in live:
            for w, l in cands:
                t2, p2 = toks + (w,), picks + ((w, l),)
                ext.append((_lm_path_score(lat, pw, committed, t2, p2, lam), t2, p2))
        top = max(ext, key=lambda e: float(e[0]))
        best = top
        if eos_id >= 0 and top[1][-1] == eos_id:
            return list(top[1]), top[0]
        live = [(t, p) for _, t, p in ext if not (eos_id >= 0 and t[-1] == eos_id)]
    return list(best[1]), best[0]


def test_proxy_log_probs_is_a_normalised_log_softmax():
    z = (np.random.default_rng(0).standard_normal(37) * 4).astype(np.float32)
    lp = cps.proxy_log_probs(z)
    assert lp.dtype == np.float32 and abs(float(np.exp(lp.astype(np.float64)).sum()) - 1.0) < 1e-6
    assert np.argmax(lp) == np.argmax(z) and np.allclose(lp - lp[0], z - z[0], atol=1e-5)


@pytest.mark.parametrize("seed", range(4))
def test_lm_proxy_wide_beam_equals_exhaustive_enumeration_from_scratch(seed):
    rng = np.random.default_rng(100 + seed)
    k, m_max, vocab = 3, 3, PROXY.vocab
    eos = vocab - 2 if seed % 2 == 0 else -1
    lat, _ = _random_lattice(rng, k, m_max, vocab, eos)
    lat["cand_cnt"][:] = rng.integers(2, m_max + 1, size=k)
    if eos >= 0:
        lat["eos_logp"][:] = lat["cand_logp"][:, 0] - f32(0.05)
    pw, committed, cache, pending = _proxy_setup(seed)
    before = cache.length
    toks, score, evals = cps.cps_path_lm(lat, 0, k, (m_max + 1) ** k, 0.4, PROXY, pw, cache, pending, eos)
    assert cache.length == before + len(pending)          # the pending tokens are committed, nothing else
    ref_toks, ref_score = _enumerate_best_lm(lat, k, 0.4, pw, committed, eos)
    assert toks == ref_toks and abs(float(score) - float(ref_score)) <= 2e-6 * max(1.0, abs(float(ref_score)))
    assert evals >= len(toks)


def test_lm_proxy_with_lambda_one_is_the_proxy_free_search():
    rng = np.random.default_rng(120)
    lat, _ = _random_lattice(rng, 6, 4, PROXY.vocab, 38)
    pw, _, cache, pending = _proxy_setup(5)
    a = cps.cps_path_lm(lat, 0, 6, 3, 1.0, PROXY, pw, cache, pending, 38)
    b = cps.cps_path(lat, 0, 6, 3, 1.0, None, LOG2, (0, 0), 38)
    assert a[0] == b[0] and a[1] == b[1] and a[2] == b[2]


def test_lm_proxy_changes_the_path_and_the_committed_tokens_matter():
    rng = np.random.default_rng(121)
    lat, _ = _random_lattice(rng, 6, 4, PROXY.vocab, -1)
    lat["cand_logp"][:] = f32(-1.0)                        # the drafter is indifferent: the proxy decides
    found = set()
    for seed in range(4):
        pw, _, cache, pending = _proxy_setup(seed)
        toks, score, _ = cps.cps_path_lm(lat, 0, 6, 4, 0.5, PROXY, pw, cache, pending, -1)
        # indifferent drafter: the score is lam * (-k) + (1 - lam) * sum of proxy log-probabilities
        assert float(score) < 0.5 * -6.0
        found.add(tuple(toks))
    assert len(found) > 1
    pw, committed, cache, pending = _proxy_setup(0)
    base = cps.cps_path_lm(lat, 0, 6, 4, 0.5, PROXY, pw, cache, pending, -1)
    other = model.KVCache(PROXY)
    model.prefill(PROXY, pw, other, [(t + 7) % 36 for t in committed[:-2]])
    moved = cps.cps_path_lm(lat, 0, 6, 4, 0.5, PROXY, pw, other, pending, -1)
    assert base[1] != moved[1]                             # same pending tokens, another history: another score
