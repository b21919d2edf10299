"""GPU parity: token lattice and path search kernels vs the CPU oracle, through the C ABI.

Bars: token ids, candidate counts, paths, path lengths: bit-exact.  Path scores: bit-exact
(float32, same unfused operation order, lattice log-scores passed as data).  lse / log-probabilities: 1e-5
absolute (the kernel sums exp() in float32 tree order, the oracle in float64; both round to float32).
"""
import numpy as np
import pytest
import torch

from oracle import cps as o_cps
from oracle import lattice as o_lat
from paper_2510_02358_amd import synth

import gpu_util as gu

pytestmark = pytest.mark.gpu

LSE_TOL = 1e-5
VOCAB = 152064


def _compare_lattice(got: dict, ref: dict, logits: np.ndarray):
    g = {k: gu.from_dev(v) for k, v in got.items()}
    assert np.array_equal(g["cand_id"], ref["cand_id"])
    assert np.max(np.abs(g["lse"] - ref["lse"])) <= LSE_TOL
    assert np.max(np.abs(g["cand_logp"] - ref["cand_logp"])) <= LSE_TOL
    assert np.max(np.abs(g["eos_logp"] - ref["eos_logp"])) <= LSE_TOL
    assert np.array_equal(g["cand_cnt"], ref["cand_cnt"])
    # internal consistency, exact: log-prob is logit - lse in float32
    rows = logits.shape[0]
    assert np.array_equal(g["cand_logp"], logits[np.arange(rows)[:, None], g["cand_id"]] - g["lse"][:, None])
    return g


@pytest.mark.parametrize("k_len,tau", [(8, 1.0), (16, 1.0), (32, 0.8)])
def test_lattice_full_vocab_batch16(k_len, tau):
    """Stress-test shape: 16 sequences x K positions x 152064 logits, top-16; every row of every array against the
    oracle (K = 32 with mass pruning on: 512 rows, 311 MB of logits)."""
    logits = synth.make_logits(16, k_len, VOCAB, seed=40 + k_len)
    eos = VOCAB - 2
    ref = o_lat.build_lattice(logits, 16, tau, eos)
    got = gu.gpu_lattice(gu.to_dev(logits), 16, tau, eos)
    _compare_lattice(got, ref, logits)


@pytest.mark.parametrize("rows,vocab,m_max", [(1, 16, 16), (3, 4099, 5), (7, 8192, 8), (5, 8193, 1), (2, 20001, 16),
                                             (33, 152064, 8), (40, 32768 + 12, 4)])
def test_lattice_ragged_shapes(rows, vocab, m_max):
    rng = np.random.default_rng(rows * 1000 + vocab)
    logits = (rng.standard_normal((rows, vocab)) * 3).astype(np.float32)
    eos = vocab - 2 if vocab > 2 else -1
    ref = o_lat.build_lattice(logits, m_max, 1.0, eos)
    got = gu.gpu_lattice(gu.to_dev(logits), m_max, 1.0, eos)
    _compare_lattice(got, ref, logits)


def test_lattice_ties_flat_rows_and_pruning():
    vocab = 12000
    rng = np.random.default_rng(5)
    logits = (rng.standard_normal((6, vocab))).astype(np.float32)
    logits[0, :] = 0.5                                   # flat: ids 0..M-1
    logits[1, [11999, 7, 8191, 8192, 4096]] = 9.0        # exact ties across tiles and wavefronts
    logits[2, :] = -np.inf
    logits[2, [5, 600, 7000, 11998]] = [1.0, 1.0, 0.0, -3.0]   # -inf elsewhere
    p = np.full(vocab, 0.05 / (vocab - 3)); p[[100, 9000, 3]] = [0.50, 0.35, 0.10]
    logits[3] = np.log(p).astype(np.float32)             # mass pruning: two survive at tau = 0.8
    p = np.full(vocab, 0.07 / (vocab - 1)); p[11000] = 0.93
    logits[4] = np.log(p).astype(np.float32)             # peaky: one survives
    ref = o_lat.build_lattice(logits, 4, 0.8, vocab - 2)
    got = gu.gpu_lattice(gu.to_dev(logits), 4, 0.8, vocab - 2)
    g = _compare_lattice(got, ref, logits)
    assert list(g["cand_id"][0]) == [0, 1, 2, 3]
    assert list(g["cand_id"][1]) == [7, 4096, 8191, 8192]
    assert list(g["cand_id"][2]) == [5, 600, 7000, 11998]
    assert g["cand_cnt"][3] == 2 and g["cand_cnt"][4] == 1 and g["cand_cnt"][0] == 4


def test_lattice_is_deterministic():
    logits = gu.to_dev(synth.make_logits(4, 8, 50000, seed=9))
    a = gu.gpu_lattice(logits, 8, 1.0, -1)
    b = gu.gpu_lattice(logits, 8, 1.0, -1)
    for k in a:
        assert torch.equal(a[k], b[k])


# ------------------------------------------------------------------------------------------ path search

def _cps_case(batch, k_len, m_max, beam, lam, eos_id, seed, vocab=VOCAB, use_table=True, peaky=False, tau=1.0):
    rng = np.random.default_rng(seed)
    # lattice built by the ORACLE from seeded logits restricted to a small random vocabulary slice per row
    rows = batch * k_len
    cand_id = np.zeros((rows, m_max), dtype=np.int32)
    cand_logp = np.zeros((rows, m_max), dtype=np.float32)
    for r in range(rows):
        ids = rng.choice(vocab - 2, size=m_max, replace=False)
        lp = np.sort(rng.standard_normal(m_max).astype(np.float32) * (3.0 if peaky else 0.7) - 8.0)[::-1]
        cand_id[r], cand_logp[r] = ids, lp
    cnt = rng.integers(1, m_max + 1, size=rows).astype(np.int32) if tau < 1.0 else np.full(rows, m_max, np.int32)
    eos_logp = (cand_logp[:, 0] - rng.uniform(0.0, 2.0, rows).astype(np.float32)).astype(np.float32)
    if eos_id >= 0:   # sometimes make EOS the clear winner so the early stop triggers at different depths
        hot = rng.random(rows) < 0.04
        eos_logp[hot] = cand_logp[hot, 0] + np.float32(6.0)
        inside = rng.random(rows) < 0.05
        cand_id[inside, m_max - 1] = eos_id
    lat = {"cand_id": cand_id, "cand_logp": cand_logp, "cand_cnt": cnt, "eos_logp": eos_logp}
    ctx = synth.make_contexts(vocab, batch, seed + 1)
    table = synth.make_ngram_table(3) if use_table else None
    ref_path, ref_len, ref_score = o_cps.cps_batch(lat, batch, k_len, beam, lam, table, synth.NGRAM_LOG2_SIZE, ctx,
                                                   eos_id)
    table_d = gu.to_dev(table) if use_table else None
    for with_ws in (True, False):   # with and without the optional scratch: same bits
        path, plen, score = gu.gpu_cps(lat, batch, k_len, m_max, beam, lam, table_d, synth.NGRAM_LOG2_SIZE, ctx,
                                       eos_id, with_ws=with_ws)
        assert np.array_equal(plen, ref_len)
        assert np.array_equal(path, ref_path)
        assert np.array_equal(score.view(np.uint32), ref_score.view(np.uint32))
    return ref_len


@pytest.mark.parametrize("k_len", [8, 16, 32, 64])
def test_cps_stress_shape_batch16_top16_beam8(k_len):
    _cps_case(16, k_len, 16, 8, 0.5, VOCAB - 2, seed=100 + k_len)


@pytest.mark.parametrize("batch,k_len,m_max,beam,lam,eos,tau", [
    (1, 1, 1, 1, 0.5, -1, 1.0), (3, 7, 4, 4, 0.5, 4094, 1.0), (2, 33, 8, 4, 0.5, -1, 1.0), (5, 20, 15, 3, 0.5, 100, 0.8),
    (2, 256, 16, 16, 0.25, 7, 0.8), (4, 12, 16, 16, 0.0, -1, 1.0), (4, 12, 6, 5, 1.0, 9, 1.0), (1, 64, 2, 16, 0.75, -1, 0.8),
])
def test_cps_shapes_and_edge_parameters(batch, k_len, m_max, beam, lam, eos, tau):
    _cps_case(batch, k_len, m_max, beam, lam, eos, seed=batch * 7 + k_len, tau=tau)


@pytest.mark.parametrize("seed", [11, 12])
def test_cps_seeded_sweep_with_inexact_lambda(seed):
    """Seeded sweep over batch, depth, M, beam, EOS and pruning with mixing weights that are NOT exact in binary
    (0.3, 0.7, 0.37): the products lambda * l_dlm and (1 - lambda) * l_ng then round, so a fused multiply-add
    anywhere in the kernel's score update would change score bits (and occasionally the kept hypotheses)."""
    rng = np.random.default_rng(seed)
    for _ in range(30):
        batch = int(rng.choice([1, 2, 5, 16]))
        k_len = int(rng.choice([1, 2, 7, 8, 31, 32, 64]))
        m_max, beam = int(rng.integers(1, 17)), int(rng.integers(1, 17))
        lam = float(rng.choice([0.3, 0.7, 0.37, 0.5]))
        eos = int(rng.choice([-1, VOCAB - 2]))
        tau = float(rng.choice([1.0, 0.8]))
        _cps_case(batch, k_len, m_max, beam, lam, eos, int(rng.integers(1 << 30)), peaky=bool(rng.random() < 0.3),
                  tau=tau)


def test_cps_without_proxy_and_peaky_lattice():
    _cps_case(4, 16, 8, 4, 0.5, -1, seed=3, use_table=False)
    lens = _cps_case(8, 24, 8, 4, 0.5, VOCAB - 2, seed=4, peaky=True)
    assert lens.min() >= 1


def test_cps_eos_first_position_and_ties():
    # EOS wins immediately: length 1
    m_max, k_len = 4, 5
    lat = {"cand_id": np.tile(np.array([[10, 11, 12, 13]], dtype=np.int32), (k_len, 1)),
           "cand_logp": np.tile(np.array([[-1.0, -1.0, -2.0, -2.0]], dtype=np.float32), (k_len, 1)),
           "cand_cnt": np.full(k_len, 4, dtype=np.int32), "eos_logp": np.full(k_len, -0.5, dtype=np.float32)}
    ctx = np.array([[1, 2]], dtype=np.int32)
    path, plen, score = gu.gpu_cps(lat, 1, k_len, m_max, 3, 1.0, None, 0, ctx, 99)
    assert plen[0] == 1 and path[0, 0] == 99 and list(path[0, 1:]) == [-1] * 4
    ref = o_cps.cps_batch(lat, 1, k_len, 3, 1.0, None, 0, ctx, 99)
    assert np.array_equal(path, ref[0]) and score[0] == ref[2][0]
    # exact score ties: lower parent, then lower rank
    path, plen, score = gu.gpu_cps(lat, 1, k_len, m_max, 3, 1.0, None, 0, ctx, -1)
    ref = o_cps.cps_batch(lat, 1, k_len, 3, 1.0, None, 0, ctx, -1)
    assert np.array_equal(path, ref[0]) and list(path[0]) == [10] * 5


def test_cps_hand_worked_narrow_beams():
    """The hand-computed example of tests/hand_cases.py on the GPU: beams 4, 2, 1 return the three hand-derived paths
    and scores (the narrower beams lose the optimum because its prefix is pruned at depth 1)."""
    import hand_cases
    log2 = 12
    lat, table, ctx, expected = hand_cases.narrow_beam_case(log2, o_cps.ngram_slot)
    for beam, want_toks, want_score in expected:
        for with_ws in (True, False):
            path, plen, score = gu.gpu_cps(lat, 1, 3, 2, beam, 0.5, gu.to_dev(table), log2,
                                           np.array([ctx], dtype=np.int32), -1, with_ws=with_ws)
            assert plen[0] == 3 and list(path[0]) == want_toks and score[0] == np.float32(want_score), beam


def test_cps_host_mirror_holds_path_length_and_raw_draft():
    """The optional pinned-memory mirror of the search: per sequence the path (tail -1), its length and the top
    candidate of every position, equal to what the device outputs and the lattice hold; with and without the
    pre-gathered proxy scores, EOS stopping some sequences early."""
    from paper_2510_02358_amd import binding as ds
    rng = np.random.default_rng(77)
    batch, k, m_max, beam, eos = 3, 11, 5, 4, VOCAB - 2
    rows = batch * k
    cand_id = np.stack([rng.choice(VOCAB - 2, size=m_max, replace=False) for _ in range(rows)]).astype(np.int32)
    cand_logp = np.sort(rng.standard_normal((rows, m_max)).astype(np.float32) - 6.0, axis=1)[:, ::-1].copy()
    eos_logp = (cand_logp[:, 0] - np.float32(1.0)).astype(np.float32)
    eos_logp[k + 4] = cand_logp[k + 4, 0] + np.float32(7.0)          # sequence 1 stops at depth 5
    lat = {"cand_id": cand_id, "cand_logp": cand_logp, "cand_cnt": np.full(rows, m_max, np.int32), "eos_logp": eos_logp}
    d = {n: gu.to_dev(v) for n, v in lat.items()}
    table = gu.to_dev(synth.make_ngram_table(3))
    proxy = ds.ds_ngram_create(table, synth.NGRAM_LOG2_SIZE)
    ctx = gu.to_dev(synth.make_contexts(VOCAB, batch, 5))
    try:
        for with_ws in (True, False):
            path = torch.empty(batch, k, dtype=torch.int32, device=gu.DEV)
            plen = torch.empty(batch, dtype=torch.int32, device=gu.DEV)
            score = torch.empty(batch, dtype=torch.float32, device=gu.DEV)
            mirror = torch.full((batch, 2 * k + 1), -9, dtype=torch.int32).pin_memory()
            ws = torch.empty(ds.ds_cps_workspace_bytes(batch, k, m_max), dtype=torch.uint8, device=gu.DEV) if with_ws else None
            ds.ds_cps_path(d["cand_id"], d["cand_logp"], d["cand_cnt"], d["eos_logp"], batch, k, m_max, beam, 0.5, proxy,
                           ctx, eos, path, plen, score, ws, host_mirror=mirror)
            torch.cuda.synchronize()
            m = mirror.numpy()
            assert np.array_equal(m[:, :k], path.cpu().numpy())
            assert np.array_equal(m[:, k], plen.cpu().numpy()) and m[1, k] == 5 and m[1, 4] == eos
            assert np.array_equal(m[:, k + 1:], cand_id[:, 0].reshape(batch, k))
            ref = o_cps.cps_batch(lat, batch, k, beam, 0.5, synth.make_ngram_table(3), synth.NGRAM_LOG2_SIZE,
                                  ctx.cpu().numpy(), eos)
            assert np.array_equal(m[:, :k], ref[0])
    finally:
        ds.ds_ngram_destroy(proxy)


def test_lattice_then_cps_end_to_end_on_device():
    """Lattice arrays stay on the device between the two calls; compared against the oracle chain fed
    with the SAME float32 logits.  Path equality can only break at float32 near-ties of scores, which
    are flagged rather than hidden."""
    batch, k_len, m_max, beam = 4, 16, 8, 4
    logits = synth.make_logits(batch, k_len, 30000, seed=77)
    eos = 29998
    got = gu.gpu_lattice(gu.to_dev(logits), m_max, 1.0, eos)
    ctx = synth.make_contexts(30000, batch, 78)
    table = synth.make_ngram_table(3)
    path, plen, score = gu.gpu_cps(got, batch, k_len, m_max, beam, 0.5, gu.to_dev(table), synth.NGRAM_LOG2_SIZE, ctx, eos)
    ref_lat = o_lat.build_lattice(logits, m_max, 1.0, eos)
    rpath, rlen, rscore = o_cps.cps_batch(ref_lat, batch, k_len, beam, 0.5, table, synth.NGRAM_LOG2_SIZE, ctx, eos)
    agree = np.mean(path == rpath)
    assert agree == 1.0, f"token agreement {agree}"
    assert np.max(np.abs(score - rscore)) < 1e-3


def test_lattice_stress_full_size_k64_sampled_rows_and_properties():
    """16 x 64 = 1024 rows x 152064 logits (622.9 MB), top-16: sampled rows against the oracle, and
    size-independent properties on every row."""
    k_len, m_max = 64, 16
    logits = synth.make_logits(16, k_len, VOCAB, seed=123)
    eos = VOCAB - 2
    got = {k: gu.from_dev(v) for k, v in gu.gpu_lattice(gu.to_dev(logits), m_max, 0.8, eos).items()}
    rows = logits.shape[0]
    sample = np.random.default_rng(0).choice(rows, size=24, replace=False)
    ref = o_lat.build_lattice(logits[sample], m_max, 0.8, eos)
    assert np.array_equal(got["cand_id"][sample], ref["cand_id"])
    assert np.array_equal(got["cand_cnt"][sample], ref["cand_cnt"])
    assert np.max(np.abs(got["lse"][sample] - ref["lse"])) <= LSE_TOL
    assert np.max(np.abs(got["cand_logp"][sample] - ref["cand_logp"])) <= LSE_TOL
    # every row: candidates are the row's largest values in order, log-prob identity, mass bound
    picked = logits[np.arange(rows)[:, None], got["cand_id"]]
    assert np.all(np.diff(picked, axis=1) <= 0)
    assert np.array_equal(picked[:, 0], logits.max(axis=1))
    kth = np.partition(logits, VOCAB - m_max, axis=1)[:, VOCAB - m_max]
    assert np.array_equal(picked[:, -1], kth)
    assert np.array_equal(got["cand_logp"], picked - got["lse"][:, None])
    assert np.array_equal(got["eos_logp"], logits[:, eos] - got["lse"])
    mass = np.exp(got["cand_logp"].astype(np.float64)).sum(axis=1)
    assert np.all(mass < 1.0) and np.all(got["cand_cnt"] >= 1) and np.all(got["cand_cnt"] <= m_max)
    lse64 = np.log(np.exp(logits[::37].astype(np.float64) - 20.0).sum(axis=1)) + 20.0
    assert np.max(np.abs(got["lse"][::37] - lse64)) <= LSE_TOL
