"""GPU parity: drafter / verifier forwards, LM head and greedy acceptance vs the CPU oracle, through the C ABI.

Bars (from the benchmark spec): logits max-abs 1e-4 in float32 mode, 2e-2 with bf16 storage and float32
accumulation.  Arg-max / accepted length must agree exactly unless the oracle's top-2 logit gap is below
twice the tolerance (a flagged near-tie).  Fed identical logits, acceptance is bit-exact.
"""
import dataclasses

import numpy as np
import pytest
import torch

from oracle import accept as o_accept
from oracle import lattice as o_lat
from oracle import model as o_model
from paper_2510_02358_amd import binding as ds
from paper_2510_02358_amd import synth

import gpu_util as gu

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-4, "bf16": 2e-2}
SMALL_BF16 = synth.ModelCfg(n_layers=2, d_model=256, n_q=4, n_kv=2, head_dim=128, d_ffn=512, vocab=4096,
                            rope_base=1.0e6, dtype="bf16")


def _check_argmax(gpu_am, ref_logits, tol):
    """Exact agreement except at flagged near-ties; returns the number of flagged rows."""
    ref_am = o_accept.greedy_argmax(ref_logits)
    flagged = 0
    for r in range(len(ref_am)):
        if gpu_am[r] != ref_am[r]:
            top2 = np.sort(ref_logits[r])[-2:]
            assert top2[1] - top2[0] < 2 * tol, f"row {r}: argmax {gpu_am[r]} vs {ref_am[r]} with a clear gap"
            flagged += 1
    return flagged


def _round_trip(cfg, w, prefix, pending_extra, k1, k2, kv_cap, seed):
    """prefill -> draft (1 pending) -> verify -> commit -> draft (several pending) -> verify; all vs oracle."""
    tol = TOL[cfg.dtype]
    gm = gu.GpuModel(cfg, w, kv_cap)
    try:
        oc = o_model.KVCache(cfg)
        ref_last = o_model.prefill(cfg, w, oc, prefix)
        got_last = gm.prefill(prefix)
        assert gm.kv_len == len(prefix)
        err = np.max(np.abs(got_last - ref_last))
        assert err <= tol, f"prefill logits err {err}"
        scale = float(np.std(ref_last))
        assert err <= 0.05 * scale, f"prefill err {err} vs logits std {scale}"

        # ---- first draft pass: one pending token
        pend = [int(np.argmax(ref_last))]
        ref_hid = o_model.draft_block(cfg, w, oc, pend, k1)
        hid = gm.draft(pend, k1)
        logits = gm.lm_head(hid)
        torch.cuda.synchronize()
        assert gm.kv_len == len(prefix) + 1 and oc.length == gm.kv_len
        h_err = np.max(np.abs(gu.from_dev(hid) - ref_hid))
        assert h_err <= (1e-2 if cfg.dtype == "bf16" else 1e-4), f"draft hidden err {h_err}"
        ref_logits = o_model.lm_head(w, ref_hid)
        l_err = np.max(np.abs(gu.from_dev(logits) - ref_logits))
        assert l_err <= tol, f"draft logits err {l_err}"
        assert l_err <= 0.05 * float(np.std(ref_logits))

        # ---- second draft pass: several pending tokens (as after an accepted prefix), different K
        ref_hid = o_model.draft_block(cfg, w, oc, pending_extra, k2)
        hid = gm.draft(pending_extra, k2)
        logits = gm.lm_head(hid)
        torch.cuda.synchronize()
        assert gm.kv_len == len(prefix) + 1 + len(pending_extra)
        ref_logits = o_model.lm_head(w, ref_hid)
        l_err = np.max(np.abs(gu.from_dev(logits) - ref_logits))
        assert l_err <= tol, f"draft-2 logits err {l_err}"

        # ---- verify against the same cache state: causal block of m + 1 rows
        rng = np.random.default_rng(seed)
        m = k1
        greedy_first = None
        block = np.concatenate([[pend[0]], rng.integers(0, cfg.n_plain_tokens, m)]).astype(np.int32)
        vc = o_model.KVCache(cfg)
        o_model.prefill(cfg, w, vc, prefix)
        gm.set_kv_len(len(prefix))          # roll the GPU cache back to the prefix (same model as verifier)
        ref_v = o_model.verify_logits(cfg, w, vc, block)
        # make the path partly right: first two tokens are the oracle's greedy choices, unless near-tied
        ref_am = o_accept.greedy_argmax(ref_v)
        block2 = block.copy()
        block2[1] = ref_am[0]
        vc.truncate(len(prefix))
        ref_v = o_model.verify_logits(cfg, w, vc, block2)
        ref_am = o_accept.greedy_argmax(ref_v)
        block2[2] = ref_am[1]
        vc.truncate(len(prefix))
        ref_v = o_model.verify_logits(cfg, w, vc, block2)
        out = gm.verify(block2, eos_id=cfg.eos_id)
        assert gm.kv_len == len(prefix)     # verify never advances the committed length
        v_err = np.max(np.abs(out["logits"] - ref_v))
        assert v_err <= tol, f"verify logits err {v_err}"
        flagged = _check_argmax(out["argmax"], ref_v, tol)
        # acceptance on the GPU's own logits is exactly the oracle rule applied to those logits
        n_acc, nxt, am, eos = o_accept.verify_greedy(out["logits"], block2[1:], cfg.eos_id)
        assert np.array_equal(out["argmax"], am)
        assert (out["n_accept"], out["next_token"], out["eos_accepted"]) == (n_acc, nxt, eos)
        if flagged == 0:
            r_acc, r_nxt, _, _ = o_accept.verify_greedy(ref_v, block2[1:], cfg.eos_id)
            assert (out["n_accept"], out["next_token"]) == (r_acc, r_nxt)
            assert out["n_accept"] >= 2
        # commit and check the cache by verifying the next block against it
        gm.set_kv_len(len(prefix) + 1 + out["n_accept"])
        vc.truncate(len(prefix) + 1 + out["n_accept"])
        nb = np.concatenate([[out["next_token"]], rng.integers(0, cfg.n_plain_tokens, 3)]).astype(np.int32)
        ref_v2 = o_model.verify_logits(cfg, w, vc, nb)
        out2 = gm.verify(nb, eos_id=cfg.eos_id)
        assert np.max(np.abs(out2["logits"] - ref_v2)) <= tol
        return flagged
    finally:
        gm.close()


def test_tiny_f32_pair_config():
    """The tiny float32 configuration: 2 layers, d=256, 4 heads x 64, FFN 688, vocab 4096, prefix 128, K=8."""
    cfg = synth.CFG_TINY
    w = synth.make_weights(cfg, 0)
    prefix = synth.make_prefix(cfg, 128, 2)
    _round_trip(cfg, w, prefix, [5, 77, 4000], 8, 5, kv_cap=192, seed=1)


def test_f32_ragged_shapes_and_random_gains():
    cfg = dataclasses.replace(synth.CFG_TINY, n_q=6, n_kv=2, head_dim=32, d_model=200, d_ffn=300, vocab=1003,
                              n_layers=3)
    w = synth.make_weights(cfg, 5, std=0.05)
    synth.randomize_norm_gains(w, 6)
    prefix = synth.make_prefix(cfg, 150, 7)
    _round_trip(cfg, w, prefix, [1, 2, 3, 4, 5, 6, 7], 13, 21, kv_cap=230, seed=2)


def test_small_bf16_two_layers_gqa():
    cfg = SMALL_BF16
    w = synth.make_weights(cfg, 10)            # N(0, 0.02): the scale the 2e-2 bar is stated for
    synth.randomize_norm_gains(w, 11)
    prefix = synth.make_prefix(cfg, 150, 12)   # prefill in two chunks, keys cross several 64-key chunks
    _round_trip(cfg, w, prefix, [9, 8, 7, 6, 5], 17, 40, kv_cap=256, seed=3)


def test_small_bf16_long_prefix_many_key_splits():
    """4200 cached tokens (66 key chunks: split counts beyond 16, a ragged last chunk) on the small bf16 model."""
    cfg = SMALL_BF16
    w = synth.make_weights(cfg, 50)
    prefix = synth.make_prefix(cfg, 4200, 51)
    _round_trip(cfg, w, prefix, [3, 1, 4, 1, 5, 9, 2, 6], 40, 7, kv_cap=4480, seed=52)


@pytest.mark.parametrize("cfg_name", ["f32", "bf16"])
def test_block_verification_is_bit_identical_to_one_token_decoding(cfg_name):
    """A row's logits do not depend on which other rows share the call: verifying m + 1 rows at once gives, bit
    for bit, the logits of decoding the same tokens one row at a time (so greedy verification reproduces the
    target's own greedy stream exactly).  Prefix lengths straddle chunk and split boundaries."""
    cfg = synth.CFG_TINY if cfg_name == "f32" else SMALL_BF16
    w = synth.make_weights(cfg, 60)
    rng = np.random.default_rng(61)
    gm = gu.GpuModel(cfg, w, 1024)
    try:
        for n_prefix, m in ((120, 9), (250, 20), (511, 33), (700, 70)):
            prefix = synth.make_prefix(cfg, n_prefix, 62 + n_prefix)
            block = rng.integers(0, cfg.n_plain_tokens, m + 1).astype(np.int32)
            gm.set_kv_len(0)
            gm.prefill(prefix, want_logits=False)
            whole = gm.verify(block)["logits"]
            for r in range(m + 1):
                gm.set_kv_len(n_prefix + r)               # rows 0 .. r-1 were written by the previous steps
                one = gm.verify(block[r:r + 1])["logits"]
                assert np.array_equal(one[0], whole[r]), (n_prefix, r)
    finally:
        gm.close()


@pytest.mark.parametrize("cfg_name", ["f32", "bf16"])
def test_lm_head_on_the_rows_the_draft_pass_left_behind(cfg_name):
    """ds_lm_head(hidden = NULL) right after a draft pass == ds_lm_head on that pass's hidden_out, bit for bit;
    in any other state the call is refused."""
    cfg = synth.CFG_TINY if cfg_name == "f32" else SMALL_BF16
    w = synth.make_weights(cfg, 70)
    gm = gu.GpuModel(cfg, w, 256)
    try:
        gm.prefill(synth.make_prefix(cfg, 90, 71), want_logits=False)
        for pending, k in (([5], 8), ([1, 2, 3], 21), ([], 33)):
            hid = gm.draft(pending, k)
            direct = torch.empty(k, cfg.vocab, dtype=torch.float32, device=gu.DEV)
            ds.ds_lm_head(gm.handle, None, k, direct, gm.ws)
            with pytest.raises(ds.DsError) as e:
                ds.ds_lm_head(gm.handle, None, k + 1, direct, gm.ws)     # wrong row count
            assert e.value.code == ds.DS_E_INVALID
            via_hidden = gm.lm_head(hid)
            torch.cuda.synchronize()
            assert torch.equal(direct, via_hidden)
        gm.verify(np.array([1, 2, 3], np.int32))                          # another forward: the rows are gone
        with pytest.raises(ds.DsError) as e:
            ds.ds_lm_head(gm.handle, None, 33, direct, gm.ws)
        assert e.value.code == ds.DS_E_INVALID
    finally:
        gm.close()


def test_bf16_lm_head_is_a_plain_gemm():
    """hidden (float32 -> IEEE half, round to nearest) x W^T with float32 accumulation: element by element the
    result stays within the rigorous rounding bound u * sum_k |x_k w_k| of one half rounding per activation
    (u = 2^-11), plus a float32 accumulation term; the weights (bf16 values in half range) are exact."""
    cfg = SMALL_BF16
    w = synth.make_weights(cfg, 20, std=0.05)
    gm = gu.GpuModel(cfg, w, 64)
    try:
        rng = np.random.default_rng(0)
        w_abs = np.abs(w["lm_head"].astype(np.float64))
        for rows in (1, 16, 17, 33, 100, 144):
            hid = rng.standard_normal((rows, cfg.d_model)).astype(np.float32)
            got = gu.from_dev(gm.lm_head(gu.to_dev(hid)))
            ref = o_model.lm_head(w, hid.astype(np.float64))
            mag = np.abs(hid.astype(np.float64)) @ w_abs.T
            bound = (2.0 ** -11 + cfg.d_model * 2.0 ** -23) * mag + 1e-7
            assert np.all(np.abs(got - ref) <= bound), rows
            # and the error is not systematically near the bound: rms well below it
            assert np.sqrt(np.mean((got - ref) ** 2)) < 0.2 * np.sqrt(np.mean(bound ** 2)), rows
    finally:
        gm.close()


def test_bf16_verify_argmax_comes_from_the_lm_head_epilogue():
    """The bf16 verifier takes each row's arg-max from per-tile records of the LM-head product, with or without
    the logits being written.  Both ways give the same verdict; the arg-max is exactly the arg-max of the logits
    the same call returns (first index on ties); and exact ties planted across tiles and inside one tile (LM-head
    rows duplicated, so the logits are bit-equal) resolve to the lowest token id."""
    cfg = SMALL_BF16
    w = dict(synth.make_weights(cfg, 90))
    lm = np.array(w["lm_head"], copy=True)
    rng = np.random.default_rng(91)
    gm = gu.GpuModel(cfg, w, 256)
    try:
        gm.prefill(synth.make_prefix(cfg, 70, 92), want_logits=False)
        block = rng.integers(0, cfg.n_plain_tokens, 34).astype(np.int32)
        for n in range(6):                      # make the first six drafted tokens the verifier's own choices
            gm.set_kv_len(70)
            block[n + 1] = gm.verify(block, want_logits=False)["argmax"][n]
        gm.set_kv_len(70)
        base = gm.verify(block)
    finally:
        gm.close()
    assert np.array_equal(base["argmax"], np.argmax(base["logits"], axis=1))
    assert base["n_accept"] >= 6
    # duplicate each of the first rows' winning LM-head row into a later tile, a lower id in another tile and
    # a neighbour in the same tile
    planted = {}
    for r in range(0, 34, 3):
        a = int(base["argmax"][r])
        for b in ((a + 1000) % cfg.vocab, (a + 2 * 128 + 5) % cfg.vocab, a ^ 1):
            if b in planted or b in base["argmax"]:
                continue
            lm[b] = lm[a]
            planted[b] = a
    w["lm_head"] = lm
    gm = gu.GpuModel(cfg, w, 256)
    try:
        gm.prefill(synth.make_prefix(cfg, 70, 92), want_logits=False)
        full = gm.verify(block)
        gm.set_kv_len(70)
        bare = gm.verify(block, want_logits=False)
        eos = int(full["argmax"][2])
        for pl in (0, 5, 33):
            dev_pl = gu.to_dev(np.array([pl], np.int32))
            gm.set_kv_len(70)
            a = gm.verify(block, path_len=dev_pl, eos_id=eos)
            gm.set_kv_len(70)
            b = gm.verify(block, path_len=dev_pl, eos_id=eos, want_logits=False)
            got = (a["n_accept"], a["next_token"], a["eos_accepted"])
            assert got == (b["n_accept"], b["next_token"], b["eos_accepted"])
            n_acc, nxt, _, eos_acc = o_accept.verify_greedy(a["logits"][:pl + 1], block[1:pl + 1], eos)
            assert got == (n_acc, nxt, eos_acc), (pl, got)
        # the widest block the library takes (144 rows: nine row blocks per workgroup) and the narrowest (one row)
        for n_rows in (ds.DS_MAX_ROWS, 1):
            wide = rng.integers(0, cfg.n_plain_tokens, n_rows).astype(np.int32)
            gm.set_kv_len(70)
            a = gm.verify(wide)
            gm.set_kv_len(70)
            b = gm.verify(wide, want_logits=False)
            assert np.array_equal(a["argmax"], np.argmax(a["logits"], axis=1))
            assert np.array_equal(a["argmax"], b["argmax"]) and a["next_token"] == b["next_token"]
    finally:
        gm.close()
    first_max = np.argmax(full["logits"], axis=1)
    assert np.array_equal(full["argmax"], first_max) and np.array_equal(bare["argmax"], first_max)
    ties = 0
    for r in range(34):
        row = full["logits"][r]
        ties += int(np.sum(row == row[first_max[r]]) > 1)
    assert ties >= 8, "the planted duplicates must produce exact ties"


LSE_TOL = 1e-5


def _check_fused_lattice(gm, hidden, rows, m_max, tau, eos_id):
    """ds_draft_lattice with and without the logits written: identical outputs; candidates, counts and log-scores
    are those the oracle builds from the logits the same call returned (ids / counts exact, float values 1e-5);
    and log-score == logit - lse exactly in float32."""
    full, logits = gm.draft_lattice(hidden, rows, m_max, tau, eos_id, want_logits=True)
    bare, _ = gm.draft_lattice(hidden, rows, m_max, tau, eos_id, want_logits=False)
    for k in full:
        assert torch.equal(full[k], bare[k]), k
    lg = gu.from_dev(logits)
    ref = o_lat.build_lattice(lg, m_max, tau, eos_id)
    g = {k: gu.from_dev(v) for k, v in full.items()}
    assert np.array_equal(g["cand_id"], ref["cand_id"])
    assert np.array_equal(g["cand_cnt"], ref["cand_cnt"])
    for k in ("lse", "cand_logp", "eos_logp"):
        assert np.max(np.abs(g[k] - ref[k])) <= LSE_TOL, k
    assert np.array_equal(g["cand_logp"], lg[np.arange(rows)[:, None], g["cand_id"]] - g["lse"][:, None])
    return g, lg


def test_bf16_lattice_from_the_lm_head_epilogue():
    """The fused LM head + lattice call on a bf16 model, against the oracle's lattice of the same logits:
    ordinary rows; rows whose best tokens all sit inside one 128-id tile (the tile is recomputed), with exact ties
    inside the cluster; an all-zero hidden row (every logit equal: ids 0 .. M-1); EOS inside and outside the
    cluster; M = 1, 8, 16; pruning on and off; 1, 33 and 144 rows."""
    cfg = SMALL_BF16
    w = dict(synth.make_weights(cfg, 95))
    lm = np.array(w["lm_head"], copy=True).astype(np.float32)
    rng = np.random.default_rng(96)
    u = rng.standard_normal(cfg.d_model).astype(np.float32)
    u /= np.linalg.norm(u)
    base = 5 * 128 + 40                       # a cluster of 12 ids inside tile 5
    for k in range(12):
        lm[base + k] = (0.30 + 0.01 * (k % 7)) * u      # (k % 7): ids base + 0 / + 7, + 1 / + 8 ... tie exactly
    lm[7 * 128 + 3] = 0.33 * u                # and one strong id in another tile
    w["lm_head"] = synth.round_to_bf16(lm)
    gm = gu.GpuModel(cfg, w, 256)
    try:
        for rows in (1, 33, 144):
            hid = rng.standard_normal((rows, cfg.d_model)).astype(np.float32)
            hid[::3] += 40.0 * u              # every third row lights the cluster up
            if rows > 4:
                hid[4] = 0.0                  # all logits equal
            for m_max, tau, eos in ((8, 1.0, base + 2), (16, 0.9, 3000), (1, 1.0, -1), (8, 0.5, 7 * 128 + 3)):
                g, lg = _check_fused_lattice(gm, gu.to_dev(hid), rows, m_max, tau, eos)
                if m_max == 8:
                    top = g["cand_id"][0]
                    assert np.sum((top >= 5 * 128) & (top < 6 * 128)) >= 7, "row 0 must draw from the cluster"
                    if rows > 4:
                        assert list(g["cand_id"][4]) == list(range(8))
        # straight after a draft pass (hidden = NULL), as the round calls it
        gm.prefill(synth.make_prefix(cfg, 50, 97), want_logits=False)
        gm.draft([3], 21)
        g, lg = _check_fused_lattice(gm, None, 21, 8, 0.95, cfg.eos_id)
        gm.verify(np.array([1, 2], np.int32))
        with pytest.raises(ds.DsError) as e:
            gm.draft_lattice(None, 21, 8, 0.95, cfg.eos_id)
        assert e.value.code == ds.DS_E_INVALID
        # the two-step form: the second step must follow the first with the same rows and EOS id
        hid = gu.to_dev(rng.standard_normal((9, cfg.d_model)).astype(np.float32))
        outs = [torch.empty(9, 8, dtype=torch.int32, device=gu.DEV), torch.empty(9, 8, device=gu.DEV),
                torch.empty(9, dtype=torch.int32, device=gu.DEV), torch.empty(9, device=gu.DEV),
                torch.empty(9, device=gu.DEV)]
        for bad_rows, bad_eos, between in ((8, 5, None), (9, 6, None), (9, 5, "forward"), (9, 5, "lm_head")):
            ds.ds_lm_head_tiles(gm.handle, hid, 9, 5, None, gm.ws)
            if between == "forward":
                gm.verify(np.array([1, 2], np.int32))
            elif between == "lm_head":
                gm.lm_head(hid)
            with pytest.raises(ds.DsError) as e:
                ds.ds_lattice_from_tiles(gm.handle, bad_rows, 8, 1.0, bad_eos, *outs, gm.ws)
            assert e.value.code == ds.DS_E_INVALID
        ds.ds_lm_head_tiles(gm.handle, hid, 9, 5, None, gm.ws)
        ds.ds_lattice_from_tiles(gm.handle, 9, 8, 1.0, 5, *outs, gm.ws)
        one_call, _ = gm.draft_lattice(hid, 9, 8, 1.0, 5, want_logits=False)
        torch.cuda.synchronize()
        assert torch.equal(outs[0], one_call["cand_id"]) and torch.equal(outs[4], one_call["lse"])
    finally:
        gm.close()


def test_bf16_vocabulary_that_the_tile_records_do_not_cover():
    """vocab = 4096 + 16 is a multiple of 16 (so the bf16 product runs) but not of 128: the LM head ends in a
    half-size workgroup, the record epilogues do not apply, and both the fused lattice call and the verifier fall
    back to the stored logits with unchanged results."""
    cfg = dataclasses.replace(SMALL_BF16, vocab=4096 + 16)
    w = synth.make_weights(cfg, 110)
    gm = gu.GpuModel(cfg, w, 256)
    try:
        gm.prefill(synth.make_prefix(cfg, 40, 111), want_logits=False)
        gm.draft([5, 6], 19)
        _check_fused_lattice(gm, None, 19, 8, 0.9, cfg.eos_id)
        block = np.random.default_rng(112).integers(0, cfg.n_plain_tokens, 20).astype(np.int32)
        full = gm.verify(block)
        gm.set_kv_len(42)
        bare = gm.verify(block, want_logits=False)
        assert np.array_equal(full["argmax"], np.argmax(full["logits"], axis=1))
        assert np.array_equal(full["argmax"], bare["argmax"]) and full["n_accept"] == bare["n_accept"]
        ref = o_model.lm_head(w, np.zeros((1, cfg.d_model)))
        assert ref.shape[1] == cfg.vocab
    finally:
        gm.close()


@pytest.mark.parametrize("vocab", [128, 1024, 8192, 33024])
def test_bf16_tile_records_seeded_sweep(vocab):
    """Seeded sweep over row counts, M, tau, EOS ids and planted runs of strong neighbouring ids with exact ties:
    the record-based lattice equals the oracle's lattice of the returned logits, with and without the logits being
    written, and the verifier's record-based arg-max equals the arg-max of its returned logits.  vocab = 128 is a
    single tile; 33024 needs two records per thread."""
    rng = np.random.default_rng(1000 + vocab)
    cfg = synth.ModelCfg(n_layers=1, d_model=256, n_q=2, n_kv=1, head_dim=128, d_ffn=256, vocab=vocab,
                         rope_base=1.0e6, dtype="bf16")
    for trial in range(2):
        w = dict(synth.make_weights(cfg, int(rng.integers(1 << 30))))
        lm = np.array(w["lm_head"], copy=True)
        u = rng.standard_normal(cfg.d_model).astype(np.float32)
        u /= np.linalg.norm(u)
        for _ in range(int(rng.integers(1, 4))):
            start, n = int(rng.integers(0, vocab - 20)), int(rng.integers(3, 18))
            for k in range(n):
                lm[start + k] = (0.3 + 0.01 * int(rng.integers(0, 5))) * u
        w["lm_head"] = synth.round_to_bf16(lm)
        gm = gu.GpuModel(cfg, w, 192)
        try:
            for sub in range(3):
                rows = int(rng.choice([1, 2, 15, 16, 17, 33, 64, 100, 144]))
                m_max = int(rng.integers(1, min(16, vocab) + 1))
                tau = float(rng.choice([1.0, 0.99, 0.9, 0.5]))
                eos = int(rng.integers(-1, vocab))
                hid = rng.standard_normal((rows, cfg.d_model)).astype(np.float32)
                hid[rng.random(rows) < 0.4] += 40.0 * u
                if rows > 2:
                    hid[1] = 0.0
                full, logits = gm.draft_lattice(gu.to_dev(hid), rows, m_max, tau, eos, want_logits=True)
                bare, _ = gm.draft_lattice(gu.to_dev(hid), rows, m_max, tau, eos, want_logits=False)
                for k in full:
                    assert torch.equal(full[k], bare[k]), (trial, sub, k)
                lg = gu.from_dev(logits)
                ref = o_lat.build_lattice(lg, m_max, tau, eos)
                g = {k: gu.from_dev(v) for k, v in full.items()}
                assert np.array_equal(g["cand_id"], ref["cand_id"]), (rows, m_max, tau, eos)
                for r in np.nonzero(g["cand_cnt"] != ref["cand_cnt"])[0]:   # only a mass within rounding of tau
                    cum = np.cumsum(np.exp(ref["cand_logp"][r].astype(np.float64)))
                    assert np.min(np.abs(cum - tau)) < 1e-5, (rows, r, cum, tau)
                for k in ("lse", "cand_logp", "eos_logp"):
                    assert np.max(np.abs(g[k] - ref[k])) <= LSE_TOL, (k, rows)
                blk = rng.integers(0, max(1, vocab - 2), int(rng.choice([1, 9, 33, 144]))).astype(np.int32)
                gm.set_kv_len(0)
                a = gm.verify(blk)
                gm.set_kv_len(0)
                b = gm.verify(blk, want_logits=False)
                assert np.array_equal(a["argmax"], np.argmax(a["logits"], axis=1))
                assert np.array_equal(a["argmax"], b["argmax"]) and a["n_accept"] == b["n_accept"]
        finally:
            gm.close()


def test_f32_fused_call_equals_the_two_separate_calls():
    cfg = synth.CFG_TINY
    w = synth.make_weights(cfg, 98)
    gm = gu.GpuModel(cfg, w, 128)
    try:
        gm.prefill(synth.make_prefix(cfg, 30, 99), want_logits=False)
        hid = gm.draft([2], 9)
        fused, logits = gm.draft_lattice(None, 9, 4, 0.9, cfg.eos_id)
        sep = gu.gpu_lattice(gm.lm_head(hid), 4, 0.9, cfg.eos_id)
        for k in fused:
            assert torch.equal(fused[k], sep[k]), k
    finally:
        gm.close()


def test_7b_layer_bf16_fused_lattice_full_vocabulary():
    """LM head 152064 x 3584 (1188 tiles), 32 rows, top-8 and top-16, straight after a draft pass."""
    cfg = synth.CFG_7B_LAYER
    w = synth.make_weights(cfg, 0)
    gm = gu.GpuModel(cfg, w, 256)
    try:
        gm.prefill(synth.make_prefix(cfg, 100, 2), want_logits=False)
        gm.draft([11], 32)
        _check_fused_lattice(gm, None, 32, 8, 0.9, cfg.eos_id)
        gm.draft([], 32)
        _check_fused_lattice(gm, None, 32, 16, 1.0, -1)
    finally:
        gm.close()
    # the same shape with a planted run of strong neighbouring ids (tile 700) and one exact tie inside it: rows that
    # light the run up have their whole top-8 in one tile, which the kernel must recompute (112 k-steps, 5 records
    # per thread)
    w = dict(w)
    lm = np.array(w["lm_head"], copy=True)
    rng = np.random.default_rng(7)
    u = rng.standard_normal(cfg.d_model).astype(np.float32)
    u /= np.linalg.norm(u)
    base = 700 * 128 + 100
    for k in range(12):
        lm[base + k] = (0.30 + 0.01 * (k % 9)) * u
    w["lm_head"] = synth.round_to_bf16(lm)
    gm = gu.GpuModel(cfg, w, 256)
    try:
        hid = rng.standard_normal((33, cfg.d_model)).astype(np.float32)
        hid[::2] += 60.0 * u
        g, lg = _check_fused_lattice(gm, gu.to_dev(hid), 33, 8, 0.9, base + 3)
        top = g["cand_id"][0]
        assert np.all((top >= 700 * 128) & (top < 701 * 128)), "row 0 must draw its whole top-8 from the planted run"
        assert not np.any((g["cand_id"][1] >= base) & (g["cand_id"][1] < base + 12))
    finally:
        gm.close()


def test_7b_layer_bf16_prefix2048_k32():
    """7B-shaped layer + LM head, prefix 2048, K = 32 draft rows, 33 verify rows (one model in both roles)."""
    cfg = synth.CFG_7B_LAYER
    w = synth.make_weights(cfg, 0)
    prefix = synth.make_prefix(cfg, 2048, 2)
    flagged = _round_trip(cfg, w, prefix, [11, 12, 13], 32, 32, kv_cap=2048 + 192, seed=4)
    print("near-tie rows flagged:", flagged)


def test_32b_layer_bf16_prefix600_k64():
    """32B-shaped layer (d=5120, 40 query / 8 KV heads, FFN 27648) with a reduced vocabulary (keeps the float64
    oracle quick; the LM-head shape is covered by the 7B test): prefix 600, K = 64, 65 verify rows, and a second
    draft with 48 pending rows + 64 mask rows (112 rows: the seven-row-block GEMM and attention paths)."""
    from dataclasses import replace
    cfg = replace(synth.CFG_32B_LAYER, vocab=16384)
    w = synth.make_weights(cfg, 6)
    prefix = synth.make_prefix(cfg, 600, 7)
    pending = [int(t) for t in synth.make_prefix(cfg, 48, 8)]
    flagged = _round_trip(cfg, w, prefix, pending, 64, 64, kv_cap=896, seed=9)
    print("near-tie rows flagged:", flagged)


def test_argument_errors_with_a_live_model():
    cfg = SMALL_BF16
    w = synth.make_weights(cfg, 30)
    gm = gu.GpuModel(cfg, w, 64)
    try:
        with pytest.raises(ds.DsError) as e:
            gm.draft([1], 64)                       # 65 rows > capacity 64
        assert e.value.code == ds.DS_E_CAPACITY and gm.kv_len == 0
        with pytest.raises(ds.DsError) as e:
            gm.draft([1] * 100, 60)                 # 160 rows > DS_MAX_ROWS
        assert e.value.code == ds.DS_E_SHAPE
        with pytest.raises(ds.DsError) as e:
            gm.set_kv_len(65)
        assert e.value.code == ds.DS_E_CAPACITY
        small_ws = torch.empty(1024, dtype=torch.uint8, device=gu.DEV)
        hid = torch.empty(4, cfg.d_model, dtype=torch.float32, device=gu.DEV)
        with pytest.raises(ds.DsError) as e:
            ds.ds_draft_block(gm.handle, None, 0, 4, cfg.mask_id, hid, small_ws)
        assert e.value.code == ds.DS_E_CAPACITY
    finally:
        gm.close()


@pytest.mark.parametrize("cfg_name", ["f32", "bf16"])
def test_degenerate_row_counts(cfg_name):
    """K = 1 draft with no pending token, and an empty path (m = 0: one verifier row)."""
    cfg = synth.CFG_TINY if cfg_name == "f32" else SMALL_BF16
    tol = TOL[cfg.dtype]
    w = synth.make_weights(cfg, 40)
    prefix = synth.make_prefix(cfg, 70, 41)
    gm = gu.GpuModel(cfg, w, 128)
    try:
        oc = o_model.KVCache(cfg)
        o_model.prefill(cfg, w, oc, prefix)
        gm.prefill(prefix, want_logits=False)
        ref_hid = o_model.draft_block(cfg, w, oc, [], 1)
        hid = gm.draft([], 1)
        logits = gu.from_dev(gm.lm_head(hid))
        assert gm.kv_len == len(prefix)
        assert np.max(np.abs(logits - o_model.lm_head(w, ref_hid))) <= tol
        last = int(prefix[-1])
        ref_v = o_model.verify_logits(cfg, w, oc, [last])
        out = gm.verify(np.array([last], dtype=np.int32), eos_id=cfg.eos_id)
        assert np.max(np.abs(out["logits"] - ref_v)) <= tol
        assert out["n_accept"] == 0 and out["next_token"] == int(out["argmax"][0])
        assert _check_argmax(out["argmax"], ref_v, tol) in (0, 1)
    finally:
        gm.close()
