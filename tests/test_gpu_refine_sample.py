"""GPU parity of the refinement update, the stochastic acceptance rule and whole rounds that use them, through
the C ABI, against the oracle.

Integer outputs are compared exactly wherever both sides decide on the same float32 numbers; where a decision
rests on a sum or a ratio the two sides round differently (float32 on the GPU, float64 in the oracle), a case is
flagged instead of compared when the ORACLE's own margin for that decision is below the stated threshold."""
import numpy as np
import pytest
import torch

from oracle import adl as o_adl
from oracle import refine as o_refine
from oracle import round as o_round
from oracle import sample as o_sample
from paper_2510_02358_amd import binding as ds
from paper_2510_02358_amd import round as rnd
from paper_2510_02358_amd import synth
from tests import gpu_util as gu
from tests import parity_util as pu

pytestmark = pytest.mark.gpu


# ---------------------------------------------------------------------------------------------------
# refinement update on given lattices: bit-exact
# ---------------------------------------------------------------------------------------------------
def test_refine_select_matches_oracle_selection_on_given_lattices():
    rng = np.random.default_rng(0)
    mask_id = 999
    for case in range(60):
        k = int(rng.integers(1, 257)) if case else 256
        m = int(rng.integers(1, 17))
        lat = {"cand_id": rng.integers(0, 900, (k, m)).astype(np.int32),
               "cand_logp": -rng.random((k, m)).astype(np.float32).cumsum(axis=1).astype(np.float32),
               "cand_cnt": rng.integers(1, m + 1, k).astype(np.int32),
               "eos_logp": -rng.random(k).astype(np.float32), "lse": rng.random(k).astype(np.float32)}
        if k > 3:  # plant ties in the confidence
            lat["cand_logp"][rng.integers(0, k, 3), 0] = lat["cand_logp"][0, 0]
        masked = rng.random(k) < 0.6
        block = np.where(masked, mask_id, rng.integers(0, 900, k)).astype(np.int32)
        n = int(rng.integers(0, masked.sum() + 2))
        d = {key: gu.to_dev(v) for key, v in lat.items()}
        blk = gu.to_dev(block)
        out = {key: torch.full_like(v, -7) for key, v in d.items()}
        ds.ds_refine_select(d["cand_id"], d["cand_logp"], d["cand_cnt"], d["eos_logp"], d["lse"], k, m, n, mask_id, blk,
                            out["cand_id"], out["cand_logp"], out["cand_cnt"], out["eos_logp"], out["lse"])
        torch.cuda.synchronize()
        upd = o_refine.select_update(lat["cand_logp"][:, 0], masked, n) if masked.any() and n > 0 else np.array([], int)
        want_block = block.copy()
        want_block[upd] = lat["cand_id"][upd, 0]
        assert np.array_equal(blk.cpu().numpy(), want_block), case
        sel = np.zeros(k, bool)
        sel[upd] = True
        for key in lat:
            got = out[key].cpu().numpy()
            assert np.array_equal(got[sel], lat[key][sel]), (case, key)
            assert np.all(got[~sel] == -7), (case, key)          # untouched rows stay untouched


# ---------------------------------------------------------------------------------------------------
# stochastic acceptance on given logits
# ---------------------------------------------------------------------------------------------------
def _pick_margin(weights, u, chosen):
    """Oracle-side distance (relative to the total) between the draw's target and the nearest boundary of the
    chosen token's cumulative interval."""
    total = float(weights.sum())
    c = np.cumsum(weights)
    target = u * total
    lo = c[chosen] - weights[chosen]
    return min(abs(target - lo), abs(c[chosen] - target)) / total


def _run_gpu_accept(p, q, block, path_len, u, eos_id):
    m, vocab = q.shape[0], p.shape[1]
    out = torch.zeros(3, dtype=torch.int32, device=gu.DEV)
    alpha = torch.zeros(max(m, 1), dtype=torch.float32, device=gu.DEV)
    ws = torch.empty(ds.ds_sample_workspace_bytes(m), dtype=torch.uint8, device=gu.DEV)
    pl = gu.to_dev(np.array([path_len], np.int32)) if path_len is not None else None
    qd = gu.to_dev(q) if m else None
    ds.ds_accept_stochastic(gu.to_dev(p), qd, m, vocab, gu.to_dev(block), pl, gu.to_dev(u), eos_id, out[0:1], out[1:2],
                            out[2:3], alpha if m else None, ws)
    torch.cuda.synchronize()
    o = out.cpu().numpy()
    return int(o[0]), int(o[1]), int(o[2]), alpha.cpu().numpy()[:m]


@pytest.mark.parametrize("vocab", [37, 1003, 4096, 152064])
def test_accept_stochastic_matches_oracle_on_identical_logits(vocab):
    rng = np.random.default_rng(vocab)
    n_cases = 8 if vocab > 100000 else 40
    flagged = compared = 0
    for case in range(n_cases):
        m = int(rng.integers(0, 9)) if case else 8
        temp = float(rng.uniform(0.5, 3.0))
        p = (rng.standard_normal((m + 1, vocab)) * temp).astype(np.float32)
        q = (p[:m] + rng.standard_normal((m, vocab)).astype(np.float32) * float(rng.uniform(0.05, 1.0))).astype(np.float32)
        path = np.array([int(np.argmax(q[i])) if rng.random() < 0.7 else int(rng.integers(0, vocab)) for i in range(m)],
                        dtype=np.int32)
        eos_id = int(path[0]) if (m and case % 5 == 0) else -1
        path_len = None if case % 3 else int(rng.integers(0, m + 1))
        block = np.concatenate([[3 % vocab], path]).astype(np.int32)
        u = rng.random(m + 1).astype(np.float32)
        if case % 7 == 3 and m:
            u[: m // 2] = 0.0                                         # force a long accepted prefix
        m_eff = m if path_len is None else min(m, path_len)
        r_acc, r_next, r_eos, r_alpha = o_sample.verify_stochastic(p[: m_eff + 1], q[:m_eff], path[:m_eff], u[:m_eff],
                                                                   float(u[m]), eos_id)
        g_acc, g_next, g_eos, g_alpha = _run_gpu_accept(p, q, block, path_len, u, eos_id)
        full_alpha = np.array([o_sample.acceptance_probability(p[i], q[i], int(path[i])) for i in range(m)])
        assert np.allclose(g_alpha, full_alpha, rtol=2e-4, atol=1e-7), case
        if np.any(np.abs(u[:m_eff] - r_alpha) < 1e-4 * np.maximum(r_alpha, 1e-3)):
            flagged += 1
            continue
        assert g_acc == r_acc, (case, g_acc, r_acc)
        pr = o_sample.softmax64(p[r_acc])
        weights = np.maximum(pr - o_sample.softmax64(q[r_acc]), 0.0) if r_acc < m_eff else pr
        # float32 sums over the vocabulary carry ~1e-6 of the total; a target closer than 5e-6 to an edge of the
        # chosen token's interval may legitimately land on the neighbouring token
        if _pick_margin(weights, float(u[m]), r_next) < 5e-6:
            flagged += 1
            continue
        compared += 1
        assert (g_next, g_eos) == (r_next, r_eos), (case, g_next, r_next)
    print(f"vocab {vocab}: compared {compared}, flagged {flagged}")
    assert compared >= n_cases // 2


def test_accept_stochastic_edge_cases():
    rng = np.random.default_rng(5)
    vocab = 513
    p = rng.standard_normal((4, vocab)).astype(np.float32)
    path = np.array([7, 8, 9], np.int32)
    block = np.concatenate([[1], path]).astype(np.int32)
    # drafter == verifier: alpha = 1 everywhere; u < 1 accepts all, the bonus comes from the last row
    u = np.array([0.999, 0.5, 0.0, 0.25], np.float32)
    acc, nxt, eos, alpha = _run_gpu_accept(p, p[:3].copy(), block, None, u, -1)
    assert acc == 3 and np.all(alpha == 1.0)
    assert nxt == o_sample.inverse_cdf(o_sample.softmax64(p[3]), 0.25)
    # u = 1 rejects even alpha = 1; the residual is empty, so the draw falls back to the verifier row
    u = np.array([1.0, 0.5, 0.0, 0.6], np.float32)
    acc, nxt, eos, _ = _run_gpu_accept(p, p[:3].copy(), block, None, u, -1)
    assert acc == 0 and nxt == o_sample.inverse_cdf(o_sample.softmax64(p[0]), 0.6)
    # empty path: only the draw from row 0; u = 0 picks the first token
    acc, nxt, eos, _ = _run_gpu_accept(p[:1], np.zeros((0, vocab), np.float32), block[:1], None,
                                       np.array([0.0], np.float32), 0)
    assert (acc, nxt, eos) == (0, 0, 1)
    # path_len = 0 behaves like the empty path although m = 3
    acc, nxt, eos, _ = _run_gpu_accept(p, p[:3].copy(), block, 0, np.array([0., 0., 0., 0.0], np.float32), -1)
    assert (acc, nxt) == (0, 0)
    # a one-hot verifier row: the draw returns that token for any uniform
    hot = np.full((1, vocab), -80.0, np.float32)
    hot[0, 300] = 40.0
    for uu in (0.0, 0.5, 0.999999):
        acc, nxt, _, _ = _run_gpu_accept(hot, np.zeros((0, vocab), np.float32), block[:1], None,
                                         np.array([uu], np.float32), -1)
        assert nxt == 300
    # host-side argument checks
    lib = ds.load()
    one = torch.zeros(4, dtype=torch.int32, device=gu.DEV).data_ptr()
    assert lib.ds_accept_stochastic(one, one, -1, 10, one, None, one, -1, one, one, one, one, one, 1024, None) == ds.DS_E_SHAPE
    assert lib.ds_accept_stochastic(one, None, 2, 10, one, None, one, -1, one, one, one, one, one, 1024, None) == ds.DS_E_INVALID
    assert lib.ds_accept_stochastic(one, one, 2, 10, one, None, one, -1, one, one, one, one, one, 8, None) == ds.DS_E_CAPACITY


# ---------------------------------------------------------------------------------------------------
# refinement, pass by pass (every pass compared on identical block contents)
# ---------------------------------------------------------------------------------------------------
TOL = 1e-4


@pytest.mark.parametrize("steps,k", [(2, 8), (3, 11), (8, 8), (4, 16)])
def test_refinement_passes_match_oracle_pass_by_pass(steps, k):
    """Each drafter pass of a refinement through the C ABI (ds_draft_block_tokens, ds_draft_lattice,
    ds_refine_select) against the oracle's pass on the same block contents: logits to 1e-4; lattice rows exact
    except rows flagged on their own near-tie; the update set exactly the oracle's selection rule applied to the
    GPU's confidences, and equal to the oracle's own set unless a deviating position's confidence is within the
    tolerance of the selection boundary; frozen rows are the rows of the pass that fixed them."""
    from oracle import lattice as o_lat
    from oracle import model as o_model
    cfg = synth.CFG_TINY
    w = synth.make_weights(cfg, 0)
    prefix = synth.make_prefix(cfg, 96, 2)
    m_max, tau, eos, mask_id = 4, 0.9, cfg.eos_id, cfg.mask_id
    gm = gu.GpuModel(cfg, w, 256)
    flagged_rows = flagged_sel = 0
    try:
        oc = o_model.KVCache(cfg)
        pending = [int(np.argmax(o_model.prefill(cfg, w, oc, prefix)))]
        gm.prefill(prefix, want_logits=False)
        block = np.full(k, mask_id, np.int32)
        blk = gu.to_dev(block)
        names = ("cand_id", "cand_logp", "cand_cnt", "eos_logp", "lse")
        frozen = {"cand_id": torch.full((k, m_max), -7, dtype=torch.int32, device=gu.DEV),
                  "cand_logp": torch.full((k, m_max), -7.0, device=gu.DEV),
                  "cand_cnt": torch.full((k,), -7, dtype=torch.int32, device=gu.DEV),
                  "eos_logp": torch.full((k,), -7.0, device=gu.DEV), "lse": torch.full((k,), -7.0, device=gu.DEV)}
        want_frozen = {n: frozen[n].cpu().numpy().copy() for n in names}
        hidden = torch.empty(k, cfg.d_model, dtype=torch.float32, device=gu.DEV)
        sizes = ds.ds_refine_update_sizes(k, steps)
        assert sizes == o_refine.update_sizes(k, steps)
        for s, n in enumerate(sizes):
            pend = gu.to_dev(np.asarray(pending, np.int32)) if s == 0 else None
            ds.ds_draft_block_tokens(gm.handle, pend, len(pending) if s == 0 else 0, blk, k, hidden, gm.ws)
            lat_g, logits_g = gm.draft_lattice(None, k, m_max, tau, eos, want_logits=True)
            y = o_model.draft_block(cfg, w, oc, pending if s == 0 else [], k, block_tokens=block)
            ref_logits = o_model.lm_head(w, y)
            assert np.max(np.abs(gu.from_dev(logits_g) - ref_logits)) <= TOL, s
            ref_lat = o_lat.build_lattice(ref_logits, m_max, tau, eos)
            g = {n: gu.from_dev(lat_g[n]) for n in names}
            flagged_rows += len(pu.lattice_rows_flagged(g["cand_id"], ref_lat["cand_id"], ref_logits, TOL))
            assert np.max(np.abs(g["cand_logp"] - ref_lat["cand_logp"])) <= 3 * TOL
            masked = block == mask_id
            ds.ds_refine_select(*[lat_g[n] for n in names], k, m_max, n, mask_id, blk, *[frozen[n] for n in names])
            torch.cuda.synchronize()
            upd = o_refine.select_update(g["cand_logp"][:, 0], masked, n)        # the rule on the GPU's own numbers
            upd_ref = o_refine.select_update(ref_lat["cand_logp"][:, 0], masked, n)
            if list(upd) != list(upd_ref):
                conf = ref_lat["cand_logp"][:, 0].astype(np.float64)
                boundary = np.sort(conf[masked])[::-1][n - 1]                   # the n-th largest confidence
                for pos in set(upd) ^ set(upd_ref):
                    assert abs(conf[pos] - boundary) < 4 * TOL, (s, pos)
                flagged_sel += 1
            block = block.copy()
            block[upd] = g["cand_id"][upd, 0]
            assert np.array_equal(blk.cpu().numpy(), block), s
            for name in names:
                want_frozen[name][upd] = g[name][upd]
                assert np.array_equal(frozen[name].cpu().numpy(), want_frozen[name]), (s, name)
        assert not np.any(block == mask_id) and len(sizes) == min(steps, k)
        print(f"PARITY-COUNTS refinement passes S={steps} K={k}: passes {len(sizes)}, lattice rows flagged "
              f"{flagged_rows}, selections flagged {flagged_sel}")
        assert flagged_rows <= 1 and flagged_sel <= 1
    finally:
        gm.close()


# ---------------------------------------------------------------------------------------------------
# whole rounds on the tiny float32 pair
# ---------------------------------------------------------------------------------------------------


def _setup(params, k_cap=16):
    cfg = synth.CFG_TINY
    dw, vw = synth.make_weights(cfg, 0), synth.make_weights(cfg, 1)
    prefix = synth.make_prefix(cfg, 96, 2)
    table = synth.make_ngram_table(3)
    dm, vm = rnd.DeviceModel(cfg, dw, 256), rnd.DeviceModel(cfg, vw, 256)
    dec = rnd.SpecDecoder(dm, vm, table, synth.NGRAM_LOG2_SIZE, params, k_cap=k_cap, keep_verify_logits=True)
    dec.start(prefix)
    st = o_round.SpecState(cfg, dw, cfg, vw, prefix)
    assert dec.tokens == st.tokens
    return cfg, dec, st, table, dm, vm


@pytest.mark.parametrize("steps", [2, 3, 8])
def test_refinement_rounds_match_oracle(steps):
    m_max, beam, lam, tau = 4, 3, 0.5, 0.9
    params = rnd.RoundParams(m_max=m_max, tau=tau, beam=beam, lam=lam, k_min=2, k_max=12, delta=2.0, rho=0.5,
                             refine_steps=steps)
    cfg, dec, st, table, dm, vm = _setup(params)
    try:
        adl = o_adl.AdlState(params.k_min, params.k_max, params.delta, params.rho)
        k, compared = 8, 0
        for t in range(4):
            got = dec.round(k)
            # the oracle's refinement once more with one extra candidate per row (same passes, same selection):
            # it shows the value just below each row's top-M, which the near-tie rule below needs
            wide, _, _ = o_refine.refine_block(cfg, st.dw, st.dcache.copy(), list(st.pending), k, steps, m_max + 1,
                                               1.0, cfg.eos_id)
            ref = o_round.spec_round(st, k, m_max, tau, beam, lam, table, synth.NGRAM_LOG2_SIZE, refine_steps=steps)
            k_ref = o_adl.adl_update(adl, k, ref["first_eos"], ref["n_accept"])
            lat = ref["lattice"]
            g_logp = dec.f_cand_logp[:k].cpu().numpy()
            same = (np.array_equal(dec.f_cand_id[:k].cpu().numpy(), lat["cand_id"])
                    and np.array_equal(dec.blk[:k].cpu().numpy(), lat["cand_id"][:, 0])
                    and list(got["path"]) == ref["path"] and got["n_accept"] == ref["n_accept"]
                    and got["next_token"] == ref["next_token"])
            if not same:
                # Later passes see what earlier passes fixed, so one flipped decision changes many rows; but it must
                # start in a row that deviates, on that row's own near-tie: two of its neighbouring candidate values
                # (the one below the top-M included) or its confidence and another row's within twice the tolerance.
                g_ids, g_blk = dec.f_cand_id[:k].cpu().numpy(), dec.blk[:k].cpu().numpy()
                dev = np.nonzero(np.any(g_ids != lat["cand_id"], axis=1) | (g_blk != lat["cand_id"][:, 0]))[0]
                conf = wide["cand_logp"][:, 0].astype(np.float64)
                origin = []
                for r in dev:
                    row_gap = np.min(-np.diff(wide["cand_logp"][r].astype(np.float64)))
                    conf_gap = np.min(np.abs(np.delete(conf, r) - conf[r])) if k > 1 else np.inf
                    if row_gap < 2 * TOL or conf_gap < 2 * TOL:
                        origin.append(int(r))
                assert len(dev) == 0 or origin, f"round {t}: rows {list(dev)} deviate, none on a near-tie of its own"
                if len(dev) == 0:   # identical lattices and drafts: only the verifier can have decided differently
                    assert list(got["path"]) == ref["path"]
                    pu.argmax_rows_flagged(dec.argmax[:len(ref["path"]) + 1].cpu().numpy(), ref["v_logits"], TOL)
                print(f"PARITY-COUNTS refinement rounds S={steps}: stopped at round {t}, origin rows {origin}")
                break
            assert np.max(np.abs(g_logp - lat["cand_logp"])) <= 2 * TOL
            assert np.array_equal(dec.f_cand_cnt[:k].cpu().numpy(), lat["cand_cnt"])
            assert got["k_next"] == k_ref and dec.tokens == st.tokens
            assert dec.d.kv_len == st.dcache.length and dec.v.kv_len == st.vcache.length
            compared += 1
            k = k_ref
        print(f"PARITY-COUNTS refinement rounds S={steps}: rounds fully compared {compared} of 4")
        assert compared >= 3
    finally:
        dec.close(); dm.close(); vm.close()


def test_stochastic_rounds_match_oracle():
    m_max, beam, lam, tau = 4, 3, 0.5, 0.9
    params = rnd.RoundParams(m_max=m_max, tau=tau, beam=beam, lam=lam, k_min=2, k_max=12, delta=2.0, rho=0.5)
    cfg, dec, st, table, dm, vm = _setup(params)
    rng = np.random.default_rng(11)
    try:
        adl = o_adl.AdlState(params.k_min, params.k_max, params.delta, params.rho)
        k, compared = 8, 0
        counts = pu.new_counts()
        for t in range(8):
            u = rng.random(k + 1).astype(np.float32)
            u[: t % 4] = 0.0                      # vary how far acceptance gets (alpha > 0 always accepts u = 0)
            got = dec.round(k, uniforms=u)
            # draft stage decision by decision (a differing path must sit on a near-tie of its own and is then
            # verified on the oracle too, so the acceptance rule is compared either way)
            ref = pu.compare_round(dec, st, got, k, params, table, TOL, counts, uniforms=u)
            k_ref = o_adl.adl_update(adl, k, got["first_eos"], ref["n_accept"])
            m_eff = len(ref["path"])
            assert list(got["path"]) == ref["path"]
            g_alpha = dec.alpha[:m_eff].cpu().numpy()
            assert np.allclose(g_alpha, ref["alpha"], rtol=5e-3, atol=1e-6)
            L = ref["n_accept"]
            pr = o_sample.softmax64(ref["v_logits"][L])
            w = np.maximum(pr - o_sample.softmax64(ref["d_logits"][L]), 0.0) if L < m_eff else pr
            # decisions within the two sides' logit noise (1e-4) of flipping: a uniform next to its acceptance
            # probability, or a draw target next to an edge of the chosen token's cumulative interval
            fragile = (np.any(np.abs(u[:m_eff] - ref["alpha"]) < 1e-2 * np.maximum(ref["alpha"], 1e-3))
                       or _pick_margin(w, float(u[k]), ref["next_token"]) < 2e-5)
            same = (got["n_accept"] == ref["n_accept"] and got["next_token"] == ref["next_token"]
                    and got["eos_accepted"] == ref["eos_accepted"])
            if not same:
                assert fragile, f"round {t}: outputs differ without a fragile decision"
                break
            assert got["k_next"] == k_ref and dec.tokens == st.tokens
            assert dec.v.kv_len == st.vcache.length
            compared += 1
            k = k_ref
        print(f"PARITY-COUNTS stochastic rounds: compared {compared} of 8, {counts}")
        assert compared >= 6
    finally:
        dec.close(); dm.close(); vm.close()
