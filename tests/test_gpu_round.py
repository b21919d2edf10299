"""GPU parity of whole rounds: the speculative loop driven through the C ABI vs the oracle loop on the tiny
float32 pair, plus the lossless invariant (committed stream == verifier's greedy decode).

End to end the two sides compute their own logits, so integer outputs can only be required to agree when
no decision sits on a float32 near-tie; such rows are detected from the ORACLE's logits and flagged."""
import numpy as np
import pytest
import torch

from oracle import adl as o_adl
from oracle import round as o_round
from paper_2510_02358_amd import round as rnd
from paper_2510_02358_amd import synth

import parity_util as pu

pytestmark = pytest.mark.gpu

TOL = 1e-4


@pytest.mark.parametrize("lam,tau", [(0.5, 1.0), (1.0, 0.8), (0.3, 0.9)])
def test_tiny_pair_rounds_match_oracle_and_are_lossless(lam, tau, record_property):
    cfg = synth.CFG_TINY
    dw, vw = synth.make_weights(cfg, 0), synth.make_weights(cfg, 1)
    prefix = synth.make_prefix(cfg, 128, 2)
    table = synth.make_ngram_table(3)
    m_max, beam, n_rounds, k1 = 4, 4, 6, 8
    params = rnd.RoundParams(m_max=m_max, tau=tau, beam=beam, lam=lam, k_min=2, k_max=12, delta=2.0, rho=0.5)
    dm, vm = rnd.DeviceModel(cfg, dw, 256), rnd.DeviceModel(cfg, vw, 256)
    dec = rnd.SpecDecoder(dm, vm, table, synth.NGRAM_LOG2_SIZE, params, k_cap=16, keep_draft_logits=True,
                          keep_verify_logits=True)
    counts = pu.new_counts()
    try:
        dec.start(prefix)
        st = o_round.SpecState(cfg, dw, cfg, vw, prefix)
        assert dec.tokens == st.tokens
        adl = o_adl.AdlState(params.k_min, params.k_max, params.delta, params.rho)
        k = k1
        for t in range(n_rounds):
            got = dec.round(k)
            ref = pu.compare_round(dec, st, got, k, params, table, TOL, counts)
            if ref is None:
                break
            counts["rounds"] += 1
            k_ref = o_adl.adl_update(adl, k, got["first_eos"], ref["n_accept"])
            assert got["k_next"] == k_ref
            assert dec.tokens == st.tokens
            assert dm.kv_len == st.dcache.length and vm.kv_len == st.vcache.length
            k = k_ref
        print("PARITY-COUNTS tiny rounds", (lam, tau), counts)
        record_property("parity_counts", counts)
        assert counts["rounds"] >= n_rounds - 1, counts
        assert counts["lattice_rows_flagged"] <= 2 and counts["verifier_rows_flagged"] <= 1, counts
        # lossless: whatever was committed is the verifier's own greedy continuation (GPU verifier vs oracle decode)
        produced = dec.tokens[len(prefix):]
        ref_stream = o_round.ar_greedy(cfg, vw, prefix, len(produced))
        if counts["verifier_rows_flagged"] == 0:
            assert produced == ref_stream
    finally:
        dec.close(); dm.close(); vm.close()


def test_bf16_rounds_do_not_depend_on_the_logits_being_written():
    """Two decoders on the same small bf16 pair, one keeping the drafter's logits in memory and one not (the lattice
    then comes from the LM-head product's tile records alone), walk through the same rounds with identical lattices,
    paths and verdicts; and the lattice is the oracle's lattice of the logits the first decoder kept."""
    from oracle import lattice as o_lat
    cfg = synth.ModelCfg(n_layers=2, d_model=256, n_q=4, n_kv=2, head_dim=128, d_ffn=512, vocab=4096,
                         rope_base=1.0e6, dtype="bf16")
    dw, vw = synth.make_weights(cfg, 10), synth.make_weights(cfg, 11)
    prefix = synth.make_prefix(cfg, 100, 12)
    table = synth.make_ngram_table(3)
    params = rnd.RoundParams(m_max=8, tau=0.95, beam=4, lam=0.5, k_min=4, k_max=32, delta=2.0, rho=0.5)
    models = [rnd.DeviceModel(cfg, w, 512) for w in (dw, vw, dw, vw)]
    a = rnd.SpecDecoder(models[0], models[1], table, synth.NGRAM_LOG2_SIZE, params, k_cap=32, keep_draft_logits=True)
    b = rnd.SpecDecoder(models[2], models[3], table, synth.NGRAM_LOG2_SIZE, params, k_cap=32)
    try:
        a.start(prefix)
        b.start(prefix)
        k = 21
        for t in range(6):
            ga, gb = a.round(k), b.round(k)
            for name in ("cand_id", "cand_logp", "cand_cnt", "eos_logp", "lse"):
                assert torch.equal(getattr(a, name)[:k], getattr(b, name)[:k]), (t, name)
            assert list(ga["path"]) == list(gb["path"]) and ga["n_accept"] == gb["n_accept"]
            assert ga["next_token"] == gb["next_token"] and ga["k_next"] == gb["k_next"]
            assert a.tokens == b.tokens
            ref = o_lat.build_lattice(a.d_logits[:k].cpu().numpy(), params.m_max, params.tau, cfg.eos_id)
            assert np.array_equal(a.cand_id[:k].cpu().numpy(), ref["cand_id"])
            assert np.array_equal(a.cand_cnt[:k].cpu().numpy(), ref["cand_cnt"])
            k = ga["k_next"]
    finally:
        a.close(); b.close()
        for m in models:
            m.close()


def test_forced_greedy_path_is_fully_accepted_on_gpu():
    """A draft equal to the verifier's own greedy continuation is accepted in full (GPU verifier)."""
    from paper_2510_02358_amd import binding as ds
    cfg = synth.CFG_TINY
    vw = synth.make_weights(cfg, 1)
    prefix = synth.make_prefix(cfg, 100, 5)
    k = 7
    greedy = o_round.ar_greedy(cfg, vw, prefix, k + 2)
    vm = rnd.DeviceModel(cfg, vw, 128)
    try:
        t = rnd.upload(np.asarray(prefix, dtype=np.int32))
        ds.ds_prefill(vm.handle, t, len(prefix), None, vm.ws)
        block = rnd.upload(np.asarray(greedy[: k + 1], dtype=np.int32))
        res = torch.zeros(3, dtype=torch.int32, device=rnd.DEV)
        am = torch.empty(k + 1, dtype=torch.int32, device=rnd.DEV)
        ds.ds_verify_block(vm.handle, block, k, None, cfg.eos_id, res[0:1], res[1:2], am, res[2:3], None, vm.ws)
        r = res.cpu().numpy()
        assert r[0] == k and r[1] == greedy[k + 1]
        assert list(am.cpu().numpy()) == greedy[1: k + 2]
        # path_len on the device limits acceptance
        pl = rnd.upload(np.array([3], dtype=np.int32))
        ds.ds_verify_block(vm.handle, block, k, pl, cfg.eos_id, res[0:1], res[1:2], am, res[2:3], None, vm.ws)
        r = res.cpu().numpy()
        assert r[0] == 3 and r[1] == greedy[4]
    finally:
        vm.close()


@pytest.mark.parametrize("cfg_name", ["f32", "bf16"])
def test_verify_carry_leaves_the_next_rounds_inputs_on_the_device(cfg_name):
    """ds_verify_block_carry returns what ds_verify_block returns and writes the committed tokens, right-aligned,
    the token before the last one and the last one into its carry buffer (nothing else of it), for no / some / all
    path tokens accepted and for a path cut by path_len; float32 model (arg-max scan) and bf16 model (per-tile
    records).  Then whole rounds: after every round of the driver, the device holds exactly what the host would
    have staged."""
    from paper_2510_02358_amd import binding as ds
    cfg = synth.CFG_TINY if cfg_name == "f32" else synth.ModelCfg(
        n_layers=2, d_model=256, n_q=4, n_kv=2, head_dim=128, d_ffn=512, vocab=4096, rope_base=1.0e6, dtype="bf16")
    dw, vw = synth.make_weights(cfg, 0), synth.make_weights(cfg, 1)
    prefix = synth.make_prefix(cfg, 90, 11)
    k, P = 6, ds.DS_MAX_ROWS
    dm, vm = rnd.DeviceModel(cfg, dw, 256), rnd.DeviceModel(cfg, vw, 256)
    dec = None
    try:
        ds.ds_prefill(vm.handle, rnd.upload(np.asarray(prefix, dtype=np.int32)), len(prefix), None, vm.ws)
        res = torch.zeros(3, dtype=torch.int32, device=rnd.DEV)
        am = torch.empty(k + 1, dtype=torch.int32, device=rnd.DEV)

        def plain(block, pl):
            ds.ds_verify_block(vm.handle, rnd.upload(block), k, pl, cfg.eos_id, res[0:1], res[1:2], am, res[2:3],
                               None, vm.ws)
            torch.cuda.synchronize()
            return res.cpu().numpy().copy(), am.cpu().numpy().copy()

        # the verifier's own greedy chain after the prefix's last token, one more settled position per call
        chain = np.full(k + 1, 3, dtype=np.int32)
        chain[0] = prefix[-1]
        for i in range(k):
            chain[i + 1] = plain(chain, None)[1][i]
        cases = []
        for n_keep, pl in ((k, None), (3, None), (0, None), (k, 2)):
            block = chain.copy()
            if n_keep < k:
                block[n_keep + 1] = (block[n_keep + 1] + 1) % cfg.n_plain_tokens      # first rejected position
            cases.append((block, pl))
        for block, pl in cases:
            pl_dev = rnd.upload(np.array([pl], dtype=np.int32)) if pl is not None else None
            want, want_am = plain(block, pl_dev)
            n, nxt = int(want[0]), int(want[1])
            assert n == (pl if pl is not None else int(np.sum(np.cumprod(block[1:] == chain[1:]))))
            carry = torch.full((P + 2,), -7, dtype=torch.int32, device=rnd.DEV)
            res.zero_(); am.zero_()
            ds.ds_verify_block_carry(vm.handle, rnd.upload(block), k, pl_dev, cfg.eos_id, res[0:1], res[1:2], am,
                                     res[2:3], None, carry, vm.ws)
            torch.cuda.synchronize()
            assert np.array_equal(res.cpu().numpy(), want) and np.array_equal(am.cpu().numpy(), want_am)
            c = carry.cpu().numpy()
            assert np.all(c[:P - 1 - n] == -7)
            assert list(c[P - 1 - n:P]) == list(block[1:1 + n]) + [nxt]
            assert c[P] == (block[n] if n > 0 else block[0]) and c[P + 1] == nxt
            # the driver's layout: the block starts at the carry buffer's last word
            io = torch.full((P + 2 + k,), -7, dtype=torch.int32, device=rnd.DEV)
            io[P + 1:] = rnd.upload(block)
            ds.ds_verify_block_carry(vm.handle, io[P + 1:], k, pl_dev, cfg.eos_id, res[0:1], res[1:2], am, res[2:3],
                                     None, io, vm.ws)
            torch.cuda.synchronize()
            assert np.array_equal(res.cpu().numpy(), want)
            assert np.array_equal(io[:P + 2].cpu().numpy(), c)
            assert np.array_equal(io[P + 2:].cpu().numpy(), block[1:])
        with pytest.raises(ds.DsError) as e:
            ds.ds_verify_block_carry(vm.handle, rnd.upload(chain), k, None, cfg.eos_id, res[0:1], res[1:2], am,
                                     res[2:3], None, None, vm.ws)
        assert e.value.code == ds.DS_E_INVALID

        # whole rounds, some of them with part of the path overwritten by the verifier's chain (accepted tokens)
        vm.set_kv_len(0)
        params = rnd.RoundParams(m_max=4, tau=0.9, beam=4, lam=0.5, k_min=2, k_max=12, delta=2.0, rho=0.5)
        dec = rnd.SpecDecoder(dm, vm, synth.make_ngram_table(3), synth.NGRAM_LOG2_SIZE, params, k_cap=16)
        dec.start(prefix)
        staged = 0
        for t in range(5):
            inject = None
            if t in (1, 3) and cfg_name == "f32":
                # tokens the verifier will accept: its greedy continuation of the committed stream
                nxt_tokens = o_round.ar_greedy(cfg, vw, dec.tokens, 3)
                inject = (rnd.upload(np.asarray(nxt_tokens, dtype=np.int32)), 2)
            was_carried = dec._carried
            got = dec.round(8, inject=inject)
            staged += 0 if was_carried else 1
            n_p = len(dec.pending)
            io = dec.io[:P + 2].cpu().numpy()
            assert dec._carried and n_p == got["n_accept"] + 1
            assert list(io[P - n_p:P]) == dec.pending
            assert io[P] == dec.tokens[-2] and io[P + 1] == dec.tokens[-1]
            if inject is not None:
                assert got["n_accept"] >= 2
        assert staged == 1          # the first round only
    finally:
        if dec is not None:
            dec.close()
        dm.close(); vm.close()


@pytest.mark.parametrize("cfg_name", ["f32", "bf16"])
def test_library_round_loop_equals_the_round_by_round_driver(cfg_name):
    """ds_rounds_run (the loop inside the library) against SpecDecoder.round() called round by round on the same
    models: the same verdicts, first-EOS indices, draft-length proposals, committed tokens and cache lengths, also
    when the two ways of driving alternate, and with the event pairs around the LM head switched on."""
    cfg = synth.CFG_TINY if cfg_name == "f32" else synth.ModelCfg(
        n_layers=2, d_model=256, n_q=4, n_kv=2, head_dim=128, d_ffn=512, vocab=4096, rope_base=1.0e6, dtype="bf16")
    dw, vw = synth.make_weights(cfg, 0), synth.make_weights(cfg, 1)
    prefix = synth.make_prefix(cfg, 100, 13)
    table = synth.make_ngram_table(3)
    params = rnd.RoundParams(m_max=4, tau=0.9, beam=4, lam=0.5, k_min=2, k_max=12, delta=2.0, rho=0.5)
    dm, vm = rnd.DeviceModel(cfg, dw, 256), rnd.DeviceModel(cfg, vw, 256)
    keys = ("k", "path_len", "n_accept", "next_token", "eos_accepted", "first_eos", "k_next", "committed")
    try:
        a = rnd.SpecDecoder(dm, vm, table, synth.NGRAM_LOG2_SIZE, params, k_cap=16)
        a.start(prefix)
        want, k = [], 8
        for _ in range(7):
            got = a.round(k)
            want.append({n: (list(got[n]) if n == "committed" else int(got[n])) for n in keys})
            k = got["k_next"]
        want_tokens, want_len = list(a.tokens), (dm.kv_len, vm.kv_len)
        a.close()

        b = rnd.SpecDecoder(dm, vm, table, synth.NGRAM_LOG2_SIZE, params, k_cap=16)
        b.start(prefix)
        got = b.run(2, 8)                                  # two rounds in the library's loop,
        one = b.round(got[-1]["k_next"])                   # one by hand,
        got.append({n: (list(one[n]) if n == "committed" else int(one[n])) for n in keys})
        pairs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(2)]
        for e0, e1 in pairs:
            e0.record(); e1.record()
        torch.cuda.synchronize()
        got += b.run(4, got[-1]["k_next"], lm_events=(2, pairs))   # and four more, two of them with events
        torch.cuda.synchronize()
        assert all(e0.elapsed_time(e1) > 0.0 for e0, e1 in pairs)
        assert [{n: r[n] for n in keys} for r in got] == want
        assert b.tokens == want_tokens and (dm.kv_len, vm.kv_len) == want_len
        assert b.pending == want[-1]["committed"]
        # a fixed draft length, and stopping at an accepted EOS (none here: all rounds run)
        b.start(prefix)
        fixed = b.run(3, 6, follow_adl=False, stop_at_eos=True)
        assert [r["k"] for r in fixed] == [6, 6, 6] and len(fixed) == 3
        b.close()
    finally:
        dm.close(); vm.close()


def _successor_pair(cfg, succ: dict, seed: int):
    """A drafter / verifier pair whose next token depends on the current token alone and is PLANTED for the tokens in
    `succ`: the layers contribute nothing (zero output projections), so the final state is the token's embedding, and
    the LM-head row of succ[t] carries a large multiple of the normalised embedding of t."""
    w = synth.make_weights(cfg, seed)
    for lw in w["layers"]:
        lw["wo"][:] = 0.0
        lw["w_down"][:] = 0.0
    for t, nxt in succ.items():
        e = w["embed"][t].astype(np.float64)
        y = e / np.sqrt(np.mean(e * e) + cfg.rms_eps)
        w["lm_head"][nxt] += (8.0 * y / np.sqrt(cfg.d_model)).astype(np.float32)
    return w


@pytest.mark.parametrize("case", ["all-accepted", "one-accepted"])
def test_library_round_loop_with_accepted_tokens_on_a_planted_successor_model(case):
    """Rounds that DO accept draft tokens, through both loop drivers, on a pair whose behaviour is known by
    construction.  The drafter fills every masked position with token 7 (the planted successor of [MASK]); the
    verifier follows the planted successors 5 -> 7 and either 7 -> 7 (every draft token accepted, K + 1 committed per
    round) or 7 -> 9 -> 7 (exactly one accepted, next token 9).  Pending counts above one, the carried tokens, the
    committed streams and the controller's proposals must agree between the library's loop and the round-by-round
    driver, and with these hand-derived verdicts."""
    cfg = synth.CFG_TINY
    succ = {cfg.mask_id: 7, 5: 7, 7: 7 if case == "all-accepted" else 9, 9: 7}
    prefix = np.concatenate([synth.make_prefix(cfg, 60, 14), [31]]).astype(np.int32)
    succ[31] = 5                                       # the verifier's first token after the prefix
    w = _successor_pair(cfg, succ, 20)
    params = rnd.RoundParams(m_max=4, tau=1.0, beam=2, lam=1.0, k_min=2, k_max=8, delta=2.0, rho=0.5)
    dm, vm = rnd.DeviceModel(cfg, w, 256), rnd.DeviceModel(cfg, w, 256)
    k = 6
    try:
        a = rnd.SpecDecoder(dm, vm, None, 0, params, k_cap=8)
        a.start(prefix)
        assert a.tokens[-1] == 5
        by_hand = [a.round(k) for _ in range(4)]
        tokens_by_hand = list(a.tokens)
        a.close()
        for t, r in enumerate(by_hand):
            assert list(r["path"]) == [7] * k
            if case == "all-accepted":
                assert (r["n_accept"], r["next_token"]) == (k, 7) and r["committed"] == [7] * (k + 1)
            else:
                assert (r["n_accept"], r["next_token"]) == (1, 9) and r["committed"] == [7, 9]
        b = rnd.SpecDecoder(dm, vm, None, 0, params, k_cap=8)
        b.start(prefix)
        in_lib = b.run(4, k, follow_adl=False, stop_at_eos=False)
        for r, q in zip(in_lib, by_hand):
            for n in ("k", "path_len", "n_accept", "next_token", "eos_accepted", "first_eos", "k_next"):
                assert r[n] == q[n], n
            assert r["committed"] == q["committed"]
        assert b.tokens == tokens_by_hand and len(b.pending) == (k + 1 if case == "all-accepted" else 2)
        # the controller's proposals followed: rounds of different K and pending counts (fresh controllers)
        b.close()
        b = rnd.SpecDecoder(dm, vm, None, 0, params, k_cap=8)
        b.start(prefix)
        followed = b.run(5, 4)
        a = rnd.SpecDecoder(dm, vm, None, 0, params, k_cap=8)
        a.start(prefix)
        kk = 4
        for r in followed:
            q = a.round(kk)
            assert (r["k"], r["n_accept"], r["next_token"], r["k_next"]) == (kk, q["n_accept"], q["next_token"], q["k_next"])
            kk = q["k_next"]
        assert a.tokens == b.tokens
        a.close(); b.close()
    finally:
        dm.close(); vm.close()


def test_gpu_ar_greedy_matches_oracle_and_injected_rounds_are_lossless():
    """The GPU's one-token-per-step greedy decode equals the oracle's; speculative rounds whose path is
    partly overwritten with that stream (synthetic acceptance) commit exactly the same stream."""
    cfg = synth.CFG_TINY
    dw, vw = synth.make_weights(cfg, 0), synth.make_weights(cfg, 1)
    prefix = synth.make_prefix(cfg, 96, 9)
    n_new = 40
    dm, vm = rnd.DeviceModel(cfg, dw, 256), rnd.DeviceModel(cfg, vw, 256)
    dec = rnd.SpecDecoder(dm, vm, synth.make_ngram_table(3), synth.NGRAM_LOG2_SIZE,
                          rnd.RoundParams(m_max=4, beam=4, lam=0.5, k_min=2, k_max=12, delta=2.0), k_cap=16)
    try:
        stream = rnd.ar_greedy(vm, prefix, n_new)
        ref = o_round.ar_greedy(cfg, vw, prefix, n_new)
        if stream != ref:   # only a float32 near-tie of the top two logits may separate the two decodes
            first = next(i for i in range(n_new) if stream[i] != ref[i])
            pytest.skip(f"greedy streams part at token {first}: near-tie case, not comparable further")
        stream_dev = rnd.upload(np.asarray(stream, dtype=np.int32))
        dec.start(prefix)
        assert dec.tokens[len(prefix)] == stream[0]
        rng = np.random.default_rng(3)
        k = 8
        accepted = []
        while len(dec.tokens) - len(prefix) + k + 1 < n_new:
            done = len(dec.tokens) - len(prefix)          # stream[done:] is what the verifier would emit next
            a = int(min(k, rng.geometric(0.3) - 1))
            got = dec.round(k, inject=(stream_dev[done:done + a], a))
            assert got["n_accept"] >= a                    # injected tokens are the verifier's own choices
            accepted.append(got["n_accept"])
            k = got["k_next"]
        produced = dec.tokens[len(prefix):]
        assert produced == stream[:len(produced)]
        assert max(accepted) >= 2 and dm.kv_len == len(dec.tokens) - len(dec.pending)
    finally:
        dec.close(); dm.close(); vm.close()
