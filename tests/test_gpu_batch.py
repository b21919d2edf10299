"""GPU tests of the batched calls (several sequences share one pass over the weights).

(1) Every row of a batched draft / verify call is bit-identical to the single-sequence call for that sequence alone:
    a row's result never depends on what else is in the call.
(2) Whole batched rounds against the oracle: the batch is n independent oracle rounds.
"""
import numpy as np
import pytest
import torch

from oracle import round as o_round
from paper_2510_02358_amd import binding as ds
from paper_2510_02358_amd import round as rnd
from paper_2510_02358_amd import synth

import gpu_util as gu

pytestmark = pytest.mark.gpu

SMALL_BF16 = synth.ModelCfg(n_layers=2, d_model=256, n_q=4, n_kv=2, head_dim=128, d_ffn=512, vocab=4096,
                            rope_base=1.0e6, dtype="bf16")


def _new_seq(gm):
    kvb = ds.ds_kv_bytes(gm.cfgc)
    k = torch.empty(kvb, dtype=torch.uint8, device=gu.DEV)
    v = torch.empty(kvb, dtype=torch.uint8, device=gu.DEV)
    return ds.ds_kv_create(gm.handle, k, v), k, v


@pytest.mark.parametrize("cfg_name", ["f32", "bf16"])
def test_batched_rows_are_bit_identical_to_single_sequence_calls(cfg_name):
    cfg = synth.CFG_TINY if cfg_name == "f32" else SMALL_BF16
    w = synth.make_weights(cfg, 300)
    synth.randomize_norm_gains(w, 301)
    rng = np.random.default_rng(302)
    gm = gu.GpuModel(cfg, w, 512)
    seqs = [_new_seq(gm) for _ in range(3)]
    kvs = [q[0] for q in seqs]
    try:
        # prefixes of different lengths (different split counts of the key axis), different pending counts
        prefixes = [synth.make_prefix(cfg, n, 310 + n) for n in (70, 130, 333)]
        pend = [[5], [9, 8, 7], [1, 2]]
        k = 9
        for s, pre in enumerate(prefixes):
            ds.ds_prefill_seq(gm.handle, kvs[s], gu.to_dev(pre), len(pre), None, gm.ws)
        hid = torch.empty(3 * k, cfg.d_model, dtype=torch.float32, device=gu.DEV)
        flat = gu.to_dev(np.asarray([t for q in pend for t in q], np.int32))
        ds.ds_draft_block_batch(gm.handle, kvs, flat, [len(q) for q in pend], k, cfg.mask_id, hid, gm.ws)
        lat_b, logits_b = gm.draft_lattice(None, 3 * k, 4, 0.9, cfg.eos_id, want_logits=True)
        torch.cuda.synchronize()
        assert [ds.ds_kv_len(kv) for kv in kvs] == [len(p) + len(q) for p, q in zip(prefixes, pend)]
        # verify: m = 9 path tokens per sequence; make the first two of sequence 1 the verifier's own choices later
        m = k
        first = rng.integers(0, cfg.n_plain_tokens, 3).astype(np.int32)
        path = rng.integers(0, cfg.n_plain_tokens, (3, m)).astype(np.int32)
        plen = np.array([m, 4, 0], np.int32)
        R = (m + 1 + 15) // 16 * 16

        def verify_batch(path_now):
            out = torch.zeros(9, dtype=torch.int32, device=gu.DEV)
            am = torch.zeros(3 * (m + 1), dtype=torch.int32, device=gu.DEV)
            lg = torch.zeros(2 * R + m + 1, cfg.vocab, dtype=torch.float32, device=gu.DEV)
            ds.ds_verify_block_batch(gm.handle, kvs, gu.to_dev(first), gu.to_dev(path_now), m, gu.to_dev(plen),
                                     cfg.eos_id, out[0:3], out[3:6], am, out[6:9], lg, gm.ws)
            torch.cuda.synchronize()
            return out.cpu().numpy(), am.cpu().numpy().reshape(3, m + 1), lg.cpu().numpy()

        res0, am0, _ = verify_batch(path)
        path2 = path.copy()
        path2[0, 0], path2[1, 0] = am0[0, 0], am0[1, 0]          # accepted first tokens in sequences 0 and 1
        res, am, lg = verify_batch(path2)
        assert res[0] >= 1 and res[1] >= 1 and res[2] == 0      # n_accept; path_len 0 accepts nothing
        # the same things, one sequence at a time, through the single-sequence calls on the built-in cache
        for s, pre in enumerate(prefixes):
            gm.set_kv_len(0)
            gm.prefill(pre, want_logits=False)
            hid1 = gm.draft(pend[s], k)
            lat1, logits1 = gm.draft_lattice(None, k, 4, 0.9, cfg.eos_id, want_logits=True)
            assert torch.equal(hid1, hid[s * k:(s + 1) * k]), s
            assert torch.equal(logits1, logits_b[s * k:(s + 1) * k]), s
            for name in lat1:
                assert torch.equal(lat1[name], lat_b[name][s * k:(s + 1) * k]), (s, name)
            block = np.concatenate([[first[s]], path2[s]]).astype(np.int32)
            one = gm.verify(block, path_len=gu.to_dev(plen[s:s + 1]), eos_id=cfg.eos_id)
            assert np.array_equal(one["logits"], lg[s * R:s * R + m + 1]), s
            assert np.array_equal(one["argmax"], am[s]), s
            assert (one["n_accept"], one["next_token"], one["eos_accepted"]) == (res[s], res[3 + s], res[6 + s]), s
    finally:
        for kv, _, _ in seqs:
            ds.ds_kv_destroy(kv)
        gm.close()


def test_batched_call_argument_errors():
    cfg = SMALL_BF16
    gm = gu.GpuModel(cfg, synth.make_weights(cfg, 320), 128)
    other = gu.GpuModel(cfg, synth.make_weights(cfg, 321), 128)
    seqs = [_new_seq(gm) for _ in range(2)]
    foreign = _new_seq(other)
    hid = torch.empty(64, cfg.d_model, dtype=torch.float32, device=gu.DEV)
    pend = gu.to_dev(np.array([1, 2], np.int32))
    try:
        with pytest.raises(ds.DsError) as e:        # the same handle twice
            ds.ds_draft_block_batch(gm.handle, [seqs[0][0], seqs[0][0]], pend, [1, 1], 8, cfg.mask_id, hid, gm.ws)
        assert e.value.code == ds.DS_E_INVALID
        with pytest.raises(ds.DsError) as e:        # a handle of another model
            ds.ds_draft_block_batch(gm.handle, [seqs[0][0], foreign[0]], pend, [1, 1], 8, cfg.mask_id, hid, gm.ws)
        assert e.value.code == ds.DS_E_INVALID
        with pytest.raises(ds.DsError) as e:        # 2 x (1 + 70) rows: 80 + 71 > 144
            ds.ds_draft_block_batch(gm.handle, [q[0] for q in seqs], pend, [1, 1], 70, cfg.mask_id, hid, gm.ws)
        assert e.value.code == ds.DS_E_SHAPE
        with pytest.raises(ds.DsError) as e:        # cache capacity 128
            ds.ds_kv_set_len(seqs[0][0], 129)
        assert e.value.code == ds.DS_E_CAPACITY
        assert [ds.ds_kv_len(q[0]) for q in seqs] == [0, 0]
    finally:
        for kv, _, _ in seqs + [foreign]:
            ds.ds_kv_destroy(kv)
        gm.close()
        other.close()


def test_batched_rounds_match_independent_oracle_rounds():
    """Three sequences with their own prefixes through four batched rounds on the tiny float32 pair: each sequence's
    lattice ids, searched path, verdict and committed tokens equal the oracle's round for that sequence alone."""
    cfg = synth.CFG_TINY
    dw, vw = synth.make_weights(cfg, 0), synth.make_weights(cfg, 1)
    table = synth.make_ngram_table(3)
    m_max, beam, lam, tau, k = 4, 4, 0.5, 0.9, 8
    params = rnd.RoundParams(m_max=m_max, tau=tau, beam=beam, lam=lam, k_min=2, k_max=12, delta=2.0, rho=0.5)
    prefixes = [synth.make_prefix(cfg, n, 330 + n) for n in (128, 40, 77)]
    dm, vm = rnd.DeviceModel(cfg, dw, 256), rnd.DeviceModel(cfg, vw, 256)
    dec = rnd.BatchSpecDecoder(dm, vm, 3, table, synth.NGRAM_LOG2_SIZE, params, k_cap=16, keep_logits=True)
    try:
        dec.start(prefixes)
        states = [o_round.SpecState(cfg, dw, cfg, vw, p) for p in prefixes]
        for s in range(3):
            assert dec.tokens[s] == states[s].tokens
        compared = 0
        for t in range(4):
            got = dec.round(k)
            d_logits = dec.d_logits[:3 * k].cpu().numpy()
            ids = dec.cand_id[:3 * k].cpu().numpy()
            for s in range(3):
                ref = o_round.spec_round(states[s], k, m_max, tau, beam, lam, table, synth.NGRAM_LOG2_SIZE)
                assert np.max(np.abs(d_logits[s * k:(s + 1) * k] - ref["d_logits"])) <= 1e-4
                assert np.array_equal(ids[s * k:(s + 1) * k], ref["lattice"]["cand_id"]), (t, s)
                assert list(got[s]["path"]) == ref["path"], (t, s)
                verdict = (got[s]["n_accept"], got[s]["next_token"], got[s]["eos_accepted"])
                assert verdict == (ref["n_accept"], ref["next_token"], ref["eos_accepted"]), (t, s)
                assert got[s]["first_eos"] == ref["first_eos"]
                assert dec.tokens[s] == states[s].tokens
                assert ds.ds_kv_len(dec.d_kv[s]) == states[s].dcache.length
                assert ds.ds_kv_len(dec.v_kv[s]) == states[s].vcache.length
                compared += 1
        print("PARITY-COUNTS batched rounds: sequence-rounds compared", compared)
    finally:
        dec.close(); dm.close(); vm.close()
