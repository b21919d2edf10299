"""Pins for the oracle's whole round and loop (no GPU): the committed stream equals the
verifier's own greedy decode (greedy verification is lossless), and a draft equal to that
greedy continuation is accepted in full."""
import numpy as np

from oracle import adl, model, round as oround
from paper_2510_02358_amd import synth

CFG = synth.ModelCfg(n_layers=2, d_model=64, n_q=4, n_kv=2, head_dim=16, d_ffn=96, vocab=96,
                     rope_base=1.0e4, dtype="f32")
LOG2 = 12


def _setup(seed_d=0, seed_v=1):
    dw = synth.make_weights(CFG, seed_d, std=0.3)
    vw = synth.make_weights(CFG, seed_v, std=0.3)
    prefix = synth.make_prefix(CFG, 12, 2)
    return dw, vw, prefix


def test_committed_stream_equals_verifier_greedy_decode():
    dw, vw, prefix = _setup()
    table = synth.make_ngram_table(3, LOG2)
    st = oround.SpecState(CFG, dw, CFG, vw, prefix)
    recs = oround.generate(st, 6, 5, adl.AdlState(2, 8, 2, 0.5), 3, 1.0, 2, 0.5, table, LOG2)
    produced = st.tokens[len(prefix):]
    ref = oround.ar_greedy(CFG, vw, prefix, len(produced))
    assert produced == ref
    assert sum(len(r["committed"]) for r in recs) + 1 == len(produced)
    # caches hold exactly the committed tokens minus the one still pending for the verifier
    assert st.vcache.length == len(st.tokens) - 1


def test_same_model_as_drafter_and_verifier_still_lossless_and_forced_greedy_path_fully_accepted():
    dw, vw, prefix = _setup()
    k = 5
    st = oround.SpecState(CFG, dw, CFG, vw, prefix)
    greedy = oround.ar_greedy(CFG, vw, prefix, k + 2)       # greedy[0] is the pending token
    r = oround.spec_round(st, k, 3, 1.0, 2, 1.0, None, LOG2, forced_path=greedy[1:k + 1])
    assert r["n_accept"] == k and r["next_token"] == greedy[k + 1]
    assert r["committed"] == greedy[1:k + 2]
    # wrong first token -> nothing accepted, correction equals the greedy token
    st = oround.SpecState(CFG, dw, CFG, vw, prefix)
    bad = [(greedy[1] + 1) % CFG.n_plain_tokens] + greedy[2:k + 1]
    r = oround.spec_round(st, k, 3, 1.0, 2, 1.0, None, LOG2, forced_path=bad)
    assert r["n_accept"] == 0 and r["next_token"] == greedy[1]
    # partial: first two right
    st = oround.SpecState(CFG, dw, CFG, vw, prefix)
    part = greedy[1:3] + [(greedy[3] + 1) % CFG.n_plain_tokens] + greedy[4:k + 1]
    r = oround.spec_round(st, k, 3, 1.0, 2, 1.0, None, LOG2, forced_path=part)
    assert r["n_accept"] == 2 and r["next_token"] == greedy[3]
    # next round still continues the greedy stream (KV rollback by truncation is right)
    r2 = oround.spec_round(st, k, 3, 1.0, 2, 1.0, None, LOG2)
    ref = oround.ar_greedy(CFG, vw, prefix, len(st.tokens) - len(prefix))
    assert st.tokens[len(prefix):] == ref
    assert st.pending == r2["committed"]


def test_rounds_with_a_tiny_lm_proxy_stay_lossless_and_keep_the_proxy_history_in_step():
    """The causal proxy only steers the search: with a tiny causal LM in its place the committed stream is still the
    verifier's greedy decode, and the proxy's cache always holds the committed tokens but the pending ones."""
    dw, vw, prefix = _setup()
    pcfg = synth.ModelCfg(n_layers=1, d_model=32, n_q=2, n_kv=1, head_dim=16, d_ffn=48, vocab=CFG.vocab,
                          rope_base=1.0e4, dtype="f32")
    pw = synth.make_weights(pcfg, 9, std=0.3)
    pcache = model.KVCache(pcfg)
    model.prefill(pcfg, pw, pcache, prefix)
    st = oround.SpecState(CFG, dw, CFG, vw, prefix)
    plain = oround.SpecState(CFG, dw, CFG, vw, prefix)
    differs = 0
    for _ in range(5):
        r = oround.spec_round(st, 5, 3, 1.0, 2, 0.3, None, LOG2, lm_proxy=(pcfg, pw, pcache))
        q = oround.spec_round(plain, 5, 3, 1.0, 2, 0.3, None, LOG2)
        differs += r["path"] != q["path"]
        assert pcache.length == len(st.tokens) - len(st.pending)
    produced = st.tokens[len(prefix):]
    assert produced == oround.ar_greedy(CFG, vw, prefix, len(produced))
    assert differs >= 1          # the proxy does steer the search


def test_rounds_on_a_pair_with_planted_successors_give_the_hand_derived_verdicts():
    """A pair whose next token is a planted function of the current token (zero output projections: the final state is
    the token's embedding; the LM-head row of the successor carries the normalised embedding).  [MASK] -> 7, 5 -> 7 and
    either 7 -> 7 (all K draft tokens accepted, next 7) or 7 -> 9 -> 7 (one accepted, next 9): worked by hand."""
    for fixed_point in (True, False):
        succ = {CFG.mask_id: 7, 31: 5, 5: 7, 7: 7 if fixed_point else 9, 9: 7}
        w = synth.make_weights(CFG, 20, std=0.3)
        for lw in w["layers"]:
            lw["wo"][:] = 0.0
            lw["w_down"][:] = 0.0
        for t, nxt in succ.items():
            e = w["embed"][t].astype(np.float64)
            y = e / np.sqrt(np.mean(e * e) + CFG.rms_eps)
            w["lm_head"][nxt] += (60.0 * y / np.sqrt(CFG.d_model)).astype(np.float32)
        prefix = np.concatenate([synth.make_prefix(CFG, 10, 3), [31]])
        st = oround.SpecState(CFG, w, CFG, w, prefix)
        assert st.tokens[-1] == 5
        k = 5
        for _ in range(3):
            r = oround.spec_round(st, k, 3, 1.0, 2, 1.0, None, LOG2)
            assert r["path"] == [7] * k
            if fixed_point:
                assert (r["n_accept"], r["next_token"], r["committed"]) == (k, 7, [7] * (k + 1))
            else:
                assert (r["n_accept"], r["next_token"], r["committed"]) == (1, 9, [7, 9])
        assert st.vcache.length == len(st.tokens) - 1 and st.dcache.length == len(st.tokens) - len(st.pending)
