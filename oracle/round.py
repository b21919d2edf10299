"""Oracle speculative round and loop (the four-stage algorithm of Sec. 3.4: draft, path search,
parallel verification, draft-length update).  Test infrastructure only.

Bookkeeping reading: both caches start with the same P prefix tokens.  `pending` holds the
tokens committed since the drafter last ran (one token before the first round: the verifier's
greedy token after the prefix).  Each round commits the accepted draft tokens plus one verifier
token (correction or bonus), so the committed stream equals the verifier's own greedy decode.
"""
from __future__ import annotations

import numpy as np

from . import accept, adl, cps, lattice, model, refine, sample


class SpecState:
    def __init__(self, dcfg, dw, vcfg, vw, prefix):
        self.dcfg, self.dw, self.vcfg, self.vw = dcfg, dw, vcfg, vw
        self.dcache = model.KVCache(dcfg)
        self.vcache = model.KVCache(vcfg)
        model.prefill(dcfg, dw, self.dcache, prefix)
        first = int(np.argmax(model.prefill(vcfg, vw, self.vcache, prefix)))
        self.tokens = [int(t) for t in prefix] + [first]  # every committed token so far
        self.pending = [first]


def spec_round(st: SpecState, k_draft: int, m_max: int, tau: float, beam: int, lam: float,
               table, log2_size: int, forced_path=None, refine_steps: int = 1, uniforms=None,
               lm_proxy=None) -> dict:
    """One round.  `forced_path` (tests only) replaces the searched path before verification.

    refine_steps > 1: the drafter refines the block over several passes and the lattice is frozen row by row
    (refinement update equation).  uniforms (float [k_draft + 1]): verify with the stochastic acceptance rule,
    u[i] deciding draft token i + 1 and u[k_draft] driving the replacement / bonus draw; needs the single-pass
    draft, whose rows are the left-to-right proxy's distributions.
    lm_proxy = (cfg, weights, KVCache holding the committed tokens but the pending ones): the path search scores with
    this tiny causal LM instead of the n-gram table (Sec. 3.2, "Scoring and search").
    """
    eos_id = st.dcfg.eos_id
    ctx = st.tokens[-2:]
    hidden = d_logits = None
    if refine_steps > 1:
        assert uniforms is None
        lat, _, _ = refine.refine_block(st.dcfg, st.dw, st.dcache, st.pending, k_draft, refine_steps, m_max, tau,
                                        eos_id)
    else:
        hidden = model.draft_block(st.dcfg, st.dw, st.dcache, st.pending, k_draft)
        d_logits = model.lm_head(st.dw, hidden)
        lat = lattice.build_lattice(d_logits, m_max, tau, eos_id)
    if lm_proxy is not None:
        path, score, _ = cps.cps_path_lm(lat, 0, k_draft, beam, lam, lm_proxy[0], lm_proxy[1], lm_proxy[2], st.pending,
                                         eos_id)
    else:
        path, score, _ = cps.cps_path(lat, 0, k_draft, beam, lam, table, log2_size, ctx, eos_id)
    if forced_path is not None:
        path = [int(t) for t in forced_path]
    block = [st.tokens[-1]] + path
    old_len = st.vcache.length
    v_logits = model.verify_logits(st.vcfg, st.vw, st.vcache, block)
    alpha = None
    if uniforms is None:
        n_acc, nxt, am, eos = accept.verify_greedy(v_logits, np.asarray(path), eos_id)
    else:
        am = accept.greedy_argmax(v_logits)
        n_acc, nxt, eos, alpha = sample.verify_stochastic(v_logits, d_logits[:len(path)], np.asarray(path),
                                                          np.asarray(uniforms)[:len(path)],
                                                          float(np.asarray(uniforms)[k_draft]), eos_id)
    st.vcache.truncate(old_len + 1 + n_acc)
    committed = path[:n_acc] + [nxt]
    st.tokens += committed
    st.pending = committed
    return {"hidden": hidden, "d_logits": d_logits, "lattice": lat, "path": path, "score": score,
            "v_logits": v_logits, "argmax": am, "n_accept": n_acc, "next_token": nxt,
            "eos_accepted": eos, "committed": committed, "alpha": alpha,
            "first_eos": adl.first_eos_index(lattice.raw_draft(lat), eos_id)}


def generate(st: SpecState, n_rounds: int, k_first: int, adl_state: adl.AdlState, m_max: int,
             tau: float, beam: int, lam: float, table, log2_size: int):
    """Run rounds until an EOS is accepted or n_rounds are done; returns the per-round records."""
    k_t = k_first
    recs = []
    for _ in range(n_rounds):
        r = spec_round(st, k_t, m_max, tau, beam, lam, table, log2_size)
        r["k"] = k_t
        k_t = adl.adl_update(adl_state, k_t, r["first_eos"], r["n_accept"])
        r["k_next"] = k_t
        recs.append(r)
        if r["eos_accepted"]:
            break
    return recs


def ar_greedy(cfg, w, prefix, n_new: int):
    """Plain greedy decoding of the verifier, one token per step (the lossless reference)."""
    cache = model.KVCache(cfg)
    out = [int(np.argmax(model.prefill(cfg, w, cache, prefix)))]
    while len(out) < n_new:
        logits = model.verify_logits(cfg, w, cache, [out[-1]])
        out.append(int(np.argmax(logits[0])))
    return out
