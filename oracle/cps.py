"""Oracle causal-consistency path search (Sec. 3.2, "Scoring and search").  Test infrastructure only.

A path pi = (pi_1 .. pi_m) through the pruned lattice is scored by the additive mixed score

    S(pi) = sum_i [ lambda * l_dlm_i(pi_i) + (1 - lambda) * l_ng_i(pi_1..i) ]

and a left-to-right beam search of width B picks one path.  EOS is always a candidate,
and nothing is expanded past the first EOS.

Readings fixed here (the paper leaves them open):
  * candidates of position i = first cand_cnt[i] lattice entries; if EOS is not among them it
    is appended as the last candidate with its own log-probability;
  * l_ng is the conditional 3-gram log-score of pi_i given the two preceding tokens (reaching
    back into the prefix at the block start), looked up in a hashed table;
  * search is depth-synchronous: every live hypothesis is extended by every candidate, the
    best B by (score descending, parent index ascending, candidate rank ascending) are kept;
    if the best kept hypothesis ends in EOS it is returned (EOS included); otherwise hypotheses
    that end in EOS are dropped and the rest go on; after the last position the best is returned;
  * no length normalisation;
  * float32, unfused: term = (lambda*l_dlm) + ((1-lambda)*l_ng); score = score + term.

The same section names a tiny causal LM as the other form of the causal proxy (cps_path_lm): there l_ng of a
hypothesis' next token w is log softmax(z)[w], z the proxy LM's logits after the committed tokens followed by the
hypothesis' tokens (a small decoder of the family in model.py that shares the vocabulary); everything else is
the search above.  The proxy's logits are float32 (model.lm_head); the log-softmax is taken in float64 and rounded
once to float32.
"""
from __future__ import annotations

import numpy as np

from . import model  # the decoder a tiny-causal-LM proxy is an instance of

f32 = np.float32
u32 = np.uint32


def ngram_slot(u: int, v: int, w: int, log2_size: int) -> int:
    """Table slot of the 3-gram (u, v, w): a multiply / xor-shift mix in uint32 arithmetic."""
    with np.errstate(over="ignore"):
        x = u32(u) * u32(0x9E3779B1)
        x = x ^ (x >> u32(15))
        x = (x + u32(v)) * u32(0x85EBCA77)
        x = x ^ (x >> u32(13))
        x = (x + u32(w)) * u32(0xC2B2AE3D)
        x = x ^ (x >> u32(16))
    return int(x & u32((1 << log2_size) - 1))


def position_candidates(lat: dict, row: int, eos_id: int):
    """[(token, l_dlm)] of one lattice row after pruning, EOS retained."""
    cnt = int(lat["cand_cnt"][row])
    cands = [(int(lat["cand_id"][row, c]), f32(lat["cand_logp"][row, c])) for c in range(cnt)]
    if eos_id >= 0 and all(tok != eos_id for tok, _ in cands):
        cands.append((int(eos_id), f32(lat["eos_logp"][row])))
    return cands


def step_term(lam: f32, l_dlm: f32, l_ng: f32) -> f32:
    one_minus = f32(f32(1.0) - lam)
    return f32(f32(lam * l_dlm) + f32(one_minus * l_ng))


def cps_path(lat: dict, row0: int, k_len: int, beam: int, lam: float, table, log2_size: int,
             ctx, eos_id: int, margins=None):
    """Beam search over lattice rows row0 .. row0+k_len-1.

    table: float32 array of 2^log2_size proxy scores, or None (then l_ng = 0).
    ctx: the two tokens that precede the block (older first).
    margins (diagnostic, optional list): per depth, the smallest score gap between neighbours among the kept
    hypotheses and the best dropped one is appended (inf if there is a single expansion), so that a test can
    tell whether a differing search result sits on a near-tie.  It changes nothing in the search.
    Returns (path tokens list, score float32, number of candidate evaluations).
    """
    lam = f32(lam)
    hyps = [(f32(0.0), [], int(ctx[0]), int(ctx[1]))]  # score, tokens, u, v
    evals = 0
    for i in range(k_len):
        cands = position_candidates(lat, row0 + i, eos_id)
        grown = []
        for b, (score, toks, u, v) in enumerate(hyps):
            for c, (w, l_dlm) in enumerate(cands):
                l_ng = f32(table[ngram_slot(u, v, w, log2_size)]) if table is not None else f32(0.0)
                grown.append((f32(score + step_term(lam, l_dlm, l_ng)), b, c))
                evals += 1
        grown.sort(key=lambda e: (-float(e[0]), e[1], e[2]))
        kept = grown[:beam]
        if margins is not None:
            top = [float(e[0]) for e in grown[:beam + 1]]
            margins.append(min((a - b for a, b in zip(top, top[1:])), default=float("inf")))
        new_hyps = []
        for rank, (score, b, c) in enumerate(kept):
            w = cands[c][0]
            toks = hyps[b][1] + [w]
            if w == eos_id and eos_id >= 0:
                if rank == 0:
                    return toks, score, evals
                continue  # finished but not best: dropped, never expanded
            new_hyps.append((score, toks, hyps[b][3], w))
        hyps = new_hyps
    return hyps[0][1], hyps[0][0], evals


def proxy_log_probs(logits_row: np.ndarray) -> np.ndarray:
    """float32 log-softmax of one row of proxy logits: log-sum-exp in float64, one rounding."""
    z = np.asarray(logits_row, dtype=np.float64)
    m = z.max()
    return (z - (m + np.log(np.exp(z - m).sum()))).astype(f32)


def cps_path_lm(lat: dict, row0: int, k_len: int, beam: int, lam: float, pcfg, pw, cache, pending,
                eos_id: int, margins=None):
    """The search of cps_path with a tiny causal LM as the proxy (Sec. 3.2, "Scoring and search").

    pcfg / pw: the proxy model; cache: its model.KVCache holding the committed tokens EXCEPT the last
    len(pending) >= 1 of them, which `pending` lists (the last committed token among them).  The pending tokens
    are appended to `cache` (they are committed); hypotheses work on copies.  Every kept hypothesis is advanced
    by one proxy step (its own copy of the cache), which yields the distribution its extensions are scored with.
    Returns (path tokens list, score float32, number of candidate evaluations).
    """
    lam = f32(lam)
    root = proxy_log_probs(model.verify_logits(pcfg, pw, cache, [int(t) for t in pending])[-1])
    hyps = [(f32(0.0), [], cache, root)]  # score, tokens, proxy cache after the tokens but the last, l_ng row
    evals = 0
    for i in range(k_len):
        cands = position_candidates(lat, row0 + i, eos_id)
        grown = []
        for b, (score, toks, _, l_ng_row) in enumerate(hyps):
            for c, (w, l_dlm) in enumerate(cands):
                grown.append((f32(score + step_term(lam, l_dlm, f32(l_ng_row[w]))), b, c))
                evals += 1
        grown.sort(key=lambda e: (-float(e[0]), e[1], e[2]))
        kept = grown[:beam]
        if margins is not None:
            top = [float(e[0]) for e in grown[:beam + 1]]
            margins.append(min((a - b for a, b in zip(top, top[1:])), default=float("inf")))
        new_hyps = []
        for rank, (score, b, c) in enumerate(kept):
            w = cands[c][0]
            toks = hyps[b][1] + [w]
            if w == eos_id and eos_id >= 0:
                if rank == 0:
                    return toks, score, evals
                continue
            if i + 1 < k_len:  # the proxy's distribution after this hypothesis: one more causal row
                child = hyps[b][2].copy()
                row = proxy_log_probs(model.verify_logits(pcfg, pw, child, [w])[-1])
            else:
                child, row = None, None
            new_hyps.append((score, toks, child, row))
        hyps = new_hyps
    return hyps[0][1], hyps[0][0], evals


def cps_batch(lat: dict, batch: int, k_len: int, beam: int, lam: float, table, log2_size: int,
              ctx: np.ndarray, eos_id: int):
    """Independent searches for `batch` sequences whose lattice rows are stacked [batch*k_len].

    Returns path int32 [batch, k_len] (unused tail = -1), path_len int32 [batch], score float32 [batch].
    """
    path = np.full((batch, k_len), -1, dtype=np.int32)
    plen = np.zeros(batch, dtype=np.int32)
    score = np.zeros(batch, dtype=np.float32)
    for s in range(batch):
        toks, sc, _ = cps_path(lat, s * k_len, k_len, beam, lam, table, log2_size, ctx[s], eos_id)
        path[s, :len(toks)] = toks
        plen[s] = len(toks)
        score[s] = sc
    return path, plen, score
