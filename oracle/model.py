"""Oracle decoder forward (drafter and verifier).  Test infrastructure only.

The paper specifies the drafter only as a Transformer with bidirectional attention that
fills `prefix ∘ [MASK]^k` in one pass (Sec. 3.1, "Inference", default S = 1) and the
verifier as an autoregressive LM evaluated over the drafted block in one parallel pass
with its KV cache (Sec. 2, "Parallel verification"; Sec. 4, "Implementation details").
The layer itself is the standard pre-RMSNorm decoder with grouped-query attention, rotary
position embedding and a SwiGLU MLP:

    h = rmsnorm(x, g1);  q,k,v = h Wq^T, h Wk^T, h Wv^T;  rotate q,k
    x = x + softmax(q k^T / sqrt(hd) + mask) v Wo^T
    h = rmsnorm(x, g2);  x = x + (silu(h Wg^T) * (h Wu^T)) Wd^T
    y = rmsnorm(x_last_layer, gf);  logits = y Wlm^T

Attention mask (the reading that makes a drafter prefix cache possible): a real-token row
sees columns up to and including itself (causal); a [MASK] row sees every column of the
sequence: whole prefix, pending tokens and all draft positions, later ones included.

All arithmetic is float64; logits are rounded once to float32.
"""
from __future__ import annotations

import numpy as np

F64 = np.float64


def matmul_t(x: np.ndarray, w: np.ndarray, chunk: int = 16384) -> np.ndarray:
    """x [rows, n_in] (f64) times w^T, w [n_out, n_in] (f32 storage) -> [rows, n_out] f64."""
    out = np.empty((x.shape[0], w.shape[0]), dtype=F64)
    for lo in range(0, w.shape[0], chunk):
        out[:, lo:lo + chunk] = x @ w[lo:lo + chunk].astype(F64).T
    return out


def rmsnorm(x: np.ndarray, gain: np.ndarray, eps: float) -> np.ndarray:
    ms = np.mean(x * x, axis=-1, keepdims=True)
    return x / np.sqrt(ms + eps) * gain.astype(F64)


def rope(x: np.ndarray, pos: np.ndarray, base: float) -> np.ndarray:
    """Rotate-half RoPE.  x [rows, heads, hd]; pos [rows] absolute positions.

    Pair (i, i + hd/2) is rotated by the angle pos * base^(-2i/hd).
    """
    hd = x.shape[-1]
    half = hd // 2
    theta = F64(base) ** (-2.0 * np.arange(half, dtype=F64) / hd)
    ang = pos.astype(F64)[:, None] * theta[None, :]
    c = np.cos(ang)[:, None, :]
    s = np.sin(ang)[:, None, :]
    x1, x2 = x[..., :half], x[..., half:]
    return np.concatenate([x1 * c - x2 * s, x2 * c + x1 * s], axis=-1)


def silu(x: np.ndarray) -> np.ndarray:
    return x / (1.0 + np.exp(-x))


class KVCache:
    """Per-layer keys (already rotated) and values of the committed tokens, [len, Hkv, hd] f64."""

    def __init__(self, cfg):
        self.k = [np.zeros((0, cfg.n_kv, cfg.head_dim), dtype=F64) for _ in range(cfg.n_layers)]
        self.v = [np.zeros((0, cfg.n_kv, cfg.head_dim), dtype=F64) for _ in range(cfg.n_layers)]

    @property
    def length(self) -> int:
        return self.k[0].shape[0]

    def truncate(self, n: int) -> None:
        assert 0 <= n <= self.length
        self.k = [a[:n] for a in self.k]
        self.v = [a[:n] for a in self.v]

    def copy(self) -> "KVCache":
        c = KVCache.__new__(KVCache)
        c.k = [a.copy() for a in self.k]
        c.v = [a.copy() for a in self.v]
        return c


def decoder_rows(cfg, w: dict, cache: KVCache, tokens: np.ndarray, sees_all: np.ndarray,
                 n_commit: int, use_rope: bool = True) -> np.ndarray:
    """Forward of `tokens` placed right after the cached tokens.

    sees_all[r] = True marks a [MASK] row (sees every column); False a real-token row
    (causal).  Keys/values of the first `n_commit` rows are appended to the cache.
    Returns the final-normed hidden states y [rows, d_model] in float64.
    """
    tokens = np.asarray(tokens)
    rows = tokens.shape[0]
    past = cache.length
    hq, hkv, hd = cfg.n_q, cfg.n_kv, cfg.head_dim
    group = hq // hkv
    pos = past + np.arange(rows)
    # visibility of column c (absolute index) from row r
    col = np.arange(past + rows)
    visible = np.asarray(sees_all, dtype=bool)[:, None] | (col[None, :] <= pos[:, None])

    x = w["embed"][tokens].astype(F64)
    for li in range(cfg.n_layers):
        lw = w["layers"][li]
        h = rmsnorm(x, lw["norm1"], cfg.rms_eps)
        q = matmul_t(h, lw["wq"]).reshape(rows, hq, hd)
        k = matmul_t(h, lw["wk"]).reshape(rows, hkv, hd)
        v = matmul_t(h, lw["wv"]).reshape(rows, hkv, hd)
        if use_rope:
            q = rope(q, pos, cfg.rope_base)
            k = rope(k, pos, cfg.rope_base)
        keys = np.concatenate([cache.k[li], k], axis=0)
        vals = np.concatenate([cache.v[li], v], axis=0)
        att = np.empty((rows, hq, hd), dtype=F64)
        for head in range(hq):
            kvh = head // group
            s = q[:, head, :] @ keys[:, kvh, :].T / np.sqrt(F64(hd))
            s = np.where(visible, s, -np.inf)
            s = s - s.max(axis=-1, keepdims=True)
            p = np.exp(s)
            p = p / p.sum(axis=-1, keepdims=True)
            att[:, head, :] = p @ vals[:, kvh, :]
        x = x + matmul_t(att.reshape(rows, hq * hd), lw["wo"])
        h = rmsnorm(x, lw["norm2"], cfg.rms_eps)
        act = silu(matmul_t(h, lw["w_gate"])) * matmul_t(h, lw["w_up"])
        x = x + matmul_t(act, lw["w_down"])
        cache.k[li] = np.concatenate([cache.k[li], k[:n_commit]], axis=0)
        cache.v[li] = np.concatenate([cache.v[li], v[:n_commit]], axis=0)
    return rmsnorm(x, w["final_norm"], cfg.rms_eps)


def lm_head(w: dict, y: np.ndarray) -> np.ndarray:
    """logits = y Wlm^T, rounded once to float32."""
    return matmul_t(y, w["lm_head"]).astype(np.float32)


def prefill(cfg, w, cache: KVCache, tokens, use_rope: bool = True) -> np.ndarray:
    """Causal forward of real tokens; commits all of them; returns last-row logits [vocab]."""
    n = len(tokens)
    y = decoder_rows(cfg, w, cache, tokens, np.zeros(n, dtype=bool), n, use_rope)
    return lm_head(w, y[-1:])[0]


def draft_block(cfg, w, cache: KVCache, pending, k_draft: int, use_rope: bool = True,
                block_tokens=None) -> np.ndarray:
    """One drafter pass: rows = pending real tokens, then the k_draft block positions.

    With block_tokens None every block position holds [MASK] (the single pass of S = 1, and the first
    pass of a refinement); otherwise block_tokens gives the current draft y^(s-1) of the refinement
    update (already fixed tokens, [MASK] elsewhere).  Block rows see the whole block either way.
    Commits only the pending rows.  Returns y of the block rows, [k_draft, d_model] float64.
    The hidden state at block row i yields the distribution of the token at that position.
    """
    pending = np.asarray(pending, dtype=np.int64)
    n_pend = pending.shape[0]
    if block_tokens is None:
        block_tokens = np.full(k_draft, cfg.mask_id, dtype=np.int64)
    block_tokens = np.asarray(block_tokens, dtype=np.int64)
    assert block_tokens.shape == (k_draft,)
    tokens = np.concatenate([pending, block_tokens])
    sees_all = np.arange(n_pend + k_draft) >= n_pend
    y = decoder_rows(cfg, w, cache, tokens, sees_all, n_pend, use_rope)
    return y[n_pend:]


def verify_logits(cfg, w, cache: KVCache, block, use_rope: bool = True) -> np.ndarray:
    """Causal forward of block = [last committed token, path...]; logits [len(block), vocab].

    Row r predicts the token that follows block[r].  All rows are appended to the cache;
    the caller truncates to `old_len + 1 + n_accept` once acceptance is known.
    """
    n = len(block)
    y = decoder_rows(cfg, w, cache, block, np.zeros(n, dtype=bool), n, use_rope)
    return lm_head(w, y)


def full_sequence(cfg, w, tokens, sees_all, use_rope: bool = True) -> np.ndarray:
    """Whole sequence from an empty cache (the recompute the cached path is checked against)."""
    cache = KVCache(cfg)
    return decoder_rows(cfg, w, cache, tokens, sees_all, 0, use_rope)
