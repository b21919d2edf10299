"""Pins for the oracle decoder forward (no GPU).

The paper prints no numeric example for the forward, so it is pinned by: an independent
third implementation in primitive PyTorch CPU ops (complex-number RoPE, explicit mask
tensor, library softmax), KV-cached == full-sequence recompute, RoPE shift invariance,
GQA == MHA with replicated heads, mask-row symmetry without RoPE, and causality.
"""
import dataclasses

import numpy as np
import pytest
import torch

from oracle import model
from paper_2510_02358_amd import synth

CFG = synth.ModelCfg(n_layers=2, d_model=64, n_q=4, n_kv=2, head_dim=16, d_ffn=96, vocab=128,
                     rope_base=1.0e4, dtype="f32")


def _weights(cfg, seed):
    w = synth.make_weights(cfg, seed, std=0.2)  # larger std: makes every term matter
    synth.randomize_norm_gains(w, seed + 100)
    return w


def _torch_forward(cfg, w, tokens, sees_all, pos0=0):
    """Independent formulation: float64 torch, RoPE by complex multiplication, SDPA-style softmax."""
    t = lambda a: torch.from_numpy(np.asarray(a, dtype=np.float64))
    rows = len(tokens)
    hq, hkv, hd = cfg.n_q, cfg.n_kv, cfg.head_dim
    pos = torch.arange(rows, dtype=torch.float64) + pos0
    inv = torch.tensor(cfg.rope_base, dtype=torch.float64) ** (
        -torch.arange(0, hd, 2, dtype=torch.float64) / hd)
    rot = torch.polar(torch.ones(rows, hd // 2, dtype=torch.float64), pos[:, None] * inv[None, :])

    def rotate(x):  # x [rows, heads, hd]; pair (i, i+hd/2) as one complex number
        z = torch.complex(x[..., : hd // 2], x[..., hd // 2:]) * rot[:, None, :]
        return torch.cat([z.real, z.imag], dim=-1)

    allowed = torch.tril(torch.ones(rows, rows, dtype=torch.bool)) | torch.from_numpy(
        np.asarray(sees_all, dtype=bool))[:, None]
    bias = torch.zeros(rows, rows, dtype=torch.float64).masked_fill(~allowed, float("-inf"))
    x = t(w["embed"])[torch.as_tensor(np.asarray(tokens, dtype=np.int64))]
    for lw in w["layers"]:
        h = x * torch.rsqrt(x.pow(2).mean(-1, keepdim=True) + cfg.rms_eps) * t(lw["norm1"])
        q = rotate((h @ t(lw["wq"]).T).view(rows, hq, hd))
        k = rotate((h @ t(lw["wk"]).T).view(rows, hkv, hd))
        v = (h @ t(lw["wv"]).T).view(rows, hkv, hd)
        k = k.repeat_interleave(hq // hkv, dim=1)
        v = v.repeat_interleave(hq // hkv, dim=1)
        s = torch.einsum("rhd,chd->hrc", q, k) / hd ** 0.5 + bias[None]
        a = torch.einsum("hrc,chd->rhd", torch.softmax(s, dim=-1), v).reshape(rows, hq * hd)
        x = x + a @ t(lw["wo"]).T
        h = x * torch.rsqrt(x.pow(2).mean(-1, keepdim=True) + cfg.rms_eps) * t(lw["norm2"])
        x = x + (torch.nn.functional.silu(h @ t(lw["w_gate"]).T) * (h @ t(lw["w_up"]).T)) @ t(lw["w_down"]).T
    y = x * torch.rsqrt(x.pow(2).mean(-1, keepdim=True) + cfg.rms_eps) * t(w["final_norm"])
    return (y @ t(w["lm_head"]).T).numpy()


def _seq(cfg, n_real, k_mask, seed):
    real = synth.make_prefix(cfg, n_real, seed)
    tokens = np.concatenate([real, np.full(k_mask, cfg.mask_id, dtype=np.int32)])
    sees_all = np.arange(n_real + k_mask) >= n_real
    return tokens, sees_all


def test_matches_independent_torch_forward():
    w = _weights(CFG, 0)
    tokens, sees_all = _seq(CFG, 9, 5, 2)
    y = model.full_sequence(CFG, w, tokens, sees_all)
    got = model.matmul_t(y, w["lm_head"])
    ref = _torch_forward(CFG, w, tokens, sees_all)
    assert np.max(np.abs(got - ref)) < 1e-9
    # and the logits really depend on the inputs at the scale we test
    assert np.std(ref) > 0.1


def test_cached_equals_full_recompute_draft_and_verify():
    w = _weights(CFG, 1)
    prefix = synth.make_prefix(CFG, 11, 3)
    pending = synth.make_prefix(CFG, 3, 4)
    k = 6
    # drafter: prefix cached, then pending + K masks
    cache = model.KVCache(CFG)
    model.prefill(CFG, w, cache, prefix)
    hid = model.draft_block(CFG, w, cache, pending, k)
    assert cache.length == len(prefix) + len(pending)  # mask rows never committed
    tokens = np.concatenate([prefix, pending, np.full(k, CFG.mask_id)])
    sees_all = np.arange(len(tokens)) >= len(prefix) + len(pending)
    full = model.full_sequence(CFG, w, tokens, sees_all)
    assert np.max(np.abs(full[-k:] - hid)) < 1e-10
    # verifier: causal block against the cache
    cache = model.KVCache(CFG)
    model.prefill(CFG, w, cache, prefix)
    block = synth.make_prefix(CFG, 5, 5)
    lg = model.verify_logits(CFG, w, cache, block)
    tokens = np.concatenate([prefix, block])
    full = model.lm_head(w, model.full_sequence(CFG, w, tokens, np.zeros(len(tokens), bool)))
    assert np.max(np.abs(full[-5:] - lg)) <= 1e-5
    # a second cached draft round after committing more tokens still equals the recompute
    cache = model.KVCache(CFG)
    model.prefill(CFG, w, cache, prefix)
    model.draft_block(CFG, w, cache, pending[:1], k)
    hid2 = model.draft_block(CFG, w, cache, pending[1:], 4)
    tokens = np.concatenate([prefix, pending, np.full(4, CFG.mask_id)])
    sees_all = np.arange(len(tokens)) >= len(prefix) + len(pending)
    full = model.full_sequence(CFG, w, tokens, sees_all)
    assert np.max(np.abs(full[-4:] - hid2)) < 1e-10


def test_rope_shift_invariance():
    """Scores depend on position differences only: shifting every position leaves logits unchanged."""
    w = _weights(CFG, 2)
    tokens, sees_all = _seq(CFG, 7, 4, 6)
    base = model.full_sequence(CFG, w, tokens, sees_all)

    # building block: rotated q.k products are unchanged when every position moves by 37
    rows = len(tokens)
    x = np.random.default_rng(0).standard_normal((rows, CFG.n_q, CFG.head_dim))
    k = np.random.default_rng(1).standard_normal((rows, CFG.n_q, CFG.head_dim))
    pos = np.arange(rows)
    s0 = np.einsum("rhd,chd->hrc", model.rope(x, pos, 1e4), model.rope(k, pos, 1e4))
    s1 = np.einsum("rhd,chd->hrc", model.rope(x, pos + 37, 1e4), model.rope(k, pos + 37, 1e4))
    assert np.max(np.abs(s0 - s1)) < 1e-9
    # whole model through the torch formulation with an offset agrees with the oracle at offset 0
    ref = _torch_forward(CFG, w, tokens, sees_all, pos0=1000)
    assert np.max(np.abs(model.matmul_t(base, w["lm_head"]) - ref)) < 1e-7


def test_rope_rotates_the_right_pairs():
    """Position 0 is the identity; a quarter turn on pair (0, hd/2) with theta_0 = 1 maps (1,0)->(0,1)."""
    hd = 8
    x = np.zeros((1, 1, hd)); x[0, 0, 0] = 1.0
    out = model.rope(x, np.array([0]), 1e4)
    assert np.allclose(out, x)
    out = model.rope(x, np.array([np.pi / 2]), 1e4)
    expect = np.zeros(hd); expect[hd // 2] = 1.0
    assert np.allclose(out[0, 0], expect, atol=1e-12)
    # pair i uses theta_i = base^(-2i/hd): at pos=1, pair 1 rotates by 10000^(-0.25) = 0.1 rad
    x = np.zeros((1, 1, hd)); x[0, 0, 1] = 1.0
    out = model.rope(x, np.array([1]), 1e4)
    assert np.isclose(out[0, 0, 1], np.cos(0.1)) and np.isclose(out[0, 0, 1 + hd // 2], np.sin(0.1))


def test_gqa_equals_mha_with_replicated_kv_heads():
    w = _weights(CFG, 3)
    tokens, sees_all = _seq(CFG, 8, 3, 7)
    y_gqa = model.full_sequence(CFG, w, tokens, sees_all)
    mha = dataclasses.replace(CFG, n_kv=CFG.n_q)
    group = CFG.n_q // CFG.n_kv
    w2 = {"embed": w["embed"], "final_norm": w["final_norm"], "lm_head": w["lm_head"], "layers": []}
    for lw in w["layers"]:
        l2 = dict(lw)
        for name in ("wk", "wv"):
            m = lw[name].reshape(CFG.n_kv, CFG.head_dim, CFG.d_model)
            l2[name] = np.repeat(m, group, axis=0).reshape(CFG.n_q * CFG.head_dim, CFG.d_model)
        w2["layers"].append(l2)
    y_mha = model.full_sequence(mha, w2, tokens, sees_all)
    assert np.max(np.abs(y_gqa - y_mha)) < 1e-10


def test_mask_rows_are_symmetric_without_rope():
    w = _weights(CFG, 4)
    tokens, sees_all = _seq(CFG, 6, 5, 8)
    y = model.full_sequence(CFG, w, tokens, sees_all, use_rope=False)
    masks = y[6:]
    assert np.max(np.abs(masks - masks[0])) < 1e-10
    # with RoPE they differ
    y = model.full_sequence(CFG, w, tokens, sees_all, use_rope=True)
    assert np.max(np.abs(y[6:] - y[6])) > 1e-4


def test_real_rows_are_causal_and_mask_rows_see_later_positions():
    w = _weights(CFG, 5)
    tokens, sees_all = _seq(CFG, 10, 0, 9)
    y0 = model.full_sequence(CFG, w, tokens, sees_all)
    t2 = tokens.copy(); t2[6] = (t2[6] + 1) % CFG.n_plain_tokens
    y1 = model.full_sequence(CFG, w, t2, sees_all)
    assert np.max(np.abs(y0[:6] - y1[:6])) == 0.0
    assert np.max(np.abs(y0[6:] - y1[6:])) > 1e-6
    # a mask row placed before real tokens is not possible in the round, but a mask row sees the
    # later mask rows: editing the LAST row's token changes the first mask row's output
    tokens, sees_all = _seq(CFG, 5, 4, 10)
    y0 = model.full_sequence(CFG, w, tokens, sees_all)
    t2 = tokens.copy(); t2[-1] = 3
    y1 = model.full_sequence(CFG, w, t2, sees_all)
    assert np.max(np.abs(y0[5] - y1[5])) > 1e-6
    assert np.max(np.abs(y0[:5] - y1[:5])) == 0.0


def test_rmsnorm_and_silu_closed_forms():
    x = np.array([[3.0, 4.0]])
    out = model.rmsnorm(x, np.array([2.0, 0.5], dtype=np.float32), 0.0)
    rms = np.sqrt(12.5)
    assert np.allclose(out, [[3 / rms * 2, 4 / rms * 0.5]])
    assert np.isclose(model.silu(np.array([0.0]))[0], 0.0)
    assert np.isclose(model.silu(np.array([2.0]))[0], 2.0 / (1 + np.exp(-2.0)))
    assert np.isclose(model.silu(np.array([-30.0]))[0], -30.0 * np.exp(-30.0), rtol=1e-6)


def test_bf16_rounding_helper_is_nearest_even():
    x = np.array([1.0, 1.0 + 2 ** -8, 1.0 + 2 ** -7, 1.0 + 3 * 2 ** -8, -2.5, 3.3895314e38], dtype=np.float32)
    r = synth.round_to_bf16(x)
    assert r[0] == 1.0 and r[1] == 1.0 and r[2] == 1.0 + 2 ** -7 and r[3] == 1.0 + 2 ** -6
    assert r[4] == -2.5
    back = torch.from_numpy(x[:5]).to(torch.bfloat16).to(torch.float32).numpy()
    assert np.array_equal(back, r[:5])
