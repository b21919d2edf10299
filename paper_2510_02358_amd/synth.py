"""Seeded synthetic inputs shared by the tests, the benchmark and the smoke run.

This module only *generates data*: configuration records, random-init weights,
random token prefixes, Gaussian logit blocks and the table behind the causal
proxy.  It contains none of the method's arithmetic (no forward pass, no
softmax, no search, no acceptance rule), so that the CPU oracle and the HIP
path can both be fed from it without sharing any logic.

Everything is drawn from numpy's PCG64 generator with a fixed seed and a fixed
draw order, so the same call always returns the same bytes.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Dict, List

import numpy as np


@dataclass(frozen=True)
class ModelCfg:
    """Shape of one pre-RMSNorm decoder (GQA attention, SwiGLU MLP, RoPE)."""

    n_layers: int
    d_model: int
    n_q: int
    n_kv: int
    head_dim: int
    d_ffn: int
    vocab: int
    rope_base: float
    rms_eps: float = 1e-6
    dtype: str = "bf16"  # "f32" or "bf16": storage type of weights / KV cache

    @property
    def mask_id(self) -> int:
        return self.vocab - 1

    @property
    def eos_id(self) -> int:
        return self.vocab - 2

    @property
    def n_plain_tokens(self) -> int:
        """Ordinary tokens are drawn from [0, vocab-2); the top two ids are EOS and MASK."""
        return self.vocab - 2


# The two model shapes the workloads use (tiny fp32 pair, 7B-shaped bf16 layer).
CFG_TINY = ModelCfg(n_layers=2, d_model=256, n_q=4, n_kv=4, head_dim=64, d_ffn=688,
                    vocab=4096, rope_base=1.0e4, dtype="f32")
CFG_7B_LAYER = ModelCfg(n_layers=1, d_model=3584, n_q=28, n_kv=4, head_dim=128, d_ffn=18944,
                        vocab=152064, rope_base=1.0e6, dtype="bf16")
CFG_32B_LAYER = ModelCfg(n_layers=1, d_model=5120, n_q=40, n_kv=8, head_dim=128, d_ffn=27648,
                         vocab=152064, rope_base=1.0e6, dtype="bf16")


def with_layers(cfg: ModelCfg, n_layers: int) -> ModelCfg:
    return replace(cfg, n_layers=n_layers)


# ----------------------------------------------------------------------------------------------
# bf16 helpers (storage conversion only)
# ----------------------------------------------------------------------------------------------

def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round fp32 to bf16 (nearest, ties to even); returns the uint16 bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rounded = u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """fp32 array whose every value is exactly representable in bf16."""
    return bf16_bits_to_f32(f32_to_bf16_bits(x))


# ----------------------------------------------------------------------------------------------
# weights
# ----------------------------------------------------------------------------------------------

LAYER_TENSORS = ("wq", "wk", "wv", "wo", "w_gate", "w_up", "w_down")


def layer_shapes(cfg: ModelCfg) -> Dict[str, tuple]:
    d, hq, hkv, hd, f = cfg.d_model, cfg.n_q, cfg.n_kv, cfg.head_dim, cfg.d_ffn
    return {
        "wq": (hq * hd, d), "wk": (hkv * hd, d), "wv": (hkv * hd, d), "wo": (d, hq * hd),
        "w_gate": (f, d), "w_up": (f, d), "w_down": (d, f),
    }


def make_weights(cfg: ModelCfg, seed: int, std: float = 0.02) -> dict:
    """Random-init weights, every matrix ~ N(0, std^2), norm gains = 1, no biases.

    Draw order: embed, then per layer wq, wk, wv, wo, w_gate, w_up, w_down, then lm_head.
    All matrices are row-major [out_features, in_features].  For a bf16 config the
    values are rounded to bf16 once here, so that both consumers see identical numbers;
    they are still returned as fp32 arrays (use `f32_to_bf16_bits` for device upload).
    """
    rng = np.random.Generator(np.random.PCG64(seed))

    def draw(shape):
        w = rng.standard_normal(shape, dtype=np.float32)
        w *= np.float32(std)
        return round_to_bf16(w) if cfg.dtype == "bf16" else w

    out = {"embed": draw((cfg.vocab, cfg.d_model)), "layers": []}
    shapes = layer_shapes(cfg)
    for _ in range(cfg.n_layers):
        lw = {name: draw(shapes[name]) for name in LAYER_TENSORS}
        lw["norm1"] = np.ones(cfg.d_model, dtype=np.float32)
        lw["norm2"] = np.ones(cfg.d_model, dtype=np.float32)
        out["layers"].append(lw)
    out["final_norm"] = np.ones(cfg.d_model, dtype=np.float32)
    out["lm_head"] = draw((cfg.vocab, cfg.d_model))
    return out


def randomize_norm_gains(weights: dict, seed: int) -> None:
    """Replace the all-ones norm gains by U[0.5, 1.5] draws (bf16-exact), in place.

    Not used by the benchmark workloads; tests use it so that a dropped or misplaced
    gain cannot hide behind gain == 1.
    """
    rng = np.random.Generator(np.random.PCG64(seed))

    def gains(n):
        return round_to_bf16(rng.uniform(0.5, 1.5, n).astype(np.float32))

    for lw in weights["layers"]:
        lw["norm1"] = gains(lw["norm1"].shape[0])
        lw["norm2"] = gains(lw["norm2"].shape[0])
    weights["final_norm"] = gains(weights["final_norm"].shape[0])


# ----------------------------------------------------------------------------------------------
# tokens, logits, proxy table
# ----------------------------------------------------------------------------------------------

def make_prefix(cfg: ModelCfg, n: int, seed: int) -> np.ndarray:
    """n ordinary token ids, uniform on [0, vocab-2)."""
    rng = np.random.Generator(np.random.PCG64(seed))
    return rng.integers(0, cfg.n_plain_tokens, size=n, dtype=np.int64).astype(np.int32)


def make_logits(batch: int, k: int, vocab: int, seed: int) -> np.ndarray:
    """fp32 logits [batch*k, vocab] = g / T, g ~ N(0,1), one temperature T ~ U[0.5, 2] per row."""
    rng = np.random.Generator(np.random.PCG64(seed))
    rows = batch * k
    temp = rng.uniform(0.5, 2.0, size=rows).astype(np.float32)
    out = np.empty((rows, vocab), dtype=np.float32)
    for r in range(rows):
        out[r] = rng.standard_normal(vocab, dtype=np.float32) / temp[r]
    return out


NGRAM_LOG2_SIZE = 22


def make_ngram_table(seed: int = 3, log2_size: int = NGRAM_LOG2_SIZE) -> np.ndarray:
    """Stand-in for a fitted 3-gram model: 2^log2_size natural-log scores.

    Values are 4*ln(u), u ~ U(0,1], clipped below at -20 (mean about -4 nats).
    """
    rng = np.random.Generator(np.random.PCG64(seed))
    u = 1.0 - rng.random(1 << log2_size)  # (0, 1]
    t = 4.0 * np.log(u)
    return np.maximum(t, -20.0).astype(np.float32)


def make_contexts(cfg_vocab: int, batch: int, seed: int) -> np.ndarray:
    """[batch, 2] ordinary tokens that precede each draft block (the proxy's left context)."""
    rng = np.random.Generator(np.random.PCG64(seed))
    return rng.integers(0, cfg_vocab - 2, size=(batch, 2), dtype=np.int64).astype(np.int32)


def layer_param_count(cfg: ModelCfg) -> int:
    return int(sum(int(np.prod(s)) for s in layer_shapes(cfg).values()))


def workload_list() -> List[str]:
    return ["cfg0_tiny_f32_round", "cfg1_7b_layer_bf16_round", "cfg3_lattice_cps"]
