"""Helpers for the GPU parity tests: move seeded inputs to the device and wrap the C-ABI calls.

PyTorch only allocates device memory here; all arithmetic happens inside libdiffuspec.so.
"""
from __future__ import annotations

import numpy as np
import torch

from paper_2510_02358_amd import binding as ds
from paper_2510_02358_amd import synth

DEV = "cuda:0"


def to_dev(a: np.ndarray, bf16: bool = False) -> torch.Tensor:
    """numpy -> device tensor; bf16=True stores the (already bf16-exact) fp32 values as bfloat16."""
    if bf16:
        bits = synth.f32_to_bf16_bits(a).reshape(a.shape)
        return torch.from_numpy(bits.view(np.int16)).to(DEV).view(torch.bfloat16)
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def from_dev(t: torch.Tensor) -> np.ndarray:
    if t.dtype == torch.bfloat16:
        return t.float().cpu().numpy()
    return t.cpu().numpy()


class GpuModel:
    """A model handle plus the device buffers it needs (weights, packed weights, KV cache, workspace)."""

    def __init__(self, cfg, weights: dict, kv_capacity: int, max_rows: int = ds.DS_MAX_ROWS):
        self.cfg = cfg
        bf = cfg.dtype == "bf16"
        self.dev_w = {
            "embed": to_dev(weights["embed"], bf), "lm_head": to_dev(weights["lm_head"], bf),
            "final_norm": to_dev(weights["final_norm"]), "layers": [],
        }
        for lw in weights["layers"]:
            d = {n: to_dev(lw[n], bf) for n in synth.LAYER_TENSORS}
            d["norm1"] = to_dev(lw["norm1"])
            d["norm2"] = to_dev(lw["norm2"])
            self.dev_w["layers"].append(d)
        self.cfgc = ds.make_cfg(cfg, kv_capacity)
        pbytes = ds.ds_model_packed_bytes(self.cfgc)
        self.packed = torch.empty(max(pbytes, 256), dtype=torch.uint8, device=DEV)
        kvb = ds.ds_kv_bytes(self.cfgc)
        self.kv_k = torch.empty(kvb, dtype=torch.uint8, device=DEV)
        self.kv_v = torch.empty(kvb, dtype=torch.uint8, device=DEV)
        self.ws = torch.empty(ds.ds_workspace_bytes(self.cfgc, max_rows), dtype=torch.uint8, device=DEV)
        self.handle = ds.ds_model_create(self.cfgc, self.dev_w, self.packed if pbytes else None, self.kv_k, self.kv_v)
        torch.cuda.synchronize()
        if bf:  # canonical matrices other than the embedding are no longer needed
            for d in self.dev_w["layers"]:
                for n in synth.LAYER_TENSORS:
                    d[n] = None
            self.dev_w["lm_head"] = None
        self.torch_dtype = torch.bfloat16 if bf else torch.float32

    def close(self):
        if self.handle:
            ds.ds_model_destroy(self.handle)
            self.handle = None

    @property
    def kv_len(self) -> int:
        return ds.ds_model_kv_len(self.handle)

    def set_kv_len(self, n: int) -> None:
        ds.ds_model_kv_set_len(self.handle, n)

    def prefill(self, tokens: np.ndarray, want_logits: bool = True):
        t = to_dev(np.asarray(tokens, dtype=np.int32))
        out = torch.empty(self.cfg.vocab, dtype=torch.float32, device=DEV) if want_logits else None
        ds.ds_prefill(self.handle, t, len(tokens), out, self.ws)
        torch.cuda.synchronize()
        return from_dev(out) if want_logits else None

    def draft(self, pending, k: int) -> torch.Tensor:
        p = to_dev(np.asarray(pending, dtype=np.int32)) if len(pending) else None
        hid = torch.empty(k, self.cfg.d_model, dtype=torch.float32, device=DEV)
        ds.ds_draft_block(self.handle, p, len(pending), k, self.cfg.mask_id, hid, self.ws)
        return hid

    def lm_head(self, hidden: torch.Tensor) -> torch.Tensor:
        rows = hidden.shape[0]
        logits = torch.empty(rows, self.cfg.vocab, dtype=torch.float32, device=DEV)
        ds.ds_lm_head(self.handle, hidden, rows, logits, self.ws)
        return logits

    def draft_lattice(self, hidden, rows: int, m_max: int, tau: float, eos_id: int, want_logits: bool = True) -> dict:
        """ds_draft_lattice; hidden None = the block rows of the preceding draft pass.  Device tensors."""
        out = {
            "cand_id": torch.empty(rows, m_max, dtype=torch.int32, device=DEV),
            "cand_logp": torch.empty(rows, m_max, dtype=torch.float32, device=DEV),
            "cand_cnt": torch.empty(rows, dtype=torch.int32, device=DEV),
            "eos_logp": torch.empty(rows, dtype=torch.float32, device=DEV),
            "lse": torch.empty(rows, dtype=torch.float32, device=DEV),
        }
        logits = torch.empty(rows, self.cfg.vocab, dtype=torch.float32, device=DEV) if want_logits else None
        ds.ds_draft_lattice(self.handle, hidden, rows, m_max, tau, eos_id, out["cand_id"], out["cand_logp"],
                            out["cand_cnt"], out["eos_logp"], out["lse"], logits, self.ws)
        torch.cuda.synchronize()
        return out, logits

    def verify(self, block, path_len=None, eos_id: int = -1, want_logits: bool = True):
        blk = block if isinstance(block, torch.Tensor) else to_dev(np.asarray(block, dtype=np.int32))
        rows = blk.shape[0]
        out = torch.zeros(3, dtype=torch.int32, device=DEV)
        am = torch.empty(rows, dtype=torch.int32, device=DEV)
        logits = torch.empty(rows, self.cfg.vocab, dtype=torch.float32, device=DEV) if want_logits else None
        ds.ds_verify_block(self.handle, blk, rows - 1, path_len, eos_id, out[0:1], out[1:2], am, out[2:3], logits,
                           self.ws)
        torch.cuda.synchronize()
        o = out.cpu().numpy()
        return {"n_accept": int(o[0]), "next_token": int(o[1]), "eos_accepted": int(o[2]),
                "argmax": am.cpu().numpy(), "logits": from_dev(logits) if want_logits else None}


def gpu_lattice(logits: torch.Tensor, m_max: int, tau: float, eos_id: int) -> dict:
    rows, vocab = logits.shape
    out = {
        "cand_id": torch.empty(rows, m_max, dtype=torch.int32, device=DEV),
        "cand_logp": torch.empty(rows, m_max, dtype=torch.float32, device=DEV),
        "cand_cnt": torch.empty(rows, dtype=torch.int32, device=DEV),
        "eos_logp": torch.empty(rows, dtype=torch.float32, device=DEV),
        "lse": torch.empty(rows, dtype=torch.float32, device=DEV),
    }
    ws = torch.empty(ds.ds_lattice_workspace_bytes(rows, vocab, m_max), dtype=torch.uint8, device=DEV)
    ds.ds_build_lattice(logits, rows, vocab, m_max, tau, eos_id, out["cand_id"], out["cand_logp"], out["cand_cnt"],
                        out["eos_logp"], out["lse"], ws)
    torch.cuda.synchronize()
    return out


def gpu_cps(lat: dict, batch: int, k: int, m_max: int, beam: int, lam: float, table, log2_size: int, ctx, eos_id: int,
            with_ws: bool = True):
    """lat: dict of device tensors (or numpy arrays, uploaded here).  Returns numpy (path, path_len, score)."""
    d = {n: (v if isinstance(v, torch.Tensor) else to_dev(v)) for n, v in lat.items()}
    path = torch.empty(batch, k, dtype=torch.int32, device=DEV)
    plen = torch.empty(batch, dtype=torch.int32, device=DEV)
    score = torch.empty(batch, dtype=torch.float32, device=DEV)
    proxy = ds.ds_ngram_create(table, log2_size) if table is not None else None
    ctx_d = ctx if isinstance(ctx, torch.Tensor) else to_dev(np.asarray(ctx, dtype=np.int32))
    ws = torch.empty(ds.ds_cps_workspace_bytes(batch, k, m_max), dtype=torch.uint8, device=DEV) if with_ws else None
    ds.ds_cps_path(d["cand_id"], d["cand_logp"], d["cand_cnt"], d["eos_logp"], batch, k, m_max, beam, lam, proxy,
                   ctx_d, eos_id, path, plen, score, ws)
    torch.cuda.synchronize()
    if proxy:
        ds.ds_ngram_destroy(proxy)
    return path.cpu().numpy(), plen.cpu().numpy(), score.cpu().numpy()
