"""Host-side driver of the speculative loop (Alg. 1): chains the C-ABI calls of one round and keeps the
bookkeeping (committed KV lengths, pending tokens, draft length).  No arithmetic of the method happens
here: drafting, lattice, path search, verification and acceptance all run inside libdiffuspec.so, and the
draft-length controller is the library's host function.

PyTorch is used for device memory only.
"""
from __future__ import annotations

import ctypes
import time
from dataclasses import dataclass
from typing import List, Optional

import numpy as np
import torch

from . import binding as ds
from . import synth

DEV = "cuda:0"


def upload(a, bf16: bool = False) -> torch.Tensor:
    if isinstance(a, torch.Tensor):  # already on the device (weights drawn there for the deep workloads)
        return a
    if bf16:
        bits = synth.f32_to_bf16_bits(a).reshape(a.shape)
        return torch.from_numpy(bits.view(np.int16)).to(DEV).view(torch.bfloat16)
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


class DeviceModel:
    """Model handle + its device buffers (weights, stream-order weights, KV cache, workspace)."""

    def __init__(self, cfg: synth.ModelCfg, weights: dict, kv_capacity: int, max_rows: int = ds.DS_MAX_ROWS):
        self.cfg = cfg
        bf = cfg.dtype == "bf16"
        dev_w = {"embed": upload(weights["embed"], bf), "lm_head": upload(weights["lm_head"], bf),
                 "final_norm": upload(weights["final_norm"]), "layers": []}
        for lw in weights["layers"]:
            d = {n: upload(lw[n], bf) for n in synth.LAYER_TENSORS}
            d["norm1"], d["norm2"] = upload(lw["norm1"]), upload(lw["norm2"])
            dev_w["layers"].append(d)
        self.cfgc = ds.make_cfg(cfg, kv_capacity)
        pbytes = ds.ds_model_packed_bytes(self.cfgc)
        self.packed = torch.empty(max(pbytes, 256), dtype=torch.uint8, device=DEV)
        kvb = ds.ds_kv_bytes(self.cfgc)
        self.kv_k = torch.zeros(kvb, dtype=torch.uint8, device=DEV)
        self.kv_v = torch.zeros(kvb, dtype=torch.uint8, device=DEV)
        self.ws = torch.empty(ds.ds_workspace_bytes(self.cfgc, max_rows), dtype=torch.uint8, device=DEV)
        self.handle = ds.ds_model_create(self.cfgc, dev_w, self.packed if pbytes else None, self.kv_k, self.kv_v)
        torch.cuda.synchronize()
        if bf:  # after packing only the embedding and the norm gains are still read
            for d in dev_w["layers"]:
                for n in synth.LAYER_TENSORS:
                    d[n] = None
            dev_w["lm_head"] = None
        self.dev_w = dev_w
        self.torch_dtype = torch.bfloat16 if bf else torch.float32

    def close(self) -> None:
        for kv, _, _ in getattr(self, "sequences", []):
            ds.ds_kv_destroy(kv)
        self.sequences = []
        if self.handle:
            ds.ds_model_destroy(self.handle)
            self.handle = None

    def new_sequence(self) -> int:
        """One more sequence's KV cache of this model (for the batched calls); returns its ds_kv handle."""
        kvb = ds.ds_kv_bytes(self.cfgc)
        k = torch.zeros(kvb, dtype=torch.uint8, device=DEV)
        v = torch.zeros(kvb, dtype=torch.uint8, device=DEV)
        kv = ds.ds_kv_create(self.handle, k, v)
        if not hasattr(self, "sequences"):
            self.sequences = []
        self.sequences.append((kv, k, v))
        return kv

    @property
    def kv_len(self) -> int:
        return ds.ds_model_kv_len(self.handle)

    def set_kv_len(self, n: int) -> None:
        ds.ds_model_kv_set_len(self.handle, n)


@dataclass
class RoundParams:
    m_max: int = 8
    tau: float = 1.0
    beam: int = 4
    lam: float = 0.5
    k_min: int = 4
    k_max: int = 64
    delta: float = 10.0
    rho: float = 0.5
    refine_steps: int = 1  # drafter passes per round (1: the single-pass round)


_hip_rt = None


def _hip_memcpy_h2d_async(dst_dev: int, src_pinned: int, n_bytes: int) -> None:
    """hipMemcpyAsync(host -> device) on the default stream, called directly: the per-round staging copy is on the
    host's critical path between a verdict and the next round's first launch, where a tensor-level copy_ costs several
    microseconds of dispatch."""
    global _hip_rt
    if _hip_rt is None:
        _hip_rt = ctypes.CDLL("libamdhip64.so")
        _hip_rt.hipMemcpyAsync.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int,
                                           ctypes.c_void_p]
        _hip_rt.hipMemcpyAsync.restype = ctypes.c_int
    rc = _hip_rt.hipMemcpyAsync(dst_dev, src_pinned, n_bytes, 1, None)
    if rc != 0:
        raise RuntimeError(f"hipMemcpyAsync failed with code {rc}")


class SpecDecoder:
    """One drafter + one verifier on one GPU, both caches holding the same prefix."""

    def __init__(self, drafter: DeviceModel, verifier: DeviceModel, table: Optional[np.ndarray], log2_size: int,
                 params: RoundParams, k_cap: int = 64, keep_draft_logits: bool = False,
                 keep_verify_logits: bool = False, lm_proxy: Optional[DeviceModel] = None):
        """lm_proxy: a small model of the same vocabulary that serves as the path search's causal proxy in place of
        the n-gram table (`table` is then ignored).  keep_draft_logits: also write the drafter's logits to `d_logits` every round (the lattice does not need
        them in memory; stochastic verification does and gets them regardless).  keep_verify_logits: also write the
        verifier's logits of the block rows to `v_logits` (tests compare them with the oracle's)."""
        if not 1 <= k_cap < ds.DS_MAX_ROWS:
            raise ValueError(f"k_cap {k_cap} outside [1, {ds.DS_MAX_ROWS})")
        if params.k_max > k_cap:
            raise ValueError(f"params.k_max {params.k_max} exceeds k_cap {k_cap}: every per-round buffer is sized "
                             "by k_cap")
        self.d, self.v, self.p = drafter, verifier, params
        self.keep_draft_logits = keep_draft_logits
        self.v_logits = (torch.empty(k_cap + 1, verifier.cfg.vocab, dtype=torch.float32, device=DEV)
                         if keep_verify_logits else None)
        self.eos_id = drafter.cfg.eos_id
        self.mask_id = drafter.cfg.mask_id
        vocab = drafter.cfg.vocab
        self.table = upload(table) if table is not None else None
        self.proxy = ds.ds_ngram_create(self.table, log2_size) if table is not None else None
        self.lm, self.lm_proxy, self.lm_mem = lm_proxy, None, None
        if lm_proxy is not None:
            if params.beam > 8:
                raise ValueError("the LM proxy carries at most 8 beam slots")
            self.lm_mem = torch.empty(ds.ds_lmproxy_bytes(lm_proxy.cfgc, params.beam), dtype=torch.uint8, device=DEV)
            self.lm_proxy = ds.ds_lmproxy_create(lm_proxy.handle, params.beam, self.lm_mem)
        self.adl = ds.ds_adl_create(params.k_min, params.k_max, params.delta, params.rho)
        m = params.m_max
        i32, f32 = torch.int32, torch.float32
        self.hidden = torch.empty(k_cap, drafter.cfg.d_model, dtype=torch.float32, device=DEV)
        self.d_logits = torch.empty(k_cap, vocab, dtype=f32, device=DEV)
        self.cand_logp = torch.empty(k_cap, m, dtype=f32, device=DEV)
        self.cand_cnt = torch.empty(k_cap, dtype=i32, device=DEV)
        self.eos_logp = torch.empty(k_cap, dtype=f32, device=DEV)
        self.lse = torch.empty(k_cap, dtype=f32, device=DEV)
        self.cps_ws = torch.empty(ds.ds_cps_workspace_bytes(1, k_cap, m), dtype=torch.uint8, device=DEV)
        # Everything the host sends per round (pending tokens, proxy context) and reads back per round (searched path,
        # its length, the candidate ids) lives in ONE device tensor, so that a round costs one host -> device and one
        # device -> host copy:   [pending, right-aligned | ctx0 | ctx1 = block[0] | path ... | path_len | pad | cand_id]
        # The last committed token is both the newer context token and the first row of the verify block.
        # (the layout the library's own round loop uses: ds_round_io_layout)
        P = ds.DS_MAX_ROWS
        self._p = P
        self._out0, self._len_at, self._cand_at, io_total = ds.ds_round_io_layout(k_cap, m)   # first int read back, ...
        self.io = torch.zeros(io_total, dtype=i32, device=DEV)
        self.ctx = self.io[P:P + 2]
        self.block = self.io[P + 1:P + 2 + k_cap]             # [last token, path...]
        self.path_len = self.io[self._len_at:self._len_at + 1]
        self.cand_id = self.io[self._cand_at:].view(k_cap, m)
        self.path_score = torch.zeros(1, dtype=f32, device=DEV)
        # n_accept, next_token, eos_accepted: pinned host memory (device-visible), so that the acceptance kernel
        # writes the round's verdict where the host reads it after the stream sync, without a copy in between
        self.result = torch.zeros(3, dtype=i32).pin_memory()
        self.result_np = self.result.numpy()
        self.argmax = torch.empty(k_cap + 1, dtype=i32, device=DEV)
        # multi-pass refinement: current draft y^(s) and the lattice frozen row by row
        self.blk = torch.zeros(k_cap, dtype=i32, device=DEV)
        self.f_cand_id = torch.empty(k_cap, m, dtype=i32, device=DEV)
        self.f_cand_logp = torch.empty(k_cap, m, dtype=f32, device=DEV)
        self.f_cand_cnt = torch.empty(k_cap, dtype=i32, device=DEV)
        self.f_eos_logp = torch.empty(k_cap, dtype=f32, device=DEV)
        self.f_lse = torch.empty(k_cap, dtype=f32, device=DEV)
        # stochastic verification: uniforms in, acceptance probabilities out
        self.u = torch.zeros(k_cap + 1, dtype=f32, device=DEV)
        self.alpha = torch.zeros(k_cap, dtype=f32, device=DEV)
        self.host = torch.empty(2 + ds.DS_MAX_ROWS, dtype=i32).pin_memory()
        self.host_np = self.host.numpy()
        self._host_ptr, self._io_ptr = self.host.data_ptr(), self.io.data_ptr()
        self.host_out = torch.empty(self.io.numel() - self._out0, dtype=i32).pin_memory()   # io[_out0:] as the host sees it
        self.host_out_np = self.host_out.numpy()
        self._host_out_ptr = self.host_out.data_ptr()
        self._cand_host_ptr = self._host_out_ptr + 4 * (self._cand_at - self._out0)
        self.host_raw0 = torch.empty(k_cap, dtype=i32).pin_memory()          # refinement rounds: the final lattice's top-1
        self.k_cap = k_cap
        self._desc = None
        self._mirrored = False
        self.tokens: List[int] = []
        self.pending: List[int] = []
        self._carried = False  # True: the device already holds the next round's pending tokens and context

    def close(self) -> None:
        if self.proxy:
            ds.ds_ngram_destroy(self.proxy)
            self.proxy = None
        if self.adl:
            ds.ds_adl_destroy(self.adl)
            self.adl = None
        if self.lm_proxy:
            ds.ds_lmproxy_destroy(self.lm_proxy)
            self.lm_proxy = None

    def start(self, prefix: np.ndarray) -> None:
        """Prefill both caches with the prefix; the verifier's greedy token after it becomes pending."""
        t = upload(np.asarray(prefix, dtype=np.int32))
        last = torch.empty(self.v.cfg.vocab, dtype=torch.float32, device=DEV)
        self.d.set_kv_len(0)
        self.v.set_kv_len(0)
        ds.ds_prefill(self.d.handle, t, len(prefix), None, self.d.ws)
        ds.ds_prefill(self.v.handle, t, len(prefix), last, self.v.ws)
        if self.lm_proxy:
            ds.ds_lmproxy_set_len(self.lm_proxy, 0)
            ds.ds_lmproxy_prefill(self.lm_proxy, t, len(prefix), self.lm.ws)
        # first pending token = verifier arg-max after the prefix: a verify call with an empty path
        # would need the token before it; the arg-max of `last` is taken by the acceptance kernel
        # through a 1-row lattice (top-1, ties to the lower id)
        cid = torch.empty(1, 1, dtype=torch.int32, device=DEV)
        clp = torch.empty(1, 1, dtype=torch.float32, device=DEV)
        tmp_i = torch.empty(1, dtype=torch.int32, device=DEV)
        tmp_f = torch.empty(2, dtype=torch.float32, device=DEV)
        ws = torch.empty(ds.ds_lattice_workspace_bytes(1, self.v.cfg.vocab, 1), dtype=torch.uint8, device=DEV)
        ds.ds_build_lattice(last, 1, self.v.cfg.vocab, 1, 1.0, -1, cid, clp, tmp_i, tmp_f[0:1], tmp_f[1:2], ws)
        torch.cuda.synchronize()
        first = int(cid.item())
        self.tokens = [int(x) for x in prefix] + [first]
        self.pending = [first]
        self._carried = False

    def enqueue_round(self, k: int, stream=None, inject=None, uniforms=None, readback: bool = False,
                      lm_events=None) -> None:
        """Enqueue draft -> LM head -> lattice -> path search -> verify for the current state.  No sync.

        inject = (device int32 tensor, a): overwrite the first `a` searched path tokens with these tokens before
        verification and let all k block positions take part in acceptance (synthetic acceptance for benchmarks
        and tests; plain device copies).
        uniforms = device float32 tensor [k + 1]: verify with the stochastic acceptance rule instead of greedy
        (u[i] decides draft token i + 1, u[k] drives the replacement / bonus draw).
        readback: also copy the searched path, its length and the candidate ids to pinned host memory; the copy is
        issued BEFORE the verifier pass (everything it reads is final by then), so it is long done when the verdict
        arrives and the round's host crossing is the verdict alone.
        lm_events = (start, end) torch events: recorded around the drafter's LM-head product alone (the two-call form
        of ds_draft_lattice; same kernels), for benchmarks that report that kernel's time.
        """
        p = self.p
        n_pend = len(self.pending)
        if not 1 <= k <= self.k_cap:
            raise ValueError(f"draft length {k} outside [1, k_cap = {self.k_cap}]")
        if n_pend + k > ds.DS_MAX_ROWS:
            raise ValueError(f"{n_pend} pending + {k} draft rows exceed {ds.DS_MAX_ROWS} rows per call")
        lat = (self.cand_id, self.cand_logp, self.cand_cnt, self.eos_logp, self.lse)
        sizes = ds.ds_refine_update_sizes(k, p.refine_steps) if p.refine_steps > 1 else [k]
        logits_out = self.d_logits if (self.keep_draft_logits or uniforms is not None) else None
        if len(sizes) <= 1:
            ds.ds_draft_block(self.d.handle, self.pending_dev, n_pend, k, self.mask_id, self.hidden, self.d.ws, stream)
            if lm_events is None:
                ds.ds_draft_lattice(self.d.handle, None, k, p.m_max, p.tau, self.eos_id, *lat, logits_out, self.d.ws,
                                    stream)
            else:
                lm_events[0].record()
                ds.ds_lm_head_tiles(self.d.handle, None, k, self.eos_id, logits_out, self.d.ws, stream)
                lm_events[1].record()
                ds.ds_lattice_from_tiles(self.d.handle, k, p.m_max, p.tau, self.eos_id, *lat, self.d.ws, stream)
        else:
            self.blk[:k].fill_(self.mask_id)
            final = (self.f_cand_id, self.f_cand_logp, self.f_cand_cnt, self.f_eos_logp, self.f_lse)
            for s, n in enumerate(sizes):
                ds.ds_draft_block_tokens(self.d.handle, self.pending_dev if s == 0 else None, n_pend if s == 0 else 0,
                                         self.blk, k, self.hidden, self.d.ws, stream)
                ds.ds_draft_lattice(self.d.handle, None, k, p.m_max, p.tau, self.eos_id, *lat, logits_out, self.d.ws,
                                    stream)
                ds.ds_refine_select(*lat, k, p.m_max, n, self.mask_id, self.blk, *final, stream)
            lat = final
        # what the host reads besides the verdict: the search kernel mirrors path, length and raw draft into pinned
        # host memory itself; rounds that change the path afterwards (injection) or search with the LM proxy copy
        self._mirrored = readback and inject is None and not self.lm_proxy
        if self.lm_proxy:  # the proxy reads the same pending tokens as the drafter did
            ds.ds_cps_path_lm(lat[0], lat[1], lat[2], lat[3], k, p.m_max, p.beam, p.lam, self.lm_proxy,
                              self.pending_dev, n_pend, self.eos_id, self.block[1:], self.path_len, self.path_score,
                              self.lm.ws, stream)
        else:
            ds.ds_cps_path(lat[0], lat[1], lat[2], lat[3], 1, k, p.m_max, p.beam, p.lam, self.proxy, self.ctx,
                           self.eos_id, self.block[1:], self.path_len, self.path_score, self.cps_ws, stream,
                           host_mirror=self.host_out if self._mirrored else None)
        self.lat_used = lat
        if inject is not None and inject[1] > 0:
            self.block[1:1 + inject[1]].copy_(inject[0][:inject[1]], non_blocking=True)
            self.path_len.fill_(k)  # the searched path may have stopped at an EOS before the injected length
        if readback and not self._mirrored:
            self.host_out.copy_(self.io[self._out0:], non_blocking=True)
            if lat[0] is not self.cand_id:  # refinement rounds keep the final lattice elsewhere
                self.host_raw0[:k].copy_(lat[0][:k, 0], non_blocking=True)
        if uniforms is None:
            # the acceptance kernel itself leaves the committed tokens where the next round's drafter pass, path
            # search and verify block read them (io[: P + 2]): no token travels host -> device between rounds
            ds.ds_verify_block_carry(self.v.handle, self.block, k, self.path_len, self.eos_id, self.result[0:1],
                                     self.result[1:2], self.argmax, self.result[2:3], self.v_logits, self.io,
                                     self.v.ws, stream)
            self._carried = True
        else:
            # the drafter rows of the path positions: with one drafter pass, the logits the lattice was built from
            ds.ds_verify_block_stochastic(self.v.handle, self.block, k, self.path_len, self.d_logits, uniforms,
                                          self.eos_id, self.result[0:1], self.result[1:2], self.result[2:3],
                                          self.alpha, self.v_logits, self.v.ws, stream)

    @property
    def pending_dev(self) -> torch.Tensor:
        """Device view of the pending tokens (the tokens committed since the drafter last ran)."""
        return self.io[self._p - len(self.pending):self._p]

    _PENDING = -0x7EADBEEF  # sentinel the host leaves in result[2] (eos_accepted is 0 or 1)

    def arm_verdict(self) -> None:
        """Before enqueueing a round: mark the verdict as outstanding (plain host store into pinned memory)."""
        self.result_np[2] = self._PENDING

    def wait_verdict(self, limit_s: float = 10.0) -> None:
        """The round's host crossing: poll the word the acceptance kernel stores last (after a system-scope fence)
        in the pinned verdict buffer.  Cheaper than a stream synchronisation by several microseconds; bounded, and
        it falls back to a synchronisation (which surfaces any device error) when the bound is hit."""
        res, t0, spins = self.result_np, None, 0
        while res[2] == self._PENDING:
            spins += 1
            if (spins & 0xFFFF) == 0:
                now = time.perf_counter()
                t0 = t0 or now
                if now - t0 > limit_s:
                    torch.cuda.current_stream().synchronize()
                    if res[2] == self._PENDING:
                        raise RuntimeError("no verdict from the acceptance kernel within %.0f s" % limit_s)

    def stage_inputs(self) -> None:
        """Host -> device: pending tokens and the proxy context (whose newer token is also the first row of the
        verify block): a few ints, one async copy."""
        self._carried = False
        n = len(self.pending)
        h = self.host_np
        h[:n] = self.pending
        h[n] = self.tokens[-2]
        h[n + 1] = self.tokens[-1]
        _hip_memcpy_h2d_async(self._io_ptr + 4 * (self._p - n), self._host_ptr, 4 * (n + 2))

    def round(self, k: int, inject=None, uniforms=None, lm_events=None) -> dict:
        """One full round including the host read-back, KV commit and the draft-length update."""
        if not self._carried:  # first round, or the last verdict came from a call that carries nothing
            self.stage_inputs()
        self._carried = False
        v_len = self.v.kv_len
        if uniforms is not None:
            if self.p.refine_steps > 1:
                raise ValueError("stochastic verification needs the single-pass draft (its rows are the left-to-right "
                                 "proxy's distribution)")
            self.u[:k + 1].copy_(uniforms if isinstance(uniforms, torch.Tensor)
                                 else torch.from_numpy(np.asarray(uniforms, dtype=np.float32)), non_blocking=False)
        self.arm_verdict()
        self.enqueue_round(k, inject=inject, uniforms=self.u if uniforms is not None else None, readback=True,
                           lm_events=lm_events)
        refined = self.lat_used[0] is not self.cand_id
        self.wait_verdict()  # the one host crossing; the path / candidate copy finished during the verifier pass
        out, res = self.host_out_np, self.result_np
        n_acc, nxt, eos = int(res[0]), int(res[1]), int(res[2])
        # the raw draft (per-position top-1 before the search) as the host sees it: s_t of the controller
        if self._mirrored:      # [path k | length | raw draft k]
            plen = int(out[k])
            path = out[:plen].copy()
            first_eos = ds.ds_adl_first_eos(self._host_out_ptr + 4 * (k + 1), k, 1, self.eos_id)
        else:
            plen = int(out[self._len_at - self._out0])
            path = out[:plen].copy()
            if refined:
                first_eos = ds.ds_adl_first_eos(self.host_raw0, k, 1, self.eos_id)
            else:
                first_eos = ds.ds_adl_first_eos(self._cand_host_ptr, k, self.p.m_max, self.eos_id)
        self.v.set_kv_len(v_len + 1 + n_acc)
        committed = [int(t) for t in path[:n_acc]] + [nxt]
        self.tokens += committed
        self.pending = committed
        k_next = ds.ds_adl_update(self.adl, k, first_eos, n_acc)
        return {"k": k, "path": path, "path_len": plen, "n_accept": n_acc, "next_token": nxt, "eos_accepted": eos,
                "committed": committed, "first_eos": first_eos, "k_next": k_next}


    def _round_desc(self) -> "ds.RoundDescC":
        if self._desc is None:
            p, d = self.p, ds.RoundDescC()
            d.drafter, d.verifier, d.proxy, d.adl = self.d.handle, self.v.handle, self.proxy, self.adl
            d.K_cap, d.M_max, d.beam, d.eos_id, d.mask_id = self.k_cap, p.m_max, p.beam, self.eos_id, self.mask_id
            d.tau, d.lam = p.tau, p.lam
            d.hidden, d.cand_logp, d.cand_cnt = self.hidden.data_ptr(), self.cand_logp.data_ptr(), self.cand_cnt.data_ptr()
            d.eos_logp, d.lse, d.io = self.eos_logp.data_ptr(), self.lse.data_ptr(), self.io.data_ptr()
            d.path_score, d.argmax = self.path_score.data_ptr(), self.argmax.data_ptr()
            d.cps_ws, d.cps_ws_bytes = self.cps_ws.data_ptr(), self.cps_ws.numel()
            d.drafter_ws, d.drafter_ws_bytes = self.d.ws.data_ptr(), self.d.ws.numel()
            d.verifier_ws, d.verifier_ws_bytes = self.v.ws.data_ptr(), self.v.ws.numel()
            d.verdict, d.host_out = self.result.data_ptr(), self.host_out.data_ptr()
            self._desc = d
        return self._desc

    def run(self, n_rounds: int, k: int, follow_adl: bool = True, stop_at_eos: bool = True, lm_events=None) -> list:
        """n_rounds rounds inside the library's own loop (ds_rounds_run): greedy verification, single-pass draft,
        n-gram proxy.  The same calls as round(), with the host's per-round work done in C.
        lm_events = (ev_every, [(start, end) torch events, already recorded once so that their handles exist]):
        round j * ev_every records pair j around the drafter's LM-head product.
        Returns one dict per round done (the fields of round())."""
        if self.p.refine_steps > 1 or self.lm_proxy:
            raise ValueError("the library's round loop drives the single-pass draft with the n-gram proxy")
        if n_rounds <= 0:
            return []
        if not self._carried:
            self.stage_inputs()
        self._carried = False
        d = self._round_desc()
        keep = None
        if lm_events is not None:
            every, pairs = lm_events
            n_ev = (n_rounds + every - 1) // every
            if len(pairs) < n_ev:
                raise ValueError(f"{n_rounds} rounds with an event pair every {every} need {n_ev} pairs")
            starts = (ctypes.c_void_p * n_ev)(*[a.cuda_event for a, _ in pairs[:n_ev]])
            ends = (ctypes.c_void_p * n_ev)(*[b.cuda_event for _, b in pairs[:n_ev]])
            d.ev_every, d.ev_start, d.ev_end, keep = every, starts, ends, (starts, ends)
        else:
            d.ev_every = 0
        records = (ds.RoundRecordC * n_rounds)()
        cap = n_rounds * (self.k_cap + 1)
        tokens = np.empty(cap, dtype=np.int32)
        try:
            done, n_tok, _ = ds.ds_rounds_run(d, n_rounds, k, follow_adl, stop_at_eos, len(self.pending), records,
                                              tokens.ctypes.data, cap)
        finally:
            d.ev_every = 0
            del keep
        out, at = [], 0
        for r in records[:done]:
            committed = [int(t) for t in tokens[at:at + r.n_accept + 1]]
            at += r.n_accept + 1
            out.append({"k": r.k, "path_len": r.path_len, "n_accept": r.n_accept, "next_token": r.next_token,
                        "eos_accepted": r.eos_accepted, "committed": committed, "first_eos": r.first_eos,
                        "k_next": r.k_next})
        assert at == n_tok
        self.tokens += [int(t) for t in tokens[:n_tok]]
        if out:
            self.pending = out[-1]["committed"]
            self._carried = True
        return out


class BatchSpecDecoder:
    """n_seq independent sequences driven through the batched calls: every round is one drafter pass, one LM head +
    lattice, one path search and one verifier pass for all of them (one stream of each model's weights), with the
    same draft length K.  Bookkeeping only, as in SpecDecoder; each sequence has its own draft-length controller,
    whose proposals are reported and left to the caller (the batch shares one K)."""

    def __init__(self, drafter: DeviceModel, verifier: DeviceModel, n_seq: int, table: Optional[np.ndarray],
                 log2_size: int, params: RoundParams, k_cap: int = 32, keep_logits: bool = False):
        if not 1 <= n_seq <= ds.DS_MAX_SEQ:
            raise ValueError(f"n_seq {n_seq} outside [1, {ds.DS_MAX_SEQ}]")
        if params.refine_steps != 1:
            raise ValueError("the batched round is the single-pass round")
        self.d, self.v, self.p, self.n, self.k_cap = drafter, verifier, params, n_seq, k_cap
        self.eos_id, self.mask_id = drafter.cfg.eos_id, drafter.cfg.mask_id
        self.d_kv = [drafter.new_sequence() for _ in range(n_seq)]
        self.v_kv = [verifier.new_sequence() for _ in range(n_seq)]
        self.table = upload(table) if table is not None else None
        self.proxy = ds.ds_ngram_create(self.table, log2_size) if table is not None else None
        self.adl = [ds.ds_adl_create(params.k_min, params.k_max, params.delta, params.rho) for _ in range(n_seq)]
        m, i32, f32 = params.m_max, torch.int32, torch.float32
        rows = n_seq * k_cap
        self.hidden = torch.empty(rows, drafter.cfg.d_model, dtype=f32, device=DEV)
        self.cand_id = torch.empty(rows, m, dtype=i32, device=DEV)
        self.cand_logp = torch.empty(rows, m, dtype=f32, device=DEV)
        self.cand_cnt = torch.empty(rows, dtype=i32, device=DEV)
        self.eos_logp = torch.empty(rows, dtype=f32, device=DEV)
        self.lse = torch.empty(rows, dtype=f32, device=DEV)
        self.cps_ws = torch.empty(ds.ds_cps_workspace_bytes(n_seq, k_cap, m), dtype=torch.uint8, device=DEV)
        # host -> device per round: [pending of all sequences | ctx [n, 2] | first [n]]; device -> host: path, path_len, cand ids
        self.n_in = ds.DS_MAX_ROWS + 3 * n_seq
        self.inp = torch.zeros(self.n_in, dtype=i32, device=DEV)
        self.inp_host = torch.zeros(self.n_in, dtype=i32).pin_memory()
        self.ctx = self.inp[ds.DS_MAX_ROWS:ds.DS_MAX_ROWS + 2 * n_seq]
        self.first = self.inp[ds.DS_MAX_ROWS + 2 * n_seq:]
        self.path = torch.zeros(n_seq * k_cap, dtype=i32, device=DEV)
        self.path_len = torch.zeros(n_seq, dtype=i32, device=DEV)
        self.path_score = torch.zeros(n_seq, dtype=f32, device=DEV)
        self.argmax = torch.zeros(n_seq * (k_cap + 1), dtype=i32, device=DEV)
        self.result = torch.zeros(3 * n_seq, dtype=i32).pin_memory()   # n_accept [n] | next_token [n] | eos_accepted [n]
        self.result_np = self.result.numpy()
        self.path_h = torch.empty(n_seq * k_cap, dtype=i32).pin_memory()
        self.plen_h = torch.empty(n_seq, dtype=i32).pin_memory()
        self.raw_h = torch.empty(rows, dtype=i32).pin_memory()
        self.d_logits = self.v_logits = None
        if keep_logits:
            self.d_logits = torch.empty(rows, drafter.cfg.vocab, dtype=f32, device=DEV)
            self.v_logits = torch.empty(ds.DS_MAX_ROWS, verifier.cfg.vocab, dtype=f32, device=DEV)
        self.tokens: List[List[int]] = [[] for _ in range(n_seq)]
        self.pending: List[List[int]] = [[] for _ in range(n_seq)]

    def close(self) -> None:
        if self.proxy:
            ds.ds_ngram_destroy(self.proxy)
            self.proxy = None
        for a in self.adl:
            ds.ds_adl_destroy(a)
        self.adl = []

    def start(self, prefixes) -> None:
        """Prefill every sequence's two caches with its prefix; the verifier's greedy token after it becomes pending."""
        vocab = self.v.cfg.vocab
        last = torch.empty(vocab, dtype=torch.float32, device=DEV)
        cid = torch.empty(1, 1, dtype=torch.int32, device=DEV)
        tmp_f = torch.empty(3, dtype=torch.float32, device=DEV)
        tmp_i = torch.empty(1, dtype=torch.int32, device=DEV)
        ws = torch.empty(ds.ds_lattice_workspace_bytes(1, vocab, 1), dtype=torch.uint8, device=DEV)
        for s, prefix in enumerate(prefixes):
            t = upload(np.asarray(prefix, dtype=np.int32))
            ds.ds_kv_set_len(self.d_kv[s], 0)
            ds.ds_kv_set_len(self.v_kv[s], 0)
            ds.ds_prefill_seq(self.d.handle, self.d_kv[s], t, len(prefix), None, self.d.ws)
            ds.ds_prefill_seq(self.v.handle, self.v_kv[s], t, len(prefix), last, self.v.ws)
            ds.ds_build_lattice(last, 1, vocab, 1, 1.0, -1, cid, tmp_f[0:1], tmp_i, tmp_f[1:2], tmp_f[2:3], ws)
            torch.cuda.synchronize()
            first = int(cid.item())
            self.tokens[s] = [int(x) for x in prefix] + [first]
            self.pending[s] = [first]

    _PENDING = -0x7EADBEEF

    def round(self, k: int) -> list:
        """One round of every sequence with draft length k; returns one record per sequence."""
        n, p = self.n, self.p
        if not 1 <= k <= self.k_cap:
            raise ValueError(f"draft length {k} outside [1, k_cap = {self.k_cap}]")
        n_pend = [len(q) for q in self.pending]
        h = self.inp_host.numpy()
        flat = [t for q in self.pending for t in q]
        if len(flat) > ds.DS_MAX_ROWS:
            raise ValueError("too many pending tokens")
        h[:len(flat)] = flat
        base = ds.DS_MAX_ROWS
        for s in range(n):
            h[base + 2 * s] = self.tokens[s][-2]
            h[base + 2 * s + 1] = self.tokens[s][-1]
            h[base + 2 * n + s] = self.tokens[s][-1]
        self.inp.copy_(self.inp_host, non_blocking=True)
        v_len = [ds.ds_kv_len(kv) for kv in self.v_kv]
        self.result_np[2 * n:] = self._PENDING
        rows = n * k
        lat = (self.cand_id, self.cand_logp, self.cand_cnt, self.eos_logp, self.lse)
        ds.ds_draft_block_batch(self.d.handle, self.d_kv, self.inp, n_pend, k, self.mask_id, self.hidden, self.d.ws)
        ds.ds_draft_lattice(self.d.handle, None, rows, p.m_max, p.tau, self.eos_id, *lat, self.d_logits, self.d.ws)
        ds.ds_cps_path(lat[0], lat[1], lat[2], lat[3], n, k, p.m_max, p.beam, p.lam, self.proxy, self.ctx, self.eos_id,
                       self.path, self.path_len, self.path_score, self.cps_ws)
        path_h, plen_h, raw_h = self.path_h[:n * k], self.plen_h, self.raw_h[:rows]
        path_h.copy_(self.path[:n * k], non_blocking=True)
        plen_h.copy_(self.path_len, non_blocking=True)
        raw_h.copy_(self.cand_id[:rows, 0], non_blocking=True)
        ds.ds_verify_block_batch(self.v.handle, self.v_kv, self.first, self.path, k, self.path_len, self.eos_id,
                                 self.result[0:n], self.result[n:2 * n], self.argmax, self.result[2 * n:3 * n],
                                 self.v_logits, self.v.ws)
        res, spins = self.result_np, 0
        while np.any(res[2 * n:] == self._PENDING):   # the round's host crossing: poll the pinned verdicts
            spins += 1
            if (spins & 0xFFFF) == 0:
                torch.cuda.current_stream().synchronize()
                if np.any(res[2 * n:] == self._PENDING):
                    raise RuntimeError("no verdict from the acceptance kernel")
        torch.cuda.current_stream().synchronize()     # the small read-back copies were issued before the verifier pass
        out = []
        paths, plens, raw = path_h.numpy().reshape(n, k), plen_h.numpy(), raw_h.numpy().reshape(n, k)
        for s in range(n):
            n_acc, nxt, eos, plen = int(res[s]), int(res[n + s]), int(res[2 * n + s]), int(plens[s])
            path = paths[s, :plen].copy()
            ds.ds_kv_set_len(self.v_kv[s], v_len[s] + 1 + n_acc)
            committed = [int(t) for t in path[:n_acc]] + [nxt]
            self.tokens[s] += committed
            self.pending[s] = committed
            first_eos = ds.ds_adl_first_eos(np.ascontiguousarray(raw[s]), k, 1, self.eos_id)
            k_next = ds.ds_adl_update(self.adl[s], k, first_eos, n_acc)
            out.append({"k": k, "path": path, "path_len": plen, "n_accept": n_acc, "next_token": nxt,
                        "eos_accepted": eos, "committed": committed, "first_eos": first_eos, "k_next": k_next})
        return out


def ar_greedy(model: DeviceModel, prefix: np.ndarray, n_new: int, timing: Optional[dict] = None) -> List[int]:
    """Plain greedy decoding of `model` on the GPU, one token per step (the baseline that speed-ups are quoted
    against, and the reference stream of the lossless check).  Every step is a ds_verify_block call with an
    empty path (one row); tokens stay on the device between steps, so there is no host sync inside the loop.
    """
    t = upload(np.asarray(prefix, dtype=np.int32))
    vocab = model.cfg.vocab
    last = torch.empty(vocab, dtype=torch.float32, device=DEV)
    model.set_kv_len(0)
    ds.ds_prefill(model.handle, t, len(prefix), last, model.ws)
    toks = torch.zeros(n_new + 1, dtype=torch.int32, device=DEV)
    scratch_f = torch.empty(3, dtype=torch.float32, device=DEV)
    scratch_i = torch.empty(4, dtype=torch.int32, device=DEV)
    ws = torch.empty(ds.ds_lattice_workspace_bytes(1, vocab, 1), dtype=torch.uint8, device=DEV)
    # first token: top-1 of the prefill logits (ties to the lower id)
    ds.ds_build_lattice(last, 1, vocab, 1, 1.0, -1, toks[0:1], scratch_f[0:1], scratch_i[0:1], scratch_f[1:2],
                        scratch_f[2:3], ws)
    base = len(prefix)
    t0, t1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0.record()
    for i in range(n_new - 1):
        ds.ds_verify_block(model.handle, toks[i:i + 1], 0, None, -1, scratch_i[1:2], toks[i + 1:i + 2],
                           scratch_i[2:3], scratch_i[3:4], None, model.ws)
        model.set_kv_len(base + i + 1)
    t1.record()
    torch.cuda.synchronize()
    if timing is not None:
        timing["decode_ms"] = t0.elapsed_time(t1)
        timing["steps"] = n_new - 1
    return [int(x) for x in toks[:n_new].cpu().numpy()]


def device_weights(cfg: synth.ModelCfg, seed: int, std: float = 0.02) -> dict:
    """Random-init weights drawn directly on the GPU (torch generator), for workloads too large to draw on
    the host in reasonable time.  Same structure as synth.make_weights; no oracle consumes these."""
    gen = torch.Generator(device=DEV)
    gen.manual_seed(seed)
    dt = torch.bfloat16 if cfg.dtype == "bf16" else torch.float32

    def draw(shape):
        return (torch.randn(shape, generator=gen, device=DEV, dtype=torch.float32) * std).to(dt)

    out = {"embed": draw((cfg.vocab, cfg.d_model)), "layers": []}
    shapes = synth.layer_shapes(cfg)
    for _ in range(cfg.n_layers):
        lw = {n: draw(shapes[n]) for n in synth.LAYER_TENSORS}
        lw["norm1"] = torch.ones(cfg.d_model, device=DEV)
        lw["norm2"] = torch.ones(cfg.d_model, device=DEV)
        out["layers"].append(lw)
    out["final_norm"] = torch.ones(cfg.d_model, device=DEV)
    out["lm_head"] = draw((cfg.vocab, cfg.d_model))
    return out
