"""Thin ctypes binding of libdiffuspec.so: same names as include/ds.h, argument marshalling only.

PyTorch supplies device memory and streams; every step of the round runs in the library's kernels.
There is no fallback: if the library has not been built, loading raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional

import numpy as np

_LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libdiffuspec.so")
_lib = None

DS_F32, DS_BF16 = 0, 1
DS_MAX_ROWS, DS_MAX_TOPM, DS_MAX_BEAM, DS_MAX_SEQ = 144, 16, 16, 8
DS_OK, DS_E_INVALID, DS_E_SHAPE, DS_E_CAPACITY, DS_E_UNSUPPORTED, DS_E_HIP = 0, -1, -2, -3, -4, -5

EXPORTS = [
    "ds_version", "ds_last_error", "ds_model_packed_bytes", "ds_workspace_bytes", "ds_kv_bytes",
    "ds_model_create", "ds_model_destroy", "ds_model_kv_len", "ds_model_kv_set_len", "ds_prefill",
    "ds_draft_block", "ds_lm_head", "ds_draft_lattice", "ds_lm_head_tiles", "ds_lattice_from_tiles", "ds_lattice_workspace_bytes", "ds_build_lattice", "ds_ngram_create",
    "ds_ngram_destroy", "ds_cps_workspace_bytes", "ds_cps_path", "ds_verify_block", "ds_adl_create", "ds_adl_destroy",
    "ds_adl_update", "ds_adl_state", "ds_sample_workspace_bytes", "ds_accept_stochastic",
    "ds_verify_block_stochastic", "ds_draft_block_tokens", "ds_refine_select", "ds_build_lattice_static",
    "ds_refine_update_sizes", "ds_adl_first_eos", "ds_model_overflow_count",
    "ds_kv_create", "ds_kv_destroy", "ds_kv_len", "ds_kv_set_len", "ds_prefill_seq", "ds_draft_block_batch",
    "ds_verify_block_batch", "ds_verify_block_carry",
    "ds_lmproxy_bytes", "ds_lmproxy_create", "ds_lmproxy_destroy", "ds_lmproxy_prefill", "ds_lmproxy_len",
    "ds_lmproxy_set_len", "ds_cps_path_lm", "ds_round_io_layout", "ds_rounds_run",
]


class DsError(RuntimeError):
    def __init__(self, code: int, text: str):
        super().__init__(f"libdiffuspec error {code}: {text}")
        self.code = code


class ModelCfgC(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("d_model", C.c_int32), ("n_q", C.c_int32), ("n_kv", C.c_int32),
                ("head_dim", C.c_int32), ("d_ffn", C.c_int32), ("vocab", C.c_int32),
                ("rope_base", C.c_float), ("rms_eps", C.c_float), ("dtype", C.c_int32),
                ("kv_capacity", C.c_int32)]


class LayerWeightsC(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("wq", "wk", "wv", "wo", "w_gate", "w_up", "w_down", "norm1", "norm2")]


class WeightsC(C.Structure):
    _fields_ = [("embed", C.c_void_p), ("layers", C.POINTER(LayerWeightsC)), ("final_norm", C.c_void_p),
                ("lm_head", C.c_void_p)]


class RoundDescC(C.Structure):
    _fields_ = [("drafter", C.c_void_p), ("verifier", C.c_void_p), ("proxy", C.c_void_p), ("adl", C.c_void_p),
                ("K_cap", C.c_int32), ("M_max", C.c_int32), ("beam", C.c_int32), ("eos_id", C.c_int32),
                ("mask_id", C.c_int32), ("tau", C.c_float), ("lam", C.c_float),
                ("hidden", C.c_void_p), ("cand_logp", C.c_void_p), ("cand_cnt", C.c_void_p), ("eos_logp", C.c_void_p),
                ("lse", C.c_void_p), ("io", C.c_void_p), ("path_score", C.c_void_p), ("argmax", C.c_void_p),
                ("cps_ws", C.c_void_p), ("cps_ws_bytes", C.c_size_t),
                ("drafter_ws", C.c_void_p), ("drafter_ws_bytes", C.c_size_t),
                ("verifier_ws", C.c_void_p), ("verifier_ws_bytes", C.c_size_t),
                ("verdict", C.c_void_p), ("host_out", C.c_void_p),
                ("ev_every", C.c_int32), ("ev_start", C.POINTER(C.c_void_p)), ("ev_end", C.POINTER(C.c_void_p))]


class RoundRecordC(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("k", "path_len", "n_accept", "next_token", "eos_accepted", "first_eos",
                                         "k_next")]


def lib_path() -> str:
    return _LIB_PATH


def load():
    """Load the shared library (once).  Raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    # torch ships its own HIP runtime (same SONAME as the system one).  Import it first so that this
    # library binds to the SAME runtime instance: streams and device pointers are shared with torch.
    import torch  # noqa: F401
    if not os.path.exists(_LIB_PATH):
        raise RuntimeError(f"{_LIB_PATH} is missing: build it with `python -m paper_2510_02358_amd.build` "
                           "(there is no CPU fallback)")
    lib = C.CDLL(_LIB_PATH)
    lib.ds_version.restype = C.c_char_p
    lib.ds_last_error.restype = C.c_char_p
    lib.ds_model_destroy.restype = None
    lib.ds_ngram_destroy.restype = None
    lib.ds_adl_destroy.restype = None
    lib.ds_kv_destroy.restype = None
    vp, i32, f32, sz = C.c_void_p, C.c_int32, C.c_float, C.c_size_t
    lib.ds_model_packed_bytes.argtypes = [C.POINTER(ModelCfgC), C.POINTER(sz)]
    lib.ds_workspace_bytes.argtypes = [C.POINTER(ModelCfgC), C.c_int, C.POINTER(sz)]
    lib.ds_kv_bytes.argtypes = [C.POINTER(ModelCfgC), C.POINTER(sz)]
    lib.ds_model_create.argtypes = [C.POINTER(ModelCfgC), C.POINTER(WeightsC), vp, sz, vp, vp, vp, C.POINTER(vp)]
    lib.ds_model_destroy.argtypes = [vp]
    lib.ds_model_overflow_count.argtypes = [vp, C.c_int, vp, C.POINTER(C.c_uint32)]
    lib.ds_kv_create.argtypes = [vp, vp, vp, C.POINTER(vp)]
    lib.ds_kv_destroy.argtypes = [vp]
    lib.ds_kv_len.argtypes = [vp, C.POINTER(C.c_int)]
    lib.ds_kv_set_len.argtypes = [vp, C.c_int]
    lib.ds_prefill_seq.argtypes = [vp, vp, vp, C.c_int, vp, vp, sz, vp]
    lib.ds_draft_block_batch.argtypes = [vp, C.POINTER(vp), C.c_int, vp, C.POINTER(C.c_int), C.c_int, i32, vp, vp, sz,
                                         vp]
    lib.ds_verify_block_batch.argtypes = [vp, C.POINTER(vp), C.c_int, vp, vp, C.c_int, vp, i32, vp, vp, vp, vp, vp, vp,
                                          sz, vp]
    lib.ds_model_kv_len.argtypes = [vp, C.POINTER(C.c_int)]
    lib.ds_model_kv_set_len.argtypes = [vp, C.c_int]
    lib.ds_prefill.argtypes = [vp, vp, C.c_int, vp, vp, sz, vp]
    lib.ds_draft_block.argtypes = [vp, vp, C.c_int, C.c_int, i32, vp, vp, sz, vp]
    lib.ds_lm_head.argtypes = [vp, vp, C.c_int, vp, vp, sz, vp]
    lib.ds_lattice_workspace_bytes.argtypes = [C.c_int, C.c_int, C.c_int, C.POINTER(sz)]
    lib.ds_lm_head_tiles.argtypes = [vp, vp, C.c_int, i32, vp, vp, sz, vp]
    lib.ds_lattice_from_tiles.argtypes = [vp, C.c_int, C.c_int, f32, i32, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.ds_draft_lattice.argtypes = [vp, vp, C.c_int, C.c_int, f32, i32, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.ds_build_lattice.argtypes = [vp, C.c_int, C.c_int, C.c_int, f32, i32, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.ds_build_lattice_static.argtypes = [vp, C.c_int, C.c_int, C.c_int, f32, i32, vp, vp, vp, vp, vp, vp]
    lib.ds_ngram_create.argtypes = [vp, C.c_int, C.POINTER(vp)]
    lib.ds_ngram_destroy.argtypes = [vp]
    lib.ds_cps_workspace_bytes.argtypes = [C.c_int, C.c_int, C.c_int, C.POINTER(sz)]
    lib.ds_cps_path.argtypes = [vp, vp, vp, vp, C.c_int, C.c_int, C.c_int, C.c_int, f32, vp, vp, i32, vp, vp, vp, vp, vp, sz,
                                vp]
    lib.ds_verify_block.argtypes = [vp, vp, C.c_int, vp, i32, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.ds_lmproxy_bytes.argtypes = [vp, C.c_int, C.POINTER(sz)]
    lib.ds_lmproxy_create.argtypes = [vp, C.c_int, vp, sz, C.POINTER(vp)]
    lib.ds_lmproxy_destroy.argtypes = [vp]
    lib.ds_lmproxy_destroy.restype = None
    lib.ds_lmproxy_prefill.argtypes = [vp, vp, C.c_int, vp, sz, vp]
    lib.ds_lmproxy_len.argtypes = [vp, C.POINTER(C.c_int)]
    lib.ds_lmproxy_set_len.argtypes = [vp, C.c_int]
    lib.ds_cps_path_lm.argtypes = [vp, vp, vp, vp, C.c_int, C.c_int, C.c_int, C.c_float, vp, vp, C.c_int, i32, vp, vp,
                                   vp, vp, sz, vp]
    ip = C.POINTER(C.c_int)
    lib.ds_round_io_layout.argtypes = [C.c_int, C.c_int, ip, ip, ip, ip]
    lib.ds_rounds_run.argtypes = [C.POINTER(RoundDescC), C.c_int, C.c_int, C.c_int, C.c_int, ip,
                                  C.POINTER(RoundRecordC), ip, vp, C.c_int, ip, vp]
    lib.ds_verify_block_carry.argtypes = [vp, vp, C.c_int, vp, i32, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.ds_sample_workspace_bytes.argtypes = [C.c_int, C.POINTER(sz)]
    lib.ds_accept_stochastic.argtypes = [vp, vp, C.c_int, C.c_int, vp, vp, vp, i32, vp, vp, vp, vp, vp, sz, vp]
    lib.ds_verify_block_stochastic.argtypes = [vp, vp, C.c_int, vp, vp, vp, i32, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.ds_draft_block_tokens.argtypes = [vp, vp, C.c_int, vp, C.c_int, vp, vp, sz, vp]
    lib.ds_refine_select.argtypes = [vp, vp, vp, vp, vp, C.c_int, C.c_int, C.c_int, i32, vp, vp, vp, vp, vp, vp, vp]
    lib.ds_adl_create.argtypes = [C.c_int, C.c_int, C.c_double, C.c_double, C.POINTER(vp)]
    lib.ds_adl_destroy.argtypes = [vp]
    lib.ds_adl_update.argtypes = [vp, C.c_int, C.c_int, C.c_int, C.POINTER(C.c_int)]
    lib.ds_refine_update_sizes.argtypes = [C.c_int, C.c_int, C.POINTER(C.c_int), C.POINTER(C.c_int)]
    lib.ds_adl_first_eos.argtypes = [vp, C.c_int, C.c_int, i32, C.POINTER(C.c_int)]
    lib.ds_adl_state.argtypes = [vp, C.POINTER(C.c_double), C.POINTER(C.c_double)]
    _lib = lib
    return lib


def _check(rc: int) -> None:
    if rc != 0:
        raise DsError(rc, load().ds_last_error().decode())


def _ptr(t) -> Optional[int]:
    """Device (or host) address of a torch tensor / raw int / None."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    return t.data_ptr()


def _stream(stream) -> Optional[int]:
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, int):
        return stream or None
    return stream.cuda_stream


def ds_version() -> str:
    return load().ds_version().decode()


def ds_last_error() -> str:
    return load().ds_last_error().decode()


def make_cfg(cfg, kv_capacity: int) -> ModelCfgC:
    return ModelCfgC(cfg.n_layers, cfg.d_model, cfg.n_q, cfg.n_kv, cfg.head_dim, cfg.d_ffn, cfg.vocab,
                     cfg.rope_base, cfg.rms_eps, DS_BF16 if cfg.dtype == "bf16" else DS_F32, kv_capacity)


def ds_model_packed_bytes(cfgc: ModelCfgC) -> int:
    out = C.c_size_t(0)
    _check(load().ds_model_packed_bytes(C.byref(cfgc), C.byref(out)))
    return out.value


def ds_workspace_bytes(cfgc: ModelCfgC, max_rows: int) -> int:
    out = C.c_size_t(0)
    _check(load().ds_workspace_bytes(C.byref(cfgc), max_rows, C.byref(out)))
    return out.value


def ds_kv_bytes(cfgc: ModelCfgC) -> int:
    out = C.c_size_t(0)
    _check(load().ds_kv_bytes(C.byref(cfgc), C.byref(out)))
    return out.value


def ds_lattice_workspace_bytes(rows: int, vocab: int, m_max: int) -> int:
    out = C.c_size_t(0)
    _check(load().ds_lattice_workspace_bytes(rows, vocab, m_max, C.byref(out)))
    return out.value


def ds_model_create(cfgc: ModelCfgC, weights: dict, packed, kv_k, kv_v, stream=None) -> int:
    """weights: {"embed", "layers": [{wq,..,norm1,norm2}], "final_norm", "lm_head"} of device tensors."""
    n = cfgc.n_layers
    layers = (LayerWeightsC * n)()
    for i, lw in enumerate(weights["layers"]):
        for name, _ in LayerWeightsC._fields_:
            setattr(layers[i], name, _ptr(lw[name]))
    wc = WeightsC(_ptr(weights["embed"]), layers, _ptr(weights["final_norm"]), _ptr(weights["lm_head"]))
    out = C.c_void_p(None)
    pbytes = packed.numel() * packed.element_size() if packed is not None else 0
    _check(load().ds_model_create(C.byref(cfgc), C.byref(wc), _ptr(packed), pbytes, _ptr(kv_k), _ptr(kv_v),
                                  _stream(stream), C.byref(out)))
    return out.value


def ds_model_destroy(model: int) -> None:
    load().ds_model_destroy(model)


def ds_model_overflow_count(model: int, reset: bool = False, stream=None) -> int:
    out = C.c_uint32(0)
    _check(load().ds_model_overflow_count(model, 1 if reset else 0, _stream(stream), C.byref(out)))
    return out.value


def ds_kv_create(model: int, kv_k, kv_v) -> int:
    out = C.c_void_p(None)
    _check(load().ds_kv_create(model, _ptr(kv_k), _ptr(kv_v), C.byref(out)))
    return out.value


def ds_kv_destroy(kv: int) -> None:
    load().ds_kv_destroy(kv)


def ds_kv_len(kv: int) -> int:
    out = C.c_int(0)
    _check(load().ds_kv_len(kv, C.byref(out)))
    return out.value


def ds_kv_set_len(kv: int, length: int) -> None:
    _check(load().ds_kv_set_len(kv, length))


def ds_prefill_seq(model: int, kv: int, tokens, n: int, last_logits, ws, stream=None) -> None:
    _check(load().ds_prefill_seq(model, kv, _ptr(tokens), n, _ptr(last_logits), _ptr(ws), _nbytes(ws), _stream(stream)))


def ds_draft_block_batch(model: int, seqs, pending, n_pend, k: int, mask_id: int, hidden_out, ws, stream=None) -> None:
    """seqs: list of ds_kv handles; n_pend: list of ints (host)."""
    n = len(seqs)
    _check(load().ds_draft_block_batch(model, (C.c_void_p * n)(*seqs), n, _ptr(pending), (C.c_int * n)(*n_pend), k,
                                       mask_id, _ptr(hidden_out), _ptr(ws), _nbytes(ws), _stream(stream)))


def ds_verify_block_batch(model: int, seqs, first, path, m: int, path_len, eos_id: int, n_accept, next_token, argmax,
                          eos_accepted, logits_out, ws, stream=None) -> None:
    n = len(seqs)
    _check(load().ds_verify_block_batch(model, (C.c_void_p * n)(*seqs), n, _ptr(first), _ptr(path), m, _ptr(path_len),
                                        eos_id, _ptr(n_accept), _ptr(next_token), _ptr(argmax), _ptr(eos_accepted),
                                        _ptr(logits_out), _ptr(ws), _nbytes(ws), _stream(stream)))


def ds_model_kv_len(model: int) -> int:
    out = C.c_int(0)
    _check(load().ds_model_kv_len(model, C.byref(out)))
    return out.value


def ds_model_kv_set_len(model: int, length: int) -> None:
    _check(load().ds_model_kv_set_len(model, length))


def _nbytes(t) -> int:
    return t.numel() * t.element_size()


def ds_prefill(model: int, tokens, n: int, last_logits, ws, stream=None) -> None:
    _check(load().ds_prefill(model, _ptr(tokens), n, _ptr(last_logits), _ptr(ws), _nbytes(ws), _stream(stream)))


def ds_draft_block(model: int, pending, n_pend: int, k: int, mask_id: int, hidden_out, ws, stream=None) -> None:
    _check(load().ds_draft_block(model, _ptr(pending), n_pend, k, mask_id, _ptr(hidden_out), _ptr(ws), _nbytes(ws),
                                 _stream(stream)))


def ds_lm_head(model: int, hidden, rows: int, logits, ws, stream=None) -> None:
    _check(load().ds_lm_head(model, _ptr(hidden), rows, _ptr(logits), _ptr(ws), _nbytes(ws), _stream(stream)))


def ds_build_lattice(logits, rows: int, vocab: int, m_max: int, tau: float, eos_id: int, cand_id, cand_logp,
                     cand_cnt, eos_logp, lse, ws, stream=None) -> None:
    _check(load().ds_build_lattice(_ptr(logits), rows, vocab, m_max, tau, eos_id, _ptr(cand_id), _ptr(cand_logp),
                                   _ptr(cand_cnt), _ptr(eos_logp), _ptr(lse), _ptr(ws),
                                   _nbytes(ws) if ws is not None else 0, _stream(stream)))


def ds_build_lattice_static(logits, rows: int, vocab: int, m_max: int, tau: float, eos_id: int, cand_id, cand_logp,
                            cand_cnt, eos_logp, lse, stream=None) -> None:
    _check(load().ds_build_lattice_static(_ptr(logits), rows, vocab, m_max, tau, eos_id, _ptr(cand_id),
                                          _ptr(cand_logp), _ptr(cand_cnt), _ptr(eos_logp), _ptr(lse), _stream(stream)))


def ds_lm_head_tiles(model: int, hidden, rows: int, eos_id: int, logits_out, ws, stream=None) -> None:
    _check(load().ds_lm_head_tiles(model, _ptr(hidden), rows, eos_id, _ptr(logits_out), _ptr(ws), _nbytes(ws),
                                   _stream(stream)))


def ds_lattice_from_tiles(model: int, rows: int, m_max: int, tau: float, eos_id: int, cand_id, cand_logp, cand_cnt,
                          eos_logp, lse, ws, stream=None) -> None:
    _check(load().ds_lattice_from_tiles(model, rows, m_max, tau, eos_id, _ptr(cand_id), _ptr(cand_logp),
                                        _ptr(cand_cnt), _ptr(eos_logp), _ptr(lse), _ptr(ws), _nbytes(ws),
                                        _stream(stream)))


def ds_draft_lattice(model: int, hidden, rows: int, m_max: int, tau: float, eos_id: int, cand_id, cand_logp, cand_cnt,
                     eos_logp, lse, logits_out, ws, stream=None) -> None:
    _check(load().ds_draft_lattice(model, _ptr(hidden), rows, m_max, tau, eos_id, _ptr(cand_id), _ptr(cand_logp),
                                   _ptr(cand_cnt), _ptr(eos_logp), _ptr(lse), _ptr(logits_out), _ptr(ws),
                                   _nbytes(ws), _stream(stream)))


def ds_ngram_create(table, log2_size: int) -> int:
    out = C.c_void_p(None)
    _check(load().ds_ngram_create(_ptr(table), log2_size, C.byref(out)))
    return out.value


def ds_ngram_destroy(handle: int) -> None:
    load().ds_ngram_destroy(handle)


def ds_cps_workspace_bytes(batch: int, k: int, m_max: int) -> int:
    out = C.c_size_t(0)
    _check(load().ds_cps_workspace_bytes(batch, k, m_max, C.byref(out)))
    return out.value


def ds_cps_path(cand_id, cand_logp, cand_cnt, eos_logp, batch: int, k: int, m_max: int, beam: int, lam: float,
                proxy: Optional[int], ctx, eos_id: int, path, path_len, path_score, ws=None, stream=None,
                host_mirror=None) -> None:
    _check(load().ds_cps_path(_ptr(cand_id), _ptr(cand_logp), _ptr(cand_cnt), _ptr(eos_logp), batch, k, m_max, beam,
                              lam, proxy, _ptr(ctx), eos_id, _ptr(path), _ptr(path_len), _ptr(path_score),
                              _ptr(host_mirror), _ptr(ws), _nbytes(ws) if ws is not None else 0, _stream(stream)))


def ds_verify_block(model: int, block, m: int, path_len, eos_id: int, n_accept, next_token, argmax, eos_accepted,
                    logits_out, ws, stream=None) -> None:
    _check(load().ds_verify_block(model, _ptr(block), m, _ptr(path_len), eos_id, _ptr(n_accept), _ptr(next_token),
                                  _ptr(argmax), _ptr(eos_accepted), _ptr(logits_out), _ptr(ws), _nbytes(ws),
                                  _stream(stream)))


def ds_lmproxy_bytes(cfg, beam: int) -> int:
    out = C.c_size_t(0)
    _check(load().ds_lmproxy_bytes(C.byref(cfg), beam, C.byref(out)))
    return out.value


def ds_lmproxy_create(model: int, beam: int, mem) -> int:
    out = C.c_void_p()
    _check(load().ds_lmproxy_create(model, beam, _ptr(mem), _nbytes(mem), C.byref(out)))
    return out.value


def ds_lmproxy_destroy(proxy: int) -> None:
    load().ds_lmproxy_destroy(proxy)


def ds_lmproxy_prefill(proxy: int, tokens, n: int, ws, stream=None) -> None:
    _check(load().ds_lmproxy_prefill(proxy, _ptr(tokens), n, _ptr(ws), _nbytes(ws), _stream(stream)))


def ds_lmproxy_len(proxy: int) -> int:
    out = C.c_int(0)
    _check(load().ds_lmproxy_len(proxy, C.byref(out)))
    return out.value


def ds_lmproxy_set_len(proxy: int, n: int) -> None:
    _check(load().ds_lmproxy_set_len(proxy, n))


def ds_cps_path_lm(cand_id, cand_logp, cand_cnt, eos_logp, k: int, m_max: int, beam: int, lam: float, proxy: int,
                   pending, n_pend: int, eos_id: int, path, path_len, path_score, ws, stream=None) -> None:
    _check(load().ds_cps_path_lm(_ptr(cand_id), _ptr(cand_logp), _ptr(cand_cnt), _ptr(eos_logp), k, m_max, beam, lam,
                                 proxy, _ptr(pending), n_pend, eos_id, _ptr(path), _ptr(path_len), _ptr(path_score),
                                 _ptr(ws), _nbytes(ws), _stream(stream)))


def ds_round_io_layout(k_cap: int, m_max: int):
    """(path_at, len_at, cand_at, total) of the round loop's device int buffer."""
    out = [C.c_int(0) for _ in range(4)]
    _check(load().ds_round_io_layout(k_cap, m_max, *[C.byref(o) for o in out]))
    return tuple(o.value for o in out)


def ds_rounds_run(desc: RoundDescC, n_rounds: int, k: int, follow_adl: bool, stop_at_eos: bool, n_pend: int,
                  records, tokens_out, tokens_cap: int, stream=None):
    """records: (RoundRecordC * n)() array; tokens_out: address of a host int32 buffer of tokens_cap entries.
    Returns (rounds_done, n_tokens, n_pend of the next round)."""
    pend, done, n_tok = C.c_int(n_pend), C.c_int(0), C.c_int(0)
    _check(load().ds_rounds_run(C.byref(desc), n_rounds, k, int(follow_adl), int(stop_at_eos), C.byref(pend), records,
                                C.byref(done), tokens_out, tokens_cap, C.byref(n_tok), _stream(stream)))
    return done.value, n_tok.value, pend.value


def ds_verify_block_carry(model: int, block, m: int, path_len, eos_id: int, n_accept, next_token, argmax,
                          eos_accepted, logits_out, carry, ws, stream=None) -> None:
    _check(load().ds_verify_block_carry(model, _ptr(block), m, _ptr(path_len), eos_id, _ptr(n_accept),
                                        _ptr(next_token), _ptr(argmax), _ptr(eos_accepted), _ptr(logits_out),
                                        _ptr(carry), _ptr(ws), _nbytes(ws), _stream(stream)))


def ds_sample_workspace_bytes(m: int) -> int:
    out = C.c_size_t(0)
    _check(load().ds_sample_workspace_bytes(m, C.byref(out)))
    return out.value


def ds_accept_stochastic(p_logits, q_logits, m: int, vocab: int, block, path_len, u, eos_id: int, n_accept,
                         next_token, eos_accepted, alpha, ws, stream=None) -> None:
    _check(load().ds_accept_stochastic(_ptr(p_logits), _ptr(q_logits), m, vocab, _ptr(block), _ptr(path_len), _ptr(u),
                                       eos_id, _ptr(n_accept), _ptr(next_token), _ptr(eos_accepted), _ptr(alpha),
                                       _ptr(ws), _nbytes(ws), _stream(stream)))


def ds_verify_block_stochastic(model: int, block, m: int, path_len, q_logits, u, eos_id: int, n_accept, next_token,
                               eos_accepted, alpha, logits_out, ws, stream=None) -> None:
    _check(load().ds_verify_block_stochastic(model, _ptr(block), m, _ptr(path_len), _ptr(q_logits), _ptr(u), eos_id,
                                             _ptr(n_accept), _ptr(next_token), _ptr(eos_accepted), _ptr(alpha),
                                             _ptr(logits_out), _ptr(ws), _nbytes(ws), _stream(stream)))


def ds_draft_block_tokens(model: int, pending, n_pend: int, block_tokens, k: int, hidden_out, ws, stream=None) -> None:
    _check(load().ds_draft_block_tokens(model, _ptr(pending), n_pend, _ptr(block_tokens), k, _ptr(hidden_out),
                                        _ptr(ws), _nbytes(ws), _stream(stream)))


def ds_refine_select(cand_id, cand_logp, cand_cnt, eos_logp, lse, k: int, m_max: int, n_update: int, mask_id: int,
                     block_tokens, out_cand_id, out_cand_logp, out_cand_cnt, out_eos_logp, out_lse,
                     stream=None) -> None:
    _check(load().ds_refine_select(_ptr(cand_id), _ptr(cand_logp), _ptr(cand_cnt), _ptr(eos_logp), _ptr(lse), k, m_max,
                                   n_update, mask_id, _ptr(block_tokens), _ptr(out_cand_id), _ptr(out_cand_logp),
                                   _ptr(out_cand_cnt), _ptr(out_eos_logp), _ptr(out_lse), _stream(stream)))


def ds_adl_create(k_min: int, k_max: int, delta: float, rho: float) -> int:
    out = C.c_void_p(None)
    _check(load().ds_adl_create(k_min, k_max, delta, rho, C.byref(out)))
    return out.value


def ds_adl_destroy(handle: int) -> None:
    load().ds_adl_destroy(handle)


def ds_adl_update(handle: int, k_t: int, first_eos: int, l_acc: int) -> int:
    out = C.c_int(0)
    _check(load().ds_adl_update(handle, k_t, first_eos, l_acc, C.byref(out)))
    return out.value


def ds_refine_update_sizes(k: int, steps: int) -> list:
    buf = (C.c_int * max(steps, 1))()
    n = C.c_int(0)
    _check(load().ds_refine_update_sizes(k, steps, buf, C.byref(n)))
    return [int(buf[i]) for i in range(n.value)]


def ds_adl_first_eos(raw_draft, k: int, stride: int, eos_id: int) -> int:
    """raw_draft: host memory (numpy int32 array or pinned torch tensor) holding token i at [i * stride]."""
    if isinstance(raw_draft, np.ndarray):
        assert raw_draft.dtype == np.int32 and raw_draft.flags["C_CONTIGUOUS"]
        addr = raw_draft.ctypes.data
    else:
        addr = _ptr(raw_draft)
    out = C.c_int(0)
    _check(load().ds_adl_first_eos(addr, k, stride, eos_id, C.byref(out)))
    return out.value


def ds_adl_state(handle: int):
    a, b = C.c_double(0), C.c_double(0)
    _check(load().ds_adl_state(handle, C.byref(a), C.byref(b)))
    return a.value, b.value
