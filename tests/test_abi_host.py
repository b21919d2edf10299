"""CPU-side checks of the C-ABI library (no GPU, no compute kernels): it loads, exports every symbol the
header declares, runs the host-only draft-length controller, and rejects bad arguments before any launch."""
import ctypes as C
import os
import re

import pytest

from paper_2510_02358_amd import binding as ds

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "ds.h")
GOLDEN = os.path.join(ROOT, "tests", "golden", "adl_traces.txt")


def _declared_symbols():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(ds_[a-z0-9_]+)\s*\(", text)))


def test_library_loads_and_exports_every_declared_symbol():
    lib = ds.load()
    declared = _declared_symbols()
    assert len(declared) >= 20
    for name in declared:
        assert hasattr(lib, name), f"{name} declared in ds.h but not exported"
    assert sorted(ds.EXPORTS) == declared
    assert "gfx950" in ds.ds_version()


def test_adl_through_the_c_abi_matches_hand_traces():
    n = 0
    for line in open(GOLDEN):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        head, steps, ks = [p.strip() for p in line.split("|")]
        k_min, k_max, delta, rho, k1 = head.split()
        h = ds.ds_adl_create(int(k_min), int(k_max), float(delta), float(rho))
        k = int(k1)
        got = []
        for s in steps.split():
            first_eos, l_acc = (int(x) for x in s.split(":"))
            k = ds.ds_adl_update(h, k, first_eos, l_acc)
            got.append(k)
        ds.ds_adl_destroy(h)
        assert got == [int(x) for x in ks.split()], line
        n += 1
    assert n >= 8


def test_adl_state_and_argument_errors():
    h = ds.ds_adl_create(4, 64, 10.0, 0.5)
    assert ds.ds_adl_update(h, 16, 0, 0) == 8
    assert ds.ds_adl_state(h) == (8.0, 0.0)
    with pytest.raises(ds.DsError) as e:
        ds.ds_adl_update(h, 0, 0, 0)
    assert e.value.code == ds.DS_E_INVALID
    ds.ds_adl_destroy(h)
    for bad in [(0, 4, 1.0, 0.5), (8, 4, 1.0, 0.5), (4, 8, -1.0, 0.5), (4, 8, 1.0, 0.0), (4, 8, 1.0, 1.5)]:
        with pytest.raises(ds.DsError):
            ds.ds_adl_create(*bad)


def test_refinement_schedule_and_first_eos_through_the_c_abi_match_the_oracle():
    """The two small host-side method steps the library owns (update-set sizes of the refinement equation, s_t of
    the generation-length signal) against the oracle's own statements of them, over every K / S of interest."""
    import numpy as np
    from oracle import adl as o_adl
    from oracle import refine as o_refine
    for k in (1, 2, 3, 7, 8, 16, 31, 32, 64, 100, 256):
        for steps in (1, 2, 3, 4, 7, 8, 10, 64, 300):
            got = ds.ds_refine_update_sizes(k, steps)
            assert got == o_refine.update_sizes(k, steps), (k, steps)
            assert sum(got) == k and len(got) == min(k, steps) and got == sorted(got, reverse=True)
    with pytest.raises(ds.DsError):
        ds.ds_refine_update_sizes(0, 2)
    rng = np.random.default_rng(0)
    for case in range(200):
        k, stride = int(rng.integers(0, 70)), int(rng.integers(1, 17))
        eos = int(rng.choice([-1, 5, 9]))
        buf = rng.integers(0, 12, size=max(k * stride, 1)).astype(np.int32)
        raw = buf[: k * stride: stride] if k else buf[:0]
        assert ds.ds_adl_first_eos(buf, k, stride, eos) == o_adl.first_eos_index(raw, eos), case
    # the columns between the strided entries are ignored
    buf = np.array([1, 9, 9, 2, 9, 9, 9, 0, 0], np.int32)
    assert ds.ds_adl_first_eos(buf, 3, 3, 9) == 3 and ds.ds_adl_first_eos(buf, 2, 3, 9) == 0


def test_bad_arguments_are_rejected_on_the_host_before_any_launch():
    lib = ds.load()
    # lattice: null pointers / bad widths
    assert lib.ds_build_lattice(None, 4, 100, 4, 1.0, -1, None, None, None, None, None, None, 0, None) == ds.DS_E_INVALID
    assert "NULL" in ds.ds_last_error()
    assert lib.ds_build_lattice(None, 0, 100, 4, 1.0, -1, None, None, None, None, None, None, 0, None) == ds.DS_OK
    one = C.c_void_p(256)
    assert lib.ds_build_lattice(one, 4, 100, 17, 1.0, -1, one, one, one, one, one, one, 1 << 20, None) == ds.DS_E_SHAPE
    assert lib.ds_build_lattice(one, 4, 100, 4, 1.0, 100, one, one, one, one, one, one, 1 << 20, None) == ds.DS_E_INVALID
    assert lib.ds_build_lattice(one, 4, 100, 4, 1.0, -1, one, one, one, one, one, one, 16, None) == ds.DS_E_CAPACITY
    # path search
    assert lib.ds_cps_path(None, None, None, None, 0, 8, 4, 4, 0.5, None, None, -1, None, None, None, None, None, 0, None) == ds.DS_OK
    assert lib.ds_cps_path(one, one, one, one, 1, 0, 4, 4, 0.5, None, one, -1, one, one, one, None, None, 0, None) == ds.DS_E_SHAPE
    assert lib.ds_cps_path(one, one, one, one, 1, 8, 4, 17, 0.5, None, one, -1, one, one, one, None, None, 0, None) == ds.DS_E_SHAPE
    assert lib.ds_cps_path(one, one, one, one, 1, 8, 4, 4, 1.5, None, one, -1, one, one, one, None, None, 0, None) == ds.DS_E_INVALID
    assert ds.ds_cps_workspace_bytes(1, 32, 8) == (32 * 729 * 4 + 255) // 256 * 256
    # stochastic acceptance and the refinement update
    assert lib.ds_accept_stochastic(one, one, -1, 10, one, None, one, -1, one, one, one, one, one, 1024, None) == ds.DS_E_SHAPE
    assert lib.ds_accept_stochastic(one, one, 144, 10, one, None, one, -1, one, one, one, one, one, 1 << 20, None) == ds.DS_E_SHAPE
    assert lib.ds_accept_stochastic(one, None, 2, 10, one, None, one, -1, one, one, one, one, one, 4096, None) == ds.DS_E_INVALID
    assert lib.ds_accept_stochastic(one, one, 2, 10, one, None, one, 10, one, one, one, one, one, 4096, None) == ds.DS_E_INVALID
    assert lib.ds_accept_stochastic(one, one, 2, 10, one, None, one, -1, one, one, one, one, one, 8, None) == ds.DS_E_CAPACITY
    assert lib.ds_accept_stochastic(one, one, 2, 300000, one, None, one, -1, one, one, one, one, one, 4096, None) == ds.DS_E_UNSUPPORTED
    assert ds.ds_sample_workspace_bytes(32) == 4352 + 512 + 256 + 256   # lse pairs, lse, control words, segment totals
    sel = [one] * 5 + [8, 4, 3, 99] + [one] * 6 + [None]
    assert lib.ds_refine_select(*(sel[:5] + [0] + sel[6:])) == ds.DS_E_SHAPE        # K = 0
    assert lib.ds_refine_select(*(sel[:5] + [257] + sel[6:])) == ds.DS_E_SHAPE      # K > 256
    assert lib.ds_refine_select(*(sel[:6] + [17] + sel[7:])) == ds.DS_E_SHAPE       # M_max > 16
    assert lib.ds_refine_select(*(sel[:7] + [-1] + sel[8:])) == ds.DS_E_SHAPE       # n_update < 0
    assert lib.ds_refine_select(*([None] + sel[1:])) == ds.DS_E_INVALID
    # model-level calls refuse a NULL handle before touching anything
    assert lib.ds_draft_block_tokens(None, None, 0, one, 4, one, one, 1 << 20, None) == ds.DS_E_INVALID
    assert lib.ds_verify_block_stochastic(None, one, 2, None, one, one, -1, one, one, one, one, None, one, 1 << 20,
                                          None) == ds.DS_E_INVALID
    assert lib.ds_lm_head(None, None, 4, one, one, 1 << 20, None) == ds.DS_E_INVALID
    assert lib.ds_draft_lattice(None, None, 4, 8, 1.0, -1, one, one, one, one, one, None, one, 1 << 20,
                                None) == ds.DS_E_INVALID
    assert lib.ds_lm_head_tiles(None, None, 4, -1, None, one, 1 << 20, None) == ds.DS_E_INVALID
    assert lib.ds_lattice_from_tiles(None, 4, 8, 1.0, -1, one, one, one, one, one, one, 1 << 20,
                                     None) == ds.DS_E_INVALID
    assert lib.ds_verify_block_carry(None, one, 2, None, -1, one, one, one, one, None, one, one, 1 << 20,
                                     None) == ds.DS_E_INVALID
    # the library's round loop
    assert ds.ds_round_io_layout(32, 8) == (146, 178, 180, 180 + 256)      # path_at, len_at, cand_at (4-aligned), total
    assert ds.ds_round_io_layout(16, 4) == (146, 162, 164, 164 + 64)
    for k_cap, m_max in ((0, 4), (144, 4), (16, 0), (16, 17)):
        with pytest.raises(ds.DsError) as e:
            ds.ds_round_io_layout(k_cap, m_max)
        assert e.value.code == ds.DS_E_SHAPE
    n_pend, done, n_tok = (C.c_int(1), C.c_int(0), C.c_int(0))
    assert lib.ds_rounds_run(None, 1, 8, 0, 0, C.byref(n_pend), None, C.byref(done), one, 16, C.byref(n_tok),
                             None) == ds.DS_E_INVALID
    desc = ds.RoundDescC()                                                  # every pointer NULL
    recs = (ds.RoundRecordC * 1)()
    assert lib.ds_rounds_run(C.byref(desc), 1, 8, 0, 0, C.byref(n_pend), recs, C.byref(done), one, 16, C.byref(n_tok),
                             None) == ds.DS_E_INVALID
    # the LM proxy of the path search
    assert lib.ds_cps_path_lm(one, one, one, one, 8, 4, 2, 0.5, None, one, 1, -1, one, one, one, one, 1 << 20,
                              None) == ds.DS_E_INVALID
    assert lib.ds_lmproxy_prefill(None, one, 4, one, 1 << 20, None) == ds.DS_E_INVALID
    assert lib.ds_lmproxy_set_len(None, 0) == ds.DS_E_INVALID
    # model configuration
    cfg = ds.ModelCfgC(1, 3584, 28, 4, 128, 18944, 152064, 1e6, 1e-6, ds.DS_BF16, 4096)
    tiny = ds.ModelCfgC(2, 256, 4, 2, 128, 512, 152064, 1e6, 1e-6, ds.DS_BF16, 4096)
    assert ds.ds_lmproxy_bytes(tiny, 4) == 4 * 4 * ds.ds_kv_bytes(tiny) + (ds.ds_lmproxy_bytes(tiny, 1) - 4 * ds.ds_kv_bytes(tiny))
    assert 16 * 1024 < ds.ds_lmproxy_bytes(tiny, 1) - 4 * ds.ds_kv_bytes(tiny) < 32 * 1024     # the search state
    for beam in (0, 9):
        with pytest.raises(ds.DsError) as e:
            ds.ds_lmproxy_bytes(tiny, beam)
        assert e.value.code == ds.DS_E_SHAPE
    assert ds.ds_model_packed_bytes(cfg) == (233046016 + 544997376) * 2 + 256   # + weight-range flag
    assert ds.ds_kv_bytes(cfg) == 4 * 4096 * 128 * 2
    assert ds.ds_workspace_bytes(cfg, 33) > 33 * 152064 * 4
    bad = ds.ModelCfgC(1, 3584, 28, 5, 128, 18944, 152064, 1e6, 1e-6, ds.DS_BF16, 4096)
    with pytest.raises(ds.DsError) as e:
        ds.ds_model_packed_bytes(bad)
    assert e.value.code == ds.DS_E_SHAPE
    bad = ds.ModelCfgC(1, 3584, 28, 4, 64, 18944, 152064, 1e6, 1e-6, ds.DS_BF16, 4096)
    with pytest.raises(ds.DsError) as e:
        ds.ds_workspace_bytes(bad, 8)
    assert e.value.code == ds.DS_E_UNSUPPORTED
    with pytest.raises(ds.DsError) as e:
        ds.ds_workspace_bytes(cfg, 145)
    assert e.value.code == ds.DS_E_SHAPE
    out = C.c_void_p(None)
    assert lib.ds_model_create(C.byref(cfg), None, None, 0, None, None, None, C.byref(out)) == ds.DS_E_INVALID
