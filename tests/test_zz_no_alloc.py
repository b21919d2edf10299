"""ds_build_lattice_static (library-held scratch, no allocation) against ds_build_lattice (caller workspace), through
the raw C ABI: two calls in a row on one GPU, the second with a smaller input, every output compared; then the
size limit.  Collected last: a failure here must not hide the parity tests."""
import ctypes as C

import numpy as np
import pytest
import torch

from oracle import lattice as o_lat
from paper_2510_02358_amd import binding as ds
from paper_2510_02358_amd import synth

pytestmark = pytest.mark.gpu

DEV = "cuda:0"
LSE_TOL = 1e-5


def _outputs(rows, m_max):
    return [torch.full((rows, m_max), -7, dtype=torch.int32, device=DEV),
            torch.full((rows, m_max), -7.0, dtype=torch.float32, device=DEV),
            torch.full((rows,), -7, dtype=torch.int32, device=DEV),
            torch.full((rows,), -7.0, dtype=torch.float32, device=DEV),
            torch.full((rows,), -7.0, dtype=torch.float32, device=DEV)]


def test_static_scratch_lattice_matches_the_workspace_entry_point_on_two_calls_in_a_row():
    lib = ds.load()
    stream = C.c_void_p(torch.cuda.current_stream().cuda_stream)
    # first a large input (40 rows of the full vocabulary, top-16: 44 segments per row), then a smaller ragged one
    for rows, vocab, m_max, tau, seed in ((40, 152064, 16, 0.8, 1), (5, 8193, 4, 1.0, 2)):
        logits_h = synth.make_logits(1, rows, vocab, seed=seed)
        eos = vocab - 2
        logits = torch.from_numpy(logits_h).to(DEV)
        want, got = _outputs(rows, m_max), _outputs(rows, m_max)
        ws = torch.empty(ds.ds_lattice_workspace_bytes(rows, vocab, m_max), dtype=torch.uint8, device=DEV)
        rc = lib.ds_build_lattice(logits.data_ptr(), rows, vocab, m_max, tau, eos, *[t.data_ptr() for t in want],
                                  ws.data_ptr(), ws.numel(), stream)
        assert rc == ds.DS_OK, ds.ds_last_error()
        rc = lib.ds_build_lattice_static(logits.data_ptr(), rows, vocab, m_max, tau, eos,
                                         *[t.data_ptr() for t in got], stream)
        assert rc == ds.DS_OK, ds.ds_last_error()
        torch.cuda.synchronize()
        for a, b in zip(want, got):
            assert torch.equal(a, b)
        # and both are the oracle's lattice
        ref = o_lat.build_lattice(logits_h, m_max, tau, eos)
        assert np.array_equal(got[0].cpu().numpy(), ref["cand_id"])
        assert np.array_equal(got[2].cpu().numpy(), ref["cand_cnt"])
        assert np.max(np.abs(got[1].cpu().numpy() - ref["cand_logp"])) <= LSE_TOL
        assert np.max(np.abs(got[3].cpu().numpy() - ref["eos_logp"])) <= LSE_TOL
        assert np.max(np.abs(got[4].cpu().numpy() - ref["lse"])) <= LSE_TOL


def test_static_scratch_lattice_rejects_sizes_beyond_its_array_before_any_launch():
    lib = ds.load()
    one = C.c_void_p(256)
    # 5000 rows at top-16 need 2.7 MB of partial records: more than the library's 2 MiB
    assert ds.ds_lattice_workspace_bytes(5000, 1000, 16) > (2 << 20)
    rc = lib.ds_build_lattice_static(one, 5000, 1000, 16, 1.0, -1, one, one, one, one, one, None)
    assert rc == ds.DS_E_CAPACITY and "scratch" in ds.ds_last_error()
    assert lib.ds_build_lattice_static(None, 0, 1000, 16, 1.0, -1, None, None, None, None, None, None) == ds.DS_OK
    assert lib.ds_build_lattice_static(None, 4, 1000, 16, 1.0, -1, None, None, None, None, None, None) == ds.DS_E_INVALID
