"""The allocation-free decode entry point against the workspace-taking one it is a variant of."""
import ctypes

import numpy as np
import pytest
import torch

from oracle import reference as oracle
from paper_2409_15104_amd import binding as pec
from paper_2409_15104_amd import synth

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _both(L, q, k, v, n_splits, out_dtype):
    """Calls pec_decode_splitkv and pec_decode_splitkv_static through the C ABI on the same inputs."""
    hq, hkv, sk = q.shape[1], k.shape[1], k.shape[0]
    shp = pec.PecShape(hq, hkv, 128, pec.PEC_F32 if out_dtype == torch.float32 else pec.PEC_BF16, 0.0, 0)
    stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    splits = n_splits or L.pec_decode_default_splits(ctypes.byref(shp), sk)
    ws = torch.empty(max(16, L.pec_decode_workspace_bytes(ctypes.byref(shp), splits)), dtype=torch.uint8, device=DEV)
    res = []
    for static in (False, True):
        out = torch.full((1, hq, 128), float("nan"), dtype=out_dtype, device=DEV)
        lse = torch.full((hq,), float("nan"), dtype=torch.float32, device=DEV)
        if static:
            rc = L.pec_decode_splitkv_static(ctypes.byref(shp), q.data_ptr(), k.data_ptr(), v.data_ptr(), sk, n_splits,
                                             out.data_ptr(), lse.data_ptr(), stream)
        else:
            rc = L.pec_decode_splitkv(ctypes.byref(shp), q.data_ptr(), k.data_ptr(), v.data_ptr(), sk, n_splits,
                                      out.data_ptr(), lse.data_ptr(), ws.data_ptr(), ws.numel(), stream)
        assert rc == 0, (static, rc)
        res.append((out, lse))
    torch.cuda.synchronize()
    return res


def test_static_scratch_decode_equals_the_workspace_decode_on_two_calls_in_a_row():
    L = pec.lib()
    # first a large call, then a smaller one (fewer heads, fewer keys, fewer ranges) that finds the
    # larger call's partials still in the buffer; then the wide-group path
    for sk, hq, hkv, n_splits, dt in ((70000, 64, 8, 0, torch.float32), (3000, 8, 2, 5, torch.bfloat16),
                                      (2100, 64, 1, 3, torch.float32), (0, 8, 2, 0, torch.float32)):
        q, k, v = [t.to(DEV) for t in synth.qkv(51 + sk, 1, sk, hq, hkv)]
        (o_ws, l_ws), (o_st, l_st) = _both(L, q, k, v, n_splits, dt)
        assert torch.equal(o_ws, o_st) and torch.equal(l_ws, l_st), (sk, hq, hkv)
        o_ref, l_ref = oracle.attention(q.cpu(), k.cpu(), v.cpu(), causal=False)
        assert np.abs(o_st.float().cpu().numpy() - o_ref).max() <= 2e-2
        fin = np.isfinite(l_ref[:, 0])
        got = l_st.cpu().numpy().astype(np.float64)
        assert np.array_equal(np.isfinite(got), fin)
        if fin.any():
            assert (np.abs(got[fin] - l_ref[fin, 0]) / np.maximum(1.0, np.abs(l_ref[fin, 0]))).max() <= 1e-3


def test_static_scratch_decode_refuses_what_does_not_fit():
    L = pec.lib()
    hq, hkv, sk = 64, 8, 4096
    q, k, v = [t.to(DEV) for t in synth.qkv(52, 1, sk, hq, hkv)]
    out = torch.zeros((1, hq, 128), dtype=torch.float32, device=DEV)
    lse = torch.zeros((hq,), dtype=torch.float32, device=DEV)
    shp = pec.PecShape(hq, hkv, 128, pec.PEC_F32, 0.0, 0)
    too_many = (8 << 20) // (hq * 129 * 4) + 1
    rc = L.pec_decode_splitkv_static(ctypes.byref(shp), q.data_ptr(), k.data_ptr(), v.data_ptr(), sk, too_many,
                                     out.data_ptr(), lse.data_ptr(), None)
    assert rc == -6 and "scratch" in pec.status_string(rc)
    torch.cuda.synchronize()
    assert torch.all(out == 0) and torch.all(lse == 0)          # nothing was launched
