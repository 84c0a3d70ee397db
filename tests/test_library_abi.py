"""CPU-side checks of the boundary: the library loads, exports every symbol the
header declares, and rejects bad arguments before touching the GPU."""
import ctypes
import os
import re

import pytest

from paper_2409_15104_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "pec_attn.h")


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(binding.LIB_PATH):
        from paper_2409_15104_amd import build

        build.build()
    return binding.lib()


def declared_functions():
    text = re.sub(r"/\*.*?\*/", "", open(HEADER).read(), flags=re.S)
    return sorted(set(re.findall(r"\b(pec_[a-z_]+)\s*\(", text)))


def test_header_symbols_are_exported(lib):
    names = declared_functions()
    assert set(names) == set(binding.EXPORTS)
    for n in names:
        assert hasattr(lib, n), n


def test_status_strings(lib):
    assert binding.status_string(0) == "ok"
    seen = {binding.status_string(s) for s in range(-5, 1)}
    assert len(seen) == 6 and "unknown status" not in seen
    assert binding.status_string(-99) == "unknown status"


def test_unknown_or_contradictory_flags_are_refused(lib):
    S = binding.PecShape
    fake = ctypes.c_void_p(0x1000)
    call = lambda flags: lib.pec_attn_chunk(ctypes.byref(S(8, 2, 128, 0, 0.0, flags)), fake, fake, fake, 0, 16, 0, 0, 1,  # noqa: E731
                                            fake, fake, None)
    for flags in (0, binding.PEC_FLAG_SIMPLE_KERNEL, binding.PEC_FLAG_SP_SEPARATE_MERGE,
                  binding.PEC_FLAG_SIMPLE_KERNEL | binding.PEC_FLAG_SP_STEP_LAUNCHES):
        assert call(flags) == 0                      # sq = 0: accepted, nothing launched
    assert call(8) == -2 and call(1 << 31) == -2     # unknown bits
    assert call(binding.PEC_FLAG_SP_SEPARATE_MERGE | binding.PEC_FLAG_SP_STEP_LAUNCHES) == -1


def test_argument_validation_happens_on_the_host(lib):
    S = binding.PecShape
    fake = ctypes.c_void_p(0x1000)     # never dereferenced: every call below must fail validation first
    odd = ctypes.c_void_p(0x1004)
    ok = S(8, 2, 128, binding.PEC_BF16, 0.0)
    call = lambda shp, q=fake, sq=16, sk=16, out=fake: lib.pec_attn_chunk(  # noqa: E731
        ctypes.byref(shp), q, fake, fake, sq, sk, 0, 0, 1, out, fake, None)
    assert call(S(8, 3, 128, 0, 0.0)) == -1          # heads do not divide
    assert call(S(8, 2, 64, 0, 0.0)) == -2           # head_dim
    assert call(S(8, 2, 128, 7, 0.0)) == -2          # dtype
    assert call(S(8, 2, 128, 0, -1.0)) == -1         # scale
    assert call(ok, sq=-1) == -1
    assert call(ok, sq=(1 << 30) + 1) == -2
    assert call(ok, q=None) == -1
    assert call(ok, q=odd) == -3
    assert call(ok, sq=0) == 0                        # empty problem: no-op
    assert lib.pec_attn_chunk(None, fake, fake, fake, 1, 1, 0, 0, 1, fake, fake, None) == -1
    assert lib.pec_attn_merge(ctypes.byref(ok), None, fake, fake, fake, 4, None) == -1
    assert lib.pec_attn_merge(ctypes.byref(ok), fake, fake, fake, fake, 0, None) == 0
    assert lib.pec_finalize(ctypes.byref(ok), fake, odd, 4, None) == -3
    # sp_prefill, one launch per ring step: several segments need a workspace
    steps = S(8, 2, 128, binding.PEC_BF16, 0.0, binding.PEC_FLAG_SP_STEP_LAUNCHES)
    assert lib.pec_sp_prefill(ctypes.byref(steps), fake, fake, fake, 64, 64, 128, 64, 1, fake, fake, None, 0, None) == -4
    assert lib.pec_sp_prefill(ctypes.byref(ok), fake, fake, fake, 64, 0, 128, 0, 1, fake, fake, fake, 1 << 30, None) == -1
    need = lib.pec_sp_workspace_bytes(ctypes.byref(ok), 64)
    assert need >= 2 * 64 * 8 * 128 * 4 + 64 * 8 * 4
    assert lib.pec_varlen_workspace_bytes(4, 1000) > 0
    assert lib.pec_attn_varlen(ctypes.byref(ok), fake, fake, fake, fake, 4, 1000, 512, 1, fake, fake, None, 0, None) == -4
    assert lib.pec_attn_varlen(ctypes.byref(ok), fake, fake, fake, fake, 0, 0, 0, 1, fake, fake, None, 0, None) == 0
    # colocated batch: workspace, null offsets, the plain kernel is refused, empty batch is a no-op
    need = lib.pec_colocated_workspace_bytes(ctypes.byref(ok), 4, 1000, 50000)
    assert need >= (50000 // 4096 + 4) * 8 * 129 * 4
    coloc = lambda shp, cq=fake, ws=fake, nbytes=1 << 40, batch=4: lib.pec_attn_colocated(  # noqa: E731
        ctypes.byref(shp), fake, fake, fake, cq, fake, batch, 1000, 50000, 1, fake, fake, ws, nbytes, None)
    assert coloc(ok, nbytes=need - 1) == -4
    assert coloc(ok, ws=None) == -4
    assert coloc(ok, cq=None) == -1
    assert coloc(S(8, 2, 128, 0, 0.0, binding.PEC_FLAG_SIMPLE_KERNEL)) == -2
    assert coloc(ok, batch=0) == 0
    # resumable sweep: pending is required, chunk a multiple of 64, no plain kernel, workspace checked
    need = lib.pec_sp_resumable_workspace_bytes(ctypes.byref(ok), 512)
    assert need >= 512 * 8 * 128 * 4 + 2 * 8 * 4
    sweep = lambda shp=ok, chunk=1024, ws=fake, nbytes=1 << 40, pending=fake, stop=fake: lib.pec_sp_prefill_resumable(  # noqa: E731
        ctypes.byref(shp), fake, fake, fake, 512, 0, 4096, chunk, 1, fake, fake, ws, nbytes, stop, pending, 0, None)
    assert sweep(pending=None) == -1
    assert sweep(chunk=1000) == -2
    assert sweep(chunk=0) == -1
    assert sweep(S(8, 2, 128, 0, 0.0, binding.PEC_FLAG_SIMPLE_KERNEL)) == -2
    assert sweep(nbytes=need - 1) == -4
    assert sweep(ws=None) == -4
    assert sweep(stop=ctypes.c_void_p(0x1002)) == -3 and sweep(pending=ctypes.c_void_p(0x1002)) == -3


def test_binding_refuses_cpu_tensors(lib):
    import torch

    q = torch.zeros(4, 2, 128, dtype=torch.bfloat16)
    with pytest.raises(ValueError):
        binding.pec_attn_chunk(q, q, q, 0, 0)
