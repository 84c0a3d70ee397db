"""ctypes binding of libpec_attn.so: argument marshalling only.

Function names and argument order follow include/pec_attn.h.  torch supplies
device memory and the current HIP stream; every step of the computation runs in
the library's kernels.  There is no fallback: a missing library or a non-zero
status raises.
"""
from __future__ import annotations

import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libpec_attn.so")

PEC_BF16, PEC_F32 = 0, 1
PEC_FLAG_SIMPLE_KERNEL, PEC_FLAG_SP_SEPARATE_MERGE, PEC_FLAG_SP_STEP_LAUNCHES = 1, 2, 4
KERNEL_NAMES = {0: "pec::fwd_il_kernel", PEC_FLAG_SIMPLE_KERNEL: "pec::fwd_simple_kernel"}

EXPORTS = (
    "pec_attn_chunk", "pec_attn_chunk_merge", "pec_attn_merge", "pec_finalize", "pec_sp_prefill",
    "pec_sp_workspace_bytes", "pec_sp_prefill_resumable", "pec_sp_resumable_workspace_bytes", "pec_sp_prefill_num_steps", "pec_sp_prefill_step", "pec_decode_splitkv", "pec_ulysses_layout", "pec_sp_select_strategy", "pec_decode_default_splits",
    "pec_decode_workspace_bytes", "pec_decode_splitkv_static", "pec_mfma_probe", "pec_hbm_read_probe", "pec_attn_colocated", "pec_colocated_workspace_bytes", "pec_attn_varlen", "pec_varlen_workspace_bytes", "pec_status_string",
)


class PecShape(ctypes.Structure):
    _fields_ = [("n_q_heads", ctypes.c_int32), ("n_kv_heads", ctypes.c_int32), ("head_dim", ctypes.c_int32),
                ("out_dtype", ctypes.c_int32), ("scale", ctypes.c_float), ("flags", ctypes.c_uint32)]


class PecSpModel(ctypes.Structure):
    _fields_ = [("d_model", ctypes.c_int64), ("n_heads", ctypes.c_int32), ("n_kv_heads", ctypes.c_int32),
                ("head_dim", ctypes.c_int32), ("seg_len", ctypes.c_int64), ("tp", ctypes.c_int32),
                ("gpus_per_node", ctypes.c_int32), ("bytes_per_element", ctypes.c_double),
                ("node_bandwidth", ctypes.c_double), ("gpu_flops", ctypes.c_double)]


class PecSpChoice(ctypes.Structure):
    _fields_ = [("attn_comm", ctypes.c_double * 2), ("attn_compute", ctypes.c_double * 2),
                ("mlp_comm", ctypes.c_double * 2), ("mlp_compute", ctypes.c_double * 2),
                ("seconds", (ctypes.c_double * 2) * 2), ("best_attn", ctypes.c_int32), ("best_mlp", ctypes.c_int32)]


class PecError(RuntimeError):
    def __init__(self, fn: str, status: int):
        self.status = status
        super().__init__("%s failed: %s (%d)" % (fn, status_string(status), status))


_lib = None


def lib() -> ctypes.CDLL:
    """Load the HIP library; raises if it has not been built (no CPU fallback exists)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(
                "libpec_attn.so is missing: run `python -m paper_2409_15104_amd.build` (hipcc, gfx950) first")
        L = ctypes.CDLL(LIB_PATH)
        vp, i64, i32, ci, sz = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32, ctypes.c_int, ctypes.c_size_t
        sp = ctypes.POINTER(PecShape)
        L.pec_attn_chunk.argtypes = [sp, vp, vp, vp, i64, i64, i64, i64, ci, vp, vp, vp]
        L.pec_attn_chunk_merge.argtypes = [sp, vp, vp, vp, i64, i64, i64, i64, ci, vp, vp, vp, vp]
        L.pec_attn_merge.argtypes = [sp, vp, vp, vp, vp, i64, vp]
        L.pec_finalize.argtypes = [sp, vp, vp, i64, vp]
        L.pec_sp_prefill.argtypes = [sp, vp, vp, vp, i64, i64, i64, i64, ci, vp, vp, vp, sz, vp]
        L.pec_sp_workspace_bytes.argtypes = [sp, i64]
        L.pec_sp_workspace_bytes.restype = sz
        L.pec_sp_prefill_resumable.argtypes = [sp, vp, vp, vp, i64, i64, i64, i64, ci, vp, vp, vp, sz, vp, vp, ci, vp]
        L.pec_sp_resumable_workspace_bytes.argtypes = [sp, i64]
        L.pec_sp_resumable_workspace_bytes.restype = sz
        L.pec_sp_prefill_num_steps.argtypes = [sp, i64, i64, i64, i64, ci]
        L.pec_sp_prefill_num_steps.restype = i64
        L.pec_sp_prefill_step.argtypes = [sp, vp, vp, vp, i64, i64, i64, i64, ci, i64, vp, vp, vp, vp]
        L.pec_decode_splitkv.argtypes = [sp, vp, vp, vp, i64, i32, vp, vp, vp, sz, vp]
        L.pec_decode_splitkv_static.argtypes = [sp, vp, vp, vp, i64, i32, vp, vp, vp]
        L.pec_decode_splitkv_static.restype = ci
        L.pec_decode_default_splits.argtypes = [sp, i64]
        L.pec_decode_default_splits.restype = i32
        L.pec_decode_workspace_bytes.argtypes = [sp, i32]
        L.pec_decode_workspace_bytes.restype = sz
        L.pec_ulysses_layout.argtypes = [vp, vp, i64, i32, i32, i32, ci, vp]
        L.pec_sp_select_strategy.argtypes = [ctypes.POINTER(PecSpModel), ctypes.POINTER(PecSpChoice)]
        L.pec_attn_varlen.argtypes = [sp, vp, vp, vp, vp, i32, i64, i32, ci, vp, vp, vp, sz, vp]
        L.pec_varlen_workspace_bytes.argtypes = [i32, i64]
        L.pec_varlen_workspace_bytes.restype = sz
        L.pec_attn_colocated.argtypes = [sp, vp, vp, vp, vp, vp, i32, i64, i64, ci, vp, vp, vp, sz, vp]
        L.pec_attn_colocated.restype = ci
        L.pec_colocated_workspace_bytes.argtypes = [sp, i32, i64, i64]
        L.pec_colocated_workspace_bytes.restype = sz
        L.pec_hbm_read_probe.argtypes = [vp, sz, vp, vp]
        L.pec_hbm_read_probe.restype = ci
        L.pec_mfma_probe.argtypes = [vp, sz, i32, vp, sz, vp]
        L.pec_mfma_probe.restype = i64
        L.pec_status_string.argtypes = [ci]
        L.pec_status_string.restype = ctypes.c_char_p
        for name in ("pec_attn_chunk", "pec_attn_chunk_merge", "pec_attn_merge", "pec_finalize", "pec_sp_prefill",
                     "pec_sp_prefill_step", "pec_decode_splitkv", "pec_ulysses_layout", "pec_sp_select_strategy",
                     "pec_attn_varlen"):
            getattr(L, name).restype = ci
        _lib = L
    return _lib


def status_string(status: int) -> str:
    return lib().pec_status_string(int(status)).decode()


def _check(fn: str, status: int) -> None:
    if status != 0:
        raise PecError(fn, status)


def _shape(q: torch.Tensor, k: torch.Tensor, out_dtype, scale: float, flags: int = 0) -> PecShape:
    return PecShape(q.shape[1], k.shape[1], q.shape[2], PEC_F32 if out_dtype == torch.float32 else PEC_BF16,
                    float(scale), int(flags))


def _ptr(t):
    return ctypes.c_void_p(t.data_ptr()) if t is not None else None


def _stream(stream):
    s = stream if stream is not None else torch.cuda.current_stream()
    return ctypes.c_void_p(s.cuda_stream)


def _require(t: torch.Tensor, dtype, name: str):
    if not (t.is_cuda and t.is_contiguous() and t.dtype == dtype):
        raise ValueError("%s must be a contiguous %s tensor on the GPU" % (name, dtype))


def pec_attn_chunk(q, k, v, q_off: int, kv_off: int, causal: bool = True, out_dtype=torch.bfloat16,
                   scale: float = 0.0, flags: int = 0, out=None, lse=None, stream=None):
    """q [sq,Hq,128], k/v [sk,Hkv,128] bf16 -> (out [sq,Hq,128] out_dtype, lse [Hq,sq] fp32)."""
    for t, n in ((q, "q"), (k, "k"), (v, "v")):
        _require(t, torch.bfloat16, n)
    sq, hq, d = q.shape
    sk = k.shape[0]
    if out is None:
        out = torch.empty((sq, hq, d), dtype=out_dtype, device=q.device)
    if lse is None:
        lse = torch.empty((hq, sq), dtype=torch.float32, device=q.device)
    _require(out, out_dtype, "out")
    _require(lse, torch.float32, "lse")
    shp = _shape(q, k, out_dtype, scale, flags)
    _check("pec_attn_chunk", lib().pec_attn_chunk(ctypes.byref(shp), _ptr(q), _ptr(k), _ptr(v), sq, sk, int(q_off),
                                                  int(kv_off), int(bool(causal)), _ptr(out), _ptr(lse),
                                                  _stream(stream)))
    return out, lse


def pec_attn_chunk_merge(q, k, v, q_off: int, kv_off: int, o_acc, lse_acc, causal: bool = True, out_final=None,
                         scale: float = 0.0, flags: int = 0, stream=None):
    """Fold one KV segment into the running fp32 (o_acc, lse_acc) in place; optionally also emit out_final."""
    for t, n in ((q, "q"), (k, "k"), (v, "v")):
        _require(t, torch.bfloat16, n)
    _require(o_acc, torch.float32, "o_acc")
    _require(lse_acc, torch.float32, "lse_acc")
    out_dtype = out_final.dtype if out_final is not None else torch.bfloat16
    shp = _shape(q, k, out_dtype, scale, flags)
    _check("pec_attn_chunk_merge",
           lib().pec_attn_chunk_merge(ctypes.byref(shp), _ptr(q), _ptr(k), _ptr(v), q.shape[0], k.shape[0], int(q_off),
                                      int(kv_off), int(bool(causal)), _ptr(o_acc), _ptr(lse_acc), _ptr(out_final),
                                      _stream(stream)))
    return o_acc, lse_acc


def pec_attn_merge(o_acc, lse_acc, o_part, lse_part, stream=None):
    """In-place exact merge of (o_part, lse_part) into (o_acc, lse_acc); o_* share a dtype (bf16 or fp32)."""
    if o_acc.dtype != o_part.dtype:
        raise ValueError("o_acc and o_part must share a dtype")
    _require(o_acc, o_acc.dtype, "o_acc")
    _require(o_part, o_acc.dtype, "o_part")
    _require(lse_acc, torch.float32, "lse_acc")
    _require(lse_part, torch.float32, "lse_part")
    sq, hq, d = o_acc.shape
    shp = PecShape(hq, hq, d, PEC_F32 if o_acc.dtype == torch.float32 else PEC_BF16, 0.0, 0)
    _check("pec_attn_merge", lib().pec_attn_merge(ctypes.byref(shp), _ptr(o_acc), _ptr(lse_acc), _ptr(o_part),
                                                  _ptr(lse_part), sq, _stream(stream)))
    return o_acc, lse_acc


def pec_finalize(o_f32, o_bf16=None, stream=None):
    _require(o_f32, torch.float32, "o_f32")
    sq, hq, d = o_f32.shape
    if o_bf16 is None:
        o_bf16 = torch.empty((sq, hq, d), dtype=torch.bfloat16, device=o_f32.device)
    shp = PecShape(hq, hq, d, PEC_BF16, 0.0, 0)
    _check("pec_finalize", lib().pec_finalize(ctypes.byref(shp), _ptr(o_f32), _ptr(o_bf16), sq, _stream(stream)))
    return o_bf16


def pec_sp_workspace_bytes(n_q_heads: int, n_kv_heads: int, s_q: int) -> int:
    shp = PecShape(n_q_heads, n_kv_heads, 128, PEC_BF16, 0.0, 0)
    return int(lib().pec_sp_workspace_bytes(ctypes.byref(shp), int(s_q)))


def pec_sp_prefill(q, k, v, q_off: int, chunk: int, causal: bool = True, out_dtype=torch.bfloat16,
                   scale: float = 0.0, flags: int = 0, out=None, lse=None, workspace=None, stream=None):
    """One ring member's prefill: q [s_q,Hq,128] at q_off vs k/v [s_kv,Hkv,128] in segments of `chunk`."""
    for t, n in ((q, "q"), (k, "k"), (v, "v")):
        _require(t, torch.bfloat16, n)
    s_q, hq, d = q.shape
    s_kv = k.shape[0]
    if out is None:
        out = torch.empty((s_q, hq, d), dtype=out_dtype, device=q.device)
    if lse is None:
        lse = torch.empty((hq, s_q), dtype=torch.float32, device=q.device)
    shp = _shape(q, k, out_dtype, scale, flags)
    if workspace is None:   # only the modes that launch once per ring step keep state between launches
        per_step = flags & (PEC_FLAG_SP_STEP_LAUNCHES | PEC_FLAG_SP_SEPARATE_MERGE)
        nbytes = int(lib().pec_sp_workspace_bytes(ctypes.byref(shp), s_q)) if per_step else 0
        workspace = torch.empty(max(16, nbytes), dtype=torch.uint8, device=q.device)
    _check("pec_sp_prefill",
           lib().pec_sp_prefill(ctypes.byref(shp), _ptr(q), _ptr(k), _ptr(v), s_q, int(q_off), s_kv, int(chunk),
                                int(bool(causal)), _ptr(out), _ptr(lse), _ptr(workspace), workspace.numel(),
                                _stream(stream)))
    return out, lse


def pec_sp_resumable_workspace_bytes(q, k) -> int:
    shp = _shape(q, k, torch.bfloat16, 0.0)
    return int(lib().pec_sp_resumable_workspace_bytes(ctypes.byref(shp), q.shape[0]))


def pec_sp_prefill_resumable(q, k, v, q_off: int, chunk: int, out, lse, workspace, pending, stop=None, resume: bool = False,
                             causal: bool = True, scale: float = 0.0, flags: int = 0, stream=None):
    """One launch of the stoppable sweep; `stop` (int32 tensor the GPU can read, or None) and `pending` (device int32
    tensor of one element) as in the C header.  Returns nothing: read `pending` to learn whether out / lse are complete."""
    for t, n in ((q, "q"), (k, "k"), (v, "v")):
        _require(t, torch.bfloat16, n)
    _require(lse, torch.float32, "lse")
    _require(pending, torch.int32, "pending")
    shp = _shape(q, k, out.dtype, scale, flags)
    stop_ptr = None
    if stop is not None:
        if stop.dtype != torch.int32:
            raise ValueError("stop must be an int32 tensor")
        stop_ptr = ctypes.c_void_p(stop.data_ptr())      # device memory or pinned host memory
    _check("pec_sp_prefill_resumable",
           lib().pec_sp_prefill_resumable(ctypes.byref(shp), _ptr(q), _ptr(k), _ptr(v), q.shape[0], int(q_off), k.shape[0],
                                          int(chunk), int(bool(causal)), _ptr(out), _ptr(lse), _ptr(workspace),
                                          workspace.numel(), stop_ptr, _ptr(pending), int(bool(resume)), _stream(stream)))


def pec_sp_prefill_num_steps(q, k, q_off: int, chunk: int, causal: bool = True) -> int:
    shp = _shape(q, k, torch.bfloat16, 0.0)
    n = int(lib().pec_sp_prefill_num_steps(ctypes.byref(shp), q.shape[0], int(q_off), k.shape[0], int(chunk),
                                           int(bool(causal))))
    if n < 0:
        raise PecError("pec_sp_prefill_num_steps", n)
    return n


def pec_sp_prefill_step(q, k, v, q_off: int, chunk: int, step: int, o_acc, lse_acc, causal: bool = True,
                        out_final=None, scale: float = 0.0, flags: int = 0, stream=None):
    """Ring step number `step` of the member's prefill, folded into the caller-kept state (o_acc, lse_acc)."""
    for t, n in ((q, "q"), (k, "k"), (v, "v")):
        _require(t, torch.bfloat16, n)
    _require(o_acc, torch.float32, "o_acc")
    _require(lse_acc, torch.float32, "lse_acc")
    out_dtype = out_final.dtype if out_final is not None else torch.bfloat16
    shp = _shape(q, k, out_dtype, scale, flags)
    _check("pec_sp_prefill_step",
           lib().pec_sp_prefill_step(ctypes.byref(shp), _ptr(q), _ptr(k), _ptr(v), q.shape[0], int(q_off), k.shape[0],
                                     int(chunk), int(bool(causal)), int(step), _ptr(o_acc), _ptr(lse_acc),
                                     _ptr(out_final), _stream(stream)))
    return o_acc, lse_acc


def pec_decode_splitkv(q, k, v, n_splits: int = 0, out_dtype=torch.float32, scale: float = 0.0, flags: int = 0, out=None, lse=None,
                       workspace=None, stream=None):
    """One new token q [1,Hq,128] against a KV-cache shard k/v [sk,Hkv,128] -> (out [1,Hq,128], lse [Hq])."""
    for t, n in ((q, "q"), (k, "k"), (v, "v")):
        _require(t, torch.bfloat16, n)
    if q.shape[0] != 1:
        raise ValueError("pec_decode_splitkv takes exactly one query token")
    hq = q.shape[1]
    sk = k.shape[0]
    shp = _shape(q, k, out_dtype, scale, flags)
    if n_splits == 0:
        n_splits = int(lib().pec_decode_default_splits(ctypes.byref(shp), sk))
    if out is None:
        out = torch.empty((1, hq, 128), dtype=out_dtype, device=q.device)
    if lse is None:
        lse = torch.empty((hq,), dtype=torch.float32, device=q.device)
    if workspace is None:
        workspace = torch.empty(max(16, int(lib().pec_decode_workspace_bytes(ctypes.byref(shp), n_splits))),
                                dtype=torch.uint8, device=q.device)
    _check("pec_decode_splitkv",
           lib().pec_decode_splitkv(ctypes.byref(shp), _ptr(q), _ptr(k), _ptr(v), sk, int(n_splits), _ptr(out),
                                    _ptr(lse), _ptr(workspace), workspace.numel(), _stream(stream)))
    return out, lse


def pec_decode_splitkv_static(q, k, v, out, lse, n_splits: int = 0, scale: float = 0.0, stream=None):
    """pec_decode_splitkv without a workspace: partials live in the library's static device buffer.
    `out` [1,Hq,128] (bf16 or fp32) and `lse` [Hq] are supplied by the caller; nothing is allocated."""
    shp = _shape(q, k, out.dtype, scale)
    _check("pec_decode_splitkv_static",
           lib().pec_decode_splitkv_static(ctypes.byref(shp), _ptr(q), _ptr(k), _ptr(v), k.shape[0], int(n_splits),
                                           _ptr(out), _ptr(lse), _stream(stream)))
    return out, lse


def pec_ulysses_layout(x, n_gpus: int, to_messages: bool, out=None, stream=None):
    """to_messages: x [s,H,128] -> [G,s,H/G,128]; otherwise x [G,s,H/G,128] -> [s,H,128] (bf16)."""
    _require(x, torch.bfloat16, "x")
    if to_messages:
        s, h, d = x.shape
        shape = (n_gpus, s, h // n_gpus, d)
    else:
        g, s, hg, d = x.shape
        h = g * hg
        shape = (s, h, d)
    if out is None:
        out = torch.empty(shape, dtype=torch.bfloat16, device=x.device)
    _check("pec_ulysses_layout", lib().pec_ulysses_layout(_ptr(x), _ptr(out), s, h, d, int(n_gpus),
                                                          int(bool(to_messages)), _stream(stream)))
    return out


def pec_sp_select_strategy(d_model, n_heads, n_kv_heads, head_dim, seg_len, tp, gpus_per_node, bytes_per_element,
                           node_bandwidth, gpu_flops) -> dict:
    """Host-only: volumes and time estimates of the four Megatron/Ulysses combinations and the best one."""
    m = PecSpModel(int(d_model), int(n_heads), int(n_kv_heads), int(head_dim), int(seg_len), int(tp),
                   int(gpus_per_node), float(bytes_per_element), float(node_bandwidth), float(gpu_flops))
    c = PecSpChoice()
    _check("pec_sp_select_strategy", lib().pec_sp_select_strategy(ctypes.byref(m), ctypes.byref(c)))
    return {"attn_comm": list(c.attn_comm), "attn_compute": list(c.attn_compute), "mlp_comm": list(c.mlp_comm),
            "mlp_compute": list(c.mlp_compute), "seconds": [list(c.seconds[0]), list(c.seconds[1])],
            "best": (int(c.best_attn), int(c.best_mlp))}


def pec_attn_colocated(q, k, v, cu_seqlens_q, cu_seqlens_k, causal: bool = True, out_dtype=torch.bfloat16,
                       scale: float = 0.0, flags: int = 0, out=None, lse=None, workspace=None, stream=None):
    """Colocated batch: q [Tq,Hq,128], k/v [Tk,Hkv,128], separate int32 offsets [B+1] for queries and keys."""
    for t, n in ((q, "q"), (k, "k"), (v, "v")):
        _require(t, torch.bfloat16, n)
    _require(cu_seqlens_q, torch.int32, "cu_seqlens_q")
    _require(cu_seqlens_k, torch.int32, "cu_seqlens_k")
    total_q, hq, d = q.shape
    total_k = k.shape[0]
    batch = cu_seqlens_q.numel() - 1
    if out is None:
        out = torch.empty((total_q, hq, d), dtype=out_dtype, device=q.device)
    if lse is None:
        lse = torch.empty((hq, total_q), dtype=torch.float32, device=q.device)
    shp = _shape(q, k, out_dtype, scale, flags)
    if workspace is None:
        workspace = torch.empty(max(16, int(lib().pec_colocated_workspace_bytes(ctypes.byref(shp), batch, total_q, total_k))),
                                dtype=torch.uint8, device=q.device)
    _check("pec_attn_colocated",
           lib().pec_attn_colocated(ctypes.byref(shp), _ptr(q), _ptr(k), _ptr(v), _ptr(cu_seqlens_q), _ptr(cu_seqlens_k),
                                    batch, total_q, total_k, int(bool(causal)), _ptr(out), _ptr(lse), _ptr(workspace),
                                    workspace.numel(), _stream(stream)))
    return out, lse


def pec_hbm_read_probe(src, sink, stream=None) -> None:
    """One streaming read of the whole tensor `src` (any dtype, contiguous, on the GPU)."""
    _check("pec_hbm_read_probe", lib().pec_hbm_read_probe(_ptr(src), (src.numel() * src.element_size()) // 16 * 16,
                                                          _ptr(sink), _stream(stream)))


def pec_mfma_probe(operands, iters: int, sink, stream=None) -> int:
    """Launches the bare-MFMA loop on `operands` (bf16, >= 8192 elements); returns the flop count of the launch."""
    _require(operands, torch.bfloat16, "operands")
    _require(sink, torch.float32, "sink")
    n = int(lib().pec_mfma_probe(_ptr(operands), operands.numel() * 2, int(iters), _ptr(sink), sink.numel(),
                                 _stream(stream)))
    if n < 0:
        raise PecError("pec_mfma_probe", n)
    return n


def pec_varlen_workspace_bytes(batch: int, total_tokens: int) -> int:
    return int(lib().pec_varlen_workspace_bytes(int(batch), int(total_tokens)))


def pec_attn_varlen(q, k, v, cu_seqlens, max_seqlen: int, causal: bool = True, out_dtype=torch.bfloat16,
                    scale: float = 0.0, flags: int = 0, out=None, lse=None, workspace=None, stream=None):
    """Packed batch: q [T,Hq,128], k/v [T,Hkv,128], cu_seqlens int32 [B+1] on the GPU."""
    for t, n in ((q, "q"), (k, "k"), (v, "v")):
        _require(t, torch.bfloat16, n)
    _require(cu_seqlens, torch.int32, "cu_seqlens")
    total, hq, d = q.shape
    batch = cu_seqlens.numel() - 1
    if out is None:
        out = torch.empty((total, hq, d), dtype=out_dtype, device=q.device)
    if lse is None:
        lse = torch.empty((hq, total), dtype=torch.float32, device=q.device)
    if workspace is None:
        workspace = torch.empty(max(16, pec_varlen_workspace_bytes(batch, total)), dtype=torch.uint8, device=q.device)
    shp = _shape(q, k, out_dtype, scale, flags)
    _check("pec_attn_varlen",
           lib().pec_attn_varlen(ctypes.byref(shp), _ptr(q), _ptr(k), _ptr(v), _ptr(cu_seqlens), batch, total,
                                 int(max_seqlen), int(bool(causal)), _ptr(out), _ptr(lse), _ptr(workspace),
                                 workspace.numel(), _stream(stream)))
    return out, lse
