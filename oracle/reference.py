"""fp64 CPU oracle for blockwise causal prefill attention -- TEST INFRASTRUCTURE ONLY.

Only ``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of
``bench.py`` may import this module.  It neither imports nor is imported by the
HIP package, and shares no arithmetic with it.

The arithmetic lives in ``pec_oracle.c`` (plain loops, fp64); this file only
marshals numpy arrays into it and writes out the segment/ring bookkeeping:

* :func:`attention`  -- Eq. 2 with the causal row softmax of Eq. 3 (section
  "LLM Foundations"), for a query segment at global offset ``q_off`` against a
  key/value segment at global offset ``kv_off``.
* :func:`merge`      -- exact combination of two partial results over disjoint
  key sets (the online-softmax step of ring attention, section "Sequence
  Parallelism for Long Requests").
* :func:`sp_prefill` -- one ring member's sweep: its query segment visits the
  KV segments in ring order, own segment first, merging as it goes.
* :func:`varlen`     -- a packed batch of independent prompts (the batched short
  prefills of section "Coordinated Prefill-Decode Colocation and
  Disaggregation"): each sequence attends only to itself, positions restart at 0.
* :func:`colocated`  -- the mixed batch of the same section: every sequence brings its own number of
  queries (the last positions of the sequence) and of keys; a decode step is one query against its
  whole cache, a prompt has as many queries as keys.

Parity pins: tests/test_oracle_pins.py.
"""
from __future__ import annotations

import ctypes
import math
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "pec_oracle.c")
# PEC_ORACLE_SANITIZE=1 selects a second build of the same source with AddressSanitizer and
# UndefinedBehaviorSanitizer (the process then has to run with libasan preloaded; see
# tests/test_oracle_sanitizers.py).
_SANITIZE = os.environ.get("PEC_ORACLE_SANITIZE", "") == "1"
_LIB = os.path.join(_HERE, "libpec_oracle_san.so" if _SANITIZE else "libpec_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile pec_oracle.c with gcc (OpenMP) next to its source."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp.%d" % os.getpid()
        flags = ["-O1", "-g", "-fno-omit-frame-pointer", "-fsanitize=address,undefined",
                 "-fno-sanitize-recover=undefined"] if _SANITIZE else ["-O2"]
        subprocess.check_call(["gcc", *flags, "-fopenmp", "-fPIC", "-shared", "-std=c11", "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        vp, i64, ci, dbl = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int, ctypes.c_double
        lib.oracle_attention.argtypes = [vp, vp, vp, ci, i64, i64, ci, ci, ci, vp, i64, ci, dbl, vp, vp, vp]
        lib.oracle_attention.restype = ci
        lib.oracle_merge.argtypes = [vp, vp, vp, vp, i64, ci, ci, vp, vp]
        lib.oracle_merge.restype = ci
        lib.oracle_num_threads.restype = ci
        _lib = lib
    return _lib


def num_threads() -> int:
    """Threads the C loops run on (OpenMP's maximum for this process)."""
    return int(_load().oracle_num_threads())


def _as_input(x):
    """-> (contiguous numpy array, dtype code). uint16 = bf16 bit patterns, else fp64."""
    if hasattr(x, "detach"):  # a torch tensor: take its bytes, no arithmetic
        t = x.detach().cpu().contiguous()
        if str(t.dtype) == "torch.bfloat16":
            import torch

            x = t.view(torch.int16).numpy().view(np.uint16)
        else:
            x = t.double().numpy()
    x = np.asarray(x)
    if x.dtype == np.uint16:
        return np.ascontiguousarray(x), 1
    return np.ascontiguousarray(x, dtype=np.float64), 0


def _ptr(a):
    return a.ctypes.data_as(ctypes.c_void_p) if a is not None else None


def attention(q, k, v, *, q_off: int = 0, kv_off: int = 0, causal: bool = True,
              scale: float | None = None, q_pos=None, return_probs: bool = False):
    """Eq. 2-3.  q [sq, Hq, d], k/v [sk, Hkv, d]  ->  out [sq, Hq, d] fp64, lse [Hq, sq] fp64.

    ``q_pos`` (int64 [sq]) gives each row's global position explicitly (used to
    check sampled rows of a long sequence); default ``q_off + arange(sq)``.
    """
    qa, dt = _as_input(q)
    ka, dtk = _as_input(k)
    va, dtv = _as_input(v)
    if not (dt == dtk == dtv):
        raise ValueError("q, k, v must share a dtype")
    sq, hq, d = qa.shape
    sk, hkv, dk = ka.shape
    if dk != d or va.shape != ka.shape:
        raise ValueError("shape mismatch")
    if scale is None:
        scale = 1.0 / math.sqrt(float(d))
    if q_pos is None:
        q_pos = q_off + np.arange(sq, dtype=np.int64)
    q_pos = np.ascontiguousarray(q_pos, dtype=np.int64)
    if q_pos.shape != (sq,):
        raise ValueError("q_pos must have one entry per query row")
    out = np.empty((sq, hq, d), dtype=np.float64)
    lse = np.empty((hq, sq), dtype=np.float64)
    probs = np.empty((hq, sq, sk), dtype=np.float64) if return_probs else None
    rc = _load().oracle_attention(_ptr(qa), _ptr(ka), _ptr(va), dt, sq, sk, hq, hkv, d,
                                  _ptr(q_pos), int(kv_off), int(bool(causal)), float(scale),
                                  _ptr(out), _ptr(lse), _ptr(probs))
    if rc != 0:
        raise ValueError("oracle_attention rejected its arguments")
    return (out, lse, probs) if return_probs else (out, lse)


def merge(o_a, lse_a, o_b, lse_b):
    """Combine two partial (O, LSE) pairs over disjoint key sets; (0, -inf) is the identity."""
    o_a = np.ascontiguousarray(o_a, dtype=np.float64)
    o_b = np.ascontiguousarray(o_b, dtype=np.float64)
    lse_a = np.ascontiguousarray(lse_a, dtype=np.float64)
    lse_b = np.ascontiguousarray(lse_b, dtype=np.float64)
    sq, hq, d = o_a.shape
    if o_b.shape != o_a.shape or lse_a.shape != (hq, sq) or lse_b.shape != (hq, sq):
        raise ValueError("shape mismatch")
    o = np.empty_like(o_a)
    lse = np.empty_like(lse_a)
    rc = _load().oracle_merge(_ptr(o_a), _ptr(lse_a), _ptr(o_b), _ptr(lse_b), sq, hq, d, _ptr(o), _ptr(lse))
    if rc != 0:
        raise ValueError("oracle_merge rejected its arguments")
    return o, lse


def ring_schedule(r: int, n_chunks: int, causal: bool = True):
    """KV chunks that ring member ``r`` visits, in order: step t brings chunk (r - t) mod P.

    Segments are contiguous and equal (the last may be short); under the causal
    mask a chunk with index above r lies wholly in the future and is skipped.
    """
    order = [(r - t) % n_chunks for t in range(n_chunks)]
    return [c for c in order if (not causal) or c <= r]


def sp_prefill(q, k, v, *, q_off: int, chunk: int, causal: bool = True, scale: float | None = None):
    """One ring member's prefill: query segment at q_off vs. all KV (from position 0) in chunks.

    Visits the chunks in ring order starting from the one containing the
    member's own first query, computing each partial by :func:`attention` and
    folding it in with :func:`merge`.
    """
    qa, _ = _as_input(q)
    ka, _ = _as_input(k)
    va, _ = _as_input(v)
    sq, hq, d = qa.shape
    sk = ka.shape[0]
    n_chunks = max(1, -(-sk // chunk))
    r = min(q_off // chunk, n_chunks - 1)
    o = np.zeros((sq, hq, d), dtype=np.float64)
    lse = np.full((hq, sq), -np.inf, dtype=np.float64)
    for t in range(n_chunks):
        c = (r - t) % n_chunks
        lo, hi = c * chunk, min(sk, (c + 1) * chunk)
        if causal and lo > q_off + sq - 1:
            continue  # wholly in the future of every local query
        o_p, lse_p = attention(qa, ka[lo:hi], va[lo:hi], q_off=q_off, kv_off=lo, causal=causal, scale=scale)
        o, lse = merge(o, lse, o_p, lse_p)
    return o, lse


def sp_prefill_states(q, k, v, *, q_off: int, chunk: int, causal: bool = True, scale: float | None = None):
    """The running (O, LSE) pair after each ring step of :func:`sp_prefill`, in order: what a
    scheduler has to keep when it pauses the prefill between two steps (section "Preemption of
    Long-Request Prefill").  The last entry is the final result; the list is empty when no
    segment is visible."""
    qa, _ = _as_input(q)
    ka, _ = _as_input(k)
    va, _ = _as_input(v)
    sq, hq, d = qa.shape
    sk = ka.shape[0]
    n_chunks = max(1, -(-sk // chunk))
    r = min(q_off // chunk, n_chunks - 1)
    o = np.zeros((sq, hq, d), dtype=np.float64)
    lse = np.full((hq, sq), -np.inf, dtype=np.float64)
    states = []
    for t in range(n_chunks):
        c = (r - t) % n_chunks
        lo, hi = c * chunk, min(sk, (c + 1) * chunk)
        if hi <= lo or (causal and lo > q_off + sq - 1):
            continue
        o_p, lse_p = attention(qa, ka[lo:hi], va[lo:hi], q_off=q_off, kv_off=lo, causal=causal, scale=scale)
        o, lse = merge(o, lse, o_p, lse_p)
        states.append((o.copy(), lse.copy()))
    return states


def ulysses_to_messages(x, n_gpus: int):
    """Segment of all heads x [s, H, d] -> the G all-to-all messages [G, s, H/G, d]: message g holds
    the heads GPU g owns (section "Sequence Parallelism of Megatron and Ulysses")."""
    x = np.asarray(x)
    s, h, d = x.shape
    return np.ascontiguousarray(x.reshape(s, n_gpus, h // n_gpus, d).transpose(1, 0, 2, 3))


def ulysses_from_messages(y):
    """Inverse: received messages [G, s, H/G, d] (ordered by source rank) -> [s, H, d]."""
    y = np.asarray(y)
    g, s, hg, d = y.shape
    return np.ascontiguousarray(y.transpose(1, 0, 2, 3).reshape(s, g * hg, d))


def varlen(q, k, v, cu_seqlens, *, causal: bool = True, scale: float | None = None):
    """Packed batch: sequence b owns rows cu[b]..cu[b+1]-1 and attends only to itself."""
    qa, _ = _as_input(q)
    ka, _ = _as_input(k)
    va, _ = _as_input(v)
    cu = [int(x) for x in np.asarray(cu_seqlens).reshape(-1)]
    total, hq, d = qa.shape
    out = np.zeros((total, hq, d), dtype=np.float64)
    lse = np.full((hq, total), -np.inf, dtype=np.float64)
    for b in range(len(cu) - 1):
        lo, hi = cu[b], cu[b + 1]
        if hi <= lo:
            continue
        o_b, l_b = attention(qa[lo:hi], ka[lo:hi], va[lo:hi], q_off=0, kv_off=0, causal=causal, scale=scale)
        out[lo:hi] = o_b
        lse[:, lo:hi] = l_b
    return out, lse


def colocated(q, k, v, cu_seqlens_q, cu_seqlens_k, *, causal: bool = True, scale: float | None = None):
    """Mixed batch of prefills and decode steps: sequence b owns query rows cu_q[b]..cu_q[b+1]-1 and key
    rows cu_k[b]..cu_k[b+1]-1; its len_q queries are the last len_q positions of its len_k tokens, so
    query i sits at position len_k - len_q + i and sees keys 0 .. len_k - len_q + i (Eq. 3)."""
    qa, _ = _as_input(q)
    ka, _ = _as_input(k)
    va, _ = _as_input(v)
    cq = [int(x) for x in np.asarray(cu_seqlens_q).reshape(-1)]
    ck = [int(x) for x in np.asarray(cu_seqlens_k).reshape(-1)]
    total, hq, d = qa.shape
    out = np.zeros((total, hq, d), dtype=np.float64)
    lse = np.full((hq, total), -np.inf, dtype=np.float64)
    for b in range(len(cq) - 1):
        q0, q1, k0, k1 = cq[b], cq[b + 1], ck[b], ck[b + 1]
        if q1 <= q0:
            continue
        o_b, l_b = attention(qa[q0:q1], ka[k0:k1], va[k0:k1], q_off=(k1 - k0) - (q1 - q0), kv_off=0, causal=causal,
                             scale=scale)
        out[q0:q1] = o_b
        lse[:, q0:q1] = l_b
    return out, lse
