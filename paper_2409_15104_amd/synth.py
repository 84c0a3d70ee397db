"""Seeded synthetic inputs shared by the tests, the benchmark and the smoke check.

Holds no arithmetic of the attention method itself: only random draws, dtype
casts and index bookkeeping, so that the HIP path and the CPU checker can be fed
the very same bytes.

Workload recipe (stand-ins for the production trace and the long-input datasets
of the paper's evaluation, section "Experiment Settings", which are not
available here): Q, K, V ~ N(0, 1) drawn in fp32 and rounded once to bf16;
short-prompt lengths log-normal with median 700 and 80 % below 2048, clipped to
[1, 8192], matching the paper's summary of the trace (about 80 % of inputs
under 2K tokens, maximum about 9K); long prompts 64K-512K tokens.
"""
from __future__ import annotations

import math
from dataclasses import dataclass

import numpy as np
import torch

HEAD_DIM = 128


@dataclass(frozen=True)
class Workload:
    name: str
    n_q_heads: int
    n_kv_heads: int
    seq: int
    chunk: int
    seed: int


# The dense configurations of the benchmark definition.
WORKLOADS = {
    "c1_mha_2k": Workload("c1_mha_2k", 8, 8, 2048, 512, 1001),
    "c2_gqa_32k": Workload("c2_gqa_32k", 32, 8, 32768, 4096, 1002),
    "c3_gqa_128k": Workload("c3_gqa_128k", 32, 8, 131072, 8192, 1003),
    "c5_gqa_512k": Workload("c5_gqa_512k", 64, 8, 524288, 16384, 1005),
}
VARLEN_SEED = 1004
VARLEN_N_SHORT = 256
VARLEN_LONG = 65536


def randn_bf16(shape, seed: int, device="cpu") -> torch.Tensor:
    """N(0,1) in fp32 from a seeded generator on ``device``, rounded once to bf16."""
    gen = torch.Generator(device=device)
    gen.manual_seed(int(seed))
    return torch.randn(*shape, generator=gen, dtype=torch.float32, device=device).to(torch.bfloat16)


def qkv(seed: int, s_q: int, s_kv: int, n_q_heads: int, n_kv_heads: int, d: int = HEAD_DIM, device="cpu"):
    """Token-major tensors q [s_q, Hq, d], k and v [s_kv, Hkv, d], bf16, from one seed."""
    q = randn_bf16((s_q, n_q_heads, d), seed * 3 + 0, device)
    k = randn_bf16((s_kv, n_kv_heads, d), seed * 3 + 1, device)
    v = randn_bf16((s_kv, n_kv_heads, d), seed * 3 + 2, device)
    return q, k, v


def qkv_with_outlier_keys(seed: int, s_q: int, s_kv: int, n_q_heads: int, n_kv_heads: int, outliers, d: int = HEAD_DIM,
                          device="cpu"):
    """``qkv`` with some key rows replaced by multiples of query rows.

    ``outliers`` is a list of (key_pos, query_row, gain): key ``key_pos`` of every KV head becomes
    ``gain`` times query row ``query_row`` of the first query head of that group, so that row's score
    against the key lies about ``gain * sqrt(d)`` above the N(0,1) bulk -- a jump of the running softmax
    maximum late in the key stream.
    """
    q, k, v = qkv(seed, s_q, s_kv, n_q_heads, n_kv_heads, d, device)
    group = n_q_heads // n_kv_heads
    k = k.clone()
    for key_pos, row, gain in outliers:
        k[key_pos] = (q[row, ::group].float() * float(gain)).to(k.dtype)
    return q, k, v


def lognormal_lengths(seed: int, n: int = VARLEN_N_SHORT, median: float = 700.0, p80: float = 2048.0,
                      max_len: int = 8192) -> np.ndarray:
    """Prompt lengths L = clip(round(exp(mu + sigma z)), 1, max_len), z ~ N(0,1).

    mu = ln(median); sigma puts the 80th percentile at ``p80`` (z_0.8 = 0.8416).
    """
    rng = np.random.default_rng(int(seed))
    mu = math.log(median)
    sigma = math.log(p80 / median) / 0.8416212335729143
    z = rng.standard_normal(n)
    return np.clip(np.rint(np.exp(mu + sigma * z)), 1, max_len).astype(np.int64)


def varlen_lengths(seed: int = VARLEN_SEED, n_short: int = VARLEN_N_SHORT, long_len: int = VARLEN_LONG,
                   long_at: str = "last") -> np.ndarray:
    """The colocated batch: ``n_short`` log-normal prompts plus one long prompt."""
    short = lognormal_lengths(seed, n_short)
    long_ = np.array([long_len], dtype=np.int64)
    if long_at == "last":
        return np.concatenate([short, long_])
    if long_at == "first":
        return np.concatenate([long_, short])
    mid = n_short // 2
    return np.concatenate([short[:mid], long_, short[mid:]])


def cu_seqlens_of(lengths) -> np.ndarray:
    """Exclusive prefix sum as int32 [B+1]."""
    cu = np.zeros(len(lengths) + 1, dtype=np.int64)
    np.cumsum(np.asarray(lengths, dtype=np.int64), out=cu[1:])
    if cu[-1] >= 2**31:
        raise ValueError("packed batch exceeds int32 token indices")
    return cu.astype(np.int32)


def sample_rows(seed: int, n_rows: int, boundaries=(), n_random: int = 64, edge: int = 4) -> np.ndarray:
    """Row indices for spot checks: first/last ``edge`` rows, two rows either side
    of every boundary, and ``n_random`` seeded-random rows; sorted, unique."""
    rows = set(range(min(edge, n_rows))) | set(range(max(0, n_rows - edge), n_rows))
    for b in boundaries:
        for r in (b - 2, b - 1, b, b + 1):
            if 0 <= r < n_rows:
                rows.add(int(r))
    rng = np.random.default_rng(int(seed))
    if n_rows > 0 and n_random > 0:
        rows |= set(int(x) for x in rng.integers(0, n_rows, size=n_random))
    return np.array(sorted(rows), dtype=np.int64)


def visible_pairs(s_q: int, s_kv: int, q_off: int, kv_off: int, causal: bool) -> int:
    """Number of (query, key) pairs a segment-vs-segment call has to evaluate:
    row i sees n_i = clamp(q_off + i - kv_off + 1, 0, s_kv) keys under the causal mask."""
    if not causal:
        return int(s_q) * int(s_kv)
    n = np.clip(q_off + np.arange(s_q, dtype=np.int64) - kv_off + 1, 0, s_kv)
    return int(n.sum())
