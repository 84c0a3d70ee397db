"""Cost model of the intra-node strategy choice of fast Sequence Parallelism -- TEST INFRASTRUCTURE ONLY.

Plain transcription, in exact rational arithmetic, of the closed forms of section "Fast Sequence
Parallelism for Long-Request Prefill": communication volume in a node and computation volume on a
GPU for Megatron SP and Ulysses SP, in the attention stage and in the MLP stage; the four
combinations are timed as (communication elements * bytes per element / node bandwidth +
computation flop / GPU flop rate) summed over the two stages, and the smallest wins (ties: the
first in the order Megatron, Ulysses).  How communication and computation time combine is not
stated in the paper; adding them is the reading taken here and in the library.

Symbols: d model dimension, N_h / N_kv query / key-value heads, d_h head dimension, s segment
length per GPU, T tensor-parallel size, G GPUs per node.
"""
from fractions import Fraction as F

MEGATRON, ULYSSES = 0, 1


def volumes(d, n_h, n_kv, d_h, s, T, G):
    d, s, T, G = F(d), F(s), F(T), F(G)
    qkv = F(n_h + n_kv) * d_h
    attn_comm = [2 * s * d * (T - 1) * G,
                 2 * s * qkv * (G - 1) + (d * qkv + d * d) * G * (T - 1) / T]
    attn_compute = [2 * s * d * qkv / T + 4 * (s * T) ** 2 * d / T + 2 * s * d * d,
                    2 * s * d * qkv + 4 * (s * G) ** 2 * d / G + 2 * s * d * d]
    mlp_comm = [2 * s * d * (T - 1) * G, 8 * d * d * (T - 1) * G / T]
    mlp_compute = [16 * s * d * d, 16 * s * d * d]
    return {"attn_comm": attn_comm, "attn_compute": attn_compute, "mlp_comm": mlp_comm, "mlp_compute": mlp_compute}


def select(d, n_h, n_kv, d_h, s, T, G, bytes_per_element, node_bandwidth, gpu_flops):
    v = volumes(d, n_h, n_kv, d_h, s, T, G)
    bpe, bw, fl = F(bytes_per_element), F(node_bandwidth), F(gpu_flops)
    seconds = [[(v["attn_comm"][a] + v["mlp_comm"][m]) * bpe / bw + (v["attn_compute"][a] + v["mlp_compute"][m]) / fl
                for m in (MEGATRON, ULYSSES)] for a in (MEGATRON, ULYSSES)]
    best = min(((a, m) for a in (0, 1) for m in (0, 1)), key=lambda am: (seconds[am[0]][am[1]], am))
    return v, seconds, best
