#!/usr/bin/env python3
"""Benchmark of the ring-style blockwise causal prefill attention path on one MI355X.

A step is one full sequential ring sweep of the workload on one GPU: every query
segment r = 0..P-1 runs pec_sp_prefill over the KV segments it can see, in ring
order, with the log-sum-exp merge folded in at every step.  Inputs are resident
in HBM before the timed region.  Prints ONE JSON line.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload c3_gqa_128k|c2_gqa_32k|c1_mha_2k|c5_gqa_512k|c4_varlen|c4_colocated|c3_preempt|decode_512k|ulysses_layout]
                  [--sp-mode resumable|sweep|step|separate] [--simple-kernel] [--share] [--no-cpu-baseline]
"""
from __future__ import annotations

import argparse
import ctypes
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2516.6      # MI355X dense bf16 matrix peak: 256 CU x 4096 flop/clk x 2.4 GHz
FLOP_PER_PAIR = 512.0          # per (query, key, head): 2*128 for q.k plus 2*128 for p.v


def timed_steps(torch, step, steps, warmup):
    """W untimed steps, then K timed ones between synchronisations.  Returns (wall ms per step over the
    whole timed region, HIP-event ms of every single step): events are recorded on torch's current
    stream, the stream every library call of this benchmark is issued on."""
    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    evs = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
    t0 = time.perf_counter()
    evs[0].record()
    for i in range(steps):
        step()
        evs[i + 1].record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3 / steps
    return wall_ms, [evs[i].elapsed_time(evs[i + 1]) for i in range(steps)]


def step_stats(ev_ms):
    xs = sorted(ev_ms)
    n = len(xs)
    med = xs[n // 2] if n % 2 else 0.5 * (xs[n // 2 - 1] + xs[n // 2])
    return {"median": round(med, 4), "min": round(xs[0], 4), "max": round(xs[-1], 4), "n": n}


def mfma_probe(torch, pec, dev, iters=20000):
    """Bare v_mfma_f32_32x32x16_bf16 loop on every compute unit: TFLOP/s on constant and on N(0,1) operands."""
    sink = torch.empty(1024 * 512, dtype=torch.float32, device=dev)
    res = {}
    for name in ("constant", "normal"):
        if name == "constant":
            ops = torch.ones(8192, dtype=torch.bfloat16, device=dev)
        else:
            gen = torch.Generator(device=dev)
            gen.manual_seed(4711)
            ops = torch.randn(8192, generator=gen, dtype=torch.float32, device=dev).to(torch.bfloat16)
        flop = pec.pec_mfma_probe(ops, iters, sink)        # warm-up launch
        torch.cuda.synchronize()
        ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        ev0.record()
        for _ in range(3):
            pec.pec_mfma_probe(ops, iters, sink)
        ev1.record()
        torch.cuda.synchronize()
        ms = ev0.elapsed_time(ev1) / 3
        res[name + "_operands_tflops"] = round(flop / (ms * 1e-3) / 1e12, 1)
        res[name + "_ms"] = round(ms, 3)
    res["what"] = ("bare v_mfma_f32_32x32x16_bf16 loop, 8 wavefronts on every compute unit, %d x 32 MFMAs per wavefront; "
                   "the chip lowers its clock under the power limit, more so on random operand data" % iters)
    return res


def hbm_read_probe(torch, pec, dev, gib=2):
    """Streaming read of a buffer far larger than the caches: the read bandwidth the memory system delivers."""
    buf = torch.empty(gib << 28, dtype=torch.float32, device=dev).normal_()
    sink = torch.zeros(1, dtype=torch.int32, device=dev)
    for _ in range(2):
        pec.pec_hbm_read_probe(buf, sink)
    torch.cuda.synchronize()
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    ev0.record()
    for _ in range(5):
        pec.pec_hbm_read_probe(buf, sink)
    ev1.record()
    torch.cuda.synchronize()
    gbs = 5.0 * buf.numel() * 4 / (ev0.elapsed_time(ev1) * 1e-3) / 1e9
    return {"read_gbs": round(gbs, 1), "what": "streaming read of %d GiB, 8 x 16-byte loads in flight per thread" % gib}


def item_fit(torch, np, pec, synth, dev):
    """Time of an unmasked pec_attn_chunk_merge launch (32 q / 8 kv heads, fp32 running state in and out) as
    T = L + n (o + tiles t): n work items per compute unit (256 query rows of one head each), `tiles` key
    tiles of 64 per item.  Least-squares fit of L (per launch), o (per work item) and t (per tile step)."""
    q, _, _ = synth.qkv(1, 32768, 16, 32, 8, device=dev)
    _, k, v = synth.qkv(2, 16, 16384, 32, 8, device=dev)
    oacc = torch.zeros(32768, 32, 128, dtype=torch.float32, device=dev)
    lse = torch.zeros(32, 32768, dtype=torch.float32, device=dev)
    rows, ys = [], []
    for sq in (2048, 4096, 8192, 16384, 32768):
        for sk in (2048, 4096, 8192, 16384):
            if sq * sk > 8192 * 32768:
                continue
            qq, kk, vv, oa, ll = q[:sq], k[:sk], v[:sk], oacc[:sq], lse[:, :sq].contiguous()
            _, ev = timed_steps(torch, lambda: pec.pec_attn_chunk_merge(qq, kk, vv, 1 << 20, 0, oa, ll, True), 10, 3)
            n, tiles = sq // 2048, sk // 64
            rows.append([1.0, n, n * tiles])
            ys.append(1e3 * sum(ev) / len(ev))
    sol = np.linalg.lstsq(np.array(rows), np.array(ys), rcond=None)[0]
    resid = float(np.abs(np.array(rows) @ sol - np.array(ys)).max())
    return {"per_launch_us": round(float(sol[0]), 2), "per_work_item_us": round(float(sol[1]), 2),
            "per_tile_step_us": round(float(sol[2]), 4), "max_residual_us": round(resid, 1), "launches_fitted": len(ys),
            "asymptotic_tflops": round(512.0 * 32 * 256 * 64 * 256 / 32 / (float(sol[2]) * 1e-6) / 1e12, 1)}


def measured_traffic(workload):
    """HBM bytes per launch of the dominant kernel, from the committed rocprofv3 counter summary of this workload
    (line 'traffic_bytes_per_launch: N' in profiles/<kernel>_<workload>_hbm_traffic.md); None if there is none."""
    path = os.path.join(ROOT, "profiles", "fwd_il_kernel_%s_hbm_traffic.md" % workload)
    try:
        for ln in open(path):
            if ln.startswith("traffic_bytes_per_launch:"):
                return float(ln.split(":")[1])
    except OSError:
        pass
    return None


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="c3_gqa_128k")
    ap.add_argument("--sp-mode", default="resumable", choices=["resumable", "sweep", "step", "separate"],
                    help="resumable: one stoppable sweep launch per ring member, stop word polled and never set (default); "
                         "sweep: the same launch without a stop word; step: one launch per ring step, merge fused; "
                         "separate: one launch per ring step plus a merge kernel")
    ap.add_argument("--simple-kernel", action="store_true", help="time the plain cross-check kernel instead of the default")
    ap.add_argument("--share", action="store_true",
                    help="time one GPU's share only: the last ring member's prefill (its query segment against all KV segments)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=15.0, help="target CPU time of the oracle sample")
    ap.add_argument("--decode-splits", type=int, default=0, help="key ranges per KV head for --workload decode_512k (0: library default)")
    ap.add_argument("--mfma-probe", action="store_true",
                    help="only measure the bare MFMA rate (constant and N(0,1) operands) and print it as one JSON line")
    ap.add_argument("--item-fit", action="store_true",
                    help="only fit launch / work-item / tile-step costs of the attention kernel from unmasked launches of "
                         "different shapes (32 q / 8 kv heads) and print them as one JSON line")
    ap.add_argument("--copy-probe", action="store_true",
                    help="only run three 1 GiB device-to-device copies (calibrates rocprofv3 FETCH_SIZE/WRITE_SIZE)")
    return ap.parse_args()


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (nothing here spans devices); use --gpus 1", file=sys.stderr)
        return 2

    import numpy as np
    import torch

    from paper_2409_15104_amd import binding as pec
    from paper_2409_15104_amd import synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    if args.copy_probe:   # known traffic: 2^30 bytes read and 2^30 bytes written per copy
        x = torch.empty(1 << 28, dtype=torch.float32, device="cuda:0").normal_()
        y = torch.empty_like(x)
        for _ in range(3):
            y.copy_(x)
        torch.cuda.synchronize()
        print(json.dumps({"copy_probe": "3 device copies of 1073741824 bytes"}))
        return 0
    pec.lib()  # fails loudly when the HIP library has not been built
    dev = "cuda:0"
    torch.cuda.set_device(0)
    if args.item_fit:
        print(json.dumps({"item_fit": item_fit(torch, np, pec, synth, dev)}), flush=True)
        return 0
    if args.mfma_probe:
        print(json.dumps({"mfma_probe": mfma_probe(torch, pec, dev), "nominal_peak_tflops": PEAK_BF16_TFLOPS}), flush=True)
        return 0
    args.kernel_flag = pec.PEC_FLAG_SIMPLE_KERNEL if args.simple_kernel else 0
    if args.simple_kernel and args.sp_mode == "resumable":
        args.sp_mode = "sweep"          # the plain kernel keeps no progress table
    mode = {"resumable": 0, "sweep": 0, "step": pec.PEC_FLAG_SP_STEP_LAUNCHES, "separate": pec.PEC_FLAG_SP_SEPARATE_MERGE}[args.sp_mode]
    args.flags = mode | args.kernel_flag

    if args.workload == "c4_varlen":
        return bench_varlen(args, torch, np, pec, synth, dev)
    if args.workload == "c4_colocated":
        return bench_colocated(args, torch, np, pec, synth, dev)
    if args.workload == "c3_preempt":
        return bench_preempt(args, torch, np, pec, synth, dev)
    if args.workload.startswith("decode"):
        return bench_decode(args, torch, np, pec, synth, dev)
    if args.workload.startswith("ulysses"):
        return bench_ulysses(args, torch, np, pec, synth, dev)

    w = synth.WORKLOADS[args.workload]
    S, C, Hq, Hkv = w.seq, w.chunk, w.n_q_heads, w.n_kv_heads
    P = S // C
    if args.share:
        return bench_share(args, torch, pec, synth, dev, w, mode)
    q, k, v = synth.qkv(w.seed, S, S, Hq, Hkv, device=dev)
    out = torch.empty_like(q)
    lse = torch.empty((P, Hq, C), dtype=torch.float32, device=dev)   # one [Hq, C] block per ring member
    ws = torch.empty(max(16, pec.pec_sp_workspace_bytes(Hq, Hkv, C), pec.pec_sp_resumable_workspace_bytes(q[:C], k)),
                     dtype=torch.uint8, device=dev)
    stop = torch.zeros(1, dtype=torch.int32, device=dev)        # the scheduler's stop word: never raised here
    pending = torch.zeros(P, dtype=torch.int32, device=dev)

    pairs = sum(synth.visible_pairs(C, min(C, S - c * C), r * C, c * C, True)
                for r in range(P) for c in range(r + 1))
    assert pairs == S * (S + 1) // 2
    flops = FLOP_PER_PAIR * Hq * pairs
    launches = P * (P + 1) // 2 if mode else P
    how = {"resumable": "one stoppable sweep launch per ring member, the segments' partial results merged by the online "
                        "softmax in registers, stop word polled at every segment boundary",
           "sweep": "one sweep launch per ring member, the segments' partial results merged in registers",
           "step": "one launch per ring step, LSE merge fused into the next step's kernel",
           "separate": "one launch per ring step, LSE merge by a separate kernel"}[args.sp_mode]

    def step():
        for r in range(P):
            lo = r * C
            if args.sp_mode == "resumable":
                pec.pec_sp_prefill_resumable(q[lo:lo + C], k, v, lo, C, out[lo:lo + C], lse[r], ws, pending[r:r + 1], stop=stop)
            else:
                pec.pec_sp_prefill(q[lo:lo + C], k, v, lo, C, True, out=out[lo:lo + C], lse=lse[r], workspace=ws,
                                   flags=args.flags)

    ms_step, ev_ms = timed_steps(torch, step, args.steps, args.warmup)
    if args.sp_mode == "resumable" and int(pending.abs().sum().item()) != 0:
        print("bench.py: a sweep did not run to its end: pending %s" % pending.tolist(), file=sys.stderr)
        return 1
    ev_ms_step = sum(ev_ms) / len(ev_ms)
    tflops = flops / (ms_step * 1e-3) / 1e12

    # Dominant kernel = the attention kernel (every launch of the timed region except in separate mode).
    # Average launch duration from HIP events on the launch stream over the timed region.
    avg_launch_ms = ev_ms_step / launches
    achieved = (flops / launches) / (avg_launch_ms * 1e-3) / 1e12
    roofline = {"bound": "mfma", "achieved": round(achieved, 2), "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                "frac": round(achieved / PEAK_BF16_TFLOPS, 4), "traffic": measured_traffic(args.workload),
                "kernel": pec.KERNEL_NAMES[args.kernel_flag], "launches_per_step": launches,
                "avg_launch_ms": round(avg_launch_ms, 4), "flop_per_launch_avg": flops / launches}

    result = {
        "metric": "prefill attention TFLOP/s and tokens/s at 128K GQA; % of bf16 MFMA peak",
        "value": round(tflops, 2), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_step, 3), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "%s: causal prefill, %d q heads / %d kv heads, d 128, seq %d as %d segments of %d, "
                               "full ring sweep with LSE merge (%s)" % (w.name, Hq, Hkv, S, P, C, how),
                   "seq_len": S, "chunk": C, "n_q_heads": Hq, "n_kv_heads": Hkv, "sp_mode": args.sp_mode,
                   "kernel": pec.KERNEL_NAMES[args.kernel_flag]},
        "tokens_per_s": round(S / (ms_step * 1e-3), 1),
        "pct_of_bf16_mfma_peak": round(100.0 * tflops / PEAK_BF16_TFLOPS, 2),
        "causal_useful_tflop_per_step": round(flops / 1e12, 3),
        "noncausal_convention_tflops": round(4.0 * 128 * Hq * S * S / (ms_step * 1e-3) / 1e12, 2),
        "ms_per_step_stats": step_stats(ev_ms),
        "roofline": roofline,
    }
    probe = mfma_probe(torch, pec, dev)     # after the timed region: the chip's bare matrix rate on this machine, now
    result["mfma_probe"] = probe
    result["pct_of_measured_mfma_peak"] = round(100.0 * tflops / probe["normal_operands_tflops"], 2)
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(args, np, torch, synth, q, k, v, w)
    print(json.dumps(result), flush=True)
    return 0


def bench_share(args, torch, pec, synth, dev, w, mode):
    """One GPU's share of the ring: the last member's query segment against every KV segment (what a GPU of
    the sequence-parallel group computes; the other members' shares are smaller under the causal mask)."""
    S, C, Hq, Hkv = w.seq, w.chunk, w.n_q_heads, w.n_kv_heads
    P = S // C
    q, k, v = synth.qkv(w.seed, C, S, Hq, Hkv, device=dev)      # Q of the one segment only
    out = torch.empty_like(q)
    lse = torch.empty((Hq, C), dtype=torch.float32, device=dev)
    ws = torch.empty(max(16, pec.pec_sp_workspace_bytes(Hq, Hkv, C), pec.pec_sp_resumable_workspace_bytes(q, k)),
                     dtype=torch.uint8, device=dev)
    stop = torch.zeros(1, dtype=torch.int32, device=dev)
    pending = torch.zeros(1, dtype=torch.int32, device=dev)
    lo = S - C
    flops = FLOP_PER_PAIR * Hq * synth.visible_pairs(C, S, lo, 0, True)
    launches = P if mode else 1

    def step():
        if args.sp_mode == "resumable":
            pec.pec_sp_prefill_resumable(q, k, v, lo, C, out, lse, ws, pending, stop=stop)
        else:
            pec.pec_sp_prefill(q, k, v, lo, C, True, out=out, lse=lse, workspace=ws, flags=args.flags)

    ms_step, ev_list = timed_steps(torch, step, args.steps, args.warmup)
    ev_mean = sum(ev_list) / len(ev_list)
    avg_launch_ms = ev_mean / launches
    tflops = flops / (ms_step * 1e-3) / 1e12
    achieved = (flops / launches) / (avg_launch_ms * 1e-3) / 1e12
    result = {
        "metric": "prefill attention TFLOP/s of one ring member's share; % of bf16 MFMA peak",
        "value": round(tflops, 2), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_step, 3), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "%s, last member's share: %d query rows at offset %d against %d keys in %d segments, "
                               "%d q heads / %d kv heads, LSE merge (%s)" % (w.name, C, lo, S, P, Hq, Hkv, args.sp_mode)},
        "tokens_per_s": round(C / (ms_step * 1e-3), 1),
        "pct_of_bf16_mfma_peak": round(100.0 * tflops / PEAK_BF16_TFLOPS, 2),
        "causal_useful_tflop_per_step": round(flops / 1e12, 3),
        "ms_per_step_stats": step_stats(ev_list),
        "roofline": {"bound": "mfma", "achieved": round(achieved, 2), "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                     "frac": round(achieved / PEAK_BF16_TFLOPS, 4), "traffic": None,
                     "kernel": pec.KERNEL_NAMES[args.kernel_flag],
                     "launches_per_step": launches, "avg_launch_ms": round(avg_launch_ms, 4)},
    }
    print(json.dumps(result), flush=True)
    return 0


def cpu_baseline(args, np, torch, synth, q, k, v, w):
    """The fp64 oracle, as it stands, on a bounded sample of the same workload: whole rows
    (all heads, full visible key range) drawn uniformly from the sequence."""
    from oracle import reference as oracle

    S, Hq = w.seq, w.n_q_heads
    k_h, v_h = k.cpu(), v.cpu()
    rng = np.random.default_rng(w.seed)

    def run(n_rows):
        rows = np.sort(rng.integers(0, S, size=n_rows))
        qs = q[torch.from_numpy(rows).to(q.device)].cpu()
        t0 = time.perf_counter()
        oracle.attention(qs, k_h, v_h, q_pos=rows, kv_off=0, causal=True)
        dt = time.perf_counter() - t0
        return dt, int((rows + 1).sum())

    dt, pairs = run(4)                                  # calibration, then the timed sample
    rate = pairs / max(dt, 1e-6)
    n_rows = int(max(4, min(4096, args.cpu_seconds * rate / (S / 2))))
    dt, pairs = run(n_rows)
    tflops = FLOP_PER_PAIR * Hq * pairs / dt / 1e12
    full_pairs = S * (S + 1) // 2
    return {"value": round(tflops, 6), "unit": "TFLOP/s", "cores": oracle.num_threads(), "kind": "oracle",
            "sample": "%d uniformly drawn query rows x %d heads over their full causal key range "
                      "(%.3g visible pairs per head, %.1f s); full workload extrapolates to %.0f s"
                      % (n_rows, Hq, pairs, dt, full_pairs / (pairs / dt)),
            "tokens_per_s_extrapolated": round(S / (full_pairs / (pairs / dt)), 3)}


def bench_varlen(args, torch, np, pec, synth, dev):
    """Colocated batch: 256 log-normal short prompts + one 65,536-token prompt, one launch."""
    Hq, Hkv = 32, 8
    lengths = synth.varlen_lengths()
    cu = synth.cu_seqlens_of(lengths)
    T = int(cu[-1])
    q, k, v = synth.qkv(synth.VARLEN_SEED, T, T, Hq, Hkv, device=dev)
    cud = torch.from_numpy(cu).to(dev)
    out = torch.empty_like(q)
    lse = torch.empty((Hq, T), dtype=torch.float32, device=dev)
    ws = torch.empty(pec.pec_varlen_workspace_bytes(len(lengths), T), dtype=torch.uint8, device=dev)
    pairs = int(sum(int(n) * (int(n) + 1) // 2 for n in lengths))
    flops = FLOP_PER_PAIR * Hq * pairs
    max_len = int(lengths.max())

    def step():
        pec.pec_attn_varlen(q, k, v, cud, max_len, True, out=out, lse=lse, workspace=ws, flags=args.kernel_flag)

    ms_step, ev_list = timed_steps(torch, step, args.steps, args.warmup)
    ev_mean = sum(ev_list) / len(ev_list)
    ev_ms = ev_mean
    tflops = flops / (ms_step * 1e-3) / 1e12
    ach = flops / (ev_ms * 1e-3) / 1e12
    result = {
        "metric": "prefill attention TFLOP/s and tokens/s of the colocated packed batch; % of bf16 MFMA peak",
        "value": round(tflops, 2), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_step, 3), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "c4_varlen: %d packed prompts (256 log-normal short + one 65536), %d tokens, "
                               "32 q / 8 kv heads, causal per sequence" % (len(lengths), T), "total_tokens": T},
        "tokens_per_s": round(T / (ms_step * 1e-3), 1),
        "pct_of_bf16_mfma_peak": round(100.0 * tflops / PEAK_BF16_TFLOPS, 2),
        "ms_per_step_stats": step_stats(ev_list),
        "roofline": {"bound": "mfma", "achieved": round(ach, 2), "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                     "frac": round(ach / PEAK_BF16_TFLOPS, 4), "traffic": None,
                     "kernel": pec.KERNEL_NAMES[args.kernel_flag]},
    }
    print(json.dumps(result), flush=True)
    return 0


def bench_colocated(args, torch, np, pec, synth, dev):
    """The colocation case of the paper: 256 log-normal short prompts batched with the decode step of a long
    request whose KV cache holds 524,288 tokens (32 q / 8 kv heads), one pec_attn_colocated call."""
    Hq, Hkv, cache = 32, 8, 524288
    short = synth.lognormal_lengths(synth.VARLEN_SEED, synth.VARLEN_N_SHORT)
    len_q = np.concatenate([short, [1]])
    len_k = np.concatenate([short, [cache]])
    cq, ck = synth.cu_seqlens_of(len_q), synth.cu_seqlens_of(len_k)
    Tq, Tk = int(cq[-1]), int(ck[-1])
    q, _, _ = synth.qkv(synth.VARLEN_SEED, Tq, 1, Hq, Hkv, device=dev)
    _, k, v = synth.qkv(synth.VARLEN_SEED + 1, 1, Tk, Hq, Hkv, device=dev)
    cqd, ckd = torch.from_numpy(cq).to(dev), torch.from_numpy(ck).to(dev)
    out = torch.empty_like(q)
    lse = torch.empty((Hq, Tq), dtype=torch.float32, device=dev)
    shp = pec.PecShape(Hq, Hkv, 128, pec.PEC_BF16, 0.0, 0)
    ws = torch.empty(int(pec.lib().pec_colocated_workspace_bytes(ctypes.byref(shp), len(len_q), Tq, Tk)), dtype=torch.uint8,
                     device=dev)
    pairs = int(sum(int(n) * (int(n) + 1) // 2 for n in short)) + cache
    flops = FLOP_PER_PAIR * Hq * pairs
    decode_bytes = 2.0 * cache * Hkv * 128 * 2                # K and V of the long request, read once

    def step():
        pec.pec_attn_colocated(q, k, v, cqd, ckd, True, out=out, lse=lse, workspace=ws)

    ms_step, ev_list = timed_steps(torch, step, args.steps, args.warmup)
    ev_ms = sum(ev_list) / len(ev_list)
    tflops = flops / (ms_step * 1e-3) / 1e12
    # for comparison: the two parts as separate calls
    qs, ks, vs = q[:Tq - 1], k[:Tk - cache], v[:Tk - cache]
    cus = torch.from_numpy(synth.cu_seqlens_of(short)).to(dev)
    ws2 = torch.empty(pec.pec_varlen_workspace_bytes(len(short), Tq - 1), dtype=torch.uint8, device=dev)
    _, ev_p = timed_steps(torch, lambda: pec.pec_attn_varlen(qs, ks, vs, cus, int(short.max()), True, out=out[:Tq - 1],
                                                            lse=lse[:, :Tq - 1].contiguous(), workspace=ws2), args.steps, 1)
    o1 = torch.empty((1, Hq, 128), dtype=torch.float32, device=dev)
    l1 = torch.empty((Hq,), dtype=torch.float32, device=dev)
    _, ev_d = timed_steps(torch, lambda: pec.pec_decode_splitkv(q[Tq - 1:], k[Tk - cache:], v[Tk - cache:], out=o1, lse=l1),
                          args.steps, 1)
    result = {
        "metric": "colocated batch (short prefills + one long-request decode step) per launch; attention TFLOP/s",
        "value": round(tflops, 2), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_step, 3), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "c4_colocated: 256 log-normal short prompts (%d tokens) + the decode step of a request with "
                               "%d cached tokens, 32 q / 8 kv heads, one pec_attn_colocated call" % (Tq - 1, cache)},
        "tokens_per_s": round(Tq / (ms_step * 1e-3), 1),
        "ms_per_step_stats": step_stats(ev_list),
        "separate_calls_ms": {"pec_attn_varlen (prefills)": round(sum(ev_p) / len(ev_p), 3),
                              "pec_decode_splitkv (decode)": round(sum(ev_d) / len(ev_d), 3)},
        "decode_bytes_per_step": decode_bytes,
        "roofline": {"bound": "mfma", "achieved": round(flops / (ev_ms * 1e-3) / 1e12, 2), "peak": PEAK_BF16_TFLOPS,
                     "unit": "TFLOP/s", "frac": round(flops / (ev_ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 4), "traffic": None,
                     "kernel": "pec::fwd_il_kernel"},
    }
    print(json.dumps(result), flush=True)
    return 0


def bench_preempt(args, torch, np, pec, synth, dev):
    """Stopping and continuing a long prefill (section "Preemption of Long-Request Prefill"): the last c3 ring member's
    sweep (8192 query rows against 131072 keys in 16 segments) with the stop word, in pinned host memory, raised by
    the host some milliseconds into the kernel.  Reported: how long after the word is raised the host sees the kernel
    gone from the GPU, and what the stop and the continuation cost on top of the uninterrupted sweep."""
    import time

    w = synth.WORKLOADS["c3_gqa_128k"]
    S, C, Hq, Hkv = w.seq, w.chunk, w.n_q_heads, w.n_kv_heads
    lo = S - C
    q, k, v = synth.qkv(w.seed, C, S, Hq, Hkv, device=dev)
    out = torch.empty_like(q)
    lse = torch.empty((Hq, C), dtype=torch.float32, device=dev)
    ws = torch.empty(pec.pec_sp_resumable_workspace_bytes(q, k), dtype=torch.uint8, device=dev)
    stop = torch.zeros(1, dtype=torch.int32).pin_memory()
    pending = torch.zeros(1, dtype=torch.int32, device=dev)
    ev = lambda: torch.cuda.Event(enable_timing=True)   # noqa: E731

    def sweep(resume):
        pec.pec_sp_prefill_resumable(q, k, v, lo, C, out, lse, ws, pending, stop=stop, resume=resume)

    _, ev_full = timed_steps(torch, lambda: sweep(False), args.steps, args.warmup)
    full_ms = sorted(ev_full)[len(ev_full) // 2]
    latencies, overheads, left = [], [], []
    trials = max(args.steps, 10)
    for t in range(trials):
        stop[0] = 0
        torch.cuda.synchronize()
        delay_s = (0.15 + 0.7 * t / max(1, trials - 1)) * full_ms * 1e-3      # 15 ... 85 % into the kernel
        e0, e1, e2, e3 = ev(), ev(), ev(), ev()
        e0.record()
        sweep(False)
        e1.record()
        t_launch = time.perf_counter()
        while time.perf_counter() - t_launch < delay_s:
            pass
        stop[0] = 1
        t_raise = time.perf_counter()
        while not e1.query():
            pass
        t_gone = time.perf_counter()
        torch.cuda.synchronize()
        n_left = int(pending.item())
        if n_left == 0:
            continue                      # the kernel was through before the word was raised
        stop[0] = 0
        e2.record()
        sweep(True)
        e3.record()
        torch.cuda.synchronize()
        if int(pending.item()) != 0:
            print("bench.py: the continued sweep did not finish", file=sys.stderr)
            return 1
        latencies.append(1e3 * (t_gone - t_raise))
        overheads.append(e0.elapsed_time(e1) + e2.elapsed_time(e3) - full_ms)
        left.append(n_left)
    if not latencies:
        print("bench.py: no sweep was interrupted", file=sys.stderr)
        return 1
    items_per_cu = max(1, (C // 256) * Hq // 256)
    result = {
        "metric": "time from raising the stop word to the prefill kernel having left the GPU (seen from the host)",
        "value": round(step_stats(latencies)["median"], 4),
        "unit": "ms", "n_gpus": 1, "steps": len(latencies), "warmup": args.warmup, "ms_per_step": round(full_ms, 3),
        "higher_is_better": False, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "c3_preempt: last ring member of c3_gqa_128k (8192 query rows, 131072 keys in 16 segments), one "
                               "stoppable sweep launch, stop word in pinned host memory raised by the host 15 ... 85 % into it, "
                               "then continued to the end"},
        "stop_latency_ms": step_stats(latencies),
        "one_key_segment_of_one_query_tile_ms": round(full_ms / (S // C) / items_per_cu, 4),
        "stop_and_continue_overhead_ms": step_stats(overheads),
        "uninterrupted_sweep_ms": round(full_ms, 3),
        "work_items_left_at_stop": {"min": min(left), "max": max(left), "of": (C // 256) * Hq},
    }
    print(json.dumps(result), flush=True)
    return 0


def bench_ulysses(args, torch, np, pec, synth, dev):
    """Head <-> sequence layout exchange (on-GPU half): segment of 16384 tokens, 64 heads, 8 GPUs."""
    s_len, H, G = 16384, 64, 8
    x = synth.randn_bf16((s_len, H, 128), 1006, dev)
    y = torch.empty((G, s_len, H // G, 128), dtype=torch.bfloat16, device=dev)
    z = torch.empty_like(x)
    algo_bytes = 2.0 * x.numel() * 2            # read once, written once

    def step():
        pec.pec_ulysses_layout(x, G, True, out=y)
        pec.pec_ulysses_layout(y, G, False, out=z)

    steps = max(args.steps, 20)
    ms_step, ev_list = timed_steps(torch, step, steps, max(args.warmup, 3))
    ev_mean = sum(ev_list) / len(ev_list)
    ev_ms = ev_mean / 2    # per kernel launch
    gbs = algo_bytes / (ev_ms * 1e-3) / 1e9
    assert torch.equal(z, x)
    result = {
        "metric": "Ulysses layout exchange, tokens/s through pack + unpack", "value": round(s_len / (ms_step * 1e-3), 1),
        "unit": "tokens/s", "n_gpus": 1, "steps": steps, "warmup": max(args.warmup, 3), "ms_per_step": round(ms_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "ulysses_layout: [16384, 64, 128] bf16 <-> [8, 16384, 8, 128], both directions per step"},
        "ms_per_step_stats": step_stats(ev_list),
        "roofline": {"bound": "hbm", "achieved": round(gbs, 1), "peak": 8000.0, "unit": "GB/s",
                     "frac": round(gbs / 8000.0, 4), "traffic": None, "kernel": "pec::ulysses_layout_kernel"},
    }
    del y, z
    probe = hbm_read_probe(torch, pec, dev)
    result["hbm_read_probe"] = probe
    result["pct_of_measured_read_bandwidth"] = round(100.0 * gbs / probe["read_gbs"], 2)
    print(json.dumps(result), flush=True)
    return 0


def bench_decode(args, torch, np, pec, synth, dev):
    """Long-request decode step: one new token against a 524,288-token KV-cache shard (64 q / 8 kv heads).
    HBM-bound: K and V are read once."""
    Hq, Hkv, sk = 64, 8, 524288
    q, k, v = synth.qkv(1005, 1, sk, Hq, Hkv, device=dev)
    shp = pec.PecShape(Hq, Hkv, 128, 1, 0.0, 0)
    n_splits = args.decode_splits or int(pec.lib().pec_decode_default_splits(ctypes.byref(shp), sk))   # key ranges per KV head
    out = torch.empty((1, Hq, 128), dtype=torch.float32, device=dev)
    lse = torch.empty((Hq,), dtype=torch.float32, device=dev)
    ws = torch.empty(n_splits * Hq * 129 * 4, dtype=torch.uint8, device=dev)
    algo_bytes = 2.0 * sk * Hkv * 128 * 2 + 2 * Hq * 128 * 2 + Hq * 4      # K + V once, q, out, lse

    def step():
        pec.pec_decode_splitkv(q, k, v, n_splits=n_splits, out=out, lse=lse, workspace=ws)

    steps = max(args.steps, 20)
    ms_step, ev_list = timed_steps(torch, step, steps, max(args.warmup, 3))
    ev_mean = sum(ev_list) / len(ev_list)
    ev_ms = ev_mean
    gbs = algo_bytes / (ev_ms * 1e-3) / 1e9
    result = {
        "metric": "decode attention step over a 512K-token KV shard", "value": round(1e3 / ms_step, 1),
        "unit": "tokens/s", "n_gpus": 1, "steps": steps, "warmup": max(args.warmup, 3), "ms_per_step": round(ms_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "decode_512k: 1 query token, 64 q / 8 kv heads, KV shard of 524288 tokens, %d key splits"
                               % n_splits},
        "ms_per_step_stats": step_stats(ev_list),
        "roofline": {"bound": "hbm", "achieved": round(gbs, 1), "peak": 8000.0, "unit": "GB/s",
                     "frac": round(gbs / 8000.0, 4), "traffic": None, "kernel": "pec::decode_kernel + pec::combine_splits_kernel"},
    }
    probe = hbm_read_probe(torch, pec, dev)
    result["hbm_read_probe"] = probe
    result["pct_of_measured_read_bandwidth"] = round(100.0 * gbs / probe["read_gbs"], 2)
    print(json.dumps(result), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
