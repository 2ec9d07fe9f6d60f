#!/usr/bin/env python3
"""Benchmark of the tensorized-attention hot path on one MI355X.

One "step" = one pass of Algorithm 1 (all hops of ta_multihop_forward) over one batch
of synthetic Q, K, V that already live in HBM.  Prints ONE JSON line:
  metric/value/unit : tokens/s of the whole multi-hop forward (B*N / step time)
  roofline          : the per-axis attention kernel against the 8 TB/s HBM peak, from
                      HIP-event timings of every hop launch (algorithmic bytes / time)
  cpu_baseline      : the CPU oracle, as it stands, timed on a bounded sample (whole
                      sequences of a few heads) on the host cores of this machine
Usage: python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload c3|c4|c2|c5]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E peak


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="c3", choices=["c2", "c3", "c4", "c5"])
    ap.add_argument("--rotate", type=int, default=3, help="independent buffer sets cycled through, so that the "
                    "256 MB Infinity Cache cannot serve one step's re-reads from the previous step")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--copy-calibration", action="store_true", help="also launch the plain copy kernel on 1 GiB a few "
                    "times, so that a hardware-counter run of this command has a transfer of known size to scale by")
    ap.add_argument("--cpu-seconds", type=float, default=15.0, help="target CPU time of the oracle sample")
    return ap.parse_args()


def make_sets(torch, w, rotate):
    """`rotate` independent (q, k, v, o, workspace) sets, generated on the device from a seed."""
    import paper_2410_20926_amd as ta
    B, N, Hq, Hkv, D = w.batch, w.seq_len, w.n_q_heads, w.n_kv_heads, w.head_dim
    plan = ta.ta_plan_create(B, Hq, Hkv, D, w.dims, ta.TA_BF16, w.causal)
    gen = torch.Generator(device="cuda")
    gen.manual_seed(w.seed)
    wsb = plan.workspace_bytes(False)
    sets = []
    for _ in range(rotate):
        q = (torch.randn(B, N, Hq, D, device="cuda", generator=gen) * w.qk_prescale).to(torch.bfloat16)
        k = (torch.randn(B, N, Hkv, D, device="cuda", generator=gen) * w.qk_prescale).to(torch.bfloat16)
        v = torch.randn(B, N, Hkv, D, device="cuda", generator=gen).to(torch.bfloat16)
        o = torch.empty(B, N, Hq, D, device="cuda", dtype=torch.bfloat16)
        ws = torch.empty(max(wsb, 256), dtype=torch.uint8, device="cuda")
        sets.append((q, k, v, o, ws))
    return plan, sets, wsb


def time_steps(torch, ta, plan, sets, wsb, steps, warmup):
    """Wall time of exactly `steps` multi-hop forwards, synchronised on both sides."""
    for i in range(warmup):
        q, k, v, o, ws = sets[i % len(sets)]
        ta.ta_multihop_forward(plan, q, k, v, o, ws, wsb, False)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        q, k, v, o, ws = sets[i % len(sets)]
        ta.ta_multihop_forward(plan, q, k, v, o, ws, wsb, False)
    torch.cuda.synchronize()
    return time.perf_counter() - t0


def time_hops(torch, ta, plan, sets, w, steps):
    """HIP-event duration of every per-axis launch, on the stream the kernels run on
    (torch's current stream, which the binding hands to the library).  Returns per hop
    position the list of durations in seconds."""
    B, N, Hq, D = w.batch, w.seq_len, w.n_q_heads, w.head_dim
    m = len(w.dims)
    o_elems = B * N * Hq * D
    per_hop = [[] for _ in range(m)]
    events = []
    for i in range(steps):
        q, k, v, o, ws = sets[i % len(sets)]
        bufs = [ws[j * plan_o_bytes(plan, w):][:o_elems * 2].view(torch.bfloat16).view(B, N, Hq, D) for j in range(2)]
        cur, kind = v, ta.TA_VIN_KV
        for pos in range(m):
            dst = o if pos == m - 1 else bufs[pos & 1]
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            ta.ta_axis_attn_forward(plan, plan.hop_axis(pos), q, k, cur, kind, dst)
            e1.record()
            events.append((pos, e0, e1))
            cur, kind = dst, ta.TA_VIN_O
    torch.cuda.synchronize()
    for pos, e0, e1 in events:
        per_hop[pos].append(e0.elapsed_time(e1) * 1e-3)
    return per_hop


def plan_o_bytes(plan, w):
    n = w.batch * w.seq_len * w.n_q_heads * w.head_dim * 2
    return (n + 255) // 256 * 256


def cpu_baseline(w, target_seconds):
    """The oracle, untuned, on whole sequences of a few query heads of the same workload
    (heads are independent, so tokens/s of the full job = N*B / (t_per_head * H_q))."""
    import numpy as np
    from oracle import tensattn_oracle as orc
    from paper_2410_20926_amd.workloads import make_inputs
    q, k, v = make_inputs(1, w.seq_len, 1, 1, w.head_dim, w.seed, "bf16", w.qk_prescale)
    heads = 0
    c0 = time.process_time()
    t0 = time.perf_counter()
    while True:
        orc.tensorized_attention_forward(q, k, v, w.dims, w.causal)
        heads += 1
        el = time.perf_counter() - t0
        if el + el / heads > target_seconds:
            break
    wall = time.perf_counter() - t0
    cpu = time.process_time() - c0
    per_head = wall / heads
    tokens_per_s = w.batch * w.seq_len / (per_head * w.batch * w.n_q_heads)
    return {
        "value": tokens_per_s, "unit": "tokens/s", "cores": max(1, int(round(cpu / wall))),
        "host_cores": len(os.sched_getaffinity(0)), "kind": "oracle",
        "sample": f"{heads} single-head passes of {w.name} (all {w.seq_len} tokens, all hops; the job has "
                  f"{w.batch * w.n_q_heads} such heads), {wall:.1f} s wall; scaled by heads",
    }


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build measures one GPU only (every box here has one); run with --gpus 1",
              file=sys.stderr)
        sys.exit(2)
    import torch
    import paper_2410_20926_amd as ta
    from paper_2410_20926_amd.workloads import WORKLOADS
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    ta.load_library()                                   # fails loudly when the HIP library is missing
    w = WORKLOADS[args.workload]
    plan, sets, wsb = make_sets(torch, w, args.rotate)
    m = len(w.dims)

    wall = time_steps(torch, ta, plan, sets, wsb, args.steps, args.warmup)
    ms_per_step = wall / args.steps * 1e3
    tokens_per_s = w.batch * w.seq_len / (wall / args.steps)

    per_hop = time_hops(torch, ta, plan, sets, w, args.steps)
    hop_bytes = [plan.hop_bytes(plan.hop_axis(pos), ta.TA_VIN_KV if pos == 0 else ta.TA_VIN_O) for pos in range(m)]
    hop_flops = [plan.hop_flops(plan.hop_axis(pos)) for pos in range(m)]
    hop_avg = [sum(ts) / len(ts) for ts in per_hop]
    hops = []
    for pos in range(m):
        axis = plan.hop_axis(pos)
        gbs = hop_bytes[pos] / hop_avg[pos] / 1e9
        hops.append({"hop": pos, "axis": axis, "n": w.dims[axis],
                     "kernel": plan.hop_kernel(axis, ta.TA_VIN_KV if pos == 0 else ta.TA_VIN_O),
                     "us": round(hop_avg[pos] * 1e6, 2), "algorithmic_bytes": hop_bytes[pos],
                     "GBps": round(gbs, 1), "frac_of_8TBps": round(gbs / HBM_PEAK_GBS, 4),
                     "TFLOPs_executed": round(hop_flops[pos] / hop_avg[pos] / 1e12, 1)})
    # the per-axis attention kernel is the only kernel on the path: all launches, averaged
    launches = sum(len(ts) for ts in per_hop)
    avg_bytes = sum(hop_bytes[pos] * len(per_hop[pos]) for pos in range(m)) / launches
    avg_dur = sum(sum(ts) for ts in per_hop) / launches
    achieved = avg_bytes / avg_dur / 1e9
    roofline = {"bound": "hbm", "kernel": hops[-1]["kernel"], "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS,
                "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": None,
                "avg_launch_us": round(avg_dur * 1e6, 2), "algorithmic_bytes_per_launch": avg_bytes,
                "launches_timed": launches, "per_hop": hops}

    if args.copy_calibration:
        nbytes = 1 << 30
        src = torch.zeros(nbytes, dtype=torch.uint8, device="cuda")
        dst = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
        for _ in range(3):
            ta.ta_copy_bytes(src, dst, nbytes)
        torch.cuda.synchronize()

    out = {
        "metric": "tensorized-attn tokens/s + per-hop HBM GB/s (% peak) at N=32k, 128k",
        "value": tokens_per_s, "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{w.name}: bf16 forward, B={w.batch}, {w.n_q_heads} query / {w.n_kv_heads} kv heads, "
                               f"D={w.head_dim}, N={w.seq_len} as {'x'.join(map(str, w.dims))}, "
                               f"{'causal' if w.causal else 'non-causal'}",
                   "rotating_buffer_sets": args.rotate},
        "roofline": roofline,
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w, args.cpu_seconds)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
