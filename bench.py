#!/usr/bin/env python3
"""Benchmark of the tensorized-attention hot path on one MI355X.

One "step" = one pass of Algorithm 1 (all hops of ta_multihop_forward; for the training
workload c5 also ta_multihop_backward) over one batch of synthetic Q, K, V (and dO) that
already live in HBM.  Prints ONE JSON line:
  metric/value/unit : tokens/s of the whole multi-hop forward (B*N / step time)
  roofline          : the per-axis attention kernel against the 8 TB/s HBM peak, from
                      HIP-event timings of every hop launch (algorithmic bytes / time)
  cpu_baseline      : the CPU oracle, as it stands, timed on a bounded sample (whole
                      sequences of a few heads) on the host cores of this machine
Usage: python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload c3|c4|c2|c5|c6|c3_rope|c4_train]
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
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="c3", choices=["c2", "c3", "c4", "c5", "c6", "c3_rope", "c4_train", "c3_w100_train"])
    ap.add_argument("--rotate", type=int, default=3, help="independent buffer sets cycled through, so that the "
                    "256 MB Infinity Cache cannot serve one step's re-reads from the previous step")
    ap.add_argument("--also", default=None, help="comma-separated further workloads measured in the same run and "
                    "reported under other_workloads (default: c2,c4,c5,c6,c3_rope,c4_train,c3_w100_train next to c3, none otherwise)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--copy-calibration", action="store_true", help="also launch the plain copy kernel on 1 GiB a few "
                    "times, so that a hardware-counter run of this command has a transfer of known size to scale by")
    ap.add_argument("--cpu-seconds", type=float, default=15.0, help="target CPU time of the oracle sample")
    args = ap.parse_args()
    if args.also is None:
        args.also = "c2,c4,c5,c6,c3_rope,c4_train,c3_w100_train" if args.workload == "c3" else ""
    return args


def make_sets(torch, w, rotate):
    """`rotate` independent (q, k, v, o, workspace) sets, generated on the device from a seed."""
    import paper_2410_20926_amd as ta
    B, N, Hq, Hkv, D = w.batch, w.seq_len, w.n_q_heads, w.n_kv_heads, w.head_dim
    plan = ta.ta_plan_create(B, Hq, Hkv, D, w.dims, ta.TA_BF16, w.causal, rope_base=w.rope_base)
    gen = torch.Generator(device="cuda")
    gen.manual_seed(w.seed)
    wsb = plan.workspace_bytes(w.backward)
    scb = plan.backward_scratch_bytes() if w.backward else 0
    sets = []
    for _ in range(rotate):
        q = (torch.randn(B, N, Hq, D, device="cuda", generator=gen) * w.qk_prescale).to(torch.bfloat16)
        k = (torch.randn(B, N, Hkv, D, device="cuda", generator=gen) * w.qk_prescale).to(torch.bfloat16)
        v = torch.randn(B, N, Hkv, D, device="cuda", generator=gen).to(torch.bfloat16)
        o = torch.empty(B, N, Hq, D, device="cuda", dtype=torch.bfloat16)
        ws = torch.empty(max(wsb, 256), dtype=torch.uint8, device="cuda")
        st = {"q": q, "k": k, "v": v, "o": o, "ws": ws}
        if w.backward:
            st["d_o"] = torch.randn(B, N, Hq, D, device="cuda", generator=gen).to(torch.bfloat16)
            st["dq"], st["dk"], st["dv"] = torch.empty_like(q), torch.empty_like(k), torch.empty_like(v)
            st["sc"] = torch.empty(max(scb, 256), dtype=torch.uint8, device="cuda")
        sets.append(st)
    return plan, sets, wsb, scb


def one_step(ta, plan, st, wsb, scb, backward):
    """One pass of the whole hot path: Algorithm 1 forward, plus the backward for a training workload."""
    ta.ta_multihop_forward(plan, st["q"], st["k"], st["v"], st["o"], st["ws"], wsb, backward)
    if backward:
        ta.ta_multihop_backward(plan, st["q"], st["k"], st["v"], st["d_o"], st["ws"], wsb,
                                st["dq"], st["dk"], st["dv"], st["sc"], scb)


def time_steps(torch, ta, plan, sets, wsb, scb, backward, steps, warmup):
    """Wall time of exactly `steps` steps, synchronised on both sides."""
    for i in range(warmup):
        one_step(ta, plan, sets[i % len(sets)], wsb, scb, backward)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        one_step(ta, plan, sets[i % len(sets)], wsb, scb, backward)
    torch.cuda.synchronize()
    return time.perf_counter() - t0


def time_hops(torch, ta, plan, sets, w, steps):
    """HIP-event duration of every per-axis launch, on the stream the kernels run on
    (torch's current stream, which the binding hands to the library).  Returns a list of
    records (direction, hop position, axis, value-input kind, seconds); direction "fwd2" is the
    fused launch of two hops (the one at `axis` and the next), which the inference forward uses
    for its last two hops when the plan offers it."""
    B, N, Hq, D = w.batch, w.seq_len, w.n_q_heads, w.head_dim
    m = len(w.dims)
    o_elems = B * N * Hq * D
    ob = plan_o_bytes(plan, w)
    events = []

    def timed(tag, fn):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        fn()
        e1.record()
        events.append(tag + (e0, e1))

    def view(buf, j):
        return buf[j * ob:][:o_elems * 2].view(torch.bfloat16).view(B, N, Hq, D)

    for i in range(steps):
        st = sets[i % len(sets)]
        q, k, v, o, ws = st["q"], st["k"], st["v"], st["o"], st["ws"]
        inter = [view(ws, j) for j in range(ws.numel() // ob)]    # as many inter-hop buffers as the plan asked for
        srcs = []
        cur, kind = v, ta.TA_VIN_KV
        fused = plan.fused_position()
        for pos in range(m):
            axis = plan.hop_axis(pos)
            if pos == fused:                             # a training step also gets the O between the two hops
                mid = inter[pos] if w.backward else None
                timed(("fwd2", pos, axis, kind), lambda: ta.ta_axis_pair_attn_forward(plan, axis, q, k, cur, kind, o, o_mid=mid))
                srcs.append((cur, kind))
                srcs.append((mid, ta.TA_VIN_O))
                break
            dst = o if pos == m - 1 else (inter[pos] if w.backward else inter[pos % len(inter)])
            timed(("fwd", pos, axis, kind), lambda: ta.ta_axis_attn_forward(plan, axis, q, k, cur, kind, dst))
            srcs.append((cur, kind))
            cur, kind = dst, ta.TA_VIN_O
        if w.backward:
            grad = st["d_o"]
            for pos in range(m - 1, -1, -1):
                x, kind = srcs[pos]
                gprev = st["dv"] if pos == 0 else view(st["sc"], pos & 1)
                axis = plan.hop_axis(pos)
                acc = pos != m - 1
                timed(("bwd", pos, axis, kind), lambda: ta.ta_axis_attn_backward(
                    plan, axis, q, k, x, kind, grad, gprev, st["dq"], st["dk"], acc))
                grad = gprev
    torch.cuda.synchronize()
    return [(d, pos, axis, kind, e0.elapsed_time(e1) * 1e-3) for d, pos, axis, kind, e0, e1 in events]


def plan_o_bytes(plan, w):
    n = w.batch * w.seq_len * w.n_q_heads * w.head_dim * 2
    return (n + 255) // 256 * 256


def _cpu_worker(job):
    """One worker process of the CPU baseline: `passes` whole single-head passes of the oracle.
    Returns (wall seconds, CPU seconds) of the timed passes."""
    name, worker, passes = job
    from oracle import tensattn_oracle as orc
    from paper_2410_20926_amd.workloads import WORKLOADS, make_inputs
    w = WORKLOADS[name]
    q, k, v, d_o = make_inputs(1, w.seq_len, 1, 1, w.head_dim, w.seed + worker, "bf16", w.qk_prescale, with_grad=True)

    def one_head():
        if w.backward:                                  # the oracle's backward runs its own forward first
            orc.tensorized_attention_backward(q, k, v, d_o, w.dims, w.causal)
        else:
            orc.tensorized_attention_forward(q, k, v, w.dims, w.causal)

    one_head()                                          # first touch of the code and the arrays, untimed
    c0, t0 = time.process_time(), time.perf_counter()
    for _ in range(passes):
        one_head()
    return time.perf_counter() - t0, time.process_time() - c0


def cpu_baseline(w, target_seconds):
    """The oracle, untuned, on whole sequences of single query heads of the same workload, on
    ALL host cores of this process: one worker process per core (heads are independent; the
    oracle's NumPy code holds the interpreter lock most of the time, so threads would not
    scale), each running the same number of single-head passes.  tokens/s of the full job =
    B * N / (wall time per head-pass * B * H_q).  Must run before this process touches the GPU:
    the workers are fresh interpreters started by multiprocessing's spawn method."""
    import multiprocessing as mp
    host_cores = len(os.sched_getaffinity(0))
    ctx = mp.get_context("spawn")
    with ctx.Pool(host_cores) as pool:
        t_one = pool.map(_cpu_worker, [(w.name, 0, 1)])[0][0]                 # sizes the sample
        passes = max(1, int(target_seconds / max(2.0 * t_one, 1e-3)))            # passes slow down when all cores are busy
        t0 = time.perf_counter()
        res = pool.map(_cpu_worker, [(w.name, i, passes) for i in range(host_cores)], chunksize=1)
        wall_all = time.perf_counter() - t0
    wall = max(r[0] for r in res)                                                # timed part of the slowest worker
    cpu = sum(r[1] for r in res)
    heads = passes * host_cores
    tokens_per_s = w.batch * w.seq_len / (wall / heads * w.batch * w.n_q_heads)
    return {
        "value": tokens_per_s, "unit": "tokens/s", "cores": max(1, int(round(cpu / wall))),
        "host_cores": host_cores, "kind": "oracle",
        "sample": f"{heads} single-head passes of {w.name} (all {w.seq_len} tokens, all hops"
                  f"{', forward + backward' if w.backward else ''}; the job has "
                  f"{w.batch * w.n_q_heads} such heads), {passes} on each of {host_cores} worker processes, {wall:.1f} s wall "
                  f"({wall_all:.1f} s with process start-up), {cpu:.1f} s CPU; one pass on an otherwise idle machine takes "
                  f"{t_one * 1e3:.0f} ms; scaled by heads",
    }


def full_attention_reference(torch, ta, workloads):
    """Plain causal attention (tensor order 1: one hop over the whole sequence, the library's
    streaming kernel) on the same GPU at the two sequence lengths, and the tensorized / full time
    ratio next to the paper's whole-model figures for the same lengths (Table 3, Llama-8B row:
    context only, another machine and a whole model)."""
    from paper_2410_20926_amd.workloads import Workload
    out = {}
    for name, paper_ratio in (("c3", 0.25), ("c4", 0.09)):
        w, tens_ms = workloads[name]
        full = Workload(f"{name}_order1", w.index, "bf16", w.batch, w.n_q_heads, w.n_kv_heads, w.head_dim, (w.seq_len,), True, w.qk_prescale)
        plan, sets, wsb, scb = make_sets(torch, full, 1)
        steps = 5 if w.seq_len <= 32768 else 3
        wall = time_steps(torch, ta, plan, sets, wsb, scb, False, steps, 1)
        ms = wall / steps * 1e3
        out[f"N={w.seq_len}"] = {"full_attention_ms": round(ms, 3), "tensorized_ms": round(tens_ms, 4), "kernel": plan.hop_kernel(0, 0),
                                 "tensorized_over_full": round(tens_ms / ms, 5), "paper_table3_llama8b_whole_model": paper_ratio}
        del sets
        torch.cuda.empty_cache()
    return out


def measure(torch, ta, w, args, steps, warmup):
    """Times `steps` whole steps and every hop launch of workload `w`; returns
    (tokens/s, ms per step, roofline record of the dominant kernel)."""
    plan, sets, wsb, scb = make_sets(torch, w, args.rotate)
    m = len(w.dims)

    wall = time_steps(torch, ta, plan, sets, wsb, scb, w.backward, steps, warmup)
    ms_per_step = wall / steps * 1e3
    tokens_per_s = w.batch * w.seq_len / (wall / steps)

    records = time_hops(torch, ta, plan, sets, w, steps)
    hops = []
    groups = {}
    for d, pos, axis, kind, sec in records:
        groups.setdefault((d, pos, axis, kind), []).append(sec)
    kernel_totals = {}                                   # kernel name -> [bytes, seconds, launches]
    for (d, pos, axis, kind), ts in groups.items():
        bwd = d == "bwd"
        if d == "fwd2":
            nbytes = plan.pair_bytes(axis, kind)
            if w.backward:                               # plus the write of the O between the two hops
                nbytes += w.batch * w.seq_len * w.n_q_heads * w.head_dim * 2
            flops = plan.hop_flops(axis, False) + plan.hop_flops(axis + 1, False)
            name = plan.pair_kernel(axis, kind)
        else:
            nbytes = plan.hop_bytes(axis, kind, bwd, bwd and pos != m - 1)
            flops = plan.hop_flops(axis, bwd)
            name = plan.hop_backward_kernel(axis, kind) if bwd else plan.hop_kernel(axis, kind)
        avg = sum(ts) / len(ts)
        gbs = nbytes / avg / 1e9
        hops.append({"pass": d, "hop": pos, "axis": axis, "n": w.dims[axis], "kernel": name, "us": round(avg * 1e6, 2),
                     "algorithmic_bytes": nbytes, "GBps": round(gbs, 1), "frac_of_8TBps": round(gbs / HBM_PEAK_GBS, 4),
                     "TFLOPs_executed": round(flops / avg / 1e12, 1)})
        tot = kernel_totals.setdefault(name, [0.0, 0.0, 0])
        tot[0] += nbytes * len(ts)
        tot[1] += sum(ts)
        tot[2] += len(ts)
    # roofline of the dominant kernel (most time in the timed region), all its launches averaged
    dom = max(kernel_totals, key=lambda k_: kernel_totals[k_][1])
    nb, sec, launches = kernel_totals[dom]
    achieved = nb / sec / 1e9
    # HBM bytes per launch from the hardware counters of an earlier rocprofv3 --pmc run of this
    # command (FETCH_SIZE and WRITE_SIZE, scaled by the copy kernel; see profiles/), when one is stored
    traffic, traffic_source = None, None
    tpath = os.path.join(ROOT, "profiles", f"traffic_{w.name}.json")
    if os.path.exists(tpath):
        rec = json.load(open(tpath)).get(dom)
        if rec:
            traffic = rec["fetch_bytes_per_launch"] + rec["write_bytes_per_launch"]
            traffic_source = (f"stored: profiles/traffic_{w.name}.json, written by `python -m paper_2410_20926_amd.counters` from the "
                              f"rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs listed in profiles/tensattn_{w.name}.txt (not measured in this run)")
    roofline = {"bound": "hbm", "kernel": dom, "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS,
                "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": traffic, "traffic_source": traffic_source,
                "avg_launch_us": round(sec / launches * 1e6, 2), "algorithmic_bytes_per_launch": nb / launches,
                "launches_timed": launches, "per_hop": hops}

    del sets
    torch.cuda.empty_cache()
    return tokens_per_s, ms_per_step, roofline


def describe(w):
    return (f"{w.name}: bf16, B={w.batch}, {w.n_q_heads} query / {w.n_kv_heads} kv heads, D={w.head_dim}, "
            f"N={w.seq_len} as {'x'.join(map(str, w.dims))}, {'forward + backward, ' if w.backward else ''}"
            f"{'causal' if w.causal else 'non-causal'}{', per-axis rotary encoding inside the hops' if w.rope_base else ''}")


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build measures one GPU only (every box here has one); run with --gpus 1",
              file=sys.stderr)
        sys.exit(2)
    from paper_2410_20926_amd.workloads import WORKLOADS
    # the CPU baseline runs first: its worker processes must exist before this process initialises the GPU
    cpu = None if args.no_cpu_baseline else cpu_baseline(WORKLOADS[args.workload], args.cpu_seconds)
    import torch
    import paper_2410_20926_amd as ta
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    ta.load_library()                                   # fails loudly when the HIP library is missing
    w = WORKLOADS[args.workload]
    tokens_per_s, ms_per_step, roofline = measure(torch, ta, w, args, args.steps, args.warmup)
    others = {}
    step_ms = {args.workload: ms_per_step}
    for name in [x for x in args.also.split(",") if x and x != args.workload]:
        ow = WORKLOADS[name]
        tps, ms, rf = measure(torch, ta, ow, args, max(5, args.steps // 2), max(2, args.warmup // 2))
        step_ms[name] = ms
        others[name] = {"tokens_per_s": tps, "ms_per_step": ms, "workload": describe(ow),
                        "roofline_kernel": rf["kernel"], "roofline_GBps": rf["achieved"], "roofline_frac": rf["frac"],
                        "per_hop": [{k_: h_[k_] for k_ in ("pass", "hop", "n", "kernel", "us", "GBps", "frac_of_8TBps")}
                                    for h_ in rf["per_hop"]]}

    # the plain copy kernel on 1 GiB (read once, written once): the copy rate this machine reaches, next to the 8 TB/s peak;
    # its launches also give the counter runs their calibration (--copy-calibration keeps that name)
    nbytes = 1 << 30
    src = torch.zeros(nbytes, dtype=torch.uint8, device="cuda")
    dst = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    copy_ms = []
    for i in range(5):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        ta.ta_copy_bytes(src, dst, nbytes)
        e1.record()
        torch.cuda.synchronize()
        if i >= 2:
            copy_ms.append(e0.elapsed_time(e1))
    del src, dst
    copy_gbs = 2 * nbytes / (sorted(copy_ms)[len(copy_ms) // 2] * 1e-3) / 1e9
    roofline["copy_GBps"] = round(copy_gbs, 1)
    roofline["frac_of_copy"] = round(roofline["achieved"] / copy_gbs, 4)

    # what the memory gives a kernel that only moves the roofline kernel's mix of reads and writes (a forward hop
    # reads Q, K and its value input and writes O): the library's streaming kernel with the nearest mix it has,
    # on about as many bytes as one launch of that kernel
    dom = [h_ for h_ in roofline["per_hop"] if h_["kernel"] == roofline["kernel"]][0]
    if dom["pass"] in ("fwd", "fwd2"):
        hv = w.n_kv_heads if dom["hop"] == 0 else w.n_q_heads     # heads of the value input: V for the first hop, an O after it
        reads, writes = w.n_q_heads + w.n_kv_heads + hv, w.n_q_heads
        mixes = ((1, 1), (4, 3), (3, 2), (2, 1), (9, 4), (3, 1))
        r_, w_ = min(mixes, key=lambda m: abs(m[0] / m[1] - reads / writes))
        units = max(1, int(dom["algorithmic_bytes"] // ((r_ + w_) * 4096)))
        src = torch.zeros(units * r_ * 4096, dtype=torch.uint8, device="cuda")
        dst = torch.empty(units * w_ * 4096, dtype=torch.uint8, device="cuda")
        mix_ms = []
        for i in range(7):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            ta.ta_stream_mix(src, dst, units, r_, w_)
            e1.record()
            torch.cuda.synchronize()
            if i >= 2:
                mix_ms.append(e0.elapsed_time(e1))
        del src, dst
        mix_gbs = units * (r_ + w_) * 4096 / (sorted(mix_ms)[len(mix_ms) // 2] * 1e-3) / 1e9
        roofline["stream_same_mix"] = {"reads_to_writes": f"{r_}:{w_}", "GBps": round(mix_gbs, 1),
                                       "achieved_over_stream": round(roofline["achieved"] / mix_gbs, 4)}
    # The fused pair moves its bytes in a pattern that LDS capacity dictates (128-byte lines of one head's rows at the
    # token pitch, the four heads of a group on four workgroups): the same traffic without the arithmetic, and for
    # comparison with 1 KB of a token's head group at a time (the pattern of the single-hop kernels).
    if roofline["kernel"] == "mfma_bf16_pair_n32" and w.head_dim == 128 and w.seq_len % 1024 == 0:
        T = w.batch * w.seq_len
        bufs = [(torch.zeros(T * w.n_q_heads * 128, dtype=torch.int16, device="cuda"), torch.zeros(T * w.n_kv_heads * 128, dtype=torch.int16, device="cuda"),
                 torch.zeros(T * w.n_q_heads * 128, dtype=torch.int16, device="cuda"), torch.empty(T * w.n_q_heads * 128, dtype=torch.int16, device="cuda"))
                for _ in range(2)]
        rates = {}
        for granule in (1, 3):
            ms = []
            for i in range(8):
                q_, k_, x_, o_ = bufs[i % 2]
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                ta.ta_stream_slabs(q_, k_, x_, o_, T, w.n_q_heads, w.n_kv_heads, granule)
                e1.record()
                torch.cuda.synchronize()
                if i >= 2:
                    ms.append(e0.elapsed_time(e1))
            rates[granule] = dom["algorithmic_bytes"] / (sorted(ms)[len(ms) // 2] * 1e-3) / 1e9
        del bufs
        roofline["stream_same_pattern"] = {"GBps": round(rates[1], 1), "achieved_over_stream": round(roofline["achieved"] / rates[1], 4),
                                           "pattern": "128-byte lines of one head's rows, one workgroup per (1,024-token slab, head)",
                                           "GBps_with_1KB_head_groups": round(rates[3], 1)}

    out = {
        "metric": "tensorized-attn tokens/s + per-hop HBM GB/s (% peak) at N=32k, 128k",
        "value": tokens_per_s, "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": describe(w), "rotating_buffer_sets": args.rotate},
        "roofline": roofline,
    }
    if others:
        out["other_workloads"] = others
    if "c3" in step_ms and "c4" in step_ms:
        out["full_attention_same_gpu"] = full_attention_reference(torch, ta, {n_: (WORKLOADS[n_], step_ms[n_]) for n_ in ("c3", "c4")})
    if cpu is not None:
        out["cpu_baseline"] = cpu
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
