"""Turns rocprofv3 output of `bench.py` runs into the figures the benchmark and the profile
summaries quote: per-kernel launch times, HBM bytes per launch and compute-unit counters.

Usage (after the rocprofv3 commands printed by `--commands`, run from the repository root):
    python -m paper_2410_20926_amd.counters WORKLOAD RAW_DIR [--out-dir profiles]
reads   RAW_DIR/prof_W/W_kernel_stats.csv               kernel trace with --stats
        RAW_DIR/prof_W_bench.json                       bench.py's JSON line of that run
        RAW_DIR/pmc_W_FETCH_SIZE/W_counter_collection.csv, RAW_DIR/pmc_W_WRITE_SIZE/...
        RAW_DIR/sq_W_1/..., RAW_DIR/sq_W_2/...          (optional) compute-unit counters
writes  OUT/tensattn_W.txt   the summary text
        OUT/traffic_W.json   {plan kernel name: {fetch_bytes_per_launch, write_bytes_per_launch}}

HBM traffic arithmetic.  rocprofv3 --pmc reports FETCH_SIZE and WRITE_SIZE per dispatch in KiB:
    bytes(dispatch) = Counter_Value * 1024 * scale,
where `scale` calibrates the counter on this machine: the same run launches the library's plain
copy kernel on 1 GiB (bench.py --copy-calibration), which reads 2^30 bytes and writes 2^30 bytes,
so scale = 2^30 / (mean over the copy launches of Counter_Value * 1024), separately for the two
counters (FETCH_SIZE has read 0.5 of the true bytes on MI355X, i.e. scale 2.000, and WRITE_SIZE
1.000).  A kernel's figure is the mean of bytes(dispatch) over all its dispatches in the run."""
from __future__ import annotations

import argparse
import collections
import csv
import json
import os
import re

PMC_SETS = ["SQ_VALU_MFMA_BUSY_CYCLES SQ_BUSY_CYCLES SQ_WAVE_CYCLES SQ_INSTS_VALU SQ_INSTS_MFMA SQ_INSTS_LDS SQ_WAIT_INST_ANY SQ_ACTIVE_INST_ANY",
            "SQ_LDS_BANK_CONFLICT SQ_LDS_IDX_ACTIVE SQ_INSTS_VMEM_RD SQ_INSTS_VMEM_WR SQ_WAVES SQ_INST_CYCLES_VMEM_RD GRBM_GUI_ACTIVE"]


def commands(wl: str, raw: str):
    bench = f"python3 bench.py --workload {wl} --no-cpu-baseline --also \"\""
    out = [f"rocprofv3 --kernel-trace --stats --output-format csv -d {raw}/prof_{wl} -o {wl} -- {bench} > {raw}/prof_{wl}_bench.json"]
    for c in ("FETCH_SIZE", "WRITE_SIZE"):
        out.append(f"rocprofv3 --pmc {c} --kernel-trace --output-format csv -d {raw}/pmc_{wl}_{c} -o {wl} -- {bench} --steps 3 --warmup 1 --copy-calibration")
    for i, cs in enumerate(PMC_SETS, 1):
        out.append(f"rocprofv3 --pmc {cs} --kernel-trace --output-format csv -d {raw}/sq_{wl}_{i} -o {wl} -- {bench} --steps 2 --warmup 1")
    return out


def short(name: str):
    """`mfma_fwd_pair_kernel<128, false, false>` from a demangled kernel symbol of the library; None for other kernels."""
    if not name.startswith("void ta::") and not name.startswith("ta::"):
        return None
    m = re.search(r"(\w+_kernel(<[^>(]*>)?)\(", name)
    return m.group(1) if m else None


def plan_name(k: str) -> str:
    """The plan's name (ta_plan_hop_kernel and friends) of a kernel instantiation."""
    base = k.split("<")[0]
    args = [x.strip() for x in k[k.index("<") + 1:k.rindex(">")].split(",")] if "<" in k else []
    if base == "mfma_fwd_pair_kernel": return "mfma_bf16_pair_n32"
    if base == "mfma_bwd_kernel": return "mfma_bf16_bwd_n32"
    if base == "mfma_bwd2_kernel": return "mfma_bf16_bwd_n64"
    if base == "mfma_bwd_stream_kernel": return "mfma_bf16_bwd_blocked"
    if base == "mfma_fwd_kernel": return "mfma_bf16_n32" if args[1] == "1" else "mfma_bf16_n64"
    if base == "mfma_fwd_shared_kernel": return ("mfma_bf16_n32" if args[1] == "1" else "mfma_bf16_n64") + "_shared" + ("_kv" if args[2] == "true" else "")
    if base == "mfma_fwd_stream_kernel": return "mfma_bf16_stream"
    if base in ("mfma_fwd_stream_shared_kernel", "mfma_fwd_stream_chunked_kernel"): return "mfma_bf16_stream_shared" + ("_kv" if args[1] == "true" else "")
    return k


def counter_rows(path: str):
    per = collections.defaultdict(lambda: collections.defaultdict(list))
    for r in csv.DictReader(open(path)):
        k = short(r["Kernel_Name"])
        if k:
            per[k][r["Counter_Name"]].append(float(r["Counter_Value"]))
    return per


def summarise(wl: str, raw: str, out_dir: str) -> str:
    out = [f"rocprofv3 summaries for workload {wl} on one MI355X (commands run from the repository root with TMPDIR=/tmp; "
           f"this text and traffic_{wl}.json were written by `python -m paper_2410_20926_amd.counters {wl} {raw}`)\n"]
    cmds = commands(wl, raw)
    stats = list(csv.DictReader(open(f"{raw}/prof_{wl}/{wl}_kernel_stats.csv")))
    bench = json.load(open(f"{raw}/prof_{wl}_bench.json"))
    out.append("== kernel trace ==")
    out.append("command: " + cmds[0])
    out.append(f"{'kernel':44s} {'calls':>6s} {'avg_us':>10s} {'min_us':>10s} {'max_us':>10s} {'pct':>6s}")
    for r in stats:
        k = short(r["Name"])
        if k:
            out.append(f"{k:44s} {r['Calls']:>6s} {float(r['AverageNs']) / 1e3:10.2f} {float(r['MinNs']) / 1e3:10.2f} {float(r['MaxNs']) / 1e3:10.2f} {r['Percentage']:>6s}")
    rf = bench["roofline"]
    out.append(f"bench.py of the same run: {bench['value'] / 1e6:.2f} M tokens/s, {bench['ms_per_step']:.3f} ms/step; roofline kernel {rf['kernel']}: "
               f"HIP-event average {rf['avg_launch_us']} us per launch over {rf['launches_timed']} launches, {rf['achieved']} GB/s algorithmic = {rf['frac'] * 100:.1f}% of 8 TB/s")
    for h in rf["per_hop"]:
        out.append(f"    {h['pass']} hop {h['hop']} axis {h['axis']} n={h['n']:3d} {h['kernel']:26s} {h['us']:9.2f} us  {h['algorithmic_bytes'] / 1e6:8.1f} MB  {h['GBps']:7.1f} GB/s  {h['frac_of_8TBps'] * 100:5.1f}%")
    out.append("(the trace average includes warm-up steps and both the whole-step and per-hop timing loops)\n")

    out.append("== HBM traffic counters (KiB per dispatch, scaled by the copy kernel of the same run; see the module's docstring) ==")
    traffic = {}
    for idx, c in enumerate(("FETCH_SIZE", "WRITE_SIZE")):
        out.append("command: " + cmds[1 + idx])
        per = counter_rows(f"{raw}/pmc_{wl}_{c}/{wl}_counter_collection.csv")
        copy = [x * 1024 for x in per["copy_kernel"][c]]
        scale = (1 << 30) / (sum(copy) / len(copy))
        out.append(f"  copy_kernel on 1 GiB: {sum(copy) / len(copy) / 1e6:.1f} MB on this counter -> scale {scale:.3f}")
        for k, d in per.items():
            if k == "copy_kernel" or k.startswith("stream_mix_kernel") or k.startswith("stream_slab"):      # the measurement aids
                continue
            v = [x * 1024 * scale for x in d[c]]
            uniq = []
            for x in v:
                if not any(abs(x - u) < 0.002 * u for u in uniq):
                    uniq.append(x)
            out.append(f"  {k}: {len(v)} launches, scaled MB per launch (distinct values): " + ", ".join(f"{u / 1e6:.1f}" for u in uniq))
            traffic.setdefault(k, {})[c] = sum(v) / len(v)

    if os.path.exists(f"{raw}/sq_{wl}_1/{wl}_counter_collection.csv"):
        out.append("\n== compute-unit counters (per launch, averaged over the launches of each kernel) ==")
        vals = collections.defaultdict(dict)
        for i in (1, 2):
            out.append("command: " + cmds[2 + i])
            for k, d in counter_rows(f"{raw}/sq_{wl}_{i}/{wl}_counter_collection.csv").items():
                if k != "copy_kernel" and not k.startswith("stream_mix_kernel") and not k.startswith("stream_slab"):
                    for c, v in d.items():
                        vals[k][c] = sum(v) / len(v)
        for k, v in vals.items():
            waves = v["SQ_WAVES"]
            gui = v["GRBM_GUI_ACTIVE"] / 8.0              # the counter sums the 8 XCDs
            out.append(f"  {k}: waves {waves:.0f}; per wave: {v['SQ_INSTS_VALU'] / waves:.0f} VALU (incl. {v['SQ_INSTS_MFMA'] / waves:.0f} MFMA), {v['SQ_INSTS_LDS'] / waves:.0f} LDS, "
                       f"{v['SQ_INSTS_VMEM_RD'] / waves:.1f} global loads, {v['SQ_INSTS_VMEM_WR'] / waves:.1f} global stores")
            out.append(f"      MFMA utilisation = SQ_VALU_MFMA_BUSY_CYCLES / (GRBM_GUI_ACTIVE/8 * 1024 SIMDs) = {100 * v['SQ_VALU_MFMA_BUSY_CYCLES'] / (gui * 1024):.1f} %")
            out.append(f"      LDS: {v['SQ_LDS_IDX_ACTIVE'] / 256 / gui * 100:.0f} % of cycles active per CU, {100 * v['SQ_LDS_BANK_CONFLICT'] / v['SQ_LDS_IDX_ACTIVE']:.0f} % of those are bank-conflict cycles")
            out.append(f"      waves waiting on an instruction (SQ_WAIT_INST_ANY / SQ_WAVE_CYCLES) = {100 * v['SQ_WAIT_INST_ANY'] / v['SQ_WAVE_CYCLES']:.0f} %")
    out.append("")
    algo = sorted(set(round(h["algorithmic_bytes"] / 1e6, 1) for h in rf["per_hop"]))
    out.append("algorithmic MB per launch (reads + writes) for comparison: " + ", ".join(map(str, algo)))
    for k, t in traffic.items():
        out.append(f"  {k}: average measured HBM traffic per launch = {(t['FETCH_SIZE'] + t['WRITE_SIZE']) / 1e6:.1f} MB (fetch {t['FETCH_SIZE'] / 1e6:.1f} + write {t['WRITE_SIZE'] / 1e6:.1f})")
    text = "\n".join(out) + "\n"
    os.makedirs(out_dir, exist_ok=True)
    open(os.path.join(out_dir, f"tensattn_{wl}.txt"), "w").write(text)
    json.dump({plan_name(k): {"fetch_bytes_per_launch": t["FETCH_SIZE"], "write_bytes_per_launch": t["WRITE_SIZE"]} for k, t in traffic.items()},
              open(os.path.join(out_dir, f"traffic_{wl}.json"), "w"), indent=1)
    return text


def main():
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("workload")
    ap.add_argument("raw_dir")
    ap.add_argument("--out-dir", default="profiles")
    ap.add_argument("--commands", action="store_true", help="print the rocprofv3 commands whose output this tool reads, and stop")
    a = ap.parse_args()
    if a.commands:
        print("\n".join(commands(a.workload, a.raw_dir)))
        return
    print(summarise(a.workload, a.raw_dir, a.out_dir))


if __name__ == "__main__":
    main()
