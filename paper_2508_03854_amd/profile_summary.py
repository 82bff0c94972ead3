"""Turns the raw output of four rocprofv3 runs of bench.py into the short summaries kept under profiles/:

    <WL>_kernel_stats.md   per-kernel durations (rocprofv3 --kernel-trace --stats) next to the bench line of that run
    <WL>_hbm_traffic.md    FETCH_SIZE / WRITE_SIZE per launch, scaled by what the same counters read for kernels of
                           known traffic (the streaming copy and the gather calibration), and L2 hit rates
    <WL>_traffic.json      bytes per step per timing record + the digest of the library they were measured on;
                           bench.py reports them as `traffic` only while the loaded library has that digest

    python -m paper_2508_03854_amd.profile_summary --workload C4 --src <dir> [--out profiles]

<dir> holds  stats/s_kernel_stats.csv, stats.log (bench's stdout/stderr of that run), and fetch/ write/ cache/ each with
p_counter_collection.csv, written by (run from the repo root, after `cd /tmp && export TMPDIR=/tmp && cd -`):

    rocprofv3 --kernel-trace --stats -d <dir>/stats -o s --output-format csv -- python3 bench.py <ARGS> > <dir>/stats.log
    rocprofv3 --pmc FETCH_SIZE --kernel-include-regex "tbe::" -d <dir>/fetch -o p --output-format csv -- python3 bench.py <ARGS>
    rocprofv3 --pmc WRITE_SIZE --kernel-include-regex "tbe::" -d <dir>/write -o p --output-format csv -- python3 bench.py <ARGS>
    rocprofv3 --pmc TCC_HIT_sum TCC_MISS_sum TCP_TCC_READ_REQ_sum TCP_TOTAL_CACHE_ACCESSES_sum --kernel-include-regex "tbe::" -d <dir>/cache -o p --output-format csv -- python3 bench.py <ARGS>

with <ARGS> = --workload <WL> --steps 5 --warmup 2 --pool 2 --no-cpu-baseline.  If <dir> also holds latency/ and issue/
(two more counter runs of the same command, listed in LATENCY_PASSES), <WL>_latency_counters.md is written too: read
latency past the vector L1, read requests in flight per compute unit, instruction counts per wavefront.
"""
from __future__ import annotations

import argparse
import collections
import csv
import glob
import json
import os

ARGS = "--workload {wl} --steps 5 --warmup 2 --pool 2 --no-cpu-baseline"

LATENCY_PASSES = {
    "latency": "TCP_TCC_READ_REQ_LATENCY_sum TCP_TCC_READ_REQ_sum TCP_PENDING_STALL_CYCLES_sum TCP_TOTAL_CACHE_ACCESSES_sum",
    "issue": "SQ_WAVES SQ_BUSY_CYCLES SQ_WAIT_INST_ANY SQ_INSTS_VMEM_RD SQ_INSTS_VALU SQ_INSTS_SALU GRBM_GUI_ACTIVE",
}
COMPUTE_UNITS = 256
XCDS = 8   # GRBM_GUI_ACTIVE comes back summed over the chip's 8 dies (8 x 2.3e9 per second of kernel time)

# kernel (name without template arguments) -> timing record of tbe_timing_read / bench.py
RECORD = {
    "forward_kernel": "forward_pool", "forward_groups_kernel": "forward_pool", "forward_hot_kernel": "forward_pool",
    "forward_long_bags_kernel": "forward_pool", "linearize_kernel": "linearize", "radix_plan_kernel": "radix_plan",
    "radix_hist_kernel": "radix_hist", "radix_binscan_kernel": "radix_binscan", "radix_scatter_kernel": "radix_scatter",
    "rle_count_kernel": "rle_count", "rle_scan_kernel": "rle_scan", "rle_write_kernel": "rle_write",
    "seg_update_kernel": "seg_update", "seg_update_wide_kernel": "seg_update", "seg_long_scan_kernel": "seg_long_list",
    "seg_long_fill_kernel": "seg_long_list", "hot_select_kernel": "seg_long_list", "seg_dense_select_kernel": "seg_long_list",
    "seg_long_units_kernel": "seg_long_list", "seg_long_bounds_kernel": "seg_long_list",
    "seg_dense_bounds_kernel": "seg_long_list", "seg_dense_partial_kernel": "seg_dense_partial",
    "seg_long_partial_kernel": "seg_long_partial", "seg_long_update_kernel": "seg_long_update",
}


def short(name: str) -> str:
    return name.replace("void ", "").split("(")[0]


def bare(name: str) -> str:
    return short(name).split("::")[-1].split("<")[0]


def find(path_glob: str) -> str:
    hits = sorted(glob.glob(path_glob, recursive=True))
    if not hits:
        raise FileNotFoundError(path_glob)
    return hits[-1]


def load_counters(src: str, sub: str):
    agg = collections.defaultdict(lambda: collections.defaultdict(list))
    for r in csv.DictReader(open(find(os.path.join(src, sub, "**", "p_counter_collection.csv")))):
        agg[short(r["Kernel_Name"])][r["Counter_Name"]].append(float(r["Counter_Value"]))
    return agg


def mean(xs):
    return sum(xs) / len(xs)


def main() -> None:
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", required=True)
    ap.add_argument("--src", required=True)
    ap.add_argument("--out", default="profiles")
    a = ap.parse_args()
    wl, src = a.workload, a.src
    args = ARGS.format(wl=wl)
    bench = json.loads([ln for ln in open(os.path.join(src, "stats.log")) if ln.startswith("{")][-1])
    steps_run = bench["steps"] + bench["warmup"] + bench["profiled_steps"]

    # ---- kernel stats
    rows = list(csv.DictReader(open(find(os.path.join(src, "stats", "**", "s_kernel_stats.csv")))))
    tbe = [r for r in rows if "tbe::" in r["Name"]]
    tot = sum(float(r["TotalDurationNs"]) for r in tbe)
    with open(os.path.join(a.out, f"{wl}_kernel_stats.md"), "w") as f:
        f.write(f"# rocprofv3 kernel stats, workload {wl}\n\nLibrary: `{bench['build']}`\n\n")
        f.write("Command (from the repo root on the MI355X box, after `cd /tmp && export TMPDIR=/tmp && cd -`):\n\n")
        f.write(f"    rocprofv3 --kernel-trace --stats -d out -o s --output-format csv -- python3 bench.py {args}\n\n")
        f.write(f"Kernels of libtbe355 only (the input generator's torch kernels are omitted); {steps_run} steps in all "
                f"({bench['warmup']} warm-up, {bench['steps']} timed, {bench['profiled_steps']} with per-kernel events) "
                "plus the calibration kernels.\n\n")
        f.write("| kernel | calls | avg us | total ms | % of tbe time |\n|---|---:|---:|---:|---:|\n")
        for r in sorted(tbe, key=lambda r: -float(r["TotalDurationNs"])):
            f.write(f"| `{short(r['Name'])}` | {r['Calls']} | {float(r['AverageNs']) / 1e3:.1f} | "
                    f"{float(r['TotalDurationNs']) / 1e6:.2f} | {100 * float(r['TotalDurationNs']) / tot:.1f} |\n")
        f.write("\nThe same run's bench line (HIP-event timings on the launch stream, per step):\n\n")
        f.write("| timing record | launches/step | avg ms (HIP events) | ms/step |\n|---|---:|---:|---:|\n")
        for k, v in sorted(bench["kernels"].items(), key=lambda kv: -kv[1]["ms_per_step"]):
            f.write(f"| {k} | {v['launches_per_step']:.0f} | {v['avg_ms']:.3f} | {v['ms_per_step']:.3f} |\n")
        f.write(f"\nbench value under the profiler: {bench['value']:.4g} lookups/s, {bench['ms_per_step']:.2f} ms/step; "
                f"dominant kernel {bench['roofline']['kernel']} avg {bench['roofline']['avg_launch_ms']:.3f} ms.\n")

    # ---- byte counters
    fetch, write, cache = load_counters(src, "fetch"), load_counters(src, "write"), load_counters(src, "cache")
    cf = [k for k in fetch if "calibration_copy" in k][0]
    copy_bytes = 2 * 1024 ** 3
    f_scale = copy_bytes / (mean(fetch[cf]["FETCH_SIZE"]) * 1024)
    w_scale = copy_bytes / (mean(write[cf]["WRITE_SIZE"]) * 1024)
    with open(os.path.join(a.out, f"{wl}_hbm_traffic.md"), "w") as f:
        f.write(f"# rocprofv3 --pmc byte counters, workload {wl}\n\nLibrary: `{bench['build']}`\n\n")
        f.write("Commands (one counter set per run; kernels filtered to the library's):\n\n")
        for c in ("FETCH_SIZE", "WRITE_SIZE", "TCC_HIT_sum TCC_MISS_sum TCP_TCC_READ_REQ_sum TCP_TOTAL_CACHE_ACCESSES_sum"):
            f.write(f"    rocprofv3 --pmc {c} --kernel-include-regex \"tbe::\" -d out -o p --output-format csv -- python3 bench.py {args}\n")
        f.write(f"\nScale factors from the streaming copy of 2 GiB (reads 2 GiB, writes 2 GiB): FETCH_SIZE reads "
                f"{mean(fetch[cf]['FETCH_SIZE']) / 1024 ** 2:.3f} GiB for it -> x{f_scale:.3f}; WRITE_SIZE reads "
                f"{mean(write[cf]['WRITE_SIZE']) / 1024 ** 2:.3f} GiB -> x{w_scale:.3f}.\n\n")
        # the gather calibration: known bytes by construction (bench prints slices x slice_bytes per case)
        g = bench.get("measured_gather") or {}
        lpr_case = {64: "hbm_1KiB", 32: None, 16: "l2_resident_256B", 8: "hbm_128B"}
        f.write("The same factors checked on gathers (bytes known by construction; launches of one kernel name averaged):\n\n")
        f.write("| calibration kernel | case | bytes gathered per launch | FETCH_SIZE x factor | ratio |\n|---|---|---:|---:|---:|\n")
        for k in sorted(fetch):
            if "calibration_gather" not in k:
                continue
            targ = k.split("<")[1].split(">")[0].replace(" ", "").split(",")
            lpr, rmw = int(targ[0]), targ[1] == "true"
            rmw_case = {32: "hbm_rmw_512B", 4: "hbm_rmw_64B", 2: "hbm_rmw_32B"}
            case = rmw_case.get(lpr) if rmw else ("infinity_cache_512B" if lpr == 32 else lpr_case.get(lpr))
            if not case or case not in g:
                continue
            known = g[case]["slices"] * g[case]["slice_bytes"]
            seen = mean(fetch[k]["FETCH_SIZE"]) * 1024 * f_scale
            f.write(f"| `{k}` | {case} | {known / 1e9:.2f} GB | {seen / 1e9:.2f} GB | {seen / known:.2f} |\n")
        f.write("\n(An L2-resident window reads next to nothing past the L2; windows beyond the caches should read ~1.0; slices "
                "of less than 128 bytes read more than they use - the L2 fetches whole 128-byte lines: 2.0 at 64 bytes, 4.0 "
                "at 32.)\n\n")
        f.write("Per launch, scaled (GB = 1e9 bytes). FETCH_SIZE counts what the L2 asks of the fabric, whether the "
                "Infinity Cache or HBM serves it. L2 hit = TCC_HIT / (TCC_HIT + TCC_MISS).\n\n")
        f.write("| kernel | launches seen | read GB | written GB | L2 hit % | L1->L2 read requests |\n|---|---:|---:|---:|---:|---:|\n")
        per_record = collections.defaultdict(float)
        for k in sorted(fetch, key=lambda k: -mean(fetch[k]["FETCH_SIZE"])):
            rd = mean(fetch[k]["FETCH_SIZE"]) * 1024 * f_scale
            wr = mean(write[k]["WRITE_SIZE"]) * 1024 * w_scale if k in write else 0.0
            h = mean(cache[k]["TCC_HIT_sum"]) if k in cache else 0.0
            m = mean(cache[k]["TCC_MISS_sum"]) if k in cache else 0.0
            rq = mean(cache[k]["TCP_TCC_READ_REQ_sum"]) if k in cache else 0.0
            n = len(fetch[k]["FETCH_SIZE"])
            f.write(f"| `{k}` | {n} | {rd / 1e9:.2f} | {wr / 1e9:.2f} | {100 * h / max(1.0, h + m):.0f} | {rq:.3g} |\n")
            rec = RECORD.get(bare(k))
            if rec:
                per_record[rec] += (rd + wr) * n / steps_run
        f.write("\nPer step and timing record (launches x bytes, summed over the kernels of a record):\n\n")
        f.write("| timing record | GB per step |\n|---|---:|\n")
        for rec, v in sorted(per_record.items(), key=lambda kv: -kv[1]):
            f.write(f"| {rec} | {v / 1e9:.2f} |\n")
        f.write(f"| all | {sum(per_record.values()) / 1e9:.2f} |\n")
    with open(os.path.join(a.out, f"{wl}_traffic.json"), "w") as f:
        json.dump({"workload": wl, "build": bench["build"], "command_args": args, "fetch_scale": f_scale,
                   "write_scale": w_scale, "bytes_per_step": {k: round(v) for k, v in sorted(per_record.items())}}, f, indent=1)
        f.write("\n")
    print(open(os.path.join(a.out, f"{wl}_hbm_traffic.md")).read())

    # ---- latency and issue counters (optional passes)
    if not all(os.path.isdir(os.path.join(src, sub)) for sub in LATENCY_PASSES):
        return
    lat, iss = load_counters(src, "latency"), load_counters(src, "issue")
    avg_us = {short(r["Name"]): float(r["AverageNs"]) / 1e3 for r in tbe}
    with open(os.path.join(a.out, f"{wl}_latency_counters.md"), "w") as f:
        f.write(f"# rocprofv3 --pmc latency and issue counters, workload {wl}\n\nLibrary: `{bench['build']}`\n\n")
        f.write("Commands (one counter set per run):\n\n")
        for c in LATENCY_PASSES.values():
            f.write(f"    rocprofv3 --pmc {c} --kernel-include-regex \"tbe::\" -d out -o p --output-format csv -- python3 bench.py {args}\n")
        f.write("\nPer launch (mean over the launches seen). `latency` = TCP_TCC_READ_REQ_LATENCY / TCP_TCC_READ_REQ: clock "
                "cycles per read request that left a vector L1. `cycles` = GRBM_GUI_ACTIVE / 8 (the counter is summed over the "
                f"8 dies). `requests / cycle / CU` = read requests / (cycles x {COMPUTE_UNITS}); x 128 bytes x 256 CUs x the "
                "clock it is the request bandwidth the kernel drew past the L1s. `in flight per CU` = that rate x latency "
                "(Little's law): the mean number of read requests one compute unit had outstanding. The calibration gathers "
                "(random slices of known size; <16>: window in L2, <32, false>: in the Infinity Cache, <64> and <8>: HBM, "
                "<32, true>: HBM, read-modify-write) show what the memory system gives each level: deeper queues buy "
                "latency, not rate. `avg us` is the kernel-trace duration of the stats run.\n\n")
        f.write("| kernel | avg us | wavefronts | VALU insts / wave | SALU insts / wave | VMEM reads / wave | L1->L2 read requests | "
                "latency (cycles) | requests / cycle / CU | in flight per CU | L1 pending-stall cycles / cycle |\n"
                "|---|---:|---:|---:|---:|---:|---:|---:|---:|---:|---:|\n")
        for k in sorted(lat, key=lambda k: -avg_us.get(k, 0.0)):
            if k not in iss:
                continue
            rq = mean(lat[k]["TCP_TCC_READ_REQ_sum"])
            lc = mean(lat[k]["TCP_TCC_READ_REQ_LATENCY_sum"]) / max(1.0, rq)
            waves = max(1.0, mean(iss[k]["SQ_WAVES"]))
            active = max(1.0, mean(iss[k]["GRBM_GUI_ACTIVE"]) / XCDS)
            stall = mean(lat[k]["TCP_PENDING_STALL_CYCLES_sum"]) / (active * COMPUTE_UNITS)
            f.write(f"| `{k}` | {avg_us.get(k, 0.0):.1f} | {waves:.3g} | {mean(iss[k]['SQ_INSTS_VALU']) / waves:.0f} | "
                    f"{mean(iss[k]['SQ_INSTS_SALU']) / waves:.0f} | {mean(iss[k]['SQ_INSTS_VMEM_RD']) / waves:.1f} | {rq:.3g} | "
                    f"{lc:.0f} | {rq / (active * COMPUTE_UNITS):.4f} | {rq * lc / (active * COMPUTE_UNITS):.1f} | {stall:.2f} |\n")


if __name__ == "__main__":
    main()
