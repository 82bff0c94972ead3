#!/usr/bin/env python3
"""Benchmark of the fused table-batched embedding step on one MI355X.

One "step" = tbe_forward + tbe_backward_rowwise_adagrad over one synthetic batch, all inputs resident in
HBM before the timed region.  Prints ONE JSON line: whole-job lookups/s, the roofline record of the
dominant kernel (duration measured live with HIP events on the launch stream) and the CPU oracle timed on
a bounded sample of the same workload.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload C2|C1|C3|C4|C5|C5I]
"""
from __future__ import annotations

import argparse
import math
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0  # MI355X published HBM3E peak

def measured_traffic(workload: str, build: str):
    """Bytes per step that the byte counters saw, per timing record, from the tracked summary that
    paper_2508_03854_amd/profile_summary.py wrote for this workload - or None when there is none, or when it was
    measured on a library built from other sources than the one loaded now (the digest in tbe_build_info())."""
    path = os.path.join(ROOT, "profiles", f"{workload}_traffic.json")
    try:
        rec = json.load(open(path))
    except (OSError, ValueError):
        return None
    if rec.get("build") != build:
        return None
    return {k: float(v) for k, v in rec.get("bytes_per_step", {}).items()}


def profiler_region(resume: bool) -> None:
    """Under `rocprofv3 --selected-regions` only the code between resume and pause is profiled; the input
    generation (tens of thousands of torch kernels) stays outside.  A no-op when the library is absent."""
    import ctypes
    try:
        lib = ctypes.CDLL("librocprofiler-sdk-roctx.so")
        (lib.roctxProfilerResume if resume else lib.roctxProfilerPause)(ctypes.c_uint64(0))
    except OSError:
        pass


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def realised_unique(cfg, batches, torch):
    """Per batch: (U_t per table) - statistics of the inputs, needed for the algorithmic byte counts."""
    out = []
    for idx, off in batches:
        bounds = off[:: cfg.B].tolist()
        out.append([int(torch.unique(idx[bounds[t]:bounds[t + 1]]).numel()) for t in range(cfg.T)])
    return out


def algorithmic_bytes(cfg, nnz, U_t, ib=8, eb=4):
    """Compulsory bytes of each kernel for one batch: every distinct row once, every index once, the pooled
    output / upstream gradient once, row and moment read-modify-write once per unique row."""
    wb = 4 if cfg.weight_dtype == "f32" else 2
    nb = cfg.T * cfg.B + 1
    rows_bytes = sum(u * d * wb for u, d in zip(U_t, cfg.D))
    U = sum(U_t)
    dense = cfg.B * cfg.sum_D * eb      # eb bytes per element of out / grad_out, ib bytes per id and offset
    return {
        "forward_pool": rows_bytes + nnz * ib + nb * ib + dense,
        "linearize": nnz * ib + nb * ib + nnz * 8,                 # ids + offsets in; key and bag id out
        "radix_hist": nnz * 4,
        "radix_plan": 0,
        "radix_scatter": nnz * 16,                                  # (key, bag id) in and out
        "radix_binscan": 0,
        "rle_count": nnz * 4,
        "rle_scan": 0,
        "rle_write": nnz * 4 + U * 8,
        "seg_dense_partial": dense,                                 # streams the gradient block of every table once
        "seg_long_list": U * 8,
        # gradient once, sorted positions and their bags, row + moment read-modify-write per unique row
        "seg_update": dense + nnz * 8 + U * 8 + 2 * rows_bytes + 8 * U,
        "seg_long_partial": dense,                                  # the hot rows touch (nearly) every bag once more
        "seg_long_update": 0,
    }


def side_mode(args, torch, W, TBE, build):
    """The widened entry points, timed the same way (HIP events per kernel on the launch stream, wall clock over the
    timed steps): one record, not the headline metric."""
    dev = "cuda"
    base = {"n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "higher_is_better": True, "scaling": "weak",
            "vs_baseline": None, "data": "synthetic", "build": build}
    if args.mode == "sync":
        # weight sync / moment sync of Algorithm 1 for M replicas held on this device, 1 GiB per replica
        tbe = TBE([16], [8], "f32")
        out = {}
        for name, dt, eb in (("f32", torch.float32, 4), ("f16", torch.float16, 2)):
            for M in (2, 4, 8):
                reps = [torch.empty((1 << 30) // eb, dtype=dt, device=dev).normal_() for _ in range(M)]
                tbe.timing_enable(True)
                for _ in range(args.warmup + args.steps):
                    tbe.replica_mean(reps)
                ms = [m for n, m in tbe.timing_read() if n == "replica_mean"][args.warmup:]
                t = sum(ms) / len(ms)
                out[f"{name}_M{M}"] = {"ms": t, "read_plus_write_GBps": 2 * M * (1 << 30) / (t * 1e-3) / 1e9}
                del reps
        best = max(v["read_plus_write_GBps"] for v in out.values())
        return dict(base, metric="GB/s read+written, replica mean (Algorithm 1 weight / moment sync) on one device",
                    value=best, unit="GB/s", ms_per_step=None, dtype="f32",
                    config={"workload": "M replicas of 1 GiB each, M in {2, 4, 8}"}, cases=out)
    # ---- the non-pooled lookup and its backward
    cfg = W.config(args.workload, rows_scale=args.rows_scale)
    io_t = {"f32": torch.float32, "f16": torch.float16, "bf16": torch.bfloat16}[args.io]
    flat = torch.empty(cfg.total_elems, dtype=cfg.torch_weight_dtype, device=dev)
    W.fill_weights(cfg, flat)
    state = torch.zeros(cfg.total_rows, dtype=torch.float32, device=dev)
    (idx, off), = W.make_batches(cfg, [0], device=dev)
    idx, toff, total = W.as_sequence(cfg, idx, off)
    if args.index_dtype == "i32":
        idx, toff = idx.to(torch.int32), toff.to(torch.int32)
    g = W.make_grad_seq(cfg, total, 0, device=dev).to(io_t)
    out = torch.empty(total, dtype=io_t, device=dev)
    tbe = TBE(cfg.rows, cfg.D, cfg.weight_dtype)
    ws = tbe.alloc_workspace(1, idx.numel())

    def step():
        tbe.lookup_seq(flat, idx, toff, out)
        tbe.backward_seq_rowwise_adagrad(g, idx, toff, flat, state, ws, lr=cfg.lr, eps=cfg.eps, momentum_scale=cfg.c)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    acc = {}
    reps = max(2, min(args.steps, 4))
    for _ in range(reps):
        tbe.timing_enable(True)
        step()
        for n, ms in tbe.timing_read():
            acc[n] = acc.get(n, 0.0) + ms / reps
    assert not tbe.poll_index_error()
    nnz = int(idx.numel())
    lookup_bytes = total * (flat.element_size() + out.element_size()) + nnz * idx.element_size()
    return dict(base, metric="lookups/sec, non-pooled lookup + its backward with row-wise AdaGrad", unit="lookups/s",
                value=nnz * args.steps / elapsed, ms_per_step=1e3 * elapsed / max(1, args.steps), dtype="f32",
                config={"workload": W.describe(cfg) + " (ids read as one sequence per table)", "index_dtype": args.index_dtype,
                        "io_dtype": args.io, "lookups_per_step": nnz, "out_bytes": total * out.element_size()},
                kernels_ms_per_step=acc,
                lookup_seq={"ms": acc.get("lookup_seq"), "read_plus_write_GBps": lookup_bytes / (acc["lookup_seq"] * 1e-3) / 1e9},
                backward_ms=sum(v for n, v in acc.items() if n != "lookup_seq"))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="C4")
    ap.add_argument("--pool", type=int, default=4, help="pre-generated batches rotated through")
    ap.add_argument("--cpu-seconds", type=float, default=10.0, help="target CPU time of the oracle baseline")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-threads", type=int, default=16, help="threads of the all-cores oracle baseline (at most the host's cores)")
    ap.add_argument("--rows-scale", type=float, default=1.0,
                    help="shrink every table's row count (profiling aid only; the result is then NOT the named workload)")
    ap.add_argument("--index-dtype", choices=["i64", "i32"], default="i64", help="ids and offsets (i32: *_ex calls)")
    ap.add_argument("--io", choices=["f32", "f16", "bf16"], default="f32",
                    help="element type of out and grad_out (16-bit: *_ex calls)")
    ap.add_argument("--optimizer", choices=["rowwise_adagrad", "sgd"], default="rowwise_adagrad")
    ap.add_argument("--momentum-scale", type=float, default=None, help="override the workload's scaling factor c")
    ap.add_argument("--graph", action="store_true",
                    help="replay one captured HIP graph per pooled batch instead of launching every kernel (small, "
                         "launch-bound workloads)")
    ap.add_argument("--copy-mib", type=int, default=2048, help="size of the streaming-copy calibration (0 = skip)")
    ap.add_argument("--gather-gib", type=int, default=16, help="buffer of the gather calibration in GiB (0 = skip)")
    ap.add_argument("--sort-stream", action="store_true",
                    help="the backward in two calls, its gradient-free half (sort / dedup) on a second stream next to "
                         "the forward of the same batch")
    ap.add_argument("--mode", choices=["step", "seq", "sync"], default="step",
                    help="step: the pooled forward + backward (the metric); seq: the non-pooled lookup and its backward "
                         "on the workload's ids read as sequences; sync: the replica mean of Algorithm 1 on one device")
    ap.add_argument("--hot-rows-min-workgroups", type=int, default=None,
                    help="tunable of the forward's on-chip hot-row path (negative: off; default: the library's)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures ONE GPU: this path has no collectives (the cross-replica weight/moment averaging and "
              "the all-to-all of the paper sit outside it). Run with --gpus 1.", file=sys.stderr)
        sys.exit(2)

    import torch
    import workloads as W
    from paper_2508_03854_amd import TBE
    from paper_2508_03854_amd.binding import build_info

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    dev = "cuda"
    if args.mode != "step":
        print(json.dumps(side_mode(args, torch, W, TBE, build_info())))
        return
    cfg = W.config(args.workload, rows_scale=args.rows_scale,
                   **({} if args.momentum_scale is None else {"c": args.momentum_scale}))
    log("workload:", W.describe(cfg), "" if args.rows_scale == 1.0 else f"[rows scaled by {args.rows_scale}]")

    # ---- inputs, generated directly in HBM
    t0 = time.time()
    flat = torch.empty(cfg.total_elems, dtype=cfg.torch_weight_dtype, device=dev)
    log("allocated tables")
    W.fill_weights(cfg, flat)
    log("tables filled")
    state = torch.zeros(cfg.total_rows, dtype=torch.float32, device=dev)
    pool = max(1, args.pool)
    batches = W.make_batches(cfg, list(range(pool)), device=dev)
    extended = args.index_dtype != "i64" or args.io != "f32"
    # the committed counter profiles cover the default call variant of the full-size workload only, and only the
    # library build they were measured on
    default_call = not extended and args.rows_scale == 1.0 and args.optimizer == "rowwise_adagrad" and \
        args.hot_rows_min_workgroups is None and not args.sort_stream
    traffic = measured_traffic(cfg.name, build_info()) if default_call else None
    io_t = {"f32": torch.float32, "f16": torch.float16, "bf16": torch.bfloat16}[args.io]
    if args.index_dtype == "i32":
        batches = [(i.to(torch.int32), o.to(torch.int32)) for i, o in batches]
    log("batches drawn")
    n_go = pool if cfg.B * cfg.sum_D * 4 * pool < 16e9 else 2
    gouts = [W.make_grad_out(cfg, k, device=dev).to(io_t) for k in range(n_go)]
    out = torch.empty(cfg.B, cfg.sum_D, dtype=io_t, device=dev)
    max_nnz = max(int(i.numel()) for i, _ in batches)
    tbe = TBE(cfg.rows, cfg.D, cfg.weight_dtype)
    if args.hot_rows_min_workgroups is not None:
        tbe.set_tunable("hot_rows_min_workgroups", args.hot_rows_min_workgroups)
    ws = tbe.alloc_workspace(cfg.B, max_nnz)
    torch.cuda.synchronize()
    log(f"inputs ready in {time.time() - t0:.1f}s; nnz/batch ~ {max_nnz}; workspace {ws.numel() / 1e6:.1f} MB")

    side = torch.cuda.Stream() if args.sort_stream else None

    def step(k):
        idx, off = batches[k % pool]
        if side is not None:   # (row-wise AdaGrad, any element types)
            main_stream = torch.cuda.current_stream()
            side.wait_stream(main_stream)
            tbe.backward_prepare(idx, off, cfg.B, ws, stream=side)
            tbe.forward_ex(flat, idx, off, cfg.B, cfg.pooling, out=out)
            main_stream.wait_stream(side)
            tbe.backward_apply_rowwise_adagrad(gouts[k % n_go], off, cfg.B, int(idx.numel()), flat, state, ws,
                                               pooling=cfg.pooling, lr=cfg.lr, eps=cfg.eps, momentum_scale=cfg.c)
            return
        if args.optimizer == "sgd":
            tbe.forward_ex(flat, idx, off, cfg.B, cfg.pooling, out=out)
            tbe.backward_sgd(gouts[k % n_go], idx, off, cfg.B, flat, ws, pooling=cfg.pooling, lr=cfg.lr)
            return
        if extended:
            tbe.forward_ex(flat, idx, off, cfg.B, cfg.pooling, out=out)
            tbe.backward_rowwise_adagrad_ex(gouts[k % n_go], idx, off, cfg.B, flat, state, ws, pooling=cfg.pooling,
                                            lr=cfg.lr, eps=cfg.eps, momentum_scale=cfg.c)
            return
        tbe.forward(flat, idx, off, cfg.B, cfg.pooling, out=out)
        tbe.backward_rowwise_adagrad(gouts[k % n_go], idx, off, cfg.B, flat, state, ws, pooling=cfg.pooling, lr=cfg.lr,
                                     eps=cfg.eps, momentum_scale=cfg.c)

    profiler_region(True)
    # ---- warm-up (also makes the moments non-zero), then the timed region
    for k in range(args.warmup):
        step(k)
    torch.cuda.synchronize()
    assert not tbe.poll_index_error()
    run = step
    if args.graph:
        # one graph per distinct (batch, grad_out) pair; the calls record kernels only (no memset, no allocation)
        assert not args.sort_stream, "--graph and --sort-stream are separate experiments"
        capture_stream = torch.cuda.Stream()
        period = pool * n_go // math.gcd(pool, n_go)
        graphs = []
        for k in range(period):
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g, stream=capture_stream):
                step(k)
            graphs.append(g)
        torch.cuda.synchronize()

        def run(k):
            graphs[k % period].replay()
    t0 = time.perf_counter()
    for k in range(args.steps):
        run(args.warmup + k)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    lookups = sum(int(batches[(args.warmup + k) % pool][0].numel()) for k in range(args.steps))
    value = lookups / elapsed
    ms_per_step = 1e3 * elapsed / max(1, args.steps)

    # ---- per-kernel durations with HIP events on the launch stream (separate loop: events add launch gaps)
    prof_steps = max(2, min(args.steps, 2 * pool))
    per_kernel = {}
    for k in range(prof_steps):
        tbe.timing_enable(True)
        step(args.warmup + args.steps + k)
        for name, ms in tbe.timing_read():
            d = per_kernel.setdefault(name, {"launches": 0, "ms": 0.0, "all": []})
            d["all"].append(ms)
            d["launches"] += 1
            d["ms"] += ms
    # streaming-copy calibration: achievable bandwidth, and the known-traffic kernel for counter scaling
    copy_gbps = None
    if args.copy_mib > 0:
        a_buf = torch.empty(args.copy_mib << 18, dtype=torch.float32, device=dev).normal_()
        b_buf = torch.empty_like(a_buf)
        tbe.timing_enable(True)
        for _ in range(4):
            tbe.calibration_copy(b_buf, a_buf)
        ms = [m for n, m in tbe.timing_read() if n == "calibration_copy"][1:]
        copy_gbps = 2.0 * a_buf.numel() * 4 / (sum(ms) / len(ms) * 1e-3) / 1e9
        del a_buf, b_buf
    # gather calibration: random slices of known size from a window that fits an L2 (2 MiB per XCD), the Infinity
    # Cache (32 MiB shared) or neither (2 GiB per XCD), and the same with every slice written back - what this box
    # delivers for the access pattern of the embedding kernels.  (Slice sizes differ per case only so that the cases
    # carry different kernel names in a profile; rates do not depend on the size from 128 bytes up.  The two small
    # read-modify-write cases are the pieces a row would be cut into if every XCD owned an eighth of its columns.)
    gather = None
    if args.gather_gib > 0:
        g_buf = torch.zeros(args.gather_gib << 30, dtype=torch.uint8, device=dev)
        sink = torch.empty(4 << 20, dtype=torch.uint8, device=dev)
        per_xcd_big = (args.gather_gib << 30) // 8
        cases = [("l2_resident_256B", 2 << 20, 256, True, False), ("infinity_cache_512B", 32 << 20, 512, False, False),
                 ("hbm_1KiB", per_xcd_big, 1024, True, False), ("hbm_128B", per_xcd_big, 128, True, False),
                 ("hbm_rmw_512B", per_xcd_big, 512, True, True), ("hbm_rmw_64B", per_xcd_big, 64, True, True),
                 ("hbm_rmw_32B", per_xcd_big, 32, True, True)]
        gather = {}
        for name, window, sl, per_xcd, wb in cases:
            n = int(4e9 // sl)
            if wb:
                n = min(n, 8 * (window // sl))
            tbe.timing_enable(True)
            for _ in range(3):
                tbe.calibration_gather(g_buf, window, sl, n, per_xcd=per_xcd, write_back=wb, sink=sink)
            ms = [m for nm, m in tbe.timing_read() if nm == "calibration_gather"][1:]
            gather[name] = {"read_GBps": n * sl / (sum(ms) / len(ms) * 1e-3) / 1e9, "slices": n, "slice_bytes": sl,
                            "window_bytes": window, "per_xcd_windows": per_xcd, "written_back": wb}
        del g_buf, sink
    tbe.timing_enable(False)
    torch.cuda.synchronize()
    profiler_region(False)
    U_all = realised_unique(cfg, batches, torch)
    nnz_all = [int(i.numel()) for i, _ in batches]
    used = [(args.warmup + args.steps + k) % pool for k in range(prof_steps)]
    alg = {}
    for k in used:
        for name, b in algorithmic_bytes(cfg, nnz_all[k], U_all[k], ib=8 if args.index_dtype == "i64" else 4,
                                         eb=4 if args.io == "f32" else 2).items():
            alg[name] = alg.get(name, 0.0) + b / len(used)   # mean over the profiled batches, per step
    kernels = {}
    for name, d in per_kernel.items():
        per_step_launches = d["launches"] / prof_steps
        avg_ms = d["ms"] / d["launches"]
        bytes_per_launch = alg.get(name, 0.0)
        kernels[name] = {"launches_per_step": per_step_launches, "avg_ms": avg_ms, "ms_per_step": d["ms"] / prof_steps,
                         "min_ms": min(d["all"]), "median_ms": sorted(d["all"])[len(d["all"]) // 2],
                         "alg_bytes_per_launch": bytes_per_launch,
                         "alg_GBps": bytes_per_launch / (avg_ms * 1e-3) / 1e9 if avg_ms > 0 else 0.0}
        measured = traffic.get(name) if traffic else None
        if measured:   # bytes the counters saw per timing record, against what the method must move
            kernels[name]["measured_bytes"] = measured
            kernels[name]["measured_GBps"] = measured / (d["ms"] / prof_steps * 1e-3) / 1e9
            if bytes_per_launch > 0:
                kernels[name]["amplification"] = measured / (bytes_per_launch * per_step_launches)
    dominant = max(kernels, key=lambda n: kernels[n]["ms_per_step"])
    dk = kernels[dominant]
    roofline = {"bound": "hbm", "kernel": dominant, "achieved": dk["alg_GBps"], "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                "frac": dk["alg_GBps"] / HBM_PEAK_GBPS, "avg_launch_ms": dk["avg_ms"],
                "alg_bytes_per_launch": dk["alg_bytes_per_launch"],
                "traffic": (traffic.get(dominant) / max(1.0, dk["launches_per_step"])) if traffic and traffic.get(dominant)
                else None}
    if gather:   # the dominant kernel's counter traffic against what the box delivers for gathers beyond the caches
        roofline["measured_hbm_gather_GBps"] = gather["hbm_1KiB"]["read_GBps"]
        if roofline["traffic"]:
            roofline["traffic_GBps"] = roofline["traffic"] / (dk["avg_ms"] * 1e-3) / 1e9
            roofline["traffic_frac_of_hbm_gather_rate"] = roofline["traffic_GBps"] / gather["hbm_1KiB"]["read_GBps"]
    fwd_ms = kernels.get("forward_pool", {}).get("ms_per_step", 0.0)
    kernel_ms = sum(k["ms_per_step"] for k in kernels.values())
    step_alg_bytes = sum(alg.get(n, 0.0) * kernels[n]["launches_per_step"] for n in kernels)
    # compulsory bytes of one whole step: the forward set + the backward set (ids are read once more by linearize)
    compulsory = alg["forward_pool"] + alg["seg_update"] + sum(nnz_all[k] for k in used) / len(used) * (8 if args.index_dtype == "i64" else 4)

    counter_bytes = (sum(traffic.values()) or None) if traffic else None
    # the whole step against the roofline: compulsory bytes of forward + backward over the measured time per step
    step_GBps = compulsory / (ms_per_step * 1e-3) / 1e9
    roofline_step = {"bound": "hbm", "achieved": step_GBps, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": step_GBps / HBM_PEAK_GBPS, "compulsory_bytes_per_step": compulsory,
                     "ms_per_step": ms_per_step}
    bwd_ms = kernel_ms - fwd_ms
    roofline_backward = {"bound": "hbm", "achieved": alg["seg_update"] / (bwd_ms * 1e-3) / 1e9 if bwd_ms > 0 else None,
                         "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                         "frac": alg["seg_update"] / (bwd_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS if bwd_ms > 0 else None,
                         "compulsory_bytes": alg["seg_update"], "ms": bwd_ms}
    wb = 4 if cfg.weight_dtype == "f32" else 2
    eb = 4 if args.io == "f32" else 2
    d_bar = cfg.total_elems / max(1, cfg.total_rows)    # row-weighted mean width; ids are spread over rows
    logical_bytes = (lookups / max(1, args.steps)) * d_bar * (wb + eb)

    # ---- CPU oracle on a bounded sample of the same workload (rank 0, N=1): whole tables, full batch size,
    #      as many leading tables as fit the time budget
    cpu = None
    cpu_all = None
    if not args.no_cpu_baseline:
        import numpy as np
        import oracle
        oracle.build()
        idx, off = batches[0]
        bounds = off[:: cfg.B].tolist()
        woff = cfg.w_offsets()
        # first table alone to estimate the cost per lookup, then extend to the budget
        def sample(nt):
            tabs = []
            for t in range(nt):
                a = flat[woff[t]:woff[t + 1]].view(cfg.rows[t], cfg.D[t]).cpu().numpy()
                tabs.append(np.ascontiguousarray(a))
            i_np = idx[:bounds[nt]].cpu().numpy()
            o_np = off[: nt * cfg.B + 1].cpu().numpy()
            doff = cfg.D_offsets()[nt]
            g_t = gouts[0][:, :doff].contiguous().cpu()
            g_np = g_t.view(torch.int16).numpy().view(np.uint16) if args.io == "bf16" else g_t.numpy()
            st = np.ascontiguousarray(state[: cfg.row_base()[nt]].cpu().numpy())
            return tabs, st, g_np, i_np, o_np

        def run(nt, reps):
            tabs, st, g_np, i_np, o_np = sample(nt)
            t0 = time.perf_counter()
            for _ in range(reps):
                oracle.forward(tabs, i_np, o_np, cfg.B, cfg.pooling, out_dtype=args.io)
                oracle.backward_rowwise_adagrad(tabs, None if args.optimizer == "sgd" else st, g_np, i_np, o_np, cfg.B,
                                                cfg.pooling, cfg.lr, cfg.eps, cfg.c, want_indices=False,
                                                grad_dtype=args.io)
            return time.perf_counter() - t0, int(i_np.size) * reps

        t1, n1 = run(1, 1)
        per_lookup = t1 / max(1, n1)
        total_nnz = int(idx.numel())
        budget_lookups = args.cpu_seconds / max(per_lookup, 1e-12)
        if budget_lookups >= total_nnz:
            nt, reps = cfg.T, max(1, int(budget_lookups // total_nnz))
        else:
            nt = 1
            while nt < cfg.T and bounds[nt + 1] <= budget_lookups:
                nt += 1
            reps = 1
        secs, n = run(nt, min(reps, 50))
        host_cores = os.cpu_count() or 1
        cpu_model = "unknown"
        try:
            for line in open("/proc/cpuinfo"):
                if line.lower().startswith("model name"):
                    cpu_model = line.split(":", 1)[1].strip()
                    break
        except OSError:
            pass
        shapes = ", ".join(f"{cfg.rows[t]}x{cfg.D[t]}" for t in range(min(nt, 8))) + (" ..." if nt > 8 else "")
        cpu = {"value": n / secs, "unit": "lookups/s", "cores": 1, "kind": "oracle",
               "sample": f"first {nt} of {cfg.T} tables (rows x D: {shapes}; {cfg.weight_dtype} weights) at full batch "
                         f"size B={cfg.B}, {min(reps, 50)} pass(es), {n} lookups in {secs:.1f}s, fwd+bwd, single thread",
               "seconds": secs, "host_cores": host_cores, "cpu_model": cpu_model}
        # the same oracle with its loop over tables split over the host's cores: plain threads, one table each per
        # round (the C oracle runs outside the interpreter lock); tables are independent in both passes
        from concurrent.futures import ThreadPoolExecutor
        workers = max(1, min(host_cores, args.cpu_threads, cfg.T))
        want = min(cfg.T, workers * max(1, int(args.cpu_seconds / max(per_lookup * bounds[1], 1e-9))))
        want = max(workers, min(want, 2 * workers))
        want = min(want, cfg.T)
        doffs = cfg.D_offsets()

        def one_table(t):
            a = np.ascontiguousarray(flat[woff[t]:woff[t + 1]].view(cfg.rows[t], cfg.D[t]).cpu().numpy())
            i_np = idx[bounds[t]:bounds[t + 1]].cpu().numpy()
            o_np = (off[t * cfg.B:(t + 1) * cfg.B + 1] - off[t * cfg.B]).cpu().numpy()
            g_t = gouts[0][:, doffs[t]:doffs[t + 1]].contiguous().cpu()
            g_np = g_t.view(torch.int16).numpy().view(np.uint16) if args.io == "bf16" else g_t.numpy()
            st = np.ascontiguousarray(state[cfg.row_base()[t]:cfg.row_base()[t + 1]].cpu().numpy())
            return [a], st, g_np, i_np, o_np

        samples = [one_table(t) for t in range(want)]        # copies from HBM: untimed

        def work(sm):
            tabs, st, g_np, i_np, o_np = sm
            oracle.forward(tabs, i_np, o_np, cfg.B, cfg.pooling, out_dtype=args.io)
            oracle.backward_rowwise_adagrad(tabs, None if args.optimizer == "sgd" else st, g_np, i_np, o_np, cfg.B,
                                            cfg.pooling, cfg.lr, cfg.eps, cfg.c, want_indices=False, grad_dtype=args.io)
            return int(i_np.size)

        t0 = time.perf_counter()
        with ThreadPoolExecutor(max_workers=workers) as ex:
            n_all = sum(ex.map(work, samples))
        secs_all = time.perf_counter() - t0
        cpu_all = {"value": n_all / secs_all, "unit": "lookups/s", "cores": workers, "kind": "oracle",
                   "sample": f"first {want} of {cfg.T} tables at full batch size B={cfg.B}, one pass, one table per thread "
                             f"at a time, {n_all} lookups in {secs_all:.1f}s, fwd+bwd",
                   "seconds": secs_all, "host_cores": host_cores, "cpu_model": cpu_model}

    result = {
        "metric": "lookups/sec, fused TBE fwd+bwd+rowwise AdaGrad (achieved HBM GB/s in roofline)",
        "value": value, "unit": "lookups/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": ("" if args.rows_scale == 1.0 else f"rows x{args.rows_scale} of ") + W.describe(cfg), "weight_dtype": cfg.weight_dtype, "index_dtype": args.index_dtype,
                   "io_dtype": args.io, "optimizer": args.optimizer,
                   "lookups_per_step": lookups / max(1, args.steps), "unique_rows_per_lookup":
                       sum(sum(u) for u in U_all) / max(1, sum(nnz_all)), "batch_pool": pool,
                   "lr": cfg.lr, "eps": cfg.eps, "momentum_scale": cfg.c,
                   "launch": "hip_graph" if args.graph else ("eager, sort on a second stream" if args.sort_stream else "eager")},
        "roofline": roofline,
        "roofline_step": roofline_step,
        "roofline_backward": roofline_backward,
        "cpu_baseline": cpu,
        "cpu_baseline_all_cores": cpu_all,
        "build": build_info(),
        "profiled_steps": prof_steps,
        "measured_gather": gather,
        "step_breakdown": {"forward_ms": fwd_ms, "backward_ms": kernel_ms - fwd_ms, "sum_kernel_ms": kernel_ms,
                           "compulsory_bytes_per_step": compulsory,
                           "compulsory_GBps_at_measured_step": compulsory / (ms_per_step * 1e-3) / 1e9,
                           "all_kernels_alg_bytes_per_step": step_alg_bytes,
                           "forward_lookups_per_s": (lookups / max(1, args.steps)) / (fwd_ms * 1e-3) if fwd_ms > 0 else None,
                           "backward_lookups_per_s": (lookups / max(1, args.steps)) / ((kernel_ms - fwd_ms) * 1e-3)
                           if kernel_ms > fwd_ms else None,
                           # cache-level throughput: one table row per lookup (forward) and one gradient slice per
                           # lookup (backward), whether served by a cache or by HBM; may exceed the HBM peak
                           "logical_gathered_GBps": logical_bytes / (ms_per_step * 1e-3) / 1e9,
                           # what the byte counters of the profiles saw leave the L2 in one step, over the measured
                           # step time (null for workloads without a committed counter profile)
                           "counter_traffic_bytes_per_step": counter_bytes,
                           "counter_traffic_GBps_at_measured_step":
                               counter_bytes / (ms_per_step * 1e-3) / 1e9 if counter_bytes else None,
                           "counter_traffic_frac_of_peak":
                               counter_bytes / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBPS if counter_bytes else None},
        "measured_copy_GBps": copy_gbps,
        "kernels": kernels,
    }
    print(json.dumps(result))


if __name__ == "__main__":
    main()
