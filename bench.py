#!/usr/bin/env python3
"""Benchmark of the row-wise top-k hot path on one MI355X.

A step is one call of the exact-mode entry point (load, min/max, binary search, select, store) over
the MaxK-GNN hidden-layer workload: N = 2^20 rows x M = 256 fp32, k = 32, seeded synthetic values
(per-row N(0,1) scaled by U(0.5,2)), already resident in HBM.  The early-stopping mode is timed the
same way and reported in the same JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W]

Before the W warm-up steps the kernel is run untimed for about 60 ms (--spinup-ms): after idle the
GPU needs ~15 ms of work before its clocks settle, and launches in that window take 15-30 % longer.

Prints exactly one JSON line on stdout; progress goes to stderr.
"""
from __future__ import annotations

import argparse
import json
import statistics
import sys
import time

PEAK_HBM_GBPS = 8000.0  # MI355X published HBM3E bandwidth
# HBM bytes per launch of the exact-mode kernel (FETCH_SIZE + WRITE_SIZE, scaled by a copy kernel of known
# size), from the rocprofv3 --pmc runs summarised under profiles/ (not measured live: counters need the
# profiler).  Keyed by (workload, k, dtype, op) at the workload's full row count.
MEASURED_TRAFFIC = {
    ("c1_maxk", 32, "f32", "pairs"): (1342397495, "profiles/rtopk_wave_kernel_c1_maxk_k32.md"),
    ("c1_maxk", 32, "bf16", "pairs"): (738399789, "profiles/rtopk_wave_kernel_c1_maxk_k32dtypebf16.md"),
    ("c1_maxk", 32, "f32", "dense"): (2147639472, "profiles/rtopk_dense_kernel_c1_maxk_k32opdense.md"),
    ("c2_w128", 16, "f32", "pairs"): (671333304, "profiles/rtopk_wave_kernel_c2_w128_k16.md"),
    ("c2_w512", 64, "f32", "pairs"): (2684437542, "profiles/rtopk_wave_kernel_c2_w512_k64.md"),
    ("c2_w1024", 128, "f32", "pairs"): (5368919951, "profiles/rtopk_wave_kernel_c2_w1024_k128.md"),
    ("c3_ties", 32, "f32", "pairs"): (2841775990, "profiles/rtopk_wave_kernel_c3_ties_k32.md"),
    ("c4_wide", 64, "f32", "pairs"): (1107526387, "profiles/rtopk_wave_kernel_c4_wide_k64.md"),
    ("x_wide32k", 256, "f32", "pairs"): (1090981092, "profiles/rtopk_block_kernel_x_wide32k_k256.md"),
}


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def spin_up(torch, fn, ms):
    """Run `fn` back to back for about `ms` milliseconds of GPU time (untimed)."""
    if ms <= 0:
        return
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    for _ in range(5):
        fn()
    b.record()
    torch.cuda.synchronize()
    per = max(a.elapsed_time(b) / 5.0, 1e-3)
    for _ in range(int(ms / per) + 1):
        fn()
    torch.cuda.synchronize()


def time_calls(torch, fn, steps, warmup):
    """Returns (wall seconds for `steps` calls, mean seconds per launch).

    Wall time is taken between two device synchronisations.  The per-launch figure comes from one pair
    of HIP events recorded on the launch stream right before the first and right after the last of the
    `steps` back-to-back launches (so it is the steady-state launch-to-launch duration on the GPU's own
    clock, without the host's synchronisation cost)."""
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    start = torch.cuda.Event(enable_timing=True)
    end = torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    start.record()
    for _ in range(steps):
        fn()
    end.record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    return wall, start.elapsed_time(end) * 1e-3 / steps


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=1000)
    ap.add_argument("--warmup", type=int, default=50)
    ap.add_argument("--spinup-ms", type=float, default=60.0,
                    help="untimed launches run for about this long before the warm-up steps, so that the GPU's "
                         "clocks have settled: the first ~15 ms after idle run 15-30%% slower")
    ap.add_argument("--workload", default="c1_maxk",
                    help="name in workloads.CONFIGS (default: the headline c1_maxk, N=2^20 x M=256)")
    ap.add_argument("--rows", type=int, default=None, help="override the workload's N")
    ap.add_argument("--k", type=int, default=None, help="default: 32 for M=256, else the workload's first k")
    ap.add_argument("--max-iter", type=int, default=8)
    ap.add_argument("--op", default="pairs", choices=("pairs", "dense"),
                    help="pairs: k (value, column) pairs per row (the headline); dense: the selected values in place "
                         "and zero elsewhere (rtopk_maxk_dense, fp32 only)")
    ap.add_argument("--dtype", default="f32", choices=("f32", "f16", "bf16"),
                    help="storage type of the rows and of the value output (16-bit types: the same matrix rounded "
                         "to nearest; the search still runs in fp32)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-parity", action="store_true")
    ap.add_argument("--with-copy", action="store_true",
                    help="also run a plain device copy of the input (1 read + 1 write of N*M*4 bytes) a few times: "
                         "the known-size kernel that scales the profiler's FETCH_SIZE / WRITE_SIZE counters")
    args = ap.parse_args()
    if args.gpus != 1:
        log("bench.py: this build runs on one GPU only (rows are independent; see the design notes on "
            "sharding). Re-run with --gpus 1.")
        sys.exit(2)

    import numpy as np
    import torch

    import paper_2409_00822_amd as R
    import workloads

    R.load_library()
    if not torch.cuda.is_available():
        log("bench.py: no GPU visible")
        sys.exit(1)

    cfg = workloads.CONFIGS[args.workload]
    N = args.rows if args.rows is not None else cfg["N"]
    M, max_iter = cfg["M"], args.max_iter
    k = args.k if args.k is not None else (32 if 32 in cfg["ks"] else cfg["ks"][0])
    u8 = cfg["idx"] == "uint8"
    log(f"generating {args.workload} input N={N} M={M} ...")
    x_host = workloads.make(args.workload, N=N)
    half = args.dtype != "f32"
    if half:
        u8 = False  # the 16-bit entry points write int32 columns
        tdt = {"f16": torch.float16, "bf16": torch.bfloat16}[args.dtype]
        x_bits = workloads.to_bits16(x_host, args.dtype)
        del x_host
        x = torch.from_numpy(x_bits.view(np.int16)).cuda().view(tdt)
        out_v = torch.empty((N, k), dtype=tdt, device="cuda")
    else:
        x = torch.from_numpy(x_host).cuda()
        out_v = torch.empty((N, k), dtype=torch.float32, device="cuda")
    out_i = torch.empty((N, k), dtype=torch.uint8 if u8 else torch.int32, device="cuda")
    torch.cuda.synchronize()

    # read the row once, write k (value, column) pairs once
    esz = 2 if half else 4
    algo_bytes = N * (esz * M + k * (esz + (1 if u8 else 4)))
    if half:
        f_exact = getattr(R, "rtopk_rowwise_exact_" + args.dtype)
        f_early = getattr(R, "rtopk_rowwise_" + args.dtype)
    else:
        f_exact = R.rtopk_rowwise_exact_u8 if u8 else R.rtopk_rowwise_exact
        f_early = R.rtopk_rowwise_u8 if u8 else R.rtopk_rowwise

    dense = args.op == "dense"
    if dense:
        assert not half, "--op dense is fp32 only"
        u8 = False
        out_d = torch.empty_like(x)
        algo_bytes = N * M * 8  # read the row once, write it once

    def exact():
        if dense:
            R.rtopk_maxk_dense(x, k, -1, out_d)
        else:
            f_exact(x, k, out_v, out_i)

    def early():
        if dense:
            R.rtopk_maxk_dense(x, k, max_iter, out_d)
        else:
            f_early(x, k, max_iter, out_v, out_i)

    log("timing exact mode ...")
    spin_up(torch, exact, args.spinup_ms)
    wall_e, launch_e = time_calls(torch, exact, args.steps, args.warmup)
    log(f"  exact: {wall_e / args.steps * 1e6:.1f} us/step wall, {launch_e * 1e6:.1f} us/launch (events)")
    log(f"timing early-stop mode (max_iter={max_iter}) ...")
    spin_up(torch, early, args.spinup_ms / 4)
    wall_s, launch_s = time_calls(torch, early, args.steps, args.warmup)
    log(f"  early: {wall_s / args.steps * 1e6:.1f} us/step wall, {launch_s * 1e6:.1f} us/launch (events)")

    copy_gbps = None
    if args.with_copy:
        y = torch.empty_like(x)
        for _ in range(5):
            y.copy_(x)
        torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(20):
            y.copy_(x)
        b.record()
        torch.cuda.synchronize()
        copy_gbps = 2 * x.numel() * x.element_size() / (a.elapsed_time(b) * 1e-3 / 20) / 1e9
        log(f"  device copy of the input (read + write): {a.elapsed_time(b) / 20 * 1e3:.1f} us, {copy_gbps:.0f} GB/s")
        del y

    parity = None
    recall = None
    cpu = None
    if not args.no_parity or not args.no_cpu_baseline:
        import oracle
    if not args.no_parity:
        log("parity against the CPU oracle on every row ...")
        def out_bits():
            if dense:
                return out_d.cpu().numpy().view(np.int32)
            if half:
                return out_v.view(torch.int16).cpu().numpy().view(np.uint16)
            return out_v.cpu().numpy().view(np.int32)

        if half:
            ev, ei = oracle.topk_exact_16(x_bits, args.dtype, k)
            sv, si = oracle.topk_earlystop_16(x_bits, args.dtype, k, max_iter)
        else:
            ev, ei = oracle.topk_exact(x_host, k)
            sv, si = oracle.topk_earlystop(x_host, k, max_iter)
            ev, sv = ev.view(np.int32), sv.view(np.int32)
        exact()
        torch.cuda.synchronize()
        if dense:
            ok_e = bool(np.array_equal(out_bits(), oracle.maxk_dense(x_host, k).view(np.int32)))
        else:
            ok_e = bool(np.array_equal(out_i.cpu().numpy().astype(np.int32), ei) and np.array_equal(out_bits(), ev))
        early()
        torch.cuda.synchronize()
        if dense:
            ok_s = bool(np.array_equal(out_bits(), oracle.maxk_dense(x_host, k, max_iter).view(np.int32)))
            gi = si
        else:
            gi = out_i.cpu().numpy().astype(np.int32)
            ok_s = bool(np.array_equal(gi, si) and np.array_equal(out_bits(), sv))
        parity = {"exact": ok_e, "early_stop": ok_s}
        recall = oracle.mean_overlap(gi, ei)
        log(f"  parity {parity}, early-stop recall vs exact {recall:.4f}")
    if not args.no_cpu_baseline:
        log("timing the CPU oracle (exact mode) on the same input ...")

        def oracle_pass():
            t0 = time.perf_counter()
            if half:
                oracle.topk_exact_16(x_bits, args.dtype, k)
            else:
                oracle.topk_exact(x_host, k)
            return time.perf_counter() - t0

        first = oracle_pass()  # warm-up, also sizes the sample: about 10 s of CPU work in all
        n_pass = int(min(100, max(8, round(10.0 / max(first, 1e-3)))))
        reps = [oracle_pass() for _ in range(n_pass)]
        t_cpu = statistics.median(reps)
        cpu = {"value": N / t_cpu, "unit": "rows/s", "cores": oracle.num_threads(), "kind": "oracle",
               "sample": f"all {N} rows of the same input, exact mode (nth_element per row, OpenMP over rows), "
                         f"median of {n_pass} passes after 1 warm-up ({sum(reps):.1f} s of CPU work)"}
        log(f"  oracle: {t_cpu:.3f} s per pass on {cpu['cores']} threads")
        # the same on one thread, on the first 65536 rows
        if not half and N >= 65536:
            threads = oracle.num_threads()
            oracle.set_num_threads(1)
            try:
                sl = x_host[:65536]
                oracle.topk_exact(sl, k)
                t1 = []
                for _ in range(5):
                    t0 = time.perf_counter()
                    oracle.topk_exact(sl, k)
                    t1.append(time.perf_counter() - t0)
                cpu["one_thread_rows_per_s"] = 65536 / statistics.median(t1)
            finally:
                oracle.set_num_threads(threads)

    traffic = MEASURED_TRAFFIC.get((args.workload, k, args.dtype, args.op), (None, None)) if N == cfg["N"] else (None, None)
    rows_per_s = N * args.steps / wall_e
    result = {
        "metric": "rows/sec, row top-k N=%d M=%d k=%d %s, exact mode (early-stop alongside)"
                  % (N, M, k, {"f32": "fp32", "f16": "fp16 rows (fp32 search)", "bf16": "bf16 rows (fp32 search)"}[args.dtype]),
        "value": rows_per_s,
        "unit": "rows/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": wall_e / args.steps * 1e3,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": "%s: N=%d x M=%d %s, %s, seed %d" % (args.workload, N, M, args.dtype, cfg["dist"], cfg["seed"]),
                   "k": k, "mode": "exact", "index_type": "uint8" if u8 else "int32", "output": args.op},
        "early_stop": {"max_iter": max_iter, "rows_per_s": N * args.steps / wall_s,
                       "ms_per_step": wall_s / args.steps * 1e3,
                       "hbm_gbps": algo_bytes / launch_s / 1e9, "recall_vs_exact": recall},
        "parity_vs_oracle": parity,
        "roofline": {"bound": "hbm", "achieved": algo_bytes / launch_e / 1e9, "peak": PEAK_HBM_GBPS,
                     "unit": "GB/s", "frac": algo_bytes / launch_e / 1e9 / PEAK_HBM_GBPS,
                     "traffic": traffic[0], "traffic_source": traffic[1],
                     "kernel": "%s, exact mode, M=%d" % ("rtopk_dense_kernel" if dense else "rtopk_wave_kernel", M),
                     "algorithmic_bytes_per_launch": algo_bytes, "avg_launch_us": launch_e * 1e6,
                     "device_copy_gbps": copy_gbps},
        "cpu_baseline": cpu,
    }
    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
