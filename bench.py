#!/usr/bin/env python3
"""Benchmark of the row-wise top-k hot path on one MI355X.

A step is one call of the exact-mode entry point (load, min/max, binary search, select, store) over
the MaxK-GNN hidden-layer workload: N = 2^20 rows x M = 256 fp32, k = 32, seeded synthetic values
(per-row N(0,1) scaled by U(0.5,2)), already resident in HBM.  The early-stopping mode is timed the
same way and reported in the same JSON line.

Two timings of the same launches are reported.  "Warm": back-to-back launches over one input and one
output buffer (`value`, `roofline.frac`); at the headline size the 256 MiB of outputs are rewritten in
place launch after launch and part of that write traffic never reaches HBM.  "Cold": the launches rotate
over enough distinct input/output buffer sets that more than 4.3 GB are touched before any byte is
touched again (`roofline.frac_cold`): the rate of a single launch inside a larger program.

    python bench.py [--gpus 1] [--steps K] [--warmup W]

Before the W warm-up steps the kernel is run untimed for about 60 ms (--spinup-ms): after idle the
GPU needs ~15 ms of work before its clocks settle, and launches in that window take 15-30 % longer.

Prints exactly one JSON line on stdout; progress goes to stderr.
"""
from __future__ import annotations

import argparse
import json
import statistics
import os
import re
import sys
import time

PEAK_HBM_GBPS = 8000.0  # MI355X published HBM3E bandwidth
ROOT = os.path.dirname(os.path.abspath(__file__))
# One pass of a "cold" measurement touches at least this many bytes before any buffer is used again.
COLD_FOOTPRINT_BYTES = 4.3e9


def profile_name(kernel, workload, k, dtype="f32", op="pairs"):
    """File under profiles/ that summarises the rocprofv3 runs of this kernel on this workload."""
    extra = ("dtype" + dtype if dtype != "f32" else "") + ("op" + op if op != "pairs" else "")
    return os.path.join("profiles", f"{kernel}_{workload}_k{k}{extra}.md")


def measured_traffic(path, mode_arg=1):
    """HBM bytes per launch (FETCH_SIZE + WRITE_SIZE, each scaled by what the same counter reads for a
    device copy of known size) from a profile summary: the `* kernel<...>: HBM read A B + write B B = C B
    per launch` line of the exact-mode kernel (its MODE template argument is 1; kernels without a mode
    have a single line).  Counters need the profiler, so this is not measured live.  None if the file or
    the line is missing."""
    full = os.path.join(ROOT, path)
    if not os.path.exists(full):
        return None
    found = []
    for line in open(full):
        m = re.match(r"\* (\w+)<([^>]*)>: HBM read [\d,]+ B \+ write [\d,]+ B = ([\d,]+) B per launch", line)
        if m:
            found.append((m.group(1), m.group(2).split(","), int(m.group(3).replace(",", ""))))
    if not found:
        return None
    if len(found) == 1:
        return found[0][2]
    for name, args, total in found:
        # MODE is the 5th template argument of rtopk_wave_kernel / rtopk_dense_kernel, the 4th of rtopk_block_kernel,
        # the 2nd of rtopk_stream_kernel
        pos = 3 if name == "rtopk_block_kernel" else (1 if name == "rtopk_stream_kernel" else 4)
        if len(args) > pos and args[pos] == str(mode_arg):
            return total
    return None


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
    ap.add_argument("--op", default="pairs", choices=("pairs", "dense", "backward", "backward_gather"),
                    help="pairs: k (value, column) pairs per row (the headline); dense: the selected values in place "
                         "and zero elsewhere (rtopk_maxk_dense, fp32 only); backward / backward_gather: the backward "
                         "edge of the MaxK non-linearity in scatter / gather form, on the columns the forward saved")
    ap.add_argument("--dtype", default="f32", choices=("f32", "f16", "bf16"),
                    help="storage type of the rows and of the value output (16-bit types: the same matrix rounded "
                         "to nearest; the search still runs in fp32)")
    ap.add_argument("--cold-sets", type=int, default=-1,
                    help="number of distinct input/output buffer sets the cold timing rotates over "
                         "(-1: as many as make one rotation touch more than 4.3 GB, at least 2; 0: skip)")
    ap.add_argument("--cold-rotate", default="both", choices=("both", "in", "out"),
                    help="which buffers the cold timing rotates (in / out: the other side stays one buffer; for "
                         "telling apart what the warm figure owes to inputs and to outputs)")
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
    half = args.dtype != "f32"
    dense = args.op == "dense"
    backward = args.op in ("backward", "backward_gather")
    if (dense or backward) and half:
        log("bench.py: --op %s is fp32 only" % args.op)
        sys.exit(2)
    if half or dense:
        u8 = False  # the 16-bit entry points write int32 columns; the dense form has no columns
    log(f"generating {args.workload} input N={N} M={M} ...")
    x_host = workloads.make(args.workload, N=N)
    x_bits = None
    tdt = torch.float32
    if half:
        tdt = {"f16": torch.float16, "bf16": torch.bfloat16}[args.dtype]
        x_bits = workloads.to_bits16(x_host, args.dtype)
        x = torch.from_numpy(x_bits.view(np.int16)).cuda().view(tdt)
    else:
        x = torch.from_numpy(x_host).cuda()
    esz = 2 if half else 4
    isz = 1 if u8 else 4
    idt = torch.uint8 if u8 else torch.int32

    # One buffer set = everything one launch reads and writes.  `fns(set)` returns the (exact, early)
    # callables on that set; set 0 is the warm one.
    if backward:
        # the columns the forward pass saves, and a seeded gradient
        _, idx0 = (R.rtopk_rowwise_exact_u8 if u8 else R.rtopk_rowwise_exact)(x, k)
        if args.op == "backward":
            g_host = workloads.normal(N, k, seed=cfg["seed"] + 100)
        else:
            g_host = workloads.normal(N, M, seed=cfg["seed"] + 100)
        g0 = torch.from_numpy(g_host).cuda()
        torch.cuda.synchronize()
        del x
        algo_bytes = N * (4 * M + k * (4 + isz))  # dense row once + k gradients + k columns, each once

        def new_set(first):
            g = g0 if first else g0.clone()
            ix = idx0 if first else idx0.clone()
            out = torch.empty((N, M) if args.op == "backward" else (N, k), dtype=torch.float32, device="cuda")
            return {"in": (g, ix), "out": (out,)}

        def fns(ins, outs):
            g, ix = ins
            (out,) = outs
            if args.op == "backward":
                f = lambda: R.rtopk_maxk_backward(g, ix, M, out)
            else:
                f = lambda: R.rtopk_maxk_backward_gather(g, ix, out)
            return f, f
    elif dense:
        algo_bytes = N * M * 8  # read the row once, write it once

        def new_set(first):
            return {"in": (x if first else x.clone(),), "out": (torch.empty_like(x),)}

        def fns(ins, outs):
            (xi,) = ins
            (od,) = outs
            return (lambda: R.rtopk_maxk_dense(xi, k, -1, od)), (lambda: R.rtopk_maxk_dense(xi, k, max_iter, od))
    else:
        algo_bytes = N * (esz * M + k * (esz + isz))  # read the row once, write k (value, column) pairs once
        if half:
            f_exact = getattr(R, "rtopk_rowwise_exact_" + args.dtype)
            f_early = getattr(R, "rtopk_rowwise_" + args.dtype)
        else:
            f_exact = R.rtopk_rowwise_exact_u8 if u8 else R.rtopk_rowwise_exact
            f_early = R.rtopk_rowwise_u8 if u8 else R.rtopk_rowwise

        def new_set(first):
            return {"in": (x if first else x.clone(),),
                    "out": (torch.empty((N, k), dtype=tdt, device="cuda"), torch.empty((N, k), dtype=idt, device="cuda"))}

        def fns(ins, outs):
            (xi,) = ins
            ov, oi = outs
            return (lambda: f_exact(xi, k, ov, oi)), (lambda: f_early(xi, k, max_iter, ov, oi))

    set0 = new_set(True)
    exact, early = fns(set0["in"], set0["out"])
    torch.cuda.synchronize()

    log("timing exact mode (warm: one input, one output buffer) ...")
    spin_up(torch, exact, args.spinup_ms)
    wall_e, launch_e = time_calls(torch, exact, args.steps, args.warmup)
    log(f"  exact: {wall_e / args.steps * 1e6:.1f} us/step wall, {launch_e * 1e6:.1f} us/launch (events)")
    if backward:
        wall_s, launch_s = wall_e, launch_e
    else:
        log(f"timing early-stop mode (max_iter={max_iter}) ...")
        spin_up(torch, early, args.spinup_ms / 4)
        wall_s, launch_s = time_calls(torch, early, args.steps, args.warmup)
        log(f"  early: {wall_s / args.steps * 1e6:.1f} us/step wall, {launch_s * 1e6:.1f} us/launch (events)")

    # Cold timing: the same launches rotating over distinct buffer sets.
    cold = None
    n_sets = args.cold_sets
    if n_sets < 0:
        n_sets = max(2, int(-(-COLD_FOOTPRINT_BYTES // algo_bytes)))
    if n_sets >= 2:
        sets = [set0] + [new_set(False) for _ in range(n_sets - 1)]
        torch.cuda.synchronize()
        pairs = []
        for i in range(n_sets):
            ins = sets[i]["in"] if args.cold_rotate in ("both", "in") else set0["in"]
            outs = sets[i]["out"] if args.cold_rotate in ("both", "out") else set0["out"]
            pairs.append(fns(ins, outs))
        state = {"i": 0}

        def rot(which):
            def f():
                pairs[state["i"] % n_sets][which]()
                state["i"] += 1
            return f

        log(f"timing exact mode (cold: rotating over {n_sets} buffer sets, rotate={args.cold_rotate}) ...")
        spin_up(torch, rot(0), args.spinup_ms / 4)
        wall_ce, launch_ce = time_calls(torch, rot(0), args.steps, args.warmup)
        log(f"  exact cold: {launch_ce * 1e6:.1f} us/launch (events)")
        launch_cs = launch_ce
        if not backward:
            spin_up(torch, rot(1), args.spinup_ms / 4)
            _, launch_cs = time_calls(torch, rot(1), args.steps, args.warmup)
            log(f"  early cold: {launch_cs * 1e6:.1f} us/launch (events)")
        cold = {"sets": n_sets, "rotate": args.cold_rotate, "bytes_per_rotation": algo_bytes * n_sets,
                "exact_us": launch_ce * 1e6, "early_us": launch_cs * 1e6}
        del sets, pairs

    copy_gbps = None
    if args.with_copy:
        src = set0["in"][0]
        y = torch.empty_like(src)
        for _ in range(5):
            y.copy_(src)
        torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(20):
            y.copy_(src)
        b.record()
        torch.cuda.synchronize()
        copy_gbps = 2 * src.numel() * src.element_size() / (a.elapsed_time(b) * 1e-3 / 20) / 1e9
        log(f"  device copy of the input (read + write): {a.elapsed_time(b) / 20 * 1e3:.1f} us, {copy_gbps:.0f} GB/s")
        del y

    parity = None
    recall = None
    cpu = None
    if not args.no_parity or not args.no_cpu_baseline:
        import oracle
    if not args.no_parity:
        log("parity against the CPU oracle on every row ...")
        if backward:
            exact()
            torch.cuda.synchronize()
            idx_h = idx0.cpu().numpy().astype(np.int32)
            got = set0["out"][0].cpu().numpy().view(np.int32)
            want = oracle.maxk_backward(g_host, idx_h, M) if args.op == "backward" else oracle.maxk_backward_gather(g_host, idx_h)
            parity = {"exact": bool(np.array_equal(got, want.view(np.int32)))}
            log(f"  parity {parity}")
        else:
            if half:
                ev, ei = oracle.topk_exact_16(x_bits, args.dtype, k)
                sv, si = oracle.topk_earlystop_16(x_bits, args.dtype, k, max_iter)
            else:
                ev, ei = oracle.topk_exact(x_host, k)
                sv, si = oracle.topk_earlystop(x_host, k, max_iter)
                ev, sv = ev.view(np.int32), sv.view(np.int32)

            def out_bits():
                o = set0["out"][0]
                if half:
                    return o.view(torch.int16).cpu().numpy().view(np.uint16)
                return o.cpu().numpy().view(np.int32)

            exact()
            torch.cuda.synchronize()
            if dense:
                ok_e = bool(np.array_equal(out_bits(), oracle.maxk_dense(x_host, k).view(np.int32)))
            else:
                ok_e = bool(np.array_equal(set0["out"][1].cpu().numpy().astype(np.int32), ei) and np.array_equal(out_bits(), ev))
            early()
            torch.cuda.synchronize()
            if dense:
                ok_s = bool(np.array_equal(out_bits(), oracle.maxk_dense(x_host, k, max_iter).view(np.int32)))
                # the columns the GPU's early-stop search selects, for the recall figure below
                gi = R.rtopk_rowwise(set0["in"][0], k, max_iter)[1].cpu().numpy()
            else:
                gi = set0["out"][1].cpu().numpy().astype(np.int32)
                ok_s = bool(np.array_equal(gi, si) and np.array_equal(out_bits(), sv))
            parity = {"exact": ok_e, "early_stop": ok_s}
            recall = oracle.mean_overlap(gi, ei)
            log(f"  parity {parity}, early-stop recall vs exact {recall:.4f}")
    if not args.no_cpu_baseline:
        if backward:
            log("timing the CPU oracle (same backward form) on the same input ...")
            idx_h = idx0.cpu().numpy().astype(np.int32)

            def oracle_pass():
                t0 = time.perf_counter()
                if args.op == "backward":
                    oracle.maxk_backward(g_host, idx_h, M)
                else:
                    oracle.maxk_backward_gather(g_host, idx_h)
                return time.perf_counter() - t0
            what = "plain loops, OpenMP over rows"
        else:
            log("timing the CPU oracle (exact mode) on the same input ...")

            def oracle_pass():
                t0 = time.perf_counter()
                if half:
                    oracle.topk_exact_16(x_bits, args.dtype, k)
                else:
                    oracle.topk_exact(x_host, k)
                return time.perf_counter() - t0
            what = "exact mode (nth_element per row, OpenMP over rows)"

        first = oracle_pass()  # warm-up, also sizes the sample: about 10 s of CPU work in all
        n_pass = int(min(100, max(8, round(10.0 / max(first, 1e-3)))))
        reps = [oracle_pass() for _ in range(n_pass)]
        t_cpu = statistics.median(reps)
        cpu = {"value": N / t_cpu, "unit": "rows/s", "cores": oracle.num_threads(), "kind": "oracle",
               "sample": f"all {N} rows of the same input, {what}, "
                         f"median of {n_pass} passes after 1 warm-up ({sum(reps):.1f} s of CPU work)"}
        log(f"  oracle: {t_cpu:.3f} s per pass on {cpu['cores']} threads")
        # the same on one thread, on the first 65536 rows
        if not half and not backward and N >= 65536:
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

    if backward:
        kernel = ("maxk_scatter_" if args.op == "backward" else "maxk_gather_") + ("rows_kernel" if M <= 2048 else "block_kernel")
    elif M > 65536:
        kernel = "rtopk_stream_kernel"
    elif M > 8192:
        kernel = "rtopk_block_kernel"
    else:
        kernel = "rtopk_dense_kernel" if dense else "rtopk_wave_kernel"
    prof = profile_name(kernel, args.workload, k, args.dtype, args.op)
    traffic = measured_traffic(prof) if N == cfg["N"] else None
    rows_per_s = N * args.steps / wall_e
    op_text = {"pairs": "row top-k", "dense": "row top-k, dense (MaxK) output", "backward": "MaxK backward (scatter)",
               "backward_gather": "MaxK backward (gather)"}[args.op]
    roofline = {"bound": "hbm", "achieved": algo_bytes / launch_e / 1e9, "peak": PEAK_HBM_GBPS,
                "unit": "GB/s", "frac": algo_bytes / launch_e / 1e9 / PEAK_HBM_GBPS,
                "traffic": traffic, "traffic_source": prof if traffic is not None else None,
                "kernel": "%s, %sM=%d" % (kernel, "" if backward else "exact mode, ", M),
                "algorithmic_bytes_per_launch": algo_bytes, "avg_launch_us": launch_e * 1e6,
                "footprint": "warm: every launch reads and writes the same buffers",
                "device_copy_gbps": copy_gbps}
    if cold is not None:
        roofline.update({"achieved_cold": algo_bytes / (cold["exact_us"] * 1e-6) / 1e9,
                         "frac_cold": algo_bytes / (cold["exact_us"] * 1e-6) / 1e9 / PEAK_HBM_GBPS,
                         "avg_launch_us_cold": cold["exact_us"],
                         "footprint_cold": "launches rotate over %d distinct buffer sets (%s): %.2f GB touched per rotation"
                                           % (cold["sets"], cold["rotate"], cold["bytes_per_rotation"] / 1e9)})
    result = {
        "metric": "rows/sec, %s N=%d M=%d k=%d %s%s"
                  % (op_text, N, M, k, {"f32": "fp32", "f16": "fp16 rows (fp32 search)", "bf16": "bf16 rows (fp32 search)"}[args.dtype],
                     "" if backward else ", exact mode (early-stop alongside)"),
        "value": rows_per_s,
        "unit": "rows/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": wall_e / args.steps * 1e3,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        # the type the path computes in: comparisons and midpoints are fp32 whatever the rows are stored as
        "dtype": "f32",
        "storage_dtype": args.dtype,
        "data": "synthetic",
        "config": {"workload": "%s: N=%d x M=%d %s, %s, seed %d" % (args.workload, N, M, args.dtype, cfg["dist"], cfg["seed"]),
                   "k": k, "mode": "backward" if backward else "exact", "index_type": "uint8" if u8 else "int32", "output": args.op},
        "early_stop": None if backward else {
            "max_iter": max_iter, "rows_per_s": N * args.steps / wall_s, "ms_per_step": wall_s / args.steps * 1e3,
            "hbm_gbps": algo_bytes / launch_s / 1e9,
            "hbm_gbps_cold": (algo_bytes / (cold["early_us"] * 1e-6) / 1e9) if cold is not None else None,
            "recall_vs_exact": recall},
        "parity_vs_oracle": parity,
        "roofline": roofline,
        "cpu_baseline": cpu,
    }
    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
