#!/usr/bin/env python3
"""Benchmark: host-resident DGEMM on one MI355X (the paper's single-GPU DGEMM experiment, Section V.A).

One step = one blasx_dgemm call on page-locked host matrices: task-ization, tile cache, inbound
tile copies, MFMA tile kernels, write-back -- the whole hot path; the call returns when C is back
in host memory.  Page-locking time is excluded, as in the paper.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps 3] [--warmup 1] [--n 32768] [--tile 1024] [--streams 4]
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

FP64_MFMA_PEAK_TFLOPS = 78.6     # MI355X dense FP64 matrix peak (published)


def cpu_baseline(np, oracle, A, B, n, rows=2048, cols=8192):
    """The oracle, as it stands, on a bounded sample of the same workload: a rows x cols block of the
    output, full inner dimension (2*rows*cols*n flop)."""
    rows, cols = min(rows, n), min(cols, n)
    a = A[:rows, :]          # views: the oracle takes the leading dimension from the strides
    b = B[:, :cols]
    c = np.zeros((rows, cols), order="F")
    t0 = time.perf_counter()
    oracle.gemm(oracle.ColMajor, oracle.NoTrans, oracle.NoTrans, 1.0, a, b, 0.0, c)
    dt = time.perf_counter() - t0
    return {
        "value": round(2.0 * rows * cols * n / dt / 1e9, 3), "unit": "GFLOP/s", "cores": oracle.threads(),
        "kind": "oracle", "seconds": round(dt, 2),
        "sample": "naive triple-loop DGEMM oracle on a %dx%d block of C with K=%d (%.1f GFLOP), all host cores"
                  % (rows, cols, n, 2.0 * rows * cols * n / 1e9),
    }


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--n", type=int, default=32768)
    ap.add_argument("--tile", type=int, default=1024)
    ap.add_argument("--streams", type=int, default=4)
    ap.add_argument("--group", type=int, default=None)
    ap.add_argument("--kchain", type=int, default=None)
    ap.add_argument("--depth", type=int, default=None)
    ap.add_argument("--sb", type=int, nargs=2, default=None)
    ap.add_argument("--shells", type=int, default=None)
    ap.add_argument("--rs", type=int, default=None)
    ap.add_argument("--prefetch", type=int, default=None)
    ap.add_argument("--wide", type=int, default=None, help="least k-steps per task for which all tasks advance together when the cache has room (default 11); 0: grouped")
    ap.add_argument("--arena-gb", type=float, default=None)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--check", action="store_true", help="also compare sampled outputs with the oracle")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="instead of the benchmark, run plain device copies of a known size (1 GiB read + 1 GiB written "
                         "per dispatch) so that HBM byte counters can be scaled")
    args = ap.parse_args()

    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build is single-GPU (one MI355X per box); run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import synth
    from paper_1510_05041_amd import blasx

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP library cannot run", file=sys.stderr)
        sys.exit(3)
    torch.cuda.set_device(0)
    if args.copy_calibration:
        src = torch.ones(2 ** 27, dtype=torch.float64, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(4):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_calibration": {"bytes_read_per_dispatch": 2 ** 30, "bytes_written_per_dispatch": 2 ** 30,
                                               "dispatches": 4}}))
        return
    lib = blasx.default()                      # raises if libblasx.so is not built

    n, T = args.n, args.tile
    # the largest configured size that the host can page-lock next to everything else
    import psutil
    need = 3 * 8 * n * n
    avail = psutil.virtual_memory().available
    while need > 0.8 * avail and n > 4096:
        n //= 2
        need = 3 * 8 * n * n
    tile_bytes = T * T * 8
    arena = int(args.arena_gb * 2 ** 30) if args.arena_gb else 3 * 8 * n * n + 512 * tile_bytes
    lib.init(arena, nstreams=args.streams)
    lib.set_tile(T)
    lib.set_cache_bytes(0)
    for name, val in (("group", args.group), ("kchain", args.kchain), ("depth", args.depth), ("shells", args.shells),
                      ("rs", args.rs), ("wide", args.wide), ("prefetch", args.prefetch)):
        if val is not None:
            lib.set_option(name, val)
    if args.sb:
        lib.set_option("sb_rows", args.sb[0])
        lib.set_option("sb_cols", args.sb[1])
    lib.set_option("profile", 1)

    t0 = time.perf_counter()
    A, ka = blasx.pinned_matrix(n, n)
    B, kb = blasx.pinned_matrix(n, n)
    C, kc = blasx.pinned_matrix(n, n)
    t_pin = time.perf_counter() - t0
    t0 = time.perf_counter()
    synth.fill(A, 0, synth.MAT_A)
    synth.fill(B, 0, synth.MAT_B)
    synth.fill(C, 0, synth.MAT_C)
    t_fill = time.perf_counter() - t0

    def step():
        lib.dgemm(blasx.ColMajor, blasx.NoTrans, blasx.NoTrans, n, n, n, 1.0, A, n, B, n, 1.0, C, n)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    lib.reset_stats()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    st = lib.get_stats()

    flop_step = 2.0 * n * n * n
    gflops = flop_step * args.steps / dt / 1e9
    launches = max(1, st["profiled_launches"])
    avg_launch_s = st["t_kernel_s"] / launches
    flop_per_launch = st["flops"] / max(1, st["launches"])
    achieved = flop_per_launch / avg_launch_s / 1e12 if avg_launch_s > 0 else 0.0

    # HBM bytes per launch from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this very command, scaled by the
    # same counters on a plain 1 GiB device copy (profiles/tile_steps_f64_nn_dgemm32768_hbm_traffic.md); they are
    # a property of the launch shape, so they are only quoted for the shape they were measured on.
    traffic = None
    shape = (n, T, lib.get_option("last_group"), lib.get_option("last_kchain"), lib.get_option("last_wide"), lib.get_option("last_ramp"))
    if shape == (32768, 1024, 16, 8, 1, 2):
        # means over the 320 launches of a call (rounds of 2, 6, 8, 8 and 8 k-tiles)
        traffic = {"hbm_bytes_per_launch": 2.839e9, "read": 2.704e9, "write": 0.1345e9, "algorithmic": 1.986e9,
                   "source": "profiles/tile_steps_f64_nn_dgemm32768_hbm_traffic.md"}
    out = {
        "metric": "host-resident DGEMM GFLOP/s on 1 MI355X", "value": round(gflops, 1), "unit": "GFLOP/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(dt / args.steps * 1e3, 2),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f64", "data": "synthetic",
        "pct_of_fp64_mfma_peak": round(100.0 * gflops / 1e3 / FP64_MFMA_PEAK_TFLOPS, 2),
        "config": {
            "workload": "DGEMM NoTrans/NoTrans M=N=K=%d fp64 column-major page-locked host matrices, uniform[-1,1] seed 0, "
                        "alpha=1 beta=1, tile %d, %d streams; timed region = library call entry to return "
                        "(inbound tile copies, kernels, write-back)" % (n, T, args.streams),
            "n": n, "tile": T, "streams": args.streams, "group": lib.get_option("last_group"), "kchain": lib.get_option("last_kchain"),
            "depth": lib.get_option("depth"), "superblock": [lib.get_option("sb_rows"), lib.get_option("sb_cols")],
            "shells": lib.get_option("shells"), "wide": lib.get_option("last_wide"), "first_round": lib.get_option("last_ramp"),
            "arena_bytes": arena,
        },
        "roofline": {
            "bound": "mfma", "achieved": round(achieved, 2), "peak": FP64_MFMA_PEAK_TFLOPS, "unit": "TFLOP/s",
            "frac": round(achieved / FP64_MFMA_PEAK_TFLOPS, 4), "traffic": traffic,
            "kernel": "tile_steps_kernel<double,NN,fast>", "launches": st["launches"],
            "flop_per_launch": flop_per_launch, "avg_launch_ms": round(avg_launch_s * 1e3, 4),
        },
        "link": {
            "h2d_GBps": round(st["bytes_h2d"] / dt / 1e9, 2), "d2h_GBps": round(st["bytes_d2h"] / dt / 1e9, 2),
            "bytes_h2d_per_step": st["bytes_h2d"] // args.steps, "bytes_d2h_per_step": st["bytes_d2h"] // args.steps,
        },
        "cache": {k: st[k] for k in ("hits", "misses", "evictions", "refetches", "peak_slots", "slot_waits")},
        "host": {"pin_seconds": round(t_pin, 2), "fill_seconds": round(t_fill, 2),
                 "issue_fraction": round(st["t_issue_s"] / max(st["t_total_s"], 1e-9), 3),
                 "kernel_busy_fraction": round(st["t_kernel_s"] / dt, 3)},
    }
    if args.check:
        import oracle
        rng = np.random.default_rng(1)
        worst = 0.0
        ntile = -(-n // T)
        for (ti, tj) in synth.sample_tiles(ntile, ntile, 16, 1):
            gi = ti * T + rng.integers(0, min(T, n - ti * T), 6)
            gj = tj * T + rng.integers(0, min(T, n - tj * T), 6)
            a = np.asfortranarray(A[gi, :])
            b = np.asfortranarray(B[:, gj])
            c0 = np.array([[synth.element(0, synth.MAT_C, int(i), int(j), n) for j in gj] for i in gi], order="F")
            want = np.zeros_like(c0, order="F")
            oracle.gemm(oracle.ColMajor, oracle.NoTrans, oracle.NoTrans, float(args.steps + args.warmup), a, b, 0.0, want)
            want += c0
            got = np.asarray(C)[np.ix_(gi, gj)]
            worst = max(worst, float(np.linalg.norm(got - want) / np.linalg.norm(want)))
        out["check"] = {"sampled_tiles": 16, "worst_normwise_rel_err": worst, "gate": 1e-13}
    if not args.no_cpu_baseline:
        import oracle
        out["cpu_baseline"] = cpu_baseline(np, oracle, A, B, n)
    lib.shutdown()
    print(json.dumps(out))


if __name__ == "__main__":
    main()
