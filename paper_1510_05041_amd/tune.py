"""Tile-size / stream-count sweep on the installed GPU (paper Section V.B: the tile size is the
one tuning parameter, and Section IV.D: the number of streams).

    python -m paper_1510_05041_amd.tune --routine dgemm --sizes 4096,8192,16384 --tiles 256,512,1024,2048

For every problem size the host matrices are page-locked once; every (tile, streams, group)
combination is then timed end to end (call entry to return, best of --reps calls after one
warm-up call) and one table per stream count is printed: rows = N, columns = T, entries =
TFLOP/s, with the best tile per row marked.  A tile or group of 0 means the library's automatic
choice (blasx_set_tile(0), option "group" = 0); the measurements behind those choices were taken
with this tool.
"""
import argparse
import json
import time

import numpy as np

from . import blasx

ROUTINES = ("dgemm", "sgemm", "dsyrk", "ssyrk", "dsyr2k", "ssyr2k", "dtrsm", "strsm", "dtrmm", "strmm", "dsymm", "ssymm")


def _fill(a, seed):
    """uniform[-1, 1) values; one random block of columns repeated (only the timing matters here)."""
    rng = np.random.default_rng(seed)
    w = min(a.shape[1], 128)
    blk = rng.uniform(-1.0, 1.0, (a.shape[0], w)).astype(a.dtype)
    for c in range(0, a.shape[1], w):
        a[:, c:c + w] = blk[:, :min(w, a.shape[1] - c)]


def _problem(lib, routine, n, k):
    """Returns (call, flop, refresh, owners) for one problem size; matrices are page-locked."""
    dt = np.float32 if routine[0] == "s" else np.float64
    CM, NT = blasx.ColMajor, blasx.NoTrans
    owners = []

    def mat(r, c, seed):
        a, own = blasx.pinned_matrix(r, c, dtype=dt)
        _fill(a, seed)
        owners.append(own)
        return a

    kind = routine[1:]
    if kind == "gemm":
        A, B, C = mat(n, k, 1), mat(k, n, 2), mat(n, n, 3)
        f = getattr(lib, routine)
        return (lambda: f(CM, NT, NT, n, n, k, 1.0, A, n, B, k, 1.0, C, n)), 2.0 * n * n * k, None, owners
    if kind == "syrk":
        A, C = mat(n, k, 1), mat(n, n, 3)
        f = getattr(lib, routine)
        return (lambda: f(CM, blasx.Lower, NT, n, k, 1.0, A, n, 1.0, C, n)), 1.0 * n * (n + 1) * k, None, owners
    if kind == "syr2k":
        A, B, C = mat(n, k, 1), mat(n, k, 2), mat(n, n, 3)
        f = getattr(lib, routine)
        return (lambda: f(CM, blasx.Lower, NT, n, k, 1.0, A, n, B, n, 1.0, C, n)), 2.0 * n * (n + 1) * k, None, owners
    if kind == "symm":
        A, B, C = mat(n, n, 1), mat(n, n, 2), mat(n, n, 3)
        f = getattr(lib, routine)
        return (lambda: f(CM, blasx.Left, blasx.Lower, n, n, 1.0, A, n, B, n, 1.0, C, n)), 2.0 * n * n * n, None, owners
    if kind == "trmm":
        A, B = mat(n, n, 1), mat(n, n, 2)
        A *= 1.0 / n                                  # keeps repeated in-place products bounded
        f = getattr(lib, routine)
        return (lambda: f(CM, blasx.Left, blasx.Lower, NT, blasx.NonUnit, n, n, 1.0, A, n, B, n)), 1.0 * n * n * n, None, owners
    if kind == "trsm":
        A, B = mat(n, n, 1), mat(n, n, 2)
        A[np.diag_indices(n)] = n + 0.5
        B0 = np.array(B[:, :1])

        def refresh():              # keep the right-hand sides bounded over repeated in-place solves
            B[...] = B0
        f = getattr(lib, routine)
        return (lambda: f(CM, blasx.Left, blasx.Lower, NT, blasx.NonUnit, n, n, 1.0, A, n, B, n)), 1.0 * n * n * n, refresh, owners
    raise ValueError(routine)


def sweep(routine, sizes, tiles, streams, groups, kdim, reps, arena_gb, out=None, wide=11, kchain=0, ramp=0, warmup_s=2.0, merge=0, order=(4, 4, 1), late_c=1):
    lib = blasx.default()
    results = []
    warm = False
    for n in sizes:
        k = kdim or n
        call, flop, refresh, owners = _problem(lib, routine, n, k)
        if not warm:
            # While the driver clears device memory that was freed just before (by the process that ran before this
            # one, say), outbound copies run at half rate: 1.5 s for 48 GiB.  Keep those calls out of the table.
            lib.init(int(arena_gb * 2 ** 30), nstreams=streams[0])
            lib.set_tile(0)
            t_end = time.perf_counter() + warmup_s
            while time.perf_counter() < t_end:
                if refresh:
                    refresh()
                call()
            warm = True
        for ns in streams:
            for T in tiles:
                for g in groups:
                    lib.init(int(arena_gb * 2 ** 30), nstreams=ns)
                    lib.set_tile(T)
                    lib.set_cache_bytes(0)
                    for name, v in dict(group=g, rs=max(32, 2 * g), kchain=kchain, depth=6, sb_rows=order[0], sb_cols=order[1], shells=order[2],
                                        profile=0, persist=0, wide=wide).items():
                        lib.set_option(name, v)
                    lib.set_option("ramp", ramp)
                    lib.set_option("merge", merge)
                    lib.set_option("late_c", late_c)
                    times = []
                    for rep in range(reps + 1):
                        if refresh:
                            refresh()
                        t0 = time.perf_counter()
                        call()
                        times.append(time.perf_counter() - t0)
                    best = min(times[1:])
                    rec = dict(routine=routine, n=n, k=k, T=T, streams=ns, group=g, ms=best * 1e3,
                               tflops=flop / best / 1e12)
                    rec["wide"] = lib.get_option("last_wide")
                    if T == 0 or g == 0:      # automatic choices: say what was chosen
                        rec["chosen_T"], rec["chosen_group"] = lib.get_option("last_tile"), lib.get_option("last_group")
                    results.append(rec)
                    print(json.dumps(rec), flush=True)
                    if out:
                        out.write(json.dumps(rec) + "\n")
                        out.flush()
        del call, owners
    lib.shutdown()
    return results


def tables(results, tiles, streams):
    lines = []
    for ns in streams:
        lines.append("streams = %d (best group per cell); TFLOP/s end to end, * = best tile of the row" % ns)
        lines.append("| N | " + " | ".join("T=%d" % t for t in tiles) + " |")
        lines.append("|---|" + "---|" * len(tiles))
        for n in sorted({r["n"] for r in results}):
            cells = []
            for T in tiles:
                c = [r for r in results if r["n"] == n and r["T"] == T and r["streams"] == ns]
                cells.append(max(c, key=lambda r: r["tflops"]) if c else None)
            top = max((c["tflops"] for c in cells if c), default=0.0)
            lines.append("| %d | " % n + " | ".join(
                "-" if c is None else "%.1f (g%d)%s" % (c["tflops"], c["group"], "*" if c["tflops"] == top else "")
                for c in cells) + " |")
        lines.append("")
    return "\n".join(lines)


def main(argv=None):
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("--routine", default="dgemm", choices=ROUTINES)
    ap.add_argument("--sizes", default="2048,4096,8192,16384")
    ap.add_argument("--k", type=int, default=0, help="inner dimension (default: same as N)")
    ap.add_argument("--tiles", default="256,512,1024,2048")
    ap.add_argument("--streams", default="4")
    ap.add_argument("--groups", default="16")
    ap.add_argument("--reps", type=int, default=3)
    ap.add_argument("--arena-gb", type=float, default=24.0)
    ap.add_argument("--wide", type=int, default=11, help="option \"wide\": least k-steps per task for which all tasks advance together; 0: never")
    ap.add_argument("--kchain", type=int, default=0, help="option \"kchain\": k-tiles per launch and task; 0: the library's choice")
    ap.add_argument("--ramp", type=int, default=0, help="option \"ramp\": k-steps per task in the first round of the wide schedule (8: as in the others); 0: the library's choice")
    ap.add_argument("--merge", type=int, default=0, help="option \"merge\": most neighbouring tiles per inbound copy (1: one copy per tile; 0: the library's choice)")
    ap.add_argument("--late-c", type=int, default=1, help="option \"late_c\": grouped schedule with room for every tile fetches C for a task's last launch only")
    ap.add_argument("--order", default="4,4,1", help="options sb_rows,sb_cols,shells: super-block shape of the task queue and whether super-blocks are visited in growing shells (1) or block row by block row (0)")
    ap.add_argument("--warmup-s", type=float, default=2.0, help="seconds of untimed calls of the first problem before anything is timed")
    ap.add_argument("--out", default="", help="also append the JSON records to this file")
    a = ap.parse_args(argv)
    ints = lambda s: [int(x) for x in s.split(",") if x]
    sizes, tiles, streams, groups = ints(a.sizes), ints(a.tiles), ints(a.streams), ints(a.groups)
    out = open(a.out, "a") if a.out else None
    res = sweep(a.routine, sizes, tiles, streams, groups, a.k, a.reps, a.arena_gb, out, a.wide, a.kchain, a.ramp, a.warmup_s, a.merge, tuple(ints(a.order)), a.late_c)
    print()
    print(tables(res, tiles, streams))


if __name__ == "__main__":
    main()
