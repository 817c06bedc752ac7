"""Host logic without a GPU: task builder, ALRU cache and scheduler, linked against the
host-only device double in tests/sim (lazy, randomly interleaved execution that honours only
stream order and event waits).  Results are compared with the oracle; counters are compared
with what the method fixes (bytes moved when everything fits, reuse under a capped cache).
"""
import itertools
import os

import numpy as np
import pytest

import oracle as ref
import synth
from paper_1510_05041_amd import _build, blasx

ORDERS = [blasx.ColMajor, blasx.RowMajor]
TRANS = [blasx.NoTrans, blasx.Trans]


@pytest.fixture(scope="module")
def sim():
    lib = blasx.Library(_build.build_sim())
    lib._lib.blasx_sim_seed.argtypes = [__import__("ctypes").c_uint64]
    yield lib
    lib.shutdown()


def setup(sim, T, nstreams=4, arena_tiles=64, cap_tiles=0, seed=1, esize=8, **opts):
    sim._lib.blasx_sim_seed(seed)
    sim.init_raw(arena_tiles * T * T * esize, nstreams)
    sim.set_tile(T)
    sim.set_cache_bytes(cap_tiles * T * T * esize)
    defaults = dict(group=4, kchain=2, depth=3, rs=8, sb_rows=2, sb_cols=2, shells=1, priority=1, profile=0, persist=0, wide=0, ramp=0,
                    merge=4, late_c=1, row_order=1, tail_cut=0, stagger_panels=2, stagger_lag=3)
    defaults.update(opts)
    for k, v in defaults.items():
        sim.set_option(k, v)
    sim.reset_stats()


def store(logical, order, pad=0, dtype=np.float64):
    r, c = logical.shape
    if order == blasx.ColMajor:
        buf = np.full((r + pad, c), np.nan, dtype=dtype, order="F")
    else:
        buf = np.full((r, c + pad), np.nan, dtype=dtype, order="C")
    v = buf[:r, :c]
    v[...] = logical
    return v


def ld_of(a, order):
    it = a.itemsize
    if order == blasx.ColMajor:
        return max(1, a.strides[1] // it if a.shape[1] > 1 else a.shape[0])
    return max(1, a.strides[0] // it if a.shape[0] > 1 else a.shape[1])


def relerr(got, want):
    return np.linalg.norm(np.asarray(got, dtype=np.float64) - want) / max(np.linalg.norm(want), 1e-300)


# ------------------------------------------------------------------ GEMM ----------

@pytest.mark.parametrize("order", ORDERS)
@pytest.mark.parametrize("ta,tb", list(itertools.product(TRANS, TRANS)))
@pytest.mark.parametrize("M,N,K", [(48, 48, 48), (37, 53, 41), (16, 80, 5), (1, 1, 1)])
def test_gemm_matches_oracle(sim, order, ta, tb, M, N, K):
    setup(sim, T=16, seed=M + N + K + ta + tb + order)
    rng = np.random.default_rng(7)
    A = rng.uniform(-1, 1, (M, K) if ta == blasx.NoTrans else (K, M))
    B = rng.uniform(-1, 1, (K, N) if tb == blasx.NoTrans else (N, K))
    C = rng.uniform(-1, 1, (M, N))
    As, Bs, Cs, Cr = store(A, order, 3), store(B, order, 1), store(C, order, 2), store(C, order, 2)
    sim.dgemm(order, ta, tb, M, N, K, 0.75, As, ld_of(As, order), Bs, ld_of(Bs, order), -0.5, Cs, ld_of(Cs, order))
    ref.gemm(order, ta, tb, 0.75, As, Bs, -0.5, Cr)
    assert relerr(Cs, np.asarray(Cr)) < 1e-14
    st = sim.get_stats()
    nt = lambda x: -(-x // 16)
    assert st["tasks"] == nt(M) * nt(N)                       # one task per output tile (Section IV.A)
    assert st["tile_steps"] == nt(M) * nt(N) * nt(K)
    assert st["bytes_d2h"] == 8 * M * N
    # everything fits: every tile of A, B and C crosses the link exactly once
    assert st["bytes_h2d"] == 8 * (M * K + K * N + M * N)
    assert st["evictions"] == 0 and st["refetches"] == 0


def test_gemm_integer_inputs_are_bit_exact_across_tilings(sim):
    M, N, K = 70, 45, 90
    A = synth.matrix(M, K, 3, 0, integers=True)
    B = synth.matrix(K, N, 3, 1, integers=True)
    C = synth.matrix(M, N, 3, 2, integers=True)
    want = 2.0 * (np.asarray(A) @ np.asarray(B)) - np.asarray(C)
    for T, kchain, group in [(16, 1, 1), (16, 4, 7), (32, 3, 4), (48, 2, 2), (128, 1, 4)]:
        setup(sim, T=T, kchain=kchain, group=group, seed=T + kchain)
        Cs = C.copy(order="F")
        sim.dgemm(blasx.ColMajor, blasx.NoTrans, blasx.NoTrans, M, N, K, 2.0, A, M, B, K, -1.0, Cs, M)
        assert np.array_equal(Cs, want), (T, kchain, group)


def test_gemm_beta_zero_never_reads_c_and_alpha_zero_never_reads_ab(sim):
    setup(sim, T=16)
    rng = np.random.default_rng(1)
    M, N, K = 40, 24, 33
    A, B = np.asfortranarray(rng.uniform(-1, 1, (M, K))), np.asfortranarray(rng.uniform(-1, 1, (K, N)))
    Cs = np.full((M, N), np.nan, order="F")
    sim.dgemm(blasx.ColMajor, blasx.NoTrans, blasx.NoTrans, M, N, K, 1.0, A, M, B, K, 0.0, Cs, M)
    assert relerr(Cs, A @ B) < 1e-14
    assert sim.get_stats()["bytes_h2d"] == 8 * (M * K + K * N)         # C was not fetched
    C = np.asfortranarray(rng.uniform(-1, 1, (M, N)))
    Cs = C.copy(order="F")
    nan = np.full((64, 64), np.nan, order="F")
    sim.reset_stats()
    sim.dgemm(blasx.ColMajor, blasx.NoTrans, blasx.NoTrans, M, N, K, 0.0, nan, 64, nan, 64, 0.5, Cs, M)
    assert np.array_equal(Cs, 0.5 * C)
    assert sim.get_stats()["bytes_h2d"] == 8 * M * N
    Cs = np.full((M, N), np.nan, order="F")
    sim.dgemm(blasx.ColMajor, blasx.NoTrans, blasx.NoTrans, M, N, K, 0.0, nan, 64, nan, 64, 0.0, Cs, M)
    assert np.array_equal(Cs, np.zeros((M, N)))
    # quick returns leave C alone and need no device
    Cs = C.copy(order="F")
    sim.dgemm(blasx.ColMajor, blasx.NoTrans, blasx.NoTrans, M, N, 0, 1.0, A, M, B, 1, 1.0, Cs, M)
    sim.dgemm(blasx.ColMajor, blasx.NoTrans, blasx.NoTrans, M, N, K, 0.0, A, M, B, K, 1.0, Cs, M)
    sim.dgemm(blasx.ColMajor, blasx.NoTrans, blasx.NoTrans, 0, N, K, 1.0, A, M, B, K, 0.0, Cs, M)
    assert np.array_equal(Cs, C)


def test_sgemm_matches_oracle(sim):
    setup(sim, T=32, esize=4)
    rng = np.random.default_rng(2)
    M, N, K = 75, 66, 100
    A = np.asfortranarray(rng.uniform(-1, 1, (M, K)).astype(np.float32))
    B = np.asfortranarray(rng.uniform(-1, 1, (N, K)).astype(np.float32))
    C = np.asfortranarray(rng.uniform(-1, 1, (M, N)).astype(np.float32))
    Cs, Cr = C.copy(order="F"), C.copy(order="F")
    sim.sgemm(blasx.ColMajor, blasx.NoTrans, blasx.Trans, M, N, K, 1.0, A, M, B, N, 1.0, Cs, M)
    ref.gemm(ref.ColMajor, ref.NoTrans, ref.Trans, 1.0, A, B, 1.0, Cr)
    assert relerr(Cs, Cr.astype(np.float64)) < 1e-6


@pytest.mark.parametrize("seed", range(6))
def test_gemm_capped_cache_evicts_and_stays_correct(sim, seed):
    """Out-of-core case in miniature: 12x12x12 tiles through a 20-slot cache."""
    T, n = 16, 12 * 16
    setup(sim, T=T, arena_tiles=64, cap_tiles=20, seed=100 + seed, group=4, kchain=2, depth=2 + seed % 3,
          nstreams=2 + seed % 3)
    A = synth.matrix(n, n, seed, 0)
    B = synth.matrix(n, n, seed, 1)
    C = synth.matrix(n, n, seed, 2)
    Cs, Cr = C.copy(order="F"), C.copy(order="F")
    sim.dgemm(blasx.ColMajor, blasx.NoTrans, blasx.NoTrans, n, n, n, 1.0, A, n, B, n, 0.0, Cs, n)
    ref.gemm(ref.ColMajor, ref.NoTrans, ref.NoTrans, 1.0, A, B, 0.0, Cr)
    assert relerr(Cs, Cr) < 1e-14
    st = sim.get_stats()
    assert st["peak_slots"] <= 20
    assert st["evictions"] > 0 and st["refetches"] > 0
    distinct = 2 * 12 * 12                                   # tiles of A and B
    assert st["misses"] == distinct + st["refetches"]
    assert st["hits"] + st["misses"] >= 2 * 12 ** 3           # two translations per tile step (+ retries)
    assert not sim._lib.blasx_sim_deadlocked()


def test_arena_too_small_is_an_error_not_a_hang(sim):
    setup(sim, T=16, arena_tiles=3)
    A = synth.matrix(64, 64, 0, 0)
    C = np.zeros((64, 64), order="F")
    rc = sim.dgemm(blasx.ColMajor, blasx.NoTrans, blasx.NoTrans, 64, 64, 64, 1.0, A, 64, A, 64, 0.0, C, 64, check=False)
    assert rc == 2


def test_argument_errors_follow_the_prototype_positions(sim):
    setup(sim, T=16)
    a = np.zeros((8, 8), order="F")
    g = lambda *args: sim.dgemm(*args, check=False)
    CM, NT = blasx.ColMajor, blasx.NoTrans
    assert g(7, NT, NT, 8, 8, 8, 1.0, a, 8, a, 8, 0.0, a, 8) == -1
    assert g(CM, 5, NT, 8, 8, 8, 1.0, a, 8, a, 8, 0.0, a, 8) == -2
    assert g(CM, NT, 5, 8, 8, 8, 1.0, a, 8, a, 8, 0.0, a, 8) == -3
    assert g(CM, NT, NT, -1, 8, 8, 1.0, a, 8, a, 8, 0.0, a, 8) == -4
    assert g(CM, NT, NT, 8, -1, 8, 1.0, a, 8, a, 8, 0.0, a, 8) == -5
    assert g(CM, NT, NT, 8, 8, -1, 1.0, a, 8, a, 8, 0.0, a, 8) == -6
    assert g(CM, NT, NT, 8, 8, 8, 1.0, a, 7, a, 8, 0.0, a, 8) == -9
    assert g(CM, NT, NT, 8, 8, 8, 1.0, a, 8, a, 7, 0.0, a, 8) == -11
    assert g(CM, NT, NT, 8, 8, 8, 1.0, a, 8, a, 8, 0.0, a, 7) == -14
    assert sim.dsyrk(CM, 0, NT, 8, 8, 1.0, a, 8, 0.0, a, 8, check=False) == -2
    assert sim.dtrsm(CM, blasx.Left, blasx.Lower, NT, 0, 8, 8, 1.0, a, 8, a, 8, check=False) == -5
    assert sim.dtrmm(CM, blasx.Left, blasx.Lower, NT, blasx.Unit, 8, 8, 1.0, a, 4, a, 8, check=False) == -10
    k2 = lambda *args: sim.dsyr2k(*args, check=False)
    UP = blasx.Upper
    assert k2(CM, 0, NT, 8, 8, 1.0, a, 8, a, 8, 0.0, a, 8) == -2
    assert k2(CM, UP, NT, 8, 8, 1.0, a, 7, a, 8, 0.0, a, 8) == -8
    assert k2(CM, UP, NT, 8, 8, 1.0, a, 8, a, 7, 0.0, a, 8) == -10
    assert k2(CM, UP, NT, 8, 8, 1.0, a, 8, a, 8, 0.0, a, 7) == -13
    sm = lambda *args: sim.dsymm(*args, check=False)
    assert sm(CM, 0, UP, 8, 8, 1.0, a, 8, a, 8, 0.0, a, 8) == -2
    assert sm(CM, blasx.Left, 0, 8, 8, 1.0, a, 8, a, 8, 0.0, a, 8) == -3
    assert sm(CM, blasx.Left, UP, 8, -2, 1.0, a, 8, a, 8, 0.0, a, 8) == -5
    assert sm(CM, blasx.Right, UP, 4, 8, 1.0, a, 7, a, 8, 0.0, a, 8) == -8
    assert sm(CM, blasx.Left, UP, 8, 8, 1.0, a, 8, a, 7, 0.0, a, 8) == -10
    assert sm(CM, blasx.Left, UP, 8, 8, 1.0, a, 8, a, 8, 0.0, a, 7) == -13
    assert sim.set_option.__self__._lib.blasx_set_tile(20) == 4


def test_set_streams_changes_the_stream_count_between_calls_and_keeps_results(sim):
    """Section IV.D: tasks progress on concurrent streams.  blasx_set_streams re-roles the streams
    of the current initialisation; every count gives the same (integer-exact) product."""
    setup(sim, T=16, nstreams=4, group=3)
    rng = np.random.default_rng(12)
    A = np.asfortranarray(rng.integers(-2, 3, (70, 50)).astype(np.float64))
    B = np.asfortranarray(rng.integers(-2, 3, (50, 60)).astype(np.float64))
    assert sim.get_option("streams") == 4
    for n in (2, 3, 4, 0, 2):
        sim.set_streams(n)
        assert sim.get_option("streams") == (n or 4)
        C = np.full((70, 60), np.nan, order="F")
        sim.dgemm(blasx.ColMajor, blasx.NoTrans, blasx.NoTrans, 70, 60, 50, 1.0, A, 70, B, 50, 0.0, C, 70)
        assert np.array_equal(C, A @ B)
    assert sim._lib.blasx_set_streams(1) == 4 and sim._lib.blasx_set_streams(5) == 4      # BLASX_ERR_CONFIG
    assert sim.get_option("streams") == 2
    sim.shutdown()
    assert sim._lib.blasx_set_streams(4) == 1                                             # BLASX_ERR_NOT_INITIALIZED


def test_host_time_is_split_into_issuing_and_waiting_and_the_device_time_is_dissected(sim):
    """t_total = t_issue + t_wait; with "profile" = 2 the call is dissected as in the paper's time
    profile (Section V.A): kernels (COMPT), copies under no kernel (COMM), and the rest of the span."""
    n = 96
    A, B = synth.matrix(n, n, 3, 0), synth.matrix(n, n, 3, 1)
    for profile in (0, 1, 2):
        setup(sim, T=16, group=4, kchain=2, profile=profile, seed=5 + profile, arena_tiles=128)
        C = np.zeros((n, n), order="F")
        sim.dgemm(blasx.ColMajor, blasx.NoTrans, blasx.NoTrans, n, n, n, 1.0, A, n, B, n, 0.0, C, n)
        st = sim.get_stats()
        assert st["t_wait_s"] >= 0 and st["t_issue_s"] >= 0
        assert abs(st["t_total_s"] - st["t_issue_s"] - st["t_wait_s"]) < 1e-9
        assert st["profiled_launches"] == (st["launches"] if profile else 0)
        if profile < 2:
            assert st["t_kernel_busy_s"] == 0 and st["t_copy_unoverlapped_s"] == 0 and st["t_device_span_s"] == 0
        else:
            # the double's clock: 5 us per launch, 2 us per tile copy, one operation at a time (an
            # interval between two events of one stream also covers what other streams ran meanwhile)
            busy, comm, span = st["t_kernel_busy_s"], st["t_copy_unoverlapped_s"], st["t_device_span_s"]
            assert busy >= st["launches"] * 5e-6 - 1e-12
            assert comm > 0 and busy + comm <= span + 1e-12
            ncopies = st["copies_h2d"] + st["copies_d2h"]
            assert ncopies == 36 * 2 + 36 and span <= st["launches"] * 5e-6 + ncopies * 2e-6 + 1e-12
    sim.set_option("profile", 0)


def test_noalloc_entry_point_host_logic(sim):
    """blasx_dgemm_noalloc on the host-only double (its static arena is 8 MiB): same results as blasx_dgemm, two calls in
    a row with the second smaller, sizes beyond the slot count refused with their own code before anything is written."""
    setup(sim, T=16, group=0, kchain=0, wide=11)
    rng = np.random.default_rng(70)
    for (M, N, K, ta, tb) in ((150, 90, 200, blasx.Trans, blasx.NoTrans), (40, 70, 33, blasx.NoTrans, blasx.Trans)):
        A = np.asfortranarray(rng.integers(-2, 3, (M, K) if ta == blasx.NoTrans else (K, M)).astype(np.float64))
        B = np.asfortranarray(rng.integers(-2, 3, (K, N) if tb == blasx.NoTrans else (N, K)).astype(np.float64))
        C0 = np.asfortranarray(rng.integers(-2, 3, (M, N)).astype(np.float64))
        C1, C2 = C0.copy(order="F"), C0.copy(order="F")
        sim.dgemm_noalloc(blasx.ColMajor, ta, tb, M, N, K, 2.0, A, A.shape[0], B, B.shape[0], -1.0, C1, M)
        sim.dgemm(blasx.ColMajor, ta, tb, M, N, K, 2.0, A, A.shape[0], B, B.shape[0], -1.0, C2, M)
        assert np.array_equal(C1, C2)
        assert np.array_equal(C1, 2.0 * ((A if ta == blasx.NoTrans else A.T) @ (B if tb == blasx.NoTrans else B.T)) - C0)
    n = 1024                                    # 3 * 64 * 64 tiles of 16 x 16 against 4096 slots
    big = np.ones((n, n), order="F")
    out = np.full((n, n), 7.0, order="F")
    assert sim.dgemm_noalloc(blasx.ColMajor, blasx.NoTrans, blasx.NoTrans, n, n, n, 1.0, big, n, big, n, 0.0, out, n, check=False) == 7
    assert "too large" in sim.last_error() and np.all(out == 7.0)
    assert sim.strerror(7).startswith("problem too large")
    a = np.zeros((8, 8), order="F")
    assert sim.dgemm_noalloc(blasx.ColMajor, blasx.NoTrans, blasx.NoTrans, 8, 8, 8, 1.0, a, 7, a, 8, 0.0, a, 8, check=False) == -9
    sim.shutdown()
    assert sim.dgemm_noalloc(blasx.ColMajor, blasx.NoTrans, blasx.NoTrans, 8, 8, 8, 1.0, a, 8, a, 8, 0.0, a, 8, check=False) == 1


def start_order(sim, C, T):
    """Tile indices (i, j) of the output tiles in the order their tasks were started, read from the test double's
    trace of inbound copies: with beta != 0 a task's first device operation is the copy of its own tile of C."""
    import ctypes
    buf = (ctypes.c_void_p * 65536)()
    sim._lib.blasx_sim_trace_h2d.restype = ctypes.c_uint64
    n = sim._lib.blasx_sim_trace_h2d(buf, 65536)
    lo, ld = C.ctypes.data, C.strides[1] // 8
    out = []
    for q in range(n):
        off = (buf[q] or 0) - lo
        if 0 <= off < C.shape[1] * ld * 8:
            e = off // 8
            out.append((int(e % ld) // T, int(e // ld) // T))
    return out


def test_reservation_station_starts_the_task_with_most_cached_operands_and_ties_go_to_queue_order(sim):
    """Alg. 1 lines 10-15 and Eq. 2: the priority of a waiting task is 2 per operand tile already in the cache; the
    station hands out the highest priority first, equal ones in queue order.  A first call leaves block row r of A and
    block column c of B in the (persistent) cache; the second call must then start task (r, c), whose operands are all
    there, then the tasks of row r and column c in queue order, then the others in queue order.  With the priorities
    switched off the same call starts in queue order."""
    T, nt, nk, r, c = 16, 4, 3, 2, 3
    rng = np.random.default_rng(33)
    A = np.asfortranarray(rng.integers(-2, 3, (nt * T, nk * T)).astype(np.float64))
    B = np.asfortranarray(rng.integers(-2, 3, (nk * T, nt * T)).astype(np.float64))
    C0 = np.asfortranarray(rng.integers(-2, 3, (nt * T, nt * T)).astype(np.float64))
    n = nt * T
    orders, misses = {}, {}
    for prio in (0, 1):
        # the station holds every task of the call, so the priorities are worked out once, when the tasks come in
        setup(sim, T=T, arena_tiles=64, group=1, rs=64, kchain=1, persist=1, priority=prio, sb_rows=2, sb_cols=2)
        W = np.zeros((T, T), order="F")
        sim.dgemm(blasx.ColMajor, blasx.NoTrans, blasx.NoTrans, T, T, nk * T, 1.0, A[r * T:, :], n, B[:, c * T:], nk * T, 0.0, W, T)
        assert np.array_equal(W, A[r * T:(r + 1) * T, :] @ B[:, c * T:(c + 1) * T])
        assert sim.get_option("cached_tiles") == 2 * nk
        C = C0.copy(order="F")
        sim._lib.blasx_sim_trace_reset()
        sim.reset_stats()
        sim.dgemm(blasx.ColMajor, blasx.NoTrans, blasx.NoTrans, n, n, nk * T, 1.0, A, n, B, nk * T, 1.0, C, n)
        assert np.array_equal(C, A @ B + C0)
        orders[prio] = start_order(sim, C, T)
        misses[prio] = sim.get_stats()["misses"]
        assert len(orders[prio]) == nt * nt and len(set(orders[prio])) == nt * nt
        sim.set_option("persist", 0)
    queue = orders[0]
    priority = lambda ij: 2 * nk * (ij[0] == r) + 2 * nk * (ij[1] == c)
    expect = sorted(queue, key=lambda ij: -priority(ij))           # stable: ties keep queue order
    assert queue[0] != (r, c) and expect[0] == (r, c)
    assert orders[1] == expect
    # room for everything: each tile is fetched once whatever the order, the cached ones never
    assert misses[0] == misses[1] == 2 * nt * nk - 2 * nk
    sim.set_option("priority", 1)


@pytest.mark.parametrize("seed", range(4))
def test_priorities_save_tile_fetches_under_a_small_cache(sim, seed):
    """What Eq. 2 is for: with a cache of 12 tiles, one task running and a station of 4 (refreshed whenever a task
    comes in), the task started next is the one that finds most of its operands still cached, and an 8 x 8-tile
    product with 4 k-tiles fetches a third fewer tiles than in queue order -- for every interleaving of the device."""
    T, nt, nk = 16, 8, 4
    rng = np.random.default_rng(34)
    A = np.asfortranarray(rng.integers(-2, 3, (nt * T, nk * T)).astype(np.float64))
    B = np.asfortranarray(rng.integers(-2, 3, (nk * T, nt * T)).astype(np.float64))
    n = nt * T
    misses = {}
    for prio in (0, 1):
        setup(sim, T=T, arena_tiles=64, cap_tiles=12, group=1, rs=4, kchain=1, priority=prio, sb_rows=2, sb_cols=2, shells=0, seed=900 + seed)
        C = np.zeros((n, n), order="F")
        sim.dgemm(blasx.ColMajor, blasx.NoTrans, blasx.NoTrans, n, n, nk * T, 1.0, A, n, B, nk * T, 0.0, C, n)
        assert np.array_equal(C, A @ B)
        st = sim.get_stats()
        assert st["misses"] == 2 * nt * nk + st["refetches"]
        misses[prio] = st["misses"]
    assert misses[1] < 0.8 * misses[0], misses
    sim.set_option("priority", 1)
    sim.set_option("shells", 1)


# ------------------------------------------------------------------ SYRK ----------

@pytest.mark.parametrize("order", ORDERS)
@pytest.mark.parametrize("uplo", [blasx.Upper, blasx.Lower])
@pytest.mark.parametrize("trans", TRANS)
@pytest.mark.parametrize("beta", [0.0, 0.7])
def test_syrk_matches_oracle_and_leaves_other_triangle(sim, order, uplo, trans, beta):
    setup(sim, T=16, seed=uplo + trans + order)
    rng = np.random.default_rng(3)
    N, K = 57, 38
    A = rng.uniform(-1, 1, (N, K) if trans == blasx.NoTrans else (K, N))
    C = rng.uniform(-1, 1, (N, N))
    other = np.triu_indices(N, 1) if uplo == blasx.Lower else np.tril_indices(N, -1)
    C[other] = 777.125
    As, Cs, Cr = store(A, order, 1), store(C, order, 2), store(C, order, 2)
    sim.dsyrk(order, uplo, trans, N, K, 1.5, As, ld_of(As, order), beta, Cs, ld_of(Cs, order))
    ref.syrk(order, uplo, trans, 1.5, As, beta, Cr)
    assert np.all(np.asarray(Cs)[other] == 777.125)
    assert relerr(Cs, np.asarray(Cr)) < 1e-14
    nt = -(-N // 16)
    assert sim.get_stats()["tasks"] == nt * (nt + 1) // 2


# ------------------------------------------------------------------ SYR2K / SYMM ---

@pytest.mark.parametrize("order", ORDERS)
@pytest.mark.parametrize("uplo", [blasx.Upper, blasx.Lower])
@pytest.mark.parametrize("trans", TRANS)
@pytest.mark.parametrize("beta", [0.0, -0.4])
def test_syr2k_matches_oracle_and_leaves_other_triangle(sim, order, uplo, trans, beta):
    setup(sim, T=16, seed=3 * uplo + trans + order, group=4)
    rng = np.random.default_rng(8)
    N, K = 53, 41
    shape = (N, K) if trans == blasx.NoTrans else (K, N)
    A, B = rng.uniform(-1, 1, shape), rng.uniform(-1, 1, shape)
    C = rng.uniform(-1, 1, (N, N))
    other = np.triu_indices(N, 1) if uplo == blasx.Lower else np.tril_indices(N, -1)
    C[other] = -55.5
    As, Bs, Cs, Cr = store(A, order, 1), store(B, order, 3), store(C, order, 2), store(C, order, 2)
    sim.dsyr2k(order, uplo, trans, N, K, 0.75, As, ld_of(As, order), Bs, ld_of(Bs, order), beta, Cs, ld_of(Cs, order))
    ref.syr2k(order, uplo, trans, 0.75, As, Bs, beta, Cr)
    assert np.all(np.asarray(Cs)[other] == -55.5)
    assert relerr(Cs, np.asarray(Cr)) < 1e-14
    nt = -(-N // 16)
    st = sim.get_stats()
    assert st["tasks"] == nt * (nt + 1) // 2
    assert st["tile_steps"] == 2 * -(-K // 16) * st["tasks"]


@pytest.mark.parametrize("order", ORDERS)
@pytest.mark.parametrize("side", [blasx.Left, blasx.Right])
@pytest.mark.parametrize("uplo", [blasx.Upper, blasx.Lower])
@pytest.mark.parametrize("beta", [0.0, 1.25])
def test_symm_matches_oracle_and_never_reads_the_other_triangle(sim, order, side, uplo, beta):
    setup(sim, T=16, seed=side + uplo + order, group=6)
    rng = np.random.default_rng(9)
    M, N = 55, 38
    na = M if side == blasx.Left else N
    A = rng.uniform(-1, 1, (na, na))
    other = np.triu_indices(na, 1) if uplo == blasx.Lower else np.tril_indices(na, -1)
    A[other] = np.nan
    B, C = rng.uniform(-1, 1, (M, N)), rng.uniform(-1, 1, (M, N))
    As, Bs, Cs, Cr = store(A, order, 2), store(B, order, 1), store(C, order, 3), store(C, order, 3)
    sim.dsymm(order, side, uplo, M, N, -1.5, As, ld_of(As, order), Bs, ld_of(Bs, order), beta, Cs, ld_of(Cs, order))
    ref.symm(order, side, uplo, -1.5, As, Bs, beta, Cr)
    assert np.all(np.isfinite(np.asarray(Cs)))
    assert relerr(Cs, np.asarray(Cr)) < 1e-14
    st = sim.get_stats()
    assert st["tasks"] == -(-M // 16) * -(-N // 16)
    assert st["tile_steps"] == st["tasks"] * -(-na // 16)


@pytest.mark.parametrize("seed", range(8))
def test_symm_capped_cache_many_interleavings(sim, seed):
    """Derived tiles (completed diagonal tiles, transposed mirror tiles) are written by kernels on the compute stream:
    under slot pressure they are evicted and rebuilt while copies and launches interleave at random."""
    side, uplo = [(blasx.Left, blasx.Lower), (blasx.Right, blasx.Upper), (blasx.Left, blasx.Upper), (blasx.Right, blasx.Lower)][seed % 4]
    setup(sim, T=16, seed=100 + seed, arena_tiles=12 + seed, group=2 + seed % 3, kchain=1 + seed % 3)
    rng = np.random.default_rng(seed)
    M, N = 96, 80
    na = M if side == blasx.Left else N
    A = rng.integers(-2, 3, (na, na)).astype(np.float64)
    full = np.tril(A) + np.tril(A, -1).T if uplo == blasx.Lower else np.triu(A) + np.triu(A, 1).T
    B = rng.integers(-2, 3, (M, N)).astype(np.float64)
    As, Bs, Cs = store(A, blasx.ColMajor), store(B, blasx.ColMajor), store(np.zeros((M, N)), blasx.ColMajor)
    sim.dsymm(blasx.ColMajor, side, uplo, M, N, 1.0, As, na, Bs, M, 0.0, Cs, M)
    assert np.array_equal(np.asarray(Cs), full @ B if side == blasx.Left else B @ full)
    st = sim.get_stats()
    assert st["evictions"] > 0


def test_symm_under_slot_pressure_and_single_precision(sim):
    # few slots: symmetrised diagonal tiles get evicted and rebuilt
    setup(sim, T=16, seed=5, arena_tiles=14, group=3)
    rng = np.random.default_rng(10)
    M, N = 80, 64
    A = np.tril(rng.integers(-2, 3, (M, M)).astype(np.float64))
    B = rng.integers(-2, 3, (M, N)).astype(np.float64)
    C = np.zeros((M, N))
    As, Bs, Cs = store(A, blasx.ColMajor), store(B, blasx.ColMajor), store(C, blasx.ColMajor)
    sim.dsymm(blasx.ColMajor, blasx.Left, blasx.Lower, M, N, 1.0, As, M, Bs, M, 0.0, Cs, M)
    S = A + np.tril(A, -1).T
    assert np.array_equal(np.asarray(Cs), S @ B)          # small integers: exact in any order
    assert sim.get_stats()["evictions"] > 0

    setup(sim, T=32, seed=6, esize=4)
    A32 = rng.uniform(-1, 1, (N, N)).astype(np.float32)
    B32, C32 = rng.uniform(-1, 1, (M, N)).astype(np.float32), rng.uniform(-1, 1, (M, N)).astype(np.float32)
    As, Bs = store(A32, blasx.RowMajor, 1, np.float32), store(B32, blasx.RowMajor, 0, np.float32)
    Cs, Cr = store(C32, blasx.RowMajor, 2, np.float32), store(C32, blasx.RowMajor, 2, np.float32)
    sim.ssymm(blasx.RowMajor, blasx.Right, blasx.Upper, M, N, 0.5, As, ld_of(As, blasx.RowMajor), Bs, ld_of(Bs, blasx.RowMajor),
              2.0, Cs, ld_of(Cs, blasx.RowMajor))
    ref.symm(blasx.RowMajor, blasx.Right, blasx.Upper, 0.5, As, Bs, 2.0, Cr)
    assert relerr(Cs, np.asarray(Cr)) < 1e-6
    Cs, Cr = store(C32[:N, :N], blasx.ColMajor, 0, np.float32), store(C32[:N, :N], blasx.ColMajor, 0, np.float32)
    Ak = store(B32.T.copy(), blasx.ColMajor, 0, np.float32)   # N x M
    Bk = store(A32[:, :1].repeat(M, 1), blasx.ColMajor, 0, np.float32)
    sim.ssyr2k(blasx.ColMajor, blasx.Upper, blasx.NoTrans, N, M, 1.0, Ak, N, Bk, N, 1.0, Cs, N)
    ref.syr2k(blasx.ColMajor, blasx.Upper, blasx.NoTrans, 1.0, Ak, Bk, 1.0, Cr)
    assert relerr(Cs, np.asarray(Cr)) < 1e-6


# ------------------------------------------------------------------ TRMM / TRSM ---

FLAGS = list(itertools.product([blasx.Left, blasx.Right], [blasx.Upper, blasx.Lower], TRANS, [blasx.NonUnit, blasx.Unit]))


def poisoned(rng, n, uplo, diag, dominant=False):
    A = rng.uniform(-1, 1, (n, n))
    A[np.diag_indices(n)] = (n + rng.uniform(0, 1, n)) if dominant else rng.uniform(1, 2, n)
    P = A.copy()
    for r in range(n):
        for c in range(n):
            outside = (r < c) if uplo == blasx.Lower else (r > c)
            if outside or (r == c and diag == blasx.Unit):
                P[r, c] = np.nan
    return P


@pytest.mark.parametrize("order", ORDERS)
@pytest.mark.parametrize("side,uplo,trans,diag", FLAGS)
def test_trmm_matches_oracle(sim, order, side, uplo, trans, diag):
    setup(sim, T=16, seed=side + uplo + trans + diag + order, group=5)
    rng = np.random.default_rng(4)
    M, N = 52, 39
    P = poisoned(rng, M if side == blasx.Left else N, uplo, diag)
    B = rng.uniform(-1, 1, (M, N))
    Ps, Bs, Br = store(P, order, 2), store(B, order, 1), store(B, order, 1)
    sim.dtrmm(order, side, uplo, trans, diag, M, N, -0.8, Ps, ld_of(Ps, order), Bs, ld_of(Bs, order))
    ref.trmm(order, side, uplo, trans, diag, -0.8, Ps, Br)
    assert np.all(np.isfinite(np.asarray(Bs)))
    assert relerr(Bs, np.asarray(Br)) < 1e-14


@pytest.mark.parametrize("order", ORDERS)
@pytest.mark.parametrize("side,uplo,trans,diag", FLAGS)
def test_trsm_matches_oracle_and_residual(sim, order, side, uplo, trans, diag):
    setup(sim, T=16, seed=3 * side + uplo + trans + diag + order, group=4)
    rng = np.random.default_rng(5)
    M, N = 45, 58
    n = M if side == blasx.Left else N
    P = poisoned(rng, n, uplo, diag, dominant=True)
    if diag == blasx.Unit:          # keep the unit-diagonal system well conditioned
        P = np.where(np.isnan(P), P, P / n)
    B = rng.uniform(-1, 1, (M, N))
    Ps, Bs, Br = store(P, order, 1), store(B, order, 2), store(B, order, 2)
    sim.dtrsm(order, side, uplo, trans, diag, M, N, 1.25, Ps, ld_of(Ps, order), Bs, ld_of(Bs, order))
    ref.trsm(order, side, uplo, trans, diag, 1.25, Ps, Br)
    X = np.asarray(Bs)
    assert np.all(np.isfinite(X))
    assert relerr(X, np.asarray(Br)) < 1e-13
    # residual ||op(A) X - alpha B|| / (||A|| ||X||), formed by the oracle's TRMM
    R = store(X, order)
    ref.trmm(order, side, uplo, trans, diag, 1.0, Ps, R)
    Tn = np.linalg.norm(np.nan_to_num(P)) + (np.sqrt(n) if diag == blasx.Unit else 0)
    assert np.linalg.norm(np.asarray(R) - 1.25 * B) / (Tn * np.linalg.norm(X)) < 1e-13


def test_trsm_large_tile_inverse_levels(sim):
    """A diagonal tile larger than the directly inverted blocks exercises the merge levels."""
    setup(sim, T=96, seed=9, group=3, arena_tiles=40)
    rng = np.random.default_rng(6)
    M, N = 200, 100
    for uplo in (blasx.Lower, blasx.Upper):
        P = poisoned(rng, M, uplo, blasx.NonUnit, dominant=True)
        B = np.asfortranarray(rng.uniform(-1, 1, (M, N)))
        Ps, Bs, Br = store(P, blasx.ColMajor), B.copy(order="F"), B.copy(order="F")
        sim.dtrsm(blasx.ColMajor, blasx.Left, uplo, blasx.NoTrans, blasx.NonUnit, M, N, 1.0, Ps, M, Bs, M)
        ref.trsm(ref.ColMajor, ref.Left, uplo, ref.NoTrans, ref.NonUnit, 1.0, Ps, Br)
        assert relerr(Bs, Br) < 1e-13


def test_trsm_alpha_zero_gives_zero_without_reading_a(sim):
    setup(sim, T=16)
    B = np.asfortranarray(np.random.default_rng(0).uniform(-1, 1, (30, 20)))
    nan = np.full((30, 30), np.nan, order="F")
    sim.dtrsm(blasx.ColMajor, blasx.Left, blasx.Lower, blasx.NoTrans, blasx.NonUnit, 30, 20, 0.0, nan, 30, B, 30)
    assert np.array_equal(B, np.zeros((30, 20)))


# ------------------------------------------------------------------ structure -----

def test_tile_counts_match_the_papers_formulas(sim):
    """tests/golden/tile_counts.txt: Section III.A tile counts, Section IV.A degree of parallelism."""
    path = os.path.join(os.path.dirname(__file__), "golden", "tile_counts.txt")
    for line in open(path):
        if line.startswith("#") or not line.strip():
            continue
        rows, cols, T, square, nonsquare, dop = map(int, line.split())
        assert (rows // T) * (cols // T) == square
        assert -(-rows // T) * -(-cols // T) - square == nonsquare
        assert square + nonsquare == dop
        if rows * cols <= 300 * 300:        # the task builder makes exactly `dop` tasks
            setup(sim, T=max(16, T - T % 16) if T >= 16 else 16)
            Teff = sim.get_option("tile")
            A = np.zeros((rows, 16), order="F")
            B = np.zeros((16, cols), order="F")
            C = np.zeros((rows, cols), order="F")
            sim.dgemm(blasx.ColMajor, blasx.NoTrans, blasx.NoTrans, rows, cols, 16, 1.0, A, rows, B, 16, 0.0, C, rows)
            assert sim.get_stats()["tasks"] == -(-rows // Teff) * -(-cols // Teff)


def test_run_to_run_reproducible_and_interleaving_independent(sim):
    n = 96
    A, B = synth.matrix(n, n, 11, 0), synth.matrix(n, n, 11, 1)
    outs = []
    # With room for every tile no scheduling decision depends on device timing, so the grouping
    # of k-steps -- and with it every rounding -- is the same whatever the interleaving.
    for seed in (1, 2, 3):
        setup(sim, T=16, seed=seed, group=6, kchain=3, arena_tiles=128)
        C = np.zeros((n, n), order="F")
        sim.dgemm(blasx.ColMajor, blasx.NoTrans, blasx.NoTrans, n, n, n, 1.0, A, n, B, n, 0.0, C, n)
        outs.append(C)
    assert np.array_equal(outs[0], outs[1]) and np.array_equal(outs[0], outs[2])
    # Under slot pressure a chain may be cut where a tile was not yet available: same sums,
    # possibly grouped differently, i.e. equal up to rounding.
    setup(sim, T=16, seed=4, group=6, kchain=3, arena_tiles=40)
    C = np.zeros((n, n), order="F")
    sim.dgemm(blasx.ColMajor, blasx.NoTrans, blasx.NoTrans, n, n, n, 1.0, A, n, B, n, 0.0, C, n)
    assert relerr(C, outs[0]) < 1e-15


# ------------------------------------------------------------------ wide mode --------------
# All tasks of a call advance together, k-chunk by k-chunk; the host C tile arrives late, in a slot
# of its own, and the last launch of a task adds the accumulated partial sums to it.

@pytest.mark.parametrize("order", ORDERS)
@pytest.mark.parametrize("ta,tb", list(itertools.product(TRANS, TRANS)))
@pytest.mark.parametrize("M,N,K,kchain", [(64, 80, 96, 2), (37, 53, 41, 1), (50, 50, 100, 3), (48, 48, 16, 4)])
def test_wide_mode_gemm_matches_oracle(sim, order, ta, tb, M, N, K, kchain):
    setup(sim, T=16, arena_tiles=400, seed=M + ta + 3 * tb + order, wide=2, group=2, kchain=kchain)
    rng = np.random.default_rng(M * K + ta)
    A = rng.uniform(-1, 1, (M, K) if ta == blasx.NoTrans else (K, M))
    B = rng.uniform(-1, 1, (K, N) if tb == blasx.NoTrans else (N, K))
    C = rng.uniform(-1, 1, (M, N))
    As, Bs, Cs, Cr = store(A, order, 1), store(B, order, 2), store(C, order, 3), store(C, order, 3)
    sim.dgemm(order, ta, tb, M, N, K, 0.75, As, ld_of(As, order), Bs, ld_of(Bs, order), -0.5, Cs, ld_of(Cs, order))
    # one launch per task leaves nothing to pipeline: such calls keep the grouped schedule
    assert sim.get_option("last_wide") == (1 if -(-K // 16) > kchain else 0)
    ref.gemm(order, ta, tb, 0.75, As, Bs, -0.5, Cr)
    assert relerr(Cs, np.asarray(Cr)) < 1e-14
    st = sim.get_stats()
    nt = -(-M // 16) * -(-N // 16)
    assert st["tasks"] == nt and st["copies_d2h"] == nt
    assert st["bytes_h2d"] == 8 * (M * K + K * N + M * N)        # every tile exactly once, C included


@pytest.mark.parametrize("ktiles,ramp,expect", [(19, 0, 3), (16, 0, 2), (24, 0, 2), (13, 0, 1), (12, 0, 2), (15, 0, 3), (19, 8, 8), (19, 5, 5), (17, 0, 1)])
def test_wide_mode_first_round_takes_the_odd_steps(sim, ktiles, ramp, expect):
    """The k loop is cut into rounds of 8 steps (6 for 12 .. 15 k-tiles, which would otherwise make two rounds only);
    what is left over goes into the first round (or 2 steps when nothing is left over), never the last."""
    M, N, K = 48, 40, 16 * ktiles - 5
    setup(sim, T=16, arena_tiles=800, seed=ktiles + ramp, wide=2, group=2, kchain=0, ramp=ramp)
    rng = np.random.default_rng(ktiles)
    A, B, C = fmat(rng, M, K), fmat(rng, K, N), fmat(rng, M, N)
    want = A @ B - 2.0 * C
    sim.dgemm(CM, NT, NT, M, N, K, 1.0, A, M, B, K, -2.0, C, M)
    kc = 6 if 12 <= ktiles < 16 else 8
    assert sim.get_option("last_wide") == 1 and sim.get_option("last_kchain") == kc
    assert sim.get_option("last_ramp") == expect
    assert np.array_equal(C, want)                       # small integers: exact in any order
    st = sim.get_stats()
    assert st["bytes_h2d"] == 8 * (M * K + K * N + M * N)
    # 9 tasks = one launch per round: the odd steps first, then full rounds (nothing left over and no explicit
    # request: the first full round is split into 2 + 6, the same number of rounds as 2 + 8 + ... + 6)
    rounds = 1 + -(-(ktiles - expect) // kc) if expect < kc else -(-ktiles // kc)
    assert st["tasks"] == 9 and st["launches"] == rounds


def test_wide_mode_last_launches_are_cut_short(sim):
    """Wide schedule: the last sixteen tasks of the last round go out as launches of "tail_cut" tasks, so that most of
    their results leave under a kernel.  Same results, same bytes, more launches."""
    M, N, K = 16 * 6, 16 * 8, 16 * 9                   # 48 tasks, 9 k-tiles: rounds of 1 + 4 + 4 with chains of 4
    A = synth.matrix(M, K, 41, 0, integers=True)
    B = synth.matrix(K, N, 41, 1, integers=True)
    C0 = synth.matrix(M, N, 41, 2, integers=True)
    want = np.asarray(A) @ np.asarray(B) - 2.0 * np.asarray(C0)
    launches = {}
    for tail in (0, 4, 2, 16):
        setup(sim, T=16, arena_tiles=800, seed=tail, wide=2, group=2, kchain=4, tail_cut=tail)
        C = C0.copy(order="F")
        sim.dgemm(CM, NT, NT, M, N, K, 1.0, A, M, B, K, -2.0, C, M)
        assert sim.get_option("last_wide") == 1 and np.array_equal(C, want), tail
        st = sim.get_stats()
        assert st["bytes_h2d"] == 8 * (M * K + K * N + M * N) and st["tasks"] == 48
        launches[tail] = st["launches"]
    assert launches[0] == launches[16] == 3 * 3         # three rounds of three launches of sixteen
    assert launches[4] == 9 + 3 and launches[2] == 9 + 7


@pytest.mark.parametrize("side", [blasx.Left, blasx.Right])
@pytest.mark.parametrize("uplo", [blasx.Lower, blasx.Upper])
@pytest.mark.parametrize("trans", TRANS)
def test_wide_solve_with_staggered_panels_of_right_hand_sides(sim, side, uplo, trans):
    """Wide triangular solve: the right-hand sides are cut into "stagger_panels" independent panels, each "stagger_lag"
    rounds behind the one before.  Any number of panels and any lag give the solution of the oracle (residual and
    elementwise), also when the cache is tight and when the lag exceeds the number of rounds."""
    rng = np.random.default_rng(uplo + 2 * trans + 5 * side)
    T = 16
    n, m = 16 * 7 - 3, 16 * 6 + 5                     # triangular order n, other extent m
    A = np.asfortranarray(rng.uniform(-1, 1, (n, n)) + n * np.eye(n))
    M, N = (n, m) if side == blasx.Left else (m, n)
    B0 = np.asfortranarray(rng.uniform(-1, 1, (M, N)))
    want = B0.copy(order="F")
    ref.trsm(blasx.ColMajor, side, uplo, trans, blasx.NonUnit, 0.5, A, want)
    for case, (panels, lag, arena) in enumerate([(1, 3, 300), (2, -1, 300), (2, 3, 300), (2, 6, 300), (3, 2, 300), (4, 1, 300), (7, 1, 300),
                                                 (2, 50, 300), (2, 3, 120), (3, 2, 100)]):
        setup(sim, T=T, arena_tiles=arena, seed=case, wide=1, group=2, kchain=0, stagger_panels=panels, stagger_lag=lag)
        B = B0.copy(order="F")
        sim.dtrsm(blasx.ColMajor, side, uplo, trans, blasx.NonUnit, M, N, 0.5, A, n, B, M)
        assert relerr(B, np.asarray(want)) < 1e-13, (panels, lag, arena)
        st = sim.get_stats()
        assert st["bytes_d2h"] == 8 * M * N
        if arena == 300:
            assert sim.get_option("last_wide") == 1, (panels, lag)
            assert st["refetches"] == 0 and st["evictions"] == 0        # every tile crosses the link once
    # no lag given: chosen per call (this one is far too small to be device-bound: none)
    setup(sim, T=T, arena_tiles=300, wide=1, group=2, kchain=0, stagger_panels=2, stagger_lag=0)
    B = B0.copy(order="F")
    sim.dtrsm(blasx.ColMajor, side, uplo, trans, blasx.NonUnit, M, N, 0.5, A, n, B, M)
    assert relerr(B, np.asarray(want)) < 1e-13


def test_wide_mode_special_cases(sim):
    rng = np.random.default_rng(31)
    n = 64
    A, B = fmat(rng, n, n), fmat(rng, n, n)
    # beta = 0: C is never read (NaN in, exact integers out); no C tile crosses the link
    setup(sim, T=16, arena_tiles=400, wide=2, group=2, kchain=2)
    C = np.full((n, n), np.nan, order="F")
    sim.dgemm(CM, NT, NT, n, n, n, 2.0, A, n, B, n, 0.0, C, n)
    assert sim.get_option("last_wide") == 1 and np.array_equal(C, 2.0 * (A @ B))
    assert sim.get_stats()["bytes_h2d"] == 2 * 8 * n * n
    # alpha = 0: A and B are never read; C <- beta C
    C0 = fmat(rng, n, n)
    C = C0.copy(order="F")
    sim.dgemm(CM, NT, NT, n, n, n, 0.0, np.full((n, n), np.nan, order="F"), n, np.full((n, n), np.nan, order="F"), n, 3.0, C, n)
    assert np.array_equal(C, 3.0 * C0)
    # integer data: bit-exact whatever the order of the partial sums, also with one launch per task (kchain >= k tiles)
    for kchain in (1, 2, 4):
        setup(sim, T=16, arena_tiles=400, wide=2, group=2, kchain=kchain, seed=kchain)
        C = C0.copy(order="F")
        sim.dgemm(CM, NT, blasx.Trans, n, n, n, 1.0, A, n, B, n, -1.0, C, n)
        assert sim.get_option("last_wide") == (1 if kchain < 4 else 0) and np.array_equal(C, A @ B.T - C0)
    # not enough room for an accumulator per task: the call falls back to the grouped schedule
    setup(sim, T=16, arena_tiles=40, wide=2, group=2, kchain=2)
    C = C0.copy(order="F")
    sim.dgemm(CM, NT, NT, n, n, n, 1.0, A, n, B, n, 1.0, C, n)
    assert sim.get_option("last_wide") == 0 and np.array_equal(C, A @ B + C0)
    # the in-place triangular product runs wide too, exact on integers
    setup(sim, T=16, arena_tiles=400, wide=2, group=2)
    L = np.asfortranarray(np.tril(fmat(rng, n, n)) + 9 * np.eye(n))
    X = B.copy(order="F")
    sim.dtrmm(CM, blasx.Left, blasx.Lower, NT, blasx.NonUnit, n, n, 1.0, L, n, X, n)
    assert sim.get_option("last_wide") == 1 and np.array_equal(X, L @ B)


@pytest.mark.parametrize("seed", range(6))
def test_wide_mode_symmetric_routines_and_tight_cache(sim, seed):
    """SYRK / SYR2K (output-triangle mask: the C tile of a diagonal task is needed even for beta = 0) and SYMM
    (derived tiles) in wide mode, with barely enough slots so that operand tiles of finished rounds are evicted."""
    rng = np.random.default_rng(40 + seed)
    n, k = 80, 256
    uplo = blasx.Lower if seed % 2 else blasx.Upper
    other = np.triu_indices(n, 1) if uplo == blasx.Lower else np.tril_indices(n, -1)
    A, B = fmat(rng, n, k), fmat(rng, n, k)
    C0 = fmat(rng, n, n)
    C0[other] = 99.0
    beta = 0.0 if seed % 3 == 0 else 2.0
    setup(sim, T=16, arena_tiles=72 + 4 * seed, wide=2, group=2, kchain=1 + seed % 3, seed=seed)
    C = C0.copy(order="F")
    sim.dsyrk(CM, uplo, NT, n, k, 1.0, A, n, beta, C, n)
    assert sim.get_option("last_wide") == 1 and sim.get_stats()["evictions"] > 0
    want = np.where(np.isin(np.arange(n * n).reshape(n, n), np.ravel_multi_index(other, (n, n))), 99.0, A @ A.T + beta * C0)
    assert np.array_equal(C, want)
    C = C0.copy(order="F")
    sim.dsyr2k(CM, uplo, NT, n, k, 1.0, A, n, B, n, beta, C, n)
    assert sim.get_option("last_wide") == 1
    want = np.where(np.isin(np.arange(n * n).reshape(n, n), np.ravel_multi_index(other, (n, n))), 99.0, A @ B.T + B @ A.T + beta * C0)
    assert np.array_equal(C, want)
    S = fmat(rng, n, n)
    full = np.tril(S) + np.tril(S, -1).T if uplo == blasx.Lower else np.triu(S) + np.triu(S, 1).T
    Bm, Cm = fmat(rng, n, 48), fmat(rng, n, 48)
    Cs = Cm.copy(order="F")
    setup(sim, T=16, arena_tiles=76 + 4 * seed, wide=2, group=2, kchain=1 + seed % 3, seed=seed)
    sim.dsymm(CM, blasx.Left, uplo, n, 48, 1.0, S, n, Bm, n, beta, Cs, n)
    assert sim.get_option("last_wide") == 1
    assert np.array_equal(Cs, full @ Bm + beta * Cm)


@pytest.mark.parametrize("order", ORDERS)
@pytest.mark.parametrize("side,uplo,trans,diag", FLAGS)
def test_wide_mode_trsm_all_flags(sim, order, side, uplo, trans, diag):
    """The triangular solve in the wide schedule: right-looking, one k-step per round, the right-hand-side tile
    fetched late and combined with the accumulated updates by the task's last update launch."""
    setup(sim, T=16, arena_tiles=300, seed=side + uplo + trans + diag + order, wide=2, group=3)
    rng = np.random.default_rng(50 + side + uplo)
    M, N = 84, 70
    n = M if side == blasx.Left else N
    P = poisoned(rng, n, uplo, diag, dominant=True)
    if diag == blasx.Unit:
        P = np.where(np.isnan(P), P, P / n)
    B = rng.uniform(-1, 1, (M, N))
    Ps, Bs, Br = store(P, order, 2), store(B, order, 1), store(B, order, 1)
    sim.dtrsm(order, side, uplo, trans, diag, M, N, 0.7, Ps, ld_of(Ps, order), Bs, ld_of(Bs, order))
    assert sim.get_option("last_wide") == 1
    ref.trsm(order, side, uplo, trans, diag, 0.7, Ps, Br)
    assert np.all(np.isfinite(np.asarray(Bs)))
    assert relerr(Bs, np.asarray(Br)) < 1e-13
    st = sim.get_stats()
    ntm, ntn = -(-M // 16), -(-N // 16)
    assert st["tasks"] == ntm * ntn
    nta = ntm if side == blasx.Left else ntn
    assert st["bytes_h2d"] >= 8 * M * N and st["copies_d2h"] == ntm * ntn
    assert st["misses"] >= nta * (nta + 1) // 2 + nta


@pytest.mark.parametrize("order", ORDERS)
@pytest.mark.parametrize("side,uplo,trans,diag", FLAGS)
def test_wide_mode_trmm_all_flags(sim, order, side, uplo, trans, diag):
    """The in-place triangular product in the wide schedule: every panel of B is pinned at once, its tiles copied in
    when first needed, and a result may only overwrite the host tile whose original has been read."""
    setup(sim, T=16, arena_tiles=300, seed=3 * side + uplo + trans + diag + order, wide=2, group=3, kchain=1 + (side + uplo) % 3)
    rng = np.random.default_rng(70 + side + trans)
    M, N = 84, 70
    P = poisoned(rng, M if side == blasx.Left else N, uplo, diag)
    B = rng.uniform(-1, 1, (M, N))
    Ps, Bs, Br = store(P, order, 2), store(B, order, 1), store(B, order, 1)
    sim.dtrmm(order, side, uplo, trans, diag, M, N, -0.8, Ps, ld_of(Ps, order), Bs, ld_of(Bs, order))
    assert sim.get_option("last_wide") == 1
    ref.trmm(order, side, uplo, trans, diag, -0.8, Ps, Br)
    assert np.all(np.isfinite(np.asarray(Bs)))
    assert relerr(Bs, np.asarray(Br)) < 1e-14
    st = sim.get_stats()
    assert st["copies_d2h"] == -(-M // 16) * -(-N // 16)
    nta = -(-(M if side == blasx.Left else N) // 16)
    assert st["bytes_h2d"] >= 8 * M * N           # every tile of B once (its original), plus the triangle of A


@pytest.mark.parametrize("side,uplo,trans", [(blasx.Left, blasx.Lower, blasx.NoTrans), (blasx.Left, blasx.Upper, blasx.Trans),
                                             (blasx.Right, blasx.Lower, blasx.NoTrans), (blasx.Right, blasx.Upper, blasx.NoTrans)])
def test_wide_product_with_staggered_panels(sim, side, uplo, trans):
    """Wide triangular product with its right-hand sides in panels that run some rounds apart: small integers, so any
    order of the sums gives the same bits; every panel count, lag and chain length, roomy and tight caches."""
    rng = np.random.default_rng(uplo + 3 * side + trans)
    n, m = 16 * 7 - 5, 16 * 6 + 3
    A = rng.integers(-2, 3, (n, n)).astype(np.float64)
    Tm = np.tril(A) if uplo == blasx.Lower else np.triu(A)
    Top = Tm if trans == blasx.NoTrans else Tm.T
    M, N = (n, m) if side == blasx.Left else (m, n)
    B = rng.integers(-2, 3, (M, N)).astype(np.float64)
    want = 2.0 * (Top @ B if side == blasx.Left else B @ Top)
    for case, (panels, lag, kchain, arena) in enumerate([(2, -1, 1, 300), (2, 1, 1, 300), (2, 3, 2, 300), (3, 2, 1, 300), (4, 1, 3, 300),
                                                         (7, 1, 1, 300), (2, 40, 1, 300), (2, 2, 1, 170), (3, 1, 2, 160)]):
        setup(sim, T=16, arena_tiles=arena, seed=case, wide=2, group=2, kchain=kchain, stagger_panels=panels, stagger_lag=lag)
        As, Bs = store(A, blasx.ColMajor), store(B, blasx.ColMajor)
        sim.dtrmm(blasx.ColMajor, side, uplo, trans, blasx.NonUnit, M, N, 2.0, As, n, Bs, M)
        assert sim.get_option("last_wide") == 1, (panels, lag, kchain, arena)
        assert np.array_equal(np.asarray(Bs), want), (panels, lag, kchain, arena)
        assert sim.get_stats()["bytes_d2h"] == 8 * M * N


@pytest.mark.parametrize("seed", range(6))
def test_wide_mode_trmm_tight_cache_many_interleavings(sim, seed):
    rng = np.random.default_rng(80 + seed)
    n, m = 96, 80
    side = blasx.Left if seed % 2 else blasx.Right
    uplo = blasx.Lower if seed % 3 else blasx.Upper
    na = n if side == blasx.Left else m
    A = rng.integers(-2, 3, (na, na)).astype(np.float64)
    Tm = np.tril(A) if uplo == blasx.Lower else np.triu(A)
    B = rng.integers(-2, 3, (n, m)).astype(np.float64)
    setup(sim, T=16, arena_tiles=150 + 3 * seed, wide=2, group=2, kchain=1 + seed % 3, seed=300 + seed)
    As, Bs = store(A, blasx.ColMajor), store(B, blasx.ColMajor)
    sim.dtrmm(blasx.ColMajor, side, uplo, blasx.NoTrans, blasx.NonUnit, n, m, 1.0, As, na, Bs, n)
    assert sim.get_option("last_wide") == 1
    assert np.array_equal(np.asarray(Bs), Tm @ B if side == blasx.Left else B @ Tm)


@pytest.mark.parametrize("seed", range(6))
def test_wide_mode_trsm_tight_cache_many_interleavings(sim, seed):
    rng = np.random.default_rng(60 + seed)
    n, m = 96, 80
    side = blasx.Left if seed % 2 else blasx.Right
    uplo = blasx.Lower if seed % 3 else blasx.Upper
    na = n if side == blasx.Left else m
    L = np.tril(rng.integers(-2, 3, (na, na)).astype(np.float64), -1) + np.eye(na)      # unit triangular, integers
    if uplo == blasx.Upper:
        L = L.T.copy()
    X = rng.integers(-2, 3, (n, m)).astype(np.float64)
    B = L @ X if side == blasx.Left else X @ L
    setup(sim, T=16, arena_tiles=116 + 3 * seed, wide=2, group=2, seed=200 + seed)
    Ls, Bs = store(L, blasx.ColMajor), store(B, blasx.ColMajor)
    sim.dtrsm(blasx.ColMajor, side, uplo, blasx.NoTrans, blasx.Unit, n, m, 1.0, Ls, na, Bs, n)
    assert sim.get_option("last_wide") == 1
    assert np.array_equal(np.asarray(Bs), X)          # small integers and a unit diagonal: the solve is exact


@pytest.mark.parametrize("nstreams", [2, 3, 4])
@pytest.mark.parametrize("group", [1, 2, 4])
def test_grouped_trsm_very_tight_cache_many_interleavings(sim, nstreams, group):
    """The diagonal solve writes into a slot taken fresh from the pool.  Under a cache of a few
    tiles that slot has just been evicted, and an inbound copy for its previous owner may still be
    queued: the solve must be ordered after it (regression: it was not, and the stale copy landed
    on top of the solved tile)."""
    n, m = 96, 80
    bad = []
    for arena_tiles in range(6, 13):
        for seed in range(4):
            side = blasx.Left if (seed + arena_tiles) % 2 else blasx.Right
            uplo = blasx.Lower if seed % 3 else blasx.Upper
            rng = np.random.default_rng(1000 + 10 * arena_tiles + seed)
            na = n if side == blasx.Left else m
            L = np.tril(rng.integers(-2, 3, (na, na)).astype(np.float64), -1) + np.eye(na)
            if uplo == blasx.Upper:
                L = L.T.copy()
            X = rng.integers(-2, 3, (n, m)).astype(np.float64)
            B = L @ X if side == blasx.Left else X @ L
            setup(sim, T=16, nstreams=nstreams, arena_tiles=arena_tiles, wide=0, group=group, kchain=1 + seed % 2,
                  seed=7000 + 97 * arena_tiles + 13 * seed + nstreams)
            Ls, Bs = store(L, blasx.ColMajor), store(B, blasx.ColMajor)
            rc = sim.dtrsm(blasx.ColMajor, side, uplo, blasx.NoTrans, blasx.Unit, n, m, 1.0, Ls, na, Bs, n, check=False)
            if rc == 2:         # BLASX_ERR_ARENA_TOO_SMALL: an honest refusal, never a wrong result
                continue
            assert rc == 0
            assert sim.get_option("last_wide") == 0
            if not np.array_equal(np.asarray(Bs), X):
                bad.append((arena_tiles, seed, side, uplo))
    assert not bad, "wrong solves under a tight cache: %r" % bad


# ------------------------------------------------------------------ automatic tile size ---

def test_tile_zero_chooses_the_tile_from_extent_type_and_cache_room(sim):
    def chosen(fn, M, N, dtype=np.float64):
        A, B, C = np.ones((M, 1), dtype=dtype, order="F"), np.ones((1, N), dtype=dtype, order="F"), np.zeros((M, N), dtype=dtype, order="F")
        fn(blasx.ColMajor, blasx.NoTrans, blasx.NoTrans, M, N, 1, 1.0, A, M, B, 1, 0.0, C, M)
        assert np.all(C == 1.0)
        return sim.get_option("last_tile")

    sim._lib.blasx_sim_seed(1)
    sim.init_raw(2 ** 31, 0)                     # 0 streams = the measured best
    sim.set_cache_bytes(0)
    sim.set_tile(0)
    sim.set_option("wide", 11)                   # the library's default: the running-set rule below depends on it
    assert sim.get_option("tile") == 0
    assert chosen(sim.dgemm, 32768, 16) == 1024
    assert chosen(sim.dgemm, 16, 16384) == 1024
    assert chosen(sim.dgemm, 4096, 16) == 1024
    assert chosen(sim.dgemm, 2048, 2048) == 1024
    assert chosen(sim.dgemm, 2000, 16) == 2000
    assert chosen(sim.dgemm, 100, 50) == 112     # one tile, rounded up to the kernel's granule
    assert chosen(sim.sgemm, 32768, 16, np.float32) == 2048      # inner dimension 1: not the wide schedule's case
    assert chosen(sim.sgemm, 6656, 16, np.float32) == 2048
    assert chosen(sim.sgemm, 6144, 16, np.float32) == 1024
    assert chosen(sim.sgemm, 4096, 16, np.float32) == 1024       # single precision below 5120: 1024
    assert chosen(sim.sgemm, 3000, 16, np.float32) == 1024
    assert chosen(sim.sgemm, 2048, 16, np.float32) == 2048       # one tile
    assert chosen(sim.sgemm, 1500, 16, np.float32) == 1504

    # the triangular solve: the tile that gives a small solve five block rows (the wide schedule's least)
    def solve_tile(fn, n, dtype):
        L = np.asfortranarray(np.eye(n, dtype=dtype))
        B = np.ones((n, 16), dtype=dtype, order="F")
        fn(blasx.ColMajor, blasx.Left, blasx.Lower, blasx.NoTrans, blasx.NonUnit, n, 16, 1.0, L, n, B, n)
        assert np.all(B == 1.0)
        return sim.get_option("last_tile")

    assert [solve_tile(sim.dtrsm, n, np.float64) for n in (2048, 2560, 4096)] == [1024, 512, 512]
    assert solve_tile(sim.strsm, 5120, np.float32) == 1024
    assert solve_tile(sim.strsm, 2560, np.float32) == 512
    assert solve_tile(sim.dtrmm, 2560, np.float64) == 512 and solve_tile(sim.dtrmm, 2048, np.float64) == 1024
    # the triangular product in single precision: 1024 whatever the order
    Ltri = np.asfortranarray(np.eye(5120, dtype=np.float32))
    Btri = np.ones((5120, 16), dtype=np.float32, order="F")
    sim.strmm(blasx.ColMajor, blasx.Left, blasx.Lower, blasx.NoTrans, blasx.NonUnit, 5120, 16, 1.0, Ltri, 5120, Btri, 5120)
    assert np.all(Btri == 1.0) and sim.get_option("last_tile") == 1024
    # a small cache: halve the tile until 64 tiles fit
    sim.set_cache_bytes(64 * 2 ** 20)
    assert chosen(sim.dgemm, 8192, 16) == 256
    sim.set_cache_bytes(0)
    # the running set: a twelfth of the tasks as a power of two: 2 for a few tiles, 4 from 5 x 5, 16 from 14 x 14 tiles;
    # 16 for the triangular routines
    sim.set_option("group", 0)
    sim.set_tile(16)
    # (a k loop too short for the wide schedule, as here with one k-tile: 8 at most)
    for n, g in ((32, 2), (64, 2), (80, 4), (96, 4), (128, 4), (160, 8), (192, 8), (400, 8)):   # at least 4 from 5 x 5 tiles
        assert chosen(sim.dgemm, n, n) == 16 and sim.get_option("last_group") == g, n
    Ak, Bk, Ck = np.ones((256, 192), order="F"), np.ones((192, 256), order="F"), np.zeros((256, 256), order="F")
    sim.dgemm(blasx.ColMajor, blasx.NoTrans, blasx.NoTrans, 256, 256, 192, 1.0, Ak, 256, Bk, 192, 0.0, Ck, 256)
    assert np.all(Ck == 192.0) and sim.get_option("last_group") == 16        # 12 k-tiles, 16 x 16 tiles: 256 / 12 -> 16
    L = np.asfortranarray(np.tril(np.ones((64, 64))) + 63 * np.eye(64))
    B = np.ones((64, 32), order="F")
    sim.dtrsm(blasx.ColMajor, blasx.Left, blasx.Lower, blasx.NoTrans, blasx.NonUnit, 64, 32, 1.0, L, 64, B, 64)
    assert sim.get_option("last_group") == 16
    sim.set_option("group", 5)
    assert chosen(sim.dgemm, 256, 256) == 16 and sim.get_option("last_group") == 5
    sim.set_tile(1024)
    assert chosen(sim.dgemm, 100, 50) == 1024 and sim.get_option("tile") == 1024
    assert sim._lib.blasx_set_tile(8) == 4 and sim._lib.blasx_set_tile(1000) == 4


# ------------------------------------------------------------------ persistent cache ------

CM, NT, TR = blasx.ColMajor, blasx.NoTrans, blasx.Trans


def fmat(rng, r, c):
    return np.asfortranarray(rng.integers(-3, 4, (r, c)).astype(np.float64))   # small integers: exact products


def test_persistent_cache_serves_later_calls_and_forgets_on_request(sim):
    setup(sim, T=16, arena_tiles=96, persist=1)
    rng = np.random.default_rng(20)
    n = 64
    A, B, B2 = fmat(rng, n, n), fmat(rng, n, n), fmat(rng, n, n)
    C = np.zeros((n, n), order="F")
    sim.dgemm(CM, NT, NT, n, n, n, 1.0, A, n, B, n, 0.0, C, n)
    first = sim.get_stats()
    assert first["misses"] == 32 and np.array_equal(C, A @ B)
    assert sim.get_option("cached_tiles") == 32              # A and B tiles stay, C tiles never do
    # same A, new right-hand side: A is not copied again
    sim.reset_stats()
    sim.dgemm(CM, NT, NT, n, n, n, 1.0, A, n, B2, n, 0.0, C, n)
    st = sim.get_stats()
    assert st["misses"] == 16 and st["bytes_h2d"] == 16 * 16 * 16 * 8 and np.array_equal(C, A @ B2)
    # the host changes A without telling: the stale tiles are used (documented), until invalidated
    A_old = A.copy()
    A[...] = fmat(rng, n, n)
    sim.dgemm(CM, NT, NT, n, n, n, 1.0, A, n, B2, n, 0.0, C, n)
    assert np.array_equal(C, A_old @ B2)
    sim.reset_stats()
    sim.invalidate(A)
    assert sim.get_stats()["invalidations"] == 16
    sim.dgemm(CM, NT, NT, n, n, n, 1.0, A, n, B2, n, 0.0, C, n)
    assert np.array_equal(C, A @ B2) and sim.get_stats()["misses"] == 16
    sim.invalidate_all()
    assert sim.get_option("cached_tiles") == 0
    # persist off: nothing survives a call
    sim.set_option("persist", 0)
    sim.reset_stats()
    sim.dgemm(CM, NT, NT, n, n, n, 1.0, A, n, B2, n, 0.0, C, n)
    sim.dgemm(CM, NT, NT, n, n, n, 1.0, A, n, B2, n, 0.0, C, n)
    assert sim.get_stats()["misses"] == 64 and sim.get_option("cached_tiles") == 0


def test_persistent_cache_forgets_what_the_library_itself_overwrites(sim):
    setup(sim, T=16, arena_tiles=128, persist=1, group=5)
    rng = np.random.default_rng(21)
    n = 48
    A, A2, B = fmat(rng, n, n), fmat(rng, n, n), fmat(rng, n, n)
    D, E = np.zeros((n, n), order="F"), np.zeros((n, n), order="F")
    sim.dgemm(CM, NT, NT, n, n, n, 1.0, A, n, B, n, 0.0, D, n)        # D = A B
    sim.dgemm(CM, NT, NT, n, n, n, 1.0, D, n, B, n, 0.0, E, n)        # D is now a cached operand
    assert np.array_equal(E, A @ B @ B)
    sim.dgemm(CM, NT, NT, n, n, n, 1.0, A2, n, B, n, 0.0, D, n)       # D overwritten by the library
    sim.dgemm(CM, NT, NT, n, n, n, 1.0, D, n, B, n, 0.0, E, n)
    assert np.array_equal(E, A2 @ B @ B)
    # in-place triangular multiply: the original tiles of B2 were cached as operands of the call
    L = np.asfortranarray(np.tril(fmat(rng, n, n)))
    B2 = fmat(rng, n, n)
    want = L @ B2
    sim.dtrmm(CM, blasx.Left, blasx.Lower, NT, blasx.NonUnit, n, n, 1.0, L, n, B2, n)
    assert np.array_equal(B2, want)
    sim.dgemm(CM, NT, NT, n, n, n, 1.0, B2, n, B, n, 0.0, E, n)
    assert np.array_equal(E, want @ B)
    # SYMM keeps the completed diagonal tiles; a change of the symmetric matrix must drop them too
    S = fmat(rng, n, n)
    sim.dsymm(CM, blasx.Left, blasx.Lower, n, n, 1.0, S, n, B, n, 0.0, E, n)
    full = np.tril(S) + np.tril(S, -1).T
    assert np.array_equal(E, full @ B)
    S[np.diag_indices(n)] += 1.0
    sim.invalidate_matrix(S, n, n, n, 8)
    sim.dsymm(CM, blasx.Left, blasx.Lower, n, n, 1.0, S, n, B, n, 0.0, E, n)
    assert np.array_equal(E, (full + np.eye(n)) @ B)


def test_persistent_cache_triangular_solve_results_and_inverses_are_reused(sim):
    setup(sim, T=16, arena_tiles=128, persist=1, group=4)
    rng = np.random.default_rng(22)
    n, m = 64, 48
    L = np.asfortranarray(np.tril(rng.uniform(-1, 1, (n, n))) + n * np.eye(n))
    X = rng.uniform(-1, 1, (n, m))
    B = np.asfortranarray(L @ X)
    sim.dtrsm(CM, blasx.Left, blasx.Lower, NT, blasx.NonUnit, n, m, 1.0, L, n, B, n)
    assert relerr(B, X) < 1e-13
    nt = n // 16
    assert sim.get_stats()["misses"] == nt * (nt + 1) // 2 + nt     # L's tiles and one inverse per diagonal tile
    # the solution tiles are cached under B's address: a product with B copies nothing but C... and W
    sim.reset_stats()
    W, E = fmat(rng, m, 32), np.zeros((n, 32), order="F")
    sim.dgemm(CM, NT, NT, n, 32, m, 1.0, B, n, W, m, 0.0, E, n)
    assert relerr(E, X @ W) < 1e-13
    assert sim.get_stats()["misses"] == (m // 16) * 2            # only W's tiles
    # a second solve with the same triangular matrix: neither its tiles nor the inverses are redone
    sim.reset_stats()
    B2 = np.asfortranarray(L @ X)
    sim.dtrsm(CM, blasx.Left, blasx.Lower, NT, blasx.NonUnit, n, m, 1.0, L, n, B2, n)
    st = sim.get_stats()
    assert relerr(B2, X) < 1e-13 and st["misses"] == 0
    assert st["bytes_h2d"] == n * m * 8                          # the right-hand sides only


def test_persistent_cache_overlap_test_is_exact_for_views_of_one_matrix(sim):
    setup(sim, T=16, arena_tiles=128, persist=1)
    rng = np.random.default_rng(23)
    P = fmat(rng, 96, 64)                       # parent; ld = 96
    A = P[0:32, 0:32]                           # operand view
    C = P[32:64, 0:32]                          # output view: same columns, other rows
    B = fmat(rng, 32, 32)
    want = A @ B
    sim.dgemm(CM, NT, NT, 32, 32, 32, 1.0, A, 96, B, 32, 0.0, C, 96)
    assert np.array_equal(C, want)
    assert sim.get_stats()["invalidations"] == 0 and sim.get_option("cached_tiles") == 8
    # an output view that does share elements with cached tiles of A
    C2 = P[16:48, 16:48]
    sim.dgemm(CM, NT, NT, 32, 32, 32, 1.0, B, 32, B, 32, 0.0, C2, 96)
    assert sim.get_stats()["invalidations"] == 1   # only A's tile (1,1) = P[16:32, 16:32] lies inside the new output
    assert np.array_equal(P[16:48, 16:48], B @ B)
    E = np.zeros((32, 32), order="F")
    sim.dgemm(CM, NT, NT, 32, 32, 32, 1.0, A, 96, B, 32, 0.0, E, 32)
    assert np.array_equal(E, P[0:32, 0:32] @ B)
    # a changed tile size empties the cache
    sim.set_tile(32)
    sim.dgemm(CM, NT, NT, 32, 32, 32, 1.0, A, 96, B, 32, 0.0, E, 32)
    assert sim.get_option("cached_tiles") == 2


def test_persistent_cache_blocked_cholesky_on_views(sim):
    """Right-looking Cholesky of a matrix in host memory built from the library's TRSM / SYRK / GEMM on views of it,
    the diagonal blocks factored on the host: every matrix is operand in one call and output in another."""
    setup(sim, T=16, arena_tiles=160, persist=1, group=4)
    rng = np.random.default_rng(24)
    n, nb = 160, 48                              # block size is not a multiple of the tile: ragged views
    Aw = np.zeros((n, n), order="F")
    for attempt in range(2):                     # the second factorisation reuses the memory of the first
        G = rng.uniform(-1, 1, (n, n))
        S = G @ G.T + n * np.eye(n)
        want = np.linalg.cholesky(S)
        Aw[...] = S                              # the host rewrites an operand of earlier calls: tell the library
        sim.invalidate(Aw)
        for k in range(0, n, nb):
            b = min(nb, n - k)
            Akk = Aw[k:k + b, k:k + b]
            Akk[...] = np.linalg.cholesky(Akk)
            sim.invalidate_matrix(Akk, n, b, b, 8)
            r = n - k - b
            if r == 0:
                break
            panel = Aw[k + b:, k:k + b]
            sim.dtrsm(CM, blasx.Right, blasx.Lower, TR, blasx.NonUnit, r, b, 1.0, Akk, n, panel, n)
            trail = Aw[k + b:, k + b:]
            sim.dsyrk(CM, blasx.Lower, NT, r, b, -1.0, panel, n, 1.0, trail, n)
        assert relerr(np.tril(Aw), want) < 1e-13
    st = sim.get_stats()
    assert st["invalidations"] > 0 and st["hits"] > 0


# ------------------------------------------------------------------ single precision ------

@pytest.mark.parametrize("side,uplo,trans,diag", FLAGS[::3])
def test_single_precision_triangular_routines(sim, side, uplo, trans, diag):
    setup(sim, T=16, esize=4, seed=side + uplo + trans + diag)
    rng = np.random.default_rng(8)
    M, N = 40, 33
    n = M if side == blasx.Left else N
    P = poisoned(rng, n, uplo, diag, dominant=True).astype(np.float32)
    if diag == blasx.Unit:
        P = np.where(np.isnan(P), P, P / n).astype(np.float32)
    B = rng.uniform(-1, 1, (M, N)).astype(np.float32)
    Ps = store(P, blasx.ColMajor, 1, dtype=np.float32)
    Bs, Br = store(B, blasx.ColMajor, dtype=np.float32), store(B, blasx.ColMajor, dtype=np.float32)
    sim.strmm(blasx.ColMajor, side, uplo, trans, diag, M, N, 0.5, Ps, ld_of(Ps, blasx.ColMajor), Bs, M)
    ref.trmm(ref.ColMajor, side, uplo, trans, diag, 0.5, Ps, Br)
    assert relerr(Bs, np.asarray(Br, dtype=np.float64)) < 1e-5
    Bs, Br = store(B, blasx.ColMajor, dtype=np.float32), store(B, blasx.ColMajor, dtype=np.float32)
    sim.strsm(blasx.ColMajor, side, uplo, trans, diag, M, N, 2.0, Ps, ld_of(Ps, blasx.ColMajor), Bs, M)
    ref.trsm(ref.ColMajor, side, uplo, trans, diag, 2.0, Ps, Br)
    assert relerr(Bs, np.asarray(Br, dtype=np.float64)) < 1e-5


def test_ssyrk_matches_oracle(sim):
    setup(sim, T=16, esize=4)
    rng = np.random.default_rng(9)
    N, K = 50, 37
    A = np.asfortranarray(rng.uniform(-1, 1, (K, N)).astype(np.float32))
    C = np.asfortranarray(rng.uniform(-1, 1, (N, N)).astype(np.float32))
    Cs, Cr = C.copy(order="F"), C.copy(order="F")
    sim.ssyrk(blasx.ColMajor, blasx.Upper, blasx.Trans, N, K, 1.0, A, K, 0.5, Cs, N)
    ref.syrk(ref.ColMajor, ref.Upper, ref.Trans, 1.0, A, 0.5, Cr)
    assert relerr(Cs, Cr.astype(np.float64)) < 1e-6
    assert np.array_equal(np.tril(Cs, -1), np.tril(C, -1))


# ------------------------------------------------------------------ seeded random problems ---

@pytest.mark.parametrize("seed", range(60))
def test_seeded_random_problems_every_routine_schedule_and_cache_size(sim, seed):
    """Routine, flags, storage order, ragged extents, schedule options and the size of the tile cache drawn from
    a seeded generator (k extents up to 30 tiles: every shape of the wide schedule's rounds), against the oracle."""
    rng = np.random.default_rng(3000 + seed)
    routine = ("gemm", "syrk", "syr2k", "symm", "trmm", "trsm")[seed % 6]
    order = int(rng.choice(ORDERS))
    uplo = int(rng.choice([blasx.Lower, blasx.Upper]))
    trans, tb = int(rng.choice(TRANS)), int(rng.choice(TRANS))
    side = int(rng.choice([blasx.Left, blasx.Right]))
    diag = int(rng.choice([blasx.NonUnit, blasx.Unit]))
    alpha = float(rng.choice([1.0, -0.5, 0.0, 2.0]))
    beta = float(rng.choice([0.0, 1.0, -1.5]))
    M, N, K = int(rng.integers(10, 130)), int(rng.integers(10, 130)), int(rng.integers(5, 480))
    setup(sim, T=16, arena_tiles=int(rng.choice([64, 100, 200, 900])), seed=seed, group=int(rng.choice([0, 2, 5, 16])),
          kchain=int(rng.choice([0, 0, 1, 3, 8])), wide=int(rng.choice([0, 2, 12])), ramp=int(rng.choice([0, 0, 1, 5, 8])),
          depth=int(rng.choice([2, 6])), persist=int(rng.choice([0, 0, 1])))
    tag = "%s order=%d M=%d N=%d K=%d uplo=%d trans=%d/%d side=%d diag=%d alpha=%g beta=%g" % (routine, order, M, N, K, uplo, trans, tb, side, diag, alpha, beta)
    if routine == "gemm":
        A = rng.uniform(-1, 1, (M, K) if trans == blasx.NoTrans else (K, M))
        B = rng.uniform(-1, 1, (K, N) if tb == blasx.NoTrans else (N, K))
        C = rng.uniform(-1, 1, (M, N))
        As, Bs, Cs, Cr = store(A, order, 1), store(B, order, 2), store(C, order, 3), store(C, order, 3)
        sim.dgemm(order, trans, tb, M, N, K, alpha, As, ld_of(As, order), Bs, ld_of(Bs, order), beta, Cs, ld_of(Cs, order))
        ref.gemm(order, trans, tb, alpha, As, Bs, beta, Cr)
        assert relerr(Cs, np.asarray(Cr)) < 1e-13, tag
    elif routine in ("syrk", "syr2k"):
        A = rng.uniform(-1, 1, (N, K) if trans == blasx.NoTrans else (K, N))
        B = rng.uniform(-1, 1, A.shape)
        C = rng.uniform(-1, 1, (N, N))
        As, Bs, Cs, Cr = store(A, order, 1), store(B, order, 2), store(C, order, 3), store(C, order, 3)
        if routine == "syrk":
            sim.dsyrk(order, uplo, trans, N, K, alpha, As, ld_of(As, order), beta, Cs, ld_of(Cs, order))
            ref.syrk(order, uplo, trans, alpha, As, beta, Cr)
        else:
            sim.dsyr2k(order, uplo, trans, N, K, alpha, As, ld_of(As, order), Bs, ld_of(Bs, order), beta, Cs, ld_of(Cs, order))
            ref.syr2k(order, uplo, trans, alpha, As, Bs, beta, Cr)
        assert relerr(Cs, np.asarray(Cr)) < 1e-13, tag
    elif routine == "symm":
        n = M if side == blasx.Left else N
        A, B, C = rng.uniform(-1, 1, (n, n)), rng.uniform(-1, 1, (M, N)), rng.uniform(-1, 1, (M, N))
        As, Bs, Cs, Cr = store(A, order, 1), store(B, order, 2), store(C, order, 3), store(C, order, 3)
        sim.dsymm(order, side, uplo, M, N, alpha, As, ld_of(As, order), Bs, ld_of(Bs, order), beta, Cs, ld_of(Cs, order))
        ref.symm(order, side, uplo, alpha, As, Bs, beta, Cr)
        assert relerr(Cs, np.asarray(Cr)) < 1e-13, tag
    else:
        n = M if side == blasx.Left else N
        P = poisoned(rng, n, uplo, diag, dominant=True)
        if diag == blasx.Unit:
            P = np.where(np.isnan(P), P, P / n)
        B = rng.uniform(-1, 1, (M, N))
        Ps, Bs, Br = store(P, order, 2), store(B, order, 1), store(B, order, 1)
        alpha = alpha if alpha != 0.0 else 0.7
        if routine == "trmm":
            sim.dtrmm(order, side, uplo, trans, diag, M, N, alpha, Ps, ld_of(Ps, order), Bs, ld_of(Bs, order))
            ref.trmm(order, side, uplo, trans, diag, alpha, Ps, Br)
        else:
            sim.dtrsm(order, side, uplo, trans, diag, M, N, alpha, Ps, ld_of(Ps, order), Bs, ld_of(Bs, order))
            ref.trsm(order, side, uplo, trans, diag, alpha, Ps, Br)
        assert np.all(np.isfinite(np.asarray(Bs))), tag
        assert relerr(Bs, np.asarray(Br)) < 1e-12, tag
    sim.set_option("persist", 0)


# ------------------------------------------------ ragged tiles in the fast kernel ----------

@pytest.mark.parametrize("seed", range(3))
def test_ragged_tiles_are_kept_zero_padded_and_run_in_the_fast_kernel(sim, seed):
    """With a tile edge that is a multiple of the macro-tile edge, ragged tile steps are flagged as zero-padded and go
    to the unpredicated kernel; the device double then reads the k padding too (its memory starts as NaN bytes), so a
    tile whose padding had not been cleared after its copy, or after it was derived on the device, shows here."""
    rng = np.random.default_rng(seed)
    T = 128
    for wide in (0, 2):
        setup(sim, T=T, seed=seed, arena_tiles=96, group=3, kchain=2, wide=wide)
        M, N, K = 300, 200, 170
        for ta, tb in itertools.product(TRANS, TRANS):
            A = rng.uniform(-1, 1, (K, M) if ta == blasx.Trans else (M, K))
            B = rng.uniform(-1, 1, (N, K) if tb == blasx.Trans else (K, N))
            C = rng.uniform(-1, 1, (M, N))
            As, Bs, Cs, Cr = store(A, blasx.ColMajor, 3), store(B, blasx.ColMajor, 1), store(C, blasx.ColMajor, 2), store(C, blasx.ColMajor, 2)
            sim.dgemm(blasx.ColMajor, ta, tb, M, N, K, 0.7, As, ld_of(As, blasx.ColMajor), Bs, ld_of(Bs, blasx.ColMajor), -0.3, Cs, ld_of(Cs, blasx.ColMajor))
            ref.gemm(blasx.ColMajor, ta, tb, 0.7, As, Bs, -0.3, Cr)
            assert relerr(Cs, np.asarray(Cr)) < 1e-14
        # SYRK / SYR2K (output-triangle mask on ragged diagonal tiles), SYMM (tiles derived on the device), TRMM
        n, k = 300, 170
        A, B, C = rng.uniform(-1, 1, (n, k)), rng.uniform(-1, 1, (n, k)), rng.uniform(-1, 1, (n, n))
        Cs, Cr = store(C, blasx.ColMajor, 1), store(C, blasx.ColMajor, 1)
        sim.dsyrk(blasx.ColMajor, blasx.Lower, blasx.NoTrans, n, k, 1.1, A.copy(order="F"), n, 0.5, Cs, ld_of(Cs, blasx.ColMajor))
        ref.syrk(blasx.ColMajor, blasx.Lower, blasx.NoTrans, 1.1, A.copy(order="F"), 0.5, Cr)
        assert relerr(Cs, np.asarray(Cr)) < 1e-14
        Cs, Cr = store(C, blasx.ColMajor, 1), store(C, blasx.ColMajor, 1)
        sim.dsyr2k(blasx.ColMajor, blasx.Upper, blasx.NoTrans, n, k, 1.1, A.copy(order="F"), n, B.copy(order="F"), n, 0.5, Cs, ld_of(Cs, blasx.ColMajor))
        ref.syr2k(blasx.ColMajor, blasx.Upper, blasx.NoTrans, 1.1, A.copy(order="F"), B.copy(order="F"), 0.5, Cr)
        assert relerr(Cs, np.asarray(Cr)) < 1e-14
        general_before = sim.get_stats()["steps_general"]
        assert general_before == 0
        for side, uplo in ((blasx.Left, blasx.Lower), (blasx.Right, blasx.Upper)):
            m2, n2 = 300, 200
            na = m2 if side == blasx.Left else n2
            S = rng.uniform(-1, 1, (na, na))
            S[np.triu_indices(na, 1) if uplo == blasx.Lower else np.tril_indices(na, -1)] = np.nan
            B2, C2 = rng.uniform(-1, 1, (m2, n2)), rng.uniform(-1, 1, (m2, n2))
            Ss, Bs, Cs, Cr = store(S, blasx.ColMajor, 2), store(B2, blasx.ColMajor), store(C2, blasx.ColMajor), store(C2, blasx.ColMajor)
            sim.dsymm(blasx.ColMajor, side, uplo, m2, n2, -1.5, Ss, ld_of(Ss, blasx.ColMajor), Bs, m2, 0.25, Cs, m2)
            ref.symm(blasx.ColMajor, side, uplo, -1.5, Ss, Bs, 0.25, Cr)
            assert np.all(np.isfinite(np.asarray(Cs)))
            assert relerr(Cs, np.asarray(Cr)) < 1e-14
        assert sim.get_stats()["steps_general"] == 0
        steps_before = sim.get_stats()["tile_steps"]
        P = poisoned(rng, 300, blasx.Lower, blasx.NonUnit)
        B3 = rng.uniform(-1, 1, (300, 200))
        Ps, Bs, Br = store(P, blasx.ColMajor, 2), store(B3, blasx.ColMajor), store(B3, blasx.ColMajor)
        sim.dtrmm(blasx.ColMajor, blasx.Left, blasx.Lower, blasx.NoTrans, blasx.NonUnit, 300, 200, -0.8, Ps, ld_of(Ps, blasx.ColMajor), Bs, 300)
        ref.trmm(blasx.ColMajor, blasx.Left, blasx.Lower, blasx.NoTrans, blasx.NonUnit, -0.8, Ps, Br)
        assert relerr(Bs, np.asarray(Br)) < 1e-14
        st = sim.get_stats()
        # the ragged diagonal steps of the triangular product run in the masked fast kernel on the padded tiles too
        assert st["tile_steps"] - steps_before == 12 and st["steps_general"] == 0
        # the solve: results become operands (padded when they are adopted); all four side / triangle cases
        for side, uplo in itertools.product((blasx.Left, blasx.Right), (blasx.Lower, blasx.Upper)):
            m3, n3 = 300, 200
            na = m3 if side == blasx.Left else n3
            P = poisoned(rng, na, uplo, blasx.NonUnit, dominant=True)
            B4 = rng.uniform(-1, 1, (m3, n3))
            Ps, Bs, Br = store(P, blasx.ColMajor, 2), store(B4, blasx.ColMajor), store(B4, blasx.ColMajor)
            before = sim.get_stats()
            sim.dtrsm(blasx.ColMajor, side, uplo, blasx.NoTrans, blasx.NonUnit, m3, n3, 1.3, Ps, ld_of(Ps, blasx.ColMajor), Bs, m3)
            ref.trsm(blasx.ColMajor, side, uplo, blasx.NoTrans, blasx.NonUnit, 1.3, Ps, Br)
            assert np.all(np.isfinite(np.asarray(Bs)))
            assert relerr(Bs, np.asarray(Br)) < 1e-13
            after = sim.get_stats()
            assert after["steps_general"] == before["steps_general"] and after["tile_steps"] > before["tile_steps"]
    # single precision: k is rounded up to 64
    setup(sim, T=128, seed=seed, arena_tiles=96, esize=4, group=3, kchain=2)
    A, B, C = (rng.uniform(-1, 1, s).astype(np.float32) for s in ((200, 170), (170, 150), (200, 150)))
    Cs, Cr = np.asfortranarray(C), np.asfortranarray(C)
    sim.sgemm(blasx.ColMajor, blasx.NoTrans, blasx.NoTrans, 200, 150, 170, 1.0, np.asfortranarray(A), 200, np.asfortranarray(B), 170, 1.0, Cs, 200)
    ref.gemm(blasx.ColMajor, blasx.NoTrans, blasx.NoTrans, 1.0, np.asfortranarray(A), np.asfortranarray(B), 1.0, Cr)
    assert relerr(Cs, np.asarray(Cr)) < 1e-6
    assert sim.get_stats()["steps_general"] == 0


@pytest.mark.parametrize("wide", [0, 2])
def test_solve_results_are_never_read_before_their_launch_when_packs_of_two_kernels_are_open(sim, wide):
    """A dependency level of more tasks than one launch holds, with a ragged last block column: the solves of the
    whole tiles and the ragged one go to different kernel instantiations, whose launch packs are open side by side
    and go out in no order of their ids.  A step that reads a solve's result must wait for that very pack."""
    T, M, N = 128, 300, 2300
    rng = np.random.default_rng(5)
    for seed in range(3):
        setup(sim, T=T, seed=seed, arena_tiles=200, group=16, kchain=0, rs=32, wide=wide)
        A = np.tril(rng.uniform(-1, 1, (M, M))) + M * np.eye(M)
        B = rng.uniform(-1, 1, (M, N))
        Bs = np.asfortranarray(B)
        sim.dtrsm(blasx.ColMajor, blasx.Left, blasx.Lower, blasx.NoTrans, blasx.NonUnit, M, N, 1.0, np.asfortranarray(A), M, Bs, M)
        X = np.linalg.solve(A, B)
        assert relerr(Bs, X) < 1e-13
        assert sim.get_option("last_wide") == (1 if wide else 0)


def test_adopted_solve_results_are_padded_for_later_calls(sim):
    """Persistent cache, tile edge 128, ragged sizes: the solution tiles of a solve stay cached under B's address; a
    later product that reads them as a k-ragged operand runs in the fast kernel on the padded extent, so their padding
    must have been cleared when they were adopted (the double's memory starts as NaN and it reads the padding)."""
    setup(sim, T=128, arena_tiles=96, persist=1, group=4)
    rng = np.random.default_rng(24)
    n, m = 300, 200
    for uplo in (blasx.Lower, blasx.Upper):
        tri = np.tril if uplo == blasx.Lower else np.triu
        L = np.asfortranarray(tri(rng.uniform(-1, 1, (n, n))) + n * np.eye(n))
        X = rng.uniform(-1, 1, (n, m))
        B = np.asfortranarray(L @ X)
        sim.dtrsm(CM, blasx.Left, uplo, NT, blasx.NonUnit, n, m, 1.0, L, n, B, n)
        assert relerr(B, X) < 1e-13
        sim.reset_stats()
        # B (n x m) as the left operand: k = m = 200 is ragged; as the transposed right operand: k = n = 300 is
        W, E = fmat(rng, m, 70), np.zeros((n, 70), order="F")
        sim.dgemm(CM, NT, NT, n, 70, m, 1.0, B, n, W, m, 0.0, E, n)
        assert np.all(np.isfinite(E)) and relerr(E, X @ W) < 1e-13
        st = sim.get_stats()
        assert st["steps_general"] == 0 and st["misses"] == 2          # only W's two tiles were copied
        V, F = fmat(rng, 90, n), np.zeros((90, m), order="F")
        sim.dgemm(CM, NT, NT, 90, m, n, 1.0, V, 90, B, n, 0.0, F, 90)
        assert np.all(np.isfinite(F)) and relerr(F, V @ X) < 1e-13
        assert sim.get_stats()["steps_general"] == 0
        sim.invalidate_all()


# ------------------------------------------------------------------ merged inbound copies ----------

@pytest.mark.parametrize("wide", [0, 3])
def test_neighbouring_tiles_share_an_inbound_copy(sim, wide):
    """Whole tiles that lie side by side in a block row of a host matrix and go to neighbouring slots are one
    strided copy: with "merge" = 4 the copy engine sees fewer copies than tiles, the bytes moved stay what the
    method fixes, and the result is bit-identical to the one-copy-per-tile run."""
    M = N = K = 128
    A = synth.matrix(M, K, 11, 0, integers=True)
    B = synth.matrix(K, N, 11, 1, integers=True)
    C = synth.matrix(M, N, 11, 2, integers=True)
    want = 2.0 * (np.asarray(A) @ np.asarray(B)) - np.asarray(C)
    seen = {}
    for merge in (1, 4, 8, 0):          # 0: the library's choice, as many tiles as make 32 MiB, at most 8
        setup(sim, T=16, arena_tiles=400, group=4, kchain=4, wide=wide, sb_rows=4, sb_cols=4, merge=merge, seed=merge)
        Cs = C.copy(order="F")
        sim.dgemm(blasx.ColMajor, blasx.NoTrans, blasx.NoTrans, M, N, K, 2.0, A, M, B, K, -1.0, Cs, M)
        assert np.array_equal(Cs, want), merge
        st = sim.get_stats()
        assert st["bytes_h2d"] == 8 * (M * K + K * N + M * N) and st["copies_h2d"] == 3 * 64
        seen[merge] = st["transfers_h2d"]
    assert seen[1] == 3 * 64
    assert seen[4] <= 0.6 * seen[1], seen        # most tiles travel in company
    assert seen[8] <= 0.6 * seen[1] and seen[0] <= 0.6 * seen[1], seen
    sim.set_option("merge", 4)


@pytest.mark.parametrize("late_c", [0, 1])
def test_grouped_schedule_with_room_fetches_c_for_the_last_launch(sim, late_c):
    """With room for every tile of the call the grouped schedule fetches a task's host C tile for its last launch only
    (option "late_c", default 1) and cuts the k loop into launches of two k-tiles; results and link bytes are the same
    either way, for every routine that reads C."""
    rng = np.random.default_rng(5 + late_c)
    M, N, K = 83, 70, 101
    setup(sim, T=16, arena_tiles=600, group=3, kchain=0, depth=3, late_c=late_c, seed=3)
    A = np.asfortranarray(rng.uniform(-1, 1, (M, K)))
    B = np.asfortranarray(rng.uniform(-1, 1, (K, N)))
    C = np.asfortranarray(rng.uniform(-1, 1, (M, N)))
    Cs, Cr = C.copy(order="F"), C.copy(order="F")
    sim.dgemm(blasx.ColMajor, blasx.NoTrans, blasx.NoTrans, M, N, K, 1.5, A, M, B, K, -0.5, Cs, M)
    ref.gemm(blasx.ColMajor, blasx.NoTrans, blasx.NoTrans, 1.5, A, B, -0.5, Cr)
    assert relerr(Cs, np.asarray(Cr)) < 1e-14
    st = sim.get_stats()
    assert st["bytes_h2d"] == 8 * (M * K + K * N + M * N) and st["bytes_d2h"] == 8 * M * N
    assert sim.get_option("last_kchain") == (2 if late_c else 4) and sim.get_option("last_wide") == 0
    # integer inputs: bit-exact whichever launch adds the host tile
    Ai = synth.matrix(M, K, 21, 0, integers=True)
    Ci = synth.matrix(M, M, 21, 2, integers=True)
    want = np.asarray(Ci).copy()
    full = 2.0 * (np.asarray(Ai) @ np.asarray(Ai).T) + 3.0 * np.asarray(Ci)
    low = np.tril_indices(M)
    want[low] = full[low]
    Cs = Ci.copy(order="F")
    sim.dsyrk(blasx.ColMajor, blasx.Lower, blasx.NoTrans, M, K, 2.0, Ai, M, 3.0, Cs, M)
    assert np.array_equal(Cs, want)
    S = np.asfortranarray(rng.uniform(-1, 1, (M, M)))
    Cs, Cr = C.copy(order="F"), C.copy(order="F")
    sim.dsymm(blasx.ColMajor, blasx.Left, blasx.Upper, M, N, 0.75, S, M, B[:M, :] if K >= M else B, K, 1.25, Cs, M)
    ref.symm(blasx.ColMajor, blasx.Left, blasx.Upper, 0.75, S, B[:M, :], 1.25, Cr)
    assert relerr(Cs, np.asarray(Cr)) < 1e-14
    sim.set_option("late_c", 1)


def test_grouped_schedule_with_room_takes_tasks_block_row_by_block_row(sim):
    """A grouped call whose tiles all fit is bound by the link; its tasks are then taken block row by block row of C
    (option "row_order", default 1), whatever the super-block options say.  Seen in the order in which the host tiles
    of C are asked for, one task running at a time."""
    T, nt = 16, 4
    n = nt * T
    A = synth.matrix(n, n, 31, 0, integers=True)
    B = synth.matrix(n, n, 31, 1, integers=True)
    C0 = synth.matrix(n, n, 31, 2, integers=True)
    seen = {}
    for row_order in (0, 1):
        setup(sim, T=T, arena_tiles=200, group=1, rs=1, kchain=0, sb_rows=2, sb_cols=2, shells=1, row_order=row_order, priority=0)
        C = C0.copy(order="F")
        sim._lib.blasx_sim_trace_reset()
        sim.dgemm(blasx.ColMajor, blasx.NoTrans, blasx.NoTrans, n, n, n, 1.0, A, n, B, n, 1.0, C, n)
        assert np.array_equal(C, np.asarray(A) @ np.asarray(B) + np.asarray(C0))
        seen[row_order] = start_order(sim, C, T)
    rows = [(i, j) for i in range(nt) for j in range(nt)]
    assert seen[1] == rows
    assert sorted(seen[0]) == rows and seen[0] != rows and seen[0][:4] == [(0, 0), (0, 1), (1, 0), (1, 1)]
    # a cache too small for that keeps the queue's order
    setup(sim, T=T, arena_tiles=24, group=1, rs=1, kchain=0, sb_rows=2, sb_cols=2, shells=1, row_order=1, priority=0)
    C = C0.copy(order="F")
    sim._lib.blasx_sim_trace_reset()
    sim.dgemm(blasx.ColMajor, blasx.NoTrans, blasx.NoTrans, n, n, n, 1.0, A, n, B, n, 1.0, C, n)
    assert np.array_equal(C, np.asarray(A) @ np.asarray(B) + np.asarray(C0))
    assert start_order(sim, C, T) == seen[0]


def test_merged_copies_under_a_tight_cache_random_problems(sim):
    """Slots change owner all the time under a tight cache: a copy that is still being gathered must go out before
    anything is ordered after one of its slots.  Every routine, random shapes, merge 1..8, against the oracle."""
    rng = np.random.default_rng(2024)
    for case in range(40):
        T = 16
        M, N, K = (int(x) for x in rng.integers(33, 130, 3))
        merge = int(rng.integers(1, 9))
        wide = int(rng.choice([0, 2]))
        arena = int(rng.integers(14, 60)) if case % 3 else int(rng.integers(200, 500))
        setup(sim, T=T, arena_tiles=arena, group=int(rng.integers(1, 5)), kchain=int(rng.integers(1, 5)), wide=wide,
              merge=merge, nstreams=int(rng.integers(2, 5)), seed=case)
        A = np.asfortranarray(rng.uniform(-1, 1, (M, K)))
        B = np.asfortranarray(rng.uniform(-1, 1, (K, N)))
        C = np.asfortranarray(rng.uniform(-1, 1, (M, N)))
        Cs, Cr = C.copy(order="F"), C.copy(order="F")
        sim.dgemm(blasx.ColMajor, blasx.NoTrans, blasx.NoTrans, M, N, K, 1.5, A, M, B, K, 0.5, Cs, M)
        ref.gemm(blasx.ColMajor, blasx.NoTrans, blasx.NoTrans, 1.5, A, B, 0.5, Cr)
        assert relerr(Cs, np.asarray(Cr)) < 1e-14, (case, M, N, K, merge, wide, arena)
        # triangular solve on the same cache: results become operands, slots are recycled at once
        L = np.asfortranarray(np.tril(rng.uniform(-1, 1, (M, M))) + M * np.eye(M))
        X = np.asfortranarray(rng.uniform(-1, 1, (M, N)))
        Xs, Xr = X.copy(order="F"), X.copy(order="F")
        sim.dtrsm(blasx.ColMajor, blasx.Left, blasx.Lower, blasx.NoTrans, blasx.NonUnit, M, N, 1.0, L, M, Xs, M)
        ref.trsm(blasx.ColMajor, blasx.Left, blasx.Lower, blasx.NoTrans, blasx.NonUnit, 1.0, L, Xr)
        assert relerr(Xs, np.asarray(Xr)) < 1e-12, (case, M, N, merge, wide, arena)
    sim.set_option("merge", 4)
