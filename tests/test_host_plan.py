"""Host planners of the library against the oracle (CPU only)."""
import itertools
from fractions import Fraction

import numpy as np
import pytest

import paper_2410_17043_amd as P
import workloads as W
from oracle import matching as OM
from oracle import planning as OP
from oracle import schedule as OS


def random_D(r, n, hi=40, zero_frac=0.25):
    D = r.integers(0, hi, size=(n, n))
    D[r.random((n, n)) < zero_frac] = 0
    return D


def check_rounds(plan, D, B, exact):
    n = len(D)
    Pm = OS.scaled_matrix(D, B)
    bm = OS.bmax(D, B)
    tol = 0 if exact else 1e-9 * float(bm) + 1e-12
    assert abs(plan["bmax"] - float(bm)) <= tol
    assert abs(plan["duration"].sum() - float(bm)) <= max(tol, 0) if plan["n_rounds"] else bm == 0
    assert plan["n_rounds"] <= n * n + 8
    carried = np.zeros((n, n))
    left = np.array([[float(v) for v in row] for row in Pm])
    for dst, tau in zip(plan["dst"], plan["duration"]):
        live = [j for j in dst if j >= 0]
        assert len(live) == len(set(live))                      # a receiver hears one sender per round
        for i, j in enumerate(dst):
            if j >= 0:
                assert i != j
                use = min(left[i, j], tau)
                left[i, j] -= use
                carried[i, j] += use
    assert np.all(np.abs(left) <= (0 if exact else 1e-9 * float(bm) + 1e-12))   # everything delivered


@pytest.mark.parametrize("n", [1, 2, 3, 4, 8, 16])
def test_aurora_order_homogeneous_matches_oracle_exactly(n):
    r = np.random.default_rng(100 + n)
    for _ in range(5):
        D = random_D(r, n)
        plan = P.aurora_order(D)
        check_rounds(plan, D, None, exact=True)
        assert plan["bmax"] == float(OS.bmax(D)) == plan["port_bound"]
        ref = OS.alg1_order(D)
        assert plan["alg1_order"].tolist() == ref["dest_order"]                 # same stated reading
        assert plan["makespan_order"] == float(ref["makespan"])
        for i in range(n):
            for j in range(n):
                s = ref["start"][i][j]
                assert plan["start"][i, j] == (-1.0 if s is None else float(s))
        # the fluid simulation divides rates by fan-in, so doubles round where the oracle's rationals do not
        assert P.aurora_simulate(D, None, plan["alg1_order"]) == pytest.approx(
            float(OS.simulate(D, None, ref["dest_order"])), rel=1e-12)
        # the order for the send buffer: candidates, choice and improvement as in the oracle (n = 16 costs the
        # exact-rational oracle a minute, so its improvement step is compared up to n = 8)
        if n <= 8:
            so = OS.send_order(D)
            assert plan["candidate_time"] == pytest.approx([float(v) for v in so["candidate_times"]], rel=1e-12)
            assert plan["order_source"] == so["source"]
            assert plan["dest_order"].tolist() == so["dest_order"]
            assert plan["order_time"] == pytest.approx(float(so["time"]), rel=1e-12)
        assert plan["order_time"] == pytest.approx(P.aurora_simulate(D, None, plan["dest_order"]), rel=1e-12)
        assert plan["order_time"] <= min(plan["candidate_time"]) * (1 + 1e-12)
        assert plan["order_time"] >= plan["bmax"] * (1 - 1e-12)


@pytest.mark.parametrize("n", [2, 3, 4, 8, 16])
def test_aurora_order_heterogeneous(n):
    r = np.random.default_rng(200 + n)
    for _ in range(5):
        D = random_D(r, n)
        B = r.uniform(0.5, 1.0, size=n)
        plan = P.aurora_order(D, B)
        check_rounds(plan, D, B, exact=False)
        assert plan["bmax"] == pytest.approx(float(OS.bmax(D, B)), rel=1e-12)
        assert plan["port_bound"] == pytest.approx(float(OS.port_bound(D, B)), rel=1e-12)
        assert plan["port_bound"] <= plan["bmax"] * (1 + 1e-12)
        # the per-destination plan is valid: complete, contention-free, not below the bound
        Pm = np.array([[float(v) for v in row] for row in OS.scaled_matrix(D, B)])
        st = plan["start"]
        assert np.array_equal(st >= 0, Pm > 0)
        for i in range(n):
            assert sorted(plan["dest_order"][i].tolist()) == list(range(n))
            for tl in ([(st[i, j], st[i, j] + Pm[i, j]) for j in range(n) if st[i, j] >= 0],
                       [(st[j, i], st[j, i] + Pm[j, i]) for j in range(n) if st[j, i] >= 0]):
                tl.sort()
                assert all(a1 >= b0 - 1e-9 for (_, b0), (a1, _) in zip(tl[:-1], tl[1:]))
        assert plan["makespan_order"] >= plan["bmax"] * (1 - 1e-12)
        got = P.aurora_simulate(D, B, plan["alg1_order"])
        assert got == pytest.approx(float(OS.simulate(D, B, plan["alg1_order"].tolist())), rel=1e-9)
        assert got >= plan["port_bound"] * (1 - 1e-9)
        for i in range(n):
            assert sorted(plan["alg1_order"][i].tolist()) == list(range(n))
        got = P.aurora_simulate(D, B, plan["dest_order"])
        assert got == pytest.approx(plan["order_time"], rel=1e-12)
        assert got == pytest.approx(float(OS.simulate(D, B, plan["dest_order"].tolist())), rel=1e-9)
        assert got <= min(plan["candidate_time"]) * (1 + 1e-12)
        # with unequal rates a fast receiver can serve two slow senders at once, so the fluid model can
        # beat the one-sender-per-receiver bound of Appendix B; the per-port bound still holds
        assert got >= plan["port_bound"] * (1 - 1e-9)


def test_simulate_all_orders_against_oracle_n4_and_figure():
    r = np.random.default_rng(7)
    D = random_D(r, 4, hi=9)
    per_src = [list(itertools.permutations([j for j in range(4) if j != i])) for i in range(4)]
    best = None
    for combo in itertools.product(*per_src):
        order = [list(c) + [i] for i, c in enumerate(combo)]
        got = P.aurora_simulate(D, None, order)
        assert got == pytest.approx(float(OS.simulate(D, None, combo)), rel=1e-12)
        best = got if best is None else min(best, got)
    assert best >= P.aurora_order(D)["bmax"]
    fig = [[0, 1, 1], [1, 0, 1], [0, 0, 0]]
    assert P.aurora_simulate(fig, None, [[1, 2, 0], [0, 2, 1], [0, 1, 2]]) == 3.0
    assert P.aurora_simulate(fig, None, [[1, 2, 0], [2, 0, 1], [0, 1, 2]]) == 2.0
    plan = P.aurora_order(fig)
    assert plan["bmax"] == 2.0 and plan["makespan_rounds"] == 2.0 and plan["makespan_order"] == 2.0
    assert plan["order_time"] == 2.0


def test_send_order_against_the_stored_brute_force_optimum():
    # the same stored cases as the oracle's pin (tests/golden/order_ratios.txt): the library's send order is never
    # better than the optimum over all whole-flow orders, and equals what the oracle's send order reaches
    from tests.test_oracle_schedule import load_order_ratios
    at_optimum = 0
    for D, B, bm, best, _alg1, send in load_order_ratios():
        plan = P.aurora_order(D, None if B is None else [float(b) for b in B])
        assert plan["bmax"] == pytest.approx(float(bm), rel=1e-12)
        assert plan["order_time"] >= float(best) * (1 - 1e-9)
        assert plan["order_time"] == pytest.approx(float(send), rel=1e-9)
        at_optimum += abs(plan["order_time"] - float(best)) <= 1e-9 * float(best)
    assert at_optimum == 20


def test_schedules_for_the_workload_matrices():
    for name in ("c1_tiny_fp32", "c2_mixtral", "c5_finegrained"):
        cfg = W.get_config(name)
        D = W.make_traffic_matrix(cfg)["D"]
        B = W.make_link_rates(cfg) if cfg.hetero_links else None
        plan = P.aurora_order(D, B)
        check_rounds(plan, D, B, exact=B is None)
        assert plan["makespan_order"] >= plan["bmax"] * (1 - 1e-12)


@pytest.mark.parametrize("na,nb", [(1, 1), (2, 2), (3, 3), (4, 4), (6, 6), (2, 4), (3, 4), (4, 8), (8, 8)])
def test_colocate_match_against_brute_force(na, nb):
    r = np.random.default_rng(300 + 10 * na + nb)
    for _ in range(4 if nb >= 8 else 8):
        Da, Db = r.integers(0, 50, size=(na, na)), r.integers(0, 50, size=(nb, nb))
        pair, bott = P.colocate_match(Da, Db)
        want, _ = OM.best_pairing_brute(Da, Db)
        assert bott == want
        Wm = OM.pair_weights(Da, Db)
        assert len(set(pair)) == na and all(0 <= j < nb for j in pair)
        assert max(Wm[i][pair[i]] for i in range(na)) == want


def test_colocate_case1_and_config4_shapes():
    r = np.random.default_rng(9)
    for n in (4, 8, 16):
        A = r.integers(0, 30, size=(n, n)); A = A + A.T
        Bm = r.integers(0, 30, size=(n, n)); Bm = Bm + Bm.T
        sa, _ = OM.send_recv(A)
        sb, _ = OM.send_recv(Bm)
        assert P.colocate_match(A, Bm)[1] == OM.case1_value(sa, sb)        # Theorem 6
    # the two colocated models of the workload: 8 experts vs 16 experts on 8 GPUs (one expert each per GPU)
    Da = W.make_traffic_matrix(W.get_config("c4a_coloc"))["D"]
    pe = W.make_traffic_matrix(W.get_config("c4b_coloc"))["per_expert"]     # [8 GPUs, 16 experts]
    Db16 = np.zeros((16, 16), dtype=np.int64)
    Db16[:8, :] = pe                                                        # expert-level receive pattern
    pair, bott = P.colocate_match(Da, Db16)
    assert bott == OM.best_pairing_threshold(Da, Db16)[0]
    assert len(set(pair)) == 8


@pytest.mark.parametrize("hetero", [False, True])
def test_aurora_chunks_follow_the_library_rounds(hetero):
    """The decomposition into rounds is not unique, so chunk lists are checked against the rounds
    the library itself returned, with the properties the oracle's chunk lists are pinned to."""
    r = np.random.default_rng(77)
    for n in (2, 3, 5, 8, 16):
        for _ in range(3):
            D = random_D(r, n, hi=200)
            B = list(r.choice([1.0, 0.8, 0.5, 0.4], size=n)) if hetero else None
            plan = P.aurora_order(D, B)
            receivers = [dict() for _ in range(plan["n_rounds"])]
            for g in range(n):
                chunks = P.aurora_chunks(D, B, g)
                got = np.zeros(n, dtype=np.int64)
                cap = np.zeros(n)                                                  # tokens the rounds so far could carry to each destination
                rr = 0
                for dest, rows in chunks:
                    assert rows > 0 and dest != g
                    rate = 1.0 if B is None else min(B[g], B[dest])
                    got[dest] += rows
                    # the chunk belongs to the round at whose end the whole tokens sent so far reach its cumulative count
                    while True:
                        assert rr < plan["n_rounds"]
                        j = plan["dst"][rr][g]
                        if j >= 0:
                            cap[j] = min(cap[j] + plan["duration"][rr] * rate if j == dest else cap[j] + plan["duration"][rr] * min(1.0 if B is None else B[g], 1.0 if B is None else B[j]), D[g][j])
                        rr += 1
                        if j == dest and np.floor(cap[dest] + 1e-6) >= got[dest]:
                            break
                    assert np.floor(cap[dest] + 1e-6) == got[dest]                 # whole tokens of the cumulative amount, no more
                    assert receivers[rr - 1].setdefault(dest, g) == g              # contention-free
                want = np.array(D[g], dtype=np.int64)
                want[g] = 0
                assert np.array_equal(got, want)
    # the same lists as the oracle when the decomposition is forced: a permutation matrix has one round
    D = np.zeros((4, 4), dtype=np.int64)
    for i, j in enumerate([2, 3, 1, 0]):
        D[i, j] = 50 + i
    for g in range(4):
        assert P.aurora_chunks(D, None, g) == OS.chunks_from_rounds(D.tolist(), None, g)[0]


def test_aurora_chunks_argument_errors():
    D = np.array([[0, 3], [4, 0]], dtype=np.int64)
    with pytest.raises(P.MoeError):
        P.aurora_chunks(D, None, 2)
    with pytest.raises(P.MoeError):
        P.aurora_chunks(D, [1.0, -1.0], 0)


def test_aurora_assign_is_theorem3():
    r = np.random.default_rng(80)
    for n in (1, 2, 5, 8, 64, 256):
        for _ in range(4):
            load = r.integers(0, 50, size=n)                      # many ties
            perf = r.choice([1.0, 0.8, 0.5, 0.4], size=n)
            assert P.aurora_assign(load, perf) == OP.thm3_assign(load.tolist(), perf.tolist())
    with pytest.raises(P.MoeError):
        P.aurora_assign([1, 2], [1.0, 0.0])
    with pytest.raises(P.MoeError):
        P.aurora_assign([1, -2], [1.0, 1.0])


def test_bottleneck_assign_and_hetero_colocation_against_the_oracle():
    r = np.random.default_rng(81)
    for n in (1, 2, 3, 5, 6):
        for _ in range(6):
            Wt = r.integers(0, 25, size=(n, n)).astype(float)
            item, v = P.aurora_bottleneck_assign(Wt)
            assert sorted(item) == list(range(n))
            assert v == OP.bottleneck_assign_brute(Wt.tolist())[0] == max(Wt[g][item[g]] for g in range(n))
    for n in (2, 3, 4):
        for _ in range(5):
            Da, Db = random_D(r, n), random_D(r, n)
            perf = r.choice([1.0, 0.8, 0.5, 0.4], size=n)
            Wp = np.array(OM.pair_weights(Da.tolist(), Db.tolist()), dtype=float)
            fa, fb = Da.sum(0) - np.diag(Da), Db.sum(0) - np.diag(Db)
            time3 = ((fa[None, :, None] + fb[None, None, :]) + 2.0 * Wp[None]) / perf[:, None, None]
            pair, gpu, v = P.colocate_hetero_match(Da, Db, time3)
            assert sorted(pair) == list(range(n)) and sorted(gpu) == list(range(n))
            assert v == max(time3[gpu[i]][i][pair[i]] for i in range(n))
            # stage one attains the traffic bottleneck; stage two is optimal for the pairs it was given
            assert max(Wp[i][pair[i]] for i in range(n)) == OM.best_pairing_brute(Da.tolist(), Db.tolist())[0]
            W2 = [[time3[g][i][pair[i]] for i in range(n)] for g in range(n)]
            assert v == OP.bottleneck_assign_brute(W2)[0]
            assert v >= OP.optimum_3d(time3.tolist()) - 1e-12
    # a large instance finishes and is a valid matching
    n = 64
    Da, Db = random_D(r, n), random_D(r, n)
    time3 = r.random((n, n, n))
    pair, gpu, v = P.colocate_hetero_match(Da, Db, time3)
    assert sorted(pair) == list(range(n)) and sorted(gpu) == list(range(n))
    assert v == max(time3[gpu[i]][i][pair[i]] for i in range(n))


def test_time_model_against_the_oracle():
    r = np.random.default_rng(82)
    for _ in range(50):
        n = int(r.integers(1, 17))
        G, N, F, Cc, A = (r.random(n) * 10 for _ in range(5))
        assert P.aurora_layer_time(G, N, F, Cc, A) == pytest.approx(
            OP.layer_time(G.tolist(), N.tolist(), F.tolist(), Cc.tolist(), A.tolist()), rel=1e-15)
        v = [float(x) for x in r.integers(0, 20, size=9)]
        got = P.aurora_colocated_time(*v)
        ref = OP.colocated_time(*v)
        assert all(got[k] == ref[k] for k in got)
    assert P.aurora_colocated_time(1, 1, 10, 10, 1, 1, 1, 1, 2)["t"] == 24      # the compute-bound example worked by hand
    with pytest.raises(P.MoeError):
        P.aurora_colocated_time(1, 1, 1, 1, 1, 1, 1, 1, -1)


def test_tile_order_and_tail_plan_cover_every_tile_once():
    """The FFN's tile numbering (a bijection for every grid) and its K-split plan for a mostly empty
    last round, run on the host by the library's own self check."""
    import ctypes as C
    from paper_2410_17043_amd import _lib
    lib = _lib.load()
    lib.moe_selfcheck_tile_order.restype = C.c_int
    lib.moe_selfcheck_tile_order.argtypes = [C.c_int32] * 4
    split = 0
    for tiles_m in list(range(1, 70)) + [81, 89, 100, 255, 2393]:
        for tiles_n in (1, 2, 3, 4, 7, 8, 11, 16, 22, 112):
            for nk in (2, 32, 44, 64, 128, 448):
                parts = lib.moe_selfcheck_tile_order(tiles_m, tiles_n, 256, nk)
                assert parts >= 1, lib.moe_last_error()
                rem = (tiles_m * tiles_n) % 256
                if parts > 1:
                    split += 1
                    assert 0 < rem <= 128 and rem * parts <= 256 and nk // parts >= 16
                    assert parts >= 4 or nk // parts >= 64
    assert split > 100
    assert lib.moe_selfcheck_tile_order(81, 112, 256, 128) == 2       # first GEMM of the Mixtral-shape share
    assert lib.moe_selfcheck_tile_order(81, 16, 256, 448) == 8        # second GEMM
    assert lib.moe_selfcheck_tile_order(0, 4, 256, 8) < 0


def test_tile_map_gathers_the_segments_of_an_expert():
    """The FFN's tile map, built on the host by the library's own self check (which verifies that every row
    lies in exactly one tile of its expert): with gathering the tile count is what the rows per expert
    need, however the segments interleave; without it, what the runs of adjacent segments need."""
    import ctypes as C
    from paper_2410_17043_amd import _lib
    lib = _lib.load()
    fn = lib.moe_selfcheck_tile_map
    fn.restype = C.c_int
    fn.argtypes = [C.POINTER(C.c_int32), C.POINTER(C.c_int32)] + [C.c_int32] * 5

    def run(lens, experts, n_local, bm, gather, R=None):
        off = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
        ex = np.asarray(experts, dtype=np.int32)
        R = int(off[-1]) if R is None else R
        rc = fn(off.ctypes.data_as(C.POINTER(C.c_int32)), ex.ctypes.data_as(C.POINTER(C.c_int32)), len(lens), R, bm,
                n_local, gather)
        assert rc >= 0, lib.moe_last_error()
        return rc

    def need(lens, experts, n_local, bm, gather):
        if gather:
            return sum(-(-sum(l for l, e in zip(lens, experts) if e == x) // bm) for x in range(n_local))
        segs = [(l, e) for l, e in zip(lens, experts) if l > 0 or not 0 <= e < n_local]   # empty segments do not count
        total, i = 0, 0
        while i < len(segs):
            j = i
            while j < len(segs) and segs[j][1] == segs[i][1]:
                j += 1
            if 0 <= segs[i][1] < n_local:
                total += -(-sum(l for l, _ in segs[i:j]) // bm)
            i = j
        return total

    # the Switch-shape share: 16 sources x 4 local experts, at most 160 rows each (the capacity)
    lens = [160, 160, 150, 97] * 16
    experts = [0, 1, 2, 3] * 16
    assert run(lens, experts, 4, 256, 1) == need(lens, experts, 4, 256, 1) == 10 + 10 + 10 + 7
    assert run(lens, experts, 4, 256, 0) == 64
    r = np.random.default_rng(5)
    for _ in range(300):
        nseg = int(r.integers(0, 60))
        n_local = int(r.integers(1, 9))
        bm = int(r.choice([64, 256]))
        lens = [int(v) for v in r.choice([0, 1, 3, 100, 255, 256, 257, 700], size=nseg)]
        experts = [int(v) for v in r.integers(-1, n_local + 1, size=nseg)]       # -1 and n_local: skipped
        for gather in (0, 1):
            assert run(lens, experts, n_local, bm, gather) == need(lens, experts, n_local, bm, gather)
    # offsets past R are clamped; 1024 segments of one row each
    assert run([10, 10, 10], [0, 1, 0], 2, 256, 1, R=25) == 2
    assert run([1] * 1024, [i % 3 for i in range(1024)], 3, 256, 1) == 2 + 2 + 2
    assert run([1] * 1024, [i % 3 for i in range(1024)], 3, 256, 0) == 1024


def test_skinny_plan_and_row_geometry_self_checks():
    """Host logic of the weight-streaming FFN kernels and of the scatter's row sharing, checked by the library's own
    invariants over the whole range of shapes, plus the values the five workloads and a decode share get."""
    import ctypes as C
    from paper_2410_17043_amd import _lib
    lib = _lib.load()
    for total in list(range(1, 70)) + [111, 112, 127, 128, 129, 224, 255, 256, 257, 448, 1000]:
        for ns in (1, 2, 3, 4, 5, 7, 8, 11, 16, 32, 44, 100, 112, 113):
            for ncu in (256, 304, 64):
                parts = lib.moe_selfcheck_skinny_plan(total, ncu, ns)
                assert parts >= 1, (total, ncu, ns)
    assert lib.moe_selfcheck_skinny_plan(224, 256, 32) == 1       # first GEMM of a Mixtral-shape expert, 32 rows
    assert lib.moe_selfcheck_skinny_plan(32, 256, 112) == 8       # second GEMM: K = 14336 in 8 pieces of 14 stages
    assert lib.moe_selfcheck_skinny_plan(0, 256, 8) < 0
    out = (C.c_int32 * 3)()
    for row16 in list(range(1, 600)) + [1024, 1536, 4096, 65536]:
        for k in (1, 2, 3, 6, 8, 9, 16):
            assert lib.moe_selfcheck_row_geometry(row16, k, out) == 0, (row16, k, list(out))
    want = {(512, 2): (1, 1), (128, 1): (4, 1), (256, 2): (2, 1), (256, 6): (1, 1), (64, 2): (8, 1), (64, 6): (2, 1),
            (1024, 2): (1, 2), (576, 3): (1, 2), (16, 2): (1, 1)}
    for (row16, k), (tpw, pieces) in want.items():
        assert lib.moe_selfcheck_row_geometry(row16, k, out) == 0
        assert (out[0], out[2]) == (tpw, pieces), (row16, k, list(out))
    assert lib.moe_selfcheck_row_geometry(0, 2, out) < 0 and lib.moe_selfcheck_row_geometry(64, 17, out) < 0
