"""Pins of the planning oracle (Theorem 3, the two-stage matching of Sec. 7.2, Eqn. 1-4 and
Table 2) to facts that do not come from the oracle itself."""
import itertools

import numpy as np
import pytest

from oracle import matching as OM
from oracle import planning as OP

# per-GPU times that grow with the tokens and shrink with the performance (the premise of
# Theorem 3, with its footnote: a faster GPU never has the slower link)
TIME_FNS = [
    lambda load, perf: load / perf,
    lambda load, perf: (load + 7.0) / perf,
    lambda load, perf: load / perf + load / (40.0 + 60.0 * perf) + 3.0 / perf,
]


def test_thm3_hand_example_and_ties():
    # loads 9 > 5 > 1 meet performances 2.0 > 1.0 > 0.5
    assert OP.thm3_assign([5, 9, 1], [1.0, 0.5, 2.0]) == [0, 2, 1]
    assert OP.thm3_assign([4, 4, 4], [1.0, 1.0, 1.0]) == [0, 1, 2]            # all tied: identity
    assert OP.thm3_assign([4, 8, 4], [1.0, 3.0, 1.0]) == [0, 1, 2]
    assert OP.thm3_assign([7], [0.3]) == [0]


@pytest.mark.parametrize("fn", range(len(TIME_FNS)))
def test_thm3_attains_the_brute_force_optimum(fn):
    r = np.random.default_rng(50 + fn)
    time_fn = TIME_FNS[fn]
    for n in (2, 3, 4, 5, 6):
        for _ in range(6):
            load = [int(v) for v in r.integers(0, 500, size=n)]
            perf = [float(v) for v in r.choice([1.0, 0.8, 0.5, 0.4], size=n)]
            a = OP.thm3_assign(load, perf)
            assert sorted(a) == list(range(n))
            t = OP.assignment_time(load, perf, a, time_fn)
            assert t == pytest.approx(OP.best_assign_brute(load, perf, time_fn), rel=1e-12)
            # the exchange argument of the proof: no swap of two experts does better
            for e1, e2 in itertools.combinations(range(n), 2):
                b = list(a)
                b[e1], b[e2] = b[e2], b[e1]
                assert OP.assignment_time(load, perf, b, time_fn) >= t - 1e-12


def test_bottleneck_assignment_two_routes_agree():
    r = np.random.default_rng(60)
    for n in (1, 2, 3, 4, 5, 6):
        for _ in range(8):
            W = r.integers(0, 30, size=(n, n)).astype(float).tolist()
            vb, _ = OP.bottleneck_assign_brute(W)
            vt, item = OP.bottleneck_assign_threshold(W)
            assert vb == vt
            assert sorted(item) == list(range(n))
            assert max(W[g][item[g]] for g in range(n)) == vt
    # by hand: the cheap diagonal is blocked by one expensive entry
    W = [[1, 9, 9], [9, 1, 9], [9, 9, 50]]
    assert OP.bottleneck_assign_threshold(W)[0] == 9


def random_D(r, n):
    D = r.integers(0, 60, size=(n, n))
    np.fill_diagonal(D, 0)
    return D.tolist()


def test_two_stage_against_the_3d_optimum():
    r = np.random.default_rng(61)
    ratios = []
    for n in (2, 3, 4):
        for _ in range(6):
            Da, Db = random_D(r, n), random_D(r, n)
            perf = [float(v) for v in r.choice([1.0, 0.8, 0.5, 0.4], size=n)]
            Wp = OM.pair_weights(Da, Db)
            fa = [sum(Da[i][j] for i in range(n)) for j in range(n)]         # tokens expert j of a processes
            fb = [sum(Db[i][j] for i in range(n)) for j in range(n)]
            time3 = [[[(fa[i] + fb[j]) / perf[g] + 2.0 * Wp[i][j] / perf[g] for j in range(n)] for i in range(n)]
                     for g in range(n)]
            v, pair, gpu = OP.two_stage(Da, Db, time3)
            assert sorted(pair) == list(range(n)) and sorted(gpu) == list(range(n))
            assert v == max(time3[gpu[i]][i][pair[i]] for i in range(n))
            opt = OP.optimum_3d(time3)
            assert v >= opt - 1e-12                                           # decoupling can only lose
            ratios.append(v / opt)
            # GPUs alike and time = the pair weight: both stages collapse to Case II, which is optimal
            same = [[[float(Wp[i][j]) for j in range(n)] for i in range(n)] for _ in range(n)]
            v2, _, _ = OP.two_stage(Da, Db, same)
            assert v2 == OP.optimum_3d(same) == OM.best_pairing_brute(Da, Db)[0]
    assert min(ratios) == pytest.approx(1.0)                                  # often optimal


def test_eqn1_by_hand_and_its_collapse_to_eqn2():
    # two GPUs: max(G+N) = 6, max(F+C) = 7, max A = 1
    assert OP.layer_time([1, 1], [3, 5], [2, 4], [5, 3], [1, 1]) == 14
    # Eqn. 2 treats the maxima separately: 1 + 5 + 4 + 5 + 1
    assert OP.layer_time_homogeneous(1, [3, 5], [2, 4], [5, 3], 1) == 16
    r = np.random.default_rng(62)
    for _ in range(50):
        n = int(r.integers(1, 9))
        g, a = float(r.random()), float(r.random())
        N = r.random(n).tolist()
        tokens = r.random(n)
        F, C = (3.0 * tokens).tolist(), (0.5 * tokens).tolist()               # observation (3): both grow with the tokens
        e1 = OP.layer_time([g] * n, N, F, C, [a] * n)
        assert e1 == pytest.approx(OP.layer_time_homogeneous(g, N, F, C, a), rel=1e-12)
        # without observation (3) Eqn. 2 is only an upper bound of Eqn. 1
        C2 = r.random(n).tolist()
        assert OP.layer_time([g] * n, N, F, C2, [a] * n) <= OP.layer_time_homogeneous(g, N, F, C2, a) + 1e-12


def test_table2_by_hand():
    # compute-bound: the GPU never idles, so the inference time is the sum of all compute
    E = OP.colocated_time(Ga=1, Gb=1, Fa=10, Fb=10, Aa=1, Ab=1, Na=1, Nb=1, NaNb=2)
    assert (E["Fa"], E["Nb"], E["Fb"], E["Ca"], E["Aa"], E["Cb"], E["Ab"], E["t"]) == (11, 2, 21, 12, 22, 22, 23, 24)
    assert OP.utilisation(1 + 10 + 10 + 1 + 1 + 1, E["t"]) == 1.0
    # communication-bound: every communication entry is the table's aggregated duration
    E = OP.colocated_time(Ga=1, Gb=1, Fa=1, Fb=1, Aa=1, Ab=1, Na=10, Nb=10, NaNb=18)
    assert (E["Na"], E["Nb"], E["Ca"], E["Cb"]) == (10, 18, 28, 36)
    assert (E["Fa"], E["Fb"], E["Aa"], E["Ab"], E["t"]) == (11, 19, 29, 37, 38)
    assert OP.utilisation(6, E["t"]) == pytest.approx(6 / 38)


def test_table2_special_cases_and_monotonicity():
    r = np.random.default_rng(63)
    names = ["Ga", "Gb", "Fa", "Fb", "Aa", "Ab", "Na", "Nb", "NaNb"]
    for _ in range(200):
        v = {k: float(r.integers(0, 20)) for k in names}
        v["NaNb"] = max(v["Na"], v["Nb"]) + float(r.integers(0, 10))           # aggregated >= each part
        v["NaNb"] = min(v["NaNb"], v["Na"] + v["Nb"])
        E = OP.colocated_time(**v)
        # computation competition: the GPU's six computations never overlap
        assert E["t"] >= v["Gb"] + v["Fa"] + v["Fb"] + v["Aa"] + v["Ab"] + v["Ga"]
        # every component ends after it may start plus its own length
        assert E["Ca"] >= E["Fa"] + v["Na"] and E["Cb"] >= E["Fb"] + v["Nb"] and E["Nb"] >= v["Gb"] + v["Nb"]
        for k in names:                                                        # longer parts never shorten the layer
            w = dict(v)
            w[k] += 1.0
            assert OP.colocated_time(**w)["t"] >= E["t"]
        # model b empty: Eqn. 2 of model a alone (its gate closes the cycle)
        alone = OP.colocated_time(Ga=v["Ga"], Gb=0, Fa=v["Fa"], Fb=0, Aa=v["Aa"], Ab=0, Na=v["Na"], Nb=0, NaNb=v["Na"])
        assert alone["t"] == OP.layer_time_homogeneous(v["Ga"], [v["Na"]], [v["Fa"]], [v["Na"]], v["Aa"])
