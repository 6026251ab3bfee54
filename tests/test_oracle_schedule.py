"""Pins of the scheduling oracle: the paper's worked example, closed forms, brute force."""
import os
from fractions import Fraction

import numpy as np
import pytest

from oracle import schedule as S

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "network_figure.txt")


def load_network_figure():
    kv = {}
    for line in open(GOLDEN):
        if line.startswith("#") or not line.strip():
            continue
        key, rest = line.split(None, 1)
        kv[key] = rest.strip()
    rows = lambda s: [[int(v) for v in r.split()] if r.strip() != "-" else [] for r in s.split("/")]
    return (rows(kv["D"]), rows(kv["order_naive"]), int(kv["time_naive"]), rows(kv["order_good"]),
            int(kv["time_good"]), int(kv["bmax"]))


def test_network_figure_example():
    D, naive, t_naive, good, t_good, bm = load_network_figure()
    assert S.simulate(D, None, naive) == t_naive
    assert S.simulate(D, None, good) == t_good
    assert S.bmax(D) == bm
    best, _ = S.brute_force_best_order(D)
    assert best == bm
    rnds, b = S.rounds(D)
    assert b == bm and sum(r[1] for r in rnds) == bm
    a = S.alg1_order(D)
    assert a["makespan"] == bm and S.simulate(D, None, a["dest_order"]) == bm


def test_bmax_closed_form_and_diagonal_ignored():
    D = [[99, 3, 4], [5, 99, 1], [2, 7, 99]]
    # rows 7, 6, 9; columns 7, 10, 5
    assert S.bmax(D) == 10
    assert S.bmax(D, [2, 2, 2]) == 5                         # uniform rate scales time
    assert S.bmax(D, [1, 1, 1]) == S.bmax(D)
    # heterogeneous: p_ij = d_ij / min(B_i, B_j)
    B = [1, 0.5, 0.25]
    rows = [3 / 0.5 + 4 / 0.25, 5 / 0.5 + 1 / 0.25, 2 / 0.25 + 7 / 0.25]
    cols = [5 / 0.5 + 2 / 0.25, 3 / 0.5 + 7 / 0.25, 4 / 0.25 + 1 / 0.25]
    assert S.bmax(D, B) == Fraction(max(rows + cols))
    assert S.port_bound(D, B) <= S.bmax(D, B)


def random_D(r, n, hi=12, zero_frac=0.3):
    D = r.integers(0, hi, size=(n, n))
    D[r.random((n, n)) < zero_frac] = 0
    return D


@pytest.mark.parametrize("hetero", [False, True])
def test_padding_and_round_invariants(hetero):
    r = np.random.default_rng(31)
    for n in (2, 3, 4, 5, 8):
        for _ in range(6):
            D = random_D(r, n)
            B = list(r.choice([1.0, 0.8, 0.5, 0.4], size=n)) if hetero else None
            P = S.scaled_matrix(D, B)
            X, bm = S.pad_to_uniform(P)
            assert bm == S.bmax(D, B)
            assert all(v >= 0 for row in X for v in row)
            for i in range(n):
                assert sum(P[i]) + sum(X[i]) == bm
                assert sum(P[j][i] + X[j][i] for j in range(n)) == bm
            rnds, b2 = S.rounds(D, B)
            assert b2 == bm
            assert sum(tau for _, tau, _ in rnds) == bm                    # attains the bound exactly
            assert len(rnds) <= max(1, n * n - 2 * n + 2)
            sent = [[Fraction(0)] * n for _ in range(n)]
            for dst, tau, real in rnds:
                live = [j for j in dst if j >= 0]
                assert len(live) == len(set(live))                          # one sender per receiver
                for i, j in enumerate(dst):
                    assert (j >= 0) == (real[i] > 0) and real[i] <= tau
                    if j >= 0:
                        assert i != j
                        sent[i][j] += real[i]
            assert sent == P                                                # everything delivered once


@pytest.mark.parametrize("hetero", [False, True])
def test_chunk_lists_follow_the_rounds(hetero):
    r = np.random.default_rng(41)
    for n in (2, 3, 5, 8):
        for _ in range(4):
            D = random_D(r, n)
            B = list(r.choice([1.0, 0.8, 0.5, 0.4], size=n)) if hetero else None
            rnds, bm = S.rounds(D, B)
            per_round_receivers = [dict() for _ in rnds]
            for g in range(n):
                chunks, which = S.chunks_from_rounds(D, B, g)
                assert which == sorted(which) and len(set(which)) == len(which)    # at most one chunk per round
                got = [0] * n
                for (j, rows), rr in zip(chunks, which):
                    dst, tau, real = rnds[rr]
                    assert j == dst[g] and j != g and rows > 0
                    rate = Fraction(1) if B is None else min(Fraction(B[g]), Fraction(B[j]))
                    assert rows < tau * rate + 1                                    # fits the round, up to one token of rounding
                    got[j] += rows
                    assert per_round_receivers[rr].setdefault(j, g) == g            # nobody else sends to j in that round
                assert got == [0 if j == g else D[g][j] for j in range(n)]          # every token exactly once
            if not hetero:
                # integer traffic on unit links: rounds have whole durations and a chunk is exactly its round's share
                for g in range(n):
                    chunks, which = S.chunks_from_rounds(D, B, g)
                    for (j, rows), rr in zip(chunks, which):
                        assert rows == rnds[rr][2][g]


def test_bmax_is_a_lower_bound_and_brute_force_meets_it_when_unit_flows():
    r = np.random.default_rng(32)
    for n in (3, 4):
        for _ in range(4):
            D = random_D(r, n, hi=6)
            best, _ = S.brute_force_best_order(D)
            assert best >= S.bmax(D)
    # unit-size flows on a full mesh: a cyclic shift order meets the bound with whole flows
    n = 4
    D = [[0 if i == j else 1 for j in range(n)] for i in range(n)]
    best, _ = S.brute_force_best_order(D)
    assert best == S.bmax(D) == n - 1


@pytest.mark.parametrize("hetero", [False, True])
def test_alg1_reading_is_valid(hetero):
    r = np.random.default_rng(33)
    for n in (2, 3, 4, 6):
        for _ in range(8):
            D = random_D(r, n)
            B = list(r.uniform(0.5, 1.0, size=n)) if hetero else None
            P = S.scaled_matrix(D, B)
            a = S.alg1_order(D, B)
            st = a["start"]
            for i in range(n):
                assert sorted(a["dest_order"][i]) == list(range(n)) and a["dest_order"][i][-1] == i
                for j in range(n):
                    assert (st[i][j] is not None) == (P[i][j] > 0)          # complete
            for i in range(n):                                              # contention-free
                for tl in ([(st[i][j], st[i][j] + P[i][j]) for j in range(n) if st[i][j] is not None],
                           [(st[j][i], st[j][i] + P[j][i]) for j in range(n) if st[j][i] is not None]):
                    tl.sort()
                    assert all(a1 >= b0 for (_, b0), (a1, _) in zip(tl[:-1], tl[1:]))
            assert a["makespan"] >= S.bmax(D, B)


def test_simulate_hand_cases():
    # two senders into one receiver share its port: 2 + 2 tokens at rate 1/2 each -> 4
    D = [[0, 0, 2], [0, 0, 2], [0, 0, 0]]
    assert S.simulate(D, None, [[2], [2], []]) == 4
    # a slow receiver bounds the flow; a slow sender likewise
    assert S.simulate([[0, 6], [0, 0]], [1, 0.5], [[1], []]) == 12
    assert S.simulate([[0, 6], [0, 0]], [0.25, 1], [[1], []]) == 24
    # staggered finish: flows of 1 and 3 into one receiver: both at 1/2 until t = 2, then the rest alone
    D = [[0, 0, 1], [0, 0, 3], [0, 0, 0]]
    assert S.simulate(D, None, [[2], [2], []]) == 4
