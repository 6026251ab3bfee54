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


def test_port_bound_hand_value():
    # off-diagonal row sums 7, 6, 9 and column sums 7, 10, 5 of the matrix below; rates 1, 1/2, 1/4.
    # Every port carries its own traffic at its own rate: sends 7/1, 6/(1/2), 9/(1/4) = 7, 12, 36;
    # receives 7/1, 10/(1/2), 5/(1/4) = 7, 20, 20.
    D = [[99, 3, 4], [5, 99, 1], [2, 7, 99]]
    B = [1, Fraction(1, 2), Fraction(1, 4)]
    assert S.port_bound(D, B) == 36
    assert S.port_bound(D) == 10 == S.bmax(D)
    # a flow runs at the slower end's rate, so Theorem 4's bound is the larger one: row 2 is 2/(1/4) + 7/(1/4)
    assert S.bmax(D, B) == 36
    # rates 1, 1/4, 1: the ports see 7, 24, 9 / 7, 40, 5; the scaled matrix has column 1 = 3/(1/4) + 7/(1/4)
    assert S.port_bound(D, [1, Fraction(1, 4), 1]) == 40 == S.bmax(D, [1, Fraction(1, 4), 1])
    # a slow sender into fast receivers: ports 2 -> 9/(1/4) = 36 sends; scaled column 0 = 5 + 2/(1/4) = 13
    assert S.port_bound(D, [1, 1, Fraction(1, 4)]) == 36
    assert S.bmax(D, [1, 1, Fraction(1, 4)]) == 36


def test_alg1_cases_worked_by_hand():
    # Four GPUs, unit rates.  Off-diagonal row sums 7, 6, 8, 6; column sums 6, 10, 6, 5: GPU 1 is the
    # bottleneck and its receiving side binds (10 = b_max), so the flows INTO GPU 1 go first, back to back in
    # ascending sender: 0->1 [0,4), 2->1 [4,9), 3->1 [9,10).  Left to send: GPU 1 6, GPU 3 5, GPUs 0 and 2 3
    # each, which is the order in which they arrange their flows.
    #  GPU 1: all three flows could start at 0; columns 0 and 2 are equally loaded (6 > column 3's 5), the
    #         larger flow wins: 1->0 [0,3); then 1->2 (column 6) before 1->3 (column 5): [3,4), [4,6).
    #  GPU 3: 3->2 fits [0,3) in front of GPU 2's busy [3,4); 3->0 must wait for GPU 0's port: [3,5).
    #  GPU 0: sends from 4 on; 0->2 [4,6); 0->3 waits for GPU 3's port (busy [4,6)): [6,7).
    #  GPU 2: 2->3 [0,2); 2->0 finds GPU 0's port busy until 5, then its own port busy [4,9): [9,10).
    D = [[0, 4, 2, 1], [3, 0, 1, 2], [1, 5, 0, 2], [2, 1, 3, 0]]
    a = S.alg1_order(D)
    assert a["start"] == [[None, 0, 4, 6], [0, None, 3, 4], [9, 4, None, 0], [3, 9, 0, None]]
    assert a["dest_order"] == [[1, 2, 3, 0], [0, 2, 3, 1], [3, 1, 0, 2], [2, 0, 1, 3]]
    assert a["makespan"] == 10 == S.bmax(D)
    # Three GPUs, every flow one unit: all loads equal, so GPU 0 is the bottleneck (lowest index), its sending
    # side counts as binding (row sum >= column sum): 0->1 [0,1), 0->2 [1,2).  GPUs 1 and 2 both have 2 left; GPU 1
    # first.  Its two flows could both start at 0, columns and sizes are equal, the lower destination wins:
    # 1->0 [0,1), then 1->2 behind GPU 2's busy [1,2): [2,3).  GPU 2: both flows can start at 1, the lower
    # destination first: 2->0 [1,2), 2->1 [2,3).
    D3 = [[0, 1, 1], [1, 0, 1], [1, 1, 0]]
    a = S.alg1_order(D3)
    assert a["start"] == [[None, 0, 1], [0, None, 2], [1, 2, None]]
    assert a["makespan"] == 3                                  # the lowest-index rule costs a unit here (b_max is 2)
    # GPU 0 sends 3 and receives 3 (the largest load, a tie between its two sides): the sending side is arranged
    # first, 0->1 [0,2), 0->2 [2,3).  Then GPU 2 (2 left): 2->0 [0,2); GPU 1: 1->0 behind it, [2,3).
    D3b = [[0, 2, 1], [1, 0, 0], [2, 0, 0]]
    a = S.alg1_order(D3b)
    assert a["start"] == [[None, 0, 2], [2, None, None], [0, None, None]]
    assert a["makespan"] == 3 == S.bmax(D3b)


@pytest.mark.parametrize("hetero", [False, True])
def test_alg1_transmission_at_the_bottleneck_is_continuous(hetero):
    # Sec. 4.2, the paragraph in front of Algorithm 1: data transmission at the bottleneck GPU should be
    # continuous, and by Theorem 2 it lasts b_max.  On the binding side of the GPU with the largest load the
    # planned flows must therefore tile [0, b_max) without a gap or an overlap.
    r = np.random.default_rng(35)
    for n in (2, 3, 4, 6, 9):
        for _ in range(8):
            D = random_D(r, n, hi=20)
            B = [Fraction(int(v), 10) for v in r.integers(4, 11, size=n)] if hetero else None
            P = S.scaled_matrix(D, B)
            bm = S.bmax(D, B)
            if bm == 0:
                continue
            rows = [sum(P[i]) for i in range(n)]
            cols = [sum(P[i][j] for i in range(n)) for j in range(n)]
            b = min(i for i in range(n) if max(rows[i], cols[i]) == bm)
            st = S.alg1_order(D, B)["start"]
            if rows[b] >= cols[b]:
                tl = sorted((st[b][j], st[b][j] + P[b][j]) for j in range(n) if P[b][j] > 0)
            else:
                tl = sorted((st[j][b], st[j][b] + P[j][b]) for j in range(n) if P[j][b] > 0)
            assert tl[0][0] == 0 and tl[-1][1] == bm
            assert all(nxt[0] == prev[1] for prev, nxt in zip(tl[:-1], tl[1:]))


@pytest.mark.parametrize("hetero", [False, True])
def test_list_order_replays_under_simulate_and_send_order_is_the_best_candidate(hetero):
    r = np.random.default_rng(36)
    for n in (2, 3, 4, 6, 8):
        for _ in range(5):
            D = random_D(r, n, hi=20)
            B = [Fraction(int(v), 10) for v in r.integers(4, 11, size=n)] if hetero else None
            order, t = S.list_order(D, B)
            # two event loops written separately (one chooses flows while it runs, the other replays a given
            # order) must agree on the completion time
            assert S.simulate(D, B, order) == t
            cands = [S.alg1_order(D, B)["dest_order"], S.rounds_order(D, B), order, S.shift_order(n)]
            so = S.send_order(D, B)
            assert so["candidate_times"] == [S.simulate(D, B, c) for c in cands]
            assert so["time"] == S.simulate(D, B, so["dest_order"]) <= min(so["candidate_times"])
            assert so["time"] >= S.port_bound(D, B)
            if not hetero:
                assert so["time"] >= S.bmax(D)
            for i, row in enumerate(so["dest_order"]):
                assert sorted(row) == list(range(n)) and row[-1] == i
            for c in cands:
                assert all(sorted(row) == list(range(n)) for row in c)
            # with no evaluation budget the improvement step changes nothing
            assert S.send_order(D, B, max_evals=0)["time"] == min(so["candidate_times"])


def load_order_ratios():
    path = os.path.join(os.path.dirname(__file__), "golden", "order_ratios.txt")
    out = []
    for line in open(path):
        if line.startswith("#") or not line.strip():
            continue
        d, b, bm, best, alg1, send = [f.strip() for f in line.split("|")]
        D = [[int(v) for v in row.split()] for row in d.split("/")]
        B = None if b == "-" else [Fraction(v) for v in b.split()]
        out.append((D, B, Fraction(bm), Fraction(best), Fraction(alg1), Fraction(send)))
    return out


def test_orders_against_the_stored_brute_force_optimum():
    # tests/golden/order_ratios.txt holds, for 24 seeded matrices on 3 and 4 GPUs (half of them with the link
    # rates of Sec. 8.1), the smallest completion time over every combination of whole-flow orders.  Algorithm 1's
    # order and the chosen send order are compared with it: never better than the optimum, not worse than what
    # was recorded, and the send order equal to the optimum wherever it was when the file was written.
    cases = load_order_ratios()
    assert len(cases) == 24
    at_optimum, alg1_at_optimum, worst = 0, 0, Fraction(1)
    for k, (D, B, bm, best, alg1, send) in enumerate(cases):
        assert S.bmax(D, B) == bm
        a = S.simulate(D, B, S.alg1_order(D, B)["dest_order"])
        s = S.send_order(D, B)["time"]
        assert best <= s <= send and best <= a <= alg1, k
        assert s <= a, k
        if send == best:
            assert s == best, k
            at_optimum += 1
        alg1_at_optimum += a == best
        worst = max(worst, s / best)
        if k < 2:                                         # the stored optimum itself, where enumeration is cheap (8 orders)
            assert S.brute_force_best_order(D, B)[0] == best
    assert at_optimum == 20 and alg1_at_optimum == 8
    assert worst == Fraction(26, 22)
