"""Pins of the colocation oracle: definition by brute force vs an independent route, Theorem 6."""
import numpy as np
import pytest

from oracle import matching as M


def sym(r, n, hi=30):
    A = r.integers(0, hi, size=(n, n))
    return A + A.T            # send == receive on every GPU (Case I)


def test_hand_cases():
    # 2 x 2: sends a = (5, 1), b = (4, 2) with symmetric matrices -> pair big with small: max(5+2, 1+4) = 7
    Da = [[0, 5], [1, 0]]
    Db = [[0, 4], [2, 0]]
    # a: send (5, 1), recv (1, 5); b: send (4, 2), recv (2, 4)
    W = M.pair_weights(Da, Db)
    assert W == [[max(9, 3), max(7, 5)], [max(5, 7), max(3, 9)]]
    assert M.best_pairing_brute(Da, Db)[0] == 7
    assert M.send_recv([[9, 1, 2], [3, 9, 4], [5, 6, 9]]) == ([3, 7, 11], [8, 7, 6])   # diagonal ignored


def test_two_routes_agree_square_and_rectangular():
    r = np.random.default_rng(41)
    for na, nb in [(1, 1), (2, 2), (3, 3), (4, 4), (5, 5), (6, 6), (2, 4), (3, 4), (3, 7), (4, 8)]:
        for _ in range(5):
            Da, Db = r.integers(0, 40, size=(na, na)), r.integers(0, 40, size=(nb, nb))
            vb, pb = M.best_pairing_brute(Da, Db)
            vt, pt = M.best_pairing_threshold(Da, Db)
            assert vb == vt
            W = M.pair_weights(Da, Db)
            for p in (pb, pt):
                assert len(set(p)) == na and all(0 <= j < nb for j in p)
                assert max(W[i][p[i]] for i in range(na)) == vb


def test_case1_is_theorem6_sorted_pairing():
    r = np.random.default_rng(42)
    for n in (2, 3, 4, 5, 6, 7):
        for _ in range(5):
            Da, Db = sym(r, n), sym(r, n)
            sa, ra = M.send_recv(Da)
            sb, rb = M.send_recv(Db)
            assert sa == ra and sb == rb
            assert M.best_pairing_brute(Da, Db)[0] == M.case1_value(sa, sb)
    assert M.case1_value([1, 5, 9], [2, 4, 8]) == max(1 + 8, 5 + 4, 9 + 2)
