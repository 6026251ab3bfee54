"""Oracle for expert colocation by bottleneck matching (TEST INFRASTRUCTURE).

Sec. 6.2: for two models with traffic matrices D_a and D_b, expert i of model a
has send total a_i (off-diagonal row sum) and receive total a_{n+i} (off-diagonal
column sum), likewise b.  Colocating expert i of a with expert j of b loads that
GPU with max(a_i + b_j, a_{n+i} + b_{n+j}) (Eqn. 5 and the edge weight of Case II).
The best colocation minimises the largest such weight over all pairings.

`best_pairing_brute` is the definition written out (every injection tried);
`best_pairing_threshold` is an independent second route (grow the threshold until
a matching saturating model a exists).  Theorem 6 (`case1_value`) covers the case
send == receive on every GPU.

Pins (tests/test_oracle_matching.py): the two routes agree; Case I inputs give
Theorem 6's sorted pairing value; hand-computed 2 x 2 and 3 x 3 examples.
"""
from __future__ import annotations

import itertools


def send_recv(D):
    n = len(D)
    send = [sum(int(D[i][j]) for j in range(n) if j != i) for i in range(n)]
    recv = [sum(int(D[j][i]) for j in range(n) if j != i) for i in range(n)]
    return send, recv


def pair_weights(Da, Db):
    sa, ra = send_recv(Da)
    sb, rb = send_recv(Db)
    return [[max(sa[i] + sb[j], ra[i] + rb[j]) for j in range(len(Db))] for i in range(len(Da))]


def best_pairing_brute(Da, Db):
    """Minimum over every injection experts(a) -> experts(b) of the largest pair weight."""
    W = pair_weights(Da, Db)
    na, nb = len(Da), len(Db)
    best, best_pair = None, None
    for perm in itertools.permutations(range(nb), na):
        v = max(W[i][perm[i]] for i in range(na)) if na else 0
        if best is None or v < best:
            best, best_pair = v, list(perm)
    return best, best_pair


def best_pairing_threshold(Da, Db):
    """Smallest edge weight w such that edges of weight <= w contain a matching of all of a."""
    W = pair_weights(Da, Db)
    na, nb = len(Da), len(Db)
    for w in sorted({W[i][j] for i in range(na) for j in range(nb)}):
        match_b = [-1] * nb

        def aug(i, seen):
            for j in range(nb):
                if W[i][j] <= w and not seen[j]:
                    seen[j] = True
                    if match_b[j] < 0 or aug(match_b[j], seen):
                        match_b[j] = i
                        return True
            return False

        if all(aug(i, [False] * nb) for i in range(na)):
            pair = [-1] * na
            for j, i in enumerate(match_b):
                if i >= 0:
                    pair[i] = j
            return w, pair
    return 0, []


def case1_value(a, b):
    """Theorem 6: sort a ascending and b descending, pair in sequence; the largest sum."""
    return max(x + y for x, y in zip(sorted(a), sorted(b, reverse=True)))
