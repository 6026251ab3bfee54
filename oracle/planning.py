"""Oracle for GPU assignment, the two-stage matching of the heterogeneous colocation
case and the inference-time expressions (TEST INFRASTRUCTURE).

Theorem 3 (Sec. 5.1): experts sorted by the number of tokens they process,
descending, go to GPUs sorted from the highest to the lowest performance.
`thm3_assign` is that sentence; `best_assign_brute` tries every assignment under
a caller-supplied per-GPU time.

Sec. 7.2: the optimum is a 3-dimensional matching (one GPU, one expert of model a,
one expert of model b per hyperedge, weight = inference time on that GPU), minimise
the largest weight: `optimum_3d` tries everything.  The paper's sub-optimal method
decouples it: first the expert-expert bottleneck matching of Sec. 6.2 Case II,
then a bottleneck matching between GPUs and the pairs found, the edge weight being
the inference time of the pair on that GPU: `two_stage`.  The paper does not print a
formula for that time; here it is an input, a table time3[g][i][j].

Eqn. 1-3 (Sec. 4.1) and Table 2 with Eqn. 4 (Sec. 6.1) are written out in
`layer_time`, `layer_time_homogeneous` and `colocated_time`.
Reading taken for Table 2: its end times of the communication components are
aggregated DURATIONS (|N^a + N^b| and so on); read as absolute times they can end
before the component is allowed to start (C^a may not start before F^a ends), and
with model b empty they would drop |C^a| from Eqn. 2.  A communication component
therefore ends at the later of the table's entry and its earliest start plus its own
duration.  The aggregated durations follow the text under the table:
|N^a + N^b + C^a| = |N^a + N^b| + |C^a| and |C^a + C^b| = |N^a + N^b|.

Pins (tests/test_oracle_planning.py): brute force over all assignments for several
monotone time functions; exchange argument of the proof; stage two against brute
force over permutations; two_stage >= optimum_3d with equality when GPUs are alike;
Eqn. 1 collapsing to Eqn. 2 and 3 under the three observations of Sec. 4.1; Table 2
by hand on a communication-bound and on a compute-bound example; model b empty gives
Eqn. 2; monotonicity in every duration.
"""
from __future__ import annotations

import itertools

from . import matching


# ------------------------------------------------------------------ Theorem 3
def thm3_assign(load, perf):
    """expert_to_gpu: the expert with the r-th largest load goes to the GPU with the
    r-th highest performance (ties: lower index first, on both sides)."""
    n = len(load)
    experts = sorted(range(n), key=lambda e: (-load[e], e))
    gpus = sorted(range(n), key=lambda g: (-perf[g], g))
    out = [0] * n
    for e, g in zip(experts, gpus):
        out[e] = g
    return out


def assignment_time(load, perf, assign, time_fn):
    """Layer time of an assignment: the slowest GPU (strict barrier between layers)."""
    return max(time_fn(load[e], perf[assign[e]]) for e in range(len(load)))


def best_assign_brute(load, perf, time_fn):
    n = len(load)
    return min(assignment_time(load, perf, list(p), time_fn) for p in itertools.permutations(range(n)))


# ------------------------------------------------------------------ Sec. 7.2
def bottleneck_assign_brute(W):
    """min over permutations s of max_g W[g][s[g]] (rows: GPUs, columns: items)."""
    n = len(W)
    best, arg = None, None
    for s in itertools.permutations(range(n)):
        v = max(W[g][s[g]] for g in range(n)) if n else 0
        if best is None or v < best:
            best, arg = v, list(s)
    return best, arg


def bottleneck_assign_threshold(W):
    """Second route: smallest weight w whose edges <= w hold a perfect matching."""
    n = len(W)
    for w in sorted({W[g][c] for g in range(n) for c in range(n)}):
        match_c = [-1] * n

        def aug(g, seen):
            for c in range(n):
                if W[g][c] <= w and not seen[c]:
                    seen[c] = True
                    if match_c[c] < 0 or aug(match_c[c], seen):
                        match_c[c] = g
                        return True
            return False

        if all(aug(g, [False] * n) for g in range(n)):
            item = [-1] * n
            for c, g in enumerate(match_c):
                item[g] = c
            return w, item
    return 0, []


def two_stage(Da, Db, time3):
    """The decoupled method: pair[i] = expert of b colocated with expert i of a (Case II on the
    traffic alone), then GPUs against pairs with weight time3[g][i][pair[i]].
    Returns (value, pair, gpu_of_pair)."""
    _, pair = matching.best_pairing_threshold(Da, Db)
    n = len(Da)
    W = [[time3[g][i][pair[i]] for i in range(n)] for g in range(n)]
    value, item_of_gpu = bottleneck_assign_threshold(W)
    gpu_of_pair = [0] * n
    for g, i in enumerate(item_of_gpu):
        gpu_of_pair[i] = g
    return value, pair, gpu_of_pair


def optimum_3d(time3):
    """The 3-dimensional bottleneck matching by exhaustion (small n only)."""
    n = len(time3)
    best = None
    for pair in itertools.permutations(range(n)):
        for gpu in itertools.permutations(range(n)):
            v = max(time3[gpu[i]][i][pair[i]] for i in range(n))
            if best is None or v < best:
                best = v
    return best


# ------------------------------------------------------------------ Eqn. 1-3
def layer_time(G, N, F, C, A):
    """Eqn. 1: max_i(|G_i| + |N_i|) + max_j(|F_j| + |C_j|) + max_k |A_k|."""
    n = len(G)
    return max(G[i] + N[i] for i in range(n)) + max(F[j] + C[j] for j in range(n)) + max(A)


def layer_time_homogeneous(G, N, F, C, A):
    """Eqn. 2 (= Eqn. 3): |G| + max|N_i| + max|F_j| + max|C_j| + |A| with scalar G and A."""
    return G + max(N) + max(F) + max(C) + A


def utilisation(compute, inference_time):
    """Sec. 8.1: computation time (Gate, FFN, Aggregation) over inference time."""
    return compute / inference_time


# ------------------------------------------------------------------ Table 2, Eqn. 4
def colocated_time(Ga, Gb, Fa, Fb, Aa, Ab, Na, Nb, NaNb):
    """End times of Table 2 and the inference time of Eqn. 4 for two colocated models.

    Scalars are the maxima over GPUs the table uses.  Na and Nb are the stand-alone
    durations of the two models' first all-to-all, NaNb the aggregated duration
    |N^a + N^b| (the bound of Theorem 2 on the summed traffic matrix).  The second
    all-to-all is the first one reversed (Sec. 2.2), and the bound of Theorem 2 does not
    change under transposition, so |C^a| = |N^a|, |C^b| = |N^b| and |C^a + C^b| = |N^a + N^b|.
    Returns a dict of end times and 't' = E_{A^b} + |G^a|.
    """
    Ca, Cb = Na, Nb
    E = {}
    E["Gb"] = Gb
    E["Na"] = Na
    E["Fa"] = max(Gb, Na) + Fa
    E["Nb"] = max(NaNb, Gb + Nb)                       # starts >= |G^b|
    E["Fb"] = max(E["Fa"], E["Nb"]) + Fb
    E["Ca"] = max(NaNb + Ca, E["Fa"] + Ca)             # |N^a+N^b+C^a| = |N^a+N^b| + |C^a|; starts >= E_{F^a}
    E["Aa"] = max(E["Fb"], E["Ca"]) + Aa
    E["Cb"] = max(NaNb + NaNb, E["Fb"] + Cb)           # |N^a+N^b+C^a+C^b| = 2 |N^a+N^b|; starts >= E_{F^b}
    E["Ab"] = max(E["Aa"], E["Cb"]) + Ab
    E["Ga"] = E["Ab"] + Ga
    E["t"] = E["Ga"]
    return E
