"""Oracle for the all-to-all transmission planning (TEST INFRASTRUCTURE).

Follows Sec. 4.2 (Theorem 2, Algorithm 1), Appendix A (the padding construction
D + X = D' and the slot-by-slot argument) and Sec. 5.2 / Appendix B (Theorem 4,
the heterogeneous extension).  All arithmetic is exact: token counts are
integers and link rates are converted to `fractions.Fraction`, so invariants such
as "the round durations sum to b_max" can be asserted with equality.

Network model (Sec. 2.4): one non-blocking switch, GPU i attached by one port of
rate B_i in each direction.

Pins (tests/test_oracle_schedule.py): the three-GPU example of the network figure
(3 time units for the naive order, 2 for the reordered one, b_max = 2), the
closed form against brute force over every per-source order for n <= 4, padding
and round invariants, homogeneous reduction of the heterogeneous bound, hand
arithmetic for the per-port bound.

`alg1_order`: Algorithm 1 does not say how tokens are arranged "to avoid
conflicts"; the rule used here is a stated reading.  Pinned about it: what the
text in front of the algorithm fixes (transmission at the bottleneck GPU runs
without a gap from time 0 for exactly b_max), validity (complete,
contention-free), two cases worked by hand that exercise the sort direction
and every tie-break, and its distance from the brute-force optimum on stored
seeded matrices (tests/golden/order_ratios.txt).  What no pin can decide is
whether the authors' own implementation breaks ties the same way: the paper
does not say.

`send_order` is what the library hands to the send buffer: the best of four
whole-flow orders under `simulate`, improved by adjacent exchanges.
"""
from __future__ import annotations

import itertools
from fractions import Fraction


def scaled_matrix(D, B=None):
    """p_ij = d_ij / min(B_i, B_j) off the diagonal, 0 on it (Appendix B; B = 1 gives Sec. 4.2)."""
    n = len(D)
    Bf = [Fraction(1)] * n if B is None else [Fraction(b) for b in B]
    return [[Fraction(0) if i == j else Fraction(int(D[i][j])) / min(Bf[i], Bf[j])
             for j in range(n)] for i in range(n)]


def bmax(D, B=None):
    """Theorem 2 / Theorem 4: the largest row or column sum of the scaled matrix."""
    P = scaled_matrix(D, B)
    n = len(P)
    rows = [sum(P[i]) for i in range(n)]
    cols = [sum(P[i][j] for i in range(n)) for j in range(n)]
    return max(rows + cols) if n else Fraction(0)


def port_bound(D, B=None):
    """The looser per-port capacity bound max(sum_j d_ij / B_i, sum_i d_ij / B_j)."""
    n = len(D)
    Bf = [Fraction(1)] * n if B is None else [Fraction(b) for b in B]
    rows = [sum(Fraction(int(D[i][j])) for j in range(n) if j != i) / Bf[i] for i in range(n)]
    cols = [sum(Fraction(int(D[i][j])) for i in range(n) if i != j) / Bf[j] for j in range(n)]
    return max(rows + cols) if n else Fraction(0)


def pad_to_uniform(P):
    """Artificial traffic X >= 0 with every row and column sum of P + X equal to b_max
    (Appendix A, step 1).  Deficits are matched greedily from the top-left corner;
    an artificial entry on the diagonal simply means that GPU idles."""
    n = len(P)
    bm = max([sum(P[i]) for i in range(n)] + [sum(P[i][j] for i in range(n)) for j in range(n)])
    r = [bm - sum(P[i]) for i in range(n)]
    c = [bm - sum(P[i][j] for i in range(n)) for j in range(n)]
    X = [[Fraction(0)] * n for _ in range(n)]
    i = j = 0
    while i < n and j < n:
        q = min(r[i], c[j])
        X[i][j] += q
        r[i] -= q
        c[j] -= q
        if r[i] == 0:
            i += 1
        elif c[j] == 0:
            j += 1
    return X, bm


def _perfect_matching(support, n):
    """Any perfect matching of the bipartite graph senders x receivers (augmenting paths)."""
    match_r = [-1] * n

    def try_row(i, seen):
        for j in range(n):
            if support[i][j] and not seen[j]:
                seen[j] = True
                if match_r[j] < 0 or try_row(match_r[j], seen):
                    match_r[j] = i
                    return True
        return False

    for i in range(n):
        if not try_row(i, [False] * n):
            return None
    sigma = [-1] * n
    for j, i in enumerate(match_r):
        sigma[i] = j
    return sigma


def rounds(D, B=None):
    """A schedule that attains b_max (Appendix A, step 2).

    D' = P + X has equal row and column sums, so its support always contains a
    perfect matching: in every time slot each GPU sends to a distinct GPU.  Taking
    a matching, running it for the smallest entry on it and subtracting repeats
    until D' is empty.  Artificial traffic is then stripped: a (sender, receiver)
    pair carries real traffic first and is idle (-1) once its real part is used up.
    Returns a list of (dst[n], duration, real[n]) with real[i] the scaled amount of
    true traffic GPU i sends in that round.
    """
    P = scaled_matrix(D, B)
    n = len(P)
    X, bm = pad_to_uniform(P)
    Dp = [[P[i][j] + X[i][j] for j in range(n)] for i in range(n)]
    left = [row[:] for row in P]
    out = []
    while any(Dp[i][j] > 0 for i in range(n) for j in range(n)):
        sigma = _perfect_matching([[Dp[i][j] > 0 for j in range(n)] for i in range(n)], n)
        assert sigma is not None, "equal row/column sums guarantee a perfect matching"
        tau = min(Dp[i][sigma[i]] for i in range(n))
        dst, real = [], []
        for i in range(n):
            j = sigma[i]
            Dp[i][j] -= tau
            use = min(left[i][j], tau)
            left[i][j] -= use
            dst.append(j if use > 0 else -1)
            real.append(use)
        out.append((dst, tau, real))
    return out, bm


def chunks_from_rounds(D, B, g):
    """Chunk list [(dest, tokens)] of GPU g for the schedule of `rounds`: one chunk per
    round in which g sends real traffic.  Tokens are whole: a chunk carries the
    cumulative real traffic g has sent to that destination by the end of the round
    (scaled amount times min(B_g, B_dest)), rounded down, minus what its earlier
    chunks carried.  The cumulative amount ends at d_g,dest exactly, so nothing is
    left over.  Returns (chunks, round_of_chunk)."""
    sched, _ = rounds(D, B)
    n = len(D)
    rate = [Fraction(1) if B is None else min(Fraction(B[g]), Fraction(B[j])) for j in range(n)]
    cum = [Fraction(0)] * n
    sent = [0] * n
    chunks, which = [], []
    for r, (dst, _tau, real) in enumerate(sched):
        j = dst[g]
        if j < 0:
            continue
        cum[j] += real[g] * rate[j]
        rows = int(cum[j]) - sent[j]                        # floor of an exact fraction
        if rows > 0:
            chunks.append((j, rows))
            which.append(r)
            sent[j] += rows
    return chunks, which


def simulate(D, B, order):
    """Completion time of an all-to-all when GPU i sends to the destinations in
    order[i] one after the other (big-switch model of Sec. 2.4).

    Fluid model: a receiver with m incoming flows gives each of them B_recv / m;
    a flow runs at min(B_send, its share).  Empty transfers are skipped.  This
    reproduces the network figure: 3 units for the naive order, 2 for the other.
    """
    n = len(D)
    Bf = [Fraction(1)] * n if B is None else [Fraction(b) for b in B]
    queue = [[j for j in order[i] if j != i and int(D[i][j]) > 0] for i in range(n)]
    cur = [None] * n          # (dst, remaining tokens)
    for i in range(n):
        if queue[i]:
            j = queue[i].pop(0)
            cur[i] = [j, Fraction(int(D[i][j]))]
    t = Fraction(0)
    while any(c is not None for c in cur):
        fan_in = [0] * n
        for c in cur:
            if c is not None:
                fan_in[c[0]] += 1
        rate = [None if c is None else min(Bf[i], Bf[c[0]] / fan_in[c[0]]) for i, c in enumerate(cur)]
        dt = min(c[1] / rate[i] for i, c in enumerate(cur) if c is not None)
        t += dt
        for i, c in enumerate(cur):
            if c is None:
                continue
            c[1] -= rate[i] * dt
            if c[1] == 0:
                cur[i] = None
                if queue[i]:
                    j = queue[i].pop(0)
                    cur[i] = [j, Fraction(int(D[i][j]))]
    return t


def brute_force_best_order(D, B=None):
    """Minimum of `simulate` over every combination of per-source destination orders."""
    n = len(D)
    per_src = [list(itertools.permutations([j for j in range(n) if j != i])) for i in range(n)]
    best, best_order = None, None
    for combo in itertools.product(*per_src):
        v = simulate(D, B, combo)
        if best is None or v < best:
            best, best_order = v, combo
    return best, best_order


def _earliest_fit(busy, t, p):
    """Earliest t' >= t such that [t', t' + p) meets none of the sorted busy intervals."""
    for lo, hi in busy:
        if t + p <= lo:
            break
        if hi > t:
            t = hi
    return t


def alg1_order(D, B=None):
    """Algorithm 1 under a stated reading (parity unpinned, see the module header).

    Time is in units of the scaled matrix p_ij; every GPU has a send timeline and
    a receive timeline, and a flow i -> j of length p_ij must occupy the same
    interval on i's send timeline and j's receive timeline ("no conflicts").
    1. The bottleneck GPU is the one with the largest max(row sum, column sum)
       (lowest index among equals).  Its flows on the binding side (its sends if
       the row sum binds, else the flows it receives) are placed back to back
       from time 0 in ascending peer index, and removed from D.
    2. While D is not empty: GPUs by descending remaining row sum (lowest index
       first among equals); each GPU in turn arranges all its remaining flows:
       repeatedly it takes the flow that can start earliest in a gap free on both
       timelines; among equals the destination with the larger total column sum,
       then the larger flow, then the lower index.  Placed flows never move.
    Returns dict(start[n][n] (None if empty), dest_order[n] (every destination:
    real flows by start time, then empty ones by index, then the GPU itself),
    makespan).
    """
    P = scaled_matrix(D, B)
    n = len(P)
    rem = [row[:] for row in P]
    send_busy = [[] for _ in range(n)]
    recv_busy = [[] for _ in range(n)]
    start = [[None] * n for _ in range(n)]
    rows = [sum(P[i]) for i in range(n)]
    cols = [sum(P[i][j] for i in range(n)) for j in range(n)]

    def earliest(i, j):
        t, p = Fraction(0), rem[i][j]
        while True:
            t1 = _earliest_fit(send_busy[i], t, p)
            t2 = _earliest_fit(recv_busy[j], t1, p)
            if t2 == t1:
                return t1
            t = t2

    def place(i, j, t0):
        start[i][j] = t0
        send_busy[i].append((t0, t0 + rem[i][j]))
        send_busy[i].sort()
        recv_busy[j].append((t0, t0 + rem[i][j]))
        recv_busy[j].sort()
        rem[i][j] = Fraction(0)

    load = [max(rows[i], cols[i]) for i in range(n)]
    b = max(range(n), key=lambda i: (load[i], -i)) if n else 0
    t = Fraction(0)
    for peer in range(n):
        i, j = (b, peer) if rows[b] >= cols[b] else (peer, b)
        if rem[i][j] > 0:
            length = rem[i][j]
            place(i, j, t)
            t += length
    while any(rem[i][j] > 0 for i in range(n) for j in range(n)):
        for i in sorted(range(n), key=lambda i: (-sum(rem[i]), i)):
            while any(rem[i][j] > 0 for j in range(n)):
                cand = [(earliest(i, j), -cols[j], -rem[i][j], j) for j in range(n) if rem[i][j] > 0]
                t0, _, _, j = min(cand)
                place(i, j, t0)
    dest_order = []
    for i in range(n):
        real = sorted([j for j in range(n) if start[i][j] is not None], key=lambda j: (start[i][j], j))
        empty = [j for j in range(n) if j != i and start[i][j] is None]
        dest_order.append(real + empty + [i])
    ends = [hi for tl in send_busy for _, hi in tl]
    return {"start": start, "dest_order": dest_order, "makespan": max([Fraction(0)] + ends)}


def rounds_order(D, B=None):
    """Whole-flow order read off the rounds of Appendix A: GPU i serves its destinations
    in the order in which they first appear in its rounds (empty ones, then i itself, last)."""
    sched, _ = rounds(D, B)
    n = len(D)
    out = []
    for i in range(n):
        first = {}
        for r, (dst, _tau, _real) in enumerate(sched):
            if dst[i] >= 0:
                first.setdefault(dst[i], r)
        real = sorted(first, key=lambda j: (first[j], j))
        out.append(real + [j for j in range(n) if j != i and j not in first] + [i])
    return out


def list_order(D, B=None):
    """Whole-flow order built while the transfer is played forward on the big switch
    (Sec. 2.4) under the sharing rule of `simulate`: whenever a GPU has nothing in
    flight it starts, among the flows it still has to send, the one whose receiver
    has the fewest flows coming in at that moment (a free port if there is one:
    Theorem 2 asks for no contention at the receiving side), then the largest flow,
    then the lowest destination.  GPUs that decide at the same instant do so by
    descending amount still to send (scaled by their rate), lowest index first,
    and see the choices made before theirs.  Returns (order, completion time); the
    time is by construction what `simulate` gives for the order.
    """
    n = len(D)
    Bf = [Fraction(1)] * n if B is None else [Fraction(b) for b in B]
    todo = [{j: Fraction(int(D[i][j])) for j in range(n) if j != i and int(D[i][j]) > 0} for i in range(n)]
    cur = [None] * n                                         # [dst, tokens left] of the flow in flight
    order = [[] for _ in range(n)]
    t = Fraction(0)
    while True:
        idle = [i for i in range(n) if cur[i] is None and todo[i]]
        for i in sorted(idle, key=lambda i: (-sum(todo[i].values()) / Bf[i], i)):
            fan_in = [0] * n
            for c in cur:
                if c is not None:
                    fan_in[c[0]] += 1
            j = min(todo[i], key=lambda j: (fan_in[j], -todo[i][j], j))
            cur[i] = [j, todo[i].pop(j)]
            order[i].append(j)
        if all(c is None for c in cur):
            break
        fan_in = [0] * n
        for c in cur:
            if c is not None:
                fan_in[c[0]] += 1
        rate = [None if c is None else min(Bf[i], Bf[c[0]] / fan_in[c[0]]) for i, c in enumerate(cur)]
        dt = min(c[1] / rate[i] for i, c in enumerate(cur) if c is not None)
        t += dt
        for i, c in enumerate(cur):
            if c is not None:
                c[1] -= rate[i] * dt
                if c[1] == 0:
                    cur[i] = None
    full = [order[i] + [j for j in range(n) if j != i and j not in order[i]] + [i] for i in range(n)]
    return full, t


def shift_order(n):
    """GPU i sends to i + 1, i + 2, ... (mod n): in step s the receivers (i + s) mod n are all different, the
    contention-free order of an all-to-all whose flows are all equal."""
    return [[(i + s) % n for s in range(1, n)] + [i] for i in range(n)]


IMPROVE_MARGIN = Fraction(1, 10 ** 9)     # an exchange must gain more than this fraction of the time


def improve_order(D, B, order, max_evals=None):
    """Hill climbing on a whole-flow order: GPU by GPU, position by position, two
    neighbouring non-empty flows of a GPU are exchanged and the exchange is kept
    when `simulate` gets smaller by more than IMPROVE_MARGIN of its value; passes
    repeat until one changes nothing or `max_evals` (default 64 n) exchanges were
    tried.  Returns (order, time)."""
    n = len(D)
    order = [list(o) for o in order]
    n_real = [sum(1 for j in order[i] if j != i and int(D[i][j]) > 0) for i in range(n)]
    for i in range(n):                                       # non-empty flows first, their relative order kept
        order[i] = ([j for j in order[i] if j != i and int(D[i][j]) > 0] +
                    [j for j in order[i] if j != i and int(D[i][j]) <= 0] + [i])
    best = simulate(D, B, order)
    budget = 64 * n if max_evals is None else max_evals
    changed = True
    while changed and budget > 0:
        changed = False
        for i in range(n):
            for p in range(n_real[i] - 1):
                if budget <= 0:
                    break
                budget -= 1
                order[i][p], order[i][p + 1] = order[i][p + 1], order[i][p]
                v = simulate(D, B, order)
                if v < best * (1 - IMPROVE_MARGIN):
                    best, changed = v, True
                else:
                    order[i][p], order[i][p + 1] = order[i][p + 1], order[i][p]
    return order, best


def send_order(D, B=None, max_evals=None):
    """The whole-flow order handed to the send buffer: the candidate with the smallest
    `simulate` among Algorithm 1's order, the order read off the rounds, the
    list order and the shifted order (the earlier candidate wins unless a later
    one is better by more than IMPROVE_MARGIN), then `improve_order`.  Returns
    dict(dest_order, time, source (0..3), candidate_times)."""
    cands = [alg1_order(D, B)["dest_order"], rounds_order(D, B), list_order(D, B)[0], shift_order(len(D))]
    times = [simulate(D, B, c) for c in cands]
    k = 0
    for c in (1, 2, 3):
        if times[c] < times[k] * (1 - IMPROVE_MARGIN):
            k = c
    order, t = improve_order(D, B, cands[k], max_evals)
    return {"dest_order": order, "time": t, "source": k, "candidate_times": times}
