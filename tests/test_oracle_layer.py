"""Pins of the layer oracle to facts that do not come from the oracle itself."""
import itertools
import math

import numpy as np
import pytest

from oracle import moe_layer as O


def rng(seed):
    return np.random.default_rng(seed)


# ------------------------------------------------------------------ gate
def test_topk_exhaustive_against_full_sort():
    r = rng(1)
    for E, k in [(2, 1), (3, 2), (5, 2), (8, 2), (8, 1), (6, 6), (7, 3)]:
        x = r.standard_normal((40, 16))
        wg = r.standard_normal((E, 16))
        b = r.standard_normal(E)
        idx, w, z = O.route(x, wg, b, k, 0)
        for t in range(40):
            # brute force: explicit dot products, then pick maxima one by one
            logits = [sum(x[t, h] * wg[e, h] for h in range(16)) + b[e] for e in range(E)]
            assert np.allclose(logits, z[t], rtol=1e-12, atol=1e-12)
            chosen, pool = [], list(range(E))
            for _ in range(k):
                best = max(pool, key=lambda e: (logits[e], -e))
                chosen.append(best)
                pool.remove(best)
            assert list(idx[t]) == chosen
            den = sum(math.exp(v - max(logits)) for v in logits)
            for j, e in enumerate(chosen):
                assert w[t, j] == pytest.approx(math.exp(logits[e] - max(logits)) / den, rel=1e-12)


def test_ties_go_to_lower_index_and_no_duplicates():
    r = rng(2)
    x = r.standard_normal((32, 8))
    base = r.standard_normal((3, 8))
    wg = np.stack([base[0], base[1], base[0], base[2], base[1], base[0]])   # rows 0=2=5, 1=4
    idx, w, z = O.route(x, wg, None, 3, 0)
    for t in range(32):
        assert len(set(idx[t])) == 3
        zt = z[t]
        for a, b in zip(idx[t][:-1], idx[t][1:]):
            assert zt[a] > zt[b] or (zt[a] == zt[b] and a < b)
        rest = [e for e in range(6) if e not in idx[t]]
        last = idx[t][-1]
        for e in rest:
            assert zt[e] < zt[last] or (zt[e] == zt[last] and e > last)


def test_softmax_mass_and_renorm():
    r = rng(3)
    x = r.standard_normal((64, 32))
    wg = r.standard_normal((8, 32))
    idx_all, w_all, _ = O.route(x, wg, None, 8, 0)
    assert np.allclose(w_all.sum(1), 1.0, atol=1e-12)            # all experts: total mass 1
    idx, w, _ = O.route(x, wg, None, 2, 0)
    assert np.array_equal(idx, idx_all[:, :2])
    assert np.allclose(w, w_all[:, :2], rtol=1e-14)               # weights are the gate mass
    idx_r, w_r, _ = O.route(x, wg, None, 2, 1)
    assert np.array_equal(idx_r, idx)
    assert np.allclose(w_r.sum(1), 1.0, atol=1e-12)
    assert np.allclose(w_r[:, 0] / w_r[:, 1], w[:, 0] / w[:, 1], rtol=1e-12)


def test_gate_shift_invariance_and_bias():
    r = rng(4)
    x = r.standard_normal((16, 8))
    wg = r.standard_normal((4, 8))
    i0, w0, _ = O.route(x, wg, None, 2, 0)
    i1, w1, _ = O.route(x, wg, np.full(4, 3.25), 2, 0)           # constant bias changes nothing
    assert np.array_equal(i0, i1) and np.allclose(w0, w1, rtol=1e-12)
    i2, _, _ = O.route(x, wg, np.array([0, 0, 100.0, 0]), 2, 0)   # huge bias forces expert 2 first
    assert np.all(i2[:, 0] == 2)


# ------------------------------------------------------------------ traffic
def test_traffic_brute_force_recount():
    r = rng(5)
    T, k, E, G = 50, 2, 8, 4
    idx = np.stack([r.permutation(E)[:k] for _ in range(T)]).astype(np.int32)
    e2g = np.arange(E) // 2
    ec, dc, nd, keep = O.traffic(idx, e2g, G, 0)
    assert nd == 0 and keep.all()
    assert [int(v) for v in ec] == [sum(1 for t in range(T) for j in range(k) if idx[t, j] == e) for e in range(E)]
    assert [int(v) for v in dc] == [sum(1 for t in range(T) for j in range(k) if idx[t, j] // 2 == d) for d in range(G)]
    assert ec.sum() == T * k == dc.sum()


def test_capacity_hand_built():
    # experts chosen by slots 0..9 (k = 1): capacity 2 keeps the first two of each expert
    idx = np.array([[0], [1], [0], [0], [1], [2], [0], [1], [1], [2]], dtype=np.int32)
    ec, dc, nd, keep = O.traffic(idx, [0, 0, 1], 2, capacity=2)
    assert list(ec) == [2, 2, 2] and list(dc) == [4, 2] and nd == 4
    assert list(keep) == [True, True, True, False, True, True, False, False, False, True]
    r = rng(6)
    idx = r.integers(0, 4, size=(200, 1)).astype(np.int32)
    raw, _, _, _ = O.traffic(idx, [0, 1, 2, 3], 4, 0)
    ec, _, nd, _ = O.traffic(idx, [0, 1, 2, 3], 4, 37)
    assert list(ec) == [min(int(c), 37) for c in raw] and nd == 200 - ec.sum()


# ------------------------------------------------------------------ dispatch
@pytest.mark.parametrize("capacity", [0, 20])
def test_dispatch_invariants_all_24_orders(capacity):
    r = rng(7)
    T, k, E, G, H = 64, 2, 8, 4, 5
    x = r.standard_normal((T, H))
    idx = np.stack([r.permutation(E)[:k] for _ in range(T)]).astype(np.int32)
    e2g = np.arange(E) // 2
    ec, dc, nd, keep = O.traffic(idx, e2g, G, capacity)
    for order in itertools.permutations(range(G)):
        d = O.dispatch(x, idx, e2g, order, capacity)
        s2r, r2s = d["slot_to_row"], d["row_to_slot"]
        n = d["n_rows"]
        assert n == T * k - nd == len(r2s)
        assert sorted(r2s.tolist()) == sorted(np.nonzero(keep)[0].tolist())       # each kept slot once
        assert all(s2r[r2s[row]] == row for row in range(n))
        assert all((s2r[s] >= 0) == bool(keep[s]) for s in range(T * k))
        assert np.array_equal(d["send_buf"], x[r2s // k])                         # bitwise row copies
        dest_of_row = e2g[idx.reshape(-1)[r2s]]
        # destinations appear as contiguous runs in exactly the requested order
        runs = [g for g, _ in itertools.groupby(dest_of_row.tolist())]
        assert runs == [g for g in order if dc[g] > 0]
        so, se = d["seg_offset"], d["seg_expert"]
        assert so[0] == 0 and so[-1] == n and len(so) == E + 1
        for i, e in enumerate(se):
            seg = r2s[so[i]:so[i + 1]]
            assert len(seg) == ec[e]
            assert np.all(idx.reshape(-1)[seg] == e)
            assert np.all(np.diff(seg) > 0)                                       # stable inside a segment


def test_chunked_dispatch_reduces_to_dispatch_and_keeps_destination_sequences():
    r = rng(70)
    T, k, E, G, H = 96, 2, 12, 4, 3
    x = r.standard_normal((T, H))
    idx = np.stack([r.permutation(E)[:k] for _ in range(T)]).astype(np.int32)
    e2g = np.arange(E) % G                                  # experts of a GPU are not contiguous ids
    flat = idx.reshape(-1)
    for capacity in (0, 11):
        ec, dc, nd, keep = O.traffic(idx, e2g, G, capacity)
        # (1) one unbounded chunk per destination IS the non-preemptive layout of `dispatch`
        for order in [(0, 1, 2, 3), (2, 0, 3, 1), (3, 2, 1, 0)]:
            a = O.dispatch(x, idx, e2g, order, capacity)
            b = O.dispatch_chunks(x, idx, e2g, [(g, 10 ** 9) for g in order], capacity)
            assert np.array_equal(a["slot_to_row"], b["slot_to_row"])
            assert np.array_equal(a["row_to_slot"], b["row_to_slot"])
            assert np.array_equal(a["send_buf"], b["send_buf"])
        # (2) an empty plan: everything is left over, destination by destination in GPU order
        a = O.dispatch(x, idx, e2g, range(G), capacity)
        b = O.dispatch_chunks(x, idx, e2g, [], capacity)
        assert np.array_equal(a["row_to_slot"], b["row_to_slot"])
        # (3) random preemptive plans, with too little, too much and unknown destinations
        whole = {g: [s for e in range(E) if e2g[e] == g for s in np.nonzero(keep & (flat == e))[0]] for g in range(G)}
        for trial in range(20):
            chunks = [(int(r.integers(-1, G + 1)), int(r.integers(0, 30))) for _ in range(int(r.integers(0, 14)))]
            d = O.dispatch_chunks(x, idx, e2g, chunks, capacity)
            r2s, s2r, co = d["row_to_slot"], d["slot_to_row"], d["chunk_offset"]
            assert d["n_rows"] == T * k - nd == len(r2s)
            assert sorted(r2s.tolist()) == sorted(np.nonzero(keep)[0].tolist())
            assert all(s2r[r2s[row]] == row for row in range(len(r2s)))
            assert np.array_equal(d["send_buf"], x[r2s // k])
            assert len(co) == len(chunks) + G + 1 and co[0] == 0 and co[-1] == len(r2s)
            got = {g: [] for g in range(G)}
            for c, (dest, rows) in enumerate(chunks + [(g, None) for g in range(G)]):
                part = r2s[co[c]:co[c + 1]].tolist()
                if not (0 <= dest < G):
                    assert part == []
                    continue
                assert all(e2g[flat[s]] == dest for s in part)              # a chunk has one destination
                if rows is not None:
                    assert len(part) <= rows
                    # a planned chunk is short only when its destination has run out
                    assert len(part) == rows or len(got[dest]) + len(part) == len(whole[dest])
                got[dest].extend(part)
            assert got == whole                                             # chunks of a destination, joined, are its sequence
            po, pe = d["piece_offset"], d["piece_expert"]
            assert po[0] == 0 and po[-1] == len(r2s) and len(po) == len(pe) + 1
            assert np.all(np.diff(po) > 0)
            cuts = set(co.tolist())
            for i, e in enumerate(pe):
                assert np.all(flat[r2s[po[i]:po[i + 1]]] == e)
                assert not any(po[i] < c < po[i + 1] for c in cuts)            # a piece never straddles a chunk
                if i + 1 < len(pe):
                    assert pe[i + 1] != e or po[i + 1] in cuts                 # maximal: a new piece needs a reason


# ------------------------------------------------------------------ FFN
def test_ffn_special_cases():
    r = rng(8)
    x = r.standard_normal((6, 4))
    eye = np.eye(4)
    silu = lambda a: a / (1 + np.exp(-a))
    assert np.allclose(O.ffn(x, eye, None, eye, 0), silu(x), rtol=1e-14)
    # closed-form scalars (H = F = 1): silu(1) = 1/(1+e^-1); tanh-GELU(1) = 0.841191990608...
    assert O.ffn([[1.0]], [[1.0]], None, [[1.0]], 0)[0, 0] == pytest.approx(1 / (1 + math.exp(-1)), rel=1e-15)
    assert O.ffn([[1.0]], [[1.0]], None, [[1.0]], 1)[0, 0] == pytest.approx(0.8411919906082768, rel=1e-12)
    assert O.ffn([[2.0]], [[1.0]], [[3.0]], [[0.5]], 2)[0, 0] == pytest.approx(0.5 * (2 / (1 + math.exp(-2))) * 6.0, rel=1e-15)
    # tanh GELU stays within 1e-3 of the erf form and they differ (so the choice is visible)
    a = np.linspace(-4, 4, 101)[:, None]
    erf_form = 0.5 * a * (1 + np.vectorize(math.erf)(a / math.sqrt(2)))
    got = O.ffn(a, [[1.0]], None, [[1.0]], 1)
    assert np.max(np.abs(got - erf_form)) < 1e-3 and np.max(np.abs(got - erf_form)) > 1e-5


def test_ffn_against_independent_triple_loop_and_orientation():
    r = rng(9)
    R, H, F = 5, 7, 3                       # non-square on purpose: a transposed operand cannot pass
    x = r.standard_normal((R, H))
    w1, wu, wd = r.standard_normal((F, H)), r.standard_normal((F, H)), r.standard_normal((H, F))
    for act in (0, 1, 2):
        ref = np.zeros((R, H))
        for i in range(R):
            hid = []
            for f in range(F):
                a = sum(w1[f, h] * x[i, h] for h in range(H))
                if act == 0:
                    v = a / (1 + math.exp(-a))
                elif act == 1:
                    v = 0.5 * a * (1 + math.tanh(math.sqrt(2 / math.pi) * (a + 0.044715 * a ** 3)))
                else:
                    v = a / (1 + math.exp(-a)) * sum(wu[f, h] * x[i, h] for h in range(H))
                hid.append(v)
            for o in range(H):
                ref[i, o] = sum(wd[o, f] * hid[f] for f in range(F))
        assert np.allclose(O.ffn(x, w1, wu, wd, act), ref, rtol=1e-12, atol=1e-14)


def test_swiglu_reduces_to_silu_mlp():
    r = rng(10)
    x = np.concatenate([r.standard_normal((9, 5)), np.ones((9, 1))], axis=1)   # last feature is 1
    w1, wd = r.standard_normal((4, 6)), r.standard_normal((6, 4))
    wu = np.zeros((4, 6)); wu[:, 5] = 1.0                                       # Wu . x == 1
    assert np.allclose(O.ffn(x, w1, wu, wd, 2), O.ffn(x, w1, None, wd, 0), rtol=1e-13)


def test_grouped_ffn_is_per_segment_ffn():
    r = rng(11)
    H, F = 6, 4
    experts = [{"w1": r.standard_normal((F, H)), "w_up": r.standard_normal((F, H)),
                "w_down": r.standard_normal((H, F))} for _ in range(3)]
    recv = r.standard_normal((10, H))
    out = O.expert_ffn(recv, [0, 3, 3, 7, 10], [2, 0, 1, 2], experts, 2)
    for lo, hi, e in [(0, 3, 2), (3, 7, 1), (7, 10, 2)]:
        for i in range(lo, hi):
            w = experts[e]
            assert np.allclose(out[i], O.ffn(recv[i:i + 1], w["w1"], w["w_up"], w["w_down"], 2)[0], rtol=1e-13)


# ------------------------------------------------------------------ combine and the whole path
def test_combine_hand_case():
    ret = np.array([[1.0, 2.0], [10.0, 20.0], [100.0, 200.0]])
    s2r = np.array([2, 0, -1, 1])
    w = np.array([[0.5, 0.25], [0.7, 0.3]])
    y = O.combine(ret, s2r, w, shared_out=np.array([[1000.0, 0.0], [0.0, 1000.0]]))
    assert np.allclose(y, [[0.5 * 100 + 0.25 * 1 + 1000, 0.5 * 200 + 0.25 * 2], [0.3 * 10, 0.3 * 20 + 1000]])


def _emulated_cluster(cfgs):
    """Step-wise pipeline over G simulated GPUs with explicit all-to-alls, in numpy."""
    G, E, k, H, act, renorm, capacity = (cfgs[n] for n in ("G", "E", "k", "H", "act", "renorm", "capacity"))
    e2g, experts, xs, wg, bias = cfgs["e2g"], cfgs["experts"], cfgs["xs"], cfgs["wg"], cfgs["bias"]
    orders = cfgs["orders"]
    routed = [O.route(xs[g], wg, bias, k, renorm) for g in range(G)]
    disp = [O.dispatch(xs[g], routed[g][0], e2g, orders[g], capacity) for g in range(G)]
    rets = [np.zeros((disp[g]["n_rows"], H)) for g in range(G)]
    for dst in range(G):                                   # first all-to-all, FFN, second all-to-all
        local = [e for e in range(E) if e2g[e] == dst]
        chunks, seg_off, seg_exp, origin = [], [0], [], []
        for src in range(G):
            d = disp[src]
            for i, e in enumerate(d["seg_expert"]):
                if e2g[e] == dst:
                    lo, hi = d["seg_offset"][i], d["seg_offset"][i + 1]
                    chunks.append(d["send_buf"][lo:hi])
                    seg_off.append(seg_off[-1] + hi - lo)
                    seg_exp.append(local.index(e))
                    origin.append((src, lo, hi))
        recv = np.concatenate(chunks) if chunks else np.zeros((0, H))
        out = O.expert_ffn(recv, seg_off, seg_exp, [experts[e] for e in local], act)
        for i, (src, lo, hi) in enumerate(origin):
            rets[src][lo:hi] = out[seg_off[i]:seg_off[i + 1]]
    return [O.combine(rets[g], disp[g]["slot_to_row"], routed[g][1]) for g in range(G)]


@pytest.mark.parametrize("act,renorm,capacity,k", [(0, 0, 0, 2), (2, 1, 0, 2), (1, 0, 5, 1), (2, 0, 9, 3)])
def test_stepwise_pipeline_reaches_the_per_token_definition(act, renorm, capacity, k):
    r = rng(12 + act)
    G, E, H, F, T = 4, 8, 6, 5, 24
    experts = [{"w1": r.standard_normal((F, H)), "w_up": r.standard_normal((F, H)) if act == 2 else None,
                "w_down": r.standard_normal((H, F))} for _ in range(E)]
    cfgs = dict(G=G, E=E, k=k, H=H, act=act, renorm=renorm, capacity=capacity,
                e2g=np.arange(E) // 2, experts=experts, xs=[r.standard_normal((T, H)) for _ in range(G)],
                wg=r.standard_normal((E, H)), bias=r.standard_normal(E),
                orders=[list(r.permutation(G)) for _ in range(G)])
    ys = _emulated_cluster(cfgs)
    for g in range(G):
        dense = O.layer_dense(cfgs["xs"][g], cfgs["wg"], cfgs["bias"], k, renorm, experts, act, capacity)
        assert np.allclose(ys[g], dense, rtol=1e-12, atol=1e-13)


def test_combine_weights_sum_to_gate_mass_minus_drops():
    r = rng(20)
    T, E, k, H = 40, 4, 2, 3
    x, wg = r.standard_normal((T, H)), r.standard_normal((E, H))
    idx, w, _ = O.route(x, wg, None, k, 0)
    cap = 12
    _, _, nd, keep = O.traffic(idx, np.arange(E), E, cap)
    assert nd > 0
    d = O.dispatch(x, idx, np.arange(E), list(range(E)), cap)
    y = O.combine(np.ones((d["n_rows"], 1)), d["slot_to_row"], w)     # every expert returns 1
    assert np.allclose(y[:, 0], (w * keep.reshape(T, k)).sum(1), rtol=1e-13)
