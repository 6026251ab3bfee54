"""Parity of the HIP path (through the C ABI) with the CPU oracle on the same seeded inputs.

Integer results (indices, counts, permutation, copied rows) must be bit-exact.  Floating
point: fp32 within 1e-5, bf16 within 2e-2, both as max|diff| / max|ref| per tensor.
"""
import dataclasses
import itertools

import numpy as np
import pytest
import torch

import workloads as W
from oracle import moe_layer as O

pytestmark = pytest.mark.gpu

TOL = {"fp32": 1e-5, "bf16": 2e-2}


@pytest.fixture(scope="module")
def H():
    from tests import harness
    assert torch.cuda.is_available(), "these tests need the MI355X"
    return harness


def small(name, **kw):
    return W.scaled(W.get_config(name), **kw)


# reduced shapes the oracle finishes in seconds; several tiles and ragged tails everywhere
ROUTE_CASES = [
    W.get_config("c1_tiny_fp32"),
    small("c1_tiny_fp32", T=3, H=4, E=2, k=1, G=2),
    small("c1_tiny_fp32", T=37, H=100, E=5, k=3, G=5),
    small("c2_mixtral", T=203, H=1032),
    small("c2_mixtral", T=64, H=4096),
    small("c3_switch", T=517, H=256),
    small("c4b_coloc", T=130, H=512),
    small("c5_finegrained", T=301, H=512),
    small("c5_finegrained", T=65, H=264, E=160, k=9, G=16),
    small("c1_tiny_fp32", T=50, H=36, E=200, k=16, G=8),
    small("c2_mixtral", T=33, H=64, E=24, k=4, G=8),
    small("c2_mixtral", T=17, H=8, E=17, k=2, G=1),              # one 16-byte chunk per row, one expert past a tile
    small("c5_finegrained", T=100, H=520, E=65, k=6, G=5),       # second pass of 64 experts holds a single expert
    small("c3_switch", T=40, H=1024, E=256, k=16, G=64),         # the limits of E, k and G
]


def route_inputs(cfg):
    inp = W.make_layer_inputs(cfg)
    if inp["gate_bias"] is None and cfg.index % 2 == 1:
        inp["gate_bias"] = np.linspace(-0.5, 0.5, cfg.E).astype(np.float32)
    return inp


@pytest.mark.parametrize("cfg", ROUTE_CASES, ids=lambda c: "%s-T%d-H%d-E%d-k%d" % (c.name, c.T, c.H, c.E, c.k))
def test_route(H, cfg):
    inp = route_inputs(cfg)
    idx_ref, w_ref, z = O.route(inp["x"], inp["w_gate"], inp["gate_bias"], cfg.k, cfg.renorm)
    margin = O.route_margin(z, cfg.k).min()
    assert margin > 1e-9, "seed gives a near tie; bit-exact indices would not be meaningful"
    sh = H.Share(cfg)
    x, wg = H.dev(inp["x"], cfg.dtype), H.dev(inp["w_gate"], cfg.dtype)
    bias = None if inp["gate_bias"] is None else torch.from_numpy(inp["gate_bias"]).to(H.DEV)
    sh.route(x, wg, bias)
    torch.cuda.synchronize()
    assert np.array_equal(H.host(sh.idx), idx_ref)
    assert H.rel_err(H.host(sh.w), w_ref) < 1e-5
    assert np.max(np.abs(H.host(sh.w) / w_ref - 1.0)) < 1e-5


@pytest.mark.parametrize("cfg", [small("c2_mixtral", T=203, H=1024), small("c5_finegrained", T=301, H=512),
                                 small("c3_switch", T=40, H=1024, E=256, k=16, G=64), small("c1_tiny_fp32", T=37, H=100, E=5, k=3, G=5)],
                         ids=lambda c: "%s-T%d-E%d-k%d" % (c.name, c.T, c.E, c.k))
def test_route_phases_diag_gives_the_results_of_moe_route_and_ordered_marks(H, cfg):
    """The timed instantiation of the gate kernel is the gate kernel: same indices and weights; its clock marks
    do not go backwards within a wave; a shape that takes the fp64 kernel reports no marks."""
    inp = route_inputs(cfg)
    sh = H.Share(cfg)
    x, wg = H.dev(inp["x"], cfg.dtype), H.dev(inp["w_gate"], cfg.dtype)
    bias = None if inp["gate_bias"] is None else torch.from_numpy(inp["gate_bias"]).to(H.DEV)
    sh.route(x, wg, bias)
    idx2, w2 = torch.full_like(sh.idx, -7), torch.full_like(sh.w, float("nan"))
    marks = torch.zeros((cfg.T // 16 + 1) * 128, dtype=torch.int64, device=H.DEV)
    tpb = H.P.moe_diag_route_phases(sh.ctx, x, wg, bias, idx2, w2, marks)
    torch.cuda.synchronize()
    assert torch.equal(idx2, sh.idx) and torch.equal(w2, sh.w)
    if cfg.dtype == "fp32" or cfg.H % 32:
        assert tpb == 0 and int(marks.abs().sum()) == 0
        return
    assert tpb in (16, 32, 64)
    nb = (cfg.T + tpb - 1) // tpb
    a = marks[:nb * 128].cpu().numpy().reshape(nb, 16, 8)
    assert int(np.abs(marks[nb * 128:].cpu().numpy()).sum()) == 0
    live = a[:, :, 0] > 0
    assert live[:, 0].all()
    t = a[:, :, :5]
    assert (np.diff(t, axis=2)[live] >= 0).all()
    ends = a[:, :, 5]
    assert ((ends == 0) | (ends >= a[:, :, 4]))[live].all()
    with pytest.raises(H.P.MoeError):
        H.P.moe_diag_route_phases(sh.ctx, x, wg, bias, idx2, w2, marks[:16])


def test_route_ties_pick_lower_index(H):
    cfg = small("c2_mixtral", T=96, H=256, E=8, k=3)
    inp = W.make_layer_inputs(cfg)
    wg = inp["w_gate"].copy()
    wg[5] = wg[1]; wg[6] = wg[1]; wg[7] = wg[2]            # duplicated gate rows: exact ties
    idx_ref, w_ref, _ = O.route(inp["x"], wg, None, cfg.k, cfg.renorm)
    sh = H.Share(cfg)
    sh.route(H.dev(inp["x"], cfg.dtype), H.dev(wg, cfg.dtype), None)
    torch.cuda.synchronize()
    assert np.array_equal(H.host(sh.idx), idx_ref)
    assert H.rel_err(H.host(sh.w), w_ref) < 1e-5


@pytest.mark.parametrize("E,k,H_", [(8, 2, 1024), (65, 6, 520), (160, 9, 264)])
def test_route_near_ties_take_the_exact_path(H, E, k, H_):
    """Gate rows that differ from one another in a single element by one bf16 step: every gap
    between logits is far below what fp32 accumulation resolves, yet far above fp64 rounding,
    so the indices are well defined and any kernel that decides them from approximate logits
    must fall back to exact ones for (nearly) every token."""
    cfg = small("c2_mixtral", T=150, H=H_, E=E, k=k, G=1)
    inp = W.make_layer_inputs(cfg)
    base = inp["w_gate"][0].astype(np.float32)
    wg = np.tile(base, (E, 1))
    for e in range(1, E):
        j = (7 * e) % H_
        bits = wg[e, j:j + 1].view(np.uint32)
        bits += np.uint32((1 + e // H_) << 16)               # next bf16 value(s) away from zero
    idx_ref, w_ref, z = O.route(inp["x"], wg, None, cfg.k, cfg.renorm)
    margin = O.route_margin(z, cfg.k)
    assert margin.max() < 1e-2
    ok = margin > 1e-9          # bf16 values have few bits, so some products coincide exactly: those tokens are skipped
    assert ok.mean() > 0.5
    sh = H.Share(cfg)
    sh.route(H.dev(inp["x"], cfg.dtype), H.dev(wg, cfg.dtype), None)
    torch.cuda.synchronize()
    assert np.array_equal(H.host(sh.idx)[ok], idx_ref[ok])
    assert H.rel_err(H.host(sh.w)[ok], w_ref[ok]) < 1e-5


DISPATCH_CASES = [
    (W.get_config("c1_tiny_fp32"), 0),
    (small("c1_tiny_fp32", T=1, H=4, E=2, k=1, G=2), 0),
    (small("c2_mixtral", T=1500, H=520), 0),
    (small("c3_switch", T=3000, H=128), None),             # config's own capacity (scaled with T)
    (small("c3_switch", T=2100, H=64), 7),
    (small("c5_finegrained", T=1111, H=136), 0),
    (small("c5_finegrained", T=700, H=64, E=160, k=9, G=16), 30),
    # more than 16384 slots: the multi-block counting path
    (small("c5_finegrained", T=3100, H=64), 0),
    (small("c3_switch", T=20011, H=32), None),
    (small("c2_mixtral", T=8193, H=64), 0),               # 16386 slots, just over the single-block limit
    (small("c2_mixtral", T=8192, H=64), 0),               # 16384 slots, the single-block limit itself
    # row lengths that pick the other copy geometries: several short rows per wave (1, 2, 4 KB rows; a ragged
    # last wave), rows longer than a wave's 8 KB cut into pieces (a whole number of pieces and a ragged one)
    (small("c2_mixtral", T=203, H=512), 0),               # 1 KB rows: 8 tokens per wave
    (small("c3_switch", T=517, H=1024), 9),               # 2 KB rows, k = 1: 4 tokens per wave, dropped slots
    (small("c5_finegrained", T=131, H=512), 0),           # 1 KB rows to 6 slots: 2 tokens per wave
    (small("c4b_coloc", T=99, H=2048), 0),                # 4 KB rows: 2 tokens per wave
    (small("c2_mixtral", T=77, H=8192), 0),               # 16 KB rows: two pieces
    (small("c1_tiny_fp32", T=50, H=2304, E=5, k=3, G=5), 0),   # 9 KB rows: a full piece and a 1 KB one
]


@pytest.mark.parametrize("cfg,cap", DISPATCH_CASES, ids=lambda v: getattr(v, "name", str(v)))
def test_traffic_and_dispatch(H, cfg, cap):
    if cap is not None:
        cfg = dataclasses.replace(cfg, capacity_factor=0.0)
    capacity = cfg.capacity if cap is None else cap
    inp = W.make_layer_inputs(cfg)
    idx_ref, _, _ = O.route(inp["x"], inp["w_gate"], inp["gate_bias"], cfg.k, cfg.renorm)
    e2g = inp["expert_to_gpu"]
    r = np.random.default_rng(cfg.seed_base)
    orders = [list(range(cfg.G)), list(r.permutation(cfg.G))]
    if cfg.name == "c1_tiny_fp32" and cfg.G == 4:
        orders = list(itertools.permutations(range(4)))     # all 24 transmission orders
    sh = H.Share(cfg)
    sh.ctx.close()
    sh.ctx = H.P.MoeCtx(cfg.T, cfg.H, cfg.E, cfg.k, cfg.G, cfg.dtype, cfg.renorm, capacity)
    x = H.dev(inp["x"], cfg.dtype)
    sh.idx.copy_(torch.from_numpy(idx_ref))
    ec, dc, nd, _ = O.traffic(idx_ref, e2g, cfg.G, capacity)
    sh.traffic(e2g)
    torch.cuda.synchronize()
    assert np.array_equal(H.host(sh.expert_count), ec)
    assert np.array_equal(H.host(sh.dest_count), dc)
    assert int(sh.n_dropped.item()) == nd
    if capacity:
        assert nd > 0
    for order in orders:
        ref = O.dispatch(inp["x"], idx_ref, e2g, order, capacity)
        sh.slot_to_row.fill_(-7); sh.row_to_slot.fill_(-7); sh.send_buf.zero_()
        sh.dispatch(x, e2g, order)
        torch.cuda.synchronize()
        n = ref["n_rows"]
        assert np.array_equal(H.host(sh.slot_to_row), ref["slot_to_row"])
        assert np.array_equal(H.host(sh.row_to_slot)[:n], ref["row_to_slot"])
        assert np.all(H.host(sh.row_to_slot)[n:] == -7)                    # nothing written past the kept rows
        assert np.array_equal(H.host(sh.seg_offset), ref["seg_offset"])
        assert np.array_equal(H.host(sh.seg_expert), ref["seg_expert"])
        assert np.array_equal(H.host(sh.send_buf)[:n], ref["send_buf"])    # bitwise row copies
        assert not H.host(sh.send_buf)[n:].any()
    # determinism: a second run gives the same bytes
    a = sh.slot_to_row.clone()
    sh.dispatch(x, e2g, orders[-1])
    torch.cuda.synchronize()
    assert torch.equal(a, sh.slot_to_row)


@pytest.mark.parametrize("cfg", [small("c2_mixtral", T=700, H=264), small("c5_finegrained", T=3000, H=64)],
                         ids=lambda c: c.name)
def test_dispatch_alone_and_after_in_place_index_rewrite(H, cfg):
    """moe_dispatch never depends on an earlier call unless rank reuse was switched on; with reuse on, the
    ranks of a moe_traffic serve exactly one directly following dispatch on the same index array."""
    inp = W.make_layer_inputs(cfg)
    e2g = inp["expert_to_gpu"]
    order = list(np.random.default_rng(3).permutation(cfg.G))
    idx_a, _, _ = O.route(inp["x"], inp["w_gate"], inp["gate_bias"], cfg.k, cfg.renorm)
    idx_b = np.ascontiguousarray(idx_a[::-1])                      # a different, still valid, routing
    x = H.dev(inp["x"], cfg.dtype)
    sh = H.Share(cfg)

    def check(idx_ref):
        ref = O.dispatch(inp["x"], idx_ref, e2g, order, cfg.capacity)
        torch.cuda.synchronize()
        assert np.array_equal(H.host(sh.slot_to_row), ref["slot_to_row"])
        assert np.array_equal(H.host(sh.seg_offset), ref["seg_offset"])
        assert np.array_equal(H.host(sh.send_buf)[:ref["n_rows"]], ref["send_buf"])

    sh.idx.copy_(torch.from_numpy(idx_a))
    sh.dispatch(x, e2g, order)                                     # fresh context: ranks computed inside
    check(idx_a)
    # default (no reuse): indices rewritten in place behind the library's back, no invalidate: still right
    sh.traffic(e2g)
    sh.idx.copy_(torch.from_numpy(idx_b))
    sh.dispatch(x, e2g, order)
    check(idx_b)
    # reuse on: traffic then dispatch (one kernel) is right ...
    sh.ctx.set_rank_reuse(True)
    sh.traffic(e2g)
    sh.dispatch(x, e2g, order)
    check(idx_b)
    # ... the ranks are used once: a rewrite after that dispatch cannot reach a stale rank
    sh.idx.copy_(torch.from_numpy(idx_a))
    sh.dispatch(x, e2g, order)
    check(idx_a)
    # ... a rewrite between traffic and dispatch is the caller's to announce
    sh.traffic(e2g)
    sh.idx.copy_(torch.from_numpy(idx_b))
    sh.ctx.invalidate()
    sh.dispatch(x, e2g, order)
    check(idx_b)
    # ... and ranks made for another pointer are never used
    sh.traffic(e2g)
    other = sh.idx.clone()
    other.copy_(torch.from_numpy(idx_a))
    H.P.moe_dispatch(sh.ctx, x, other, e2g, order, sh.send_buf, sh.slot_to_row, sh.row_to_slot, sh.seg_offset,
                     sh.seg_expert)
    check(idx_a)
    # ... nor after a moe_route on the context (it rewrites the indices)
    sh.idx.copy_(torch.from_numpy(idx_b))
    sh.traffic(e2g)
    sh.route(x, H.dev(inp["w_gate"], cfg.dtype), None if inp["gate_bias"] is None else torch.from_numpy(inp["gate_bias"]).float().to(H.DEV))
    sh.dispatch(x, e2g, order)
    check(idx_a)


CHUNK_CASES = [small("c2_mixtral", T=300, H=264), small("c3_switch", T=700, H=128), small("c5_finegrained", T=260, H=64),
               small("c3_switch", T=40, H=64),                 # most experts get no token at all
               small("c1_tiny_fp32", T=37, H=100, E=5, k=3, G=5), small("c5_finegrained", T=3000, H=64, E=160, k=9, G=16),
               small("c2_mixtral", T=203, H=512), small("c3_switch", T=517, H=1024),      # several short rows per wave
               small("c2_mixtral", T=77, H=8192)]                                          # long rows in pieces


@pytest.mark.parametrize("cfg", CHUNK_CASES, ids=lambda c: "%s-T%d-E%d-k%d-G%d" % (c.name, c.T, c.E, c.k, c.G))
def test_dispatch_chunks(H, cfg):
    """Send buffer in the layout of a preemptive plan: bit-exact against the oracle for plans that
    cover too little, too much, nothing, name no GPU, and for the plan of the Appendix A rounds."""
    P = H.P
    inp = W.make_layer_inputs(cfg)
    idx_ref, _, _ = O.route(inp["x"], inp["w_gate"], inp["gate_bias"], cfg.k, cfg.renorm)
    e2g = inp["expert_to_gpu"]
    _, dc, _, _ = O.traffic(idx_ref, e2g, cfg.G, cfg.capacity)
    r = np.random.default_rng(cfg.seed_base + 9)
    plans = [[], [(g, 10 ** 9) for g in r.permutation(cfg.G)]]
    plans.append([(int(r.integers(-1, cfg.G + 1)), int(r.integers(-2, max(2, 2 * dc.max() // 3)))) for _ in range(40)])
    plans.append([(int(r.integers(0, cfg.G)), int(r.integers(0, 9))) for _ in range(4096)])     # the largest plan allowed
    # the traffic matrix of the workload with this GPU's measured row, planned by the library
    g = 0
    D = np.array(W.make_traffic_matrix(cfg)["D"], dtype=np.int64)
    D[g] = dc
    plans.append(P.aurora_chunks(D, None, g))
    sh = H.Share(cfg)
    x = H.dev(inp["x"], cfg.dtype)
    sh.idx.copy_(torch.from_numpy(idx_ref))
    for chunks in plans:
        ref = O.dispatch_chunks(inp["x"], idx_ref, e2g, chunks, cfg.capacity)
        nc = len(chunks) + cfg.G
        plan = P.MoeChunkPlan(sh.ctx, e2g, chunks)
        co = torch.full((nc + 1,), -7, dtype=torch.int32, device=H.DEV)
        po = torch.full((nc + cfg.E + 1,), -7, dtype=torch.int32, device=H.DEV)
        pe = torch.full((nc + cfg.E,), -7, dtype=torch.int32, device=H.DEV)
        npieces = torch.zeros(1, dtype=torch.int32, device=H.DEV)
        sh.send_buf.zero_()
        sh.slot_to_row.fill_(-9)
        sh.row_to_slot.fill_(-9)
        P.moe_dispatch_chunks(sh.ctx, plan, x, sh.idx, sh.send_buf, sh.slot_to_row, sh.row_to_slot, co, po, pe, npieces)
        torch.cuda.synchronize()
        n = ref["n_rows"]
        assert np.array_equal(H.host(sh.slot_to_row), ref["slot_to_row"])
        assert np.array_equal(H.host(sh.row_to_slot)[:n], ref["row_to_slot"])
        assert np.array_equal(H.host(sh.send_buf)[:n], ref["send_buf"])                     # bitwise row copies
        assert np.array_equal(H.host(co), ref["chunk_offset"])
        m = int(npieces.item())
        assert m == len(ref["piece_expert"])
        assert np.array_equal(H.host(po)[:m + 1], ref["piece_offset"])
        assert np.array_equal(H.host(pe)[:m], ref["piece_expert"])
        plan.close()


def make_segments(r, R, nseg, n_local):
    cuts = np.sort(r.integers(0, R + 1, size=nseg - 1))
    off = [0] + [int(c) for c in cuts] + [R]
    exp = [int(v) for v in r.integers(0, n_local, size=nseg)]
    return off, exp


FFN_CASES = [
    # dtype, act, R, H, F, n_local, nseg
    ("fp32", 0, 300, 64, 128, 2, 5),
    ("fp32", 1, 77, 36, 52, 3, 4),
    ("fp32", 2, 130, 64, 128, 2, 6),
    ("bf16", 2, 700, 256, 384, 2, 5),
    ("bf16", 2, 1, 128, 128, 1, 1),
    ("bf16", 1, 523, 256, 512, 3, 7),
    ("bf16", 0, 300, 128, 256, 2, 3),
    ("bf16", 2, 1029, 512, 1408, 4, 9),
    # few tiles and a long K: the tiles of the last, mostly empty round are cut along K into pieces
    ("bf16", 2, 300, 2048, 2048, 1, 1),
    ("bf16", 1, 700, 2048, 2304, 3, 6),
    ("bf16", 0, 257, 3072, 2048, 2, 2),
    # a last round that is between a quarter and half full: two and three pieces of 64 k-tiles
    ("bf16", 2, 700, 4096, 4608, 1, 1),
    ("bf16", 2, 500, 6144, 5120, 1, 1),
    # many short segments with the experts interleaved (several sources, several local experts): tiles
    # gather rows from all segments of an expert
    ("bf16", 1, 2000, 256, 512, 4, 64),
    ("bf16", 2, 1500, 384, 256, 3, 200),
    ("bf16", 0, 900, 2048, 2304, 2, 31),                   # with pieces along K as well
    ("bf16", 2, 3000, 256, 256, 64, 1024),                 # the limits: 64 local experts, 1024 segments (many of them empty)
    ("bf16", 1, 5000, 128, 256, 32, 300),
    # shares of at most 64 rows: the weight-streaming kernels (64-row tiles, tiles cut along K when they are few)
    ("bf16", 2, 16, 2048, 2048, 1, 1),
    ("bf16", 2, 64, 1024, 1408, 2, 3),
    ("bf16", 1, 33, 512, 768, 1, 1),                       # GELU, one row past a 32-row MFMA tile
    ("bf16", 0, 64, 2048, 2304, 3, 9),                     # gathered tiles
    ("bf16", 2, 60, 4096, 1536, 4, 40),                    # more segments than rows in most tiles
    ("bf16", 2, 64, 256, 128, 64, 64),                     # one row per segment, 64 local experts: 64 tiles of one row
    ("bf16", 1, 50, 128, 12800, 2, 2),                     # 100 stages of K in the second GEMM, many pieces
    # just past that path
    ("bf16", 1, 65, 512, 768, 1, 1),
    ("bf16", 2, 250, 256, 128, 64, 250),
]


@pytest.mark.parametrize("dtype,act,R,Hd,F,n_local,nseg", FFN_CASES)
def test_expert_ffn(H, dtype, act, R, Hd, F, n_local, nseg):
    cfg = small("c2_mixtral" if dtype == "bf16" else "c1_tiny_fp32", H=Hd, F=F, act=act, dtype=dtype)
    r = np.random.default_rng(R * 7 + F)
    recv = W.round_to_dtype(r.standard_normal((R, Hd)).astype(np.float32), dtype)
    experts = [W.make_expert_weights(cfg, e) for e in range(n_local)]
    off, exp = make_segments(r, R, nseg, n_local)
    ref = O.expert_ffn(recv, off, exp, experts, act)
    out = H.run_ffn(H.dev(recv, dtype), off, exp, [H.weights_to_dev(w, dtype) for w in experts], Hd, F, act, dtype)
    got = H.host(out)
    assert np.isfinite(got).all()
    H.assert_close(got, ref, dtype)


@pytest.mark.parametrize("which", [1, 2])
def test_ffn_phases_diag_gives_the_results_of_moe_expert_ffn_and_ordered_marks(H, which):
    """The timed instantiation of the GEMM kernel is the GEMM kernel: bitwise the same output; its clock marks do
    not go backwards; blocks that found no tile stop after the first mark; a share of the streaming kernels is refused."""
    Hd, F, R, act = 512, 1408, 700, 2
    cfg = small("c2_mixtral", H=Hd, F=F)
    r = np.random.default_rng(3)
    recv = W.round_to_dtype(r.standard_normal((R, Hd)).astype(np.float32), "bf16")
    experts = [H.weights_to_dev(W.make_expert_weights(cfg, e), "bf16") for e in range(2)]
    off, exp = make_segments(r, R, 5, 2)
    x = H.dev(recv, "bf16")
    ref = H.run_ffn(x, off, exp, experts, Hd, F, act, "bf16")
    i32 = dict(dtype=torch.int32, device=H.DEV)
    so, se = torch.tensor(off, **i32), torch.tensor(exp, **i32)
    ws = torch.empty(H.P.moe_ffn_workspace_bytes(R, Hd, F, act, "bf16"), dtype=torch.uint8, device=H.DEV)
    out = torch.full_like(ref, float("nan"))
    marks = torch.zeros(H.P.ffn_phase_marks_len(R, len(exp), Hd, F, act, which), dtype=torch.int64, device=H.DEV)
    H.P.moe_diag_ffn_phases(x, R, so, se, len(exp), experts, Hd, F, act, "bf16", out, ws, which, marks)
    torch.cuda.synchronize()
    rows = np.zeros(R, dtype=bool)
    for a, b in zip(off[:-1], off[1:]):
        rows[a:b] = True
    assert torch.equal(out[torch.from_numpy(rows).to(H.DEV)], ref[torch.from_numpy(rows).to(H.DEV)])
    a = marks.cpu().numpy().reshape(-1, 4, 4)
    ran = a[:, 0, 3] > 0                                           # blocks that had a tile (the others stop after mark 0)
    assert ran.sum() >= 3                                          # a few tiles at least
    assert (np.diff(a[ran], axis=2) >= 0).all()
    assert (a[~ran][:, :, 1:] == 0).all()
    with pytest.raises(H.P.MoeError):
        H.P.moe_diag_ffn_phases(x, R, so, se, len(exp), experts, Hd, F, act, "bf16", out, ws, which, marks[:64])
    with pytest.raises(H.P.MoeError):
        H.P.moe_diag_ffn_phases(x, 40, torch.tensor([0, 40], **i32), torch.tensor([0], **i32), 1, experts, Hd, F, act, "bf16", out, ws,
                                which, marks)


def test_expert_ffn_leaves_rows_outside_segments_untouched(H):
    cfg = small("c2_mixtral", H=128, F=256)
    r = np.random.default_rng(5)
    recv = W.to_bf16_grid(r.standard_normal((400, 128)).astype(np.float32))
    experts = [W.make_expert_weights(cfg, 0)]
    out = H.run_ffn(H.dev(recv, "bf16"), [10, 10, 300], [0, 0], [H.weights_to_dev(experts[0], "bf16")], 128, 256, 2, "bf16")
    got = H.host(out)
    assert np.isnan(got[:10]).all() and np.isnan(got[300:]).all() and np.isfinite(got[10:300]).all()
    ref = O.expert_ffn(recv[10:300], [0, 290], [0], experts, 2)
    H.assert_close(got[10:300], ref, "bf16")


def test_expert_ffn_rows_beyond_the_32_bit_offsets_of_a_gathered_tile(H):
    """R * F * 2 bytes above 4 GiB: tiles may no longer gather rows from distant segments (their row offsets
    are 32-bit byte offsets), so only adjacent segments of an expert share tiles.  Sampled rows against the
    oracle, plus: no row outside the segments is written."""
    Hd, F, R, n_local = 128, 16384, 140000, 2
    assert R * F * 2 > 2 ** 32
    cfg = small("c2_mixtral", H=Hd, F=F)
    r = np.random.default_rng(99)
    recv = W.round_to_dtype(r.standard_normal((R, Hd)).astype(np.float32), "bf16")
    experts = [W.make_expert_weights(cfg, e) for e in range(n_local)]
    off = [0, 300, 300, 20000, 20100, 60000, 60001, 99000, 99000, 120000, 139000]     # the last 1000 rows: no segment
    exp = [0, 1, 1, 0, 1, 0, 1, 1, 0, 0]
    out = H.run_ffn(H.dev(recv, "bf16"), off, exp, [H.weights_to_dev(w, "bf16") for w in experts], Hd, F, 2, "bf16")
    assert torch.isnan(out[139000:]).all().item() and torch.isfinite(out[:139000]).all().item()
    rows = np.unique(np.concatenate([r.integers(0, 139000, size=150), np.array(off[:-1]), np.array(off[1:]) - 1]))
    rows = rows[(rows >= 0) & (rows < 139000)]
    seg = np.searchsorted(np.array(off), rows, side="right") - 1
    got = H.host(out[torch.from_numpy(rows).to(H.DEV)])
    ref = np.stack([O.ffn(recv[i:i + 1], experts[exp[g]]["w1"], experts[exp[g]]["w_up"], experts[exp[g]]["w_down"], 2)[0]
                    for i, g in zip(rows, seg)])
    H.assert_close(got, ref, "bf16")


@pytest.mark.parametrize("run", [1, 2])
def test_mfma_run_sum_stays_inside_the_error_model_of_the_gate(H, run):
    """The gate certifies indices with the bound |run sum - exact| <= run * 1.05 * 2^-18 * sum |x_i w_i| on what
    v_mfma_f32_16x16x32_bf16 returns.  The instruction is fed random and adversarial operands (wide exponent
    spread, one huge term among many just too small to register, cancelling giants) and held to that bound;
    the exact sums come from rationals-free fp64 (products of bf16 are exact, 64 of them add exactly enough)."""
    r = np.random.default_rng(17 + run)
    K = 32 * run
    fam = []
    a = r.standard_normal((512, 16, K)); b = 0.02 * r.standard_normal((512, 16, K)); fam.append((a, b))
    a = r.standard_normal((512, 16, K)) * 2.0 ** r.integers(-12, 13, size=(512, 16, K))
    b = r.standard_normal((512, 16, K)) * 2.0 ** r.integers(-12, 13, size=(512, 16, K)); fam.append((a, b))
    for q in range(16, 34):                                # one term 2^q, the others a hair below each power of two near its last place
        for small in (1.0, 1.9921875, 3.984375, 7.96875, 15.9375):
            a = np.full((1, 16, K), small); b = np.ones((1, 16, K))
            pos = int(r.integers(0, K))
            a[:, :, pos] = 2.0 ** (q // 2); b[:, :, pos] = 2.0 ** (q - q // 2)
            fam.append((a, b))
            a2, b2 = a.copy(), b.copy()                    # and with a cancelling partner
            a2[:, :, (pos + 5) % K] = -2.0 ** (q // 2); b2[:, :, (pos + 5) % K] = 2.0 ** (q - q // 2)
            fam.append((a2, b2))
    worst = 0.0
    for a, b in fam:
        a, b = W.to_bf16_grid(a.astype(np.float32)), W.to_bf16_grid(b.astype(np.float32))
        d = torch.empty((a.shape[0], 16, 16), dtype=torch.float32, device=H.DEV)
        H.P.moe_diag_mfma_run_sum(H.dev(a, "bf16"), H.dev(b, "bf16"), d)
        torch.cuda.synchronize()
        a64, b64 = a.astype(np.float64), b.astype(np.float64)
        exact = np.einsum("tik,tjk->tij", a64, b64)
        mass = np.einsum("tik,tjk->tij", np.abs(a64), np.abs(b64))
        worst = max(worst, float(np.max(np.abs(H.host(d).astype(np.float64) - exact) / mass)))
    print("worst |error| / sum|x w| for a chain of %d: %.3e = %.3f * 2^-18" % (run, worst, worst * 2.0 ** 18))
    assert worst <= run * 1.05 * 2.0 ** -18


COMBINE_CASES = [W.get_config("c1_tiny_fp32"), small("c2_mixtral", T=333, H=520), small("c3_switch", T=1000, H=64),
                 small("c5_finegrained", T=257, H=264),
                 # k outside 1, 2, 6: the loop kernel (a whole number of groups of four rows, a ragged one, the limit)
                 small("c2_mixtral", T=211, H=520, E=24, k=4), small("c1_tiny_fp32", T=37, H=100, E=5, k=3, G=5),
                 small("c5_finegrained", T=65, H=264, E=160, k=9, G=16), small("c3_switch", T=40, H=1024, E=256, k=16, G=64)]


@pytest.mark.parametrize("cfg", COMBINE_CASES, ids=lambda c: "%s-T%d-H%d-k%d" % (c.name, c.T, c.H, c.k))
@pytest.mark.parametrize("with_shared", [False, True])
def test_combine(H, cfg, with_shared):
    inp = W.make_layer_inputs(cfg)
    idx_ref, w_ref, _ = O.route(inp["x"], inp["w_gate"], inp["gate_bias"], cfg.k, cfg.renorm)
    cap = cfg.capacity
    d = O.dispatch(inp["x"], idx_ref, inp["expert_to_gpu"], list(range(cfg.G)), cap)
    r = np.random.default_rng(11)
    S = cfg.T * cfg.k
    ret = W.round_to_dtype(r.standard_normal((S, cfg.H)).astype(np.float32), cfg.dtype)
    shared = W.round_to_dtype(r.standard_normal((cfg.T, cfg.H)).astype(np.float32), cfg.dtype) if with_shared else None
    w32 = w_ref.astype(np.float32)
    ref = O.combine(ret[:d["n_rows"]], d["slot_to_row"], w32, shared)
    sh = H.Share(cfg)
    sh.slot_to_row.copy_(torch.from_numpy(d["slot_to_row"]))
    sh.w.copy_(torch.from_numpy(w32))
    sh.combine(H.dev(ret, cfg.dtype), None if shared is None else H.dev(shared, cfg.dtype))
    torch.cuda.synchronize()
    assert H.rel_err(H.host(sh.y), ref) < (1e-6 if cfg.dtype == "fp32" else 2 ** -8)
