"""Degenerate sizes and the error behaviour of the device entry points (nothing here may fault:
every bad argument must be turned into a status before any launch)."""
import numpy as np
import pytest
import torch

import workloads as W
from oracle import moe_layer as O

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def H():
    from tests import harness
    assert torch.cuda.is_available()
    return harness


def test_one_token_one_expert_whole_path(H):
    """T = 1, E = 1, k = 1, G = 1: every stage with its smallest input."""
    cfg = W.scaled(W.get_config("c1_tiny_fp32"), T=1, H=8, F=12, E=1, k=1, G=1)
    res = H.run_emulated_cluster(cfg)
    inp = res["inputs"][0]
    ref = O.layer_dense(inp["x"], inp["w_gate"], inp["gate_bias"], 1, cfg.renorm, res["experts"], cfg.act, cfg.capacity, None)
    assert H.rel_err(res["y"][0], ref) < 1e-5


def test_empty_ffn_calls_return_ok_and_touch_nothing(H):
    P = H.P
    w = H.weights_to_dev(W.make_expert_weights(W.scaled(W.get_config("c2_mixtral"), H=128, F=128), 0), "bf16")
    ws = torch.empty(P.moe_ffn_workspace_bytes(16, 128, 128, 2, "bf16"), dtype=torch.uint8, device=H.DEV)
    recv = torch.zeros((16, 128), dtype=torch.bfloat16, device=H.DEV)
    out = torch.full((16, 128), 3.0, dtype=torch.bfloat16, device=H.DEV)
    so = torch.tensor([0, 0], dtype=torch.int32, device=H.DEV)
    se = torch.tensor([0], dtype=torch.int32, device=H.DEV)
    P.moe_expert_ffn(recv, 0, so, se, 1, [w], 128, 128, 2, "bf16", out, ws)          # no rows
    P.moe_expert_ffn(recv, 16, so, se, 0, [w], 128, 128, 2, "bf16", out, ws)         # no segments
    P.moe_expert_ffn(recv, 16, so, se, 1, [w], 128, 128, 2, "bf16", out, ws)         # one empty segment
    torch.cuda.synchronize()
    assert torch.all(out == 3.0)


def test_all_slots_dropped_by_capacity_of_one(H):
    """capacity = 1: every expert keeps exactly its first slot; combine gives w * row for those only."""
    cfg = W.scaled(W.get_config("c3_switch"), T=300, H=64, E=8, G=4)
    inp = W.make_layer_inputs(cfg)
    idx_ref, w_ref, _ = O.route(inp["x"], inp["w_gate"], inp["gate_bias"], cfg.k, cfg.renorm)
    P = H.P
    ctx = P.MoeCtx(cfg.T, cfg.H, cfg.E, cfg.k, cfg.G, cfg.dtype, cfg.renorm, 1)
    sh = H.Share(cfg)
    sh.ctx = ctx
    x = H.dev(inp["x"], cfg.dtype)
    sh.idx.copy_(torch.from_numpy(idx_ref))
    sh.traffic(inp["expert_to_gpu"])
    sh.dispatch(x, inp["expert_to_gpu"], list(range(cfg.G)))
    torch.cuda.synchronize()
    d = O.dispatch(inp["x"], idx_ref, inp["expert_to_gpu"], list(range(cfg.G)), 1)
    assert d["n_rows"] == len(set(idx_ref.reshape(-1).tolist()))
    assert np.array_equal(H.host(sh.slot_to_row), d["slot_to_row"])
    assert int(H.host(sh.n_dropped)[0]) == cfg.T * cfg.k - d["n_rows"]
    assert np.array_equal(H.host(sh.send_buf)[:d["n_rows"]], d["send_buf"])


def test_bad_arguments_are_statuses_not_launches(H):
    P = H.P
    cfg = W.scaled(W.get_config("c2_mixtral"), T=64, H=256, F=256)
    sh = H.Share(cfg)
    x = torch.zeros((cfg.T, cfg.H), dtype=torch.bfloat16, device=H.DEV)
    wg = torch.zeros((cfg.E, cfg.H), dtype=torch.bfloat16, device=H.DEV)
    e2g = list(np.arange(cfg.E) // (cfg.E // cfg.G))
    order = list(range(cfg.G))
    # misaligned row pointers
    raw = torch.zeros(cfg.T * cfg.H + 8, dtype=torch.bfloat16, device=H.DEV)
    with pytest.raises(P.MoeError):
        P.moe_route(sh.ctx, raw[1:1 + cfg.T * cfg.H].view(cfg.T, cfg.H), wg, None, sh.idx, sh.w)
    with pytest.raises(P.MoeError):
        P.moe_dispatch(sh.ctx, raw[1:1 + cfg.T * cfg.H].view(cfg.T, cfg.H), sh.idx, e2g, order, sh.send_buf, sh.slot_to_row,
                       sh.row_to_slot, sh.seg_offset, sh.seg_expert)
    # destination order that is no permutation, expert on a GPU that does not exist
    with pytest.raises(P.MoeError):
        P.moe_dispatch(sh.ctx, x, sh.idx, e2g, [0] * cfg.G, sh.send_buf, sh.slot_to_row, sh.row_to_slot, sh.seg_offset,
                       sh.seg_expert)
    with pytest.raises(P.MoeError):
        P.moe_traffic(sh.ctx, sh.idx, [cfg.G] * cfg.E, sh.expert_count, sh.dest_count, sh.n_dropped)
    # shapes the context refuses
    for bad in (dict(E=257), dict(k=17), dict(G=65), dict(k=cfg.E + 1), dict(T=0), dict(H=3)):
        kw = dict(T=cfg.T, H=cfg.H, E=cfg.E, k=cfg.k, G=cfg.G)
        kw.update(bad)
        with pytest.raises(P.MoeError):
            P.MoeCtx(kw["T"], kw["H"], kw["E"], kw["k"], kw["G"], "bf16")
    # expert FFN: workspace too small, sizes the bf16 kernel does not take, too many segments
    w = H.weights_to_dev(W.make_expert_weights(cfg, 0), "bf16")
    recv = torch.zeros((32, cfg.H), dtype=torch.bfloat16, device=H.DEV)
    out = torch.zeros_like(recv)
    so = torch.tensor([0, 32], dtype=torch.int32, device=H.DEV)
    se = torch.tensor([0], dtype=torch.int32, device=H.DEV)
    small_ws = torch.empty(1024, dtype=torch.uint8, device=H.DEV)
    with pytest.raises(P.MoeError):
        P.moe_expert_ffn(recv, 32, so, se, 1, [w], cfg.H, cfg.F, 2, "bf16", out, small_ws)
    ws = torch.empty(P.moe_ffn_workspace_bytes(32, cfg.H, cfg.F, 2, "bf16"), dtype=torch.uint8, device=H.DEV)
    with pytest.raises(P.MoeError):
        P.moe_expert_ffn(recv, 32, so, se, 1, [w], cfg.H - 64, cfg.F, 2, "bf16", out, ws)
    with pytest.raises(P.MoeError):
        P.moe_expert_ffn(recv, 32, so, se, 1025, [w], cfg.H, cfg.F, 2, "bf16", out, ws)
    with pytest.raises(P.MoeError):
        P.moe_expert_ffn(recv, 32, so, se, 1, [w] * 65, cfg.H, cfg.F, 2, "bf16", out, ws)
    assert P.moe_ffn_workspace_bytes(-1, cfg.H, cfg.F, 2, "bf16") == 0
    # chunk plans: too many chunks; a plan made for another shape
    with pytest.raises(P.MoeError):
        P.MoeChunkPlan(sh.ctx, e2g, [(0, 1)] * 4097)
    other = H.Share(W.scaled(cfg, E=16, G=8, T=64))
    plan = P.MoeChunkPlan(other.ctx, list(np.arange(16) // 2), [(0, 5)])
    i32 = dict(dtype=torch.int32, device=H.DEV)
    with pytest.raises(P.MoeError):
        P.moe_dispatch_chunks(sh.ctx, plan, x, sh.idx, sh.send_buf, sh.slot_to_row, sh.row_to_slot, torch.zeros(64, **i32),
                              torch.zeros(64, **i32), torch.zeros(64, **i32), torch.zeros(1, **i32))
    torch.cuda.synchronize()                                    # nothing was launched, nothing is pending
