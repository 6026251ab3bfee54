"""moe_dispatch_noalloc (static device scratch, no allocation) against moe_dispatch: bit-exact, on two
calls in a row, the second with a smaller input that takes the other rank-pass path."""
import numpy as np
import pytest
import torch

import workloads as W
from oracle import moe_layer as O

pytestmark = pytest.mark.gpu


def one_call(H, cfg, seed):
    P = H.P
    inp = W.make_layer_inputs(cfg)
    e2g = inp["expert_to_gpu"]
    order = list(np.random.default_rng(seed).permutation(cfg.G))
    idx_ref, _, _ = O.route(inp["x"], inp["w_gate"], inp["gate_bias"], cfg.k, cfg.renorm)
    x = H.dev(inp["x"], cfg.dtype)
    a, b = H.Share(cfg), H.Share(cfg)                      # a: through a context; b: the buffers of the static call
    for sh in (a, b):
        sh.idx.copy_(torch.from_numpy(idx_ref))
    a.dispatch(x, e2g, order)
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    P.moe_dispatch_noalloc((cfg.T, cfg.H, cfg.E, cfg.k, cfg.G, cfg.dtype, cfg.renorm, cfg.capacity), x, b.idx, e2g, order,
                           b.send_buf, b.slot_to_row, b.row_to_slot, b.seg_offset, b.seg_expert)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    ref = O.dispatch(inp["x"], idx_ref, e2g, order, cfg.capacity)
    n = ref["n_rows"]
    for name in ("slot_to_row", "seg_offset", "seg_expert"):
        assert torch.equal(getattr(a, name), getattr(b, name)), name
    assert torch.equal(a.row_to_slot[:n], b.row_to_slot[:n])
    assert torch.all(b.row_to_slot[n:] == -7)
    assert torch.equal(a.send_buf, b.send_buf)             # rows past the kept count stay zero in both
    assert np.array_equal(H.host(b.slot_to_row), ref["slot_to_row"])
    assert np.array_equal(H.host(b.send_buf)[:n], ref["send_buf"])


def test_noalloc_dispatch_matches_dispatch_twice_in_a_row():
    from tests import harness as H
    assert torch.cuda.is_available()
    big = W.scaled(W.get_config("c5_finegrained"), T=3500, H=64)          # 21000 slots, 64 experts: three-kernel rank pass
    small = W.scaled(W.get_config("c3_switch"), T=700, H=128)             # 700 slots, capacity drops: one-block rank pass
    one_call(H, big, 1)
    one_call(H, small, 2)
    one_call(H, W.scaled(W.get_config("c2_mixtral"), T=300, H=264), 3)    # 8 experts, k = 2


def test_noalloc_dispatch_rejects_what_does_not_fit():
    from tests import harness as H
    P = H.P
    t = torch.zeros(16, dtype=torch.int32, device=H.DEV)
    with pytest.raises(P.MoeError) as ei:                                  # 2^20 + 16 slots: beyond the static scratch
        P.moe_dispatch_noalloc(((1 << 16) + 1, 64, 64, 16, 16, "bf16", 0, 0), t, t, [e // 4 for e in range(64)], list(range(16)),
                               t, t, t, t, t)
    assert ei.value.name == "MOE_ESHAPE"
    with pytest.raises(P.MoeError):                                        # the shape checks of moe_ctx_create apply
        P.moe_dispatch_noalloc((8, 64, 8, 9, 4, "bf16", 0, 0), t, t, [0] * 8, list(range(4)), t, t, t, t, t)
