"""The whole path (route -> dispatch -> all-to-all -> expert FFN -> all-to-all -> combine) over an
emulated cluster, against the per-token definition y_t = sum_j w_tj FFN_{e_tj}(x_t) (+ shared)."""
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
    assert torch.cuda.is_available()
    return harness


def check_cluster(H, cfg, n_shared=0, chunked=False):
    res = H.run_emulated_cluster(cfg, n_shared=n_shared, chunked=chunked)
    inp0 = res["inputs"][0]
    worst = 0.0
    for g in range(cfg.G):
        ref = O.layer_dense(res["inputs"][g]["x"], inp0["w_gate"], inp0["gate_bias"], cfg.k, cfg.renorm,
                            res["experts"], cfg.act, cfg.capacity, res["shared"] or None)
        err, _rms = H.assert_close(res["y"][g], ref, cfg.dtype, g)
        worst = max(worst, err)
    # the measured traffic matrix is what the oracle counts
    for g in range(cfg.G):
        idx, _, _ = O.route(res["inputs"][g]["x"], inp0["w_gate"], inp0["gate_bias"], cfg.k, cfg.renorm)
        _, dc, _, _ = O.traffic(idx, inp0["expert_to_gpu"], cfg.G, cfg.capacity)
        assert np.array_equal(res["D"][g], dc)
    return worst


def test_c1_tiny_full_layer(H):
    check_cluster(H, W.get_config("c1_tiny_fp32"))


@pytest.mark.parametrize("name,kw,n_shared", [
    ("c2_mixtral", dict(T=96, H=256, F=384, G=4), 0),
    ("c3_switch", dict(T=200, H=128, F=256, E=16, G=4), 0),            # capacity drops on every GPU
    ("c4b_coloc", dict(T=64, H=128, F=256, G=4), 0),
    ("c5_finegrained", dict(T=80, H=128, F=128, E=16, G=4), 2),        # two shared experts on every token
])
def test_reduced_configs_full_layer(H, name, kw, n_shared):
    cfg = W.scaled(W.get_config(name), **kw)
    check_cluster(H, cfg, n_shared)


@pytest.mark.parametrize("name,kw", [
    ("c1_tiny_fp32", dict()),
    ("c2_mixtral", dict(T=96, H=256, F=384, G=4)),
    ("c3_switch", dict(T=200, H=128, F=256, E=16, G=4)),               # capacity drops on every GPU
])
def test_full_layer_with_the_preemptive_send_plan(H, name, kw):
    """Same layer, send buffers laid out chunk by chunk for the rounds of the library's schedule."""
    cfg = W.scaled(W.get_config(name), **kw) if kw else W.get_config(name)
    check_cluster(H, cfg, chunked=True)


def test_two_colocated_models_concurrent_streams_match_serial(H):
    """Two models' experts share the GPU: their FFNs on two streams give the bits of the serial run."""
    P = H.P
    out = {}
    cases = {"a": W.scaled(W.get_config("c4a_coloc"), H=512, F=1792), "b": W.scaled(W.get_config("c4b_coloc"), H=256, F=640)}
    data = {}
    for key, cfg in cases.items():
        r = np.random.default_rng(cfg.seed_base)
        R = 900 if key == "a" else 1500
        recv = H.dev(W.to_bf16_grid(r.standard_normal((R, cfg.H)).astype(np.float32)), "bf16")
        w = H.weights_to_dev(W.make_expert_weights(cfg, 0), "bf16")
        so = torch.tensor([0, R // 3, R], dtype=torch.int32, device=H.DEV)
        se = torch.tensor([0, 0], dtype=torch.int32, device=H.DEV)
        ws = torch.empty(P.moe_ffn_workspace_bytes(R, cfg.H, cfg.F, cfg.act, "bf16"), dtype=torch.uint8, device=H.DEV)
        data[key] = (cfg, R, recv, w, so, se, ws)

    def launch(key, out_t):
        cfg, R, recv, w, so, se, ws = data[key]
        P.moe_expert_ffn(recv, R, so, se, 2, [w], cfg.H, cfg.F, cfg.act, "bf16", out_t, ws)

    serial = {k: torch.zeros((data[k][1], data[k][0].H), dtype=torch.bfloat16, device=H.DEV) for k in cases}
    for k in cases:
        launch(k, serial[k])
    torch.cuda.synchronize()
    conc = {k: torch.zeros_like(serial[k]) for k in cases}
    streams = {k: torch.cuda.Stream() for k in cases}            # default priority
    for rep in range(3):
        for k in cases:
            conc[k].zero_()
        for k in cases:
            streams[k].wait_stream(torch.cuda.current_stream())  # the zero fill above is ordered before the FFN
            with torch.cuda.stream(streams[k]):
                launch(k, conc[k])
        for k in cases:
            torch.cuda.current_stream().wait_stream(streams[k])
        torch.cuda.synchronize()
        for k in cases:
            assert torch.equal(conc[k], serial[k])
    for k, (cfg, R, recv, w, *_rest) in data.items():
        ref = O.ffn(H.host(recv), H.host(w["w1"]), H.host(w["w_up"]), H.host(w["w_down"]), cfg.act)
        H.assert_close(H.host(serial[k]), ref, "bf16", k)
