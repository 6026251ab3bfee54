"""Full-size parity in the launch configuration bench.py times: the whole step runs on the GPU at the
workload's real shape; integer results are compared in full with the oracle, floating-point results on
sampled rows / tokens the oracle computes one by one."""
import numpy as np
import pytest
import torch

import workloads as W
from oracle import moe_layer as O

pytestmark = pytest.mark.gpu
TOL = {"fp32": 1e-5, "bf16": 2e-2}


@pytest.fixture(scope="module")
def env():
    import bench
    import paper_2410_17043_amd as P
    from tests import harness
    assert torch.cuda.is_available()
    return bench, P, harness


def check_share(H, cfg, wl):
    """One share after its step ran: integers in full, floating point on sampled rows and tokens."""
    inp, g = wl["inp"], wl["g"]
    e2g = inp["expert_to_gpu"]
    T, k = cfg.T, cfg.k

    # gate: indices bit-exact on every token, weights within 1e-5
    idx_ref, w_ref, z = O.route(inp["x"], inp["w_gate"], inp["gate_bias"], k, cfg.renorm)
    assert O.route_margin(z, k).min() > 1e-9
    assert np.array_equal(H.host(wl["idx"]), idx_ref)
    assert np.max(np.abs(H.host(wl["w"]) / w_ref - 1.0)) < 1e-5

    # traffic row and permutation: exact, in full
    ec, dc, nd, keep = O.traffic(idx_ref, e2g, cfg.G, cfg.capacity)
    assert np.array_equal(H.host(wl["expert_count"]), ec)
    assert np.array_equal(H.host(wl["dest_count"]), dc)
    assert int(wl["n_dropped"].item()) == nd
    ref = O.dispatch(inp["x"], idx_ref, e2g, list(wl["dest_order"]), cfg.capacity)
    n = ref["n_rows"]
    s2r = H.host(wl["slot_to_row"])
    assert np.array_equal(s2r, ref["slot_to_row"])
    assert np.array_equal(H.host(wl["row_to_slot"])[:n], ref["row_to_slot"])
    assert np.array_equal(H.host(wl["seg_offset"]), ref["seg_offset"])
    assert np.array_equal(H.host(wl["seg_expert"]), ref["seg_expert"])
    r = np.random.default_rng(cfg.seed_base + 77)
    rows = np.unique(np.concatenate([r.integers(0, n, size=512), [0, n - 1]]))
    got_rows = wl["send_buf"][torch.from_numpy(rows).to(H.DEV)]
    assert np.array_equal(H.host(got_rows), ref["send_buf"][rows])             # bitwise row copies

    # expert FFN on sampled received rows, every segment covered, including first and last rows of tiles
    off, exp, local = wl["ffn_off"], wl["ffn_exp"], wl["local"]
    R = wl["R"]
    experts = {li: W.make_expert_weights(cfg, e) for li, e in enumerate(local) if li in set(exp)}
    worst = 0.0
    for i, li in enumerate(exp):
        lo, hi = off[i], off[i + 1]
        pick = np.unique(np.concatenate([r.integers(lo, hi, size=6), [lo, hi - 1]]))
        rin = H.host(wl["recv"][torch.from_numpy(pick).to(H.DEV)])
        wgt = experts[li]
        want = O.ffn(rin, wgt["w1"], wgt.get("w_up"), wgt["w_down"], cfg.act)
        got = H.host(wl["ffn_out"][torch.from_numpy(pick).to(H.DEV)])
        worst = max(worst, H.assert_close(got, want, cfg.dtype, ("segment", i))[0])
    assert worst < TOL[cfg.dtype], worst
    assert off[-1] == R

    # combine on sampled tokens (the oracle gets only the rows those tokens need)
    toks = np.unique(np.concatenate([r.integers(0, T, size=200), [0, T - 1]]))
    need = np.unique(s2r.reshape(T, k)[toks].ravel())
    need = need[need >= 0]
    ret_rows = H.host(wl["ret"][torch.from_numpy(need).to(H.DEV)]) if len(need) else np.zeros((0, cfg.H))
    remap = {int(row): i for i, row in enumerate(need)}
    s2r_small = np.array([[remap.get(int(v), -1) if v >= 0 else -1 for v in s2r.reshape(T, k)[t]] for t in toks]).ravel()
    # shared experts, by their definition: the sum of every shared expert's FFN over the token (the GPU runs
    # one FFN with stacked weights); first the shared output alone, then inside the combine
    shared_ref = None
    if cfg.n_shared:
        xt = inp["x"][toks]
        for s_ in range(cfg.n_shared):
            sw = W.make_expert_weights(cfg, s_, shared=True)
            o = O.ffn(xt, sw["w1"], sw["w_up"], sw["w_down"], cfg.act)
            shared_ref = o if shared_ref is None else shared_ref + o
        got_sh = H.host(wl["shared_out"][torch.from_numpy(toks).to(H.DEV)])
        H.assert_close(got_sh, shared_ref, cfg.dtype, "shared experts")
        shared_ref = got_sh                                  # combine adds what the GPU stored (rounded to bf16)
    else:
        assert wl["shared_out"] is None
    want = O.combine(ret_rows, s2r_small, H.host(wl["w"])[toks], shared_ref)
    got = H.host(wl["y"][torch.from_numpy(toks).to(H.DEV)])
    assert H.rel_err(got, want) < 2 ** -8 and H.rms_rel_err(got, want) < 2 ** -9

    # loop-back rows really went through: the self segment of the return buffer equals the FFN output rows
    for (r0, lo, hi) in wl["self_spans"]:
        assert torch.equal(wl["ret"][lo:hi], wl["ffn_out"][r0:r0 + hi - lo])


@pytest.mark.parametrize("name", ["c2_mixtral", "c3_switch", "c4a_coloc", "c4b_coloc", "c5_finegrained"])
def test_full_size_step(env, name):
    bench, P, H = env
    cfg = W.get_config(name)
    wl = bench.build_workload(cfg, torch, P, W)
    assert (wl["shared_out"] is not None) == (cfg.n_shared > 0)
    wl["step"]()
    torch.cuda.synchronize()
    check_share(H, cfg, wl)


def test_full_size_colocated_gpu(env):
    """Two models on one GPU as the colocation places them: model a's expert and the block of model b's experts
    that colocate_match pairs with it, both steps at full size, the two expert FFNs on two HIP streams.  The
    concurrent run must give the bits of the one-stream run, and each share is checked against the oracle."""
    bench, P, H = env
    from oracle import matching as OM
    co = bench.build_coloc(torch, P, W)
    ca, cb, wa, wb = co["ca"], co["cb"], co["wa"], co["wb"]
    # the pairing: a valid injection whose largest edge weight is the brute-force-checked bottleneck value
    Da, Db = W.make_traffic_matrix(ca)["D"], W.make_traffic_matrix(cb)["D"]
    Wm = OM.pair_weights(Da, Db)
    assert sorted(co["pair"]) == list(range(8))
    assert max(Wm[i][co["pair"][i]] for i in range(8)) == co["bottleneck"] == OM.best_pairing_threshold(Da, Db)[0]
    # placement reached the shares: b's two experts on the GPU under test are the block paired with a's expert
    g = co["g"]
    assert wa["local"] == [g] and wb["local"] == [2 * co["pair"][g], 2 * co["pair"][g] + 1]
    assert g == int(np.argmax(co["Dn"].sum(axis=0)))
    co["step_serial"]()
    torch.cuda.synchronize()
    serial = [w_[k].clone() for w_ in (wa, wb) for k in ("ffn_out", "y")]
    for rep in range(2):
        for w_ in (wa, wb):
            w_["ffn_out"].zero_()
            w_["y"].zero_()
        torch.cuda.synchronize()                             # the zero fills are done before the side stream starts
        co["step"]()
        torch.cuda.synchronize()
        conc = [w_[k] for w_ in (wa, wb) for k in ("ffn_out", "y")]
        assert all(torch.equal(a, b) for a, b in zip(serial, conc)), rep
    check_share(H, ca, wa)
    check_share(H, cb, wb)
