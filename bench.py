#!/usr/bin/env python3
"""Benchmark of one GPU's share of an expert-parallel MoE layer on one MI355X.

A step is one pass of the whole hot path over one batch of synthetic input:
route -> traffic -> dispatch -> expert FFN over the rows this GPU receives -> combine.
The workload is the Mixtral-shape share: 4096 local tokens, hidden 4096, SwiGLU
4096 -> 14336 -> 4096, 8 experts top-2 over 8 simulated GPUs; the GPU under test hosts
the most popular expert and receives the largest column of a Zipf(1.0) traffic matrix.
All inputs are resident in HBM before the timed region.  One JSON line is printed.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0         # MI355X HBM3E
# HBM-side bytes per launch of the first FFN GEMM at c2_mixtral from rocprofv3 counters (FETCH_SIZE x 2.0 +
# WRITE_SIZE x 1.0, see profiles/bench_c2_mixtral_layer_share.md); None once the kernel has changed since.
GEMM1_TRAFFIC_BYTES = {"c2_mixtral": 3.9033e6 * 1024 * 2.0 + 6.6752e5 * 1024}


def build_workload(cfg, torch, P, W, share="bottleneck"):
    """Everything a step needs, resident on the GPU.  Returns a dict of tensors and the step closure."""
    dev = "cuda:0"
    tdt = P.TORCH_DTYPE[cfg.dtype]

    def to_dev(a):
        return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(dev).to(tdt).contiguous()

    traffic = W.make_traffic_matrix(cfg)
    D = traffic["D"].copy()
    received = D.sum(axis=0)
    if share == "median":
        g = int(np.argsort(received, kind="stable")[len(received) // 2])
    else:
        g = int(np.argmax(received))                        # the GPU that receives most sets the layer time
    inp = W.make_layer_inputs(cfg, g)
    e2g = inp["expert_to_gpu"]
    local = [e for e in range(cfg.E) if e2g[e] == g]
    x, wg = to_dev(inp["x"]), to_dev(inp["w_gate"])
    bias = None if inp["gate_bias"] is None else torch.from_numpy(inp["gate_bias"]).to(dev)
    experts = []
    for e in local:
        w = W.make_expert_weights(cfg, e)
        experts.append({k: (to_dev(v) if v is not None else None) for k, v in w.items()})
    table = P.expert_table(experts)

    T, k, H, F, E, G = cfg.T, cfg.k, cfg.H, cfg.F, cfg.E, cfg.G
    S = T * k
    ctx = P.MoeCtx(T, H, E, k, G, cfg.dtype, cfg.renorm, cfg.capacity)
    ctx.set_rank_reuse(True)      # in the step moe_dispatch directly follows moe_traffic on the same indices
    i32 = dict(dtype=torch.int32, device=dev)
    idx = torch.zeros((T, k), **i32)
    w = torch.zeros((T, k), dtype=torch.float32, device=dev)
    expert_count, dest_count, n_dropped = torch.zeros(E, **i32), torch.zeros(G, **i32), torch.zeros(1, **i32)
    send_buf = torch.zeros((S, H), dtype=tdt, device=dev)
    s2r, r2s = torch.zeros(S, **i32), torch.zeros(S, **i32)
    seg_offset, seg_expert = torch.zeros(E + 1, **i32), torch.zeros(E, **i32)
    y = torch.zeros((T, H), dtype=tdt, device=dev)

    # set-up pass: this GPU's own row of the traffic matrix is the measured one
    P.moe_route(ctx, x, wg, bias, idx, w)
    P.moe_traffic(ctx, idx, e2g, expert_count, dest_count, n_dropped)
    torch.cuda.synchronize()
    own_expert = expert_count.cpu().numpy().astype(np.int64)
    D[g] = dest_count.cpu().numpy()
    traffic["per_expert"][g] = own_expert
    rates = W.make_link_rates(cfg) if cfg.hetero_links else None
    plan = P.aurora_order(D, rates)                          # offline plan from the statistics
    dest_order = plan["dest_order"][g]
    P.moe_dispatch(ctx, x, idx, e2g, dest_order, send_buf, s2r, r2s, seg_offset, seg_expert)
    torch.cuda.synchronize()
    so = seg_offset.cpu().numpy()
    se = seg_expert.cpu().numpy()

    # received rows: sources in the order their flow to g starts in the plan, expert-sorted inside a source
    start_to_g = plan["start"][:, g]
    sources = sorted(range(G), key=lambda i: (start_to_g[i] if (i != g and start_to_g[i] >= 0) else np.inf, i))
    off, exp, self_spans = [0], [], []
    for i in sources:
        for li, e in enumerate(local):
            n = int(traffic["per_expert"][i][e])
            if n == 0:
                continue
            if i == g:
                p = int(np.nonzero(se == e)[0][0])
                self_spans.append((off[-1], int(so[p]), int(so[p + 1])))
            off.append(off[-1] + n)
            exp.append(li)
    R = off[-1]
    recv = torch.empty((R, H), dtype=tdt, device=dev)
    chunk = 4096
    for r0 in range(0, R, chunk):                            # rows from other GPUs: seeded N(0,1)
        n = min(chunk, R - r0)
        recv[r0:r0 + n] = to_dev(W.generate.make_rows(cfg, W.generate.S_RECV, n, sub=r0 // chunk))
    ffn_off = torch.tensor(off, **i32)
    ffn_exp = torch.tensor(exp, **i32)
    ffn_out = torch.empty((R, H), dtype=tdt, device=dev)
    ws = torch.empty(P.moe_ffn_workspace_bytes(R, H, F, cfg.act, cfg.dtype), dtype=torch.uint8, device=dev)
    ret = torch.empty((S, H), dtype=tdt, device=dev)
    for r0 in range(0, S, chunk):                            # rows returned by other GPUs: seeded N(0,1)
        n = min(chunk, S - r0)
        ret[r0:r0 + n] = to_dev(W.generate.make_rows(cfg, W.generate.S_RET, n, sub=r0 // chunk))
    # a plain device copy of known size (256 MiB read + 256 MiB written): the reference that the
    # FETCH_SIZE / WRITE_SIZE hardware counters of a profiled run are scaled by
    calib_src = torch.empty(256 << 20, dtype=torch.uint8, device=dev)
    calib_dst = torch.empty_like(calib_src)
    calib_dst.copy_(calib_src)
    del calib_src, calib_dst
    torch.cuda.synchronize()

    b_route = P.bind_route(ctx, x, wg, bias, idx, w)
    b_traffic = P.bind_traffic(ctx, idx, e2g, expert_count, dest_count, n_dropped)
    b_dispatch = P.bind_dispatch(ctx, x, idx, e2g, dest_order, send_buf, s2r, r2s, seg_offset, seg_expert)
    b_ffn = P.bind_expert_ffn(recv, R, ffn_off, ffn_exp, len(exp), table, H, F, cfg.act, cfg.dtype, ffn_out, ws)
    b_combine = P.bind_combine(ctx, ret, s2r, w, None, y)

    # the same send buffer laid out for the preemptive plan of the schedule's rounds: timed beside the
    # stages for information, not part of the step (it writes buffers of its own)
    chunks = P.aurora_chunks(D, rates, g)
    chunk_plan = P.MoeChunkPlan(ctx, e2g, chunks)
    nc = len(chunks) + G
    c_send = torch.zeros((S, H), dtype=tdt, device=dev)
    c_s2r, c_r2s = torch.zeros(S, **i32), torch.zeros(S, **i32)
    c_off, p_off, p_exp, n_pieces = torch.zeros(nc + 1, **i32), torch.zeros(nc + E + 1, **i32), torch.zeros(nc + E, **i32), torch.zeros(1, **i32)
    b_dispatch_chunks = P.bind_dispatch_chunks(ctx, chunk_plan, x, idx, c_send, c_s2r, c_r2s, c_off, p_off, p_exp, n_pieces)

    def cur():
        return torch.cuda.current_stream().cuda_stream

    def step():
        st = cur()
        b_route(st)
        b_traffic(st)
        b_dispatch(st)
        for (r0, lo, hi) in self_spans:                      # loop-back part of the first all-to-all
            recv[r0:r0 + hi - lo].copy_(send_buf[lo:hi], non_blocking=True)
        b_ffn(st)
        for (r0, lo, hi) in self_spans:                      # loop-back part of the second all-to-all
            ret[lo:hi].copy_(ffn_out[r0:r0 + hi - lo], non_blocking=True)
        b_combine(st)

    def traffic_then(b):
        def fn():
            b_traffic(cur())
            b(cur())
        return fn

    # a dispatch reuses the slot ranks of the moe_traffic in front of it, as in the step, so the two dispatch
    # stages are timed as a pair with moe_traffic and main() subtracts the traffic stage
    stages = {"route": lambda: b_route(cur()), "traffic": lambda: b_traffic(cur()),
              "traffic+dispatch": traffic_then(b_dispatch),
              "expert_ffn": lambda: b_ffn(cur()), "combine": lambda: b_combine(cur()),
              "traffic+dispatch_chunks": traffic_then(b_dispatch_chunks)}
    ffn_timed = lambda: P.moe_expert_ffn_timed(recv, R, ffn_off, ffn_exp, len(exp), table, H, F, cfg.act, cfg.dtype,
                                               ffn_out, ws)
    n_kept = int(so[-1])
    return dict(step=step, stages=stages, ffn_timed=ffn_timed, R=R, g=g, n_kept=n_kept, inp=inp, y=y,
                idx=idx, w=w, expert_count=expert_count, dest_count=dest_count, n_dropped=n_dropped,
                send_buf=send_buf, slot_to_row=s2r, row_to_slot=r2s, seg_offset=seg_offset, seg_expert=seg_expert,
                recv=recv, ffn_out=ffn_out, ret=ret, ffn_off=off, ffn_exp=exp, local=local, dest_order=dest_order,
                self_spans=self_spans, n_chunks=len(chunks), D=D, rates=rates, plan=plan, keep=(ctx, x, wg, bias, experts, table, ws, chunk_plan))


def box_reference(torch, wl, cfg):
    """What this very box sustains, for orientation beside the published peaks: a plain device copy
    (256 MiB read + 256 MiB written) and, for bf16 workloads, the vendor library's GEMM of the first FFN
    GEMM's shape (one projection, no activation; torch.matmul -> hipBLASLt).  Neither is on the product path."""
    dev = wl["recv"].device
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
    src = torch.empty(256 << 20, dtype=torch.uint8, device=dev)
    dst = torch.empty_like(src)
    dst.copy_(src)
    ev[0].record()
    for _ in range(5):
        dst.copy_(src)
    ev[1].record()
    ev[1].synchronize()
    out = {"copy_GBps": round(5 * 2 * (256 << 20) / (ev[0].elapsed_time(ev[1]) * 1e-3) / 1e9, 1)}
    del src, dst
    if cfg.dtype == "bf16":
        w1 = wl["keep"][4][0]["w1"]                              # [F, H] of the first local expert
        recv = wl["recv"]
        c = recv @ w1.t()
        torch.cuda.synchronize()
        ev[0].record()
        for _ in range(5):
            c = recv @ w1.t()
        ev[1].record()
        ev[1].synchronize()
        flops = 5 * 2.0 * recv.shape[0] * w1.shape[0] * w1.shape[1]
        out["vendor_gemm_bf16_TFLOPs"] = round(flops / (ev[0].elapsed_time(ev[1]) * 1e-3) / 1e12, 1)
        out["vendor_gemm_shape"] = [int(recv.shape[0]), int(w1.shape[0]), int(w1.shape[1])]
    return out


PAPER_LINK_GBPS = 12.5        # the 100 Gbps port of the paper's simulation set-up (Sec. 8.1), in GB/s


def paper_model(cfg, wl, stage_ms, P):
    """The paper's own metrics for this synthetic traffic matrix (Sec. 4.1 Eqn. 3, Sec. 8.1), with the
    computation times measured here and the all-to-alls modelled on the big switch of Sec. 2.4:
    inference time = |G| + max|N_i| + max|F_i| + max|C_i| + |A| where G = route + traffic + dispatch,
    F = expert FFN, A = combine on the GPU under test (the one that receives most), and the
    communication time of a transmission order is its completion time on ports of PAPER_LINK_GBPS
    (token rows of H elements).  Orders: the library's (Algorithm 1), the bound of Theorem 2 / 4 that the
    rounds of Appendix A attain, shortest flow first, and a seeded random order."""
    D, rates, plan = wl["D"], wl["rates"], wl["plan"]
    G_ = cfg.G
    row_bytes = cfg.H * (2 if cfg.dtype == "bf16" else 4)
    ms_per_unit = row_bytes / (PAPER_LINK_GBPS * 1e9) * 1e3          # one token over a rate-1 port
    off = D.astype(np.float64).copy()
    np.fill_diagonal(off, 0.0)
    sjf = np.array([sorted(range(G_), key=lambda j: (off[i, j], j)) for i in range(G_)], dtype=np.int32)
    rng = np.random.default_rng(cfg.seed_base + 77)
    rcs = np.array([rng.permutation(G_) for _ in range(G_)], dtype=np.int32)
    comm = {"theorem_bound": plan["bmax"] * ms_per_unit,
            "aurora_order": P.aurora_simulate(D, rates, plan["dest_order"]) * ms_per_unit,
            "shortest_first": P.aurora_simulate(D, rates, sjf) * ms_per_unit,
            "random_order": P.aurora_simulate(D, rates, rcs) * ms_per_unit}
    g_ms = stage_ms["route"] + stage_ms["traffic"] + stage_ms["dispatch"]
    f_ms, a_ms = stage_ms["expert_ffn"], stage_ms["combine"]
    out = {"link_GBps": PAPER_LINK_GBPS, "comm_ms_one_all_to_all": {k: round(v, 4) for k, v in comm.items()}}
    for k, c in comm.items():
        # the second all-to-all is the first reversed: same duration (Sec. 2.2)
        t = P.aurora_layer_time([g_ms], [c], [f_ms], [c], [a_ms])
        out["inference_ms_" + k] = round(t, 4)
        out["gpu_utilisation_" + k] = round((g_ms + f_ms + a_ms) / t, 4)
    return out


def capture(torch, fn, reps=1):
    """Record `reps` calls of fn into a HIP graph on a side stream (default priority)."""
    g = torch.cuda.CUDAGraph()
    s = torch.cuda.Stream()
    s.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(s):
        fn()                                                 # one eager call on the capture stream first
    torch.cuda.synchronize()
    with torch.cuda.graph(g, stream=s):
        for _ in range(reps):
            fn()
    return g


def time_graph(torch, g, launches, per_launch):
    """Average milliseconds per recorded call: events around `launches` replays on the current stream."""
    g.replay()
    torch.cuda.synchronize()
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    for _ in range(launches):
        g.replay()
    b.record()
    b.synchronize()
    return a.elapsed_time(b) / (launches * per_launch)


def cpu_baseline(cfg, wl, W):
    """The oracle, as it stands, on the whole share (about 15 s of fp64 numpy), on this machine's host cores."""
    from oracle import moe_layer as O
    frac = 1
    Ts = max(1, cfg.T // frac)
    Rs = max(1, wl["R"] // frac)
    inp = wl["inp"]
    x = inp["x"][:Ts]
    experts = [W.make_expert_weights(cfg, e) for e in range(cfg.E) if inp["expert_to_gpu"][e] == wl["g"]][:1]
    rows = W.generate.make_rows(cfg, W.generate.S_RECV, Rs)
    t0 = time.perf_counter()
    idx, w, _ = O.route(x, inp["w_gate"], inp["gate_bias"], cfg.k, cfg.renorm)
    O.traffic(idx, inp["expert_to_gpu"], cfg.G, cfg.capacity)
    d = O.dispatch(x, idx, inp["expert_to_gpu"], list(range(cfg.G)), cfg.capacity)
    out = O.expert_ffn(rows, [0, Rs], [0], experts, cfg.act)
    ret = np.resize(out, (d["n_rows"], cfg.H))
    O.combine(ret, d["slot_to_row"], w)
    dt = time.perf_counter() - t0
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        cores = os.cpu_count() or 1
    return {"value": Ts / dt, "unit": "tokens/s", "cores": int(cores), "kind": "oracle",
            "sample": "1/%d of the share: %d local tokens routed/dispatched/combined and %d received rows through "
                      "the expert FFN (inputs generated outside the timed region), fp64 numpy, one run of %.1f s"
                      % (frac, Ts, Rs, dt)}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="c2_mixtral")
    ap.add_argument("--share", choices=["bottleneck", "median"], default="bottleneck",
                    help="which GPU's share to run: the one that receives most rows (sets the layer time) or the median one")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-graph", action="store_true", help="launch every kernel from Python instead of replaying a HIP graph")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU's share of the layer; there is no multi-GPU path in this library "
              "(run with --gpus 1)", file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_2410_17043_amd as P
    import workloads as W
    import workloads.generate  # noqa: F401

    if not torch.cuda.is_available():
        print("bench.py needs the MI355X (no CPU fallback exists)", file=sys.stderr)
        sys.exit(2)
    cfg = W.get_config(args.workload)
    wl = build_workload(cfg, torch, P, W, args.share)
    step = wl["step"]

    # The step is recorded once into a HIP graph (no memset nodes: the library clears nothing with
    # hipMemsetAsync) and replayed; replays are checked against the eager result before timing.
    step()
    torch.cuda.synchronize()
    y_eager = wl["y"].clone()
    use_graph = not args.no_graph
    if use_graph:
        g_step = capture(torch, step)
        for _ in range(3):
            wl["y"].zero_()
            g_step.replay()
            torch.cuda.synchronize()
            if not torch.equal(wl["y"], y_eager):
                print("graph replay differs from the eager step", file=sys.stderr)
                sys.exit(3)
        run_step = g_step.replay
    else:
        run_step = step
    for _ in range(args.warmup):
        run_step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    for _ in range(args.steps):
        run_step()
    b.record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3 / args.steps
    ms_per_step = a.elapsed_time(b) / args.steps

    reps = max(3, args.steps // 2)
    stage_ms = {}
    for name, fn in wl["stages"].items():                   # GPU time of each stage: 10 calls per graph replay
        per = 10 if name != "expert_ffn" else 1
        stage_ms[name] = time_graph(torch, capture(torch, fn, per), reps, per)
    stage_ms["dispatch"] = stage_ms.pop("traffic+dispatch") - stage_ms["traffic"]
    stage_ms["dispatch_chunks (not in the step)"] = stage_ms.pop("traffic+dispatch_chunks") - stage_ms["traffic"]
    gemm_ms = np.mean([wl["ffn_timed"]() for _ in range(reps)], axis=0)   # tile map, GEMM1 (+act), GEMM2

    R, T, k, H, F, b_el = wl["R"], cfg.T, cfg.k, cfg.H, cfg.F, (2 if cfg.dtype == "bf16" else 4)
    n_up = 2 if cfg.act == 2 else 1
    flops_gemm1 = 2.0 * n_up * R * H * F
    flops_gemm2 = 2.0 * R * H * F
    achieved = flops_gemm1 / (gemm_ms[1] * 1e-3) / 1e12
    bytes_dispatch = T * H * b_el + wl["n_kept"] * H * b_el + T * k * 12
    bytes_combine = wl["n_kept"] * H * b_el + T * H * b_el + T * k * 8
    bytes_route = T * H * b_el + cfg.E * H * b_el + T * k * 8
    line = {
        "metric": "MoE-layer tokens/sec on 1 MI355X", "value": T / (ms_per_step * 1e-3), "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": cfg.dtype, "data": "synthetic",
        "config": {"workload": cfg.name, "T": T, "H": H, "F": F, "E": cfg.E, "k": k, "G": cfg.G,
                   "received_rows": R, "gpu_under_test": wl["g"], "share": args.share, "act": cfg.act},
        "wall_ms_per_step": wall_ms, "launch": "hip graph replay" if use_graph else "eager",
        "stage_ms": {n: round(v, 4) for n, v in stage_ms.items()},
        "stage_rate": {
            "route_GBps": bytes_route / (stage_ms["route"] * 1e-3) / 1e9,
            "dispatch_GBps": bytes_dispatch / (stage_ms["dispatch"] * 1e-3) / 1e9,
            "combine_GBps": bytes_combine / (stage_ms["combine"] * 1e-3) / 1e9,
            "ffn_TFLOPs": (flops_gemm1 + flops_gemm2) / (stage_ms["expert_ffn"] * 1e-3) / 1e12,
            "ffn_mfma_util": (flops_gemm1 + flops_gemm2) / (stage_ms["expert_ffn"] * 1e-3) / 1e12 / PEAK_BF16_TFLOPS,
            "gemm2_TFLOPs": flops_gemm2 / (gemm_ms[2] * 1e-3) / 1e12,
            "tilemap_ms": float(gemm_ms[0]),
        },
        "roofline": {"kernel": "gemm_bf16_kernel<SwiGLU> (first FFN GEMM with the activation)", "bound": "mfma",
                     "achieved": achieved, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                     "frac": achieved / PEAK_BF16_TFLOPS, "traffic": GEMM1_TRAFFIC_BYTES.get(cfg.name) if args.share == "bottleneck" else None,
                     "launch_ms": float(gemm_ms[1]), "flops_per_launch": flops_gemm1},
    }
    line["paper_model"] = paper_model(cfg, wl, stage_ms, P)
    line["box_reference"] = box_reference(torch, wl, cfg)
    if not args.no_cpu_baseline:
        line["cpu_baseline"] = cpu_baseline(cfg, wl, W)
    print(json.dumps(line))


if __name__ == "__main__":
    main()
