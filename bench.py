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
# WRITE_SIZE x 1.0, see profiles/bench_c2_mixtral_layer_share.md), valid for the kernel source whose SHA-256
# starts with the digest below; reported as null as soon as ffn.hip differs from what the counters saw.
GEMM1_TRAFFIC = {"c2_mixtral": {"bytes": 3.9033e6 * 1024 * 2.0 + 6.6752e5 * 1024, "ffn_hip_sha256": "05411752ca640057"}}


def gemm1_traffic_bytes(name):
    rec = GEMM1_TRAFFIC.get(name)
    if rec is None:
        return None
    import hashlib
    with open(os.path.join(ROOT, "paper_2410_17043_amd", "csrc", "ffn.hip"), "rb") as f:
        digest = hashlib.sha256(f.read()).hexdigest()
    return rec["bytes"] if digest.startswith(rec["ffn_hip_sha256"]) else None


def build_workload(cfg, torch, P, W, share="bottleneck", placement=None):
    """Everything a step needs, resident on the GPU.  Returns a dict of tensors and the step closure.

    placement = None: experts in contiguous blocks (expert e on GPU e // E_loc), the GPU under test chosen by
    `share`.  placement = (g, unit_of_gpu): GPU p of the cluster holds the tokens and the expert block that
    the workload generator calls GPU unit_of_gpu[p] (the result of a colocation), and GPU g is under test."""
    dev = "cuda:0"
    tdt = P.TORCH_DTYPE[cfg.dtype]

    def to_dev(a):
        return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(dev).to(tdt).contiguous()

    traffic = W.make_traffic_matrix(cfg)
    if placement is not None:
        g, unit_of_gpu = int(placement[0]), [int(u) for u in placement[1]]
        assert sorted(unit_of_gpu) == list(range(cfg.G))
        traffic = {"D": traffic["D"][np.ix_(unit_of_gpu, unit_of_gpu)], "per_expert": traffic["per_expert"][unit_of_gpu]}
    else:
        unit_of_gpu = list(range(cfg.G))
    D = traffic["D"].copy()
    received = D.sum(axis=0)
    if placement is not None:
        pass
    elif share == "median":
        g = int(np.argsort(received, kind="stable")[len(received) // 2])
    else:
        g = int(np.argmax(received))                        # the GPU that receives most sets the layer time
    inp = W.make_layer_inputs(cfg, unit_of_gpu[g])
    gpu_of_unit = np.argsort(np.asarray(unit_of_gpu))
    inp["expert_to_gpu"] = gpu_of_unit[inp["expert_to_gpu"]].astype(np.int32)
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
    # shared experts (applied to every local token, weight 1): their outputs add up, which equals ONE expert
    # whose inner dimension is the concatenation of theirs, so the weights are stacked once here and one
    # grouped-FFN call over the local tokens feeds moe_combine's shared_out
    shared_out, b_shared, shared_keep = None, None, None
    if cfg.n_shared:
        sw = [W.make_expert_weights(cfg, s_, shared=True) for s_ in range(cfg.n_shared)]
        cat = {"w1": to_dev(np.concatenate([v["w1"] for v in sw])),
               "w_up": to_dev(np.concatenate([v["w_up"] for v in sw])) if sw[0]["w_up"] is not None else None,
               "w_down": to_dev(np.concatenate([v["w_down"] for v in sw], axis=1))}
        Fs = F * cfg.n_shared
        sh_table = P.expert_table([cat])
        sh_off, sh_exp = torch.tensor([0, T], **i32), torch.tensor([0], **i32)
        sh_ws = torch.empty(P.moe_ffn_workspace_bytes(T, H, Fs, cfg.act, cfg.dtype), dtype=torch.uint8, device=dev)
        shared_out = torch.empty((T, H), dtype=tdt, device=dev)
        b_shared = P.bind_expert_ffn(x, T, sh_off, sh_exp, 1, sh_table, H, Fs, cfg.act, cfg.dtype, shared_out, sh_ws)
        shared_keep = (cat, sh_table, sh_off, sh_exp, sh_ws)
    b_combine = P.bind_combine(ctx, ret, s2r, w, shared_out, y)

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

    def front():                                             # Gate, traffic row, send buffer, loop-back of the first all-to-all
        st = cur()
        b_route(st)
        b_traffic(st)
        b_dispatch(st)
        for (r0, lo, hi) in self_spans:
            recv[r0:r0 + hi - lo].copy_(send_buf[lo:hi], non_blocking=True)

    def ffn():                                               # routed experts over the received rows, shared experts over the local tokens
        st = cur()
        b_ffn(st)
        if b_shared is not None:
            b_shared(st)

    def back():                                              # loop-back of the second all-to-all, Aggregation
        for (r0, lo, hi) in self_spans:
            ret[lo:hi].copy_(ffn_out[r0:r0 + hi - lo], non_blocking=True)
        b_combine(cur())

    def step():
        front()
        ffn()
        back()

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
    if b_shared is not None:
        stages["shared_ffn"] = lambda: b_shared(cur())
    ffn_timed = lambda: P.moe_expert_ffn_timed(recv, R, ffn_off, ffn_exp, len(exp), table, H, F, cfg.act, cfg.dtype,
                                               ffn_out, ws)
    n_kept = int(so[-1])
    return dict(step=step, front=front, ffn=ffn, back=back, stages=stages, ffn_timed=ffn_timed, R=R, g=g, n_kept=n_kept, inp=inp, y=y,
                shared_out=shared_out, x=x, unit_of_gpu=unit_of_gpu, shared_keep=shared_keep,
                idx=idx, w=w, expert_count=expert_count, dest_count=dest_count, n_dropped=n_dropped,
                send_buf=send_buf, slot_to_row=s2r, row_to_slot=r2s, seg_offset=seg_offset, seg_expert=seg_expert,
                recv=recv, ffn_out=ffn_out, ret=ret, ffn_off=off, ffn_exp=exp, ffn_off_dev=ffn_off, ffn_exp_dev=ffn_exp, local=local, dest_order=dest_order,
                self_spans=self_spans, n_chunks=len(chunks), D=D, rates=rates, plan=plan, keep=(ctx, x, wg, bias, experts, table, ws, chunk_plan))


def box_reference(torch, wl, cfg, P):
    """What this very box sustains, for orientation beside the published peaks.  None of it is on the product
    path.  copy_GBps: a plain device copy (256 MiB read + 256 MiB written, torch).  copy_1r2w_GBps: the
    library's reference kernel that reads the token block of this workload once and writes it twice with
    streaming 16-byte accesses (the send buffer's traffic without indexing).  mfma_only_TFLOPs: the
    library's register-only loop of independent v_mfma_f32_32x32x16_bf16 on one wave per SIMD of every compute
    unit, about 5 ms long (no LDS, no memory traffic: the ceiling of the matrix cores at the clock this box
    grants them).  vendor_gemm_bf16_TFLOPs: hipBLASLt's GEMM of one projection of the first FFN GEMM."""
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
    x = wl["x"]
    d0, d1 = torch.empty_like(x), torch.empty_like(x)
    P.moe_diag_copy_1r2w(x, d0, d1)
    ms = [P.moe_diag_copy_1r2w(x, d0, d1, 10) for _ in range(5)]         # 10 launches back to back, like the stage timings
    nbytes = 3 * x.numel() * x.element_size()
    out["copy_1r2w_GBps"] = round(nbytes / (float(np.mean(ms)) * 1e-3) / 1e9, 1)
    out["copy_1r2w_us"] = round(float(np.mean(ms)) * 1e3, 2)
    out["copy_1r2w_bytes"] = nbytes
    del d0, d1
    n_cu = torch.cuda.get_device_properties(dev).multi_processor_count
    sink = torch.empty(n_cu * 256, dtype=torch.float32, device=dev)
    P.moe_diag_mfma_only(n_cu, 1024, sink)
    runs = [P.moe_diag_mfma_only(n_cu, 16384, sink) for _ in range(5)]
    out["mfma_only_TFLOPs"] = round(float(np.mean([f / (m * 1e-3) / 1e12 for m, f in runs])), 1)
    out["mfma_only_ms"] = round(float(np.mean([m for m, _ in runs])), 3)
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


def blas_threads():
    """Threads the host BLAS behind numpy uses (the oracle's matmuls run there)."""
    try:
        from threadpoolctl import threadpool_info
        n = [p_.get("num_threads", 1) for p_ in threadpool_info()]
        if n:
            return int(max(n))
    except Exception:
        pass
    return int(os.cpu_count() or 1)


CPU_MAX_ROWS = 65536          # the oracle's FFN leg is bounded to this many received rows (10-30 s of host work)


def cpu_baseline(cfg, wl, W):
    """The oracle, as it stands, on the share (about 15 s of fp64 numpy at the Mixtral shape), on this machine's
    host cores: the whole share when it has at most CPU_MAX_ROWS received rows, else the first 1/frac of its
    local tokens and of its received rows.  Returns (seconds, tokens, rows, frac)."""
    from oracle import moe_layer as O
    frac = max(1, -(-wl["R"] // CPU_MAX_ROWS))
    Ts, Rs = max(1, cfg.T // frac), max(1, wl["R"] // frac)
    inp = wl["inp"]
    x = inp["x"][:Ts]
    experts = [W.make_expert_weights(cfg, e) for e in wl["local"]]
    shared = [W.make_expert_weights(cfg, s_, shared=True) for s_ in range(cfg.n_shared)]
    rows = W.generate.make_rows(cfg, W.generate.S_RECV, Rs)
    off = [min(o, Rs) for o in wl["ffn_off"]]
    exp = wl["ffn_exp"]
    t0 = time.perf_counter()
    idx, w, _ = O.route(x, inp["w_gate"], inp["gate_bias"], cfg.k, cfg.renorm)
    O.traffic(idx, inp["expert_to_gpu"], cfg.G, cfg.capacity)
    d = O.dispatch(x, idx, inp["expert_to_gpu"], list(wl["dest_order"]), cfg.capacity)
    out = O.expert_ffn(rows, off, exp, experts, cfg.act)
    sh = None
    for sw in shared:
        o = O.ffn(x, sw["w1"], sw["w_up"], sw["w_down"], cfg.act)
        sh = o if sh is None else sh + o
    ret = np.resize(out, (d["n_rows"], cfg.H))
    O.combine(ret, d["slot_to_row"], w, sh)
    return time.perf_counter() - t0, Ts, Rs, frac


def cpu_baseline_line(cfgs_wls, W):
    parts = [cpu_baseline(cfg, wl, W) for cfg, wl in cfgs_wls]
    dt, toks = sum(p_[0] for p_ in parts), sum(p_[1] for p_ in parts)
    out = {"value": toks / dt, "unit": "tokens/s", "cores": blas_threads(), "kind": "oracle",
           "sample": "1/%d of the share, one run of %.1f s: %s; fp64 numpy (matmuls in the host BLAS on `cores` threads, "
                     "the per-token loops of route/dispatch/combine on one); the received rows are regenerated from "
                     "the same seeds outside the timed region instead of being read back from the GPU, and the "
                     "returned rows are the FFN output recycled to the send-buffer row count"
                     % (parts[0][3], dt, " + ".join("%d local tokens routed/dispatched/combined in the step's transmission order, "
                                       "%d received rows through the expert FFN" % (p_[1], p_[2]) for p_ in parts))}
    # the tiny fp32 configuration on one thread (whole layer over its 4 simulated GPUs, per-token definition)
    try:
        from threadpoolctl import threadpool_limits
        from oracle import moe_layer as O
        c1 = W.get_config("c1_tiny_fp32")
        inputs = [W.make_layer_inputs(c1, g_) for g_ in range(c1.G)]
        experts = [W.make_expert_weights(c1, e) for e in range(c1.E)]
        with threadpool_limits(limits=1):
            t0 = time.perf_counter()
            for g_ in range(c1.G):
                O.layer_dense(inputs[g_]["x"], inputs[0]["w_gate"], inputs[0]["gate_bias"], c1.k, c1.renorm, experts, c1.act,
                              c1.capacity)
            out["c1_tiny_fp32_single_thread_tokens_per_s"] = c1.G * c1.T / (time.perf_counter() - t0)
    except Exception as e:                                   # informative only
        out["c1_tiny_fp32_single_thread_tokens_per_s"] = None
        out["c1_note"] = repr(e)
    return out


def measure_step(torch, step, outputs, args):
    """Times `step` (HIP-graph replay unless --no-graph; replays are first checked against the eager result on
    `outputs`).  Returns (GPU ms per step from events, wall ms per step, launch mode)."""
    step()
    torch.cuda.synchronize()
    eager = [o.clone() for o in outputs]
    use_graph = not args.no_graph
    if use_graph:
        g_step = capture(torch, step)
        for _ in range(3):                                   # no memset nodes are recorded by the library; check anyway
            for o in outputs:
                o.zero_()
            g_step.replay()
            torch.cuda.synchronize()
            if not all(torch.equal(o, e) for o, e in zip(outputs, eager)):
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
    return a.elapsed_time(b) / args.steps, wall_ms, "hip graph replay" if use_graph else "eager"


def measure_stages(torch, wl, cfg, reps):
    """GPU time of every stage (10 calls per graph replay; the FFN once), the FFN's kernels by HIP events, and
    the rates against the algorithmic work."""
    stage_ms = {}
    for name, fn in wl["stages"].items():
        per = 10 if name not in ("expert_ffn", "shared_ffn") else 1
        stage_ms[name] = time_graph(torch, capture(torch, fn, per), reps, per)
    stage_ms["dispatch"] = stage_ms.pop("traffic+dispatch") - stage_ms["traffic"]
    stage_ms["dispatch_chunks (not in the step)"] = stage_ms.pop("traffic+dispatch_chunks") - stage_ms["traffic"]
    gemm_ms = np.mean([wl["ffn_timed"]() for _ in range(reps)], axis=0)   # tile map, GEMM1 (+act), GEMM2
    R, T, k, H, F, b_el = wl["R"], cfg.T, cfg.k, cfg.H, cfg.F, (2 if cfg.dtype == "bf16" else 4)
    n_up = 2 if cfg.act == 2 else 1
    flops_gemm1 = 2.0 * n_up * R * H * F
    flops_gemm2 = 2.0 * R * H * F
    bytes_dispatch = T * H * b_el + wl["n_kept"] * H * b_el + T * k * 12
    bytes_combine = wl["n_kept"] * H * b_el + T * H * b_el + T * k * 8 + (T * H * b_el if cfg.n_shared else 0)
    bytes_route = T * H * b_el + cfg.E * H * b_el + T * k * 8
    rate = {
        "route_GBps": bytes_route / (stage_ms["route"] * 1e-3) / 1e9,
        "dispatch_GBps": bytes_dispatch / (stage_ms["dispatch"] * 1e-3) / 1e9,
        "combine_GBps": bytes_combine / (stage_ms["combine"] * 1e-3) / 1e9,
        "ffn_TFLOPs": (flops_gemm1 + flops_gemm2) / (stage_ms["expert_ffn"] * 1e-3) / 1e12,
        "ffn_mfma_util": (flops_gemm1 + flops_gemm2) / (stage_ms["expert_ffn"] * 1e-3) / 1e12 / PEAK_BF16_TFLOPS,
        "gemm2_TFLOPs": flops_gemm2 / (gemm_ms[2] * 1e-3) / 1e12,
        "tilemap_ms": float(gemm_ms[0]),
    }
    if cfg.n_shared:
        rate["shared_ffn_TFLOPs"] = 2.0 * (n_up + 1) * T * H * F * cfg.n_shared / (stage_ms["shared_ffn"] * 1e-3) / 1e12
    if cfg.dtype == "bf16":
        rate["decode_share"] = decode_share(torch, wl, cfg, reps)
        rate["route_phases_us"] = route_phases(torch, wl, cfg)
        if wl["R"] > 64:
            rate["ffn_tile_phases_us"] = {"gemm1": ffn_tile_phases(torch, wl, cfg, 1), "gemm2": ffn_tile_phases(torch, wl, cfg, 2)}
    achieved = flops_gemm1 / (gemm_ms[1] * 1e-3) / 1e12
    roof = {"kernel": "gemm_bf16_kernel<%s> (first FFN GEMM with the activation)" % {0: "SiLU", 1: "GELU", 2: "SwiGLU"}[cfg.act],
            "bound": "mfma", "achieved": achieved, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
            "frac": achieved / PEAK_BF16_TFLOPS, "traffic": None, "launch_ms": float(gemm_ms[1]),
            "flops_per_launch": flops_gemm1}
    return stage_ms, rate, roof


def route_phases(torch, wl, cfg, calls=20):
    """Where the gate kernel's time goes, from the library's timed instantiation of it (moe_diag_route_phases;
    not the kernel the step runs): microseconds from the first block's start to each phase boundary, median
    over the waves of all blocks of the last of `calls` back-to-back calls, and the latest end."""
    import paper_2410_17043_amd as P
    ctx, x, wg, bias = wl["keep"][0], wl["keep"][1], wl["keep"][2], wl["keep"][3]
    marks = torch.zeros((cfg.T // 16 + 1) * 128, dtype=torch.int64, device=x.device)
    idx, w = torch.empty_like(wl["idx"]), torch.empty_like(wl["w"])
    tpb = 0
    for _ in range(calls):
        marks.zero_()
        tpb = P.moe_diag_route_phases(ctx, x, wg, bias, idx, w, marks)
    torch.cuda.synchronize()
    if tpb == 0:
        return None
    nb = (cfg.T + tpb - 1) // tpb
    a = marks[:nb * 128].cpu().numpy().reshape(nb, 16, 8)
    used = a[:, :, 0] > 0                                     # waves that exist
    t0 = a[:, :, 0][used].min()
    rel = (a[:, :, :6] - t0) * 0.01                           # the wall clock ticks at 100 MHz
    rel[:, :, 5] = np.where(a[:, :, 5] == 0, rel[:, :, 4], rel[:, :, 5])
    names = ["start", "own_loop_done", "all_waves_done", "tiles_added", "selected", "end"]
    out = {n: round(float(np.median(rel[:, :, i][used])), 2) for i, n in enumerate(names)}
    out["end_max"] = round(float(rel[:, :, 5][used].max()), 2)
    out["tokens_evaluated_again"] = int(a[:, 0, 6].sum())
    out["tokens_per_block"] = tpb
    return out


def ffn_tile_phases(torch, wl, cfg, which, calls=3):
    """Where the time of a tile of an FFN GEMM goes, from the library's timed instantiation of the GEMM kernel
    (moe_diag_ffn_phases; not the kernel the step runs): median microseconds per whole tile spent before the loop
    (first operands on their way), in the loop and after it (activation and stores)."""
    import paper_2410_17043_amd as P
    recv, R, table, ws, out = wl["recv"], wl["R"], wl["keep"][5], wl["keep"][6], wl["ffn_out"]
    off, exp = wl["ffn_off_dev"], wl["ffn_exp_dev"]
    marks = torch.zeros(P.ffn_phase_marks_len(R, len(wl["ffn_exp"]), cfg.H, cfg.F, cfg.act, which), dtype=torch.int64, device=recv.device)
    for _ in range(calls):
        marks.zero_()
        P.moe_diag_ffn_phases(recv, R, off, exp, len(wl["ffn_exp"]), table, cfg.H, cfg.F, cfg.act, cfg.dtype, out, ws, which, marks)
    torch.cuda.synchronize()
    a = marks.cpu().numpy().reshape(-1, 4, 4)[:, 0, :]          # wave 0 of every block
    a = a[(a[:, 0] > 0) & (a[:, 3] > 0)]
    nk_whole = (a[:, 2] - a[:, 1])
    whole = a[nk_whole >= 0.9 * np.median(nk_whole)]              # the pieces of tail tiles have shorter loops
    d = np.diff(whole, axis=1) * 0.01                             # the wall clock ticks at 100 MHz
    return {"before_loop": round(float(np.median(d[:, 0])), 2), "loop": round(float(np.median(d[:, 1])), 2),
            "after_loop": round(float(np.median(d[:, 2])), 2), "tiles": int(len(whole))}


def decode_share(torch, wl, cfg, reps, rows=32):
    """The expert FFN over a decode-sized share, for information beside the stages (not part of the step): the
    first `rows` received rows as one segment of the first local expert.  Every weight of that expert is used
    once, so the figure of merit is the rate at which the weights stream."""
    import paper_2410_17043_amd as P
    dev = wl["recv"].device
    i32 = dict(dtype=torch.int32, device=dev)
    rows = min(rows, wl["R"])
    off, exp = torch.tensor([0, rows], **i32), torch.tensor([0], **i32)
    out = torch.empty((rows, cfg.H), dtype=wl["recv"].dtype, device=dev)
    ws = torch.empty(P.moe_ffn_workspace_bytes(rows, cfg.H, cfg.F, cfg.act, cfg.dtype), dtype=torch.uint8, device=dev)
    table = wl["keep"][5]
    b = P.bind_expert_ffn(wl["recv"], rows, off, exp, 1, table, cfg.H, cfg.F, cfg.act, cfg.dtype, out, ws)
    ms = time_graph(torch, capture(torch, lambda: b(torch.cuda.current_stream().cuda_stream), 10), reps, 10)
    w_bytes = (3 if cfg.act == 2 else 2) * cfg.H * cfg.F * 2
    return {"rows": rows, "ffn_us": round(ms * 1e3, 1), "weights_GBps": round(w_bytes / (ms * 1e-3) / 1e9, 1)}


def config_of(cfg, wl, share):
    return {"workload": cfg.name, "T": cfg.T, "H": cfg.H, "F": cfg.F, "E": cfg.E, "k": cfg.k, "G": cfg.G,
            "received_rows": wl["R"], "gpu_under_test": wl["g"], "share": share, "act": cfg.act,
            "shared_experts": cfg.n_shared}


def run_single(args, torch, P, W):
    cfg = W.get_config(args.workload)
    wl = build_workload(cfg, torch, P, W, args.share)
    ms_per_step, wall_ms, launch = measure_step(torch, wl["step"], [wl["y"]], args)
    stage_ms, rate, roof = measure_stages(torch, wl, cfg, max(3, args.steps // 2))
    if args.share == "bottleneck":
        roof["traffic"] = gemm1_traffic_bytes(cfg.name)
    line = {
        "metric": "MoE-layer tokens/sec on 1 MI355X", "value": cfg.T / (ms_per_step * 1e-3), "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": cfg.dtype, "data": "synthetic",
        "config": config_of(cfg, wl, args.share),
        "wall_ms_per_step": wall_ms, "launch": launch,
        "stage_ms": {n: round(v, 4) for n, v in stage_ms.items()}, "stage_rate": rate, "roofline": roof,
    }
    line["paper_model"] = paper_model(cfg, wl, stage_ms, P)
    line["box_reference"] = box_reference(torch, wl, cfg, P)
    if not args.no_cpu_baseline:
        line["cpu_baseline"] = cpu_baseline_line([(cfg, wl)], W)
    return line


def build_coloc(torch, P, W):
    """The colocated GPU of Sec. 6: model a (8 experts, one per GPU) and model b (16 experts, two per GPU) on
    the same 8 GPUs.  colocate_match pairs a's expert p with the block of b's experts that lives on one GPU
    (Sec. 6.2 Case II on the two 8 x 8 traffic matrices), so GPU p hosts a's expert p and b's block pair[p];
    the GPU under test is the one that receives most rows of both models together."""
    ca, cb = W.get_config("c4a_coloc"), W.get_config("c4b_coloc")
    Da, Db = W.make_traffic_matrix(ca)["D"], W.make_traffic_matrix(cb)["D"]
    pair, bott = P.colocate_match(Da, Db)
    pair = [int(v) for v in pair]
    Dn = Da + Db[np.ix_(pair, pair)]
    g = int(np.argmax(Dn.sum(axis=0)))
    wa = build_workload(ca, torch, P, W, placement=(g, list(range(ca.G))))
    wb = build_workload(cb, torch, P, W, placement=(g, pair))
    side = torch.cuda.Stream()                               # default priority

    def ffn_two_streams():
        main_s = torch.cuda.current_stream()
        side.wait_stream(main_s)
        wa["ffn"]()
        with torch.cuda.stream(side):
            wb["ffn"]()
        main_s.wait_stream(side)

    def ffn_serial():
        wa["ffn"]()
        wb["ffn"]()

    def step_with(ffn):
        def step():
            wa["front"]()
            wb["front"]()
            ffn()
            wa["back"]()
            wb["back"]()
        return step

    return dict(ca=ca, cb=cb, wa=wa, wb=wb, pair=pair, bottleneck=float(bott), g=g, Dn=Dn,
                ffn_two_streams=ffn_two_streams, ffn_serial=ffn_serial, step=step_with(ffn_two_streams),
                step_serial=step_with(ffn_serial), keep=side)


def run_coloc(args, torch, P, W):
    co = build_coloc(torch, P, W)
    ca, cb, wa, wb = co["ca"], co["cb"], co["wa"], co["wb"]
    ms_per_step, wall_ms, launch = measure_step(torch, co["step"], [wa["y"], wb["y"]], args)
    reps = max(3, args.steps // 2)
    ms_serial = time_graph(torch, capture(torch, co["step_serial"]), reps, 1)
    ffn_two = time_graph(torch, capture(torch, co["ffn_two_streams"]), reps, 1)
    ffn_ser = time_graph(torch, capture(torch, co["ffn_serial"]), reps, 1)
    sa, ra, roof = measure_stages(torch, wa, ca, reps)
    sb, rb, _ = measure_stages(torch, wb, cb, reps)
    line = {
        "metric": "MoE-layer tokens/sec on 1 MI355X", "value": (ca.T + cb.T) / (ms_per_step * 1e-3), "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": ca.dtype, "data": "synthetic",
        "config": {"workload": "c4_coloc", "model_a": config_of(ca, wa, "colocated"), "model_b": config_of(cb, wb, "colocated"),
                   "pair": co["pair"], "bottleneck_weight": co["bottleneck"], "gpu_under_test": co["g"],
                   "step": "both models' gate/traffic/dispatch, the two expert FFNs on two HIP streams, both combines"},
        "wall_ms_per_step": wall_ms, "launch": launch,
        "coloc": {"step_two_streams_ms": ms_per_step, "step_one_stream_ms": ms_serial,
                  "ffn_two_streams_ms": ffn_two, "ffn_one_stream_ms": ffn_ser},
        "stage_ms": {"model_a": {n: round(v, 4) for n, v in sa.items()}, "model_b": {n: round(v, 4) for n, v in sb.items()}},
        "stage_rate": {"model_a": ra, "model_b": rb}, "roofline": roof,
    }
    line["box_reference"] = box_reference(torch, wa, ca, P)
    if not args.no_cpu_baseline:
        line["cpu_baseline"] = cpu_baseline_line([(ca, wa), (cb, wb)], W)
    return line


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="c2_mixtral",
                    help="c2_mixtral (default), c1_tiny_fp32, c3_switch, c4a_coloc, c4b_coloc, c5_finegrained, or "
                         "c4_coloc: both colocated models on the GPU that colocate_match gives them")
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
    line = run_coloc(args, torch, P, W) if args.workload == "c4_coloc" else run_single(args, torch, P, W)
    print(json.dumps(line))


if __name__ == "__main__":
    main()
