"""Thin Python binding of the C ABI: argument marshalling only.

Device entry points take torch tensors that already live on the GPU (torch is used
for device memory and streams, nothing else) and enqueue work on torch's current
stream.  Every step of the path runs in the library's own kernels.
"""
from __future__ import annotations

import ctypes as C

import numpy as np
import torch

from . import _lib
from ._lib import moe_shape, moe_expert_w, aurora_schedule

F32, BF16 = 0, 1
ACT_SILU_MLP, ACT_GELU_MLP, ACT_SWIGLU = 0, 1, 2
_DT = {torch.float32: F32, torch.bfloat16: BF16, "fp32": F32, "bf16": BF16}
TORCH_DTYPE = {F32: torch.float32, BF16: torch.bfloat16, "fp32": torch.float32, "bf16": torch.bfloat16}


class MoeError(RuntimeError):
    def __init__(self, fn, status):
        lib = _lib.load()
        self.status = status
        self.name = lib.moe_status_str(status).decode()
        super().__init__("%s failed: %s (%s)" % (fn, self.name, lib.moe_last_error().decode()))


def _check(fn, rc):
    if rc != 0:
        raise MoeError(fn, rc)


def _ptr(t):
    if t is None:
        return None
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError("device entry points need contiguous GPU tensors")
    return C.c_void_p(t.data_ptr())


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _i32_array(values):
    a = np.ascontiguousarray(values, dtype=np.int32)
    return a, a.ctypes.data_as(C.POINTER(C.c_int32))


class MoeCtx:
    """Owner of a moe_ctx (small scan scratch on the current device)."""

    def __init__(self, T, H, E, k, G, dtype, renorm=0, capacity=0):
        self.lib = _lib.load()
        self.shape = moe_shape(T, H, E, k, G, _DT[dtype], renorm, capacity)
        self.handle = C.c_void_p()
        _check("moe_ctx_create", self.lib.moe_ctx_create(C.byref(self.handle), C.byref(self.shape)))

    def set_rank_reuse(self, enable=True):
        """Let a dispatch that directly follows a moe_traffic on the same index array reuse its slot ranks."""
        _check("moe_ctx_set_rank_reuse", self.lib.moe_ctx_set_rank_reuse(self.handle, 1 if enable else 0))

    def invalidate(self):
        """Forget cached slot ranks (needed only with rank reuse on, after rewriting topk_idx in place)."""
        _check("moe_ctx_invalidate", self.lib.moe_ctx_invalidate(self.handle))

    def close(self):
        if self.handle:
            self.lib.moe_ctx_destroy(self.handle)
            self.handle = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class Bound:
    """A C call with its arguments marshalled once; calling it only enqueues the work.

    Keeps the Python objects that own the argument memory alive.  The stream is the one
    that was current when the call was bound, unless `stream` is given at call time.
    """

    __slots__ = ("fn", "name", "args", "keep", "stream_pos")

    def __init__(self, fn, name, args, keep, stream_pos):
        self.fn, self.name, self.args, self.keep, self.stream_pos = fn, name, list(args), keep, stream_pos

    def __call__(self, stream=None):
        if stream is not None:
            self.args[self.stream_pos] = C.c_void_p(stream)
        rc = self.fn(*self.args)
        if rc != 0:
            raise MoeError(self.name, rc)


def bind_route(ctx, x, w_gate, gate_bias, topk_idx, topk_w):
    return Bound(ctx.lib.moe_route, "moe_route", (ctx.handle, _ptr(x), _ptr(w_gate), _ptr(gate_bias), _ptr(topk_idx),
                                                  _ptr(topk_w), _stream()), (ctx, x, w_gate, gate_bias, topk_idx, topk_w), 6)


def bind_traffic(ctx, topk_idx, expert_to_gpu, expert_count, dest_count, n_dropped):
    a, e2g = _i32_array(expert_to_gpu)
    return Bound(ctx.lib.moe_traffic, "moe_traffic", (ctx.handle, _ptr(topk_idx), e2g, _ptr(expert_count),
                                                      _ptr(dest_count), _ptr(n_dropped), _stream()),
                 (ctx, topk_idx, a, expert_count, dest_count, n_dropped), 6)


def bind_dispatch(ctx, x, topk_idx, expert_to_gpu, dest_order, send_buf, slot_to_row, row_to_slot, seg_offset,
                  seg_expert):
    a, e2g = _i32_array(expert_to_gpu)
    b, order = _i32_array(dest_order)
    return Bound(ctx.lib.moe_dispatch, "moe_dispatch",
                 (ctx.handle, _ptr(x), _ptr(topk_idx), e2g, order, _ptr(send_buf), _ptr(slot_to_row), _ptr(row_to_slot),
                  _ptr(seg_offset), _ptr(seg_expert), _stream()),
                 (ctx, x, topk_idx, a, b, send_buf, slot_to_row, row_to_slot, seg_offset, seg_expert), 10)


def bind_expert_ffn(recv, R, seg_offset, seg_expert, nseg, experts, H, F, act, dtype, out, workspace):
    tab = experts if isinstance(experts, C.Array) else expert_table(experts)
    return Bound(_lib.load().moe_expert_ffn, "moe_expert_ffn",
                 (_ptr(recv), R, _ptr(seg_offset), _ptr(seg_expert), nseg, tab, len(tab), H, F, act, _DT[dtype],
                  _ptr(out), _ptr(workspace), workspace.numel() * workspace.element_size(), _stream()),
                 (recv, seg_offset, seg_expert, tab, experts, out, workspace), 14)


def bind_combine(ctx, ret, slot_to_row, topk_w, shared_out, y):
    return Bound(ctx.lib.moe_combine, "moe_combine", (ctx.handle, _ptr(ret), _ptr(slot_to_row), _ptr(topk_w),
                                                      _ptr(shared_out), _ptr(y), _stream()),
                 (ctx, ret, slot_to_row, topk_w, shared_out, y), 6)


def moe_route(ctx, x, w_gate, gate_bias, topk_idx, topk_w):
    _check("moe_route", ctx.lib.moe_route(ctx.handle, _ptr(x), _ptr(w_gate), _ptr(gate_bias), _ptr(topk_idx),
                                          _ptr(topk_w), _stream()))


def moe_traffic(ctx, topk_idx, expert_to_gpu, expert_count, dest_count, n_dropped):
    _, e2g = _i32_array(expert_to_gpu)
    _check("moe_traffic", ctx.lib.moe_traffic(ctx.handle, _ptr(topk_idx), e2g, _ptr(expert_count), _ptr(dest_count),
                                              _ptr(n_dropped), _stream()))


def moe_dispatch(ctx, x, topk_idx, expert_to_gpu, dest_order, send_buf, slot_to_row, row_to_slot, seg_offset,
                 seg_expert):
    _a, e2g = _i32_array(expert_to_gpu)
    _b, order = _i32_array(dest_order)
    _check("moe_dispatch", ctx.lib.moe_dispatch(ctx.handle, _ptr(x), _ptr(topk_idx), e2g, order, _ptr(send_buf),
                                                _ptr(slot_to_row), _ptr(row_to_slot), _ptr(seg_offset),
                                                _ptr(seg_expert), _stream()))


def moe_dispatch_noalloc(shape, x, topk_idx, expert_to_gpu, dest_order, send_buf, slot_to_row, row_to_slot, seg_offset,
                         seg_expert):
    """moe_dispatch without a context: `shape` is (T, H, E, k, G, dtype, renorm, capacity)."""
    T, H, E, k, G, dtype, renorm, capacity = shape
    sh = moe_shape(T, H, E, k, G, _DT[dtype], renorm, capacity)
    _a, e2g = _i32_array(expert_to_gpu)
    _b, order = _i32_array(dest_order)
    _check("moe_dispatch_noalloc", _lib.load().moe_dispatch_noalloc(
        C.byref(sh), _ptr(x), _ptr(topk_idx), e2g, order, _ptr(send_buf), _ptr(slot_to_row), _ptr(row_to_slot),
        _ptr(seg_offset), _ptr(seg_expert), _stream()))


class MoeChunkPlan:
    """Owner of a moe_chunk_plan: a preemptive send plan [(dest, rows), ...] for one GPU."""

    def __init__(self, ctx, expert_to_gpu, chunks):
        self.ctx, self.lib = ctx, ctx.lib
        self.n_chunks = len(chunks)
        _a, e2g = _i32_array(expert_to_gpu)
        _d, dest = _i32_array([c[0] for c in chunks] or [0])
        _r, rows = _i32_array([c[1] for c in chunks] or [0])
        self.handle = C.c_void_p()
        _check("moe_chunk_plan_create", self.lib.moe_chunk_plan_create(ctx.handle, e2g, self.n_chunks, dest, rows,
                                                                       C.byref(self.handle)))

    def close(self):
        if self.handle:
            self.lib.moe_chunk_plan_destroy(self.handle)
            self.handle = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def moe_dispatch_chunks(ctx, plan, x, topk_idx, send_buf, slot_to_row, row_to_slot, chunk_offset, piece_offset,
                        piece_expert, n_pieces):
    _check("moe_dispatch_chunks", ctx.lib.moe_dispatch_chunks(
        ctx.handle, plan.handle, _ptr(x), _ptr(topk_idx), _ptr(send_buf), _ptr(slot_to_row), _ptr(row_to_slot),
        _ptr(chunk_offset), _ptr(piece_offset), _ptr(piece_expert), _ptr(n_pieces), _stream()))


def bind_dispatch_chunks(ctx, plan, x, topk_idx, send_buf, slot_to_row, row_to_slot, chunk_offset, piece_offset,
                         piece_expert, n_pieces):
    return Bound(ctx.lib.moe_dispatch_chunks, "moe_dispatch_chunks",
                 (ctx.handle, plan.handle, _ptr(x), _ptr(topk_idx), _ptr(send_buf), _ptr(slot_to_row), _ptr(row_to_slot),
                  _ptr(chunk_offset), _ptr(piece_offset), _ptr(piece_expert), _ptr(n_pieces), _stream()),
                 (ctx, plan, x, topk_idx, send_buf, slot_to_row, row_to_slot, chunk_offset, piece_offset, piece_expert,
                  n_pieces), 11)


def moe_ffn_workspace_bytes(R_max, H, F, act, dtype):
    return int(_lib.load().moe_ffn_workspace_bytes(R_max, H, F, act, _DT[dtype]))


def expert_table(experts):
    """HOST array of moe_expert_w from a list of dicts of device tensors (w1, w_up or None, w_down)."""
    arr = (moe_expert_w * len(experts))()
    for i, w in enumerate(experts):
        arr[i].w1 = w["w1"].data_ptr()
        arr[i].w_up = w["w_up"].data_ptr() if w.get("w_up") is not None else None
        arr[i].w_down = w["w_down"].data_ptr()
    return arr


def moe_expert_ffn(recv, R, seg_offset, seg_expert, nseg, experts, H, F, act, dtype, out, workspace):
    """`experts` is either a list of weight dicts or a table made by expert_table()."""
    tab = experts if isinstance(experts, C.Array) else expert_table(experts)
    _check("moe_expert_ffn", _lib.load().moe_expert_ffn(
        _ptr(recv), R, _ptr(seg_offset), _ptr(seg_expert), nseg, tab, len(tab), H, F, act, _DT[dtype], _ptr(out),
        _ptr(workspace), workspace.numel() * workspace.element_size(), _stream()))


def moe_expert_ffn_timed(recv, R, seg_offset, seg_expert, nseg, experts, H, F, act, dtype, out, workspace):
    """Measurement twin of moe_expert_ffn; returns (ms_tilemap, ms_gemm1, ms_gemm2) and synchronises."""
    tab = experts if isinstance(experts, C.Array) else expert_table(experts)
    ms = (C.c_float * 3)()
    _check("moe_expert_ffn_timed", _lib.load().moe_expert_ffn_timed(
        _ptr(recv), R, _ptr(seg_offset), _ptr(seg_expert), nseg, tab, len(tab), H, F, act, _DT[dtype], _ptr(out),
        _ptr(workspace), workspace.numel() * workspace.element_size(), _stream(), ms))
    return tuple(ms)


def ffn_phase_marks_len(R, nseg, H, F, act, which_gemm):
    tiles_n = -(-F // (128 if act == ACT_SWIGLU else 256)) if which_gemm == 1 else -(-H // 256)
    return (((R + 255) // 256 + nseg) * tiles_n + 256) * 16


def moe_diag_ffn_phases(recv, R, seg_offset, seg_expert, nseg, experts, H, F, act, dtype, out, workspace, which_gemm, marks):
    """moe_expert_ffn with GEMM `which_gemm` (1 or 2) timed from inside (see the header); `marks` is a zeroed int64
    device tensor of at least ffn_phase_marks_len(...) elements."""
    tab = experts if isinstance(experts, C.Array) else expert_table(experts)
    _check("moe_diag_ffn_phases", _lib.load().moe_diag_ffn_phases(
        _ptr(recv), R, _ptr(seg_offset), _ptr(seg_expert), nseg, tab, len(tab), H, F, act, _DT[dtype], _ptr(out),
        _ptr(workspace), workspace.numel() * workspace.element_size(), which_gemm, _ptr(marks), marks.numel(), _stream()))


def moe_combine(ctx, ret, slot_to_row, topk_w, shared_out, y):
    _check("moe_combine", ctx.lib.moe_combine(ctx.handle, _ptr(ret), _ptr(slot_to_row), _ptr(topk_w),
                                              _ptr(shared_out), _ptr(y), _stream()))


def moe_diag_mfma_run_sum(a, b, d):
    """d[t] = a chain of bf16 MFMAs (16x16x32, zero start) over a[t], b[t]; a, b [n,16,32*run] bf16, d [n,16,16] fp32."""
    _check("moe_diag_mfma_run_sum", _lib.load().moe_diag_mfma_run_sum(_ptr(a), _ptr(b), _ptr(d), a.shape[0], a.shape[2] // 32,
                                                                       _stream()))


def moe_diag_route_phases(ctx, x, w_gate, gate_bias, topk_idx, topk_w, marks):
    """moe_route with clock marks (see the header); `marks` is a zeroed int64 device tensor.  Returns tokens per block."""
    tpb = C.c_int32()
    _check("moe_diag_route_phases", ctx.lib.moe_diag_route_phases(ctx.handle, _ptr(x), _ptr(w_gate), _ptr(gate_bias), _ptr(topk_idx),
                                                                   _ptr(topk_w), _ptr(marks), marks.numel(), C.byref(tpb), _stream()))
    return tpb.value


def moe_diag_mfma_only(n_blocks, iters, sink):
    """Register-only MFMA loop; returns (milliseconds, floating-point operations issued).  Synchronises."""
    ms, flop = C.c_float(), C.c_double()
    _check("moe_diag_mfma_only", _lib.load().moe_diag_mfma_only(n_blocks, iters, _ptr(sink), _stream(), C.byref(ms),
                                                                 C.byref(flop)))
    return ms.value, flop.value


def moe_diag_copy_1r2w(src, dst0, dst1, reps=1):
    """dst0 = dst1 = src, `reps` launches back to back; returns milliseconds per launch.  Synchronises."""
    ms = C.c_float()
    nbytes = src.numel() * src.element_size()
    _check("moe_diag_copy_1r2w", _lib.load().moe_diag_copy_1r2w(_ptr(src), _ptr(dst0), _ptr(dst1), nbytes, reps, _stream(),
                                                                 C.byref(ms)))
    return ms.value


# ------------------------------------------------------------------ host planners (no GPU needed)
def _i64_matrix(D):
    a = np.ascontiguousarray(D, dtype=np.int64)
    return a, a.ctypes.data_as(C.POINTER(C.c_int64))


def _f64_array(B):
    if B is None:
        return None, None
    a = np.ascontiguousarray(B, dtype=np.float64)
    return a, a.ctypes.data_as(C.POINTER(C.c_double))


def aurora_order(D, B=None):
    """Plan one all-to-all; returns a dict of numpy arrays and scalars (the C struct is freed here)."""
    lib = _lib.load()
    Dm, Dp = _i64_matrix(D)
    n = Dm.shape[0]
    _Bm, Bp = _f64_array(B)
    s = aurora_schedule()
    _check("aurora_order", lib.aurora_order(n, Dp, Bp, C.byref(s)))
    try:
        nr = s.n_rounds
        out = {
            "n": n, "n_rounds": nr,
            "duration": np.array([s.duration[r] for r in range(nr)], dtype=np.float64),
            "dst": np.array([s.dst[i] for i in range(nr * n)], dtype=np.int32).reshape(nr, n),
            "dest_order": np.array([s.dest_order[i] for i in range(n * n)], dtype=np.int32).reshape(n, n),
            "alg1_order": np.array([s.alg1_order[i] for i in range(n * n)], dtype=np.int32).reshape(n, n),
            "start": np.array([s.start[i] for i in range(n * n)], dtype=np.float64).reshape(n, n),
            "bmax": s.bmax, "port_bound": s.port_bound, "makespan_rounds": s.makespan_rounds,
            "makespan_order": s.makespan_order, "order_time": s.order_time,
            "candidate_time": [s.candidate_time[c] for c in range(4)], "order_source": s.order_source,
        }
    finally:
        lib.aurora_schedule_free(C.byref(s))
    return out


def aurora_chunks(D, B, g):
    """Plan the all-to-all and return GPU g's chunk list [(dest, rows), ...] under its rounds."""
    lib = _lib.load()
    Dm, Dp = _i64_matrix(D)
    n = Dm.shape[0]
    _Bm, Bp = _f64_array(B)
    s = aurora_schedule()
    _check("aurora_order", lib.aurora_order(n, Dp, Bp, C.byref(s)))
    try:
        dest = (C.c_int32 * max(s.n_rounds, 1))()
        rows = (C.c_int32 * max(s.n_rounds, 1))()
        nc = C.c_int32()
        _check("aurora_chunks", lib.aurora_chunks(C.byref(s), Dp, Bp, g, dest, rows, C.byref(nc)))
        return [(int(dest[i]), int(rows[i])) for i in range(nc.value)]
    finally:
        lib.aurora_schedule_free(C.byref(s))


def aurora_simulate(D, B, order):
    lib = _lib.load()
    Dm, Dp = _i64_matrix(D)
    _Bm, Bp = _f64_array(B)
    _o, op = _i32_array(order)
    t = C.c_double()
    _check("aurora_simulate", lib.aurora_simulate(Dm.shape[0], Dp, Bp, op, C.byref(t)))
    return t.value


def colocate_match(Da, Db):
    lib = _lib.load()
    A, Ap = _i64_matrix(Da)
    Bm, Bp = _i64_matrix(Db)
    pair = (C.c_int32 * A.shape[0])()
    bott = C.c_double()
    _check("colocate_match", lib.colocate_match(A.shape[0], Bm.shape[0], Ap, Bp, pair, C.byref(bott)))
    return list(pair), bott.value


def aurora_assign(load, perf):
    """Theorem 3: expert_to_gpu for one expert per GPU."""
    lib = _lib.load()
    L = np.ascontiguousarray(load, dtype=np.int64)
    Pf = np.ascontiguousarray(perf, dtype=np.float64)
    out = (C.c_int32 * len(L))()
    _check("aurora_assign", lib.aurora_assign(len(L), L.ctypes.data_as(C.POINTER(C.c_int64)),
                                              Pf.ctypes.data_as(C.POINTER(C.c_double)), out))
    return list(out)


def aurora_bottleneck_assign(W):
    lib = _lib.load()
    Wm = np.ascontiguousarray(W, dtype=np.float64)
    n = Wm.shape[0]
    item = (C.c_int32 * n)()
    v = C.c_double()
    _check("aurora_bottleneck_assign", lib.aurora_bottleneck_assign(n, Wm.ctypes.data_as(C.POINTER(C.c_double)), item,
                                                                    C.byref(v)))
    return list(item), v.value


def colocate_hetero_match(Da, Db, time3):
    """Two-stage matching of Sec. 7.2; returns (pair, gpu_of_pair, value)."""
    lib = _lib.load()
    A, Ap = _i64_matrix(Da)
    Bm, Bp = _i64_matrix(Db)
    T3 = np.ascontiguousarray(time3, dtype=np.float64)
    n = A.shape[0]
    pair, gpu = (C.c_int32 * n)(), (C.c_int32 * n)()
    v = C.c_double()
    _check("colocate_hetero_match", lib.colocate_hetero_match(n, Ap, Bp, T3.ctypes.data_as(C.POINTER(C.c_double)), pair,
                                                              gpu, C.byref(v)))
    return list(pair), list(gpu), v.value


def aurora_layer_time(G, N, F, Cc, A):
    lib = _lib.load()
    arrs = [np.ascontiguousarray(a, dtype=np.float64) for a in (G, N, F, Cc, A)]
    t = C.c_double()
    _check("aurora_layer_time", lib.aurora_layer_time(len(arrs[0]), *[a.ctypes.data_as(C.POINTER(C.c_double)) for a in arrs],
                                                      C.byref(t)))
    return t.value


def aurora_colocated_time(Ga, Gb, Fa, Fb, Aa, Ab, Na, Nb, NaNb):
    """Table 2 / Eqn. 4; returns a dict of end times with 't' the inference time."""
    lib = _lib.load()
    out = _lib.aurora_coloc_times()
    _check("aurora_colocated_time", lib.aurora_colocated_time(Ga, Gb, Fa, Fb, Aa, Ab, Na, Nb, NaNb, C.byref(out)))
    return {k: getattr(out, k) for k, _ in out._fields_}
