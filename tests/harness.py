"""Test-side plumbing: moves seeded host arrays to the GPU and calls the C ABI through
the Python binding.  No arithmetic of the method lives here."""
from __future__ import annotations

import numpy as np
import torch

import paper_2410_17043_amd as P

DEV = "cuda:0"


def dev(a, dtype):
    """float32 host array (values already representable in `dtype`) -> device tensor of `dtype`."""
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(DEV).to(P.TORCH_DTYPE[dtype]).contiguous()


def host(t):
    return t.detach().float().cpu().numpy() if t.is_floating_point() else t.detach().cpu().numpy()


def weights_to_dev(w, dtype):
    return {k: (dev(v, dtype) if v is not None else None) for k, v in w.items()}


class Share:
    """One simulated GPU's share of the layer, run step by step through the library."""

    def __init__(self, cfg, T=None):
        self.cfg = cfg
        self.T = T or cfg.T
        self.ctx = P.MoeCtx(self.T, cfg.H, cfg.E, cfg.k, cfg.G, cfg.dtype, cfg.renorm, cfg.capacity)
        S = self.T * cfg.k
        i32 = dict(dtype=torch.int32, device=DEV)
        self.idx = torch.full((self.T, cfg.k), -7, **i32)
        self.w = torch.full((self.T, cfg.k), float("nan"), dtype=torch.float32, device=DEV)
        self.expert_count = torch.full((cfg.E,), -7, **i32)
        self.dest_count = torch.full((cfg.G,), -7, **i32)
        self.n_dropped = torch.full((1,), -7, **i32)
        self.send_buf = torch.zeros((S, cfg.H), dtype=P.TORCH_DTYPE[cfg.dtype], device=DEV)
        self.slot_to_row = torch.full((S,), -7, **i32)
        self.row_to_slot = torch.full((S,), -7, **i32)
        self.seg_offset = torch.full((cfg.E + 1,), -7, **i32)
        self.seg_expert = torch.full((cfg.E,), -7, **i32)
        self.y = torch.zeros((self.T, cfg.H), dtype=P.TORCH_DTYPE[cfg.dtype], device=DEV)

    def route(self, x, wg, bias):
        P.moe_route(self.ctx, x, wg, bias, self.idx, self.w)

    def traffic(self, e2g):
        P.moe_traffic(self.ctx, self.idx, e2g, self.expert_count, self.dest_count, self.n_dropped)

    def dispatch(self, x, e2g, dest_order):
        P.moe_dispatch(self.ctx, x, self.idx, e2g, dest_order, self.send_buf, self.slot_to_row, self.row_to_slot,
                       self.seg_offset, self.seg_expert)

    def combine(self, ret, shared_out=None):
        P.moe_combine(self.ctx, ret, self.slot_to_row, self.w, shared_out, self.y)


def run_ffn(recv, seg_offset, seg_expert, experts, H, F, act, dtype):
    """recv: device [R,H]; seg_offset / seg_expert: host int lists; experts: list of device weight dicts."""
    R = recv.shape[0]
    so = torch.tensor(np.asarray(seg_offset, dtype=np.int32), device=DEV)
    se = torch.tensor(np.asarray(seg_expert, dtype=np.int32), device=DEV)
    ws = torch.empty(max(P.moe_ffn_workspace_bytes(R, H, F, act, dtype), 256), dtype=torch.uint8, device=DEV)
    out = torch.full((R, H), float("nan"), dtype=P.TORCH_DTYPE[dtype], device=DEV)
    P.moe_expert_ffn(recv, R, so, se, len(seg_expert), experts, H, F, act, dtype, out, ws)
    torch.cuda.synchronize()
    return out


def rel_err(got, ref):
    """Normwise error: max |got - ref| / max |ref|."""
    ref = np.asarray(ref, dtype=np.float64)
    return float(np.max(np.abs(np.asarray(got, dtype=np.float64) - ref)) / max(np.max(np.abs(ref)), 1e-300))
