"""MI355X-native MoE-layer share (Aurora's data-parallel hot path): HIP kernels behind a C ABI.

Importing this package loads libaurora_moe.so; it raises if the library has not been
built (`python paper_2410_17043_amd/build.py`).  There is no CPU or PyTorch fallback.
"""
from . import _lib

_lib.load()

from .api import (  # noqa: E402
    F32, BF16, ACT_SILU_MLP, ACT_GELU_MLP, ACT_SWIGLU, TORCH_DTYPE, MoeError, MoeCtx, moe_route, moe_traffic,
    moe_dispatch, moe_dispatch_noalloc, MoeChunkPlan, moe_dispatch_chunks, aurora_chunks, moe_ffn_workspace_bytes, expert_table, moe_expert_ffn, moe_expert_ffn_timed, moe_combine, aurora_order,
    aurora_simulate, colocate_match, aurora_assign, aurora_bottleneck_assign, colocate_hetero_match, aurora_layer_time,
    aurora_colocated_time, Bound, bind_route, bind_traffic, bind_dispatch, bind_dispatch_chunks, bind_expert_ffn,
    bind_combine, moe_diag_mfma_only, moe_diag_copy_1r2w, moe_diag_mfma_run_sum, moe_diag_route_phases, moe_diag_ffn_phases, ffn_phase_marks_len)

__all__ = ["F32", "BF16", "ACT_SILU_MLP", "ACT_GELU_MLP", "ACT_SWIGLU", "TORCH_DTYPE", "MoeError", "MoeCtx",
           "moe_route", "moe_traffic", "moe_dispatch", "moe_dispatch_noalloc", "MoeChunkPlan", "moe_dispatch_chunks", "aurora_chunks", "moe_ffn_workspace_bytes", "expert_table",
           "moe_expert_ffn", "moe_expert_ffn_timed", "moe_combine", "aurora_order", "aurora_simulate", "colocate_match", "aurora_assign", "aurora_bottleneck_assign", "colocate_hetero_match",
           "aurora_layer_time", "aurora_colocated_time", "Bound", "bind_route", "bind_traffic", "bind_dispatch", "bind_dispatch_chunks",
           "bind_expert_ffn", "bind_combine", "moe_diag_mfma_only", "moe_diag_copy_1r2w", "moe_diag_mfma_run_sum",
           "moe_diag_route_phases", "moe_diag_ffn_phases", "ffn_phase_marks_len"]
