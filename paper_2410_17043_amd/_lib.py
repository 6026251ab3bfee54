"""ctypes loader for libaurora_moe.so (the C ABI declared in include/aurora_moe.h)."""
from __future__ import annotations

import ctypes as C
import os

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libaurora_moe.so")


class moe_shape(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("T", "H", "E", "k", "G", "dtype", "renorm", "capacity")]


class moe_expert_w(C.Structure):
    _fields_ = [("w1", C.c_void_p), ("w_up", C.c_void_p), ("w_down", C.c_void_p)]


class aurora_schedule(C.Structure):
    _fields_ = [("n", C.c_int32), ("n_rounds", C.c_int32), ("duration", C.POINTER(C.c_double)),
                ("dst", C.POINTER(C.c_int32)), ("dest_order", C.POINTER(C.c_int32)),
                ("alg1_order", C.POINTER(C.c_int32)),
                ("start", C.POINTER(C.c_double)), ("bmax", C.c_double), ("port_bound", C.c_double),
                ("makespan_rounds", C.c_double), ("makespan_order", C.c_double), ("order_time", C.c_double),
                ("candidate_time", C.c_double * 4), ("order_source", C.c_int32)]


class aurora_coloc_times(C.Structure):
    _fields_ = [(k, C.c_double) for k in ("Gb", "Na", "Fa", "Nb", "Fb", "Ca", "Aa", "Cb", "Ab", "Ga", "t")]


_vp, _i32, _sz = C.c_void_p, C.c_int32, C.c_size_t
_pd, _pi64, _pi32 = C.POINTER(C.c_double), C.POINTER(C.c_int64), C.POINTER(C.c_int32)
SIGNATURES = {
    "moe_status_str": (C.c_char_p, [C.c_int]),
    "moe_last_error": (C.c_char_p, []),
    "moe_ctx_create": (C.c_int, [C.POINTER(_vp), C.POINTER(moe_shape)]),
    "moe_ctx_destroy": (C.c_int, [_vp]),
    "moe_ctx_invalidate": (C.c_int, [_vp]),
    "moe_ctx_set_rank_reuse": (C.c_int, [_vp, _i32]),
    "moe_route": (C.c_int, [_vp, _vp, _vp, _vp, _vp, _vp, _vp]),
    "moe_traffic": (C.c_int, [_vp, _vp, C.POINTER(_i32), _vp, _vp, _vp, _vp]),
    "moe_dispatch": (C.c_int, [_vp, _vp, _vp, C.POINTER(_i32), C.POINTER(_i32), _vp, _vp, _vp, _vp, _vp, _vp]),
    "moe_dispatch_noalloc": (C.c_int, [C.POINTER(moe_shape), _vp, _vp, C.POINTER(_i32), C.POINTER(_i32), _vp, _vp, _vp, _vp,
                                       _vp, _vp]),
    "moe_chunk_plan_create": (C.c_int, [_vp, C.POINTER(_i32), _i32, C.POINTER(_i32), C.POINTER(_i32), C.POINTER(_vp)]),
    "moe_chunk_plan_destroy": (C.c_int, [_vp]),
    "moe_dispatch_chunks": (C.c_int, [_vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp]),
    "moe_ffn_workspace_bytes": (_sz, [_i32, _i32, _i32, _i32, _i32]),
    "moe_expert_ffn": (C.c_int, [_vp, _i32, _vp, _vp, _i32, C.POINTER(moe_expert_w), _i32, _i32, _i32, _i32, _i32,
                                 _vp, _vp, _sz, _vp]),
    "moe_expert_ffn_timed": (C.c_int, [_vp, _i32, _vp, _vp, _i32, C.POINTER(moe_expert_w), _i32, _i32, _i32, _i32, _i32,
                                       _vp, _vp, _sz, _vp, C.POINTER(C.c_float)]),
    "moe_diag_ffn_phases": (C.c_int, [_vp, _i32, _vp, _vp, _i32, C.POINTER(moe_expert_w), _i32, _i32, _i32, _i32, _i32,
                                      _vp, _vp, _sz, _i32, _vp, _sz, _vp]),
    "moe_combine": (C.c_int, [_vp, _vp, _vp, _vp, _vp, _vp, _vp]),
    "moe_diag_mfma_run_sum": (C.c_int, [_vp, _vp, _vp, _i32, _i32, _vp]),
    "moe_diag_mfma_only": (C.c_int, [_i32, _i32, _vp, _vp, C.POINTER(C.c_float), C.POINTER(C.c_double)]),
    "moe_diag_route_phases": (C.c_int, [_vp, _vp, _vp, _vp, _vp, _vp, _vp, C.c_size_t, C.POINTER(C.c_int32), _vp]),
    "moe_diag_copy_1r2w": (C.c_int, [_vp, _vp, _vp, _sz, _i32, _vp, C.POINTER(C.c_float)]),
    "moe_selfcheck_tile_order": (C.c_int, [_i32, _i32, _i32, _i32]),
    "moe_selfcheck_skinny_plan": (C.c_int, [_i32, _i32, _i32]),
    "moe_selfcheck_row_geometry": (C.c_int, [_i32, _i32, _pi32]),
    "moe_selfcheck_tile_map": (C.c_int, [_pi32, _pi32, _i32, _i32, _i32, _i32, _i32]),
    "aurora_order": (C.c_int, [_i32, C.POINTER(C.c_int64), C.POINTER(C.c_double), C.POINTER(aurora_schedule)]),
    "aurora_schedule_free": (None, [C.POINTER(aurora_schedule)]),
    "aurora_chunks": (C.c_int, [C.POINTER(aurora_schedule), C.POINTER(C.c_int64), C.POINTER(C.c_double), _i32,
                                C.POINTER(_i32), C.POINTER(_i32), C.POINTER(_i32)]),
    "aurora_simulate": (C.c_int, [_i32, C.POINTER(C.c_int64), C.POINTER(C.c_double), C.POINTER(_i32),
                                  C.POINTER(C.c_double)]),
    "aurora_assign": (C.c_int, [_i32, _pi64, _pd, _pi32]),
    "aurora_bottleneck_assign": (C.c_int, [_i32, _pd, _pi32, _pd]),
    "colocate_hetero_match": (C.c_int, [_i32, _pi64, _pi64, _pd, _pi32, _pi32, _pd]),
    "aurora_layer_time": (C.c_int, [_i32, _pd, _pd, _pd, _pd, _pd, _pd]),
    "aurora_colocated_time": (C.c_int, [C.c_double] * 9 + [C.POINTER(aurora_coloc_times)]),
    "colocate_match": (C.c_int, [_i32, _i32, C.POINTER(C.c_int64), C.POINTER(C.c_int64), C.POINTER(_i32),
                                 C.POINTER(C.c_double)]),
}

_lib = None


def load():
    """Load the built library; raises if it is missing (there is no fallback path)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(
                "libaurora_moe.so is not built: run `python paper_2410_17043_amd/build.py` "
                "(this package has no CPU or PyTorch fallback)")
        lib = C.CDLL(LIB_PATH)
        for name, (res, args) in SIGNATURES.items():
            fn = getattr(lib, name)
            fn.restype, fn.argtypes = res, args
        _lib = lib
    return _lib
