"""The C-ABI library loads, exports every symbol the header declares, and validates
arguments before touching the GPU (no compute calls here)."""
import ctypes as C
import os
import re

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "aurora_moe.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = re.findall(r"\b([a-z_][a-z0-9_]*)\s*\([^;{}]*\)\s*;", text)
    return sorted(set(n for n in names if n.startswith(("moe_", "aurora_", "colocate_"))))


def test_every_declared_symbol_is_exported_and_bound():
    from paper_2410_17043_amd import _lib
    lib = _lib.load()
    names = declared_functions()
    assert {"moe_route", "moe_traffic", "moe_dispatch", "moe_expert_ffn", "moe_combine", "aurora_order",
            "colocate_match", "moe_ctx_create", "moe_ctx_destroy", "moe_ffn_workspace_bytes", "moe_status_str",
            "moe_last_error", "aurora_schedule_free", "aurora_simulate", "moe_ctx_invalidate",
            "moe_expert_ffn_timed"} <= set(names)
    for n in names:
        assert hasattr(lib, n), n
        assert n in _lib.SIGNATURES, n


def test_status_strings_and_shape_validation():
    import paper_2410_17043_amd as P
    from paper_2410_17043_amd import _lib
    lib = _lib.load()
    assert lib.moe_status_str(0) == b"MOE_OK" and lib.moe_status_str(-2) == b"MOE_ESHAPE"
    bad = [dict(T=0, H=64, E=8, k=2, G=4), dict(T=8, H=64, E=8, k=9, G=4), dict(T=8, H=64, E=300, k=2, G=4),
           dict(T=8, H=6, E=8, k=2, G=4), dict(T=8, H=64, E=8, k=2, G=65)]
    codes = []
    for kw in bad:
        with pytest.raises(P.MoeError) as ei:
            P.MoeCtx(dtype="bf16", **kw)
        codes.append(ei.value.name)
        assert str(ei.value)
    assert codes == ["MOE_EINVAL", "MOE_ESHAPE", "MOE_ESHAPE", "MOE_EALIGN", "MOE_ESHAPE"]
    assert P.moe_ffn_workspace_bytes(100, 128, 256, 2, "bf16") >= 100 * 256 * 2
    assert P.moe_ffn_workspace_bytes(100, 128, 256, 7, "bf16") == 0
    rc = lib.moe_expert_ffn(None, 0, None, None, 0, None, 0, 0, 0, 0, 0, None, None, 0, None)
    assert rc == -1 and b"NULL" in lib.moe_last_error()


def test_planner_argument_errors():
    import paper_2410_17043_amd as P
    with pytest.raises(P.MoeError):
        P.aurora_order([[0, -1], [1, 0]])
    with pytest.raises(P.MoeError):
        P.aurora_order([[0, 1], [1, 0]], B=[1.0, 0.0])
    with pytest.raises(P.MoeError):
        P.aurora_simulate([[0, 1], [1, 0]], None, [[1, 1], [0, 1]])
    with pytest.raises(P.MoeError):
        P.colocate_match(np.zeros((3, 3)), np.zeros((2, 2)))
