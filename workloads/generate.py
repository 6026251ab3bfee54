"""Seeded generators for every synthetic input.

Seeds follow ``1000 * config index (+ offset) + stream id`` so that every array
can be regenerated on its own.  Stream ids:

    0  activations x[T, H]            ~ N(0, 1)
    1  gate weight Wg[E, H]           ~ N(0, 0.02)
    2  traffic matrix draws
    3  link rates B[G]                ~ U[0.5, 1.0]
    4  rows received from other GPUs  ~ N(0, 1)
    5  rows returned by other GPUs    ~ N(0, 1)
    10 + e   weights of routed expert e   ~ N(0, 0.02)
    200 + s  weights of shared expert s   ~ N(0, 0.02)

Arrays are returned as float32 whose values are exactly representable in the
config's storage dtype (rounded once, round-to-nearest-even for bf16), so the
same host array can be handed to a bf16 device tensor and to an fp64 CPU
computation without either side seeing different numbers.
"""
from __future__ import annotations

import numpy as np

from .configs import LayerConfig, ACT_SWIGLU

S_X, S_WGATE, S_TRAFFIC, S_LINK, S_RECV, S_RET = 0, 1, 2, 3, 4, 5
S_EXPERT, S_SHARED = 10, 200


def rng_for(cfg: LayerConfig, stream: int, sub: int = 0) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=[cfg.seed_base + stream, sub]))


def to_bf16_grid(a: np.ndarray) -> np.ndarray:
    """Round float32 values to the nearest bf16-representable value (ties to even)."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32).astype(np.uint64)
    lsb = (u >> 16) & 1
    u = (u + 0x7FFF + lsb) & 0xFFFF0000
    return u.astype(np.uint32).view(np.float32).reshape(a.shape)


def round_to_dtype(a: np.ndarray, dtype: str) -> np.ndarray:
    if dtype == "bf16":
        return to_bf16_grid(a)
    if dtype == "fp32":
        return np.ascontiguousarray(a, dtype=np.float32)
    raise ValueError(dtype)


def _normal(rng, shape, sigma, dtype):
    a = rng.standard_normal(size=shape, dtype=np.float32)
    if sigma != 1.0:
        a *= np.float32(sigma)
    return round_to_dtype(a, dtype)


def zipf_popularity(E: int, s: float) -> np.ndarray:
    """pop_e proportional to (e + 1) ** -s, normalised; s = 0 gives uniform."""
    r = np.arange(1, E + 1, dtype=np.float64)
    p = r ** (-float(s))
    return p / p.sum()


def make_layer_inputs(cfg: LayerConfig, gpu: int = 0) -> dict:
    """Activations and gate parameters of one simulated GPU.

    The gate weight is the same on every simulated GPU; the activations depend
    on ``gpu``.  ``gate_bias`` is log(popularity), which skews the local routing
    the same way the synthetic traffic of the other GPUs is skewed; it is None
    when the config has uniform popularity.
    """
    x = _normal(rng_for(cfg, S_X, gpu), (cfg.T, cfg.H), 1.0, cfg.dtype)
    wg = _normal(rng_for(cfg, S_WGATE), (cfg.E, cfg.H), 0.02, cfg.dtype)
    bias = None
    if cfg.zipf_s > 0.0:
        bias = np.log(zipf_popularity(cfg.E, cfg.zipf_s)).astype(np.float32)
    e2g = (np.arange(cfg.E, dtype=np.int32) // cfg.E_loc).astype(np.int32)
    return {"x": x, "w_gate": wg, "gate_bias": bias, "expert_to_gpu": e2g}


def make_expert_weights(cfg: LayerConfig, expert: int, shared: bool = False) -> dict:
    """Weights of one expert, stored [out, in] row-major: w1[F,H], (w_up[F,H]), w_down[H,F]."""
    rng = rng_for(cfg, (S_SHARED if shared else S_EXPERT) + expert)
    w = {"w1": _normal(rng, (cfg.F, cfg.H), 0.02, cfg.dtype)}
    w["w_up"] = _normal(rng, (cfg.F, cfg.H), 0.02, cfg.dtype) if cfg.act == ACT_SWIGLU else None
    w["w_down"] = _normal(rng, (cfg.H, cfg.F), 0.02, cfg.dtype)
    return w


def make_traffic_matrix(cfg: LayerConfig) -> dict:
    """Synthetic G x G traffic matrix in token-slots.

    Every simulated GPU holds T tokens; each token picks k distinct experts
    without replacement with probabilities given by the Zipf popularity (a
    Gumbel top-k draw).  ``per_expert[i, e]`` is the number of slots GPU i sends
    to expert e, clipped to the per-source capacity when the config has one;
    ``D[i, j]`` sums it over the experts hosted on GPU j (contiguous blocks of
    E / G experts).  The diagonal holds the self traffic.
    """
    pop = zipf_popularity(cfg.E, cfg.zipf_s)
    per_expert = np.zeros((cfg.G, cfg.E), dtype=np.int64)
    for i in range(cfg.G):
        rng = rng_for(cfg, S_TRAFFIC, i)
        keys = np.log(pop)[None, :] + rng.gumbel(size=(cfg.T, cfg.E))
        picks = np.argpartition(-keys, cfg.k - 1, axis=1)[:, :cfg.k]
        per_expert[i] = np.bincount(picks.ravel(), minlength=cfg.E)
    if cfg.capacity > 0:
        per_expert = np.minimum(per_expert, cfg.capacity)
    D = per_expert.reshape(cfg.G, cfg.G, cfg.E_loc).sum(axis=2)
    return {"per_expert": per_expert, "D": D}


def make_link_rates(cfg: LayerConfig) -> np.ndarray:
    if not cfg.hetero_links:
        return np.ones(cfg.G, dtype=np.float64)
    return rng_for(cfg, S_LINK).uniform(0.5, 1.0, size=cfg.G)


def make_rows(cfg: LayerConfig, stream: int, n_rows: int, sub: int = 0) -> np.ndarray:
    """N(0, 1) rows standing in for activations that arrive from other GPUs."""
    return _normal(rng_for(cfg, stream, sub), (n_rows, cfg.H), 1.0, cfg.dtype)
