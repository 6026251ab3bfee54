"""The five layer-share workloads (shapes only).

Each entry describes ONE simulated GPU's share of an expert-parallel MoE layer:
T local tokens of width H are gated over E experts (top-k); the E experts are
spread over G simulated GPUs, E/G per GPU.  The paper's own traces (LIMoE
statistics on COCO / ImageNet, Sec. 8.1) are not available, so these shapes and
a Zipf expert popularity stand in for them.
"""
from __future__ import annotations

import dataclasses
import math
from dataclasses import dataclass

ACT_SILU_MLP = 0   # W2 . silu(W1 . x)
ACT_GELU_MLP = 1   # W2 . gelu_tanh(W1 . x)
ACT_SWIGLU = 2     # Wd . (silu(Wg . x) * (Wu . x))


@dataclass(frozen=True)
class LayerConfig:
    name: str
    index: int            # 1..5, used in the seed
    dtype: str            # "fp32" | "bf16"
    T: int                # local tokens on the GPU under test (and on every simulated GPU)
    H: int                # hidden size
    F: int                # expert inner size
    E: int                # routed experts
    k: int                # experts per token
    G: int                # simulated GPUs
    act: int              # ACT_*
    renorm: int           # 1: top-k weights divided by their sum
    capacity_factor: float = 0.0   # 0 = no capacity limit
    zipf_s: float = 0.0            # 0 = uniform popularity
    n_shared: int = 0              # shared experts applied to every local token
    hetero_links: bool = False     # per-GPU link rates U[0.5, 1.0] for the host scheduler
    seed_offset: int = 0           # separates two configs that share an index

    @property
    def seed_base(self) -> int:
        return 1000 * self.index + self.seed_offset

    @property
    def E_loc(self) -> int:
        return self.E // self.G

    @property
    def capacity(self) -> int:
        """Rows kept per expert per source GPU (0 = unlimited)."""
        if self.capacity_factor <= 0.0:
            return 0
        return int(math.ceil(self.capacity_factor * self.T * self.k / self.E))

    @property
    def n_mats(self) -> int:
        return 3 if self.act == ACT_SWIGLU else 2

    @property
    def ffn_flops_per_row(self) -> int:
        return 2 * self.n_mats * self.H * self.F


CONFIGS = {
    "c1_tiny_fp32": LayerConfig("c1_tiny_fp32", 1, "fp32", T=256, H=64, F=128, E=8, k=2, G=4,
                                act=ACT_SILU_MLP, renorm=0),
    "c2_mixtral": LayerConfig("c2_mixtral", 2, "bf16", T=4096, H=4096, F=14336, E=8, k=2, G=8,
                              act=ACT_SWIGLU, renorm=1, zipf_s=1.0),
    "c3_switch": LayerConfig("c3_switch", 3, "bf16", T=8192, H=1024, F=4096, E=64, k=1, G=16,
                             act=ACT_GELU_MLP, renorm=0, capacity_factor=1.25, zipf_s=1.2),
    "c4a_coloc": LayerConfig("c4a_coloc", 4, "bf16", T=2048, H=4096, F=14336, E=8, k=2, G=8,
                             act=ACT_SWIGLU, renorm=1),
    "c4b_coloc": LayerConfig("c4b_coloc", 4, "bf16", T=4096, H=2048, F=5632, E=16, k=2, G=8,
                             act=ACT_SWIGLU, renorm=1, seed_offset=500),
    "c5_finegrained": LayerConfig("c5_finegrained", 5, "bf16", T=16384, H=2048, F=1408, E=64, k=6,
                                  G=16, act=ACT_SWIGLU, renorm=0, zipf_s=1.1, n_shared=2,
                                  hetero_links=True),
}


def get_config(name: str) -> LayerConfig:
    return CONFIGS[name]


def scaled(cfg: LayerConfig, **overrides) -> LayerConfig:
    """A copy of a config with some sizes replaced (used for reduced parity cases)."""
    return dataclasses.replace(cfg, **overrides)
