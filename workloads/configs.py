"""The five workload configurations, in the paper's notation.

M   routed (base) experts per MoE layer           (paper Sec. 2.1)
k   experts selected per token                    (paper Sec. 2.1)
N   maximum number of adapters in one batch       (paper Sec. 3.1)
E_max  slots reserved per adapter                 (paper Sec. 3.1)
P = M + N*E_max  slots of the virtual weight tensor (paper Sec. 4.1)
H   hidden size, I expert intermediate size, S shared experts (DeepSeek-V2-Lite shape)
"""
from __future__ import annotations

from dataclasses import dataclass, replace

BASE_SEED = 250817624


@dataclass(frozen=True)
class MoEConfig:
    name: str
    index: int            # position in the configuration list; enters the seed
    H: int
    M: int
    I: int
    S: int
    k: int
    T: int
    N: int
    E_max: int
    dtype: str            # "f32" or "bf16": storage type of tokens and expert weights
    tuned_lo: int         # each adapter tunes U{tuned_lo..tuned_hi} experts per layer
    tuned_hi: int
    aid_dist: str         # "uniform" or "zipf" over the N+1 classes (0 = base model)
    zipf_s: float = 1.1
    gate_bias: float = 0.0  # added to the gate logit of experts tuned by the token's adapter
    L: int = 1            # stacked MoE layers
    weight_std: float = 0.02
    integer_only: bool = False

    @property
    def P(self) -> int:
        return self.M + self.N * self.E_max

    @property
    def seed(self) -> int:
        return BASE_SEED * 10 + self.index

    def with_(self, **kw) -> "MoEConfig":
        return replace(self, **kw)


CONFIGS = (
    # C0: tiny fp32 layer, the oracle finishes it in milliseconds.
    MoEConfig("c0_tiny_f32", 0, H=256, M=8, I=128, S=1, k=2, T=64, N=2, E_max=2,
              dtype="f32", tuned_lo=2, tuned_hi=2, aid_dist="uniform"),
    # C1: DeepSeek-V2-Lite-shaped layer, decode batch.
    MoEConfig("c1_dsv2lite_decode", 1, H=2048, M=64, I=1408, S=2, k=6, T=64, N=4, E_max=16,
              dtype="bf16", tuned_lo=6, tuned_hi=6, aid_dist="uniform"),
    # C2: same shape, 8K-token prefill, 20 adapters, skewed popularity, specialised gates.
    MoEConfig("c2_dsv2lite_prefill", 2, H=2048, M=64, I=1408, S=2, k=6, T=8192, N=20, E_max=16,
              dtype="bf16", tuned_lo=2, tuned_hi=16, aid_dist="zipf", zipf_s=1.1, gate_bias=2.0),
    # C3: integer-only reroute/permute microbenchmark.
    MoEConfig("c3_reroute_permute_int", 3, H=0, M=64, I=0, S=0, k=6, T=1 << 20, N=20, E_max=16,
              dtype="bf16", tuned_lo=2, tuned_hi=16, aid_dist="uniform", integer_only=True),
    # C4: 26 stacked C1-shaped layers, 20 adapters, one 256-token decode step.
    MoEConfig("c4_dsv2lite_stack26", 4, H=2048, M=64, I=1408, S=2, k=6, T=256, N=20, E_max=16,
              dtype="bf16", tuned_lo=2, tuned_hi=16, aid_dist="uniform", L=26),
)


def get_config(name_or_index) -> MoEConfig:
    if isinstance(name_or_index, int):
        return CONFIGS[name_or_index]
    for c in CONFIGS:
        if c.name == name_or_index or c.name.split("_")[0] == name_or_index:
            return c
    raise KeyError(name_or_index)
