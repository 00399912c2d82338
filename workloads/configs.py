"""The five benchmark/parity workloads (shapes, radii, seeds).

VAR's 256x256 scale list (1,2,3,4,5,6,8,10,13,16 -> 680 tokens) is the one the
paper prints (Section 2, implementation details); the 512x512 and 2K-style
lists are the benchmark's own.  Seeds: the tiny case uses seed 0; the others
use 1..4 in order.  Q, K, V are drawn in that order from one generator.
"""
from dataclasses import dataclass
from typing import Optional, Tuple


@dataclass(frozen=True)
class Workload:
    name: str
    scales: Tuple[int, ...]
    batch: int
    heads: int
    head_dim: int
    dtype: str                 # "f32" | "bf16"
    radius: int
    n_sink: int
    q_scales: Optional[Tuple[int, int]]   # [begin, end) query scales; None = all
    seed: int
    input_scale: float         # multiplies the N(0,1) draws
    sm_scale: float
    cfg_share: bool = False

    @property
    def q_range(self):
        return (0, len(self.scales)) if self.q_scales is None else self.q_scales


VAR256 = (1, 2, 3, 4, 5, 6, 8, 10, 13, 16)
VAR512 = (1, 2, 3, 4, 6, 9, 13, 18, 24, 32)
VAR2K = (1, 2, 3, 4, 6, 9, 13, 18, 24, 32, 48, 64, 96, 128)

CONFIGS = {
    "tiny_f32": Workload("tiny_f32", (1, 2, 3, 4), 1, 1, 64, "f32", 1, 0, None, 0, 1.0, 0.125),
    "var_d16": Workload("var_d16", VAR256, 2, 16, 64, "bf16", 2, 0, None, 1, 0.125, 0.125),
    "var_d30_kvstep": Workload("var_d30_kvstep", VAR256, 16, 30, 64, "bf16", 3, 0, (9, 10), 2,
                               1.0, 0.125),
    "var_d36_512": Workload("var_d36_512", VAR512, 8, 36, 64, "bf16", 4, 0, None, 3, 1.0, 0.125),
    "var_2k_cfg": Workload("var_2k_cfg", VAR2K, 2, 16, 64, "bf16", 4, 0, None, 4, 1.0, 0.125,
                           cfg_share=True),
}


def get(name: str) -> Workload:
    return CONFIGS[name]
