"""Seeded synthetic inputs shaped like the paper's VAR workloads.

Shared by the oracle-side tests and the HIP-side tests/bench.  Holds no part of
the method's arithmetic: only shapes, seeds and random tensors.
"""
from .configs import CONFIGS, Workload, get  # noqa: F401
from .gen import (bf16_bits, make_attn_map, make_cfg_share, make_qkv, make_workload_qkv, seq_len,  # noqa: F401
                  to_oracle_array)
