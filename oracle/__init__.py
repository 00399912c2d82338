"""fp64 CPU oracle for LiteVAR's windowed attention.  TEST INFRASTRUCTURE ONLY.

Importable from tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg;
the product package never imports it and it never imports the product package.
"""
from .oracle import (  # noqa: F401
    allowed, attn, attn_probs, attn_qkv8, band_part_columns, calibrate, calibrate_band, cfg_share,
    dequantize_rows, expand_radii,
    index_sets, mask_dense, num_threads, quantize_rows, row_counts, scale_offsets, seq_len,
    token_coords,
)
