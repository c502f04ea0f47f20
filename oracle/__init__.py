"""CPU oracle for the LCD table-lookup linear layer.  TEST INFRASTRUCTURE ONLY.

Only ``tests/``, ``__graft_entry__.smoke()`` and ``bench.py``'s ``cpu_baseline`` leg may
import this package.  It shares no code with ``paper_2506_12038_amd`` and never imports it.
"""
from .lcd_oracle import (
    build_oracle,
    half_to_double,
    dequant,
    smooth,
    lut_matmul,
    bucket_matmul,
    input_transform,
    quantised_lut_matmul,
    num_threads,
)
from .metrics import parity_errors
from .cluster_oracle import assign_nearest, cluster_counts, merge_closest, merge_closest_stored, round_to_half

__all__ = [
    "build_oracle", "half_to_double", "dequant", "smooth", "lut_matmul", "bucket_matmul",
    "input_transform", "quantised_lut_matmul", "num_threads", "parity_errors",
    "assign_nearest", "cluster_counts", "merge_closest", "merge_closest_stored", "round_to_half",
]
