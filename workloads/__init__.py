"""Seeded synthetic inputs for the AnTKV online path.

This package only draws random tensors and picks codebook entries from them.  It
holds none of the method's arithmetic (no encoding, no anchor scores, no
attention) and is the one module that both the CPU oracle's tests and the HIP
path's tests consume, so that both sides see identical inputs.
"""
from .configs import CONFIGS, Workload, anchor_count
from .generator import (
    normal_fp16,
    outlier_channels,
    make_qkv,
    make_decode_query,
    make_codebooks,
    random_codes,
    random_anchor_sets,
)

__all__ = [
    "CONFIGS",
    "Workload",
    "anchor_count",
    "normal_fp16",
    "outlier_channels",
    "make_qkv",
    "make_decode_query",
    "make_codebooks",
    "random_codes",
    "random_anchor_sets",
]
