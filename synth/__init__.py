"""Seeded synthetic inputs shared by the CPU oracle's tests and the HIP path's tests.

This package holds the input recipe only: token layout of a VGGT global-attention
layer, a smooth random field with per-frame shifts, and the Q/K/V projections.
None of the method's arithmetic (reordering, matching, merging, attention,
unmerging) lives here.
"""
from .vggt_tokens import CONFIGS, Workload, workload, make_qkv  # noqa: F401
