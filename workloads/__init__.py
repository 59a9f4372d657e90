"""Seeded synthetic inputs shaped like the paper's video-attention workloads.

This package holds input *data* recipes only (shapes, seeds, value
distributions).  None of the method's arithmetic lives here: no pooling, no
window geometry, no selection, no attention.  Both the CPU oracle's tests and
the GPU path's tests/bench draw their inputs from here so that they see the
same bits.
"""
from .generate import (CONFIGS, Workload, get_workload, make_ar1_proxy, make_head, make_qkv,  # noqa: F401
                       tiny_case)
