"""Seeded synthetic video-feature workloads for Temporal Token Fusion.

This package only produces input tensors (and the bookkeeping needed to redraw single
tokens).  It contains none of the method's arithmetic: no similarity, no anchor rule,
no gating.  Both the CPU oracle's tests and the GPU path's tests draw inputs from here.
"""
from .ttf_gen import (  # noqa: F401
    CONFIGS,
    ClipBatch,
    WorkloadConfig,
    bf16_bits_to_f32,
    f32_to_bf16_bits,
    make_clip_batch,
    similarity_field,
)
