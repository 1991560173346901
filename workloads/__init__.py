"""Seeded synthetic inputs shared by the CPU oracle's tests and the HIP path's tests and bench.

This package holds input generation and storage-format helpers only.  None of the
method's arithmetic (codes, matching, merging, selection, attention) lives here.
"""
from .synth import (  # noqa: F401
    CONFIGS,
    Codec,
    FrameStream,
    PromptSet,
    bf16_bits_to_f32,
    f32_to_bf16_bits,
    make_codec,
    make_sign_matrix,
    to_f32,
    to_storage,
)
