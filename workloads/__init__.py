"""Seeded synthetic inputs shared by the tests, the bench and the oracle's callers.

This package holds no arithmetic of the method itself (no U-Net op, no scheduler,
no guidance, no similarity filter): only random tensors, the weight-blob filler
and the table of workload shapes.  It imports neither the oracle nor the HIP
binding.
"""
from .synth import (  # noqa: F401
    CONFIGS,
    IMAGE_STAGE,
    image_frames,
    MINI_CONFIGS,
    normal,
    make_weights,
    round_to_bf16,
    ssf_frames,
    stream_inputs,
)
