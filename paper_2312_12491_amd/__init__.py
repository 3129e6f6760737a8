"""MI355X-native Stream Batch denoising step (StreamDiffusion, arXiv 2312.12491).

Thin ctypes binding over libsdstream.so (hand-written HIP for gfx950).  PyTorch is used by callers for
device memory and streams only; every step of the path runs in the library's kernels.  There is no CPU
fallback: importing works without a GPU (so the symbols can be checked), creating an engine does not.
"""
from .binding import (  # noqa: F401
    CFG_FULL, CFG_NONE, CFG_ONETIME, CFG_SELF, Engine, SdstreamError, config_from_dict, lib, ssf_decide,
    ssf_decide_hard, ssf_static,
)
