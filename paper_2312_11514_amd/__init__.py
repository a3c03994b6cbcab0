"""MI355X-native sparse-FFN hot path of "LLM in a flash" (arXiv 2312.11514).

The product is the C-ABI library declared in include/lif.h (HIP kernels for gfx950);
this package is the thin ctypes binding over it.  There is no CPU fallback: importing
`binding` without a built liblif.so raises.
"""
from .binding import (  # noqa: F401
    LifError, Layer, load_library, LIF_OK, LIF_INVALID_ARG, LIF_BAD_STATE, LIF_CAPACITY, LIF_HIP_ERROR,
    LIF_F32, LIF_F16, FFN_SKIP_DEAD, FFN_FULL_BUNDLE, PRED_LOWRANK, PRED_GATE, KERNEL_NAMES, profile_read, profile_handoff,
    profile_handoff_bytes,
)
