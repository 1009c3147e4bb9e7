"""MI355X-native per-tensor FP8 linear layer with the fused TWEO penalty, and W8A8 INT8 linear.

The product is the C-ABI library declared in include/tweo.h (HIP kernels under
csrc/); `binding` marshals torch tensors into it and `synth` generates the
seeded workloads.
"""
from . import synth  # noqa: F401
from .binding import *  # noqa: F401,F403
from .binding import load, TweoError, LIB_PATH  # noqa: F401
