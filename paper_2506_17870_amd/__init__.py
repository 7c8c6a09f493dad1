"""NestQuant nested-integer hot path for AMD MI355X (gfx950): hand-written HIP kernels
behind a C ABI (include/nq.h) with a thin ctypes binding.  PyTorch is used only for device
memory and streams."""
from .binding import *  # noqa: F401,F403
from .binding import NestedWeight, NQError, make_cfg, make_epilogue, nq_cfg, nq_conv_shape, nq_epilogue, nq_weight  # noqa: F401
