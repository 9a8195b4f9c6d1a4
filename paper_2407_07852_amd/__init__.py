"""MI355X-native DiLoCo optimizer hot path: fused AdamW inner step, fused outer step
(pseudo-gradient, optional FP16 rounding, mean over k workers, Nesterov SGD, broadcast) and the
gradient-scaler inf/NaN check, as hand-written gfx950 HIP kernels behind a C ABI
(include/diloco.h).  This package is the ctypes binding of that library."""
from .binding import *  # noqa: F401,F403
from .binding import DiLoCo, DilocoError, lib  # noqa: F401
