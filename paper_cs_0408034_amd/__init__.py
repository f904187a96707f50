"""MI355X-native pLogP collective-tuning sweep (arXiv cs/0408034, Section 3).

`plogp` is the thin binding over the C-ABI HIP library (libplogp.so); every
step of the method runs in that library's gfx950 kernels.
"""
from . import plogp  # noqa: F401
