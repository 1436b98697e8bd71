"""MI355X-native W8A8 + step-cache + variance-compensation DiT sampler step.

The work is done by hand-written HIP kernels behind a C ABI (include/qc.h,
built to libqc.so); this package is only the ctypes binding.  PyTorch supplies
device memory and the current stream, nothing else."""
from .binding import *  # noqa: F401,F403
from .binding import __all__  # noqa: F401
