"""EntropyCache denoising step for MI355X: HIP kernels behind a C ABI (libec.so) and a thin
ctypes binding.  Build the library first (`python -m paper_2603_18489_amd.build`)."""
from .binding import *  # noqa: F401,F403
