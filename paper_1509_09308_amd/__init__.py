"""MI355X-native Winograd F(m x m, 3 x 3) convolution: HIP kernels behind a C ABI (libwino.so)
with a thin ctypes binding.  See include/wino.h for the contract of every entry point."""
from .binding import *  # noqa: F401,F403
from . import binding, build, synth  # noqa: F401
