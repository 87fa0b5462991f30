"""MI355X-native WaveTune hot path: tile-parameterised MFMA GEMM + wave-aware config selection.

Everything runs in libwt.so (HIP kernels and C++ host code behind the C ABI of include/wt.h);
this package is the thin binding.  Build with `python -m paper_2604_10187_amd.build`.
"""
from .binding import *  # noqa: F401,F403
from .binding import EXPORTS, LIB_PATH, WtError, lib, make_grid, status_string  # noqa: F401
