"""DeTAG hot path on one MI355X: hand-written HIP kernels behind a C ABI
(include/detag.h, built into libdetag.so) and this thin ctypes binding.

Importing the package loads nothing; the shared library is loaded on first
use and its absence is an error, never a fallback.
"""
from .binding import *  # noqa: F401,F403
from .binding import Context, Factors, Topology, DetagError, detag_create, lib, LIB_PATH, EXPORTS  # noqa: F401
from .memory import padded_ld, new_matrix  # noqa: F401
