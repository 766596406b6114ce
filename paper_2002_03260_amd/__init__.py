"""dft3d for MI355X: thin Python binding over the C-ABI library (see include/dft3d.h).

Importing this package does not load the shared library; the first call does, and fails
loudly if it has not been built (there is no CPU fallback).
"""
from .binding import (  # noqa: F401
    BACKWARD, FFT, FLAG_3M, FLAG_ADJOINT, FLAG_BF16X3, FLAG_CLOBBER_INPUT, FLAG_COMPLEX128, FLAG_UNFUSED, FORWARD, KDFT, Dft3dError, Plan,
    device_copy, generate_matrix, generate_points_matrix, generate_twiddle, library_path, load_library,
)
