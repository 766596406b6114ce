"""ctypes front end of the fp64 CPU oracle (``dft3d_oracle.c``).  TEST INFRASTRUCTURE ONLY.

Only the tests, ``__graft_entry__.smoke()`` and the CPU-baseline leg of ``bench.py`` may import
this module.  It shares nothing with the HIP library and does not import it.

The functions mirror the C file:

* :func:`dft_matrix`       -- rows of the per-axis transform matrix (paper Eq. 3, Eq. 12)
* :func:`points_matrix`    -- Vandermonde matrix of arbitrary evaluation points (paper Eq. 3 as written)
* :func:`dft3d_points`     -- the transform at arbitrary per-axis evaluation points (Eq. 10 in general form)
* :func:`mode_contract`    -- one mode product (paper Eq. 2 applied along a tensor index)
* :func:`dft3d`            -- the 3-D transform one axis at a time (paper Eq. 10 / Eq. 11)
* :func:`dft3d_brute`      -- the literal triple sum of Eq. 10 (tiny inputs; pins ``dft3d``)
* :func:`dft3d_sampled`    -- selected output slabs of a large transform (same sums, only the
  requested output frequencies along the first axis are evaluated)
* :func:`dft3d_pencils`    -- selected output pencils along the first axis, likewise
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "dft3d_oracle.c")
_LIB = os.path.join(_HERE, "libdft3d_oracle.so")

FORWARD = -1
BACKWARD = +1

_lib = None


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (fp64, OpenMP, no fast-math).  Returns the library path."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c99", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
               _SRC, "-o", _LIB, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        i64, dp, fp, ip = ctypes.c_int64, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int
        lib.oracle_num_threads.restype = ctypes.c_int
        lib.oracle_dft_matrix.argtypes = [i64, i64, ctypes.c_void_p, dp, ip, dp]
        lib.oracle_dft_matrix.restype = None
        lib.oracle_points_matrix.argtypes = [i64, i64, dp, dp]
        lib.oracle_points_matrix.restype = None
        lib.oracle_mode_contract.argtypes = [i64, i64, i64, i64, dp, dp, dp]
        lib.oracle_mode_contract.restype = None
        lib.oracle_mode_contract_f32.argtypes = [i64, i64, i64, i64, dp, fp, dp]
        lib.oracle_mode_contract_f32.restype = None
        lib.oracle_dft3d.argtypes = [i64, i64, i64, fp, dp, dp, dp, dp, ip, ip]
        lib.oracle_dft3d.restype = ctypes.c_int
        lib.oracle_dft3d_brute.argtypes = [i64, i64, i64, fp, dp, dp, dp, dp, ip]
        lib.oracle_dft3d_brute.restype = None
        _lib = lib
    return _lib


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def _ptr(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _coords(c, n):
    if c is None:
        return None
    c = np.ascontiguousarray(c, dtype=np.float64)
    if c.shape != (n,):
        raise ValueError(f"coordinate array must have shape ({n},), got {c.shape}")
    return c


def dft_matrix(n: int, coords=None, sign: int = FORWARD, ks=None) -> np.ndarray:
    """Rows ``ks`` (default 0..n-1) of the n-column transform matrix, complex128."""
    c = _coords(coords, n)
    if ks is None:
        K, ksa = n, None
    else:
        ksa = np.ascontiguousarray(ks, dtype=np.int64)
        K = ksa.shape[0]
    M = np.empty((K, n), dtype=np.complex128)
    _load().oracle_dft_matrix(K, n, _ptr(ksa), _ptr(c), int(sign), _ptr(M))
    return M


def points_matrix(z, n: int) -> np.ndarray:
    """K x n Vandermonde matrix ``M[r, j] = z_r**(-j)`` of paper Eq. 3 for arbitrary points ``z``."""
    z = np.ascontiguousarray(z, dtype=np.complex128)
    if z.ndim != 1 or np.any(z == 0):
        raise ValueError("points must be a 1-D array of non-zero complex numbers")
    M = np.empty((z.shape[0], n), dtype=np.complex128)
    _load().oracle_points_matrix(z.shape[0], n, _ptr(z), _ptr(M))
    return M


def dft3d_points(x: np.ndarray, points) -> np.ndarray:
    """General form of Eq. 10: X(z1_a, z2_b, z3_c) for per-axis evaluation points.

    ``points[j]`` is a 1-D complex array of points for axis j, or None for the N-th roots of
    unity.  Output shape (len(points[0]), len(points[1]), len(points[2]))."""
    x = _check_input(x)
    y = x
    for axis in (2, 1, 0):
        n = x.shape[axis]
        M = dft_matrix(n) if points[axis] is None else points_matrix(points[axis], n)
        y = mode_contract(M, y, axis)
    return y


def dft3d_adjoint(y: np.ndarray, shape=None, coords=(None, None, None), points=None) -> np.ndarray:
    """Conjugate transpose of the transform of Eq. 10 applied to ``y``:

        out[n1, n2, n3] = sum_{k1,k2,k3} conj(M1[k1,n1]) conj(M2[k2,n2]) conj(M3[k3,n3]) y[k1,k2,k3]

    with the per-axis matrices M_j of the forward transform: sample coordinates ``coords`` (square
    matrices, Eq. 3 read as in the benchmark configuration) or evaluation ``points`` (K x N matrices,
    Eq. 3 as printed; then ``shape`` gives the n_j).  One axis at a time, in fp64."""
    y = _check_input(y)
    if points is None:
        shape = y.shape
        Ms = [dft_matrix(n, coords[j]) for j, n in enumerate(shape)]
    else:
        if shape is None:
            raise ValueError("the adjoint of a point transform needs the shape of the data space")
        Ms = [dft_matrix(n) if points[j] is None else points_matrix(points[j], n) for j, n in enumerate(shape)]
    out = y
    for axis in (2, 1, 0):
        out = mode_contract(np.ascontiguousarray(Ms[axis].conj().T), out, axis)
    return out


def mode_contract(M: np.ndarray, x: np.ndarray, axis: int) -> np.ndarray:
    """``out[..., k, ...] = sum_n M[k, n] x[..., n, ...]`` along ``axis`` in fp64.

    A complex64 ``x`` is promoted element by element inside the C loop (exactly), anything
    else is converted to complex128 first."""
    M = np.ascontiguousarray(M, dtype=np.complex128)
    f32 = isinstance(x, np.ndarray) and x.dtype == np.complex64
    x = np.ascontiguousarray(x) if f32 else np.ascontiguousarray(x, dtype=np.complex128)
    axis = axis % x.ndim
    K, N = M.shape
    if x.shape[axis] != N:
        raise ValueError("matrix / tensor size mismatch")
    O = int(np.prod(x.shape[:axis], dtype=np.int64))
    I = int(np.prod(x.shape[axis + 1:], dtype=np.int64))
    out = np.empty(x.shape[:axis] + (K,) + x.shape[axis + 1:], dtype=np.complex128)
    fn = _load().oracle_mode_contract_f32 if f32 else _load().oracle_mode_contract
    fn(O, N, I, K, _ptr(M), _ptr(x), _ptr(out))
    return out


def _check_input(x):
    x = np.ascontiguousarray(x)
    if x.dtype != np.complex64 or x.ndim != 3:
        raise ValueError("oracle input must be a 3-D complex64 array")
    return x


def dft3d(x: np.ndarray, coords=(None, None, None), sign: int = FORWARD) -> np.ndarray:
    """3-D transform of a complex64 tensor, evaluated in fp64; complex128 result.

    ``sign=BACKWARD`` applies the positive exponent and the 1/(n1 n2 n3) factor and is only
    defined here for uniform axes."""
    x = _check_input(x)
    n1, n2, n3 = x.shape
    cs = [_coords(c, n) for c, n in zip(coords, x.shape)]
    if sign == BACKWARD and any(c is not None for c in cs):
        raise ValueError("backward transform is only defined for uniform axes")
    out = np.empty(x.shape, dtype=np.complex128)
    rc = _load().oracle_dft3d(n1, n2, n3, _ptr(x), _ptr(out), _ptr(cs[0]), _ptr(cs[1]),
                              _ptr(cs[2]), int(sign), 1 if sign == BACKWARD else 0)
    if rc != 0:
        raise MemoryError("oracle scratch allocation failed")
    return out


def dft3d_brute(x: np.ndarray, coords=(None, None, None), sign: int = FORWARD) -> np.ndarray:
    """Literal O(E^2) evaluation of the defining sum (unscaled).  Tiny inputs only."""
    x = _check_input(x)
    if x.size > 4096:
        raise ValueError("brute-force oracle is limited to 4096 points")
    n1, n2, n3 = x.shape
    cs = [_coords(c, n) for c, n in zip(coords, x.shape)]
    out = np.empty(x.shape, dtype=np.complex128)
    _load().oracle_dft3d_brute(n1, n2, n3, _ptr(x), _ptr(out), _ptr(cs[0]), _ptr(cs[1]),
                               _ptr(cs[2]), int(sign))
    return out


def dft3d_sampled(x: np.ndarray, k1s, coords=(None, None, None), sign: int = FORWARD,
                  slab_chunk: int = 64) -> np.ndarray:
    """Output slabs ``X[k1, :, :]`` for the frequencies ``k1s`` of a (possibly huge) tensor.

    The sum over the first index is taken with the matching rows of M1 only, streaming the
    input in chunks of ``slab_chunk`` planes so the fp64 copy stays small; modes 2 and 3 are
    then applied in full to the reduced (len(k1s), n2, n3) tensor.  Unscaled (forward use)."""
    if x.ndim != 3 or x.dtype != np.complex64:
        raise ValueError("oracle input must be a 3-D complex64 array")
    n1, n2, n3 = x.shape
    k1s = np.asarray(k1s, dtype=np.int64)
    M1 = dft_matrix(n1, coords[0], sign, ks=k1s)            # (len(k1s), n1)
    acc = np.zeros((len(k1s), n2, n3), dtype=np.complex128)
    for a0 in range(0, n1, slab_chunk):
        a1 = min(n1, a0 + slab_chunk)
        acc += mode_contract(M1[:, a0:a1], np.asarray(x[a0:a1]), axis=0)
    y = mode_contract(dft_matrix(n2, coords[1], sign), acc, axis=1)
    return mode_contract(dft_matrix(n3, coords[2], sign), y, axis=2)


def dft3d_pencils(x: np.ndarray, k2s, k3s, coords=(None, None, None), sign: int = FORWARD) -> np.ndarray:
    """Output pencils ``X[:, k2, k3]`` for every pair in ``k2s`` x ``k3s``: shape (n1, len(k2s), len(k3s)).

    Modes 3 and 2 are taken with the matching matrix rows only, mode 1 in full.  Unscaled."""
    if x.ndim != 3 or x.dtype != np.complex64:
        raise ValueError("oracle input must be a 3-D complex64 array")
    n1, n2, n3 = x.shape
    M3 = dft_matrix(n3, coords[2], sign, ks=np.asarray(k3s, dtype=np.int64))
    M2 = dft_matrix(n2, coords[1], sign, ks=np.asarray(k2s, dtype=np.int64))
    y = mode_contract(M3, x, axis=2)             # (n1, n2, |k3s|)
    y = mode_contract(M2, y, axis=1)             # (n1, |k2s|, |k3s|)
    return mode_contract(dft_matrix(n1, coords[0], sign), y, axis=0)
