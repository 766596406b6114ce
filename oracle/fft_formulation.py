"""fp64 CPU statement of the paper's FFT formulation, step by step.  TEST INFRASTRUCTURE ONLY.

Paper, Section III-B.  With the global index split  n = P*l + beta  (Eq. 13; l = 0..N/P-1,
beta = 0..P-1) the uniform N-point transform of Eq. 12 becomes (Eq. 14 / Eq. 15)

    X_k = sum_beta exp(-2 pi i beta k / N) * Xt_k(beta),
    Xt_k(beta) = sum_l x[P*l + beta] exp(-2 pi i l k / (N/P))                      (Eq. 16)

Xt is an (N/P)-point transform ("local transform"), periodic in k with period N/P; the outer
sum is the "phase adjustment".  Notation used in this repository:  B = P (number of beta
values, second-stage length),  A = N/P (first-stage length),  k = k_a + A*k_b.

Two evaluations of the phase adjustment are given:

* :func:`phase_adjust_literal` -- the outer sum of Eq. 15 exactly as written, with the N x P
  matrix of phase shifts exp(-2 pi i beta k / N);
* the factored steps the GPU kernels execute, which use
  exp(-2 pi i beta k / N) = exp(-2 pi i beta k_a / N) * exp(-2 pi i beta k_b / B):
  :func:`twiddle` (f1's elementwise factor), :func:`second_stage` (f2, a B-point transform
  over beta) and :func:`reorder` (f3, k = k_a + A*k_b placed in order).

All functions act along one axis of an n-D complex array, in complex128, with numpy's
``einsum`` / elementwise ops as the only primitives.  ``sign`` = -1 forward, +1 backward
(backward here is unscaled; the 3-D wrapper applies 1/(N1 N2 N3) once at the end).
Nothing here imports or is imported by the HIP library.
"""
from __future__ import annotations

import numpy as np

FORWARD = -1
BACKWARD = +1


def _split_view(x, axis, A, B):
    """View ``axis`` (length A*B) as two axes [A][B], slow index first."""
    x = np.asarray(x, dtype=np.complex128)
    axis = axis % x.ndim
    if x.shape[axis] != A * B:
        raise ValueError("axis length must equal A*B")
    return x.reshape(x.shape[:axis] + (A, B) + x.shape[axis + 1:]), axis


def _merge_view(y, axis):
    return y.reshape(y.shape[:axis] + (y.shape[axis] * y.shape[axis + 1],) + y.shape[axis + 2:])


def _root_table(rows, cols, period, sign):
    """exp(sign * 2 pi i * (r*c mod period) / period), r < rows, c < cols; integer reduction."""
    r = np.arange(rows, dtype=np.int64)[:, None]
    c = np.arange(cols, dtype=np.int64)[None, :]
    return np.exp(sign * 2j * np.pi * (((r * c) % period).astype(np.float64) / period))


def local_transform(x, axis, A, B, sign=FORWARD):
    """Eq. 16: Xt[k_a, beta] = sum_l x[B*l + beta] exp(sign 2 pi i l k_a / A); slots [k_a][beta]."""
    v, axis = _split_view(x, axis, A, B)                 # [.., l, beta, ..]
    FA = _root_table(A, A, A, sign)                      # [k_a, l]
    y = np.moveaxis(np.tensordot(FA, v, axes=([1], [axis])), 0, axis)
    return _merge_view(y, axis)


def phase_adjust_literal(xt, axis, A, B, sign=FORWARD):
    """Outer sum of Eq. 15 as written: X[k] = sum_beta exp(sign 2 pi i beta k / N) Xt[k mod A, beta].

    Input slots [k_a][beta]; output is in natural order k = 0..N-1."""
    N = A * B
    v, axis = _split_view(xt, axis, A, B)                # [.., k_a, beta, ..]
    v = np.moveaxis(v, (axis, axis + 1), (0, 1))         # [k_a, beta, rest..]
    phi = _root_table(N, B, N, sign)                     # [k, beta]
    out = np.empty((N,) + v.shape[2:], dtype=np.complex128)
    for k in range(N):
        out[k] = np.tensordot(phi[k], v[k % A], axes=([0], [0]))
    return np.moveaxis(out, 0, axis)


def twiddle(xt, axis, A, B, sign=FORWARD):
    """Elementwise factor of step f1: Z[k_a, beta] = exp(sign 2 pi i beta k_a / N) Xt[k_a, beta]."""
    v, axis = _split_view(xt, axis, A, B)
    T = _root_table(A, B, A * B, sign)                   # [k_a, beta]
    shape = [1] * v.ndim
    shape[axis], shape[axis + 1] = A, B
    return _merge_view(v * T.reshape(shape), axis)


def first_stage(x, axis, A, B, sign=FORWARD):
    """Step f1: the A-point local transform followed by the twiddle factor."""
    return twiddle(local_transform(x, axis, A, B, sign), axis, A, B, sign)


def second_stage(z, axis, A, B, sign=FORWARD):
    """Step f2: W[k_a, k_b] = sum_beta exp(sign 2 pi i beta k_b / B) Z[k_a, beta]; slots [k_a][k_b]."""
    v, axis = _split_view(z, axis, A, B)
    FB = _root_table(B, B, B, sign)                      # [k_b, beta]
    y = np.moveaxis(np.tensordot(FB, v, axes=([1], [axis + 1])), 0, axis + 1)
    return _merge_view(y, axis)


def reorder(w, axis, A, B):
    """Step f3: slots [k_a][k_b] -> natural order k = k_a + A*k_b, i.e. slots [k_b][k_a]."""
    v, axis = _split_view(w, axis, A, B)
    return _merge_view(np.swapaxes(v, axis, axis + 1), axis)


def fft_axis(x, axis, A, B, sign=FORWARD):
    """One axis of the FFT formulation via the factored steps f1, f2, f3 (unscaled)."""
    return reorder(second_stage(first_stage(x, axis, A, B, sign), axis, A, B, sign), axis, A, B)


def fft_axis_literal(x, axis, A, B, sign=FORWARD):
    """One axis via Eq. 16 then the outer sum of Eq. 15 as written (unscaled)."""
    return phase_adjust_literal(local_transform(x, axis, A, B, sign), axis, A, B, sign)


def fft3d(x, splits, sign=FORWARD):
    """3-D transform by repeating the 1-D scheme along each axis (end of Section III-B).

    ``splits`` = ((A1, B1), (A2, B2), (A3, B3)).  Backward is scaled by 1/(N1 N2 N3)."""
    y = np.asarray(x, dtype=np.complex128)
    for axis, (A, B) in enumerate(splits):
        y = fft_axis(y, axis, A, B, sign)
    if sign == BACKWARD:
        y = y / y.size
    return y
