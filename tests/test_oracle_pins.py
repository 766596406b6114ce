"""Pins for the CPU oracle: it is checked against things other than itself.

The paper prints no worked numeric example, so the pins are what the mathematics fixes:
brute force on tiny inputs (Eq. 10 literally), closed forms, invariants, special cases that
reduce to a library routine (numpy's pocketfft, numpy einsum) and exact small matrices.
"""
import os

import numpy as np
import pytest

from oracle import dft3d_oracle as orc
from oracle import fft_formulation as ff
import dft3d_workloads as wl

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def rel_l2(a, b):
    return np.linalg.norm((a - b).ravel()) / max(np.linalg.norm(b.ravel()), 1e-300)


def rand_c64(shape, seed):
    return wl.draw_complex(shape, "normal", seed)


# --------------------------------------------------------------------------- P7: exact matrices
def _read_golden_matrices():
    mats = {}
    with open(os.path.join(GOLDEN, "dft_small_matrices.txt")) as f:
        lines = [ln.strip() for ln in f if ln.strip() and not ln.startswith("#")]
    i = 0
    while i < len(lines):
        n = int(lines[i]); i += 1
        rows = []
        for _ in range(n):
            rows.append([complex(*map(float, p.split(","))) for p in lines[i].split()]); i += 1
        mats[n] = np.array(rows)
    return mats


def test_small_matrices_match_textbook_values():
    for n, G in _read_golden_matrices().items():
        M = orc.dft_matrix(n)
        assert np.max(np.abs(M - G)) < 1e-15, n
        # backward matrix is the conjugate
        assert np.max(np.abs(orc.dft_matrix(n, sign=orc.BACKWARD) - G.conj())) < 1e-15


def test_matrix_is_vandermonde_in_row_points():
    # Eq. 3: row k is 1, z_k^-1, z_k^-2, ... : consecutive entries have a constant ratio
    for n, coords in ((12, None), (9, np.sort(np.random.default_rng(3).random(9)))):
        M = orc.dft_matrix(n, coords)
        assert np.allclose(np.abs(M), 1.0, atol=1e-15)
        if coords is None:
            ratio = M[:, 1:] / M[:, :-1]
            assert np.allclose(ratio, ratio[:, :1], atol=1e-13)
            assert np.allclose(M[:, 0], 1.0)
        else:
            # nonuniform reading: column n is geometric in the integer frequency k
            ratio = M[1:, :] / M[:-1, :]
            assert np.allclose(ratio, ratio[:1, :], atol=1e-12)
            assert np.allclose(M[0, :], 1.0)


def test_uniform_matrix_unitary_up_to_scale():
    # Section III-A: with uniform sampling the matrix holds roots of unity; V V^H = N I
    for n in (5, 8, 30):
        M = orc.dft_matrix(n)
        assert np.allclose(M @ M.conj().T, n * np.eye(n), atol=1e-11)


def test_matrix_rows_subset():
    n = 20
    ks = [0, 3, 19, 7]
    c = np.sort(np.random.default_rng(5).random(n))
    for coords in (None, c):
        full = orc.dft_matrix(n, coords)
        assert np.array_equal(orc.dft_matrix(n, coords, ks=ks), full[ks])


# --------------------------------------------------------------------------- mode product
@pytest.mark.parametrize("shape,axis,K", [((3, 5, 4), 0, 3), ((3, 5, 4), 1, 7), ((3, 5, 4), 2, 2),
                                          ((1, 6, 1), 1, 6), ((2, 1, 3), 1, 4)])
def test_mode_contract_matches_einsum(shape, axis, K):
    rng = np.random.default_rng(11)
    x = rng.standard_normal(shape) + 1j * rng.standard_normal(shape)
    M = rng.standard_normal((K, shape[axis])) + 1j * rng.standard_normal((K, shape[axis]))
    got = orc.mode_contract(M, x, axis)
    sub = ["kn,nbc->kbc", "kn,anc->akc", "kn,abn->abk"][axis]
    want = np.einsum(sub, M, x)
    assert got.shape == want.shape
    assert rel_l2(got, want) < 1e-14


# --------------------------------------------------------------------------- P1: brute force
@pytest.mark.parametrize("shape", [(4, 4, 4), (3, 4, 5), (1, 7, 2), (5, 1, 1)])
@pytest.mark.parametrize("nonuniform", [(False, False, False), (True, True, True),
                                        (False, True, False)])
def test_per_axis_matches_brute_force(shape, nonuniform):
    x = rand_c64(shape, 101 + sum(shape))
    rng = np.random.default_rng(7)
    coords = tuple(np.sort(rng.random(n)) if nu else None for n, nu in zip(shape, nonuniform))
    a = orc.dft3d(x, coords)
    b = orc.dft3d_brute(x, coords)
    assert rel_l2(a, b) < 1e-13


def test_brute_force_backward_sign():
    x = rand_c64((3, 4, 2), 5)
    a = orc.dft3d(x, sign=orc.BACKWARD) * x.size       # undo the 1/E scaling
    b = orc.dft3d_brute(x, sign=orc.BACKWARD)
    assert rel_l2(a, b) < 1e-13


# --------------------------------------------------------------------------- P2: closed forms
def test_delta_at_origin_gives_ones():
    x = np.zeros((6, 5, 8), np.complex64); x[0, 0, 0] = 1
    assert np.max(np.abs(orc.dft3d(x) - 1.0)) < 1e-14


def test_shifted_delta_gives_plane_wave():
    shape = (6, 5, 8); a, b, c = 2, 4, 3
    x = np.zeros(shape, np.complex64); x[a, b, c] = 1
    k1, k2, k3 = np.meshgrid(*[np.arange(n) for n in shape], indexing="ij")
    want = np.exp(-2j * np.pi * (a * k1 / shape[0] + b * k2 / shape[1] + c * k3 / shape[2]))
    assert np.max(np.abs(orc.dft3d(x) - want)) < 1e-13


def test_single_exponential_gives_one_bin():
    shape = (8, 4, 16); f = (3, 1, 11)
    n1, n2, n3 = np.meshgrid(*[np.arange(n) for n in shape], indexing="ij")
    x = np.exp(2j * np.pi * (f[0] * n1 / shape[0] + f[1] * n2 / shape[1] + f[2] * n3 / shape[2]))
    x = x.astype(np.complex64)
    X = orc.dft3d(x)
    E = np.prod(shape)
    assert abs(X[f] - E) < 1e-4 * E            # input was rounded to fp32
    X[f] = 0
    assert np.max(np.abs(X)) < 1e-4 * E
    # exactly representable case: all-ones input -> E at bin 0, 0 elsewhere
    X1 = orc.dft3d(np.ones(shape, np.complex64))
    assert abs(X1[0, 0, 0] - E) < 1e-10
    X1[0, 0, 0] = 0
    assert np.max(np.abs(X1)) < 1e-10


# --------------------------------------------------------------------------- P3: separable
def test_separable_input():
    shape = (7, 9, 6)
    rng = np.random.default_rng(21)
    coords = (None, np.sort(rng.random(9)), None)
    a, b, c = [wl.draw_complex((n,), "uniform", 30 + i) for i, n in enumerate(shape)]
    x = np.einsum("a,b,c->abc", a, b, c).astype(np.complex64)
    # the 1-D factors as they were actually rounded into x are not recoverable, so compare
    # with the transform of the exactly-separable fp64 tensor within the fp32 rounding of x
    Ma, Mb, Mc = [orc.dft_matrix(n, cc) for n, cc in zip(shape, coords)]
    want = np.einsum("a,b,c->abc", Ma @ a.astype(complex), Mb @ b.astype(complex),
                     Mc @ c.astype(complex))
    got = orc.dft3d(x, coords)
    assert rel_l2(got, want) < 5e-7


# --------------------------------------------------------------------------- P4: invariants
def test_linearity():
    shape = (5, 6, 4)
    # small integer parts and power-of-two scalars: the combination is exact in fp32
    x, y = wl.gaussian_integers(shape, 1), wl.gaussian_integers(shape, 2)
    z64 = 2 * x.astype(np.complex128) + 0.5j * y.astype(np.complex128)
    z = z64.astype(np.complex64)
    assert np.array_equal(z.astype(np.complex128), z64)
    assert rel_l2(orc.dft3d(z), 2 * orc.dft3d(x) + 0.5j * orc.dft3d(y)) < 1e-14


def test_parseval_uniform():
    x = rand_c64((8, 6, 10), 3)
    X = orc.dft3d(x)
    lhs = np.sum(np.abs(X) ** 2)
    rhs = x.size * np.sum(np.abs(x.astype(np.complex128)) ** 2)
    assert abs(lhs - rhs) < 1e-12 * rhs


def test_forward_backward_roundtrip():
    x = rand_c64((4, 6, 8), 4)
    X = orc.dft3d(x)
    # the oracle takes complex64 input; X is not representable, so invert with matrices
    y = X
    for ax, n in enumerate(x.shape):
        y = orc.mode_contract(orc.dft_matrix(n, sign=orc.BACKWARD), y, ax)
    y /= x.size
    assert rel_l2(y, x.astype(np.complex128)) < 1e-14
    # and the packaged backward transform agrees with numpy's ifftn convention
    assert rel_l2(orc.dft3d(x, sign=orc.BACKWARD), np.fft.ifftn(x.astype(np.complex128))) < 1e-13


def test_mode_order_independence():
    x = rand_c64((5, 4, 6), 8).astype(np.complex128)
    Ms = [orc.dft_matrix(n) for n in x.shape]
    a = x
    for ax in (2, 0, 1):
        a = orc.mode_contract(Ms[ax], a, ax)
    assert rel_l2(a, orc.dft3d(x.astype(np.complex64))) < 1e-14


def test_nonuniform_on_uniform_grid_equals_uniform():
    shape = (8, 16, 4)
    x = rand_c64(shape, 9)
    coords = tuple(np.arange(n) / n for n in shape)
    assert np.array_equal(orc.dft3d(x, coords), orc.dft3d(x))
    # non-power-of-two: n/N is rounded, agreement to rounding only
    shape = (6, 5, 7)
    x = rand_c64(shape, 10)
    coords = tuple(np.arange(n) / n for n in shape)
    assert rel_l2(orc.dft3d(x, coords), orc.dft3d(x)) < 1e-14


# --------------------------------------------------------------------------- P5: library routine
@pytest.mark.parametrize("shape", [(8, 8, 8), (6, 10, 15), (32, 32, 32), (1, 1, 9), (64, 3, 48)])
def test_matches_numpy_fftn(shape):
    x = rand_c64(shape, 40 + shape[0])
    want = np.fft.fftn(x.astype(np.complex128))
    assert rel_l2(orc.dft3d(x), want) < 1e-12


@pytest.mark.parametrize("shape", [(6, 10, 15), (16, 16, 16), (1, 12, 40)])
def test_mode_products_on_a_complex128_tensor_match_numpy_fftn(shape):
    """The composition the complex128 parity tests use as their oracle (matrix per axis, modes
    z, y, x on a full-precision complex128 tensor), pinned to the library FFT in both directions."""
    rng = np.random.default_rng(77 + shape[1])
    x = rng.standard_normal(shape) + 1j * rng.standard_normal(shape)
    for sign, want in ((orc.FORWARD, np.fft.fftn(x)), (orc.BACKWARD, np.fft.ifftn(x) * x.size)):
        y = x
        for axis in (2, 1, 0):
            y = orc.mode_contract(orc.dft_matrix(shape[axis], None, sign), y, axis)
        assert rel_l2(y, want) < 1e-13


# --------------------------------------------------------------------------- P6: nonuniform closed forms
def test_nonuniform_delta_dirichlet_sum():
    n = 16
    rng = np.random.default_rng(77)
    c = np.sort(rng.random(n))
    j = 5
    x = np.zeros((1, 1, n), np.complex64); x[0, 0, j] = 1
    X = orc.dft3d(x, (None, None, c))[0, 0]
    # column j of the matrix: geometric sequence in k with ratio exp(-2 pi i c_j)
    q = np.exp(-2j * np.pi * c[j])
    assert abs(X[0] - 1) < 1e-15
    assert np.allclose(X[1:] / X[:-1], q, atol=1e-13)
    assert abs(X.sum() - (1 - q ** n) / (1 - q)) < 1e-12


def test_nonuniform_shifted_grid_is_modulated_fft():
    # samples at (n + s)/N: X[k] = exp(-2 pi i k s / N) * FFT(x)[k]
    n, s = 12, 0.3
    x = rand_c64((1, n, 1), 12)
    c = (np.arange(n) + s) / n
    X = orc.dft3d(x, (None, c, None))[0, :, 0]
    want = np.exp(-2j * np.pi * np.arange(n) * s / n) * np.fft.fft(x[0, :, 0].astype(complex))
    assert rel_l2(X, want) < 1e-13


def test_nonuniform_axis_is_not_transposed():
    # two samples at distinct coordinates: X[k] = x0 e^{-2 pi i k c0} + x1 e^{-2 pi i k c1};
    # a transposed matrix would put the coordinate on the output index instead.
    c = np.array([0.125, 0.5])
    x = np.array([1.0, 2.0], np.complex64).reshape(2, 1, 1)
    X = orc.dft3d(x, (c, None, None))[:, 0, 0]
    assert np.allclose(X, [3.0, np.exp(-2j * np.pi * 0.125) + 2 * np.exp(-2j * np.pi * 0.5)])


# --------------------------------------------------------------------------- arbitrary evaluation points (Eq. 1-3 as written)
def test_points_matrix_is_polynomial_evaluation():
    # X(z_k) = sum_n x_n z_k^{-n} is the polynomial with coefficients x_n evaluated at 1/z_k
    rng = np.random.default_rng(8)
    n, K = 11, 7
    z = (0.8 + 0.4 * rng.random(K)) * np.exp(2j * np.pi * rng.random(K))      # off the unit circle
    x = rng.standard_normal(n) + 1j * rng.standard_normal(n)
    M = orc.points_matrix(z, n)
    want = np.polyval(x[::-1], 1.0 / z)
    assert np.allclose(M @ x, want, rtol=1e-12, atol=1e-12)
    assert np.allclose(M[:, 0], 1.0)
    assert np.allclose(M[:, 1:] / M[:, :-1], (1.0 / z)[:, None], rtol=1e-12)


def test_points_on_roots_of_unity_reproduce_the_uniform_transform():
    shape = (6, 8, 5)
    x = rand_c64(shape, 19)
    pts = tuple(np.exp(2j * np.pi * np.arange(n) / n) for n in shape)
    assert rel_l2(orc.dft3d_points(x, pts), orc.dft3d(x)) < 1e-13
    assert rel_l2(orc.dft3d_points(x, (None, pts[1], None)), orc.dft3d(x)) < 1e-13


def test_points_rectangular_output_matches_brute_polynomial():
    shape = (3, 4, 5)
    rng = np.random.default_rng(9)
    x = rand_c64(shape, 20)
    pts = [0.9 * np.exp(2j * np.pi * rng.random(k)) for k in (2, 6, 4)]
    X = orc.dft3d_points(x, pts)
    assert X.shape == (2, 6, 4)
    xc = x.astype(np.complex128)
    for a, za in enumerate(pts[0]):
        for b, zb in enumerate(pts[1]):
            for c, zc in enumerate(pts[2]):
                w = (za ** -np.arange(3))[:, None, None] * (zb ** -np.arange(4))[None, :, None] * \
                    (zc ** -np.arange(5))[None, None, :]
                assert abs(X[a, b, c] - np.sum(xc * w)) < 1e-12 * np.sum(np.abs(xc * w))


# --------------------------------------------------------------------------- adjoint
def test_adjoint_on_uniform_axes_is_unscaled_inverse_fft():
    """On uniform axes M^H = conj(M): the adjoint is numpy's ifftn times the number of points."""
    shape = (6, 10, 7)
    y = rand_c64(shape, 23)
    ref = np.fft.ifftn(y.astype(np.complex128)) * np.prod(shape)
    assert rel_l2(orc.dft3d_adjoint(y), ref) < 1e-13


def test_adjoint_satisfies_the_inner_product_identity():
    """<A x, y> = <x, A^H y> with A the (pinned) forward transform: nonuniform coordinates, and
    rectangular point matrices off the unit circle.  A transposed index, a missing conjugate or a
    wrong axis order breaks the identity."""
    rng = np.random.default_rng(12)
    shape = (5, 6, 4)
    coords = tuple(np.sort(rng.random(n)) for n in shape)
    x, y = rand_c64(shape, 24), rand_c64(shape, 25)
    lhs = np.vdot(y.astype(np.complex128), orc.dft3d(x, coords))          # <y, A x>
    rhs = np.vdot(orc.dft3d_adjoint(y, coords=coords), x.astype(np.complex128))
    assert abs(lhs - rhs) < 1e-12 * abs(lhs)

    pts = [0.95 * np.exp(2j * np.pi * rng.random(k)) for k in (3, 7, 6)]
    yk = rand_c64((3, 7, 6), 26)
    lhs = np.vdot(yk.astype(np.complex128), orc.dft3d_points(x, pts))
    back = orc.dft3d_adjoint(yk, shape=shape, points=pts)
    assert back.shape == shape
    rhs = np.vdot(back, x.astype(np.complex128))
    assert abs(lhs - rhs) < 1e-12 * abs(lhs)


def test_adjoint_of_a_single_frequency_is_the_conjugate_matrix_row():
    """y = delta at frequency (a, b, c) -> out[n] = conj(M1[a,n1]) conj(M2[b,n2]) conj(M3[c,n3]),
    written out from the definition M[k, n] = exp(-2 pi i k c[n])."""
    rng = np.random.default_rng(13)
    shape = (4, 5, 6)
    coords = tuple(np.sort(rng.random(n)) for n in shape)
    y = np.zeros(shape, np.complex64)
    a, b, c = 3, 1, 4
    y[a, b, c] = 1.0
    want = np.exp(2j * np.pi * a * coords[0])[:, None, None] * np.exp(2j * np.pi * b * coords[1])[None, :, None] * \
        np.exp(2j * np.pi * c * coords[2])[None, None, :]
    assert np.max(np.abs(orc.dft3d_adjoint(y, coords=coords) - want)) < 1e-13


# --------------------------------------------------------------------------- sampled slabs
def test_sampled_slabs_equal_full():
    shape = (10, 6, 7)
    x = rand_c64(shape, 13)
    rng = np.random.default_rng(2)
    coords = (np.sort(rng.random(10)), None, np.sort(rng.random(7)))
    full = orc.dft3d(x, coords)
    ks = [0, 9, 4]
    got = orc.dft3d_sampled(x, ks, coords, slab_chunk=3)
    assert rel_l2(got, full[ks]) < 1e-14


def test_pencils_equal_full():
    shape = (9, 6, 7)
    x = rand_c64(shape, 14)
    rng = np.random.default_rng(4)
    coords = (None, np.sort(rng.random(6)), np.sort(rng.random(7)))
    full = orc.dft3d(x, coords)
    k2s, k3s = [5, 0], [3, 6, 1]
    got = orc.dft3d_pencils(x, k2s, k3s, coords)
    assert rel_l2(got, full[:, k2s][:, :, k3s]) < 1e-14


def test_mode_contract_complex64_input_is_promoted_exactly():
    x = rand_c64((4, 3000, 2), 15)
    M = orc.dft_matrix(3000, ks=[1, 7])
    assert np.array_equal(orc.mode_contract(M, x, 1), orc.mode_contract(M, x.astype(np.complex128), 1))


# --------------------------------------------------------------------------- FFT formulation (Eq. 12-16)
@pytest.mark.parametrize("N,A,B", [(8, 2, 4), (8, 4, 2), (16, 4, 4), (15, 3, 5), (15, 5, 3),
                                   (32, 4, 8), (12, 1, 12), (12, 12, 1)])
def test_fft_axis_factored_literal_and_library_agree(N, A, B):
    rng = np.random.default_rng(N * 100 + A)
    x = rng.standard_normal((3, N, 2)) + 1j * rng.standard_normal((3, N, 2))
    want = np.fft.fft(x, axis=1)
    assert rel_l2(ff.fft_axis_literal(x, 1, A, B), want) < 1e-13
    assert rel_l2(ff.fft_axis(x, 1, A, B), want) < 1e-13
    wantb = np.fft.ifft(x, axis=1) * N
    assert rel_l2(ff.fft_axis(x, 1, A, B, sign=ff.BACKWARD), wantb) < 1e-13
    assert rel_l2(ff.fft_axis_literal(x, 1, A, B, sign=ff.BACKWARD), wantb) < 1e-13


def test_local_transform_is_periodic_subsequence_dft():
    # Eq. 16: for each beta, the A-point transform of the stride-B subsequence
    N, A, B = 24, 4, 6
    rng = np.random.default_rng(6)
    x = rng.standard_normal(N) + 1j * rng.standard_normal(N)
    xt = ff.local_transform(x, 0, A, B).reshape(A, B)
    for beta in range(B):
        assert np.allclose(xt[:, beta], np.fft.fft(x[beta::B]), atol=1e-13)


def test_fft_steps_on_each_axis_and_3d():
    shape = (8, 12, 16)
    splits = ((2, 4), (3, 4), (4, 4))
    x = rand_c64(shape, 17)
    X = orc.dft3d(x)
    assert rel_l2(ff.fft3d(x, splits), X) < 1e-13
    assert rel_l2(ff.fft3d(x, splits, sign=ff.BACKWARD), orc.dft3d(x, sign=orc.BACKWARD)) < 1e-13
    for ax, (A, B) in enumerate(splits):
        want = np.fft.fft(x.astype(np.complex128), axis=ax)
        assert rel_l2(ff.fft_axis(x, ax, A, B), want) < 1e-13


def test_reorder_places_ka_plus_A_kb():
    A, B = 3, 4
    w = np.arange(A * B).astype(np.complex128)      # slot k_a*B + k_b holds that number
    out = ff.reorder(w, 0, A, B)
    for ka in range(A):
        for kb in range(B):
            assert out[ka + A * kb] == ka * B + kb


# --------------------------------------------------------------------------- planted mistakes are caught
def test_pins_would_catch_a_sign_or_transpose_error():
    # sanity of the pins themselves: a conjugated or transposed matrix fails them
    n = 8
    c = np.sort(np.random.default_rng(1).random(n))
    M = orc.dft_matrix(n, c)
    x = rand_c64((1, 1, n), 3)
    good = orc.dft3d(x, (None, None, c))[0, 0]
    assert rel_l2(M @ x[0, 0].astype(complex), good) < 1e-14
    assert rel_l2(M.T @ x[0, 0].astype(complex), good) > 1e-2
    assert rel_l2(M.conj() @ x[0, 0].astype(complex), good) > 1e-2
