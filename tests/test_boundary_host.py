"""CPU-side checks of the C-ABI library: it loads, exports what the header declares, its host
generator rounds like the fp64 oracle says it should, and argument errors come back as status
codes.  No kernel is launched here."""
import ctypes
import os
import re

import numpy as np
import pytest

import paper_2002_03260_amd as dft
from paper_2002_03260_amd import binding
from oracle import dft3d_oracle as orc

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    from paper_2002_03260_amd import build

    if build.is_stale():
        build.build()
    return dft.load_library()


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "dft3d.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(dft3d_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol(lib):
    names = declared_symbols()
    assert len(names) >= 16
    for n in names:
        assert hasattr(lib, n), n
    assert sorted(binding.EXPORTS) == names


def ulp32(x):
    return np.spacing(np.abs(x).astype(np.float32)).astype(np.float64)



def test_binding_constants_match_the_header():
    """Flags, formulations, directions and status codes of the Python binding equal the header's."""
    import re

    import paper_2002_03260_amd as dft
    from paper_2002_03260_amd import binding

    text = open(os.path.join(ROOT, "include", "dft3d.h")).read()
    flags = {m.group(1): int(m.group(2)) for m in re.finditer(r"#define\s+DFT3D_FLAG_(\w+)\s+(\d+)u", text)}
    assert flags == {"CLOBBER_INPUT": dft.FLAG_CLOBBER_INPUT, "UNFUSED": dft.FLAG_UNFUSED, "3M": dft.FLAG_3M,
                     "BF16X3": dft.FLAG_BF16X3, "COMPLEX128": dft.FLAG_COMPLEX128, "ADJOINT": dft.FLAG_ADJOINT}
    assert len(set(flags.values())) == len(flags) and all(v & (v - 1) == 0 for v in flags.values())
    enums = {m.group(1): int(m.group(2)) for m in re.finditer(r"DFT3D_(\w+)\s*=\s*(-?\d+)", text)}
    assert enums["KDFT"] == dft.KDFT and enums["FFT"] == dft.FFT
    assert enums["FORWARD"] == dft.FORWARD and enums["BACKWARD"] == dft.BACKWARD
    assert int(re.search(r"#define\s+DFT3D_MAX_PASSES\s+(\d+)", text).group(1)) == 16
    assert binding.EXPORTS == sorted(set(binding.EXPORTS)) or len(binding.EXPORTS) == len(set(binding.EXPORTS))


@pytest.mark.parametrize("n,nonuniform", [(2, False), (4, False), (8, False), (30, False), (37, False),
                                          (256, False), (2048, False), (128, True), (45, True)])
def test_generated_matrix_is_oracle_matrix_rounded_once(lib, n, nonuniform):
    c = np.sort(np.random.default_rng(n).random(n)) if nonuniform else None
    M = dft.generate_matrix(n, c)
    O = orc.dft_matrix(n, c)
    for part in (np.real, np.imag):
        err = np.abs(part(M).astype(np.float64) - part(O))
        # one rounding to fp32 of a value computed to ~1e-16 (k*c carries ~k*1e-16 for nonuniform)
        assert np.all(err <= 0.5 * ulp32(part(O)) + 1e-12)
    Mb = dft.generate_matrix(n, c, dft.BACKWARD)
    assert np.array_equal(Mb, M.conj())


@pytest.mark.parametrize("n", [4, 8, 16, 64, 12, 20])
def test_quarter_turn_entries_are_exact(lib, n):
    M = dft.generate_matrix(n)
    k, j = np.meshgrid(np.arange(n), np.arange(n), indexing="ij")
    r = (k * j) % n
    for q, val in ((0, 1), (1, -1j), (2, -1), (3, 1j)):
        if (q * n) % 4:
            continue
        mask = r == q * n // 4
        assert np.all(M[mask] == np.complex64(val))
    assert np.all(np.abs(np.abs(M.astype(np.complex128)) - 1) < 1e-7)


def test_uniform_coordinates_reproduce_uniform_matrix_bitwise(lib):
    for n in (8, 64, 512):
        assert np.array_equal(dft.generate_matrix(n, np.arange(n) / n), dft.generate_matrix(n))


def test_points_matrix_is_oracle_matrix_rounded_once(lib):
    rng = np.random.default_rng(12)
    for K, n in ((5, 9), (64, 64), (3, 300)):
        z = (0.97 + 0.06 * rng.random(K)) * np.exp(2j * np.pi * rng.random(K))
        M = dft.generate_points_matrix(z, n)
        O = orc.points_matrix(z, n)
        err = np.abs(M.astype(np.complex128) - O)
        assert np.all(err <= 0.75 * ulp32(np.abs(O)) * np.sqrt(2) + 1e-10 * np.abs(O))
    # points on the unit circle at the roots of unity reproduce the uniform matrix
    n = 32
    z = np.exp(2j * np.pi * np.arange(n) / n)
    assert np.max(np.abs(dft.generate_points_matrix(z, n) - dft.generate_matrix(n))) < 1.3e-7
    with pytest.raises(dft.Dft3dError):
        dft.generate_points_matrix(np.array([0.0 + 0.0j]), 4)          # zero point
    with pytest.raises(dft.Dft3dError):
        dft.generate_points_matrix(np.array([1e-3 + 0.0j]), 64)        # overflows fp32


def test_twiddle_table(lib):
    for A, B in ((16, 32), (32, 64), (3, 5), (1, 7), (7, 1)):
        T = dft.generate_twiddle(A, B)
        want = np.exp(-2j * np.pi * ((np.outer(np.arange(A), np.arange(B)) % (A * B)) / (A * B)))
        assert np.max(np.abs(T - want)) < 6.1e-8
        assert np.array_equal(dft.generate_twiddle(A, B, dft.BACKWARD), T.conj())
        assert np.all(T[0, :] == 1) and np.all(T[:, 0] == 1)


def test_argument_errors_are_status_codes(lib):
    h = ctypes.c_void_p()
    st = lib.dft3d_plan_create(ctypes.byref(h), 0, 4, 4, dft.KDFT, None, None, None)
    assert lib.dft3d_status_string(st) == b"DFT3D_ERR_INVALID_ARG" and not h
    assert b"axis 0" in lib.dft3d_last_error()
    st = lib.dft3d_plan_create(None, 4, 4, 4, dft.KDFT, None, None, None)
    assert lib.dft3d_status_string(st) == b"DFT3D_ERR_INVALID_ARG"
    st = lib.dft3d_plan_create(ctypes.byref(h), 4, 4, 4, 7, None, None, None)
    assert lib.dft3d_status_string(st) == b"DFT3D_ERR_INVALID_ARG"
    c = (ctypes.c_double * 4)(0.0, 0.1, 0.2, 0.3)
    st = lib.dft3d_plan_create(ctypes.byref(h), 4, 4, 4, dft.FFT, ctypes.cast(c, ctypes.c_void_p), None, None)
    assert lib.dft3d_status_string(st) == b"DFT3D_ERR_UNSUPPORTED" and not h
    st = lib.dft3d_plan_create_ex(ctypes.byref(h), 4, 4, 4, dft.KDFT, None, None, None, None, 0x80)
    assert lib.dft3d_status_string(st) == b"DFT3D_ERR_INVALID_ARG"
    # NULL plans
    assert lib.dft3d_plan_destroy(None) == 0
    assert lib.dft3d_plan_workspace_bytes(None) == 0
    st = lib.dft3d_exec(None, None, None, dft.FORWARD, None)
    assert lib.dft3d_status_string(st) == b"DFT3D_ERR_INVALID_ARG"
    st = lib.dft3d_generate_matrix(0, None, dft.FORWARD, None, None)
    assert lib.dft3d_status_string(st) == b"DFT3D_ERR_INVALID_ARG"
    assert lib.dft3d_status_string(99) == b"DFT3D_ERR_UNKNOWN"


def test_axis_order_query_rejects_null(lib):
    """The plan query for the order of the passes is host code: NULL arguments come back as a status."""
    order = (ctypes.c_int * 3)()
    st = lib.dft3d_plan_axis_order(None, order)
    assert lib.dft3d_status_string(st) == b"DFT3D_ERR_INVALID_ARG"


def test_plan_arguments_rejected_before_any_device_work(lib):
    """Non-finite coordinates, contraction variants on an FFT plan and extents the kernels cannot
    index come back as status codes from checks that run before the first device call."""
    h = ctypes.c_void_p()
    for bad in (float("nan"), float("inf"), -float("inf")):
        c = (ctypes.c_double * 4)(0.0, 0.1, bad, 0.3)
        st = lib.dft3d_plan_create(ctypes.byref(h), 4, 4, 4, dft.KDFT, None, ctypes.cast(c, ctypes.c_void_p), None)
        assert lib.dft3d_status_string(st) == b"DFT3D_ERR_INVALID_ARG" and not h
        assert b"not finite" in lib.dft3d_last_error()
        re = np.empty((4, 4), np.float32)
        im = np.empty((4, 4), np.float32)
        st = lib.dft3d_generate_matrix(4, ctypes.cast(c, ctypes.c_void_p), dft.FORWARD,
                                       re.ctypes.data_as(ctypes.c_void_p), im.ctypes.data_as(ctypes.c_void_p))
        assert lib.dft3d_status_string(st) == b"DFT3D_ERR_INVALID_ARG"
    for fl in (dft.FLAG_3M, dft.FLAG_BF16X3, dft.FLAG_3M | dft.FLAG_BF16X3):
        st = lib.dft3d_plan_create_ex(ctypes.byref(h), 8, 8, 8, dft.FFT, None, None, None, None, fl)
        assert lib.dft3d_status_string(st) == b"DFT3D_ERR_UNSUPPORTED" and not h
    # ny*nz (and nx*ny) are 32-bit quantities inside the kernels
    st = lib.dft3d_plan_create(ctypes.byref(h), 1, 1 << 16, 1 << 15, dft.KDFT, None, None, None)
    assert lib.dft3d_status_string(st) == b"DFT3D_ERR_UNSUPPORTED" and not h
    assert b"2^31" in lib.dft3d_last_error()
    st = lib.dft3d_plan_create(ctypes.byref(h), 1 << 16, 1 << 15, 1, dft.FFT, None, None, None)
    assert lib.dft3d_status_string(st) == b"DFT3D_ERR_UNSUPPORTED" and not h
    st = lib.dft3d_plan_create(ctypes.byref(h), (1 << 24) + 1, 1, 1, dft.FFT, None, None, None)
    assert lib.dft3d_status_string(st) == b"DFT3D_ERR_INVALID_ARG" and not h
    # the entry point that allocates nothing validates like exec
    st = lib.dft3d_exec_noalloc(None, None, None, dft.FORWARD, None)
    assert lib.dft3d_status_string(st) == b"DFT3D_ERR_INVALID_ARG"


def test_a_matrix_too_large_for_the_host_is_a_status_code_not_an_abort(lib):
    """A KDFT axis of 2^24 points needs a 2^48-entry matrix: the failed host allocation must come
    back as DFT3D_ERR_ALLOC (no C++ exception may cross the C boundary)."""
    h = ctypes.c_void_p()
    st = lib.dft3d_plan_create(ctypes.byref(h), 1 << 24, 1, 1, dft.KDFT, None, None, None)
    assert lib.dft3d_status_string(st) == b"DFT3D_ERR_ALLOC" and not h
    assert b"memory" in lib.dft3d_last_error()
    st = lib.dft3d_plan_create_points(ctypes.byref(h), 1 << 24, 1, 1, 1 << 24, 1, 1, None, None, None, 0)
    assert lib.dft3d_status_string(st) == b"DFT3D_ERR_ALLOC" and not h


def test_plan_creation_without_a_gpu_fails_loudly(lib):
    import torch

    if torch.cuda.is_available():
        pytest.skip("a GPU is present")
    with pytest.raises(dft.Dft3dError) as ei:
        dft.Plan((8, 8, 8), dft.KDFT)
    assert ei.value.status_name in ("DFT3D_ERR_ALLOC", "DFT3D_ERR_HIP")
