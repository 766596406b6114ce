"""GPU parity: the HIP path, called through the C ABI, against the fp64 CPU oracle.

Bar (relative L2 error in fp64, complex64 arithmetic on the GPU): <= 2e-5 for every transform
and every single step; bit-exact where all arithmetic is exact in fp32 (N in {2, 4} with small
Gaussian-integer inputs).  Next to the relative L2 distance every comparison asserts an
element-wise bound: max|err| <= 1e-4 * rms|ref| (5 to 50 times what the fp32 paths measure).
"""
import sys

import numpy as np
import pytest

import dft3d_workloads as wl
from oracle import dft3d_oracle as orc
from oracle import fft_formulation as ff

pytestmark = pytest.mark.gpu

TOL = 2e-5


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def rel_l2(got, want):
    got = np.asarray(got, dtype=np.complex128)
    d = np.linalg.norm((got - want).ravel())
    return d / max(np.linalg.norm(want.ravel()), 1e-300)


ELEMENTWISE = 1e-4     # bound on max|err| / rms|ref|


def report(name, got, want):
    got = np.asarray(got, dtype=np.complex128)
    r = rel_l2(got, want)
    m = np.max(np.abs(got - want)) if got.size else 0.0
    rms = np.sqrt(np.mean(np.abs(want) ** 2)) if got.size else 0.0
    say(f"[parity] {name}: relL2={r:.3e} max|err|={m:.3e} rms|ref|={rms:.3e} max|ref|={np.max(np.abs(want)):.3e}")
    assert m <= ELEMENTWISE * rms + 1e-300, f"{name}: max|err| {m:.3e} exceeds {ELEMENTWISE:g} * rms|ref| {rms:.3e}"
    return r


@pytest.fixture(scope="module")
def dft(gpu_device):
    import paper_2002_03260_amd as d

    d.load_library()
    return d


def to_dev(x):
    import torch

    return torch.from_numpy(np.ascontiguousarray(x)).to("cuda")


def to_host(t):
    import torch

    torch.cuda.synchronize()
    return t.cpu().numpy()


# ------------------------------------------------------------------------------------ KDFT
KDFT_SHAPES = [(4, 4, 4), (5, 7, 3), (1, 1, 9), (9, 1, 1), (17, 33, 20), (32, 32, 32),
               (64, 48, 80), (130, 20, 258), (24, 200, 36), (16, 64, 48), (3, 32, 16), (64, 16, 144),
               (128, 192, 64), (320, 64, 128)]


@pytest.mark.parametrize("shape", KDFT_SHAPES)
def test_kdft_uniform_matches_oracle(dft, shape):
    say(f"case kdft uniform {shape}")
    x = wl.draw_complex(shape, "normal", 1000 + sum(shape))
    want = orc.dft3d(x)
    with dft.Plan(shape, dft.KDFT) as p:
        got = to_host(p.exec(to_dev(x)))
    assert report(f"kdft {shape}", got, want) <= TOL


@pytest.mark.parametrize("shape", [(6, 10, 12), (40, 33, 70), (128, 16, 32)])
def test_kdft_nonuniform_matches_oracle(dft, shape):
    say(f"case kdft nonuniform {shape}")
    x = wl.draw_complex(shape, "uniform", 2000 + sum(shape))
    rng = np.random.default_rng(5)
    coords = (np.sort(rng.random(shape[0])), None, np.sort(rng.random(shape[2])))
    want = orc.dft3d(x, coords)
    with dft.Plan(shape, dft.KDFT, coords=coords) as p:
        got = to_host(p.exec(to_dev(x)))
    assert report(f"kdft nonuniform {shape}", got, want) <= TOL


@pytest.mark.parametrize("axis", [0, 1, 2])
@pytest.mark.parametrize("shape", [(20, 36, 28), (128, 130, 64), (3, 5, 260)])
def test_single_mode_contraction(dft, shape, axis):
    say(f"case mode_contract {shape} axis {axis}")
    x = wl.draw_complex(shape, "normal", 3000 + axis)
    M = orc.dft_matrix(shape[axis])
    want = orc.mode_contract(M, x, axis)
    with dft.Plan(shape, dft.KDFT) as p:
        got = to_host(p.mode_contract(axis, to_dev(x)))
        assert report(f"mode {axis} {shape}", got, want) <= TOL
        # backward: conjugate matrix, scaled by 1/N
        wantb = orc.mode_contract(orc.dft_matrix(shape[axis], sign=orc.BACKWARD), x, axis) / shape[axis]
        gotb = to_host(p.mode_contract(axis, to_dev(x), direction=dft.BACKWARD))
        assert report(f"mode {axis} {shape} backward", gotb, wantb) <= TOL


def test_kdft_backward_and_roundtrip(dft):
    shape = (32, 48, 64)
    say(f"case kdft backward {shape}")
    x = wl.draw_complex(shape, "normal", 77)
    with dft.Plan(shape, dft.KDFT) as p:
        xd = to_dev(x)
        X = p.exec(xd)
        got = to_host(p.exec(xd, direction=dft.BACKWARD))
        assert report("kdft backward", got, orc.dft3d(x, sign=orc.BACKWARD)) <= TOL
        back = to_host(p.exec(X, direction=dft.BACKWARD))
        assert report("kdft roundtrip", back, x.astype(np.complex128)) <= TOL


@pytest.mark.parametrize("shape", [(256, 256, 256), (300, 260, 270), (128, 512, 130)])
def test_kdft_three_product_scheme(dft, shape):
    """DFT3D_FLAG_3M: three real products per complex product; same tolerance as the default."""
    say(f"case kdft 3M {shape}")
    x = wl.draw_complex(shape, "normal", 2500 + sum(shape))
    want = orc.dft3d(x)
    with dft.Plan(shape, dft.KDFT, flags=dft.FLAG_3M) as p:
        xd = to_dev(x)
        got = to_host(p.exec(xd))
        assert report(f"kdft 3M {shape}", got, want) <= TOL
        gotb = to_host(p.exec(xd, direction=dft.BACKWARD))
        assert report(f"kdft 3M backward {shape}", gotb, orc.dft3d(x, sign=orc.BACKWARD)) <= TOL
    with dft.Plan(shape, dft.KDFT) as p:
        ref4 = to_host(p.exec(to_dev(x)))
        report(f"kdft 4M {shape} (for comparison)", ref4, want)


@pytest.mark.parametrize("shape,ks", [((6, 10, 12), (4, 10, 20)), ((40, 33, 70), (33, 50, 70)),
                                      ((128, 64, 96), (200, 64, 130))])
def test_kdft_arbitrary_evaluation_points(dft, shape, ks):
    """Eq. 1 - Eq. 3 as written: arbitrary points of the z-plane per axis, rectangular matrices."""
    say(f"case kdft points {shape} -> {ks}")
    x = wl.draw_complex(shape, "uniform", 2600 + sum(shape))
    rng = np.random.default_rng(6)
    pts = []
    for n, k in zip(shape, ks):
        # moduli close to 1 so z^-n stays well inside fp32 range over the whole axis
        pts.append((1.0 + (rng.random(k) - 0.5) / n) * np.exp(2j * np.pi * rng.random(k)))
    pts[1] = None if ks[1] == shape[1] else pts[1]
    want = orc.dft3d_points(x, pts)
    with dft.Plan(shape, dft.KDFT, points=pts) as p:
        assert p.out_shape == tuple(ks)
        xd = to_dev(x)
        got = to_host(p.exec(xd))
        assert got.shape == tuple(ks)
        assert report(f"kdft points {shape}->{ks}", got, want) <= TOL
        with pytest.raises(dft.Dft3dError):
            p.exec(xd, direction=dft.BACKWARD)
        # single modes, in exec order
        y = x.astype(np.complex128)
        yd = xd
        for axis in (2, 1, 0):
            M = orc.dft_matrix(shape[axis]) if pts[axis] is None else orc.points_matrix(pts[axis], shape[axis])
            y = orc.mode_contract(M, y, axis)
            yd = p.mode_contract(axis, yd)
            assert report(f"points mode {axis}", to_host(yd), y) <= TOL


@pytest.mark.parametrize("shape,flags", [((128, 128, 128), 0), ((50, 128, 72), 0), ((128, 256, 128), "3M"),
                                         ((128, 128, 256), "BF16X3"), ((1, 96, 40), 0)])
def test_kdft_adjoint_of_nonuniform_transform(dft, shape, flags):
    """DFT3D_FLAG_ADJOINT on a plan with sample coordinates: out = (M_x (x) M_y (x) M_z)^H in."""
    say(f"case kdft adjoint {shape} {flags}")
    fl = dft.FLAG_ADJOINT | {0: 0, "3M": dft.FLAG_3M, "BF16X3": dft.FLAG_BF16X3}[flags]
    rng = np.random.default_rng(8)
    coords = tuple(np.sort(rng.random(n)) for n in shape)
    coords = (coords[0], None, coords[2])              # one uniform axis among them
    y = wl.draw_complex(shape, "normal", 2650 + sum(shape))
    want = orc.dft3d_adjoint(y, coords=coords)
    with dft.Plan(shape, dft.KDFT, coords=coords, flags=fl) as p:
        yd = to_dev(y)
        assert report(f"kdft adjoint {shape}", to_host(p.exec(yd)), want) <= TOL
        with pytest.raises(dft.Dft3dError):
            p.exec(yd, direction=dft.BACKWARD)
        for axis in range(3):
            MH = orc.dft_matrix(shape[axis], coords[axis]).conj().T
            got = to_host(p.mode_contract(axis, yd))
            assert report(f"adjoint mode {axis}", got, orc.mode_contract(MH, y, axis)) <= TOL
    with pytest.raises(dft.Dft3dError):
        dft.Plan(shape, dft.FFT, flags=dft.FLAG_ADJOINT)


@pytest.mark.parametrize("shape,ks", [((6, 10, 12), (4, 10, 20)), ((128, 64, 96), (200, 64, 130))])
def test_kdft_adjoint_of_point_transform(dft, shape, ks):
    """ADJOINT of the K x N point matrices: a kx x ky x kz tensor goes back to nx x ny x nz."""
    say(f"case kdft points adjoint {ks} -> {shape}")
    rng = np.random.default_rng(10)
    pts = [(1.0 + (rng.random(k) - 0.5) / n) * np.exp(2j * np.pi * rng.random(k)) for n, k in zip(shape, ks)]
    pts[1] = None if ks[1] == shape[1] else pts[1]
    y = wl.draw_complex(ks, "uniform", 2660 + sum(ks))
    want = orc.dft3d_adjoint(y, shape=shape, points=pts)
    with dft.Plan(shape, dft.KDFT, points=pts, flags=dft.FLAG_ADJOINT) as p:
        assert p.shape == tuple(ks) and p.out_shape == tuple(shape)
        got = to_host(p.exec(to_dev(y)))
        assert got.shape == tuple(shape)
        assert report(f"kdft points adjoint {ks}->{shape}", got, want) <= TOL


@pytest.mark.parametrize("shape", [(128, 128, 128), (256, 256, 256), (128, 384, 256), (130, 256, 128),
                                   (130, 200, 258), (33, 129, 40), (1, 7, 300), (200, 1, 1)])
@pytest.mark.parametrize("three_m", [False, True])
def test_kdft_bf16_split_scheme(dft, shape, three_m):
    """DFT3D_FLAG_BF16X3: three bf16 levels per fp32 number on the bf16 matrix cores; same tolerance.
    Whole 128 x 128 tiles or not, every mode must take the bf16 kernel (edge tiles are masked).
    DFT3D_FLAG_3M on top changes nothing for these modes (the bf16 kernel always uses three real products)."""
    say(f"case kdft bf16x3 {shape} three_m={three_m}")
    x = wl.draw_complex(shape, "normal", 2700 + sum(shape))
    want = orc.dft3d(x)
    with dft.Plan(shape, dft.KDFT, flags=dft.FLAG_BF16X3 | (dft.FLAG_3M if three_m else 0)) as p:
        assert [p.mode_kernel(axis) for axis in range(3)] == ["k_contract_bf16x3"] * 3
        xd = to_dev(x)
        got = to_host(p.exec(xd))
        assert report(f"kdft bf16x3 {shape}", got, want) <= TOL
        gotb = to_host(p.exec(xd, direction=dft.BACKWARD))
        assert report(f"kdft bf16x3 backward {shape}", gotb, orc.dft3d(x, sign=orc.BACKWARD)) <= TOL
        for axis in range(3):
            M = orc.dft_matrix(shape[axis])
            gm = to_host(p.mode_contract(axis, xd))
            assert report(f"bf16x3 mode {axis}", gm, orc.mode_contract(M, x, axis)) <= TOL


TOL_F64 = 1e-12     # fp64 unit roundoff 1.1e-16, three modes of length <= 2^11 on either side: ~1e-14 expected


def _oracle_c128(x, coords=(None, None, None), sign=None):
    """The transform of a complex128 tensor from the oracle's own mode products (z, y, x)."""
    sign = orc.FORWARD if sign is None else sign
    y = x
    for axis in (2, 1, 0):
        y = orc.mode_contract(orc.dft_matrix(x.shape[axis], coords[axis], sign), y, axis)
    return y / x.size if sign == orc.BACKWARD else y


@pytest.mark.parametrize("shape", [(6, 10, 12), (40, 33, 70), (64, 64, 64), (128, 130, 64), (3, 5, 260),
                                   (1, 256, 192), (2, 2, 2), (32, 16, 40), (16, 32, 7), (256, 256, 256)])
def test_kdft_complex128(dft, shape):
    """DFT3D_FLAG_COMPLEX128: complex128 tensors, fp64 matrices, fp64 matrix cores."""
    import torch

    say(f"case kdft complex128 {shape}")
    x = wl.draw_complex128(shape, 8100 + sum(shape))
    want = _oracle_c128(x)
    with dft.Plan(shape, dft.KDFT, flags=dft.FLAG_COMPLEX128) as p:
        xd = torch.from_numpy(x).to("cuda")
        got = p.exec(xd).cpu().numpy()
        assert got.dtype == np.complex128
        assert report(f"kdft complex128 {shape}", got, want) <= TOL_F64
        assert np.array_equal(xd.cpu().numpy(), x), "input must be left intact"
        gotb = p.exec(xd, direction=dft.BACKWARD).cpu().numpy()
        assert report(f"kdft complex128 backward {shape}", gotb, _oracle_c128(x, sign=orc.BACKWARD)) <= TOL_F64
        back = p.exec(torch.from_numpy(got).to("cuda"), direction=dft.BACKWARD).cpu().numpy()
        assert report(f"kdft complex128 round trip {shape}", back, x) <= TOL_F64
        for axis in range(3):
            gm = p.mode_contract(axis, xd).cpu().numpy()
            assert report(f"complex128 mode {axis}", gm,
                          orc.mode_contract(orc.dft_matrix(shape[axis]), x, axis)) <= TOL_F64
    with dft.Plan(shape, dft.KDFT, flags=dft.FLAG_COMPLEX128 | dft.FLAG_CLOBBER_INPUT) as p:
        assert p.workspace_bytes() == 0
        got = p.exec(torch.from_numpy(x).to("cuda")).cpu().numpy()
        assert report(f"kdft complex128 clobber {shape}", got, want) <= TOL_F64


@pytest.mark.parametrize("shape,ks,adjoint", [((6, 10, 12), (4, 10, 20), False), ((40, 33, 70), (33, 50, 70), False),
                                              ((64, 48, 40), (80, 48, 130), True)])
def test_kdft_complex128_evaluation_points(dft, shape, ks, adjoint):
    """DFT3D_FLAG_COMPLEX128 on a plan of arbitrary evaluation points (Eq. 1 - 3 as printed, rectangular
    Vandermonde matrices kept in fp64), and on its conjugate transpose."""
    import torch

    say(f"case complex128 points {shape} -> {ks} adjoint={adjoint}")
    rng = np.random.default_rng(8400 + sum(shape))
    points = []
    for j in range(3):
        if ks[j] == shape[j] and j == 1:
            points.append(None)                 # this axis keeps the roots of unity
        else:
            radius = np.exp(rng.uniform(-0.3, 0.3, ks[j]) / shape[j])        # |z|^-n stays within e^(+-0.3)
            points.append(radius * np.exp(2j * np.pi * rng.random(ks[j])))
    Ms = [orc.dft_matrix(shape[j]) if points[j] is None else orc.points_matrix(points[j], shape[j]) for j in range(3)]
    flags = dft.FLAG_COMPLEX128 | (dft.FLAG_ADJOINT if adjoint else 0)
    with dft.Plan(shape, dft.KDFT, points=points, flags=flags) as p:
        if adjoint:
            y = wl.draw_complex128(tuple(ks), 8401)
            want = y
            for axis in (2, 1, 0):
                want = orc.mode_contract(np.ascontiguousarray(Ms[axis].conj().T), want, axis)
            got = p.exec(torch.from_numpy(y).to("cuda")).cpu().numpy()
        else:
            x = wl.draw_complex128(shape, 8402)
            want = x
            for axis in (2, 1, 0):
                want = orc.mode_contract(Ms[axis], want, axis)
            got = p.exec(torch.from_numpy(x).to("cuda")).cpu().numpy()
        assert got.dtype == np.complex128 and got.shape == want.shape
        assert report(f"complex128 points {shape}->{ks}", got, want) <= TOL_F64


def test_kdft_complex128_nonuniform(dft):
    import torch

    shape = (24, 40, 36)
    rng = np.random.default_rng(8200)
    coords = tuple(np.sort(rng.random(n)) for n in shape)
    x = wl.draw_complex128(shape, 8201)
    with dft.Plan(shape, dft.KDFT, coords=coords, flags=dft.FLAG_COMPLEX128) as p:
        got = p.exec(torch.from_numpy(x).to("cuda")).cpu().numpy()
    assert report("kdft complex128 nonuniform", got, _oracle_c128(x, coords)) <= TOL_F64


@pytest.mark.parametrize("shape,split", [((8, 12, 30), (2, 3, 5)), ((64, 32, 128), None), ((36, 20, 48), (6, 4, 8)),
                                         ((1, 256, 512), None), ((128, 64, 64), None), ((6, 5, 7), (3, 1, 7))])
def test_fft_formulation_complex128(dft, shape, split):
    """DFT3D_FLAG_COMPLEX128 on an FFT plan: per axis first stage with the fp64 twiddle in its epilogue
    and second stage (the x / y re-ordering folded into its stores), z re-ordering pass, all in fp64."""
    import torch

    say(f"case fft complex128 {shape} split {split}")
    x = wl.draw_complex128(shape, 8300 + sum(shape))
    want = _oracle_c128(x)
    xd = torch.from_numpy(x).to("cuda")
    with dft.Plan(shape, dft.FFT, split=split, flags=dft.FLAG_COMPLEX128) as p:
        got = p.exec(xd).cpu().numpy()
        assert got.dtype == np.complex128
        assert report(f"fft complex128 {shape}", got, want) <= TOL_F64
        assert np.array_equal(xd.cpu().numpy(), x), "input must be left intact"
        gotb = p.exec(xd, direction=dft.BACKWARD).cpu().numpy()
        assert report(f"fft complex128 backward {shape}", gotb, _oracle_c128(x, sign=orc.BACKWARD)) <= TOL_F64
        back = p.exec(torch.from_numpy(got).to("cuda"), direction=dft.BACKWARD).cpu().numpy()
        assert report(f"fft complex128 round trip {shape}", back, x) <= TOL_F64
        # single steps against the oracle's literal steps (fp64 throughout)
        for axis in range(3):
            A, B = p.split(axis)
            z = ff.first_stage(x, axis, A, B)
            assert report(f"c128 f1 axis {axis}", p.fft_first_stage(axis, xd).cpu().numpy(), z) <= TOL_F64
            w = ff.second_stage(x, axis, A, B)
            assert report(f"c128 f2 axis {axis}", p.fft_second_stage(axis, xd, reorder=False).cpu().numpy(), w) <= TOL_F64
            assert report(f"c128 f2+reorder axis {axis}", p.fft_second_stage(axis, xd, reorder=True).cpu().numpy(),
                          ff.reorder(w, axis, A, B)) <= TOL_F64
            moved = p.fft_reorder(1 << axis, xd).cpu().numpy()
            assert np.array_equal(moved, ff.reorder(x, axis, A, B)), "re-ordering is pure data movement"
        with pytest.raises(dft.Dft3dError):
            p.fft_phase(0, xd)
    with dft.Plan(shape, dft.FFT, split=split, flags=dft.FLAG_COMPLEX128 | dft.FLAG_CLOBBER_INPUT) as p:
        assert p.workspace_bytes() == 0
        got = p.exec(torch.from_numpy(x).to("cuda")).cpu().numpy()
        assert report(f"fft complex128 clobber {shape}", got, want) <= TOL_F64


def test_complex128_plan_restrictions(dft):
    with pytest.raises(dft.Dft3dError) as e:
        dft.Plan((8, 8, 8), dft.FFT, flags=dft.FLAG_COMPLEX128 | dft.FLAG_UNFUSED)
    assert e.value.status_name == "DFT3D_ERR_UNSUPPORTED"
    with pytest.raises(dft.Dft3dError):
        dft.Plan((8, 8, 8), dft.KDFT, flags=dft.FLAG_COMPLEX128 | dft.FLAG_3M)
    import torch

    with dft.Plan((8, 8, 8), dft.KDFT, flags=dft.FLAG_COMPLEX128) as p:
        with pytest.raises(ValueError):
            p.exec(torch.zeros((8, 8, 8), dtype=torch.complex64, device="cuda"))


def test_plan_reports_the_kernel_of_each_mode(dft):
    with dft.Plan((256, 256, 256), dft.KDFT) as p:
        assert [p.mode_kernel(a) for a in range(3)] == ["k_contract_s", "k_contract_s", "k_contract_c"]
    with dft.Plan((256, 256, 256), dft.KDFT, flags=dft.FLAG_3M) as p:
        assert [p.mode_kernel(a) for a in range(3)] == ["k_contract_s (3M)", "k_contract_s (3M)", "k_contract_c (3M)"]
    with dft.Plan((64, 64, 64), dft.KDFT) as p:
        assert p.mode_kernel(0) == "k_contract_sr" and p.mode_kernel(2) == "k_contract_c"
    with dft.Plan((64, 64, 64), dft.KDFT, flags=dft.FLAG_COMPLEX128) as p:
        assert p.mode_kernel(1) == "k_contract_f64"
    with dft.Plan((64, 64, 64), dft.FFT) as p:
        assert p.mode_kernel(0) == "butterflies + second stage"           # 64 = 8 x 8 (FFT plans: how the axis runs)


def test_fft_plan_reports_how_each_axis_runs(dft):
    with dft.Plan((512, 48, 1024), dft.FFT) as p:
        assert p.mode_kernel(0) == "fused" and p.mode_kernel(2) == "fused"
        assert p.mode_kernel(1) == "first stage + second stage"          # 48 = 6 x 8
    with dft.Plan((1, 8192, 8192), dft.FFT) as p:
        assert p.mode_kernel(0) == "identity"
        assert p.mode_kernel(1) == p.mode_kernel(2) == "butterflies + fused second stage"
    with dft.Plan((8, 8192, 24), dft.FFT) as p:
        assert p.mode_kernel(0) == "butterflies + second stage"           # 8 = 2 x 4
        assert p.mode_kernel(1) == "first stage + second stage"           # inner extent 24: 8192 = 64 x 128
    with dft.Plan((16, 16, 16), dft.FFT, flags=dft.FLAG_UNFUSED) as p:
        assert p.mode_kernel(1) == "first stage, twiddle pass, second stage"


def test_kdft_clobber_input(dft):
    shape = (16, 24, 40)
    x = wl.draw_complex(shape, "normal", 78)
    with dft.Plan(shape, dft.KDFT, flags=dft.FLAG_CLOBBER_INPUT) as p:
        assert p.workspace_bytes() == 0
        got = to_host(p.exec(to_dev(x)))
    assert report("kdft clobber", got, orc.dft3d(x)) <= TOL


@pytest.mark.parametrize("shape", [(2, 2, 2), (4, 4, 4), (2, 4, 2), (4, 2, 4)])
def test_exact_arithmetic_is_bitwise(dft, shape):
    # every matrix entry is 0 / +-1 and the inputs are small integers: fp32 is exact
    say(f"case exact {shape}")
    x = wl.gaussian_integers(shape, 31)
    want = orc.dft3d(x)
    # the oracle's own entries carry ~1e-16 (libm cos(pi/2) is not 0): exact result = nearest integer
    assert np.max(np.abs(want - np.round(want))) < 1e-12
    with dft.Plan(shape, dft.KDFT) as p:
        got = to_host(p.exec(to_dev(x)))
    assert np.array_equal(got.astype(np.complex128), np.round(want))
    with dft.Plan(shape, dft.FFT) as p:
        got = to_host(p.exec(to_dev(x)))
    assert np.array_equal(got.astype(np.complex128), np.round(want))


def test_generated_matrix_on_device_equals_host_generator(dft):
    # contracting the identity along an axis returns the matrix the device holds
    n = 48
    shape = (n, 1, n)
    x = np.zeros(shape, np.complex64)
    x[np.arange(n), 0, np.arange(n)] = 1            # x[a, 0, c] = delta(a, c)
    rng = np.random.default_rng(3)
    c = np.sort(rng.random(n))
    with dft.Plan(shape, dft.KDFT, coords=(c, None, None)) as p:
        got = to_host(p.mode_contract(0, to_dev(x)))[:, 0, :]     # got[k, c] = M[k, c]
    assert np.array_equal(got, dft.generate_matrix(n, c))


# ------------------------------------------------------------------------------------ FFT steps
FFT_CASES = [((16, 16, 16), None), ((8, 12, 30), (2, 3, 5)), ((64, 32, 128), None),
             ((36, 20, 48), (6, 4, 8)), ((32, 32, 512), (4, 8, 16)), ((6, 5, 7), (3, 1, 7)),
             # strided stages with 16 / 32 / 64-point matrices and inner extents that are multiples of 16
             ((4, 2048, 16), None), ((2, 4096, 16), (0, 64, 0)), ((512, 3, 48), (16, 0, 0)), ((1024, 1, 80), (16, 0, 0)),
             # first factor 2, 4 or 8 (butterflies in an element-wise pass), second factor of 512, 1024 or 2048 points
             # on the fused kernels: 8192 = 4 x 2048 by default
             ((2, 1024, 32), (0, 2, 0)), ((1024, 2, 16), (2, 0, 0)), ((3, 2, 4096), (0, 0, 2)), ((2, 3, 8192), None),
             ((8192, 1, 16), None), ((1, 4096, 48), (0, 8, 0)), ((2, 2, 8192), (0, 0, 8)), ((1, 8192, 64), (0, 4, 16))]


@pytest.mark.parametrize("shape,split", FFT_CASES)
def test_fft_steps_match_oracle_steps(dft, shape, split):
    say(f"case fft steps {shape} split {split}")
    x = wl.draw_complex(shape, "normal", 4000 + sum(shape))
    xd = to_dev(x)
    with dft.Plan(shape, dft.FFT, split=split) as p:
        for axis in range(3):
            A, B = p.split(axis)
            assert A * B == shape[axis]
            say(f"  axis {axis}: A={A} B={B}")
            loc = ff.local_transform(x, axis, A, B)
            got = to_host(p.fft_first_stage(axis, xd, fuse_twiddle=False))
            assert report(f"f1 no-twiddle axis {axis}", got, loc) <= TOL
            z = ff.first_stage(x, axis, A, B)
            got = to_host(p.fft_first_stage(axis, xd, fuse_twiddle=True))
            assert report(f"f1 axis {axis}", got, z) <= TOL
            got = to_host(p.fft_phase(axis, xd))
            assert report(f"phase axis {axis}", got, ff.twiddle(x, axis, A, B)) <= TOL
            w = ff.second_stage(x, axis, A, B)
            got = to_host(p.fft_second_stage(axis, xd, reorder=False))
            assert report(f"f2 axis {axis}", got, w) <= TOL
            got = to_host(p.fft_second_stage(axis, xd, reorder=True))
            assert report(f"f2+reorder axis {axis}", got, ff.reorder(w, axis, A, B)) <= TOL
            # pure data movement: exact
            got = to_host(p.fft_reorder(1 << axis, xd))
            assert np.array_equal(got, ff.reorder(x, axis, A, B).astype(np.complex64))
        want = x.astype(np.complex128)
        for axis in range(3):
            A, B = p.split(axis)
            want = ff.reorder(want, axis, A, B)
        assert np.array_equal(to_host(p.fft_reorder(7, xd)), want.astype(np.complex64))


@pytest.mark.parametrize("shape,split", [((5, 7, 256), None), ((16, 9, 512), None), ((3, 3, 1024), None),
                                         ((2, 5, 2048), None), ((1, 3, 4096), None),
                                         ((4, 4, 512), (2, 2, 16)), ((33, 1, 256), None),
                                         # 512, 1024 and 2048 default to 16 x (C*16) with the second factor split
                                         # once more inside the kernel; the last case has more rows than the
                                         # launch has waves.  32 x 32 and 32 x 64 are the kernels without that.
                                         ((9, 250, 2048), None), ((40, 100, 512), None),
                                         ((3, 3, 1024), (1, 1, 32)), ((2, 5, 2048), (1, 1, 32))])
def test_fft_fused_axis_kernel(dft, shape, split):
    """The single-kernel z-axis pass equals first stage + twiddle + second stage + re-ordering."""
    say(f"case fft fused axis {shape} split {split}")
    x = wl.draw_complex(shape, "normal", 4500 + sum(shape))
    xd = to_dev(x)
    with dft.Plan(shape, dft.FFT, split=split) as p:
        A, B = p.split(2)
        want = ff.fft_axis(x, 2, A, B)
        got = to_host(p.fft_axis(2, xd))
        assert report(f"fused z axis {A}x{B}", got, want) <= TOL
        assert rel_l2(got, np.fft.fft(x.astype(np.complex128), axis=2)) <= TOL
        wantb = ff.fft_axis(x, 2, A, B, sign=ff.BACKWARD) / shape[2]
        gotb = to_host(p.fft_axis(2, xd, direction=dft.BACKWARD))
        assert report(f"fused z axis {A}x{B} backward", gotb, wantb) <= TOL
        with pytest.raises(dft.Dft3dError):
            p.fft_axis(0, xd)       # axis length shape[0] has no fused kernel in these cases


@pytest.mark.parametrize("shape,split", [((256, 3, 16), None), ((2, 512, 48), None), ((1024, 1, 32), None),
                                         ((3, 256, 160), None), ((512, 5, 16), (16, 1, 4)),
                                         # inner extents that are multiples of 32: tiles of 32 columns
                                         ((512, 2, 32), None), ((3, 512, 96), None), ((512, 1, 352), None),
                                         # multiples of 64 with rows at least 32 KiB apart: 64-column tiles
                                         ((512, 1, 64), None), ((2, 512, 192), None), ((512, 3, 64), None),
                                         ((512, 64, 64), None), ((512, 3, 2112), None),
                                         # 2048 = 32 x (4*16) on a strided axis: first stage of 32 points
                                         ((2048, 1, 16), (32, 1, 1)), ((2, 2048, 48), (1, 32, 1)), ((2048, 3, 16), (32, 1, 1)),
                                         ((2048, 2, 4112), (32, 1, 1)),
                                         # 2048 = 16 x (8*16): second factor split once more inside the kernel
                                         ((2048, 1, 16), (16, 1, 1)), ((2, 2048, 48), (1, 16, 1)),
                                         ((2048, 3, 32), (16, 1, 1)), ((2048, 2, 4112), (16, 1, 1)),
                                         # 1024 = 16 x (4*16), against 32 x 32 by default
                                         ((1024, 1, 32), (16, 1, 1)), ((2, 1024, 48), (1, 16, 1)),
                                         ((1024, 5, 1040), (16, 1, 1)), ((1024, 3, 1056), (16, 1, 1)),
                                         # 1024 = 32 x (2*16)
                                         ((1024, 1, 32), (32, 1, 1)), ((2, 1024, 48), (1, 32, 1)),
                                         ((1024, 3, 1056), (32, 1, 1))])
def test_fft_fused_strided_axis_kernel(dft, shape, split):
    """The single-kernel x / y pass equals first stage + twiddle + second stage + re-ordering."""
    say(f"case fft fused strided axis {shape} split {split}")
    x = wl.draw_complex(shape, "normal", 4600 + sum(shape))
    xd = to_dev(x)
    with dft.Plan(shape, dft.FFT, split=split) as p:
        axis = 0 if shape[0] >= 256 else 1
        say(f"  kernel split {p.split(axis)}")
        A, B = p.split(axis)
        want = ff.fft_axis(x, axis, A, B)
        got = to_host(p.fft_axis(axis, xd))
        assert report(f"fused axis {axis} {A}x{B}", got, want) <= TOL
        assert rel_l2(got, np.fft.fft(x.astype(np.complex128), axis=axis)) <= TOL
        wantb = ff.fft_axis(x, axis, A, B, sign=ff.BACKWARD) / shape[axis]
        gotb = to_host(p.fft_axis(axis, xd, direction=dft.BACKWARD))
        assert report(f"fused axis {axis} {A}x{B} backward", gotb, wantb) <= TOL


@pytest.mark.parametrize("shape,split", FFT_CASES + [((64, 64, 64), None), ((128, 16, 256), None),
                                                     ((256, 512, 256), None), ((256, 256, 24), None)])
@pytest.mark.parametrize("flags", [0, 2])
def test_fft_exec_matches_oracle(dft, shape, split, flags):
    say(f"case fft exec {shape} split {split} flags {flags}")
    x = wl.draw_complex(shape, "normal", 5000 + sum(shape))
    want = orc.dft3d(x)
    with dft.Plan(shape, dft.FFT, split=split, flags=flags) as p:
        xd = to_dev(x)
        got = to_host(p.exec(xd))
        assert report(f"fft exec {shape}", got, want) <= TOL
        assert np.array_equal(to_host(xd), x), "input must be left intact"
        gotb = to_host(p.exec(xd, direction=dft.BACKWARD))
        assert report(f"fft exec backward {shape}", gotb, orc.dft3d(x, sign=orc.BACKWARD)) <= TOL


@pytest.mark.parametrize("shape,split", [((2, 1024, 1024), (0, 2, 2)), ((1, 4096, 1024), (0, 8, 2)),
                                         ((1024, 1, 1024), (2, 0, 2)), ((1, 1024, 4096), (0, 2, 8)),
                                         ((4, 16, 4096), (2, 2, 4))])
@pytest.mark.parametrize("flags", [0, 1])
def test_fft_first_factor_in_butterflies_exec(dft, shape, split, flags):
    """Splits R x M with R = 2, 4, 8: where the z axis and the axis transformed after it both start with the
    butterfly pass, the second one reads through the z re-ordering (one pass fewer); with CLOBBER_INPUT the
    pass count has to stay odd."""
    say(f"case fft radix exec {shape} split {split} flags {flags}")
    x = wl.draw_complex(shape, "normal", 5100 + sum(shape))
    want = orc.dft3d(x)
    with dft.Plan(shape, dft.FFT, split=split, flags=flags) as p:
        got = to_host(p.exec(to_dev(x)))
        assert report(f"fft radix exec {shape}", got, want) <= TOL
        gotb = to_host(p.exec(to_dev(x), direction=dft.BACKWARD))
        assert report(f"fft radix exec backward {shape}", gotb, orc.dft3d(x, sign=orc.BACKWARD)) <= TOL


@pytest.mark.parametrize("shape", [(1, 96, 160), (1, 1, 256), (1, 256, 1), (40, 1, 48), (1, 1, 1), (1, 256, 512)])
@pytest.mark.parametrize("form", ["kdft", "fft"])
@pytest.mark.parametrize("flags", [0, 1])
def test_lower_dimensional_transforms(dft, shape, form, flags):
    """Axes of length 1 (2-D and 1-D transforms) take no pass; the result is still the 3-D definition."""
    import torch

    say(f"case {form} {shape} flags {flags}")
    x = wl.draw_complex(shape, "normal", 7000 + sum(shape))
    want = orc.dft3d(x)
    with dft.Plan(shape, dft.KDFT if form == "kdft" else dft.FFT, flags=flags) as p:
        got = to_host(p.exec(to_dev(x)))
        assert report(f"{form} {shape} flags {flags}", got, want) <= TOL
        gotb = to_host(p.exec(to_dev(x), direction=dft.BACKWARD))
        assert report(f"{form} backward {shape}", gotb, orc.dft3d(x, sign=orc.BACKWARD)) <= TOL
        if flags == 0:
            p.enable_profiling(1)
            p.exec(to_dev(x))
            torch.cuda.synchronize()
            npass = len(p.read_profile(0))
            live = sum(1 for n in shape if n > 1)
            if form == "kdft":
                assert npass == max(live, 1)


def test_kdft_and_fft_agree(dft):
    import torch

    shape = (64, 128, 256)
    x = wl.draw_complex(shape, "normal", 6000)
    xd = to_dev(x)
    with dft.Plan(shape, dft.KDFT) as pk, dft.Plan(shape, dft.FFT) as pf:
        a = pk.exec(xd)
        b = pf.exec(xd)
        torch.cuda.synchronize()
        r = (torch.linalg.vector_norm((a - b).to(torch.complex128)) /
             torch.linalg.vector_norm(a.to(torch.complex128))).item()
    say(f"[parity] kdft vs fft {shape}: relL2={r:.3e}")
    assert r <= 2 * TOL


@pytest.mark.parametrize("variant", ["fp32", "3M", "BF16X3", "BF16X3+3M", "FFT", "FFT-nested", "FFT-radix", "small"])
def test_power_of_two_scaling_is_exact(dft, variant):
    """exec(2^s x) must equal 2^s exec(x) bit for bit (s = -60, +60): scaling by a power of two
    commutes with every rounding of every path unless the path hides an assumption on the range of
    its data (a fixed-point step, a clamp, an underflowing piece of the bf16 split)."""
    import torch

    # ("FFT-nested": 512 and 1024 points run the kernels that split the second factor once more, with their
    # butterflies in vector arithmetic; "FFT-radix": 8192 = 4 x 2048 with the first factor as a butterfly pass,
    # and the y axis (8 x 8) reading through the z re-ordering)
    shape = {"small": (32, 32, 32), "FFT-nested": (16, 512, 1024), "FFT-radix": (1, 64, 8192)}.get(variant, (128, 256, 128))
    form = dft.FFT if variant.startswith("FFT") else dft.KDFT
    flags = {"fp32": 0, "3M": dft.FLAG_3M, "BF16X3": dft.FLAG_BF16X3, "BF16X3+3M": dft.FLAG_BF16X3 | dft.FLAG_3M,
             "FFT": 0, "FFT-nested": 0, "FFT-radix": 0, "small": 0}[variant]
    say(f"case scaling {variant} {shape}")
    x = wl.draw_complex(shape, "normal", 9100)
    with dft.Plan(shape, form, flags=flags) as p:
        base = to_host(p.exec(to_dev(x)))
        assert report(f"scaling base {variant}", base, orc.dft3d(x)) <= TOL
        for s in (-60, 60):
            xs = (x * np.float32(2.0 ** s)).astype(np.complex64)
            assert np.array_equal(xs * np.float32(2.0 ** -s), x), "the scaled input itself must be exact"
            got = to_host(p.exec(to_dev(xs)))
            want = (base * np.float32(2.0 ** s)).astype(np.complex64)
            assert np.all(np.isfinite(got.view(np.float32)))
            assert np.array_equal(got.view(np.uint32), want.view(np.uint32)), f"{variant}: scaling by 2^{s} is not exact"


@pytest.mark.parametrize("variant", ["fp32", "3M", "BF16X3", "BF16X3+3M", "FFT", "FFT-nested", "FFT-radix"])
def test_input_magnitudes_spanning_eighty_binades(dft, variant):
    """Every element carries its own power-of-two factor 2^e, e uniform in [-40, 40]: the result is
    dominated by the large elements and must still meet the tolerance against the oracle."""
    shape = {"FFT-nested": (16, 512, 1024), "FFT-radix": (1, 64, 8192)}.get(variant, (128, 128, 256))
    form = dft.FFT if variant.startswith("FFT") else dft.KDFT
    flags = {"fp32": 0, "3M": dft.FLAG_3M, "BF16X3": dft.FLAG_BF16X3, "BF16X3+3M": dft.FLAG_BF16X3 | dft.FLAG_3M,
             "FFT": 0, "FFT-nested": 0, "FFT-radix": 0}[variant]
    say(f"case wide magnitudes {variant} {shape}")
    rng = np.random.default_rng(9200)
    e = rng.integers(-40, 41, size=shape)
    x = (wl.draw_complex(shape, "normal", 9201) * np.exp2(e).astype(np.float32)).astype(np.complex64)
    want = orc.dft3d(x)
    with dft.Plan(shape, form, flags=flags) as p:
        got = to_host(p.exec(to_dev(x)))
    assert report(f"wide magnitudes {variant}", got, want) <= TOL


def test_buffer_checks_misaligned_and_overlapping(dft):
    """Pointers that are not 16-byte aligned, and a workspace that overlaps the input or the output, are
    INVALID_ARG (no kernel is launched)."""
    import ctypes

    import torch

    lib = dft.load_library()
    shape = (8, 8, 40)
    n = 8 * 8 * 40
    big = torch.zeros(4 * n + 8, dtype=torch.complex64, device="cuda")
    base = big.data_ptr()
    assert base % 16 == 0
    vp = ctypes.c_void_p

    def status(fn, *a):
        return lib.dft3d_status_string(fn(*a))

    with dft.Plan(shape, dft.KDFT) as p:
        ws_bytes = p.workspace_bytes()
        assert ws_bytes == n * 8
        # misaligned workspace
        assert status(lib.dft3d_plan_set_workspace, p._h, vp(base + 8), ws_bytes) == b"DFT3D_ERR_INVALID_ARG"
        # too small
        assert status(lib.dft3d_plan_set_workspace, p._h, vp(base), ws_bytes - 8) == b"DFT3D_ERR_INVALID_ARG"
        x, out, ws = base, base + n * 8, base + 2 * n * 8
        assert status(lib.dft3d_plan_set_workspace, p._h, vp(ws), ws_bytes) == b"DFT3D_OK"
        assert status(lib.dft3d_exec, p._h, vp(x), vp(out), dft.FORWARD, None) == b"DFT3D_OK"
        # misaligned in / out
        assert status(lib.dft3d_exec, p._h, vp(x + 8), vp(out), dft.FORWARD, None) == b"DFT3D_ERR_INVALID_ARG"
        assert b"aligned" in lib.dft3d_last_error()
        assert status(lib.dft3d_exec, p._h, vp(x), vp(out + 8), dft.FORWARD, None) == b"DFT3D_ERR_INVALID_ARG"
        # partial overlap of in and out
        assert status(lib.dft3d_exec, p._h, vp(x), vp(x + 16), dft.FORWARD, None) == b"DFT3D_ERR_INVALID_ARG"
        assert b"overlap" in lib.dft3d_last_error()
        # workspace overlapping the output, then the input
        assert status(lib.dft3d_plan_set_workspace, p._h, vp(out + 16), ws_bytes) == b"DFT3D_OK"
        assert status(lib.dft3d_exec, p._h, vp(x), vp(out), dft.FORWARD, None) == b"DFT3D_ERR_INVALID_ARG"
        assert b"workspace overlaps" in lib.dft3d_last_error()
        assert status(lib.dft3d_plan_set_workspace, p._h, vp(x + 16 * 8), ws_bytes) == b"DFT3D_OK"
        assert status(lib.dft3d_exec, p._h, vp(x), vp(base + 3 * n * 8), dft.FORWARD, None) == b"DFT3D_ERR_INVALID_ARG"
        # single steps check their tensors the same way
        assert status(lib.dft3d_mode_contract, p._h, 2, vp(x + 8), vp(out), dft.FORWARD, None) == b"DFT3D_ERR_INVALID_ARG"
        assert status(lib.dft3d_mode_contract, p._h, 2, vp(x), vp(x), dft.FORWARD, None) == b"DFT3D_ERR_INVALID_ARG"
        assert status(lib.dft3d_plan_set_workspace, p._h, None, 0) == b"DFT3D_OK"
    torch.cuda.synchronize()


# ------------------------------------------------------------------------------------ the named configurations
def test_cfg1_kdft_32(dft):
    w = wl.WORKLOADS["cfg1"]
    x = wl.make_input(w)
    with dft.Plan(w.shape, dft.KDFT) as p:
        got = to_host(p.exec(to_dev(x)))
    assert report(w.name, got, orc.dft3d(x)) <= TOL


def test_cfg4_kdft_nonuniform_128(dft):
    w = wl.WORKLOADS["cfg4"]
    x = wl.make_input(w)
    coords = wl.make_coords(w)
    with dft.Plan(w.shape, dft.KDFT, coords=coords) as p:
        got = to_host(p.exec(to_dev(x)))
    assert report(w.name, got, orc.dft3d(x, coords)) <= TOL


def test_cfg2_kdft_256(dft):
    w = wl.WORKLOADS["cfg2"]
    say(f"case {w.name}")
    x = wl.make_input(w)
    with dft.Plan(w.shape, dft.KDFT) as p:
        got = to_host(p.exec(to_dev(x)))
    say("  gpu done, running oracle")
    assert report(w.name, got, orc.dft3d(x)) <= TOL


# ------------------------------------------------------------------------------------ boundary behaviour on the device
def test_exec_argument_errors(dft):
    import torch

    shape = (8, 8, 40)      # (axes of at most 32 points would need no workspace)
    x = to_dev(wl.draw_complex(shape, "normal", 1))
    with dft.Plan(shape, dft.KDFT) as p:
        with pytest.raises(dft.Dft3dError) as ei:      # no workspace set
            p._lib.dft3d_exec  # noqa: B018
            from paper_2002_03260_amd.binding import _check
            import ctypes
            _check(p._lib.dft3d_exec(p._h, ctypes.c_void_p(x.data_ptr()),
                                     ctypes.c_void_p(torch.empty_like(x).data_ptr()), dft.FORWARD, None))
        assert ei.value.status_name == "DFT3D_ERR_INVALID_ARG"
        with pytest.raises(dft.Dft3dError):            # in place
            p.exec(x, out=x)
        with pytest.raises(dft.Dft3dError):            # bad direction
            p.exec(x, direction=0)
    rng = np.random.default_rng(0)
    with dft.Plan(shape, dft.KDFT, coords=(np.sort(rng.random(8)), None, None)) as p:
        with pytest.raises(dft.Dft3dError) as ei:
            p.exec(x, direction=dft.BACKWARD)
        assert ei.value.status_name == "DFT3D_ERR_UNSUPPORTED"


@pytest.mark.parametrize("form,shape", [("KDFT", (32, 32, 32)), ("KDFT", (128, 128, 128)), ("FFT", (64, 256, 256))])
def test_exec_replayed_from_a_hip_graph(dft, form, shape):
    """exec only launches kernels, so a caller may capture it into a HIP graph (what pays for the
    small, launch-bound sizes).  Several replays, with eager work and synchronisations in between,
    must each reproduce the eager result bit for bit, and that result is the oracle's."""
    import torch
    say(f"case graph replay {form} {shape}")
    formulation = dft.KDFT if form == "KDFT" else dft.FFT
    x = wl.draw_complex(shape, "normal", 2900 + sum(shape))
    want = orc.dft3d(x)
    with dft.Plan(shape, formulation) as p:
        xd = to_dev(x)
        p.ensure_workspace()
        eager = p.exec(xd).clone()
        torch.cuda.synchronize()
        assert report(f"graph eager {form} {shape}", to_host(eager), want) <= TOL
        out = torch.empty_like(xd)
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            p.exec(xd, out)                      # warm-up on the capture stream
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=side):
            p.exec(xd, out)
        for rep in range(4):
            out.fill_(0)                          # a fill kernel, not a memset node inside the graph
            torch.cuda.synchronize()
            g.replay()
            torch.cuda.synchronize()
            assert torch.equal(out, eager), f"replay {rep} differs from the eager result"
            other = p.exec(xd)                    # eager work between the replays
            torch.cuda.synchronize()
            assert torch.equal(other, eager)
        del g


@pytest.mark.parametrize("shape", [(32, 32, 32), (5, 7, 3), (1, 1, 8), (32, 1, 17), (2, 31, 32), (1, 1, 1)])
def test_kdft_single_launch_small_shapes(dft, shape):
    """Axes of at most 32 points: exec runs all three modes in one launch (no workspace).  Forward,
    backward, nonuniform coordinates, adjoint; the arithmetic flags change nothing here."""
    say(f"case kdft single launch {shape}")
    x = wl.draw_complex(shape, "normal", 3000 + sum(shape))
    xd = to_dev(x)
    with dft.Plan(shape, dft.KDFT) as p:
        assert p.workspace_bytes() == 0
        assert report(f"small fwd {shape}", to_host(p.exec(xd)), orc.dft3d(x)) <= TOL
        assert report(f"small bwd {shape}", to_host(p.exec(xd, direction=dft.BACKWARD)),
                      orc.dft3d(x, sign=orc.BACKWARD)) <= TOL
        # the single-launch path and the per-mode kernels are different code: they must agree too
        y = xd
        for axis in (2, 1, 0):
            y = p.mode_contract(axis, y)
        assert report(f"small exec vs modes {shape}", to_host(p.exec(xd)), to_host(y).astype(np.complex128)) <= TOL
    with dft.Plan(shape, dft.KDFT, flags=dft.FLAG_3M | dft.FLAG_BF16X3) as p:
        assert p.mode_kernel(0) == "k_kdft_small"
        assert report(f"small flags {shape}", to_host(p.exec(xd)), orc.dft3d(x)) <= TOL
    rng = np.random.default_rng(14)
    coords = tuple(np.sort(rng.random(n)) for n in shape)
    with dft.Plan(shape, dft.KDFT, coords=coords) as p:
        assert report(f"small nonuniform {shape}", to_host(p.exec(xd)), orc.dft3d(x, coords)) <= TOL
    with dft.Plan(shape, dft.KDFT, coords=coords, flags=dft.FLAG_ADJOINT) as p:
        assert report(f"small adjoint {shape}", to_host(p.exec(xd)), orc.dft3d_adjoint(x, coords=coords)) <= TOL


def _sweep_case(seed):
    """A seeded random configuration: shape (mixing tiny sizes with sizes next to the tile edges),
    formulation, flags, direction."""
    rng = np.random.default_rng(5000 + seed)
    pool = [1, 2, 3, 5, 8, 15, 16, 17, 24, 31, 32, 33, 48, 63, 64, 65, 80, 96, 127, 128, 129, 130, 160, 192, 256]
    while True:
        shape = tuple(int(rng.choice(pool)) for _ in range(3))
        if np.prod(shape) <= 1_500_000:
            break
    form = "FFT" if rng.random() < 0.45 else "KDFT"
    backward = bool(rng.random() < 0.4)
    flags = []
    if rng.random() < 0.3:
        flags.append("CLOBBER_INPUT")
    if form == "KDFT":
        if rng.random() < 0.3:
            flags.append("3M")
        if rng.random() < 0.2:
            flags.append("BF16X3")
        nonuniform = (not backward) and rng.random() < 0.3
    else:
        if rng.random() < 0.25 and "CLOBBER_INPUT" not in flags:
            flags.append("UNFUSED")
        nonuniform = False
    return shape, form, tuple(flags), backward, nonuniform


@pytest.mark.parametrize("seed", range(128))
def test_random_configuration_sweep(dft, seed):
    """Whole transforms of seeded random shapes / formulations / flags / directions against the oracle:
    every dispatch decision (fast or masked tiles, fused or staged axes, skipped axes, ping-pong
    parity with CLOBBER_INPUT, the single-launch path) is taken by some case."""
    shape, form, flags, backward, nonuniform = _sweep_case(seed)
    say(f"case sweep {seed}: {shape} {form} {flags} backward={backward} nonuniform={nonuniform}")
    rng = np.random.default_rng(6000 + seed)
    coords = tuple(np.sort(rng.random(n)) for n in shape) if nonuniform else (None, None, None)
    fl = 0
    for f in flags:
        fl |= getattr(dft, "FLAG_" + f)
    x = wl.draw_complex(shape, "normal", 7000 + seed)
    sign = orc.BACKWARD if backward else orc.FORWARD
    want = orc.dft3d(x, coords, sign=sign)
    formulation = dft.FFT if form == "FFT" else dft.KDFT
    try:
        plan = dft.Plan(shape, formulation, coords=coords, flags=fl)
    except dft.Dft3dError as e:
        assert e.status_name == "DFT3D_ERR_UNSUPPORTED", e
        pytest.skip(f"combination not offered: {e}")
    with plan as p:
        xd = to_dev(x)
        try:
            got = to_host(p.exec(xd, direction=dft.BACKWARD if backward else dft.FORWARD))
        except dft.Dft3dError as e:
            assert e.status_name == "DFT3D_ERR_UNSUPPORTED", e
            pytest.skip(f"combination not offered: {e}")
        assert report(f"sweep {seed} {shape} {form} {flags}", got, want) <= TOL
