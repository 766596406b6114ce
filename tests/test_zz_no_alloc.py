"""The entry point that allocates nothing (dft3d_exec_noalloc) against dft3d_exec, through the C ABI.

Same kernels in the same order, only the intermediate tensor lives in the library's static scratch
array instead of the caller's workspace, so the two outputs must be bit-identical.  Two calls in a
row share the array, the second with a smaller tensor."""
import ctypes

import numpy as np
import pytest

import dft3d_workloads as wl

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def dft(gpu_device):
    import paper_2002_03260_amd as d

    d.load_library()
    return d


def _both(dft, shape, form, coords=(None, None, None), seed=1, flags=0, direction=None):
    """(dft3d_exec output, dft3d_exec_noalloc output) of one seeded input, called through ctypes."""
    import torch

    lib = dft.load_library()
    direction = dft.FORWARD if direction is None else direction
    x = torch.from_numpy(wl.draw_complex(shape, "normal", seed)).to("cuda")
    with dft.Plan(shape, form, coords=coords, flags=flags) as p:
        want = p.exec(x, direction=direction)
        torch.cuda.synchronize()
        got = torch.full_like(x, float("nan"))
        stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
        st = lib.dft3d_exec_noalloc(p._h, ctypes.c_void_p(x.data_ptr()), ctypes.c_void_p(got.data_ptr()),
                                    direction, stream)
        assert st == 0, lib.dft3d_last_error().decode()
        torch.cuda.synchronize()
    return want.cpu().numpy(), got.cpu().numpy(), x.cpu().numpy()


def test_exec_noalloc_two_calls_in_a_row_equal_exec(dft):
    from oracle import dft3d_oracle as orc

    # first call: the nonuniform 128^3 configuration (its intermediate fills half of the scratch array)
    w = wl.WORKLOADS["cfg4"]
    coords = wl.make_coords(w)
    want, got, x = _both(dft, w.shape, dft.KDFT, coords, seed=w.seed)
    assert np.array_equal(want.view(np.uint32), got.view(np.uint32))
    ref = orc.dft3d(x, coords)
    assert np.linalg.norm((got - ref).ravel()) / np.linalg.norm(ref.ravel()) <= 2e-5
    # second call right after it: a smaller, ragged tensor in the FFT formulation, then backward KDFT
    want, got, x = _both(dft, (40, 72, 96), dft.FFT, seed=7)
    assert np.array_equal(want.view(np.uint32), got.view(np.uint32))
    ref = orc.dft3d(x)
    assert np.linalg.norm((got - ref).ravel()) / np.linalg.norm(ref.ravel()) <= 2e-5
    want, got, _ = _both(dft, (33, 50, 17), dft.KDFT, seed=8, direction=dft.BACKWARD)
    assert np.array_equal(want.view(np.uint32), got.view(np.uint32))


def test_exec_noalloc_rejects_what_does_not_fit(dft):
    import torch

    lib = dft.load_library()
    shape = (256, 256, 128)                     # 64 MiB intermediate > 32 MiB scratch
    x = torch.zeros(shape, dtype=torch.complex64, device="cuda")
    out = torch.empty_like(x)
    with dft.Plan(shape, dft.KDFT) as p:
        assert p.workspace_bytes() > 32 << 20
        st = lib.dft3d_exec_noalloc(p._h, ctypes.c_void_p(x.data_ptr()), ctypes.c_void_p(out.data_ptr()),
                                    dft.FORWARD, None)
        assert lib.dft3d_status_string(st) == b"DFT3D_ERR_UNSUPPORTED"
        assert b"scratch" in lib.dft3d_last_error()
        with pytest.raises(dft.Dft3dError):
            p.exec_noalloc(x, out)
