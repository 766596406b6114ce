"""ctypes binding of libdft3d.so.  Argument marshalling only: every step runs in the library.

Tensors are torch complex64 CUDA(HIP) tensors, contiguous, shape (nx, ny, nz); the binding
passes ``data_ptr()`` and the current torch stream's handle.  torch is used for device memory
and streams only.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence

import numpy as np

from . import build as _build

KDFT = 0
FFT = 1
FORWARD = -1
BACKWARD = 1
FLAG_CLOBBER_INPUT = 1
FLAG_UNFUSED = 2
FLAG_3M = 4
FLAG_BF16X3 = 8
FLAG_COMPLEX128 = 16
FLAG_ADJOINT = 32

EXPORTS = [
    "dft3d_plan_create", "dft3d_plan_create_ex", "dft3d_plan_create_points",
    "dft3d_plan_get_output_shape", "dft3d_generate_points_matrix", "dft3d_plan_destroy",
    "dft3d_plan_workspace_bytes", "dft3d_plan_set_workspace", "dft3d_plan_get_split", "dft3d_plan_axis_order", "dft3d_plan_mode_kernel",
    "dft3d_exec", "dft3d_exec_noalloc", "dft3d_plan_enable_profiling", "dft3d_plan_read_profile", "dft3d_mode_contract", "dft3d_fft_first_stage", "dft3d_fft_phase",
    "dft3d_fft_second_stage", "dft3d_fft_axis", "dft3d_fft_reorder", "dft3d_device_copy", "dft3d_generate_matrix",
    "dft3d_generate_twiddle", "dft3d_status_string", "dft3d_last_error",
]

_lib = None


class Dft3dError(RuntimeError):
    def __init__(self, status: int, name: str, message: str):
        super().__init__(f"{name}: {message}")
        self.status = status
        self.status_name = name


def library_path() -> str:
    return _build.lib_path()


def load_library():
    """Load libdft3d.so (built beforehand by build.build()); raises if it is missing."""
    global _lib
    if _lib is not None:
        return _lib
    path = library_path()
    if not os.path.exists(path):
        raise FileNotFoundError(
            f"{path} has not been built; run `python -m paper_2002_03260_amd.build` "
            "(or __graft_entry__.build()) first -- there is no fallback path")
    lib = ctypes.CDLL(path)
    vp, i64, ci, u32 = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int, ctypes.c_uint32
    lib.dft3d_plan_create.argtypes = [ctypes.POINTER(vp), i64, i64, i64, ci, vp, vp, vp]
    lib.dft3d_plan_create_ex.argtypes = [ctypes.POINTER(vp), i64, i64, i64, ci, vp, vp, vp, vp, u32]
    lib.dft3d_plan_create_points.argtypes = [ctypes.POINTER(vp), i64, i64, i64, i64, i64, i64, vp, vp, vp, u32]
    lib.dft3d_plan_get_output_shape.argtypes = [vp, ctypes.POINTER(i64), ctypes.POINTER(i64), ctypes.POINTER(i64)]
    lib.dft3d_generate_points_matrix.argtypes = [i64, i64, vp, vp, vp]
    lib.dft3d_plan_destroy.argtypes = [vp]
    lib.dft3d_plan_workspace_bytes.argtypes = [vp]
    lib.dft3d_plan_workspace_bytes.restype = ctypes.c_size_t
    lib.dft3d_plan_set_workspace.argtypes = [vp, vp, ctypes.c_size_t]
    lib.dft3d_plan_get_split.argtypes = [vp, ci, ctypes.POINTER(i64), ctypes.POINTER(i64)]
    lib.dft3d_plan_axis_order.argtypes = [vp, ctypes.POINTER(ci)]
    lib.dft3d_plan_mode_kernel.argtypes = [vp, ci, ctypes.c_char_p, ctypes.c_size_t]
    lib.dft3d_exec.argtypes = [vp, vp, vp, ci, vp]
    lib.dft3d_exec_noalloc.argtypes = [vp, vp, vp, ci, vp]
    lib.dft3d_plan_enable_profiling.argtypes = [vp, ci]
    lib.dft3d_plan_read_profile.argtypes = [vp, ci, ctypes.POINTER(ctypes.c_float), ctypes.POINTER(ci)]
    lib.dft3d_mode_contract.argtypes = [vp, ci, vp, vp, ci, vp]
    lib.dft3d_fft_first_stage.argtypes = [vp, ci, vp, vp, ci, ci, vp]
    lib.dft3d_fft_phase.argtypes = [vp, ci, vp, vp, ci, vp]
    lib.dft3d_fft_second_stage.argtypes = [vp, ci, vp, vp, ci, ci, vp]
    lib.dft3d_fft_axis.argtypes = [vp, ci, vp, vp, ci, vp]
    lib.dft3d_fft_reorder.argtypes = [vp, ci, vp, vp, vp]
    lib.dft3d_device_copy.argtypes = [vp, vp, ctypes.c_size_t, ci, vp]
    lib.dft3d_generate_matrix.argtypes = [i64, vp, ci, vp, vp]
    lib.dft3d_generate_twiddle.argtypes = [i64, i64, ci, vp, vp]
    for name in EXPORTS:
        fn = getattr(lib, name)
        if name in ("dft3d_status_string", "dft3d_last_error"):
            fn.restype = ctypes.c_char_p
        elif name != "dft3d_plan_workspace_bytes":
            fn.restype = ctypes.c_int
    lib.dft3d_status_string.argtypes = [ci]
    lib.dft3d_last_error.argtypes = []
    _lib = lib
    return lib


def _check(status: int):
    if status != 0:
        lib = load_library()
        raise Dft3dError(status, lib.dft3d_status_string(status).decode(),
                         lib.dft3d_last_error().decode())


def _host_coords(c, n):
    if c is None:
        return None
    a = np.ascontiguousarray(c, dtype=np.float64)
    if a.shape != (n,):
        raise ValueError(f"coordinate array must have shape ({n},)")
    return a


def _np_ptr(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def generate_matrix(n: int, coords=None, direction: int = FORWARD) -> np.ndarray:
    """The n x n axis matrix exactly as the library rounds it (host call, complex64)."""
    c = _host_coords(coords, n)
    re = np.empty((n, n), np.float32)
    im = np.empty((n, n), np.float32)
    _check(load_library().dft3d_generate_matrix(n, _np_ptr(c), direction, _np_ptr(re), _np_ptr(im)))
    return (re + 1j * im).astype(np.complex64)


def generate_points_matrix(z, n: int) -> np.ndarray:
    """The K x n Vandermonde matrix z_r**(-j) as the library rounds it (host call, complex64)."""
    z = np.ascontiguousarray(z, dtype=np.complex128)
    K = z.shape[0]
    re = np.empty((K, n), np.float32)
    im = np.empty((K, n), np.float32)
    _check(load_library().dft3d_generate_points_matrix(K, n, _np_ptr(z), _np_ptr(re), _np_ptr(im)))
    return (re + 1j * im).astype(np.complex64)


def generate_twiddle(A: int, B: int, direction: int = FORWARD) -> np.ndarray:
    """The A x B twiddle table T[k_a, beta] as the library rounds it (host call, complex64)."""
    re = np.empty((A, B), np.float32)
    im = np.empty((A, B), np.float32)
    _check(load_library().dft3d_generate_twiddle(A, B, direction, _np_ptr(re), _np_ptr(im)))
    return (re + 1j * im).astype(np.complex64)


def _stream_handle(stream) -> Optional[int]:
    import torch

    s = torch.cuda.current_stream() if stream is None else stream
    return ctypes.c_void_p(s.cuda_stream)


def device_copy(src, dst, variant: int = 0, stream=None):
    """Copy one contiguous CUDA tensor into another of the same byte size with the library's copy kernel."""
    nbytes = src.numel() * src.element_size()
    if nbytes != dst.numel() * dst.element_size():
        raise ValueError("size mismatch")
    _check(load_library().dft3d_device_copy(ctypes.c_void_p(src.data_ptr()), ctypes.c_void_p(dst.data_ptr()),
                                            nbytes, variant, _stream_handle(stream)))
    return dst


class Plan:
    """Owns one dft3d_plan.  Methods mirror the C entry points one to one."""

    def __init__(self, shape: Sequence[int], formulation: int = KDFT, coords=(None, None, None),
                 split: Optional[Sequence[int]] = None, flags: int = 0, points=None):
        self._lib = load_library()
        self._h = ctypes.c_void_p()
        self.shape = tuple(int(s) for s in shape)
        if len(self.shape) != 3:
            raise ValueError("shape must have three entries")
        self.formulation = formulation
        self.flags = flags
        self.out_shape = self.shape
        self._workspace = None
        if points is not None:
            # general form of the transform: arbitrary evaluation points per axis (None = roots of unity)
            zs = [None if z is None else np.ascontiguousarray(z, dtype=np.complex128) for z in points]
            ks = [n if z is None else int(z.shape[0]) for z, n in zip(zs, self.shape)]
            _check(self._lib.dft3d_plan_create_points(ctypes.byref(self._h), *self.shape, *ks,
                                                      _np_ptr(zs[0]), _np_ptr(zs[1]), _np_ptr(zs[2]), flags))
            self.out_shape = tuple(ks)
            if flags & FLAG_ADJOINT:      # `shape` describes the forward transform; the adjoint maps back
                self.shape, self.out_shape = self.out_shape, self.shape
            return
        cs = [_host_coords(c, n) for c, n in zip(coords, self.shape)]
        sp = None
        if split is not None:
            sp = (ctypes.c_int64 * 3)(*[int(s) for s in split])
        _check(self._lib.dft3d_plan_create_ex(ctypes.byref(self._h), *self.shape, formulation,
                                              _np_ptr(cs[0]), _np_ptr(cs[1]), _np_ptr(cs[2]),
                                              ctypes.cast(sp, ctypes.c_void_p) if sp else None,
                                              flags))

    # -- lifetime ---------------------------------------------------------------------------
    def destroy(self):
        if getattr(self, "_h", None) is not None and self._h:
            self._lib.dft3d_plan_destroy(self._h)
            self._h = ctypes.c_void_p()
        self._workspace = None

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass

    def __enter__(self):
        return self

    def __exit__(self, *exc):
        self.destroy()

    # -- workspace --------------------------------------------------------------------------
    def workspace_bytes(self) -> int:
        return int(self._lib.dft3d_plan_workspace_bytes(self._h))

    def set_workspace(self, tensor):
        """Give the plan a torch CUDA tensor as workspace (kept alive by this object)."""
        nbytes = 0 if tensor is None else tensor.numel() * tensor.element_size()
        ptr = None if tensor is None else ctypes.c_void_p(tensor.data_ptr())
        _check(self._lib.dft3d_plan_set_workspace(self._h, ptr, nbytes))
        self._workspace = tensor

    def ensure_workspace(self, device="cuda"):
        import torch

        need = self.workspace_bytes()
        if need and self._workspace is None:
            self.set_workspace(torch.empty(need // 8, dtype=torch.complex64, device=device))

    def split(self, axis: int):
        a, b = ctypes.c_int64(), ctypes.c_int64()
        _check(self._lib.dft3d_plan_get_split(self._h, axis, ctypes.byref(a), ctypes.byref(b)))
        return int(a.value), int(b.value)

    def axis_order(self):
        """Axes in the order dft3d_exec transforms them."""
        order = (ctypes.c_int * 3)()
        _check(self._lib.dft3d_plan_axis_order(self._h, order))
        return tuple(int(v) for v in order)

    def mode_kernel(self, axis: int) -> str:
        """Name of the kernel family that contracts mode ``axis`` of a KDFT plan; for an FFT plan, how
        exec transforms the axis ("fused", "butterflies + fused second stage", ...)."""
        buf = ctypes.create_string_buffer(64)
        _check(self._lib.dft3d_plan_mode_kernel(self._h, axis, buf, len(buf)))
        return buf.value.decode()

    # -- per-pass timing -------------------------------------------------------------------
    def enable_profiling(self, max_execs: int):
        _check(self._lib.dft3d_plan_enable_profiling(self._h, int(max_execs)))

    def read_profile(self, exec_index: int):
        """Milliseconds of each kernel of exec number ``exec_index`` (stream must be synchronised)."""
        ms = (ctypes.c_float * 16)()
        n = ctypes.c_int()
        _check(self._lib.dft3d_plan_read_profile(self._h, int(exec_index), ms, ctypes.byref(n)))
        return [float(ms[i]) for i in range(n.value)]

    # -- execution --------------------------------------------------------------------------
    def _tensors(self, x, out, in_shape=None, out_shape=None):
        import torch

        in_shape = self.shape if in_shape is None else in_shape
        out_shape = self.out_shape if out_shape is None else out_shape
        dtype = torch.complex128 if (self.flags & FLAG_COMPLEX128) else torch.complex64
        if x.dtype != dtype or not x.is_cuda or not x.is_contiguous():
            raise ValueError(f"input must be a contiguous {dtype} CUDA tensor")
        if tuple(x.shape) != tuple(in_shape):
            raise ValueError(f"input shape {tuple(x.shape)} does not match {tuple(in_shape)}")
        if out is None:
            out = torch.empty(tuple(out_shape), dtype=dtype, device=x.device)
        elif (out.dtype != dtype or not out.is_cuda or not out.is_contiguous()
              or tuple(out.shape) != tuple(out_shape)):
            raise ValueError(f"output must be a contiguous {dtype} CUDA tensor of shape {tuple(out_shape)}")
        return ctypes.c_void_p(x.data_ptr()), ctypes.c_void_p(out.data_ptr()), out

    def stage_shapes(self, axis):
        """Shapes mode_contract reads and writes for ``axis`` (modes are applied z, y, x)."""
        n, k = self.shape, self.out_shape
        cur = [n[j] if j <= axis else k[j] for j in range(3)]
        nxt = list(cur)
        nxt[axis] = k[axis]
        return tuple(cur), tuple(nxt)

    def exec(self, x, out=None, direction: int = FORWARD, stream=None):
        xi, oi, out = self._tensors(x, out)
        if self.workspace_bytes():
            self.ensure_workspace(x.device)
        _check(self._lib.dft3d_exec(self._h, xi, oi, direction, _stream_handle(stream)))
        return out

    def exec_noalloc(self, x, out, direction: int = FORWARD, stream=None):
        """dft3d_exec_noalloc: the intermediate lives in the library's static scratch array; the caller
        brings the output tensor and nothing is allocated."""
        xi, oi, out = self._tensors(x, out)
        _check(self._lib.dft3d_exec_noalloc(self._h, xi, oi, direction, _stream_handle(stream)))
        return out

    def mode_contract(self, axis, x, out=None, direction: int = FORWARD, stream=None):
        xi, oi, out = self._tensors(x, out, *self.stage_shapes(axis))
        _check(self._lib.dft3d_mode_contract(self._h, axis, xi, oi, direction, _stream_handle(stream)))
        return out

    def fft_first_stage(self, axis, x, out=None, direction: int = FORWARD, fuse_twiddle: bool = True,
                        stream=None):
        xi, oi, out = self._tensors(x, out)
        _check(self._lib.dft3d_fft_first_stage(self._h, axis, xi, oi, direction,
                                               1 if fuse_twiddle else 0, _stream_handle(stream)))
        return out

    def fft_phase(self, axis, x, out=None, direction: int = FORWARD, stream=None):
        xi, oi, out = self._tensors(x, out)
        _check(self._lib.dft3d_fft_phase(self._h, axis, xi, oi, direction, _stream_handle(stream)))
        return out

    def fft_second_stage(self, axis, x, out=None, direction: int = FORWARD, reorder: bool = False,
                         stream=None):
        xi, oi, out = self._tensors(x, out)
        _check(self._lib.dft3d_fft_second_stage(self._h, axis, xi, oi, direction,
                                                1 if reorder else 0, _stream_handle(stream)))
        return out

    def fft_axis(self, axis, x, out=None, direction: int = FORWARD, stream=None):
        xi, oi, out = self._tensors(x, out)
        _check(self._lib.dft3d_fft_axis(self._h, axis, xi, oi, direction, _stream_handle(stream)))
        return out

    def fft_reorder(self, axes_mask, x, out=None, stream=None):
        xi, oi, out = self._tensors(x, out)
        _check(self._lib.dft3d_fft_reorder(self._h, axes_mask, xi, oi, _stream_handle(stream)))
        return out
