"""Seeded synthetic inputs for the five benchmark configurations, shared by tests and bench.

This module holds NO transform arithmetic: it only draws random tensors and coordinates and
names the workloads.  It serves both the HIP path and the CPU oracle so that they see the
same bits.  The paper uses no dataset (its inputs are unspecified arrays of the sizes in its
evaluation section), so every input here is a stand-in with the shapes, value distributions
and grid structure the configurations name.

seed = 200203260 + (1-based configuration index).
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Optional, Tuple

import numpy as np

SEED_BASE = 200203260

KDFT = 0
FFT = 1


@dataclass(frozen=True)
class Workload:
    name: str
    index: int                      # 1-based configuration index
    shape: Tuple[int, int, int]
    formulation: int                # KDFT or FFT (cfg 5 runs both)
    dist: str                       # "uniform" = U[-1,1), "normal" = N(0,1)
    nonuniform: bool = False
    splits: Optional[Tuple[Tuple[int, int], ...]] = None   # (A, B) per axis for FFT

    @property
    def seed(self) -> int:
        return SEED_BASE + self.index

    @property
    def elements(self) -> int:
        return int(np.prod(self.shape, dtype=np.int64))


WORKLOADS = {
    "cfg1": Workload("cfg1_kdft_32", 1, (32, 32, 32), KDFT, "uniform"),
    "cfg2": Workload("cfg2_kdft_256", 2, (256, 256, 256), KDFT, "normal"),
    "cfg3": Workload("cfg3_fft_512", 3, (512, 512, 512), FFT, "normal",
                     splits=((16, 32),) * 3),
    "cfg4": Workload("cfg4_kdft_nonuniform_128", 4, (128, 128, 128), KDFT, "uniform",
                     nonuniform=True),
    "cfg5": Workload("cfg5_2048", 5, (2048, 2048, 2048), KDFT, "normal",
                     splits=((16, 128),) * 3),
}

# Beyond the five configurations: the paper's two-dimensional size (Section IV, strong-scaling
# figure of the 2-D KDFT), given as a 3-D shape whose first axis has length 1.
EXTRA_WORKLOADS = {
    "2d-8192": Workload("next_2d_8192", 6, (1, 8192, 8192), KDFT, "normal",
                        splits=((1, 1), (4, 2048), (4, 2048))),
}


def draw_complex(shape, dist: str, seed: int) -> np.ndarray:
    """complex64 tensor whose real and imaginary parts are iid ``dist`` from ``seed``."""
    rng = np.random.default_rng(seed)
    n = int(np.prod(shape, dtype=np.int64))
    if dist == "uniform":
        buf = rng.random(2 * n, dtype=np.float32) * np.float32(2.0) - np.float32(1.0)
    elif dist == "normal":
        buf = rng.standard_normal(2 * n, dtype=np.float32)
    else:
        raise ValueError(dist)
    return buf.view(np.complex64).reshape(shape)


def draw_complex128(shape, seed: int) -> np.ndarray:
    """complex128 tensor with iid N(0,1) real and imaginary parts (full fp64 mantissas)."""
    rng = np.random.default_rng(seed)
    n = int(np.prod(shape, dtype=np.int64))
    return rng.standard_normal(2 * n).view(np.complex128).reshape(shape)


def make_input(w: Workload) -> np.ndarray:
    """Host input tensor of a workload (not for cfg5: 64 GiB does not fit a host array here)."""
    if w.elements > (1 << 30):
        raise ValueError("use make_input_device for tensors this large")
    return draw_complex(w.shape, w.dist, w.seed)


def make_coords(w: Workload):
    """Per-axis sample coordinates: None for uniform axes, else sorted iid U[0,1) fp64."""
    if not w.nonuniform:
        return (None, None, None)
    rng = np.random.default_rng(w.seed + 1000)
    return tuple(np.sort(rng.random(n)) for n in w.shape)


def make_input_device(w: Workload, device="cuda", out=None):
    """Input generated on the device plane by plane from a seeded torch generator (into the tensor
    ``out`` when one is given: the same values, no new allocation).

    Used for tensors the host cannot hold; whoever needs the values on the host reads them
    back from the device, so the generator need not be reproducible elsewhere."""
    import torch

    n1, n2, n3 = w.shape
    if out is not None:
        if tuple(out.shape) != (n1, n2, n3) or out.dtype != torch.complex64 or not out.is_contiguous():
            raise ValueError("out must be a contiguous complex64 tensor of the workload's shape")
        device = out.device
    g = torch.Generator(device=device)
    g.manual_seed(w.seed)
    x = out if out is not None else torch.empty((n1, n2, n3), dtype=torch.complex64, device=device)
    xr = torch.view_as_real(x)
    chunk = max(1, (1 << 27) // (n2 * n3))
    for a0 in range(0, n1, chunk):
        a1 = min(n1, a0 + chunk)
        if w.dist == "normal":
            xr[a0:a1].normal_(0.0, 1.0, generator=g)
        else:
            xr[a0:a1].uniform_(-1.0, 1.0, generator=g)
    return x


def gaussian_integers(shape, seed: int, lo: int = -3, hi: int = 4) -> np.ndarray:
    """complex64 tensor with small integer real and imaginary parts (exact-arithmetic tests)."""
    rng = np.random.default_rng(seed)
    re = rng.integers(lo, hi, size=shape).astype(np.float32)
    im = rng.integers(lo, hi, size=shape).astype(np.float32)
    return (re + 1j * im).astype(np.complex64)
