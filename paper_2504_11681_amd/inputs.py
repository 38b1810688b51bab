"""Seeded synthetic inputs for the spectral-convolution workloads.

This module holds none of the method's arithmetic: it only draws the random
tensors that both the GPU path and the test oracle consume, so that both sides
read the same fp32 bits.  The paper evaluates on synthetic problem sizes only
(Sec. 5), so these tensors are the workload itself.

Recipe: x re/im ~ N(0, 1); W re/im ~ N(0, var = 1/C_in) (std 1/sqrt(C_in)), one
W[C_in, C_out] shared by all modes; values are drawn in float64 by NumPy's
PCG64 and rounded to float32 once.  Every batch element has its own stream
(seed, tag, b), so a test can regenerate a single batch element of a large
workload without materialising the rest.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np


@dataclass(frozen=True)
class Workload:
    name: str
    dims: int        # 1 or 2 transformed axes
    B: int
    C_in: int
    C_out: int
    N: int           # length of every transformed axis
    K: int           # retained low modes per transformed axis
    seed: int

    @property
    def spatial(self):
        return (self.N,) * self.dims

    @property
    def compulsory_bytes(self) -> int:
        """x read once + y written once + W read once, complex64."""
        pts = self.N ** self.dims
        return 8 * self.B * pts * (self.C_in + self.C_out) + 8 * self.C_in * self.C_out


# The five benchmark configurations (index = position in the baseline's list).
CONFIGS = [
    Workload("cfg1_1d_B4_C16_N64_K16", 1, 4, 16, 16, 64, 16, 0),
    Workload("cfg2_1d_B64_C64_N256_K64", 1, 64, 64, 64, 256, 64, 1),
    Workload("cfg3_1d_B256_C128_N1024_K128", 1, 256, 128, 128, 1024, 128, 2),
    Workload("cfg4_2d_B32_C64_N256x256_K64x64", 2, 32, 64, 64, 256, 64, 3),
]


def sweep_configs():
    """The hidden-dimension sweep: B=512, N=256, C in {32,64,128,256}, K in {32,64,128}, seed 4."""
    out = []
    for C in (32, 64, 128, 256):
        for K in (32, 64, 128):
            out.append(Workload(f"cfg5_1d_B512_C{C}_N256_K{K}", 1, 512, C, C, 256, K, 4))
    return out


_TAG_X, _TAG_W = 1, 2


def make_x_element(seed: int, b: int, C_in: int, spatial) -> np.ndarray:
    """Batch element b of x: complex64 [C_in, *spatial]."""
    rng = np.random.Generator(np.random.PCG64(np.random.SeedSequence([seed, _TAG_X, b])))
    shape = (C_in,) + tuple(spatial) + (2,)
    v = rng.standard_normal(shape, dtype=np.float32)
    return v.view(np.complex64)[..., 0]


def make_x(seed: int, B: int, C_in: int, spatial) -> np.ndarray:
    """x: complex64 [B, C_in, *spatial]."""
    out = np.empty((B, C_in) + tuple(spatial), dtype=np.complex64)
    for b in range(B):
        out[b] = make_x_element(seed, b, C_in, spatial)
    return out


def make_W(seed: int, C_in: int, C_out: int) -> np.ndarray:
    """W: complex64 [C_in, C_out], re/im ~ N(0, 1/C_in)."""
    rng = np.random.Generator(np.random.PCG64(np.random.SeedSequence([seed, _TAG_W])))
    v = rng.standard_normal((C_in, C_out, 2)) / np.sqrt(float(C_in))
    return v.astype(np.float32).view(np.complex64)[..., 0]


def make_workload(w: Workload):
    return make_x(w.seed, w.B, w.C_in, w.spatial), make_W(w.seed, w.C_in, w.C_out)
