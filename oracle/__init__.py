"""TEST INFRASTRUCTURE -- not part of the product path.

ctypes front end of the float64 CPU oracle in ``tfno_oracle.c`` (the plain
definition of the TurboFNO spectral convolution, Sec. 2.1 / 3.1 / 3.3 of the
paper).  Only tests, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of
``bench.py`` may import this package.  It imports nothing from the HIP package
and the HIP package imports nothing from here.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "tfno_oracle.c")
_LIB = os.path.join(_HERE, "libtfno_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (fp64, OpenMP over batch elements)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off",
               _SRC, "-o", _LIB, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        c_int, c_void = ctypes.c_int, ctypes.c_void_p
        for name in ("oracle_spectral_conv1d", "oracle_spectral_conv2d", "oracle_spectral_conv1d_permode",
                     "oracle_spectral_conv1d_real", "oracle_fno1d_real"):
            fn = getattr(lib, name)
            fn.restype = c_int
            fn.argtypes = [c_void, c_void, c_void] + [c_int] * 6
        for name in ("oracle_spectral_conv2d_rect", "oracle_spectral_conv2d_permode", "oracle_fno2d_real"):
            fn = getattr(lib, name)
            fn.restype = c_int
            fn.argtypes = [c_void, c_void, c_void] + [c_int] * 8
        lib.oracle_forward_spectrum1d.restype = c_int
        lib.oracle_forward_spectrum1d.argtypes = [c_void, c_void, c_int, c_int]
        for name in ("oracle_fft_c128", "oracle_fft_radix2_c128", "oracle_dft_direct_c128"):
            fn = getattr(lib, name)
            fn.restype = None
            fn.argtypes = [c_void, c_void, c_int, c_int]
        _lib = lib
    return _lib


def _c64(a: np.ndarray) -> np.ndarray:
    a = np.ascontiguousarray(a)
    if a.dtype != np.complex64:
        raise TypeError("oracle inputs are complex64 (the fp32 bits the GPU also reads)")
    return a


def spectral_conv1d(x: np.ndarray, W: np.ndarray, K: int, threads: int = 0):
    """y[B,C_out,N] (complex128) for x[B,C_in,N], W[C_in,C_out] (complex64).

    Returns (y, threads_used)."""
    x, W = _c64(x), _c64(W)
    B, C_in, N = x.shape
    C_in2, C_out = W.shape
    assert C_in2 == C_in
    y = np.empty((B, C_out, N), dtype=np.complex128)
    used = _load().oracle_spectral_conv1d(x.ctypes.data, W.ctypes.data, y.ctypes.data,
                                          B, C_in, C_out, N, K, threads)
    if used < 0:
        raise ValueError("oracle_spectral_conv1d: bad arguments")
    return y, used


def spectral_conv2d(x: np.ndarray, W: np.ndarray, K: int, threads: int = 0):
    """y[B,C_out,N,N] (complex128) for x[B,C_in,N,N], W[C_in,C_out] (complex64)."""
    x, W = _c64(x), _c64(W)
    B, C_in, N, N2 = x.shape
    assert N == N2
    C_in2, C_out = W.shape
    assert C_in2 == C_in
    y = np.empty((B, C_out, N, N), dtype=np.complex128)
    used = _load().oracle_spectral_conv2d(x.ctypes.data, W.ctypes.data, y.ctypes.data,
                                          B, C_in, C_out, N, K, threads)
    if used < 0:
        raise ValueError("oracle_spectral_conv2d: bad arguments")
    return y, used


def spectral_conv2d_rect(x: np.ndarray, W: np.ndarray, K1: int, K2: int, threads: int = 0):
    """y[B,C_out,N1,N2] (complex128) for x[B,C_in,N1,N2], W[C_in,C_out] (complex64); modes k1 < K1, k2 < K2."""
    x, W = _c64(x), _c64(W)
    B, C_in, N1, N2 = x.shape
    C_in2, C_out = W.shape
    assert C_in2 == C_in
    y = np.empty((B, C_out, N1, N2), dtype=np.complex128)
    used = _load().oracle_spectral_conv2d_rect(x.ctypes.data, W.ctypes.data, y.ctypes.data,
                                               B, C_in, C_out, N1, N2, K1, K2, threads)
    if used < 0:
        raise ValueError("oracle_spectral_conv2d_rect: bad arguments")
    return y, used


def spectral_conv1d_permode(x: np.ndarray, W: np.ndarray, threads: int = 0):
    """y[B,C_out,N] for x[B,C_in,N] and an own weight matrix per retained mode, W[C_in,C_out,K] (complex64)."""
    x, W = _c64(x), _c64(W)
    B, C_in, N = x.shape
    C_in2, C_out, K = W.shape
    assert C_in2 == C_in
    y = np.empty((B, C_out, N), dtype=np.complex128)
    used = _load().oracle_spectral_conv1d_permode(x.ctypes.data, W.ctypes.data, y.ctypes.data,
                                                  B, C_in, C_out, N, K, threads)
    if used < 0:
        raise ValueError("oracle_spectral_conv1d_permode: bad arguments")
    return y, used


def spectral_conv2d_permode(x: np.ndarray, W: np.ndarray, threads: int = 0):
    """y[B,C_out,N1,N2] for x[B,C_in,N1,N2] and per-mode weights W[C_in,C_out,K1,K2] (complex64)."""
    x, W = _c64(x), _c64(W)
    B, C_in, N1, N2 = x.shape
    C_in2, C_out, K1, K2 = W.shape
    assert C_in2 == C_in
    y = np.empty((B, C_out, N1, N2), dtype=np.complex128)
    used = _load().oracle_spectral_conv2d_permode(x.ctypes.data, W.ctypes.data, y.ctypes.data,
                                                  B, C_in, C_out, N1, N2, K1, K2, threads)
    if used < 0:
        raise ValueError("oracle_spectral_conv2d_permode: bad arguments")
    return y, used


def spectral_conv1d_real(x: np.ndarray, W: np.ndarray, K: int, threads: int = 0):
    """Real-valued layer: y[B,C_out,N] (float64) for REAL x[B,C_in,N] (float32), W[C_in,C_out] (complex64), K <= N/2."""
    x = np.ascontiguousarray(x)
    if x.dtype != np.float32:
        raise TypeError("the real-valued oracle takes float32 input (the bits the GPU also reads)")
    W = _c64(W)
    B, C_in, N = x.shape
    C_in2, C_out = W.shape
    assert C_in2 == C_in
    y = np.empty((B, C_out, N), dtype=np.float64)
    used = _load().oracle_spectral_conv1d_real(x.ctypes.data, W.ctypes.data, y.ctypes.data, B, C_in, C_out, N, K, threads)
    if used < 0:
        raise ValueError("oracle_spectral_conv1d_real: bad arguments")
    return y, used


def fno1d_real(x: np.ndarray, W: np.ndarray, threads: int = 0):
    """The 1-D Fourier layer of FNO models on real fields: x[B,C_in,N] float32, W[C_in,C_out,M] complex64 (one matrix
    per mode 0..M-1 of the half spectrum), y[B,C_out,N] float64."""
    x = np.ascontiguousarray(x)
    if x.dtype != np.float32:
        raise TypeError("x must be float32")
    W = _c64(W)
    B, C_in, N = x.shape
    C_in2, C_out, M = W.shape
    assert C_in2 == C_in
    y = np.empty((B, C_out, N), dtype=np.float64)
    used = _load().oracle_fno1d_real(x.ctypes.data, W.ctypes.data, y.ctypes.data, B, C_in, C_out, N, M, threads)
    if used < 0:
        raise ValueError("oracle_fno1d_real: bad arguments")
    return y, used


def fno2d_real(x: np.ndarray, W: np.ndarray, threads: int = 0):
    """The 2-D Fourier layer of FNO models on real fields: x[B,C_in,N1,N2] float32, W[C_in,C_out,2*M1,M2] complex64
    (first-axis frequencies -M1..M1-1 at index k1 + M1, last-axis 0..M2-1), y[B,C_out,N1,N2] float64."""
    x = np.ascontiguousarray(x)
    if x.dtype != np.float32:
        raise TypeError("x must be float32")
    W = _c64(W)
    B, C_in, N1, N2 = x.shape
    C_in2, C_out, J, M2 = W.shape
    assert C_in2 == C_in and J % 2 == 0
    y = np.empty((B, C_out, N1, N2), dtype=np.float64)
    used = _load().oracle_fno2d_real(x.ctypes.data, W.ctypes.data, y.ctypes.data, B, C_in, C_out, N1, N2, J // 2, M2, threads)
    if used < 0:
        raise ValueError("oracle_fno2d_real: bad arguments")
    return y, used


def forward_spectrum1d(x: np.ndarray) -> np.ndarray:
    """Untruncated, unscaled forward spectra of x[C,N] (complex64) -> complex128."""
    x = _c64(x)
    C, N = x.shape
    out = np.empty((C, N), dtype=np.complex128)
    if _load().oracle_forward_spectrum1d(x.ctypes.data, out.ctypes.data, C, N) != 0:
        raise ValueError("oracle_forward_spectrum1d: bad arguments")
    return out


def _xform(name: str, v: np.ndarray, sign: int) -> np.ndarray:
    v = np.ascontiguousarray(v, dtype=np.complex128)
    out = np.empty_like(v)
    getattr(_load(), name)(v.ctypes.data, out.ctypes.data, v.shape[0], sign)
    return out


def fft(v, sign=-1):
    """The transform the oracle uses (direct for N<=32 or non power of two, radix-2 else)."""
    return _xform("oracle_fft_c128", v, sign)


def fft_radix2(v, sign=-1):
    return _xform("oracle_fft_radix2_c128", v, sign)


def dft_direct(v, sign=-1):
    return _xform("oracle_dft_direct_c128", v, sign)
