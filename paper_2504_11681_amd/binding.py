"""ctypes binding of libtfno.so: argument marshalling only.

Every step of the spectral convolution runs inside the HIP library; PyTorch is used for device
allocation and streams.  The functions mirror the C ABI in ``include/tfno.h`` name for name.  There is
no CPU fallback: if the library has not been built, loading raises.
"""
from __future__ import annotations

import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libtfno.so")

OK, ERR_NULL, ERR_SHAPE, ERR_UNSUPPORTED, ERR_ALIAS, ERR_WORKSPACE, ERR_HIP, ERR_ALIGN = range(8)

EXPORTS = (
    "tfno_spectral_conv1d",
    "tfno_spectral_conv2d",
    "tfno_spectral_conv1d_staged",
    "tfno_spectral_conv2d_staged",
    "tfno_spectral_conv1d_pruned",
    "tfno_spectral_conv1d_fft_gemm",
    "tfno_spectral_conv1d_gemm_ifft",
    "tfno_spectral_conv1d_auto",
    "tfno_spectral_conv2d_rect",
    "tfno_spectral_conv2d_rect_staged",
    "tfno_spectral_conv2d_permode",
    "tfno_spectral_conv1d_permode",
    "tfno_spectral_conv1d_real",
    "tfno_fno2d_real",
    "tfno_fno2d_real_workspace_bytes",
    "tfno_fno1d_real",
    "tfno_fno1d_real_workspace_bytes",
    "tfno_spectral_conv2d_noalloc",
    "tfno_spectral_conv2d_strips",
    "tfno_workspace_bytes",
    "tfno_workspace_bytes_2d",
    "tfno_set_workspace",
    "tfno_status_string",
    "tfno_version",
)

CONV_EXPORTS = EXPORTS[:8]   # the entry points with the (x, W, y, B, C_in, C_out, N, K, stream) signature
RECT_EXPORTS = EXPORTS[8:11]  # (x, W, y, B, C_in, C_out, N1, N2, K1, K2, stream)

_lib = None
_workspace = None     # the torch tensor currently registered as workspace (kept alive here)


class TfnoError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)} (status {status})")


def lib() -> ctypes.CDLL:
    """Loads libtfno.so (built in-tree by ``python -m paper_2504_11681_amd.build``)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2504_11681_amd.build` "
                               "(there is no fallback path)")
        L = ctypes.CDLL(LIB_PATH)
        vp, ci = ctypes.c_void_p, ctypes.c_int
        for name in CONV_EXPORTS + ("tfno_spectral_conv1d_permode", "tfno_spectral_conv1d_real",
                                    "tfno_spectral_conv2d_noalloc"):
            fn = getattr(L, name)
            fn.restype = ci
            fn.argtypes = [vp, vp, vp, ci, ci, ci, ci, ci, vp]
        for name in RECT_EXPORTS + ("tfno_spectral_conv2d_strips",):
            fn = getattr(L, name)
            fn.restype = ci
            fn.argtypes = [vp, vp, vp] + [ci] * 7 + [vp]
        L.tfno_fno2d_real.restype = ci
        L.tfno_fno2d_real.argtypes = [vp, vp, vp] + [ci] * 7 + [vp]
        L.tfno_fno2d_real_workspace_bytes.restype = ctypes.c_size_t
        L.tfno_fno2d_real_workspace_bytes.argtypes = [ci] * 7
        L.tfno_fno1d_real.restype = ci
        L.tfno_fno1d_real.argtypes = [vp, vp, vp] + [ci] * 5 + [vp]
        L.tfno_fno1d_real_workspace_bytes.restype = ctypes.c_size_t
        L.tfno_fno1d_real_workspace_bytes.argtypes = [ci] * 5
        L.tfno_workspace_bytes.restype = ctypes.c_size_t
        L.tfno_workspace_bytes.argtypes = [ci] * 7
        L.tfno_workspace_bytes_2d.restype = ctypes.c_size_t
        L.tfno_workspace_bytes_2d.argtypes = [ci] * 8
        L.tfno_set_workspace.restype = ci
        L.tfno_set_workspace.argtypes = [vp, ctypes.c_size_t]
        L.tfno_status_string.restype = ctypes.c_char_p
        L.tfno_status_string.argtypes = [ci]
        L.tfno_version.restype = ci
        L.tfno_version.argtypes = []
        _lib = L
    return _lib


def status_string(status: int) -> str:
    return lib().tfno_status_string(status).decode()


def version() -> int:
    return lib().tfno_version()


def workspace_bytes(dims: int, variant, B: int, C_in: int, C_out: int, N: int, K: int) -> int:
    """variant: 0 / False = fused entry point, 1 / True = staged twin, 2 = spectral_conv1d_pruned,
    3 = spectral_conv1d_fft_gemm, 4 = spectral_conv1d_gemm_ifft, 5 = spectral_conv1d_auto,
    6 = spectral_conv1d_permode."""
    return lib().tfno_workspace_bytes(dims, int(variant), B, C_in, C_out, N, K)


def workspace_bytes_2d(variant, B: int, C_in: int, C_out: int, N1: int, N2: int, K1: int, K2: int) -> int:
    """2-D entry points with per-axis sizes: variant 0 / False = spectral_conv2d_rect, 1 / True = its staged
    twin, 6 = spectral_conv2d_permode."""
    return lib().tfno_workspace_bytes_2d(int(variant), B, C_in, C_out, N1, N2, K1, K2)


def set_workspace(tensor) -> None:
    """Registers a torch device tensor (any dtype) as the library workspace; None clears it."""
    global _workspace
    if tensor is None:
        st = lib().tfno_set_workspace(None, 0)
    else:
        st = lib().tfno_set_workspace(tensor.data_ptr(), tensor.numel() * tensor.element_size())
    if st != OK:
        raise TfnoError(st, "tfno_set_workspace")
    _workspace = tensor


def ensure_workspace(nbytes: int, device) -> None:
    """Makes sure a registered workspace of at least nbytes exists (allocates with torch if not).

    The workspace is one buffer per process, shared by every stream.  Before a larger one replaces it the device is
    synchronised, so no kernel enqueued earlier on any stream still reads or writes the old buffer when torch frees
    it.  A HIP graph captured with the old buffer keeps the old address: growing the workspace invalidates such
    graphs (capture after the largest shape has been run once, or register a buffer of the final size up front with
    ``set_workspace``)."""
    import torch
    if nbytes == 0:
        return
    if _workspace is None or _workspace.numel() * _workspace.element_size() < nbytes or _workspace.device != device:
        if _workspace is not None:
            torch.cuda.synchronize(_workspace.device)
        set_workspace(torch.empty(nbytes, dtype=torch.uint8, device=device))


def _call(name: str, dims: int, variant, x, W, y, K: int, stream):
    import torch
    for t, what in ((x, "x"), (W, "W"), (y, "y")):
        if t.dtype != torch.complex64 or not t.is_contiguous() or not t.is_cuda:
            raise TypeError(f"{what} must be a contiguous complex64 device tensor")
    if x.dim() != 2 + dims or y.dim() != 2 + dims or W.dim() != 2:
        raise ValueError("x, y must be [B, C, N] (1-D) or [B, C, N, N] (2-D); W must be [C_in, C_out]")
    B, C_in, N = x.shape[0], x.shape[1], x.shape[2]
    C_out = W.shape[1]
    if W.shape[0] != C_in or tuple(y.shape) != (B, C_out) + tuple(x.shape[2:]) or any(s != N for s in x.shape[2:]):
        raise ValueError("inconsistent tensor shapes")
    ensure_workspace(workspace_bytes(dims, variant, B, C_in, C_out, N, K), x.device)
    if stream is None:
        stream = torch.cuda.current_stream(x.device).cuda_stream
    st = getattr(lib(), name)(x.data_ptr(), W.data_ptr(), y.data_ptr(), B, C_in, C_out, N, K, stream)
    if st != OK:
        raise TfnoError(st, name)
    return y


def spectral_conv1d(x, W, y, K: int, stream=None):
    return _call("tfno_spectral_conv1d", 1, False, x, W, y, K, stream)


def spectral_conv2d(x, W, y, K: int, stream=None):
    return _call("tfno_spectral_conv2d", 2, False, x, W, y, K, stream)


NOALLOC_SCRATCH_BYTES = 32 << 20     # TFNO_NOALLOC_SCRATCH_BYTES of the header


def spectral_conv2d_noalloc(x, W, y, K: int, stream=None):
    """tfno_spectral_conv2d with the library's own scratch array: allocates nothing and registers no workspace."""
    import torch
    for t, what in ((x, "x"), (W, "W"), (y, "y")):
        if t.dtype != torch.complex64 or not t.is_contiguous() or not t.is_cuda:
            raise TypeError(f"{what} must be a contiguous complex64 device tensor")
    if x.dim() != 4 or y.dim() != 4 or W.dim() != 2 or x.shape[2] != x.shape[3]:
        raise ValueError("x, y must be [B, C, N, N]; W must be [C_in, C_out]")
    B, C_in, N = x.shape[0], x.shape[1], x.shape[2]
    C_out = W.shape[1]
    if W.shape[0] != C_in or tuple(y.shape) != (B, C_out, N, N):
        raise ValueError("inconsistent tensor shapes")
    if stream is None:
        stream = torch.cuda.current_stream(x.device).cuda_stream
    st = lib().tfno_spectral_conv2d_noalloc(x.data_ptr(), W.data_ptr(), y.data_ptr(), B, C_in, C_out, N, K, stream)
    if st != OK:
        raise TfnoError(st, "tfno_spectral_conv2d_noalloc")
    return y


def spectral_conv1d_staged(x, W, y, K: int, stream=None):
    return _call("tfno_spectral_conv1d_staged", 1, True, x, W, y, K, stream)


def spectral_conv2d_staged(x, W, y, K: int, stream=None):
    return _call("tfno_spectral_conv2d_staged", 2, True, x, W, y, K, stream)


def spectral_conv1d_pruned(x, W, y, K: int, stream=None):
    return _call("tfno_spectral_conv1d_pruned", 1, 2, x, W, y, K, stream)


def spectral_conv1d_fft_gemm(x, W, y, K: int, stream=None):
    return _call("tfno_spectral_conv1d_fft_gemm", 1, 3, x, W, y, K, stream)


def spectral_conv1d_gemm_ifft(x, W, y, K: int, stream=None):
    return _call("tfno_spectral_conv1d_gemm_ifft", 1, 4, x, W, y, K, stream)


def spectral_conv1d_auto(x, W, y, K: int, stream=None):
    return _call("tfno_spectral_conv1d_auto", 1, 5, x, W, y, K, stream)


def _call_rect(name: str, variant, x, W, y, K1: int, K2: int, stream):
    import torch
    for t, what in ((x, "x"), (W, "W"), (y, "y")):
        if t.dtype != torch.complex64 or not t.is_contiguous() or not t.is_cuda:
            raise TypeError(f"{what} must be a contiguous complex64 device tensor")
    if x.dim() != 4 or y.dim() != 4 or W.dim() != 2:
        raise ValueError("x, y must be [B, C, N1, N2]; W must be [C_in, C_out]")
    B, C_in, N1, N2 = x.shape
    C_out = W.shape[1]
    if W.shape[0] != C_in or tuple(y.shape) != (B, C_out, N1, N2):
        raise ValueError("inconsistent tensor shapes")
    ensure_workspace(workspace_bytes_2d(variant, B, C_in, C_out, N1, N2, K1, K2), x.device)
    if stream is None:
        stream = torch.cuda.current_stream(x.device).cuda_stream
    st = getattr(lib(), name)(x.data_ptr(), W.data_ptr(), y.data_ptr(), B, C_in, C_out, N1, N2, K1, K2, stream)
    if st != OK:
        raise TfnoError(st, name)
    return y


def spectral_conv2d_rect(x, W, y, K1: int, K2: int, stream=None):
    return _call_rect("tfno_spectral_conv2d_rect", False, x, W, y, K1, K2, stream)


def spectral_conv2d_rect_staged(x, W, y, K1: int, K2: int, stream=None):
    return _call_rect("tfno_spectral_conv2d_rect_staged", True, x, W, y, K1, K2, stream)


def spectral_conv2d_strips(x, W, y, K1: int, K2: int, stream=None):
    """The paper's 2-D pipeline on request (first-axis FFT, fused 1-D kernel on the retained rows, first-axis iFFT)."""
    return _call_rect("tfno_spectral_conv2d_strips", 7, x, W, y, K1, K2, stream)


def _call_permode(name: str, dims: int, x, W, y, stream):
    import torch
    for t, what in ((x, "x"), (W, "W"), (y, "y")):
        if t.dtype != torch.complex64 or not t.is_contiguous() or not t.is_cuda:
            raise TypeError(f"{what} must be a contiguous complex64 device tensor")
    if x.dim() != 2 + dims or y.dim() != 2 + dims or W.dim() != 2 + dims:
        raise ValueError("x, y must be [B, C, spatial...]; W must be [C_in, C_out, modes...]")
    B, C_in = x.shape[0], x.shape[1]
    C_out = W.shape[1]
    if W.shape[0] != C_in or tuple(y.shape) != (B, C_out) + tuple(x.shape[2:]):
        raise ValueError("inconsistent tensor shapes")
    if stream is None:
        stream = torch.cuda.current_stream(x.device).cuda_stream
    if dims == 1:
        N, K = x.shape[2], W.shape[2]
        ensure_workspace(workspace_bytes(1, 6, B, C_in, C_out, N, K), x.device)
        st = lib().tfno_spectral_conv1d_permode(x.data_ptr(), W.data_ptr(), y.data_ptr(), B, C_in, C_out, N, K, stream)
    else:
        N1, N2, K1, K2 = x.shape[2], x.shape[3], W.shape[2], W.shape[3]
        ensure_workspace(workspace_bytes_2d(6, B, C_in, C_out, N1, N2, K1, K2), x.device)
        st = lib().tfno_spectral_conv2d_permode(x.data_ptr(), W.data_ptr(), y.data_ptr(), B, C_in, C_out, N1, N2, K1, K2,
                                                stream)
    if st != OK:
        raise TfnoError(st, name)
    return y


def spectral_conv1d_permode(x, W, y, stream=None):
    """W: [C_in, C_out, K], an own weight matrix per retained mode."""
    return _call_permode("tfno_spectral_conv1d_permode", 1, x, W, y, stream)


def spectral_conv2d_permode(x, W, y, stream=None):
    """W: [C_in, C_out, K1, K2]."""
    return _call_permode("tfno_spectral_conv2d_permode", 2, x, W, y, stream)


def spectral_conv1d_real(x, W, y, K: int, stream=None):
    """Real-valued layer: x [B, C_in, N] and y [B, C_out, N] float32 device tensors, W [C_in, C_out] complex64."""
    import torch
    if x.dtype != torch.float32 or y.dtype != torch.float32 or W.dtype != torch.complex64:
        raise TypeError("x, y must be float32 and W complex64")
    for t, what in ((x, "x"), (W, "W"), (y, "y")):
        if not t.is_contiguous() or not t.is_cuda:
            raise TypeError(f"{what} must be a contiguous device tensor")
    if x.dim() != 3 or y.dim() != 3 or W.dim() != 2:
        raise ValueError("x, y must be [B, C, N]; W must be [C_in, C_out]")
    B, C_in, N = x.shape
    C_out = W.shape[1]
    if W.shape[0] != C_in or tuple(y.shape) != (B, C_out, N):
        raise ValueError("inconsistent tensor shapes")
    if stream is None:
        stream = torch.cuda.current_stream(x.device).cuda_stream
    st = lib().tfno_spectral_conv1d_real(x.data_ptr(), W.data_ptr(), y.data_ptr(), B, C_in, C_out, N, K, stream)
    if st != OK:
        raise TfnoError(st, "tfno_spectral_conv1d_real")
    return y


def fno2d_real(x, W, y, stream=None):
    """The 2-D Fourier layer of FNO models on real fields: x [B, C_in, N1, N2] and y [B, C_out, N1, N2] float32,
    W [C_in, C_out, 2*M1, M2] complex64 (first-axis frequencies -M1..M1-1, last-axis 0..M2-1)."""
    import torch
    if x.dtype != torch.float32 or y.dtype != torch.float32 or W.dtype != torch.complex64:
        raise TypeError("x, y must be float32 and W complex64")
    for t, what in ((x, "x"), (W, "W"), (y, "y")):
        if not t.is_contiguous() or not t.is_cuda:
            raise TypeError(f"{what} must be a contiguous device tensor")
    if x.dim() != 4 or y.dim() != 4 or W.dim() != 4 or W.shape[2] % 2:
        raise ValueError("x, y must be [B, C, N1, N2]; W must be [C_in, C_out, 2*M1, M2]")
    B, C_in, N1, N2 = x.shape
    C_out, M1, M2 = W.shape[1], W.shape[2] // 2, W.shape[3]
    if W.shape[0] != C_in or tuple(y.shape) != (B, C_out, N1, N2):
        raise ValueError("inconsistent tensor shapes")
    ensure_workspace(lib().tfno_fno2d_real_workspace_bytes(B, C_in, C_out, N1, N2, M1, M2), x.device)
    if stream is None:
        stream = torch.cuda.current_stream(x.device).cuda_stream
    st = lib().tfno_fno2d_real(x.data_ptr(), W.data_ptr(), y.data_ptr(), B, C_in, C_out, N1, N2, M1, M2, stream)
    if st != OK:
        raise TfnoError(st, "tfno_fno2d_real")
    return y


def fno1d_real(x, W, y, stream=None):
    """The 1-D Fourier layer of FNO models on real fields: x [B, C_in, N], y [B, C_out, N] float32,
    W [C_in, C_out, M] complex64 (one matrix per mode 0..M-1)."""
    import torch
    if x.dtype != torch.float32 or y.dtype != torch.float32 or W.dtype != torch.complex64:
        raise TypeError("x, y must be float32 and W complex64")
    for t, what in ((x, "x"), (W, "W"), (y, "y")):
        if not t.is_contiguous() or not t.is_cuda:
            raise TypeError(f"{what} must be a contiguous device tensor")
    if x.dim() != 3 or y.dim() != 3 or W.dim() != 3:
        raise ValueError("x, y must be [B, C, N]; W must be [C_in, C_out, M]")
    B, C_in, N = x.shape
    C_out, M = W.shape[1], W.shape[2]
    if W.shape[0] != C_in or tuple(y.shape) != (B, C_out, N):
        raise ValueError("inconsistent tensor shapes")
    ensure_workspace(lib().tfno_fno1d_real_workspace_bytes(B, C_in, C_out, N, M), x.device)
    if stream is None:
        stream = torch.cuda.current_stream(x.device).cuda_stream
    st = lib().tfno_fno1d_real(x.data_ptr(), W.data_ptr(), y.data_ptr(), B, C_in, C_out, N, M, stream)
    if st != OK:
        raise TfnoError(st, "tfno_fno1d_real")
    return y
