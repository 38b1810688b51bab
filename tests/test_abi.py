"""CPU-side checks of the C ABI: the library loads, exports every declared symbol, and rejects bad
arguments on the host before any launch (no compute call needs a GPU here)."""
import ctypes
import os
import re

import pytest

from paper_2504_11681_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def L():
    if not os.path.exists(binding.LIB_PATH):
        from paper_2504_11681_amd import build
        build.build(verbose=False)
    return binding.lib()


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "tfno.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(tfno_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(L):
    names = declared_symbols()
    assert set(names) == set(binding.EXPORTS)
    for n in names:
        assert getattr(L, n) is not None


def test_version_and_status_strings(L):
    assert binding.version() >= 100
    seen = {binding.status_string(s) for s in range(8)}
    assert len(seen) == 8 and all(seen)


FAKE = 0x10000000  # never dereferenced: all of these calls fail validation before any launch


def call(L, name, x, W, y, B, Ci, Co, N, K):
    return getattr(L, name)(x, W, y, B, Ci, Co, N, K, None)


@pytest.mark.parametrize("name", binding.CONV_EXPORTS + ("tfno_spectral_conv1d_permode", "tfno_spectral_conv2d_noalloc"))
def test_argument_errors_are_caught_on_the_host(L, name):
    x, W, y = FAKE, FAKE + (1 << 26), FAKE + (2 << 26)
    assert call(L, name, None, W, y, 2, 4, 4, 64, 16) == binding.ERR_NULL
    assert call(L, name, x, None, y, 2, 4, 4, 64, 16) == binding.ERR_NULL
    assert call(L, name, x, W, None, 2, 4, 4, 64, 16) == binding.ERR_NULL
    any_n = name.endswith("_staged") or name.endswith("_auto")          # these also take N that is no power of two
    for bad in [(-1, 4, 4, 64, 16), (2, 0, 4, 64, 16), (2, 4, 0, 64, 16), (2, 4, 4, 48, 16), (2, 4, 4, 64, 0),
                (2, 4, 4, 64, 65), (2, 4, 4, 1, 1), (2, 4, 4, 8192, 16), (2, 4, 4, -64, 16), (2, 4, 4, 5000, 16)]:
        if any_n and bad[3] == 48:
            continue
        assert call(L, name, x, W, y, *bad) == binding.ERR_SHAPE, bad
    # y overlapping x or W
    assert call(L, name, x, W, x, 2, 4, 4, 64, 16) == binding.ERR_ALIAS
    assert call(L, name, x, W, x + 8, 2, 4, 4, 64, 16) == binding.ERR_ALIAS
    assert call(L, name, x, W, W, 2, 4, 4, 64, 16) == binding.ERR_ALIAS
    # complex64 elements move as 8-byte words
    for (dx, dw, dy) in ((4, 0, 0), (0, 4, 0), (0, 0, 4), (1, 0, 0)):
        assert call(L, name, x + dx, W + dw, y + dy, 2, 4, 4, 64, 16) == binding.ERR_ALIGN
    # empty batch: valid, nothing to do, pointers may be NULL
    assert call(L, name, None, None, None, 0, 4, 4, 64, 16) == binding.OK


@pytest.mark.parametrize("name", binding.RECT_EXPORTS + ("tfno_spectral_conv2d_strips",))
def test_rect_argument_errors_are_caught_on_the_host(L, name):
    x, W, y = FAKE, FAKE + (1 << 26), FAKE + (2 << 26)
    fn = getattr(L, name)
    good = (2, 4, 4, 64, 128, 16, 32)
    assert fn(None, W, y, *good, None) == binding.ERR_NULL
    assert fn(x, None, y, *good, None) == binding.ERR_NULL
    assert fn(x, W, None, *good, None) == binding.ERR_NULL
    for bad in [(-1, 4, 4, 64, 128, 16, 32), (2, 0, 4, 64, 128, 16, 32), (2, 4, 0, 64, 128, 16, 32),
                (2, 4, 4, 48, 128, 16, 32), (2, 4, 4, 64, 96, 16, 32), (2, 4, 4, 64, 128, 0, 32),
                (2, 4, 4, 64, 128, 16, 0), (2, 4, 4, 64, 128, 65, 32), (2, 4, 4, 64, 128, 16, 129),
                (2, 4, 4, 1, 128, 1, 32), (2, 4, 4, 64, 8192, 16, 32), (2, 4, 4, 128, 64, 16, 128)]:
        if name.endswith("_staged") and (bad[3] in (48, 96) or bad[4] in (48, 96)):
            continue                                                    # the staged twin takes any 2 <= N <= 4096
        assert fn(x, W, y, *bad, None) == binding.ERR_SHAPE, bad
    assert fn(x, W, x, *good, None) == binding.ERR_ALIAS
    assert fn(x, W, W, *good, None) == binding.ERR_ALIAS
    assert fn(None, None, None, 0, 4, 4, 64, 128, 16, 32, None) == binding.OK


def test_rect_workspace_and_unsupported_shapes(L):
    x, W, y = FAKE, FAKE + (1 << 26), FAKE + (2 << 26)
    # image kernels: truncated K1 x K2 spectra of input and output
    assert binding.workspace_bytes_2d(0, 2, 3, 5, 64, 256, 16, 64) == 8 * 2 * 16 * 64 * (3 + 5)
    # strip pipeline (K1 = 8 is not an image-kernel mode count): two [B, C, K1, N2] strips
    assert binding.workspace_bytes_2d(0, 2, 3, 5, 32, 256, 8, 64) == 8 * 2 * 8 * 256 * (3 + 5)
    assert binding.workspace_bytes_2d(0, 2, 3, 5, 64, 256, 12, 40) == 8 * 2 * 16 * 64 * (3 + 5)   # runs as 16 x 64
    assert binding.workspace_bytes_2d(1, 2, 3, 5, 32, 64, 8, 16) == 8 * 2 * (3 * 2048 + 3 * 128 + 5 * 128 + 5 * 2048)
    # the square case is the square entry point's
    assert binding.workspace_bytes_2d(0, 2, 3, 5, 64, 64, 16, 16) == binding.workspace_bytes(2, 0, 2, 3, 5, 64, 16)
    assert binding.workspace_bytes_2d(1, 2, 3, 5, 64, 64, 16, 16) == binding.workspace_bytes(2, 1, 2, 3, 5, 64, 16)
    assert binding.workspace_bytes_2d(0, 2, 3, 5, 48, 64, 16, 16) == 0
    assert binding.workspace_bytes_2d(2, 2, 3, 5, 64, 64, 16, 16) == 0        # the 1-D-only variants
    assert L.tfno_set_workspace(None, 0) == binding.OK
    assert L.tfno_spectral_conv2d_rect(x, W, y, 2, 4, 4, 64, 128, 16, 32, None) == binding.ERR_WORKSPACE
    # last axis not covered by the fused 1-D kernel and not an image-kernel shape
    assert L.tfno_spectral_conv2d_rect(x, W, y, 2, 4, 4, 64, 2048, 16, 32, None) == binding.ERR_UNSUPPORTED
    assert L.tfno_spectral_conv2d_rect(x, W, y, 2, 4, 4, 64, 32, 16, 8, None) == binding.ERR_UNSUPPORTED
    # the strip pipeline on request: strips also for a shape that the other entry point runs on the image kernels
    assert binding.workspace_bytes_2d(7, 2, 3, 5, 64, 256, 16, 64) == 8 * 2 * 16 * 256 * (3 + 5)
    assert binding.workspace_bytes_2d(7, 2, 3, 5, 32, 256, 5, 40) == 8 * 2 * 5 * 256 * (3 + 5)
    assert binding.workspace_bytes_2d(7, 2, 3, 5, 64, 2048, 16, 32) == 0
    assert binding.workspace_bytes(1, 7, 2, 3, 5, 256, 64) == 0                # 2-D only
    assert L.tfno_spectral_conv2d_strips(x, W, y, 2, 4, 4, 64, 128, 16, 32, None) == binding.ERR_WORKSPACE
    assert L.tfno_spectral_conv2d_strips(x, W, y, 2, 4, 4, 64, 2048, 16, 32, None) == binding.ERR_UNSUPPORTED


def test_real_layer_argument_checks(L):
    x, W, y = FAKE, FAKE + (1 << 26), FAKE + (2 << 26)
    f = L.tfno_spectral_conv1d_real
    assert f(None, W, y, 2, 4, 4, 64, 16, None) == binding.ERR_NULL
    assert f(x, W, y, 2, 4, 4, 64, 64, None) == binding.ERR_SHAPE          # K <= N / 2
    assert f(x, W, y, 2, 4, 4, 64, 33, None) == binding.ERR_SHAPE
    assert f(x, W, y, 2, 4, 4, 48, 16, None) == binding.ERR_SHAPE
    assert f(x, W, y, 2, 4, 4, 2048, 128, None) == binding.ERR_UNSUPPORTED
    assert f(x, W, y, 2, 4, 4, 32, 8, None) == binding.ERR_UNSUPPORTED
    assert f(x, W, y, 2, 4, 4, 1024, 300, None) == binding.ERR_UNSUPPORTED         # built sizes end at 256
    assert f(x, W, y, 2, 4, 4, 1024, 512, None) == binding.ERR_UNSUPPORTED
    # float tensors: y right behind x (4 B per element) does not overlap, y inside x does
    assert f(x, W, x + 4 * 2 * 4 * 64 - 4, 2, 4, 4, 64, 16, None) == binding.ERR_ALIAS
    assert f(x, W, W, 2, 4, 4, 64, 16, None) == binding.ERR_ALIAS
    # the real-valued kernels move pairs of floats
    assert f(x + 4, W, y, 2, 4, 4, 64, 16, None) == binding.ERR_ALIGN
    assert f(x, W, y + 4, 2, 4, 4, 64, 16, None) == binding.ERR_ALIGN
    assert f(None, None, None, 0, 4, 4, 64, 16, None) == binding.OK


def test_fno2d_argument_checks_and_workspace(L):
    x, W, y = FAKE, FAKE + (1 << 26), FAKE + (2 << 26)
    f = L.tfno_fno2d_real
    assert L.tfno_set_workspace(None, 0) == binding.OK
    assert f(None, W, y, 2, 4, 4, 64, 64, 12, 12, None) == binding.ERR_NULL
    assert f(x, W, y, 2, 4, 4, 64, 64, 33, 12, None) == binding.ERR_SHAPE           # 2 M1 <= N1
    assert f(x, W, y, 2, 4, 4, 64, 64, 12, 33, None) == binding.ERR_SHAPE           # 2 M2 <= N2
    assert f(x, W, y, 2, 4, 4, 48, 64, 12, 12, None) == binding.ERR_SHAPE
    assert f(x, W, y, 2, 4, 4, 512, 64, 12, 12, None) == binding.ERR_UNSUPPORTED
    assert f(x, W, y, 2, 4, 4, 256, 256, 40, 12, None) == binding.ERR_UNSUPPORTED   # 2 M1 > 64
    assert f(x, W, x, 2, 4, 4, 64, 64, 12, 12, None) == binding.ERR_ALIAS
    assert f(x, W, y + 4, 2, 4, 4, 64, 64, 12, 12, None) == binding.ERR_ALIGN
    assert f(x, W, y, 2, 4, 4, 64, 64, 12, 12, None) == binding.ERR_WORKSPACE
    assert f(None, None, None, 0, 4, 4, 64, 64, 12, 12, None) == binding.OK
    wsb = L.tfno_fno2d_real_workspace_bytes
    assert wsb(2, 3, 5, 64, 128, 12, 20) == 8 * 2 * 32 * 32 * (3 + 5)               # blocks of 24 x 20 run as 32 x 32
    assert wsb(2, 3, 5, 64, 128, 8, 16) == 8 * 2 * 16 * 16 * (3 + 5)
    assert wsb(2, 3, 5, 512, 128, 8, 16) == 0
    assert wsb(2, 3, 5, 64, 128, 40, 16) == 0


def test_fno1d_argument_checks_and_workspace(L):
    x, W, y = FAKE, FAKE + (1 << 26), FAKE + (2 << 26)
    f = L.tfno_fno1d_real
    assert L.tfno_set_workspace(None, 0) == binding.OK
    assert f(None, W, y, 2, 4, 4, 64, 12, None) == binding.ERR_NULL
    assert f(x, W, y, 2, 4, 4, 64, 33, None) == binding.ERR_SHAPE            # 2 M <= N
    assert f(x, W, y, 2, 4, 4, 512, 16, None) == binding.ERR_UNSUPPORTED
    assert f(x, W, y, 2, 4, 4, 1024, 200, None) == binding.ERR_UNSUPPORTED
    assert f(x, W, x, 2, 4, 4, 64, 12, None) == binding.ERR_ALIAS
    assert f(x + 4, W, y, 2, 4, 4, 64, 12, None) == binding.ERR_ALIGN
    assert f(x, W, y, 2, 4, 4, 64, 12, None) == binding.ERR_WORKSPACE
    assert f(None, None, None, 0, 4, 4, 64, 12, None) == binding.OK
    assert L.tfno_fno1d_real_workspace_bytes(4, 16, 16, 64, 12) == binding.workspace_bytes(1, 2, 4, 16, 16, 64, 16)
    assert L.tfno_fno1d_real_workspace_bytes(4, 16, 16, 512, 12) == 0


def test_fused_entry_points_report_unsupported_shapes(L):
    x, W, y = FAKE, FAKE + (1 << 26), FAKE + (2 << 26)
    assert call(L, "tfno_spectral_conv1d_permode", x, W, y, 2, 4, 4, 512, 64) == binding.ERR_UNSUPPORTED
    assert call(L, "tfno_spectral_conv1d_permode", x, W, y, 2, 4, 4, 4096, 512) == binding.ERR_UNSUPPORTED
    assert L.tfno_spectral_conv2d_permode(x, W, y, 2, 4, 4, 32, 256, 8, 64, None) == binding.ERR_UNSUPPORTED
    # the per-mode weight tensor is C_in * C_out * K elements long: y inside its tail is an alias
    assert call(L, "tfno_spectral_conv1d_permode", x, W, W + 8 * (4 * 4 * 16 - 1), 2, 4, 4, 64, 16) == binding.ERR_ALIAS
    assert call(L, "tfno_spectral_conv1d", x, W, y, 2, 4, 4, 2048, 128) == binding.ERR_UNSUPPORTED
    assert call(L, "tfno_spectral_conv1d", x, W, y, 2, 4, 4, 32, 8) == binding.ERR_UNSUPPORTED
    assert call(L, "tfno_spectral_conv1d", x, W, y, 2, 4, 4, 1024, 300) == binding.ERR_UNSUPPORTED     # K' = 512 > 256
    assert call(L, "tfno_spectral_conv1d_pruned", x, W, y, 2, 4, 4, 512, 64) == binding.ERR_UNSUPPORTED
    assert call(L, "tfno_spectral_conv2d", x, W, y, 2, 4, 4, 32, 8) == binding.ERR_UNSUPPORTED
    for name in ("tfno_spectral_conv1d_fft_gemm", "tfno_spectral_conv1d_gemm_ifft"):
        assert call(L, name, x, W, y, 2, 4, 4, 1024, 128) == binding.ERR_UNSUPPORTED
        assert call(L, name, x, W, y, 2, 4, 4, 256, 200) == binding.ERR_UNSUPPORTED                   # K' = 256
        assert call(L, name, x, W, y, 2, 4, 4, 64, 32) == binding.ERR_UNSUPPORTED


def test_workspace_contract(L):
    assert binding.workspace_bytes(1, False, 4, 16, 16, 64, 16) == 0
    assert binding.workspace_bytes(1, True, 4, 16, 16, 64, 16) == 8 * 4 * (16 * 64 + 16 * 16 + 16 * 16 + 16 * 64)
    # 2-D image kernels keep the truncated K x K spectra of input and output; the strip pipeline (shapes the
    # image kernels do not cover, here K = 8) keeps two [B, C, K, N] strips
    assert binding.workspace_bytes(2, False, 2, 3, 5, 64, 16) == 8 * 2 * 16 * 16 * (3 + 5)
    assert binding.workspace_bytes(2, False, 2, 3, 5, 64, 8) == 8 * 2 * 16 * 16 * (3 + 5)      # K = 8 runs as 16
    assert binding.workspace_bytes(2, False, 2, 3, 5, 512, 64) == 8 * 2 * 64 * 512 * (3 + 5)   # strip pipeline
    assert binding.workspace_bytes(2, True, 2, 3, 5, 64, 16) == 8 * 2 * (3 * 4096 + 3 * 256 + 5 * 256 + 5 * 4096)
    # pruned 1-D variant: truncated spectra of input and output, joint mode index padded to 128-mode tiles
    assert binding.workspace_bytes(1, 2, 4, 16, 16, 64, 16) == 8 * 128 * (16 + 16)
    assert binding.workspace_bytes(1, 2, 256, 128, 128, 1024, 128) == 8 * 256 * 128 * (128 + 128)
    # mode counts between the built sizes run on the next built size: K = 48 -> 64
    assert binding.workspace_bytes(1, 2, 4, 16, 16, 64, 48) == binding.workspace_bytes(1, 2, 4, 16, 16, 64, 64)
    assert binding.workspace_bytes(1, 2, 4, 16, 16, 512, 64) == 0         # no pruned kernels for N = 512
    assert binding.workspace_bytes(2, 2, 4, 16, 16, 64, 16) == 0          # 1-D only
    # partially fused variants: one truncated spectrum, the output's (3: FFT + CGEMM) or the input's (4: CGEMM + iFFT)
    assert binding.workspace_bytes(1, 3, 4, 16, 48, 256, 64) == 8 * 2 * 128 * 48
    assert binding.workspace_bytes(1, 4, 4, 16, 48, 256, 64) == 8 * 2 * 128 * 16
    assert binding.workspace_bytes(1, 3, 4, 16, 48, 1024, 64) == 0        # N in {128, 256} only
    assert binding.workspace_bytes(1, 4, 4, 16, 48, 256, 16) == binding.workspace_bytes(1, 4, 4, 16, 48, 256, 32)
    assert binding.workspace_bytes(1, 4, 4, 16, 48, 256, 200) == 0        # K in (128, 256]: no partially fused kernel
    # per-shape dispatch: the workspace of the variant it picks
    assert binding.workspace_bytes(1, 5, 4, 16, 48, 256, 64) == 0                         # fused
    assert binding.workspace_bytes(1, 5, 4, 16, 200, 256, 64) == 0                        # fused (256 outputs per workgroup)
    assert binding.workspace_bytes(1, 5, 4, 16, 200, 128, 64) == 0                        # N = 128, K = 64: fused
    assert binding.workspace_bytes(1, 5, 4, 16, 200, 128, 32) == 8 * 128 * 16             # N = 128, K = 32: CGEMM + iFFT
    assert binding.workspace_bytes(1, 5, 4, 16, 200, 128, 20) == 8 * 128 * 16             # ... also for K rounded up to 32
    assert binding.workspace_bytes(1, 5, 2, 3, 4, 2048, 100) == binding.workspace_bytes(1, 2, 2, 3, 4, 2048, 128)  # pruned, K' = 128
    assert binding.workspace_bytes(1, 5, 2, 3, 4, 32, 5) == binding.workspace_bytes(1, 1, 2, 3, 4, 32, 5)          # staged
    assert binding.workspace_bytes(1, 5, 2, 3, 4, 4096, 512) == binding.workspace_bytes(1, 2, 2, 3, 4, 4096, 512)  # pruned
    assert binding.workspace_bytes(1, 2, 2, 3, 4, 4096, 512) == 8 * 1024 * (3 + 4)
    assert binding.workspace_bytes(1, 2, 2, 3, 4, 2048, 64) == binding.workspace_bytes(1, 2, 2, 3, 4, 2048, 128)
    # per-mode weights: the pruned variant's buffers (1-D), the image kernels' (2-D)
    assert binding.workspace_bytes(1, 6, 4, 16, 48, 256, 64) == binding.workspace_bytes(1, 2, 4, 16, 48, 256, 64)
    assert binding.workspace_bytes(1, 6, 4, 16, 48, 2048, 256) == 0       # N <= 1024 only
    assert binding.workspace_bytes_2d(6, 2, 3, 5, 64, 256, 16, 64) == 8 * 2 * 16 * 64 * (3 + 5)
    assert binding.workspace_bytes_2d(6, 2, 3, 5, 32, 256, 8, 64) == 0    # image-kernel shapes only
    assert binding.workspace_bytes(1, 7, 4, 16, 48, 256, 64) == 0
    assert binding.workspace_bytes(3, True, 2, 3, 5, 64, 16) == 0
    assert binding.workspace_bytes(1, True, 2, 3, 5, 48, 16) == 8 * 2 * (3 * 48 + 3 * 16 + 5 * 16 + 5 * 48)   # staged: any N
    assert binding.workspace_bytes(1, False, 2, 3, 5, 48, 16) == 0
    assert binding.workspace_bytes(1, True, 2, 3, 5, 4097, 16) == 0
    x, W, y = FAKE, FAKE + (1 << 26), FAKE + (2 << 26)
    assert L.tfno_set_workspace(None, 0) == binding.OK
    # staged needs a workspace: none registered -> error, still no launch
    assert call(L, "tfno_spectral_conv1d_staged", x, W, y, 2, 4, 4, 64, 16) == binding.ERR_WORKSPACE
    assert call(L, "tfno_spectral_conv2d", x, W, y, 2, 4, 4, 64, 16) == binding.ERR_WORKSPACE
    need = binding.workspace_bytes(1, True, 2, 4, 4, 64, 16)
    ws = FAKE + (3 << 26)
    assert L.tfno_set_workspace(ws, need - 1) == binding.OK
    assert call(L, "tfno_spectral_conv1d_staged", x, W, y, 2, 4, 4, 64, 16) == binding.ERR_WORKSPACE
    assert L.tfno_set_workspace(ws + 4, need) == binding.ERR_SHAPE       # misaligned
    assert L.tfno_set_workspace(None, 16) == binding.ERR_NULL
    # workspace overlapping a tensor
    assert L.tfno_set_workspace(x, need) == binding.OK
    assert call(L, "tfno_spectral_conv1d_staged", x, W, y, 2, 4, 4, 64, 16) == binding.ERR_ALIAS
    assert L.tfno_set_workspace(None, 0) == binding.OK


def test_noalloc_entry_point_refuses_shapes_beyond_its_scratch_on_the_host(L):
    """The shape check of tfno_spectral_conv2d_noalloc runs before any HIP call: a shape whose intermediates exceed
    the built-in scratch array is TFNO_ERR_WORKSPACE."""
    x, W, y = FAKE, FAKE + (1 << 40), FAKE + (2 << 40)
    assert binding.workspace_bytes(2, 0, 32, 64, 64, 256, 64) > binding.NOALLOC_SCRATCH_BYTES
    assert L.tfno_spectral_conv2d_noalloc(x, W, y, 32, 64, 64, 256, 64, None) == binding.ERR_WORKSPACE
    text = open(os.path.join(ROOT, "include", "tfno.h")).read()
    m = re.search(r"#define TFNO_NOALLOC_SCRATCH_BYTES \((\d+)u << (\d+)\)", text)
    assert m and int(m.group(1)) << int(m.group(2)) == binding.NOALLOC_SCRATCH_BYTES
