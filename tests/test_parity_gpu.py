"""Parity of the HIP path (through the C ABI) against the float64 oracle on the same seeded inputs.

Tolerance (fp32 path vs fp64 oracle): relative L2 error <= 1e-5 and max abs error <= 1e-4 * max|y|.
"""
import sys

import numpy as np
import pytest

from paper_2504_11681_amd import inputs

pytestmark = pytest.mark.gpu

REL_L2, MAX_ABS = 1e-5, 1e-4


@pytest.fixture(scope="module")
def gpu():
    import torch
    from paper_2504_11681_amd import binding
    assert torch.cuda.is_available(), "these tests need the MI355X"
    binding.lib()   # fails loudly when the HIP library is missing
    return torch, binding


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def check(got: np.ndarray, want: np.ndarray, what=""):
    got = got.astype(np.complex128)
    err = got - want
    rel = np.linalg.norm(err.ravel()) / np.linalg.norm(want.ravel())
    mx = np.max(np.abs(err)) / np.max(np.abs(want))
    say(f"   {what}: rel_l2={rel:.3e} max_abs/max|y|={mx:.3e}")
    assert rel <= REL_L2, f"{what}: relative L2 {rel:.3e}"
    assert mx <= MAX_ABS, f"{what}: max abs {mx:.3e}"


def close(got, want, what):
    """Both halves of the tolerance, silently (for the sweeps)."""
    err = np.asarray(got) - want
    rel = np.linalg.norm(err.ravel()) / np.linalg.norm(want.ravel())
    mx = np.max(np.abs(err)) / np.max(np.abs(want))
    assert rel <= REL_L2, f"{what}: relative L2 {rel:.3e}"
    assert mx <= MAX_ABS, f"{what}: max abs {mx:.3e}"


def run_gpu(gpu, fn_name, x, W, K):
    torch, binding = gpu
    xd = torch.from_numpy(x).cuda()
    Wd = torch.from_numpy(W).cuda()
    yd = torch.full((x.shape[0], W.shape[1]) + x.shape[2:], float("nan"), dtype=torch.complex64, device="cuda")
    getattr(binding, fn_name)(xd, Wd, yd, K)
    torch.cuda.synchronize()
    return yd.cpu().numpy()


def oracle_fn(oracle_mod, dims):
    return oracle_mod.spectral_conv1d if dims == 1 else oracle_mod.spectral_conv2d


# (B, C_in, C_out, N, K): several tiles, ragged channel counts, every supported N of the fused kernel
SMALL_1D = [
    (4, 16, 16, 64, 16),        # benchmark configuration 1
    (3, 5, 7, 64, 8),
    (2, 33, 40, 64, 64),        # K = N: no truncation
    (3, 9, 70, 128, 32),
    (2, 37, 17, 128, 128),
    (64, 64, 64, 256, 64),      # benchmark configuration 2
    (5, 19, 130, 256, 32),
    (2, 40, 33, 256, 16),
    (3, 24, 96, 256, 128),
    (3, 32, 96, 256, 64),       # whole channel blocks, but the last 128-output slab is only partly there
    (2, 64, 96, 128, 32),
    (2, 16, 160, 256, 32),
    (2, 20, 40, 256, 256),
    (3, 21, 66, 512, 64),
    (2, 35, 10, 512, 256),
    (2, 16, 100, 512, 32),
    (3, 13, 129, 1024, 128),
    (2, 20, 30, 1024, 32),
    (2, 9, 64, 1024, 256),
    (1, 1, 1, 1024, 64),
    (2, 32, 128, 1024, 128),
    (1, 48, 256, 1024, 64),
    (2, 16, 128, 1024, 128),
    (128, 16, 128, 1024, 64),   # half a chip of workgroups: the symmetric-wave kernel by default (below: the four-wave one)
    (70, 9, 130, 1024, 128),    # ... with masks (70 rows x 2 slabs)
    (130, 16, 64, 1024, 64),    # at most 64 outputs: the four-wave kernel whatever the batch
    (130, 16, 65, 1024, 64),    # one output more: the symmetric-wave kernel, slab half empty
]


@pytest.mark.parametrize("shape", SMALL_1D, ids=lambda s: "B%d_Ci%d_Co%d_N%d_K%d" % s)
@pytest.mark.parametrize("fn", ["spectral_conv1d", "spectral_conv1d_staged"])
def test_1d_small(gpu, oracle_mod, fn, shape):
    B, Ci, Co, N, K = shape
    say(f"[case] {fn} {shape}")
    x = inputs.make_x(100 + N + K, B, Ci, (N,))
    W = inputs.make_W(100 + N + K, Ci, Co)
    want, _ = oracle_mod.spectral_conv1d(x, W, K)
    got = run_gpu(gpu, fn, x, W, K)
    check(got, want, fn)


# unfused variant with pruned transforms (three kernels): narrow path N <= 256, wide path N = 1024
PRUNED_1D = [(4, 16, 16, 64, 16), (3, 5, 7, 64, 64), (2, 33, 40, 64, 32), (3, 9, 70, 128, 32), (2, 37, 17, 128, 128),
             (2, 5, 3, 128, 16), (64, 64, 64, 256, 64), (5, 19, 130, 256, 32), (2, 40, 33, 256, 16), (3, 24, 96, 256, 128),
             (2, 20, 40, 256, 256), (3, 13, 129, 1024, 128), (1, 1, 1, 1024, 64), (2, 20, 30, 1024, 64),
             (7, 3, 2, 256, 16),
             # 64 < C_in <= 128: the contraction with all of W resident in LDS (ragged channels and outputs, an odd
             # number of mode tiles, several tile pairs per workgroup, whole blocks)
             (5, 70, 65, 256, 64), (3, 97, 130, 1024, 128), (600, 128, 128, 256, 128), (9, 128, 64, 256, 128), (2, 100, 20, 128, 64),
             # long pencils (N1 x 256 decomposition): odd pencil counts, K / N1 from 16 to 256, no truncation
             (2, 5, 7, 2048, 128), (3, 3, 5, 2048, 256), (1, 1, 1, 2048, 2048), (2, 8, 8, 2048, 1024),
             (2, 6, 9, 4096, 256), (1, 3, 2, 4096, 1024), (1, 2, 2, 4096, 4096), (2, 33, 70, 4096, 512),
             (1, 4, 4, 2048, 512), (1, 2, 3, 4096, 2048)]


@pytest.mark.parametrize("shape", PRUNED_1D, ids=lambda s: "B%d_Ci%d_Co%d_N%d_K%d" % s)
def test_1d_pruned_variant(gpu, oracle_mod, shape):
    B, Ci, Co, N, K = shape
    say(f"[case] spectral_conv1d_pruned {shape}")
    x = inputs.make_x(300 + N + K, B, Ci, (N,))
    W = inputs.make_W(300 + N + K, Ci, Co)
    want, _ = oracle_mod.spectral_conv1d(x, W, K)
    check(run_gpu(gpu, "spectral_conv1d_pruned", x, W, K), want, "pruned")


# partially fused variants (FFT + CGEMM kernel then pruned inverse; pruned forward then CGEMM + iFFT kernel)
PARTIAL_1D = [(3, 20, 40, 256, 64), (2, 16, 128, 256, 32), (1, 33, 65, 256, 128), (2, 8, 32, 128, 32),
              (3, 13, 129, 128, 64), (2, 32, 64, 128, 128), (5, 1, 1, 256, 32), (2, 64, 96, 256, 128),
              (70, 16, 32, 256, 64)]


@pytest.mark.parametrize("fn", ["spectral_conv1d_fft_gemm", "spectral_conv1d_gemm_ifft"])
@pytest.mark.parametrize("shape", PARTIAL_1D, ids=lambda s: "B%d_Ci%d_Co%d_N%d_K%d" % s)
def test_1d_partially_fused_variants(gpu, oracle_mod, shape, fn):
    B, Ci, Co, N, K = shape
    say(f"[case] {fn} {shape}")
    x = inputs.make_x(500 + N + K, B, Ci, (N,))
    W = inputs.make_W(500 + N + K, Ci, Co)
    want, _ = oracle_mod.spectral_conv1d(x, W, K)
    check(run_gpu(gpu, fn, x, W, K), want, fn)


# per-shape dispatch: CGEMM + iFFT variant (C_out > 128 where it exists), fused kernel, pruned kernels for long
# pencils, staged path
AUTO_1D = [(2, 16, 256, 256, 64), (3, 20, 130, 128, 32), (2, 16, 64, 256, 64), (2, 9, 200, 1024, 128),
           (2, 4, 4, 2048, 100), (2, 5, 3, 256, 48), (2, 40, 300, 256, 128), (2, 9, 20, 4096, 512), (3, 5, 6, 2048, 256)]


@pytest.mark.parametrize("shape", AUTO_1D, ids=lambda s: "B%d_Ci%d_Co%d_N%d_K%d" % s)
def test_1d_auto_dispatch(gpu, oracle_mod, shape):
    B, Ci, Co, N, K = shape
    say(f"[case] spectral_conv1d_auto {shape}")
    x = inputs.make_x(600 + N + K, B, Ci, (N,))
    W = inputs.make_W(600 + N + K, Ci, Co)
    want, _ = oracle_mod.spectral_conv1d(x, W, K)
    check(run_gpu(gpu, "spectral_conv1d_auto", x, W, K), want, "auto")


def random_shapes(seed, count):
    """Seeded random shapes (B, C_in, C_out, N, K) that every 1-D entry point accepts, small enough for the oracle."""
    rng = np.random.default_rng(seed)
    out = []
    for _ in range(count):
        N = int(rng.choice([128, 256]))
        K = int(rng.choice([k for k in (32, 64, 128) if k <= N]))
        out.append((int(rng.integers(1, 6)), int(rng.integers(1, 80)), int(rng.integers(1, 300)), N, K))
    return out


@pytest.mark.parametrize("shape", random_shapes(2025, 12), ids=lambda s: "B%d_Ci%d_Co%d_N%d_K%d" % s)
def test_1d_random_shapes_all_entry_points(gpu, oracle_mod, shape):
    """Every 1-D entry point on the same random shape (odd channel counts exercise all the masks)."""
    B, Ci, Co, N, K = shape
    x = inputs.make_x(700 + Ci + Co, B, Ci, (N,))
    W = inputs.make_W(700 + Ci + Co, Ci, Co)
    want, _ = oracle_mod.spectral_conv1d(x, W, K)
    for fn in ("spectral_conv1d", "spectral_conv1d_auto", "spectral_conv1d_pruned", "spectral_conv1d_fft_gemm",
               "spectral_conv1d_gemm_ifft", "spectral_conv1d_staged"):
        say(f"[case] {fn} random {shape}")
        check(run_gpu(gpu, fn, x, W, K), want, fn)


def test_1d_pruned_unsupported_shapes(gpu):
    torch, binding = gpu
    for (N, K) in [(512, 64), (32, 8), (1024, 200), (16, 16)]:
        x = torch.zeros((1, 2, N), dtype=torch.complex64, device="cuda")
        W = torch.zeros((2, 2), dtype=torch.complex64, device="cuda")
        y = torch.zeros((1, 2, N), dtype=torch.complex64, device="cuda")
        with pytest.raises(binding.TfnoError) as e:
            binding.spectral_conv1d_pruned(x, W, y, K)
        assert e.value.status == binding.ERR_UNSUPPORTED, (N, K)


STAGED_ONLY_1D = [(2, 3, 4, 2, 1), (2, 3, 4, 4, 3), (3, 6, 5, 32, 5), (2, 4, 4, 2048, 100), (1, 2, 3, 4096, 4096),
                  (2, 5, 3, 256, 48),
                  # lengths that are not powers of two (direct-sum transform)
                  (2, 3, 4, 3, 2), (3, 5, 4, 48, 12), (2, 4, 6, 421, 24), (1, 3, 2, 1000, 1000), (2, 2, 2, 85, 85),
                  (1, 2, 2, 4095, 7)]


@pytest.mark.parametrize("shape", STAGED_ONLY_1D, ids=lambda s: "B%d_Ci%d_Co%d_N%d_K%d" % s)
def test_1d_staged_general_shapes(gpu, oracle_mod, shape):
    B, Ci, Co, N, K = shape
    say(f"[case] staged {shape}")
    x = inputs.make_x(7, B, Ci, (N,))
    W = inputs.make_W(7, Ci, Co)
    want, _ = oracle_mod.spectral_conv1d(x, W, K)
    check(run_gpu(gpu, "spectral_conv1d_staged", x, W, K), want, "staged")


# image kernels (N in {64,128,256}, K in {16,32,64}) and, for the other shapes, the strip pipeline
SMALL_2D = [(2, 3, 5, 64, 16), (1, 8, 8, 64, 8), (2, 5, 33, 128, 32), (1, 4, 3, 256, 64), (1, 2, 2, 64, 64),
            (1, 3, 2, 64, 32), (1, 3, 2, 128, 16), (2, 2, 2, 128, 64), (1, 2, 3, 256, 16), (1, 2, 2, 256, 32),
            (3, 7, 70, 256, 64), (1, 2, 2, 128, 128), (1, 2, 2, 512, 64)]


@pytest.mark.parametrize("shape", SMALL_2D, ids=lambda s: "B%d_Ci%d_Co%d_N%d_K%d" % s)
@pytest.mark.parametrize("fn", ["spectral_conv2d", "spectral_conv2d_staged"])
def test_2d_small(gpu, oracle_mod, fn, shape):
    B, Ci, Co, N, K = shape
    say(f"[case] {fn} {shape}")
    x = inputs.make_x(200 + N + K, B, Ci, (N, N))
    W = inputs.make_W(200 + N + K, Ci, Co)
    want, _ = oracle_mod.spectral_conv2d(x, W, K)
    check(run_gpu(gpu, fn, x, W, K), want, fn)


def test_staged_lengths_that_are_not_powers_of_two(gpu, oracle_mod):
    """2-D staged twin on 85 x 48 and 421 x 12 grids, and the 1-D per-shape dispatch falling back to the staged path."""
    for (B, Ci, Co, N1, N2, K1, K2) in [(2, 3, 2, 85, 48, 12, 12), (1, 2, 3, 12, 421, 5, 20), (1, 2, 2, 64, 100, 16, 30)]:
        say(f"[case] staged rect {(B, Ci, Co, N1, N2, K1, K2)}")
        x = inputs.make_x(1500 + N1 + N2, B, Ci, (N1, N2))
        W = inputs.make_W(1500 + N1 + N2, Ci, Co)
        want, _ = oracle_mod.spectral_conv2d_rect(x, W, K1, K2)
        check(run_gpu_rect(gpu, "spectral_conv2d_rect_staged", x, W, K1, K2), want, "staged rect, any N")
    x = inputs.make_x(1501, 2, 3, (300,))
    W = inputs.make_W(1501, 3, 4)
    want, _ = oracle_mod.spectral_conv1d(x, W, 40)
    check(run_gpu(gpu, "spectral_conv1d_auto", x, W, 40), want, "auto, N = 300")


def test_2d_staged_general_shape(gpu, oracle_mod):
    B, Ci, Co, N, K = 2, 3, 2, 32, 5
    x = inputs.make_x(9, B, Ci, (N, N))
    W = inputs.make_W(9, Ci, Co)
    want, _ = oracle_mod.spectral_conv2d(x, W, K)
    check(run_gpu(gpu, "spectral_conv2d_staged", x, W, K), want, "staged2d")


def run_gpu_rect(gpu, fn_name, x, W, K1, K2):
    torch, binding = gpu
    xd = torch.from_numpy(x).cuda()
    Wd = torch.from_numpy(W).cuda()
    yd = torch.full((x.shape[0], W.shape[1]) + x.shape[2:], float("nan"), dtype=torch.complex64, device="cuda")
    getattr(binding, fn_name)(xd, Wd, yd, K1, K2)
    torch.cuda.synchronize()
    return yd.cpu().numpy()


# every (N1, N2, K1, K2) instantiation of the image kernels
RECT_IMAGE = [(n1, n2, k1, k2) for n1 in (64, 128, 256) for n2 in (64, 128, 256) for k1 in (16, 32, 64)
              for k2 in (16, 32, 64)]


@pytest.mark.parametrize("shape", RECT_IMAGE, ids=lambda s: "N%dx%d_K%dx%d" % s)
def test_2d_rect_image_kernels(gpu, oracle_mod, shape):
    N1, N2, K1, K2 = shape
    B, Ci, Co = 2, 3, 2
    say(f"[case] spectral_conv2d_rect {shape}")
    x = inputs.make_x(300 + N1 + 2 * N2 + K1 + 3 * K2, B, Ci, (N1, N2))
    W = inputs.make_W(300 + N1 + 2 * N2 + K1 + 3 * K2, Ci, Co)
    want, _ = oracle_mod.spectral_conv2d_rect(x, W, K1, K2)
    check(run_gpu_rect(gpu, "spectral_conv2d_rect", x, W, K1, K2), want, "rect")


# (B, C_in, C_out, N1, N2, K1, K2): ragged channels on the image kernels, strip-pipeline shapes (first axis or mode
# count outside the image kernels' set), and shapes only the staged twin takes
RECT_MIXED = [(3, 7, 70, 64, 256, 16, 64), (2, 33, 5, 256, 64, 64, 16), (1, 66, 130, 128, 256, 32, 16),
              (2, 3, 4, 32, 256, 8, 64), (1, 2, 3, 512, 64, 100, 16), (2, 3, 2, 16, 1024, 16, 128),
              (1, 2, 2, 1024, 128, 64, 128), (2, 2, 3, 2, 64, 1, 8)]
RECT_STAGED_ONLY = [(2, 3, 2, 8, 32, 3, 5), (1, 2, 2, 64, 16, 64, 16), (2, 2, 3, 128, 4, 7, 2), (1, 1, 1, 2, 2048, 2, 100)]


@pytest.mark.parametrize("shape", RECT_MIXED, ids=lambda s: "B%d_Ci%d_Co%d_N%dx%d_K%dx%d" % s)
@pytest.mark.parametrize("fn", ["spectral_conv2d_rect", "spectral_conv2d_rect_staged"])
def test_2d_rect_mixed(gpu, oracle_mod, fn, shape):
    B, Ci, Co, N1, N2, K1, K2 = shape
    say(f"[case] {fn} {shape}")
    x = inputs.make_x(400 + N1 + K2, B, Ci, (N1, N2))
    W = inputs.make_W(400 + N1 + K2, Ci, Co)
    want, _ = oracle_mod.spectral_conv2d_rect(x, W, K1, K2)
    check(run_gpu_rect(gpu, fn, x, W, K1, K2), want, fn)


# the paper's 2-D pipeline on request: image-kernel shapes (where the default entry point takes the other path), shapes
# it serves anyway, modes between the built sizes on both axes
STRIPS_2D = [(3, 7, 70, 64, 256, 16, 64), (2, 33, 5, 256, 64, 64, 16), (2, 8, 8, 64, 64, 16, 16), (2, 3, 4, 32, 256, 8, 64),
             (1, 5, 3, 128, 128, 20, 12), (2, 16, 16, 256, 256, 64, 64)]


@pytest.mark.parametrize("shape", STRIPS_2D, ids=lambda s: "B%d_Ci%d_Co%d_N%dx%d_K%dx%d" % s)
def test_2d_strip_pipeline_on_request(gpu, oracle_mod, shape):
    B, Ci, Co, N1, N2, K1, K2 = shape
    say(f"[case] spectral_conv2d_strips {shape}")
    x = inputs.make_x(450 + N1 + K2, B, Ci, (N1, N2))
    W = inputs.make_W(450 + N1 + K2, Ci, Co)
    want, _ = oracle_mod.spectral_conv2d_rect(x, W, K1, K2)
    check(run_gpu_rect(gpu, "spectral_conv2d_strips", x, W, K1, K2), want, "strips")


@pytest.mark.parametrize("shape", RECT_STAGED_ONLY, ids=lambda s: "B%d_Ci%d_Co%d_N%dx%d_K%dx%d" % s)
def test_2d_rect_staged_general_shapes(gpu, oracle_mod, shape):
    torch, binding = gpu
    B, Ci, Co, N1, N2, K1, K2 = shape
    say(f"[case] staged rect {shape}")
    x = inputs.make_x(500 + N1 + K2, B, Ci, (N1, N2))
    W = inputs.make_W(500 + N1 + K2, Ci, Co)
    want, _ = oracle_mod.spectral_conv2d_rect(x, W, K1, K2)
    check(run_gpu_rect(gpu, "spectral_conv2d_rect_staged", x, W, K1, K2), want, "staged rect")
    with pytest.raises(binding.TfnoError) as e:
        run_gpu_rect(gpu, "spectral_conv2d_rect", x, W, K1, K2)
    assert e.value.status == binding.ERR_UNSUPPORTED


def test_2d_rect_square_case_is_bitwise_the_square_entry_point(gpu):
    x = inputs.make_x(77, 2, 5, (128, 128))
    W = inputs.make_W(77, 5, 6)
    a = run_gpu_rect(gpu, "spectral_conv2d_rect", x, W, 32, 32)
    b = run_gpu(gpu, "spectral_conv2d", x, W, 32)
    assert np.array_equal(a.view(np.float32), b.view(np.float32))


# per-mode weights (B, C_in, C_out, N, K): several batch groups, ragged channels, K below / equal / above one tile
PERMODE_1D = [(4, 16, 16, 64, 16), (19, 5, 7, 64, 64), (9, 33, 40, 128, 32), (3, 9, 70, 128, 128), (17, 6, 18, 256, 256),
              (1, 1, 1, 256, 16), (2, 20, 30, 1024, 64), (11, 13, 17, 1024, 128), (8, 3, 2, 256, 128),
              # mode counts between the built sizes (weights hold exactly K matrices)
              (3, 5, 7, 64, 12), (9, 9, 4, 256, 100), (4, 6, 6, 1024, 72), (2, 3, 3, 128, 1),
              # batches and output counts that fill 64 x 64 tiles per mode (ragged last tiles, channel mask, surplus modes)
              (250, 16, 128, 256, 128), (256, 9, 120, 256, 100)]


@pytest.mark.parametrize("shape", PERMODE_1D, ids=lambda s: "B%d_Ci%d_Co%d_N%d_K%d" % s)
def test_1d_permode(gpu, oracle_mod, shape):
    torch, binding = gpu
    B, Ci, Co, N, K = shape
    say(f"[case] spectral_conv1d_permode {shape}")
    x = inputs.make_x(700 + N + K, B, Ci, (N,))
    W = np.ascontiguousarray(inputs.make_W(700 + N + K, Ci, Co * K).reshape(Ci, Co, K))
    want, _ = oracle_mod.spectral_conv1d_permode(x, W)
    xd, Wd = torch.from_numpy(x).cuda(), torch.from_numpy(W).cuda()
    yd = torch.full((B, Co, N), float("nan"), dtype=torch.complex64, device="cuda")
    binding.spectral_conv1d_permode(xd, Wd, yd)
    torch.cuda.synchronize()
    check(yd.cpu().numpy(), want, "permode 1d")


# (B, C_in, C_out, N1, N2, K1, K2)
PERMODE_2D = [(2, 3, 5, 64, 64, 16, 16), (9, 5, 33, 128, 64, 32, 16), (1, 4, 3, 256, 256, 64, 64), (10, 2, 2, 64, 256, 16, 64),
              (3, 17, 9, 128, 128, 64, 32), (2, 3, 4, 64, 128, 12, 20), (9, 2, 3, 256, 64, 33, 5),
              (120, 20, 112, 64, 64, 16, 16)]


@pytest.mark.parametrize("shape", PERMODE_2D, ids=lambda s: "B%d_Ci%d_Co%d_N%dx%d_K%dx%d" % s)
def test_2d_permode(gpu, oracle_mod, shape):
    torch, binding = gpu
    B, Ci, Co, N1, N2, K1, K2 = shape
    say(f"[case] spectral_conv2d_permode {shape}")
    x = inputs.make_x(800 + N1 + K2, B, Ci, (N1, N2))
    W = np.ascontiguousarray(inputs.make_W(800 + N1 + K2, Ci, Co * K1 * K2).reshape(Ci, Co, K1, K2))
    want, _ = oracle_mod.spectral_conv2d_permode(x, W)
    xd, Wd = torch.from_numpy(x).cuda(), torch.from_numpy(W).cuda()
    yd = torch.full((B, Co, N1, N2), float("nan"), dtype=torch.complex64, device="cuda")
    binding.spectral_conv2d_permode(xd, Wd, yd)
    torch.cuda.synchronize()
    check(yd.cpu().numpy(), want, "permode 2d")


def test_large_batch_uses_64_bit_offsets(gpu, oracle_mod):
    """B = 2^18 (1 GiB tensors, 2^18 workgroups): sampled batch elements against the oracle, including the last, whose
    byte offset is past 2^31; the rest of the batch is filled on the device and only checked to be written."""
    torch, binding = gpu
    B, Ci, Co, N, K = 1 << 18, 8, 8, 64, 16
    say(f"[case] large batch 1-D B={B}")
    gen = torch.Generator(device="cuda").manual_seed(5)
    xd = torch.view_as_complex(torch.randn((B, Ci, N, 2), generator=gen, device="cuda", dtype=torch.float32))
    Wn = inputs.make_W(5, Ci, Co)
    sample = [0, 1, B // 2 + 3, B - 1]
    for b in sample:
        xd[b] = torch.from_numpy(inputs.make_x_element(5, b, Ci, (N,))).cuda()
    Wd = torch.from_numpy(Wn).cuda()
    for fn in ("spectral_conv1d", "spectral_conv1d_pruned"):
        yd = torch.full((B, Co, N), float("nan"), dtype=torch.complex64, device="cuda")
        getattr(binding, fn)(xd, Wd, yd, K)
        torch.cuda.synchronize()
        assert not torch.isnan(torch.view_as_real(yd)).any().item(), "some outputs were never written"
        for b in sample:
            want, _ = oracle_mod.spectral_conv1d(inputs.make_x_element(5, b, Ci, (N,))[None], Wn, K)
            check(yd[b].cpu().numpy()[None], want, f"{fn} b={b}")
        del yd
    del xd
    torch.cuda.empty_cache()


def test_many_small_images_2d(gpu, oracle_mod):
    """32768 images of 64 x 64 (1 GiB): sampled batch elements against the oracle."""
    torch, binding = gpu
    B, Ci, Co, N, K = 4096, 8, 8, 64, 16
    say(f"[case] many images 2-D B={B}")
    gen = torch.Generator(device="cuda").manual_seed(6)
    xd = torch.view_as_complex(torch.randn((B, Ci, N, N, 2), generator=gen, device="cuda", dtype=torch.float32))
    Wn = inputs.make_W(6, Ci, Co)
    sample = [0, B // 3, B - 1]
    for b in sample:
        xd[b] = torch.from_numpy(inputs.make_x_element(6, b, Ci, (N, N))).cuda()
    Wd = torch.from_numpy(Wn).cuda()
    yd = torch.full((B, Co, N, N), float("nan"), dtype=torch.complex64, device="cuda")
    binding.spectral_conv2d(xd, Wd, yd, K)
    torch.cuda.synchronize()
    assert not torch.isnan(torch.view_as_real(yd)).any().item(), "some outputs were never written"
    for b in sample:
        want, _ = oracle_mod.spectral_conv2d(inputs.make_x_element(6, b, Ci, (N, N))[None], Wn, K)
        check(yd[b].cpu().numpy()[None], want, f"2d b={b}")
    del xd, yd
    torch.cuda.empty_cache()


def test_entry_points_replay_from_a_hip_graph(gpu):
    """The entry points only enqueue kernels on the caller's stream, so they can be captured once their first (eager)
    call has been made: three replays, with eager work and synchronisation in between, each bitwise equal to eager."""
    torch, binding = gpu
    say("[case] HIP graph capture of the fused 1-D and the three-kernel 2-D entry points")
    x1 = torch.from_numpy(inputs.make_x(11, 8, 24, (256,))).cuda()
    W1 = torch.from_numpy(inputs.make_W(11, 24, 40)).cuda()
    y1 = torch.zeros((8, 40, 256), dtype=torch.complex64, device="cuda")
    x2 = torch.from_numpy(inputs.make_x(12, 2, 5, (64, 128))).cuda()
    W2 = torch.from_numpy(inputs.make_W(12, 5, 6)).cuda()
    y2 = torch.zeros((2, 6, 64, 128), dtype=torch.complex64, device="cuda")
    binding.spectral_conv1d(x1, W1, y1, 64)
    binding.spectral_conv2d_rect(x2, W2, y2, 16, 32)
    torch.cuda.synchronize()
    want1, want2 = y1.clone(), y2.clone()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    g = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(g, stream=side):
            st = torch.cuda.current_stream().cuda_stream
            binding.spectral_conv1d(x1, W1, y1, 64, st)
            binding.spectral_conv2d_rect(x2, W2, y2, 16, 32, st)
    torch.cuda.current_stream().wait_stream(side)
    for _ in range(3):
        y1.zero_()
        y2.zero_()
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(torch.view_as_real(y1), torch.view_as_real(want1))
        assert torch.equal(torch.view_as_real(y2), torch.view_as_real(want2))


# real-valued layer (B, C_in, C_out, N, K): every N of the fused kernel, ragged channels, K = N/2
REAL_1D = [(4, 16, 16, 64, 16), (3, 5, 7, 64, 8), (2, 33, 40, 64, 32), (3, 9, 70, 128, 32), (2, 37, 17, 128, 64),
           (64, 64, 64, 256, 64), (5, 19, 130, 256, 32), (2, 40, 33, 256, 16), (3, 24, 96, 256, 128), (2, 17, 9, 512, 32),
           (2, 8, 40, 512, 256), (3, 13, 129, 1024, 128), (1, 1, 1, 1024, 64), (2, 20, 30, 1024, 32), (2, 16, 64, 1024, 256),
           (2, 128, 128, 1024, 128),
           # N = 1024 on the symmetric-wave kernel: whole blocks without the deep pipeline, K = 64 deep, and a mode
           # count between the built sizes (stays on the four-wave kernel, which masks bins)
           (2, 16, 128, 1024, 64), (2, 64, 256, 1024, 64), (2, 9, 11, 1024, 100),
           # enough workgroups for the symmetric-wave kernel by default (smaller batches run the four-wave kernel)
           (128, 16, 128, 1024, 64), (70, 9, 130, 1024, 128),
           # at most 64 outputs: the four-wave kernel whatever the batch; one more: the symmetric-wave kernel
           (130, 16, 64, 1024, 64), (130, 16, 65, 1024, 64)]


@pytest.mark.parametrize("shape", REAL_1D, ids=lambda s: "B%d_Ci%d_Co%d_N%d_K%d" % s)
def test_1d_real_layer(gpu, oracle_mod, shape):
    torch, binding = gpu
    B, Ci, Co, N, K = shape
    say(f"[case] spectral_conv1d_real {shape}")
    x = np.ascontiguousarray(inputs.make_x(900 + N + K, B, Ci, (N,)).real)          # float32, N(0, 1)
    W = inputs.make_W(900 + N + K, Ci, Co)
    want, _ = oracle_mod.spectral_conv1d_real(x, W, K)
    xd, Wd = torch.from_numpy(x).cuda(), torch.from_numpy(W).cuda()
    yd = torch.full((B, Co, N), float("nan"), dtype=torch.float32, device="cuda")
    binding.spectral_conv1d_real(xd, Wd, yd, K)
    torch.cuda.synchronize()
    got = yd.cpu().numpy().astype(np.float64)
    rel = np.linalg.norm((got - want).ravel()) / np.linalg.norm(want.ravel())
    mx = np.max(np.abs(got - want)) / np.max(np.abs(want))
    say(f"   real: rel_l2={rel:.3e} max_abs/max|y|={mx:.3e}")
    assert rel <= REL_L2 and mx <= MAX_ABS


# mode counts between the built kernel sizes (the FNO literature uses 12, 20, 24, 48 ...): the kernels run the next
# built size and zero the surplus bins before the contraction.  (B, C_in, C_out, N, K)
ANY_K_1D = [(3, 5, 7, 64, 12), (2, 16, 40, 128, 20), (2, 33, 17, 256, 48), (3, 9, 70, 256, 100), (2, 8, 8, 256, 1),
            (2, 12, 20, 512, 40), (2, 24, 130, 1024, 24), (2, 32, 128, 1024, 100), (1, 3, 200, 256, 33), (2, 4, 4, 64, 5)]


@pytest.mark.parametrize("shape", ANY_K_1D, ids=lambda s: "B%d_Ci%d_Co%d_N%d_K%d" % s)
def test_1d_any_mode_count(gpu, oracle_mod, shape):
    torch, binding = gpu
    B, Ci, Co, N, K = shape
    x = inputs.make_x(1000 + N + K, B, Ci, (N,))
    W = inputs.make_W(1000 + N + K, Ci, Co)
    want, _ = oracle_mod.spectral_conv1d(x, W, K)
    fns = ["spectral_conv1d", "spectral_conv1d_auto", "spectral_conv1d_staged"]
    if binding.workspace_bytes(1, 2, B, Ci, Co, N, K):
        fns.append("spectral_conv1d_pruned")
    if binding.workspace_bytes(1, 3, B, Ci, Co, N, K):
        fns += ["spectral_conv1d_fft_gemm", "spectral_conv1d_gemm_ifft"]
    for fn in fns:
        say(f"[case] {fn} {shape}")
        check(run_gpu(gpu, fn, x, W, K), want, fn)
    if 2 * K <= N:
        xr = np.ascontiguousarray(x.real)
        wantr, _ = oracle_mod.spectral_conv1d_real(xr, W, K)
        yd = torch.full((B, Co, N), float("nan"), dtype=torch.float32, device="cuda")
        binding.spectral_conv1d_real(torch.from_numpy(xr).cuda(), torch.from_numpy(W).cuda(), yd, K)
        torch.cuda.synchronize()
        got = yd.cpu().numpy().astype(np.float64)
        assert np.linalg.norm((got - wantr).ravel()) / np.linalg.norm(wantr.ravel()) <= REL_L2
        assert np.max(np.abs(got - wantr)) / np.max(np.abs(wantr)) <= MAX_ABS


# (B, C_in, C_out, N1, N2, K1, K2): image kernels with rounded mode counts, strip pipeline with a rounded last axis,
# long pencils
ANY_K_2D = [(2, 3, 5, 64, 64, 12, 12), (1, 5, 33, 128, 256, 20, 48), (2, 4, 3, 256, 128, 64, 33), (1, 2, 2, 64, 256, 1, 5),
            (2, 3, 4, 32, 256, 8, 40), (1, 2, 3, 512, 64, 100, 12)]


@pytest.mark.parametrize("shape", ANY_K_2D, ids=lambda s: "B%d_Ci%d_Co%d_N%dx%d_K%dx%d" % s)
def test_2d_any_mode_count(gpu, oracle_mod, shape):
    B, Ci, Co, N1, N2, K1, K2 = shape
    say(f"[case] spectral_conv2d_rect {shape}")
    x = inputs.make_x(1100 + N1 + K2, B, Ci, (N1, N2))
    W = inputs.make_W(1100 + N1 + K2, Ci, Co)
    want, _ = oracle_mod.spectral_conv2d_rect(x, W, K1, K2)
    check(run_gpu_rect(gpu, "spectral_conv2d_rect", x, W, K1, K2), want, "rect any K")


def test_long_pencils_any_mode_count(gpu, oracle_mod):
    for (B, Ci, Co, N, K) in [(2, 5, 7, 2048, 100), (1, 3, 4, 4096, 300), (2, 4, 4, 4096, 17)]:
        say(f"[case] long pencils any K {(B, Ci, Co, N, K)}")
        x = inputs.make_x(1200 + N + K, B, Ci, (N,))
        W = inputs.make_W(1200 + N + K, Ci, Co)
        want, _ = oracle_mod.spectral_conv1d(x, W, K)
        for fn in ("spectral_conv1d_pruned", "spectral_conv1d_auto"):
            check(run_gpu(gpu, fn, x, W, K), want, fn)


# the 2-D FNO layer on real fields (B, C_in, C_out, N1, N2, M1, M2): block sizes that are built sizes and others,
# every row length, M1 at its maximum
FNO_2D = [(2, 3, 5, 64, 64, 12, 12), (2, 4, 4, 64, 64, 8, 16), (1, 5, 9, 128, 128, 16, 16), (3, 2, 3, 256, 256, 32, 64),
          (2, 3, 2, 64, 256, 5, 40), (2, 6, 3, 256, 64, 20, 7), (1, 17, 33, 128, 64, 1, 1), (9, 2, 2, 64, 128, 32, 32),
          (2, 3, 3, 128, 256, 24, 20)]


@pytest.mark.parametrize("shape", FNO_2D, ids=lambda s: "B%d_Ci%d_Co%d_N%dx%d_M%dx%d" % s)
def test_fno2d_real_layer(gpu, oracle_mod, shape):
    torch, binding = gpu
    B, Ci, Co, N1, N2, M1, M2 = shape
    say(f"[case] fno2d_real {shape}")
    x = np.ascontiguousarray(inputs.make_x(1300 + N1 + M2, B, Ci, (N1, N2)).real)
    W = np.ascontiguousarray(inputs.make_W(1300 + N1 + M2, Ci, Co * 2 * M1 * M2).reshape(Ci, Co, 2 * M1, M2))
    want, _ = oracle_mod.fno2d_real(x, W)
    yd = torch.full((B, Co, N1, N2), float("nan"), dtype=torch.float32, device="cuda")
    binding.fno2d_real(torch.from_numpy(x).cuda(), torch.from_numpy(W).cuda(), yd)
    torch.cuda.synchronize()
    got = yd.cpu().numpy().astype(np.float64)
    rel = np.linalg.norm((got - want).ravel()) / np.linalg.norm(want.ravel())
    mx = np.max(np.abs(got - want)) / np.max(np.abs(want))
    say(f"   fno2d: rel_l2={rel:.3e} max_abs/max|y|={mx:.3e}")
    assert rel <= REL_L2 and mx <= MAX_ABS


# the 1-D FNO layer on real fields (B, C_in, C_out, N, M)
FNO_1D = [(4, 16, 16, 64, 16), (3, 5, 7, 64, 12), (9, 33, 40, 128, 20), (17, 6, 18, 256, 128), (2, 20, 30, 1024, 64),
          (11, 13, 17, 1024, 100), (2, 3, 3, 128, 1), (8, 3, 2, 256, 33)]


@pytest.mark.parametrize("shape", FNO_1D, ids=lambda s: "B%d_Ci%d_Co%d_N%d_M%d" % s)
def test_fno1d_real_layer(gpu, oracle_mod, shape):
    torch, binding = gpu
    B, Ci, Co, N, M = shape
    say(f"[case] fno1d_real {shape}")
    x = np.ascontiguousarray(inputs.make_x(1400 + N + M, B, Ci, (N,)).real)
    W = np.ascontiguousarray(inputs.make_W(1400 + N + M, Ci, Co * M).reshape(Ci, Co, M))
    want, _ = oracle_mod.fno1d_real(x, W)
    yd = torch.full((B, Co, N), float("nan"), dtype=torch.float32, device="cuda")
    binding.fno1d_real(torch.from_numpy(x).cuda(), torch.from_numpy(W).cuda(), yd)
    torch.cuda.synchronize()
    got = yd.cpu().numpy().astype(np.float64)
    rel = np.linalg.norm((got - want).ravel()) / np.linalg.norm(want.ravel())
    mx = np.max(np.abs(got - want)) / np.max(np.abs(want))
    say(f"   fno1d: rel_l2={rel:.3e} max_abs/max|y|={mx:.3e}")
    assert rel <= REL_L2 and mx <= MAX_ABS


def test_every_1d_shape_either_runs_or_is_reported_unsupported(gpu, oracle_mod):
    """Sweeps N and K over their whole range for every 1-D entry point: a call must end in TFNO_OK or
    TFNO_ERR_UNSUPPORTED (never a launch error from a shape the dispatch accepted but no kernel was built for), and
    what runs must match the oracle."""
    torch, binding = gpu
    B, Ci, Co = 2, 3, 2
    ran = 0
    for e in range(1, 13):
        N = 1 << e
        x = inputs.make_x(1600 + e, B, Ci, (N,))
        xd = torch.from_numpy(x).cuda()
        xr = np.ascontiguousarray(x.real)
        xrd = torch.from_numpy(xr).cuda()
        W = inputs.make_W(1600 + e, Ci, Co)
        Wd = torch.from_numpy(W).cuda()
        ks = sorted({k for k in (1, 2, 3, 5, 8, 12, 16, 24, 32, 48, 64, 100, 128, 200, 256, 300, 512, 1000, 1024, 2048, 4096,
                                 N // 2, N) if 1 <= k <= N})
        for K in ks:
            want = None
            for fn in ("spectral_conv1d", "spectral_conv1d_pruned", "spectral_conv1d_fft_gemm", "spectral_conv1d_gemm_ifft",
                       "spectral_conv1d_auto"):
                yd = torch.full((B, Co, N), float("nan"), dtype=torch.complex64, device="cuda")
                try:
                    getattr(binding, fn)(xd, Wd, yd, K)
                except binding.TfnoError as err:
                    assert err.status == binding.ERR_UNSUPPORTED, (fn, N, K, err.status)
                    assert fn != "spectral_conv1d_auto", (N, K)
                    continue
                torch.cuda.synchronize()
                if want is None:
                    want, _ = oracle_mod.spectral_conv1d(x, W, K)
                got = yd.cpu().numpy().astype(np.complex128)
                close(got, want, (fn, N, K))
                ran += 1
            if 2 * K <= N:
                Wm = np.ascontiguousarray(np.repeat(W[:, :, None], K, axis=2))
                Wmd = torch.from_numpy(Wm).cuda()
                wantr = None
                for fn, args in (("spectral_conv1d_real", (xrd, Wd)), ("fno1d_real", (xrd, Wmd))):
                    yd = torch.full((B, Co, N), float("nan"), dtype=torch.float32, device="cuda")
                    try:
                        if fn == "fno1d_real":
                            binding.fno1d_real(*args, yd)
                        else:
                            binding.spectral_conv1d_real(*args, yd, K)
                    except binding.TfnoError as err:
                        assert err.status == binding.ERR_UNSUPPORTED, (fn, N, K, err.status)
                        continue
                    torch.cuda.synchronize()
                    if wantr is None:
                        wantr, _ = oracle_mod.spectral_conv1d_real(xr, W, K)     # equal matrices: the same operator
                    got = yd.cpu().numpy().astype(np.float64)
                    close(got, wantr, (fn, N, K))
                    ran += 1
    say(f"   {ran} (entry point, N, K) combinations ran and matched the oracle")
    assert ran > 400


def test_every_2d_shape_either_runs_or_is_reported_unsupported(gpu, oracle_mod):
    """The same sweep for the 2-D entry points over N1, N2 in {32 .. 512} and mode counts from 1 to N/2."""
    torch, binding = gpu
    B, Ci, Co = 1, 2, 2
    ran = 0
    for N1 in (32, 64, 128, 256, 512):
        for N2 in (32, 64, 128, 256, 512):
            x = inputs.make_x(1700 + N1 + 3 * N2, B, Ci, (N1, N2))
            xd = torch.from_numpy(x).cuda()
            xr = np.ascontiguousarray(x.real)
            xrd = torch.from_numpy(xr).cuda()
            W = inputs.make_W(1700 + N1, Ci, Co)
            Wd = torch.from_numpy(W).cuda()
            for (K1, K2) in sorted({(1, 1), (5, 12), (16, 16), (24, 40), (64, 64), (N1 // 2, N2 // 2), (12, N2 // 2)}):
                if K1 > N1 or K2 > N2:
                    continue
                want, _ = oracle_mod.spectral_conv2d_rect(x, W, K1, K2)
                Wm = np.broadcast_to(W[:, :, None, None], (Ci, Co, K1, K2)).copy()
                for fn, args in (("spectral_conv2d_rect", (xd, Wd)), ("spectral_conv2d_permode", (xd, torch.from_numpy(Wm).cuda()))):
                    yd = torch.full((B, Co, N1, N2), float("nan"), dtype=torch.complex64, device="cuda")
                    try:
                        if fn == "spectral_conv2d_rect":
                            binding.spectral_conv2d_rect(*args, yd, K1, K2)
                        else:
                            binding.spectral_conv2d_permode(*args, yd)
                    except binding.TfnoError as err:
                        assert err.status == binding.ERR_UNSUPPORTED, (fn, N1, N2, K1, K2, err.status)
                        continue
                    torch.cuda.synchronize()
                    got = yd.cpu().numpy().astype(np.complex128)
                    close(got, want, (fn, N1, N2, K1, K2))
                    ran += 1
                M1 = K1 // 2
                if M1 >= 1 and 2 * K2 <= N2:
                    Wf = np.ascontiguousarray(inputs.make_W(1700 + K1 + K2, Ci, Co * 2 * M1 * K2).reshape(Ci, Co, 2 * M1, K2))
                    yd = torch.full((B, Co, N1, N2), float("nan"), dtype=torch.float32, device="cuda")
                    try:
                        binding.fno2d_real(xrd, torch.from_numpy(Wf).cuda(), yd)
                    except binding.TfnoError as err:
                        assert err.status == binding.ERR_UNSUPPORTED, ("fno2d_real", N1, N2, M1, K2, err.status)
                        continue
                    torch.cuda.synchronize()
                    wantf, _ = oracle_mod.fno2d_real(xr, Wf)
                    got = yd.cpu().numpy().astype(np.float64)
                    close(got, wantf, ("fno2d", N1, N2, M1, K2))
                    ran += 1
    say(f"   {ran} (entry point, N1, N2, K1, K2) combinations ran and matched the oracle")
    assert ran > 150


def test_channel_count_sweep(gpu, oracle_mod):
    """Ragged and boundary channel counts (around every tile size of the kernels) on the main entry points."""
    torch, binding = gpu
    vals = [1, 2, 3, 7, 8, 9, 15, 16, 17, 31, 32, 33, 63, 64, 65, 95, 96, 127, 128, 129, 160, 255, 256, 257]
    rs = np.random.default_rng(77)
    pairs = [(int(rs.choice(vals)), int(rs.choice(vals))) for _ in range(20)] + [(1, 257), (257, 1), (129, 129)]
    for idx, (Ci, Co) in enumerate(pairs):
        N, K, B = (256, 64, 2) if idx % 3 else (1024, 128, 1)
        x = inputs.make_x(1800 + idx, B, Ci, (N,))
        W = inputs.make_W(1800 + idx, Ci, Co)
        want, _ = oracle_mod.spectral_conv1d(x, W, K)
        fns = ["spectral_conv1d", "spectral_conv1d_pruned", "spectral_conv1d_auto"]
        if N == 256:
            fns += ["spectral_conv1d_fft_gemm", "spectral_conv1d_gemm_ifft"]
        for fn in fns:
            got = run_gpu(gpu, fn, x, W, K).astype(np.complex128)
            close(got, want, (fn, Ci, Co, N))
        xr = np.ascontiguousarray(x.real)
        wantr, _ = oracle_mod.spectral_conv1d_real(xr, W, K)
        yd = torch.full((B, Co, N), float("nan"), dtype=torch.float32, device="cuda")
        binding.spectral_conv1d_real(torch.from_numpy(xr).cuda(), torch.from_numpy(W).cuda(), yd, K)
        torch.cuda.synchronize()
        got = yd.cpu().numpy().astype(np.float64)
        close(got, wantr, ("real", Ci, Co, N))
        # 2-D image kernels, mode CGEMM and per-mode contraction with the same channel counts
        x2 = inputs.make_x(1900 + idx, 1, Ci, (64, 64))
        want2, _ = oracle_mod.spectral_conv2d(x2, W, 16)
        got = run_gpu(gpu, "spectral_conv2d", x2, W, 16).astype(np.complex128)
        close(got, want2, ("2d", Ci, Co))
        Wm = np.broadcast_to(W[:, :, None, None], (Ci, Co, 16, 16)).copy()
        yd = torch.full((1, Co, 64, 64), float("nan"), dtype=torch.complex64, device="cuda")
        binding.spectral_conv2d_permode(torch.from_numpy(x2).cuda(), torch.from_numpy(Wm).cuda(), yd)
        torch.cuda.synchronize()
        got = yd.cpu().numpy().astype(np.complex128)
        close(got, want2, ("2d permode", Ci, Co))
    say(f"   {len(pairs)} channel-count pairs on 8-9 entry points each")


def test_batch_size_sweep(gpu, oracle_mod):
    """Odd and boundary batch sizes on the kernels that group pencils, tiles or images (pruned sweeps, two long
    pencils per sweep, mode tiles shared by batch elements, the batch groups of the per-mode contraction)."""
    torch, binding = gpu
    Ci, Co = 3, 5
    for B in (1, 2, 3, 5, 7, 8, 9, 15, 16, 17, 31, 33, 65):
        for (fn, N, K) in (("spectral_conv1d_pruned", 64, 16), ("spectral_conv1d_pruned", 256, 32),
                           ("spectral_conv1d_pruned", 2048, 128), ("spectral_conv1d_gemm_ifft", 128, 32),
                           ("spectral_conv1d", 64, 8)):
            x = inputs.make_x(2000 + B + N, B, Ci, (N,))
            W = inputs.make_W(2000 + B + N, Ci, Co)
            want, _ = oracle_mod.spectral_conv1d(x, W, K)
            got = run_gpu(gpu, fn, x, W, K).astype(np.complex128)
            close(got, want, (fn, B, N, K))
        for (N, K) in ((64, 16), (256, 12)):
            x = inputs.make_x(2100 + B + N, B, Ci, (N,))
            Wm = np.ascontiguousarray(inputs.make_W(2100 + B + N, Ci, Co * K).reshape(Ci, Co, K))
            want, _ = oracle_mod.spectral_conv1d_permode(x, Wm)
            yd = torch.full((B, Co, N), float("nan"), dtype=torch.complex64, device="cuda")
            binding.spectral_conv1d_permode(torch.from_numpy(x).cuda(), torch.from_numpy(Wm).cuda(), yd)
            torch.cuda.synchronize()
            got = yd.cpu().numpy().astype(np.complex128)
            close(got, want, ("permode", B, N, K))
            xr = np.ascontiguousarray(x.real)
            wantr, _ = oracle_mod.fno1d_real(xr, Wm)
            yr = torch.full((B, Co, N), float("nan"), dtype=torch.float32, device="cuda")
            binding.fno1d_real(torch.from_numpy(xr).cuda(), torch.from_numpy(Wm).cuda(), yr)
            torch.cuda.synchronize()
            got = yr.cpu().numpy().astype(np.float64)
            close(got, wantr, ("fno1d", B, N, K))
        x2 = np.ascontiguousarray(inputs.make_x(2200 + B, B, Ci, (64, 64)).real)
        Wf = np.ascontiguousarray(inputs.make_W(2200 + B, Ci, Co * 24 * 12).reshape(Ci, Co, 24, 12))
        wantf, _ = oracle_mod.fno2d_real(x2, Wf)
        yf = torch.full((B, Co, 64, 64), float("nan"), dtype=torch.float32, device="cuda")
        binding.fno2d_real(torch.from_numpy(x2).cuda(), torch.from_numpy(Wf).cuda(), yf)
        torch.cuda.synchronize()
        got = yf.cpu().numpy().astype(np.float64)
        close(got, wantf, ("fno2d", B))


def test_wide_output_slabs_with_ragged_channels(gpu, oracle_mod):
    """Batches large enough that the fused kernel keeps its widest output slabs (small batches are given narrower
    ones to fill the chip), with channel counts that leave the last slab, the last 32-output tile and the last
    channel block partly empty."""
    for (B, Ci, Co, N, K) in [(140, 5, 70, 64, 16), (150, 9, 130, 128, 32), (140, 33, 40, 256, 64), (130, 20, 96, 512, 64),
                              (135, 7, 100, 256, 128), (132, 17, 33, 1024, 32), (140, 3, 129, 64, 64)]:
        say(f"[case] wide slabs {(B, Ci, Co, N, K)}")
        x = inputs.make_x(2300 + N + K, B, Ci, (N,))
        W = inputs.make_W(2300 + N + K, Ci, Co)
        want, _ = oracle_mod.spectral_conv1d(x, W, K)
        check(run_gpu(gpu, "spectral_conv1d", x, W, K), want, "fused, wide slabs")
        if 2 * K <= N:
            torch, binding = gpu
            xr = np.ascontiguousarray(x.real)
            wantr, _ = oracle_mod.spectral_conv1d_real(xr, W, K)
            yd = torch.full((B, Co, N), float("nan"), dtype=torch.float32, device="cuda")
            binding.spectral_conv1d_real(torch.from_numpy(xr).cuda(), torch.from_numpy(W).cuda(), yd, K)
            torch.cuda.synchronize()
            got = yd.cpu().numpy().astype(np.float64)
            close(got, wantr, "real layer")


# N = 256 has three more fused kernels behind the dispatch: the single-operand-tile kernel (K = 128, more batch rows
# than CUs; two workgroups per CU), the eight-wave kernel (256 outputs per workgroup for C_out > 128, and 32 or 64 for
# batches of at most 256 workgroups) and the two-group kernel (C_out > 128: 256 outputs per workgroup).  Shapes that reach each of them with whole and ragged channel blocks, absent output slabs and mode counts
# between the built sizes.  (B, C_in, C_out, N, K)
N256_SPECIAL = [
    (300, 5, 70, 256, 128),      # single tile, masked, 128-output slab partly empty
    (260, 20, 33, 256, 100),     # single tile, masked, 64-output slab, K rounded up to 128
    (257, 9, 30, 256, 128),      # single tile, masked, 32-output slab
    (258, 16, 64, 256, 128),     # single tile, whole blocks
    # (the 256-output kernels take over from 192 batch rows on)
    (193, 64, 256, 256, 48),     # two-group kernel, K rounded up to 64
    (192, 64, 160, 256, 64),     # two-group kernel, three of eight output slabs absent
    (200, 96, 192, 256, 32),     # two-group kernel, six 16-channel blocks
    (192, 128, 256, 256, 128),   # eight-wave kernel, whole blocks
    (195, 70, 200, 256, 128),    # eight-wave kernel, masked
    (200, 48, 136, 256, 32),     # eight-wave kernel (48 channels are not whole 32-channel blocks), masked
    (191, 64, 256, 256, 64),     # one row short of the rule: the four-wave kernel, two 128-output slabs per row
    # at most 256 workgroups of 32 (K <= 64: or 64) outputs: eight waves with those slabs
    (64, 20, 33, 256, 64),       # 32-output slabs, masked, the second slab holds one channel
    (8, 64, 256, 256, 128),      # 32-output slabs, exactly 256 workgroups, whole blocks
    (100, 33, 100, 256, 48),     # 64-output slabs (400 workgroups of 32 outputs would be too many), K rounded up
    (256, 8, 64, 256, 32),       # 64-output slabs, exactly 256 workgroups
    (257, 5, 64, 256, 32),       # one row more: the four-wave kernel
    (150, 33, 100, 256, 64),     # 300 workgroups of 64 outputs: the four-wave kernel
    (100, 7, 100, 256, 128),     # K = 128 has no 64-output eight-wave kernel: the four-wave kernel
    # N = 128, K = 64 with more batch rows than CUs: the single-operand-tile kernel (two workgroups per CU)
    (300, 20, 70, 128, 64), (260, 32, 33, 128, 50), (258, 64, 128, 128, 64), (257, 5, 9, 128, 64),
    (300, 16, 200, 128, 64),     # ... two slabs per row; the dispatch keeps the fused kernel here
    (300, 16, 200, 128, 32),     # ... and takes the CGEMM + iFFT variant at K = 32
    # N = 128, K <= 32, 33 .. 64 outputs, more than two batch rows per CU: single operand tile, the partial sums of the
    # split contraction added in turns into one epilogue tile (three workgroups per CU)
    (600, 20, 40, 128, 32), (520, 32, 64, 128, 32), (513, 5, 40, 128, 16), (600, 64, 33, 128, 20), (530, 32, 64, 128, 16),
    (512, 32, 64, 128, 32),      # one row short of the rule: the double-buffered kernel
    (600, 32, 32, 128, 32),      # 32 outputs: the double-buffered kernel, four partial sums side by side
    # ... and the same form with four output tiles: N = 128 (whole channel blocks only), N = 64 (any channel count)
    (520, 32, 128, 128, 32), (513, 64, 256, 128, 16), (520, 32, 130, 128, 32), (520, 20, 128, 128, 32),
    (600, 32, 128, 64, 16), (520, 20, 96, 64, 32), (513, 9, 70, 64, 8), (512, 32, 128, 64, 16),
    # N = 64, at most 32 outputs, more than three batch rows per CU: single operand tile, four workgroups per CU;
    # N = 128 likewise for a single half-empty block of input channels
    (800, 32, 32, 64, 16), (770, 16, 20, 64, 32), (769, 5, 9, 64, 8), (768, 32, 32, 64, 16),
    (600, 16, 16, 128, 32), (520, 9, 30, 128, 16), (600, 17, 16, 128, 32),
    # N = 256, K <= 64, more than four batch rows per CU, whole channel blocks: single operand tile, three workgroups per CU
    (1025, 16, 32, 256, 32), (1100, 32, 64, 256, 64), (1030, 16, 128, 256, 32), (1026, 32, 64, 256, 20),
    (1030, 16, 128, 256, 64),    # K = 64 with 128 outputs would spill there: the double-buffered kernel
    (1030, 24, 64, 256, 32),     # 24 channels are not whole blocks: the double-buffered kernel
]


@pytest.mark.parametrize("shape", N256_SPECIAL, ids=lambda s: "B%d_Ci%d_Co%d_N%d_K%d" % s)
def test_n256_dispatched_kernels(gpu, oracle_mod, shape):
    B, Ci, Co, N, K = shape
    say(f"[case] N = 256 dispatch {shape}")
    x = inputs.make_x(2400 + Ci + K, B, Ci, (N,))
    W = inputs.make_W(2400 + Ci + K, Ci, Co)
    want, _ = oracle_mod.spectral_conv1d(x, W, K)
    check(run_gpu(gpu, "spectral_conv1d", x, W, K), want, "fused")
    check(run_gpu(gpu, "spectral_conv1d_auto", x, W, K), want, "auto")


def test_round_trip_identity_and_determinism(gpu):
    """K = N, W = I gives y = x; two runs give bitwise equal output."""
    torch, binding = gpu
    N, C = 256, 48
    x = inputs.make_x(3, 4, C, (N,))
    W = np.eye(C, dtype=np.complex64)
    a = run_gpu(gpu, "spectral_conv1d", x, W, N)
    b = run_gpu(gpu, "spectral_conv1d", x, W, N)
    assert np.array_equal(a.view(np.float32), b.view(np.float32))
    check(a, x.astype(np.complex128), "round trip")


def test_empty_batch_and_error_paths(gpu):
    torch, binding = gpu
    x = torch.zeros((0, 4, 64), dtype=torch.complex64, device="cuda")
    W = torch.zeros((4, 4), dtype=torch.complex64, device="cuda")
    y = torch.zeros((0, 4, 64), dtype=torch.complex64, device="cuda")
    binding.spectral_conv1d(x, W, y, 16)
    binding.spectral_conv1d_staged(x, W, y, 16)
    x = torch.zeros((1, 4, 64), dtype=torch.complex64, device="cuda")
    with pytest.raises(binding.TfnoError) as e:
        binding.spectral_conv1d(x, W, x, 16)           # y aliases x
    assert e.value.status == binding.ERR_ALIAS
    y = torch.zeros((1, 4, 64), dtype=torch.complex64, device="cuda")
    with pytest.raises(binding.TfnoError) as e:
        binding.spectral_conv1d(x, W, y, 65)
    assert e.value.status == binding.ERR_SHAPE
    torch.cuda.synchronize()


# Scaling the input or the weights by a power of two only changes exponents, so every entry point must return the
# scaled result bit for bit: the transforms multiply by twiddles and add, and the contraction splits each operand into
# three BF16 terms whose exponent range is that of float32.  A split that lost low-order terms to underflow, or a
# path that mixed scaled and unscaled quantities, would show here.
@pytest.mark.parametrize("entry,shape", [("spectral_conv1d", (3, 24, 40, 1024, 128)), ("spectral_conv1d", (5, 32, 64, 256, 128)),
                                         ("spectral_conv1d", (4, 64, 256, 256, 64)), ("spectral_conv1d_pruned", (3, 70, 65, 256, 64)),
                                         ("spectral_conv2d", (2, 8, 8, 64, 16))],
                         ids=lambda v: v if isinstance(v, str) else "x".join(map(str, v)))
def test_power_of_two_scaling_is_exact(gpu, entry, shape):
    B, Ci, Co, N, K = shape
    say(f"[case] scaling {entry} {shape}")
    dims = (N, N) if entry.endswith("2d") else (N,)
    x = inputs.make_x(4242, B, Ci, dims)
    W = inputs.make_W(4242, Ci, Co)
    base = run_gpu(gpu, entry, x, W, K)
    assert np.isfinite(base.view(np.float32)).all()
    for ex, ew in ((30, 0), (-30, 0), (0, 25), (-20, -20), (40, -45)):
        got = run_gpu(gpu, entry, x * np.float32(2.0 ** ex), W * np.float32(2.0 ** ew), K)
        want = base * np.float32(2.0 ** (ex + ew))
        assert np.array_equal(got.view(np.float32), want.view(np.float32)), (entry, shape, ex, ew)


def test_workspace_growth_does_not_disturb_earlier_work_on_another_stream(gpu, oracle_mod):
    """A call that uses the workspace is enqueued on a side stream behind a long queue of other launches; a call
    with a larger workspace need follows on the default stream at once.  The binding synchronises the device before
    it replaces the registered buffer, so the first call still finds its intermediates: its result must match the
    oracle."""
    torch, binding = gpu
    binding.set_workspace(None)                               # start from no workspace at all
    xa = inputs.make_x(2500, 6, 24, (256,)); Wa = inputs.make_W(2500, 24, 40)
    xb = inputs.make_x(2501, 24, 48, (256,)); Wb = inputs.make_W(2501, 48, 64)
    xad, Wad = torch.from_numpy(xa).cuda(), torch.from_numpy(Wa).cuda()
    xbd, Wbd = torch.from_numpy(xb).cuda(), torch.from_numpy(Wb).cuda()
    ya = torch.full((6, 40, 256), float("nan"), dtype=torch.complex64, device="cuda")
    yb = torch.full((24, 64, 256), float("nan"), dtype=torch.complex64, device="cuda")
    filler = torch.empty(1 << 26, dtype=torch.float32, device="cuda")
    side = torch.cuda.Stream()
    torch.cuda.synchronize()
    with torch.cuda.stream(side):
        for _ in range(20):
            filler.fill_(1.0)                                 # keeps the side stream busy ahead of the call
        binding.spectral_conv1d_pruned(xad, Wad, ya, 64, stream=side.cuda_stream)
    binding.spectral_conv1d_pruned(xbd, Wbd, yb, 64)          # needs a larger workspace
    torch.cuda.synchronize()
    check(ya.cpu().numpy(), oracle_mod.spectral_conv1d(xa, Wa, 64)[0], "first call (side stream)")
    check(yb.cpu().numpy(), oracle_mod.spectral_conv1d(xb, Wb, 64)[0], "second call (larger workspace)")


# ----------------------------------------------------- full benchmark sizes, every batch element

def full_size_inputs(torch, w):
    Wn = inputs.make_W(w.seed, w.C_in, w.C_out)
    xd = torch.empty((w.B, w.C_in) + w.spatial, dtype=torch.complex64, device="cuda")
    for b in range(w.B):
        xd[b] = torch.from_numpy(inputs.make_x_element(w.seed, b, w.C_in, w.spatial)).cuda()
    return xd, Wn, torch.from_numpy(Wn).cuda()


def full_size_run(gpu, w, fn_name, xd, Wd):
    """The whole workload in the launch configuration the benchmark times; the output starts as NaN."""
    torch, binding = gpu
    yd = torch.full((w.B, w.C_out) + w.spatial, float("nan"), dtype=torch.complex64, device="cuda")
    getattr(binding, fn_name)(xd, Wd, yd, w.K)
    torch.cuda.synchronize()
    assert not torch.isnan(torch.view_as_real(yd)).any().item(), f"{fn_name}: some outputs were never written"
    return yd


def whole_batch_against_oracle(gpu, oracle_mod, w, fn_name, xd, Wn, yd, chunk=16):
    """Every batch element of the full-size output against the oracle, `chunk` elements at a time (the float64 result
    of the 2-D configuration would not fit comfortably at once): the tolerance must hold for every chunk and the
    relative L2 error for every single batch element (each is one workgroup row or one group of images on the GPU,
    so a fault tied to a compute unit, an XCD residue or a grid slab shows up in its own element)."""
    say(f"[case] {fn_name} {w.name}: all {w.B} batch elements against the oracle")
    worst = 0.0
    for b0 in range(0, w.B, chunk):
        b1 = min(w.B, b0 + chunk)
        xb = xd[b0:b1].cpu().numpy()
        want, _ = oracle_fn(oracle_mod, w.dims)(xb, Wn, w.K)
        got = yd[b0:b1].cpu().numpy().astype(np.complex128)
        close(got, want, f"{fn_name} {w.name} b={b0}..{b1 - 1}")
        err = np.linalg.norm((got - want).reshape(b1 - b0, -1), axis=1) / np.linalg.norm(want.reshape(b1 - b0, -1), axis=1)
        assert err.max() <= REL_L2, (fn_name, w.name, b0 + int(err.argmax()), float(err.max()))
        worst = max(worst, float(err.max()))
    say(f"   worst batch element: rel_l2={worst:.3e}")


def whole_batch_against_reference(gpu, oracle_mod, w, fn_name, xd, Wn, yd, y_ref, sample_b):
    """A variant's full-size output: every batch row against the fused kernel's output on the device (which
    whole_batch_against_oracle has tied to the oracle; two float32 paths agree to a few rounding errors), and the
    batch elements `sample_b` against the oracle itself."""
    torch, _ = gpu
    say(f"[case] {fn_name} {w.name}: all rows against the fused output, b={sample_b} against the oracle")
    d = torch.view_as_real(yd - y_ref).reshape(w.B, -1).double().norm(dim=1)
    r = torch.view_as_real(y_ref).reshape(w.B, -1).double().norm(dim=1)
    rel = (d / r).max().item()
    say(f"   worst row against the fused output: rel_l2={rel:.3e}")
    assert rel <= 5e-6, (fn_name, w.name, rel)
    for b in sample_b:
        want, _ = oracle_fn(oracle_mod, w.dims)(xd[b:b + 1].cpu().numpy(), Wn, w.K)
        check(yd[b].cpu().numpy()[None], want, f"{fn_name} {w.name} b={b}")


def full_size_config(gpu, oracle_mod, w, fused_fn, others):
    torch, _ = gpu
    xd, Wn, Wd = full_size_inputs(torch, w)
    y_ref = full_size_run(gpu, w, fused_fn, xd, Wd)
    whole_batch_against_oracle(gpu, oracle_mod, w, fused_fn, xd, Wn, y_ref)
    # E|y|^2 = 4 (K/N)^dims for these input distributions: a property that holds at any size
    e2 = torch.mean(torch.abs(y_ref.view(-1)[: 1 << 24]) ** 2).item()
    assert abs(e2 / (4 * (w.K / w.N) ** w.dims) - 1) < 0.05
    for fn_name, sample_b in others:
        yd = full_size_run(gpu, w, fn_name, xd, Wd)
        whole_batch_against_reference(gpu, oracle_mod, w, fn_name, xd, Wn, yd, y_ref, sample_b)
        del yd
    del xd, y_ref
    torch.cuda.empty_cache()


def test_config3_full_size(gpu, oracle_mod):
    full_size_config(gpu, oracle_mod, inputs.CONFIGS[2], "spectral_conv1d",
                     [("spectral_conv1d_staged", [0, 255]), ("spectral_conv1d_pruned", [101]), ("spectral_conv1d_auto", [7])])


def test_config4_full_size(gpu, oracle_mod):
    full_size_config(gpu, oracle_mod, inputs.CONFIGS[3], "spectral_conv2d", [("spectral_conv2d_staged", [0, 31])])


@pytest.mark.parametrize("w", inputs.sweep_configs(), ids=lambda w: w.name)
def test_config5_sweep_full_size(gpu, oracle_mod, w):
    full_size_config(gpu, oracle_mod, w, "spectral_conv1d",
                     [("spectral_conv1d_auto", [0, 511]), ("spectral_conv1d_staged", [257]), ("spectral_conv1d_pruned", [3]),
                      ("spectral_conv1d_fft_gemm", [509]), ("spectral_conv1d_gemm_ifft", [2, 508])])


SYM_1D = [(2, 32, 128, 1024, 128),   # two blocks of loads in flight (even block count >= 4), no masks
          (1, 48, 256, 1024, 64),
          (2, 16, 128, 1024, 128),   # unmasked, two blocks only
          (3, 13, 129, 1024, 128),   # masked
          (1, 1, 1, 1024, 64)]


@pytest.mark.parametrize("kernel", ["ws", "generic", "sym"])
def test_alternative_n1024_kernels_in_a_child_process(gpu, oracle_mod, tmp_path, kernel):
    """N = 1024 runs the symmetric-wave kernel by default when the grid fills half the chip (K in {64, 128}) and the
    four-wave kernel below that; TFNO_KERNEL (read once per process) selects the wave-specialised kernel (ws), the
    four-wave kernel (generic) or the symmetric-wave kernel (sym) for every batch size.  The real-valued layer follows
    the same switch."""
    import os
    import subprocess
    import textwrap
    say(f"[case] TFNO_KERNEL={kernel} child process")
    out = str(tmp_path / f"{kernel}.npz")
    code = textwrap.dedent(f"""
        import numpy as np, torch
        from paper_2504_11681_amd import binding, inputs
        res = {{}}
        for i, (B, Ci, Co, N, K) in enumerate({SYM_1D!r}):
            x = inputs.make_x(40 + i, B, Ci, (N,)); W = inputs.make_W(40 + i, Ci, Co)
            y = torch.empty((B, Co, N), dtype=torch.complex64, device='cuda')
            binding.spectral_conv1d(torch.from_numpy(x).cuda(), torch.from_numpy(W).cuda(), y, K)
            torch.cuda.synchronize()
            res['y%d' % i] = y.cpu().numpy()
            if K <= N // 2:
                yr = torch.empty((B, Co, N), dtype=torch.float32, device='cuda')
                binding.spectral_conv1d_real(torch.from_numpy(np.ascontiguousarray(x.real)).cuda(), torch.from_numpy(W).cuda(), yr, K)
                torch.cuda.synchronize()
                res['r%d' % i] = yr.cpu().numpy()
        np.savez({out!r}, **res)
    """)
    env = dict(os.environ, TFNO_KERNEL=kernel)
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    subprocess.run([sys.executable, "-c", code], check=True, env=env, cwd=root, timeout=110)
    got = np.load(out)
    for i, (B, Ci, Co, N, K) in enumerate(SYM_1D):
        x = inputs.make_x(40 + i, B, Ci, (N,)); W = inputs.make_W(40 + i, Ci, Co)
        check(got["y%d" % i], oracle_mod.spectral_conv1d(x, W, K)[0], f"{kernel} {(B, Ci, Co, N, K)}")
        wantr = oracle_mod.spectral_conv1d_real(np.ascontiguousarray(x.real), W, K)[0]
        gotr = got["r%d" % i].astype(np.float64)
        assert np.linalg.norm((gotr - wantr).ravel()) <= 1e-5 * np.linalg.norm(wantr.ravel()), (kernel, "real", i)
        assert np.abs(gotr - wantr).max() <= 1e-4 * np.abs(wantr).max(), (kernel, "real", i)


def test_fp32_contraction_kernels_in_a_child_process(gpu, oracle_mod, tmp_path):
    """TFNO_CONTRACTION=f32 (read once per process) selects the FP32-MFMA contraction kernels: the generic fused
    1-D kernel for N = 1024 and the FP32 mode CGEMM of the 2-D path.  A child process runs both and saves the
    results; they are compared with the oracle here."""
    import os
    import subprocess
    import textwrap
    say("[case] TFNO_CONTRACTION=f32 child process")
    out = str(tmp_path / "f32.npz")
    code = textwrap.dedent(f"""
        import numpy as np, torch
        from paper_2504_11681_amd import binding, inputs
        x1 = inputs.make_x(31, 2, 20, (1024,)); W1 = inputs.make_W(31, 20, 40)
        y1 = torch.empty((2, 40, 1024), dtype=torch.complex64, device='cuda')
        binding.spectral_conv1d(torch.from_numpy(x1).cuda(), torch.from_numpy(W1).cuda(), y1, 128)
        x2 = inputs.make_x(32, 2, 5, (128, 128)); W2 = inputs.make_W(32, 5, 70)
        y2 = torch.empty((2, 70, 128, 128), dtype=torch.complex64, device='cuda')
        binding.spectral_conv2d(torch.from_numpy(x2).cuda(), torch.from_numpy(W2).cuda(), y2, 32)
        torch.cuda.synchronize()
        np.savez({out!r}, y1=y1.cpu().numpy(), y2=y2.cpu().numpy())
    """)
    env = dict(os.environ, TFNO_CONTRACTION="f32")
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    subprocess.run([sys.executable, "-c", code], check=True, env=env, cwd=root, timeout=110)
    got = np.load(out)
    x1 = inputs.make_x(31, 2, 20, (1024,)); W1 = inputs.make_W(31, 20, 40)
    check(got["y1"], oracle_mod.spectral_conv1d(x1, W1, 128)[0], "f32 1-D N=1024")
    x2 = inputs.make_x(32, 2, 5, (128, 128)); W2 = inputs.make_W(32, 5, 70)
    check(got["y2"], oracle_mod.spectral_conv2d(x2, W2, 32)[0], "f32 2-D 128x128")
