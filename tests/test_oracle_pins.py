"""Pins for the float64 oracle: none of them re-types the oracle's own formula.

They check it against brute force, closed forms, invariants and NumPy's FFT
(library special case), chosen so that a dropped term, a wrong sign or index, a
transposed W or a wrong normalisation fails at least one of them.
"""
import os

import numpy as np
import pytest

from paper_2504_11681_amd import inputs

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
rng = np.random.default_rng(1234)


def crandn(*shape):
    return (rng.standard_normal(shape) + 1j * rng.standard_normal(shape)).astype(np.complex64)


# ---------------------------------------------------------------- transform --

@pytest.mark.parametrize("N", [1, 2, 4, 8, 16, 32, 64, 128, 1024])
@pytest.mark.parametrize("sign", [-1, +1])
def test_radix2_equals_brute_force(oracle_mod, N, sign):
    v = crandn(N).astype(np.complex128)
    a = oracle_mod.fft_radix2(v, sign)
    b = oracle_mod.dft_direct(v, sign)
    assert np.max(np.abs(a - b)) <= 1e-12 * max(1.0, N) * np.max(np.abs(b))


@pytest.mark.parametrize("N", [3, 5, 12, 32, 64, 256])
def test_transform_matches_numpy_fft(oracle_mod, N):
    v = crandn(N).astype(np.complex128)
    assert np.allclose(oracle_mod.fft(v, -1), np.fft.fft(v), rtol=0, atol=1e-11 * N)
    assert np.allclose(oracle_mod.fft(v, +1), np.fft.ifft(v) * N, rtol=0, atol=1e-11 * N)


@pytest.mark.parametrize("N", [8, 64, 256])
def test_unit_impulse_gives_all_ones(oracle_mod, N):
    v = np.zeros(N, dtype=np.complex128)
    v[0] = 1.0
    assert np.allclose(oracle_mod.fft(v, -1), np.ones(N), atol=1e-14)
    # shifted impulse: a pure phase ramp with the forward (negative) sign
    v[:] = 0
    v[1] = 1.0
    k = np.arange(N)
    assert np.allclose(oracle_mod.fft(v, -1), np.exp(-2j * np.pi * k / N), atol=1e-13)


def test_parseval_on_untruncated_forward_stage(oracle_mod):
    x = crandn(5, 128)
    Xh = oracle_mod.forward_spectrum1d(x)
    lhs = np.sum(np.abs(x.astype(np.complex128)) ** 2, axis=-1)
    rhs = np.sum(np.abs(Xh) ** 2, axis=-1) / 128
    assert np.allclose(lhs, rhs, rtol=1e-13)


# ------------------------------------------------------------------- 1-D op --

def dirichlet(N, K):
    """D(n) = (1/N) sum_{k<K} exp(2 pi i k n / N), closed form."""
    n = np.arange(N)
    out = np.empty(N, dtype=np.complex128)
    out[0] = K / N
    nz = n[1:]
    out[1:] = (1 - np.exp(2j * np.pi * K * nz / N)) / (1 - np.exp(2j * np.pi * nz / N)) / N
    return out


@pytest.mark.parametrize("N,K", [(64, 16), (256, 64), (64, 64), (32, 8), (128, 1)])
def test_impulse_closed_form(oracle_mod, N, K):
    C_in, C_out, c0 = 3, 4, 1
    x = np.zeros((2, C_in, N), dtype=np.complex64)
    x[0, c0, 0] = 1.0
    x[1, c0, 0] = 2.0 - 1.0j
    W = crandn(C_in, C_out)
    y, _ = oracle_mod.spectral_conv1d(x, W, K)
    D = dirichlet(N, K)
    for o in range(C_out):
        assert np.allclose(y[0, o], W[c0, o].astype(np.complex128) * D, atol=1e-13)
        assert np.allclose(y[1, o], (2.0 - 1.0j) * W[c0, o].astype(np.complex128) * D, atol=1e-13)


@pytest.mark.parametrize("N,K", [(64, 16), (256, 64), (1024, 128)])
def test_single_exponential_selects_low_bins_only(oracle_mod, N, K):
    """x = exp(2 pi i k0 n/N): passes (times W) iff k0 < K; bins N-K..N-1 are NOT kept."""
    C_in, C_out, c0 = 2, 3, 0
    W = crandn(C_in, C_out)
    n = np.arange(N)
    for k0 in [0, 1, K - 1, K, K + 1, N // 2, N - K, N - 1]:
        x = np.zeros((1, C_in, N), dtype=np.complex128)
        x[0, c0] = np.exp(2j * np.pi * k0 * n / N)
        x32 = x.astype(np.complex64)
        y, _ = oracle_mod.spectral_conv1d(x32, W, K)
        # the fp32-rounded exponential leaks ~1e-7 into other bins
        if k0 < K:
            want = W[c0].astype(np.complex128)[:, None] * x32[0, c0].astype(np.complex128)[None, :]
            assert np.max(np.abs(y[0] - want)) < 5e-6
        else:
            assert np.max(np.abs(y[0])) < 5e-6


@pytest.mark.parametrize("N", [16, 64, 256])
def test_round_trip_identity(oracle_mod, N):
    C = 5
    x = crandn(3, C, N)
    W = np.eye(C, dtype=np.complex64)
    y, _ = oracle_mod.spectral_conv1d(x, W, N)
    assert np.max(np.abs(y - x)) < 1e-13 * N


def test_projection_is_idempotent_and_energy(oracle_mod):
    N, K, C = 128, 32, 4
    x = crandn(2, C, N)
    W = np.eye(C, dtype=np.complex64)
    y, _ = oracle_mod.spectral_conv1d(x, W, K)
    y32 = y.astype(np.complex64)
    y2, _ = oracle_mod.spectral_conv1d(y32, W, K)
    assert np.max(np.abs(y2 - y32)) < 1e-6          # fp32 rounding of the re-fed input only
    Xh = oracle_mod.forward_spectrum1d(x[0])
    assert np.allclose(np.sum(np.abs(y[0]) ** 2, -1), np.sum(np.abs(Xh[:, :K]) ** 2, -1) / N, rtol=1e-12)


def test_linearity_in_x_and_W(oracle_mod):
    N, K, Ci, Co = 64, 16, 6, 5
    # small integers are exact in fp32, so a*x1 + x2 is representable
    x1 = (rng.integers(-8, 9, (2, Ci, N)) + 1j * rng.integers(-8, 9, (2, Ci, N))).astype(np.complex64)
    x2 = (rng.integers(-8, 9, (2, Ci, N)) + 1j * rng.integers(-8, 9, (2, Ci, N))).astype(np.complex64)
    W1 = (rng.integers(-4, 5, (Ci, Co)) + 1j * rng.integers(-4, 5, (Ci, Co))).astype(np.complex64)
    W2 = (rng.integers(-4, 5, (Ci, Co)) + 1j * rng.integers(-4, 5, (Ci, Co))).astype(np.complex64)
    f = lambda x, W: oracle_mod.spectral_conv1d(x, W, K)[0]
    a = 3 - 2j
    assert np.allclose(f((a * x1 + x2).astype(np.complex64), W1), a * f(x1, W1) + f(x2, W1), atol=1e-10)
    assert np.allclose(f(x1, (a * W1 + W2).astype(np.complex64)), a * f(x1, W1) + f(x1, W2), atol=1e-10)


def test_commutation_with_channel_mixing(oracle_mod):
    """W is mode independent, so conv(x, W) = P(x . W) = (P x) . W with P = conv(., I)."""
    N, K, Ci, Co = 128, 32, 7, 3
    x = (rng.integers(-8, 9, (2, Ci, N)) + 1j * rng.integers(-8, 9, (2, Ci, N))).astype(np.complex64)
    W = (rng.integers(-4, 5, (Ci, Co)) + 1j * rng.integers(-4, 5, (Ci, Co))).astype(np.complex64)
    direct, _ = oracle_mod.spectral_conv1d(x, W, K)
    mixed_first = np.einsum("bcn,co->bon", x, W).astype(np.complex64)      # exact in fp32 (small ints)
    a, _ = oracle_mod.spectral_conv1d(mixed_first, np.eye(Co, dtype=np.complex64), K)
    Px, _ = oracle_mod.spectral_conv1d(x, np.eye(Ci, dtype=np.complex64), K)
    b = np.einsum("bcn,co->bon", Px, W.astype(np.complex128))
    assert np.allclose(direct, a, atol=1e-10)
    assert np.allclose(direct, b, atol=1e-10)


def test_W_orientation_and_no_conjugate(oracle_mod):
    """One-hot W[c0,o0] = i routes channel c0 to output o0, multiplied by +i (not -i), and only there."""
    N, K, Ci, Co, c0, o0 = 32, 32, 3, 4, 2, 1
    x = crandn(1, Ci, N)
    W = np.zeros((Ci, Co), dtype=np.complex64)
    W[c0, o0] = 1j
    y, _ = oracle_mod.spectral_conv1d(x, W, K)
    for o in range(Co):
        want = 1j * x[0, c0].astype(np.complex128) if o == o0 else 0
        assert np.max(np.abs(y[0, o] - want)) < 1e-12


@pytest.mark.parametrize("cfg", inputs.CONFIGS[:2], ids=lambda c: c.name)
def test_against_numpy_pipeline_on_benchmark_inputs(oracle_mod, cfg):
    x, W = inputs.make_workload(cfg)
    y, _ = oracle_mod.spectral_conv1d(x, W, cfg.K)
    Xh = np.fft.fft(x.astype(np.complex128), axis=-1)[..., :cfg.K]
    Yh = np.einsum("bck,co->bok", Xh, W.astype(np.complex128))
    pad = np.zeros((cfg.B, cfg.C_out, cfg.N), dtype=np.complex128)
    pad[..., :cfg.K] = Yh
    ref = np.fft.ifft(pad, axis=-1)
    assert np.max(np.abs(ref - y)) < 1e-12
    # E|y|^2 = 4K/N for these distributions (loose statistical sanity)
    assert abs(np.mean(np.abs(y) ** 2) / (4 * cfg.K / cfg.N) - 1) < 0.2


# ------------------------------------------------------------------- 2-D op --

def test_2d_matches_numpy_fft2(oracle_mod):
    B, Ci, Co, N, K = 2, 3, 4, 64, 16
    x = crandn(B, Ci, N, N)
    W = crandn(Ci, Co)
    y, _ = oracle_mod.spectral_conv2d(x, W, K)
    Xh = np.fft.fft2(x.astype(np.complex128))[..., :K, :K]
    Yh = np.einsum("bcxy,co->boxy", Xh, W.astype(np.complex128))
    pad = np.zeros((B, Co, N, N), dtype=np.complex128)
    pad[..., :K, :K] = Yh
    ref = np.fft.ifft2(pad)
    assert np.max(np.abs(ref - y)) < 1e-12


def test_2d_single_exponential_corner_only(oracle_mod):
    N, K = 32, 8
    W = crandn(1, 1)
    n1, n2 = np.meshgrid(np.arange(N), np.arange(N), indexing="ij")
    for (k1, k2), keep in [((0, 0), True), ((K - 1, K - 1), True), ((3, 5), True), ((K, 0), False),
                           ((0, K), False), ((N - 1, 0), False), ((0, N - 1), False), ((N - 1, N - 1), False)]:
        x = np.exp(2j * np.pi * (k1 * n1 + k2 * n2) / N)[None, None].astype(np.complex64)
        y, _ = oracle_mod.spectral_conv2d(x, W, K)
        if keep:
            assert np.max(np.abs(y[0, 0] - W[0, 0].astype(np.complex128) * x[0, 0])) < 5e-6
        else:
            assert np.max(np.abs(y)) < 5e-6


def test_2d_round_trip_and_separability(oracle_mod):
    N, C = 32, 3
    x = crandn(2, C, N, N)
    I = np.eye(C, dtype=np.complex64)
    y, _ = oracle_mod.spectral_conv2d(x, I, N)
    assert np.max(np.abs(y - x)) < 1e-12
    # P_2d = P_axis1 o P_axis2: apply the 1-D operator along the last axis, then along the first
    K = 8
    y2, _ = oracle_mod.spectral_conv2d(x, I, K)
    rows = x.transpose(0, 2, 1, 3).reshape(2 * N, C, N)                       # [(b,n1), c, n2]
    p_last, _ = oracle_mod.spectral_conv1d(np.ascontiguousarray(rows), I, K)
    p_last = p_last.reshape(2, N, C, N).transpose(0, 2, 1, 3)                 # [b, c, n1, n2]
    F = np.fft.fft(p_last, axis=2)
    F[:, :, K:, :] = 0
    both = np.fft.ifft(F, axis=2)
    assert np.max(np.abs(both - y2)) < 1e-6   # p_last is fed back in fp32


def test_2d_transposed_image_gives_transposed_result(oracle_mod):
    """Axis handling: swapping the two spatial axes of x swaps them in y."""
    N, K = 32, 8
    x = crandn(1, 2, N, N)
    W = crandn(2, 2)
    y, _ = oracle_mod.spectral_conv2d(x, W, K)
    yt, _ = oracle_mod.spectral_conv2d(np.ascontiguousarray(x.transpose(0, 1, 3, 2)), W, K)
    assert np.max(np.abs(yt.transpose(0, 1, 3, 2) - y)) < 1e-12


# ------------------------------------------------- 2-D op on a non-square grid --

@pytest.mark.parametrize("N1,N2,K1,K2", [(32, 64, 8, 16), (64, 32, 16, 4), (16, 128, 16, 32), (12, 20, 5, 3)])
def test_rect_matches_numpy_fft2(oracle_mod, N1, N2, K1, K2):
    B, Ci, Co = 2, 3, 2
    x = crandn(B, Ci, N1, N2)
    W = crandn(Ci, Co)
    y, _ = oracle_mod.spectral_conv2d_rect(x, W, K1, K2)
    Xh = np.fft.fft2(x.astype(np.complex128))[..., :K1, :K2]
    pad = np.zeros((B, Co, N1, N2), dtype=np.complex128)
    pad[..., :K1, :K2] = np.einsum("bcxy,co->boxy", Xh, W.astype(np.complex128))
    assert np.max(np.abs(np.fft.ifft2(pad) - y)) < 1e-12


def test_rect_single_exponential_keeps_each_axis_own_modes(oracle_mod):
    """A plane wave (k1, k2) survives iff k1 < K1 AND k2 < K2: catches swapped axis lengths or swapped mode counts."""
    N1, N2, K1, K2 = 16, 64, 4, 24
    W = crandn(1, 1)
    n1, n2 = np.meshgrid(np.arange(N1), np.arange(N2), indexing="ij")
    for (k1, k2), keep in [((0, 0), True), ((K1 - 1, K2 - 1), True), ((2, 20), True), ((K1, 0), False),
                           ((0, K2), False), ((3, K2), False), ((K1, K2 - 1), False), ((N1 - 1, N2 - 1), False)]:
        x = np.exp(2j * np.pi * (k1 * n1 / N1 + k2 * n2 / N2))[None, None].astype(np.complex64)
        y, _ = oracle_mod.spectral_conv2d_rect(x, W, K1, K2)
        if keep:
            assert np.max(np.abs(y[0, 0] - W[0, 0].astype(np.complex128) * x[0, 0])) < 5e-6
        else:
            assert np.max(np.abs(y)) < 5e-6


def test_rect_transpose_swaps_axes_and_square_case_is_the_square_function(oracle_mod):
    N1, N2, K1, K2 = 32, 16, 8, 2
    x = crandn(1, 2, N1, N2)
    W = crandn(2, 3)
    y, _ = oracle_mod.spectral_conv2d_rect(x, W, K1, K2)
    yt, _ = oracle_mod.spectral_conv2d_rect(np.ascontiguousarray(x.transpose(0, 1, 3, 2)), W, K2, K1)
    assert np.max(np.abs(yt.transpose(0, 1, 3, 2) - y)) < 1e-12
    xs = crandn(1, 2, 32, 32)
    a, _ = oracle_mod.spectral_conv2d_rect(xs, W, 8, 8)
    b, _ = oracle_mod.spectral_conv2d(xs, W, 8)
    assert np.array_equal(a, b)


def test_rect_with_one_row_is_the_1d_operator(oracle_mod):
    """N1 = K1 = 1 reduces the 2-D operator to the 1-D one along the last axis."""
    B, Ci, Co, N, K = 2, 3, 2, 64, 16
    x = crandn(B, Ci, 1, N)
    W = crandn(Ci, Co)
    y2, _ = oracle_mod.spectral_conv2d_rect(x, W, 1, K)
    y1, _ = oracle_mod.spectral_conv1d(np.ascontiguousarray(x[:, :, 0, :]), W, K)
    assert np.max(np.abs(y2[:, :, 0, :] - y1)) < 1e-13


# ------------------------------------------------------ per-mode weights --

def test_permode_1d_matches_numpy_einsum(oracle_mod):
    B, Ci, Co, N, K = 3, 4, 5, 64, 12
    x = crandn(B, Ci, N)
    W = crandn(Ci, Co, K)
    y, _ = oracle_mod.spectral_conv1d_permode(x, W)
    Xh = np.fft.fft(x.astype(np.complex128))[..., :K]
    pad = np.zeros((B, Co, N), dtype=np.complex128)
    pad[..., :K] = np.einsum("bik,iok->bok", Xh, W.astype(np.complex128))
    assert np.max(np.abs(np.fft.ifft(pad) - y)) < 1e-12


def test_permode_2d_matches_numpy_einsum(oracle_mod):
    B, Ci, Co, N1, N2, K1, K2 = 2, 3, 2, 16, 32, 5, 7
    x = crandn(B, Ci, N1, N2)
    W = crandn(Ci, Co, K1, K2)
    y, _ = oracle_mod.spectral_conv2d_permode(x, W)
    Xh = np.fft.fft2(x.astype(np.complex128))[..., :K1, :K2]
    pad = np.zeros((B, Co, N1, N2), dtype=np.complex128)
    pad[..., :K1, :K2] = np.einsum("bixy,ioxy->boxy", Xh, W.astype(np.complex128))
    assert np.max(np.abs(np.fft.ifft2(pad) - y)) < 1e-12


def test_permode_with_equal_matrices_is_the_shared_weight_operator(oracle_mod):
    x = crandn(2, 3, 32)
    W = crandn(3, 4)
    a, _ = oracle_mod.spectral_conv1d_permode(x, np.ascontiguousarray(np.repeat(W[:, :, None], 8, axis=2)))
    b, _ = oracle_mod.spectral_conv1d(x, W, 8)
    assert np.array_equal(a, b)
    x2 = crandn(1, 3, 16, 8)
    a, _ = oracle_mod.spectral_conv2d_permode(x2, np.ascontiguousarray(np.broadcast_to(W[:, :, None, None], (3, 4, 4, 2))))
    b, _ = oracle_mod.spectral_conv2d_rect(x2, W, 4, 2)
    assert np.array_equal(a, b)


def test_permode_plane_wave_picks_its_own_matrix(oracle_mod):
    """A plane wave of mode k is multiplied by W[:, :, k] and by no other matrix: catches a wrong mode index, a
    transposed (k1, k2) and a wrong channel orientation."""
    N, K = 32, 6
    W = crandn(2, 3, K)
    n = np.arange(N)
    for k in range(K):
        x = np.zeros((1, 2, N), dtype=np.complex64)
        x[0, 1] = np.exp(2j * np.pi * k * n / N)
        y, _ = oracle_mod.spectral_conv1d_permode(x, W)
        want = W[1, :, k].astype(np.complex128)[:, None] * x[0, 1].astype(np.complex128)[None, :]
        assert np.max(np.abs(y[0] - want)) < 5e-6
    N1, N2, K1, K2 = 8, 16, 3, 5
    W2 = crandn(1, 1, K1, K2)
    n1, n2 = np.meshgrid(np.arange(N1), np.arange(N2), indexing="ij")
    for (k1, k2) in [(0, 0), (2, 4), (1, 3), (2, 0), (0, 4)]:
        x = np.exp(2j * np.pi * (k1 * n1 / N1 + k2 * n2 / N2))[None, None].astype(np.complex64)
        y, _ = oracle_mod.spectral_conv2d_permode(x, W2)
        assert np.max(np.abs(y[0, 0] - W2[0, 0, k1, k2].astype(np.complex128) * x[0, 0])) < 5e-6


# ------------------------------------------------------ real-valued layer --

@pytest.mark.parametrize("N,K", [(64, 16), (32, 16), (128, 1), (12, 5), (256, 64)])
def test_real_matches_numpy_rfft_irfft(oracle_mod, N, K):
    B, Ci, Co = 2, 3, 4
    x = rng.standard_normal((B, Ci, N)).astype(np.float32)
    W = crandn(Ci, Co)
    y, _ = oracle_mod.spectral_conv1d_real(x, W, K)
    half = np.zeros((B, Co, N // 2 + 1), dtype=np.complex128)
    half[..., :K] = np.einsum("bck,co->bok", np.fft.rfft(x.astype(np.float64))[..., :K], W.astype(np.complex128))
    assert np.max(np.abs(np.fft.irfft(half, n=N) - y)) < 1e-12


def test_real_is_twice_the_real_part_of_the_complex_operator_minus_the_mean_term(oracle_mod):
    """For real x: y_real = 2 Re(y_c2c) - Re(mean term), the identity a C2C-based kernel uses (bin 0 counted once)."""
    B, Ci, Co, N, K = 2, 3, 2, 64, 12
    x = rng.standard_normal((B, Ci, N)).astype(np.float32)
    W = crandn(Ci, Co)
    yr, _ = oracle_mod.spectral_conv1d_real(x, W, K)
    yc, _ = oracle_mod.spectral_conv1d(x.astype(np.complex64), W, K)
    y0, _ = oracle_mod.spectral_conv1d(x.astype(np.complex64), W, 1)          # the k = 0 term alone
    assert np.max(np.abs(yr - (2 * yc.real - y0.real))) < 1e-12


def test_real_cosine_closed_form(oracle_mod):
    """x = cos(2 pi k n / N) with k < K and real w gives w x; with k >= K it gives 0; a constant passes with Re(w)."""
    N, K = 64, 8
    n = np.arange(N)
    W = np.array([[0.75 - 0.5j]], dtype=np.complex64)
    for k, keep in [(3, True), (7, True), (8, False), (20, False)]:
        x = np.cos(2 * np.pi * k * n / N)[None, None].astype(np.float32)
        y, _ = oracle_mod.spectral_conv1d_real(x, W, K)
        # W X[k] e^{i t} + conj(W X[k]) e^{-i t} with X[k] = N/2: |W| cos(t + arg W)
        want = np.abs(W[0, 0]) * np.cos(2 * np.pi * k * n / N + np.angle(W[0, 0])) if keep else np.zeros(N)
        assert np.max(np.abs(y[0, 0] - want)) < 5e-6
    y, _ = oracle_mod.spectral_conv1d_real(np.ones((1, 1, N), dtype=np.float32), W, K)
    assert np.max(np.abs(y - 0.75)) < 1e-12


@pytest.mark.parametrize("N,M", [(64, 16), (32, 16), (12, 5), (128, 1)])
def test_fno1d_matches_numpy_rfft_einsum_irfft(oracle_mod, N, M):
    B, Ci, Co = 2, 3, 4
    x = rng.standard_normal((B, Ci, N)).astype(np.float32)
    W = crandn(Ci, Co, M)
    y, _ = oracle_mod.fno1d_real(x, W)
    half = np.zeros((B, Co, N // 2 + 1), dtype=np.complex128)
    half[..., :M] = np.einsum("bix,iox->box", np.fft.rfft(x.astype(np.float64))[..., :M], W.astype(np.complex128))
    assert np.max(np.abs(np.fft.irfft(half, n=N) - y)) < 1e-12
    # equal matrices: the shared-weight real layer
    Ws = crandn(Ci, Co)
    a, _ = oracle_mod.fno1d_real(x, np.ascontiguousarray(np.repeat(Ws[:, :, None], M, axis=2)))
    b, _ = oracle_mod.spectral_conv1d_real(x, Ws, M)
    assert np.array_equal(a, b)


# ------------------------------------------------------ FNO 2-D layer on real fields --

@pytest.mark.parametrize("N1,N2,M1,M2", [(16, 16, 4, 4), (32, 16, 6, 8), (8, 64, 4, 12), (64, 32, 1, 1), (12, 20, 3, 5)])
def test_fno2d_matches_numpy_rfft2_irfft2(oracle_mod, N1, N2, M1, M2):
    """The reference formulation: rfft2, the two low-frequency corners with their own weights, irfft2."""
    B, Ci, Co = 2, 3, 2
    x = rng.standard_normal((B, Ci, N1, N2)).astype(np.float32)
    W = crandn(Ci, Co, 2 * M1, M2)
    y, _ = oracle_mod.fno2d_real(x, W)
    xf = np.fft.rfft2(x.astype(np.float64))
    out = np.zeros((B, Co, N1, N2 // 2 + 1), dtype=np.complex128)
    Wd = W.astype(np.complex128)
    out[:, :, :M1, :M2] = np.einsum("bixy,ioxy->boxy", xf[:, :, :M1, :M2], Wd[:, :, M1:, :])       # k1 = 0 .. M1-1
    out[:, :, -M1:, :M2] = np.einsum("bixy,ioxy->boxy", xf[:, :, -M1:, :M2], Wd[:, :, :M1, :])     # k1 = -M1 .. -1
    assert np.max(np.abs(np.fft.irfft2(out, s=(N1, N2)) - y)) < 1e-12


def test_fno2d_plane_wave_picks_its_mode(oracle_mod):
    """cos(2 pi (k1 n1/N1 + k2 n2/N2)) is scaled and phase-shifted by W[.., k1 + M1, k2] alone (k2 > 0): catches a wrong
    sign of k1, swapped blocks and swapped axes."""
    N1, N2, M1, M2 = 16, 32, 3, 5
    W = crandn(1, 1, 2 * M1, M2)
    n1, n2 = np.meshgrid(np.arange(N1), np.arange(N2), indexing="ij")
    for (k1, k2) in [(2, 3), (-3, 1), (-1, 4), (0, 2)]:
        ph = 2 * np.pi * (k1 * n1 / N1 + k2 * n2 / N2)
        x = np.cos(ph)[None, None].astype(np.float32)
        y, _ = oracle_mod.fno2d_real(x, W)
        w = W[0, 0, k1 + M1, k2].astype(np.complex128)
        assert np.max(np.abs(y[0, 0] - np.abs(w) * np.cos(ph + np.angle(w)))) < 5e-6
    x = np.cos(2 * np.pi * (M1 * n1 / N1 + 2 * n2 / N2))[None, None].astype(np.float32)      # k1 = M1: outside
    assert np.max(np.abs(oracle_mod.fno2d_real(x, W)[0])) < 5e-6
