/*
 * TEST INFRASTRUCTURE -- NOT PART OF THE PRODUCT PATH.
 *
 * Float64 CPU oracle for the FNO Fourier-layer spectral convolution of
 * TurboFNO (arxiv 2504.11681).  Only tests, the smoke check and the
 * benchmark's cpu_baseline leg may link or call this file.  It shares no
 * code, header, table or constant with the HIP library.
 *
 * What it computes is the plain definition of the operator (Sec. 2.1: forward
 * FFT, truncation to the low modes, complex linear layer over the hidden
 * dimension, zero padding back to full length, inverse FFT; Sec. 3.1 fixes the
 * GEMM shape M = batch x modes, N = OutputDim, K = HiddenDim, i.e. ONE weight
 * matrix shared by every mode; Sec. 3.3 fixes which bins survive: the first
 * K of N along each transformed axis).  Fusion, pruning, built-in truncation
 * and built-in padding (Sec. 3.3, Sec. 4) only skip or reorder exact
 * arithmetic, so the definition itself is the oracle:
 *
 *   Xh[b,c,k] = sum_n  x[b,c,n] exp(-2 pi i k n / N)            k = 0..K-1
 *   Yh[b,o,k] = sum_c  Xh[b,c,k] W[c,o]
 *   y [b,o,n] = (1/N) sum_{k<K} Yh[b,o,k] exp(+2 pi i k n / N)   n = 0..N-1
 *
 * and in 2-D the same with (n1,n2), (k1,k2) in [0,K)x[0,K), scale 1/N^2; for a
 * non-square grid N1 x N2 each axis keeps its own first K1 / K2 bins, scale
 * 1/(N1 N2).
 *
 * Readings taken where the paper is silent: forward exponent negative, inverse
 * positive and scaled by 1/N per axis (the cuFFT/PyTorch convention the paper
 * benchmarks against, Sec. 5); no conjugation of W; W is [C_in, C_out]
 * row-major; tensors are [B, C, N] / [B, C, N, N] row-major interleaved
 * (re, im).
 *
 * No blocking, no pruning, no fusion: a full N-point transform is taken and
 * bins are then discarded / zero-filled.  Transform: direct O(N^2) DFT for
 * N <= 32 or N not a power of two, textbook recursive radix-2
 * decimation-in-time otherwise.  Contraction: naive triple loop.
 */
#include <complex.h>
#include <math.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

typedef double complex cplx;

static const double TWO_PI = 6.283185307179586476925286766559;

/* out[k] = sum_n in[n] exp(sign * 2 pi i k n / N), strided input/output. */
void oracle_dft_direct(const cplx *in, long istride, cplx *out, long ostride, int N, int sign)
{
    for (int k = 0; k < N; ++k) {
        cplx acc = 0.0;
        for (int n = 0; n < N; ++n) {
            /* reduce k*n mod N before forming the angle: keeps the argument small */
            long kn = ((long)k * (long)n) % N;
            double ang = sign * TWO_PI * (double)kn / (double)N;
            acc += in[n * istride] * (cos(ang) + I * sin(ang));
        }
        out[k * ostride] = acc;
    }
}

/* Recursive radix-2 decimation in time.  N power of two.  tmp: N scratch. */
static void fft_rec(const cplx *in, long istride, cplx *out, int N, int sign, cplx *tmp)
{
    if (N == 1) { out[0] = in[0]; return; }
    int h = N / 2;
    /* even samples -> out[0..h), odd samples -> out[h..N), each transformed */
    fft_rec(in,           2 * istride, tmp,     h, sign, out);
    fft_rec(in + istride, 2 * istride, tmp + h, h, sign, out + h);
    for (int k = 0; k < h; ++k) {
        double ang = sign * TWO_PI * (double)k / (double)N;
        cplx w = cos(ang) + I * sin(ang);
        cplx e = tmp[k], o = w * tmp[h + k];
        out[k]     = e + o;
        out[k + h] = e - o;
    }
}

static int is_pow2(int n) { return n > 0 && (n & (n - 1)) == 0; }

/* Full N-point transform of a strided sequence into a contiguous buffer.
 * out and scratch hold N elements each; no scaling. */
void oracle_fft(const cplx *in, long istride, cplx *out, int N, int sign, cplx *scratch)
{
    if (N <= 32 || !is_pow2(N))
        oracle_dft_direct(in, istride, out, 1, N, sign);
    else
        fft_rec(in, istride, out, N, sign, scratch);
}

/* Same, forcing the radix-2 path (N power of two); for the pin tests. */
void oracle_fft_radix2(const cplx *in, long istride, cplx *out, int N, int sign, cplx *scratch)
{
    fft_rec(in, istride, out, N, sign, scratch);
}

/* ------------------------------------------------------------------ 1-D -- */

/* Weight applied to mode m (of M retained modes) between input channel c and output channel o.
 * per_mode = 0: one matrix W[C_in, C_out] shared by every mode, the GEMM of Sec. 3.1.
 * per_mode = 1: W[C_in, C_out, M], an own matrix per retained mode, modes innermost -- the learned
 * transformation of the Fourier layer as the FNO model the paper accelerates defines it (Sec. 1,
 * Sec. 2.1 step 3); in 2-D the mode index is m = k1 K2 + k2. */
static cplx weight(const float *W, int c, int o, int C_out, size_t m, size_t M, int per_mode)
{
    size_t idx = per_mode ? ((size_t)c * C_out + o) * M + m : (size_t)c * C_out + o;
    return (double)W[2 * idx] + I * (double)W[2 * idx + 1];
}

/* One batch element.  x: [C_in, N] c64 (float pairs).  W: [C_in, C_out] c64.
 * y: [C_out, N] complex double.  Xh_full (optional, may be NULL): [C_in, N]
 * untruncated forward spectra, for the Parseval pin. */
static void conv1d_one(const float *x, const float *W, cplx *y, cplx *Xh_full,
                       int C_in, int C_out, int N, int K, int per_mode)
{
    cplx *sig = malloc(sizeof(cplx) * N);
    cplx *spec = malloc(sizeof(cplx) * N);
    cplx *scr = malloc(sizeof(cplx) * N);
    cplx *Xh = malloc(sizeof(cplx) * (size_t)C_in * K);   /* truncated */
    cplx *Yh = malloc(sizeof(cplx) * (size_t)C_out * K);

    /* forward transform of every input channel, keep bins 0..K-1 (Sec. 3.3) */
    for (int c = 0; c < C_in; ++c) {
        for (int n = 0; n < N; ++n)
            sig[n] = (double)x[2 * ((size_t)c * N + n)] + I * (double)x[2 * ((size_t)c * N + n) + 1];
        oracle_fft(sig, 1, spec, N, -1, scr);
        if (Xh_full) memcpy(Xh_full + (size_t)c * N, spec, sizeof(cplx) * N);
        for (int k = 0; k < K; ++k) Xh[(size_t)c * K + k] = spec[k];
    }
    /* complex linear layer over the hidden dimension (Sec. 3.1: the same W for every mode; per_mode: W[.,.,k]) */
    for (int o = 0; o < C_out; ++o)
        for (int k = 0; k < K; ++k) {
            cplx acc = 0.0;
            for (int c = 0; c < C_in; ++c) acc += Xh[(size_t)c * K + k] * weight(W, c, o, C_out, (size_t)k, (size_t)K, per_mode);
            Yh[(size_t)o * K + k] = acc;
        }
    /* zero-pad to N, inverse transform, scale 1/N */
    for (int o = 0; o < C_out; ++o) {
        for (int k = 0; k < N; ++k) spec[k] = (k < K) ? Yh[(size_t)o * K + k] : 0.0;
        oracle_fft(spec, 1, sig, N, +1, scr);
        for (int n = 0; n < N; ++n) y[(size_t)o * N + n] = sig[n] / (double)N;
    }
    free(sig); free(spec); free(scr); free(Xh); free(Yh);
}

/* x: [B, C_in, N] c64;  W: [C_in, C_out] c64;  y: [B, C_out, N] complex128.
 * Batch elements are independent and are spread over `threads` host threads.
 * Returns the number of threads actually used, or -1 on bad arguments. */
static int conv1d_batch(const float *x, const float *W, double *y,
                        int B, int C_in, int C_out, int N, int K, int threads, int per_mode)
{
    if (!x || !W || !y || B < 0 || C_in <= 0 || C_out <= 0 || N <= 0 || K <= 0 || K > N) return -1;
    int used = 1;
#ifdef _OPENMP
    if (threads > 0) omp_set_num_threads(threads);
    #pragma omp parallel
    {
        #pragma omp single
        used = omp_get_num_threads();
        #pragma omp for schedule(dynamic, 1)
        for (int b = 0; b < B; ++b)
            conv1d_one(x + 2 * (size_t)b * C_in * N, W, (cplx *)y + (size_t)b * C_out * N, NULL,
                       C_in, C_out, N, K, per_mode);
    }
#else
    (void)threads;
    for (int b = 0; b < B; ++b)
        conv1d_one(x + 2 * (size_t)b * C_in * N, W, (cplx *)y + (size_t)b * C_out * N, NULL,
                   C_in, C_out, N, K, per_mode);
#endif
    return used;
}

int oracle_spectral_conv1d(const float *x, const float *W, double *y,
                           int B, int C_in, int C_out, int N, int K, int threads)
{
    return conv1d_batch(x, W, y, B, C_in, C_out, N, K, threads, 0);
}

/* The same with an own weight matrix per retained mode: W is [C_in, C_out, K]. */
int oracle_spectral_conv1d_permode(const float *x, const float *W, double *y,
                                   int B, int C_in, int C_out, int N, int K, int threads)
{
    return conv1d_batch(x, W, y, B, C_in, C_out, N, K, threads, 1);
}

/* Real-valued variant (the R2C / C2R transforms FNO layers apply to real fields; Sec. 2.1 describes the same
 * pipeline for the C2C case the paper measures).  x: [B, C_in, N] float32 REAL, W: [C_in, C_out] c64,
 * y: [B, C_out, N] float64 REAL, K <= N/2:
 *
 *   Xh[b,c,k] = sum_n x[b,c,n] exp(-2 pi i k n / N),  k < K          (the first K bins of the R2C transform)
 *   Yh[b,o,k] = sum_c Xh[b,c,k] W[c,o]
 *   y[b,o,:]  = C2R_N(Yh padded with zeros to N/2 + 1 bins)
 *
 * where C2R is the inverse transform of the Hermitian extension: F[0] = Re Yh[0], F[k] = Yh[k] and
 * F[N-k] = conj(Yh[k]) for 0 < k < K, zero elsewhere; y = (1/N) * inverse DFT of F, whose imaginary part
 * vanishes and is dropped. */
static void conv1d_real_one(const float *x, const float *W, double *y, int C_in, int C_out, int N, int K, int per_mode)
{
    cplx *sig = malloc(sizeof(cplx) * N), *spec = malloc(sizeof(cplx) * N), *scr = malloc(sizeof(cplx) * N);
    cplx *Xh = malloc(sizeof(cplx) * (size_t)C_in * K), *Yh = malloc(sizeof(cplx) * (size_t)C_out * K);
    for (int c = 0; c < C_in; ++c) {
        for (int n = 0; n < N; ++n) sig[n] = (double)x[(size_t)c * N + n];
        oracle_fft(sig, 1, spec, N, -1, scr);
        for (int k = 0; k < K; ++k) Xh[(size_t)c * K + k] = spec[k];
    }
    for (int o = 0; o < C_out; ++o)
        for (int k = 0; k < K; ++k) {
            cplx acc = 0.0;
            for (int c = 0; c < C_in; ++c) acc += Xh[(size_t)c * K + k] * weight(W, c, o, C_out, (size_t)k, (size_t)K, per_mode);
            Yh[(size_t)o * K + k] = acc;
        }
    for (int o = 0; o < C_out; ++o) {
        for (int k = 0; k < N; ++k) spec[k] = 0.0;
        spec[0] = creal(Yh[(size_t)o * K]);
        for (int k = 1; k < K; ++k) {
            spec[k] = Yh[(size_t)o * K + k];
            spec[N - k] = conj(Yh[(size_t)o * K + k]);
        }
        oracle_fft(spec, 1, sig, N, +1, scr);
        for (int n = 0; n < N; ++n) y[(size_t)o * N + n] = creal(sig[n]) / (double)N;
    }
    free(sig); free(spec); free(scr); free(Xh); free(Yh);
}

static int conv1d_real_batch(const float *x, const float *W, double *y,
                             int B, int C_in, int C_out, int N, int K, int threads, int per_mode)
{
    if (!x || !W || !y || B < 0 || C_in <= 0 || C_out <= 0 || N <= 0 || K <= 0 || 2 * K > N) return -1;
    int used = 1;
#ifdef _OPENMP
    if (threads > 0) omp_set_num_threads(threads);
    #pragma omp parallel
    {
        #pragma omp single
        used = omp_get_num_threads();
        #pragma omp for schedule(dynamic, 1)
        for (int b = 0; b < B; ++b)
            conv1d_real_one(x + (size_t)b * C_in * N, W, y + (size_t)b * C_out * N, C_in, C_out, N, K, per_mode);
    }
#else
    (void)threads;
    for (int b = 0; b < B; ++b)
        conv1d_real_one(x + (size_t)b * C_in * N, W, y + (size_t)b * C_out * N, C_in, C_out, N, K, per_mode);
#endif
    return used;
}

int oracle_spectral_conv1d_real(const float *x, const float *W, double *y,
                                int B, int C_in, int C_out, int N, int K, int threads)
{
    return conv1d_real_batch(x, W, y, B, C_in, C_out, N, K, threads, 0);
}

/* The 1-D Fourier layer of FNO models on real fields: as above with an own weight matrix per retained mode,
 * W [C_in, C_out, M] (M = K modes). */
int oracle_fno1d_real(const float *x, const float *W, double *y,
                      int B, int C_in, int C_out, int N, int M, int threads)
{
    return conv1d_real_batch(x, W, y, B, C_in, C_out, N, M, threads, 1);
}

/* Untruncated forward spectra of one [C, N] block (no scaling): Xh[c,k], k < N. */
int oracle_forward_spectrum1d(const float *x, double *Xh, int C, int N)
{
    if (!x || !Xh || C <= 0 || N <= 0) return -1;
    cplx *sig = malloc(sizeof(cplx) * N), *scr = malloc(sizeof(cplx) * N);
    for (int c = 0; c < C; ++c) {
        for (int n = 0; n < N; ++n)
            sig[n] = (double)x[2 * ((size_t)c * N + n)] + I * (double)x[2 * ((size_t)c * N + n) + 1];
        oracle_fft(sig, 1, (cplx *)Xh + (size_t)c * N, N, -1, scr);
    }
    free(sig); free(scr);
    return 0;
}

/* ------------------------------------------------------------------ 2-D -- */

/* In-place full 2-D transform of an N1 x N2 row-major image (no scaling):
 * every row along the last axis (length N2), then every column along the
 * first (length N1).  line and scr hold max(N1, N2) values. */
static void fft2_inplace(cplx *img, int N1, int N2, int sign, cplx *line, cplx *scr)
{
    for (int r = 0; r < N1; ++r) {
        oracle_fft(img + (size_t)r * N2, 1, line, N2, sign, scr);
        memcpy(img + (size_t)r * N2, line, sizeof(cplx) * N2);
    }
    for (int c = 0; c < N2; ++c) {
        oracle_fft(img + c, N2, line, N1, sign, scr);
        for (int r = 0; r < N1; ++r) img[(size_t)r * N2 + c] = line[r];
    }
}

/* One batch element.  x: [C_in, N1, N2] c64;  y: [C_out, N1, N2] complex double.
 * Each transformed axis keeps its own first K_i of N_i bins (Sec. 3.2 / 3.3: the
 * 2-D transform is separable and truncation / padding act per axis). */
static void conv2d_one(const float *x, const float *W, cplx *y,
                       int C_in, int C_out, int N1, int N2, int K1, int K2, int per_mode)
{
    size_t NN = (size_t)N1 * N2, KK = (size_t)K1 * K2;
    int NL = N1 > N2 ? N1 : N2;
    cplx *img = malloc(sizeof(cplx) * NN);
    cplx *line = malloc(sizeof(cplx) * NL), *scr = malloc(sizeof(cplx) * NL);
    cplx *Xh = malloc(sizeof(cplx) * C_in * KK);
    cplx *Yh = malloc(sizeof(cplx) * C_out * KK);

    for (int c = 0; c < C_in; ++c) {
        const float *xc = x + 2 * (size_t)c * NN;
        for (size_t i = 0; i < NN; ++i) img[i] = (double)xc[2 * i] + I * (double)xc[2 * i + 1];
        fft2_inplace(img, N1, N2, -1, line, scr);
        /* keep the single low corner [0,K1) x [0,K2) */
        for (int k1 = 0; k1 < K1; ++k1)
            for (int k2 = 0; k2 < K2; ++k2)
                Xh[c * KK + (size_t)k1 * K2 + k2] = img[(size_t)k1 * N2 + k2];
    }
    for (int o = 0; o < C_out; ++o)
        for (size_t m = 0; m < KK; ++m) {
            cplx acc = 0.0;
            for (int c = 0; c < C_in; ++c) acc += Xh[c * KK + m] * weight(W, c, o, C_out, m, KK, per_mode);
            Yh[o * KK + m] = acc;
        }
    double scale = 1.0 / ((double)N1 * (double)N2);
    for (int o = 0; o < C_out; ++o) {
        for (size_t i = 0; i < NN; ++i) img[i] = 0.0;
        for (int k1 = 0; k1 < K1; ++k1)
            for (int k2 = 0; k2 < K2; ++k2)
                img[(size_t)k1 * N2 + k2] = Yh[o * KK + (size_t)k1 * K2 + k2];
        fft2_inplace(img, N1, N2, +1, line, scr);
        cplx *yo = y + (size_t)o * NN;
        for (size_t i = 0; i < NN; ++i) yo[i] = img[i] * scale;
    }
    free(img); free(line); free(scr); free(Xh); free(Yh);
}

/* x: [B, C_in, N1, N2] c64;  W: [C_in, C_out] c64;  y: [B, C_out, N1, N2] complex128.
 * Modes kept: k1 < K1 along the first axis, k2 < K2 along the last. */
static int conv2d_batch(const float *x, const float *W, double *y, int B, int C_in, int C_out,
                        int N1, int N2, int K1, int K2, int threads, int per_mode)
{
    if (!x || !W || !y || B < 0 || C_in <= 0 || C_out <= 0 || N1 <= 0 || N2 <= 0 || K1 <= 0 || K2 <= 0 ||
        K1 > N1 || K2 > N2)
        return -1;
    int used = 1;
    size_t NN = (size_t)N1 * N2;
#ifdef _OPENMP
    if (threads > 0) omp_set_num_threads(threads);
    #pragma omp parallel
    {
        #pragma omp single
        used = omp_get_num_threads();
        #pragma omp for schedule(dynamic, 1)
        for (int b = 0; b < B; ++b)
            conv2d_one(x + 2 * (size_t)b * C_in * NN, W, (cplx *)y + (size_t)b * C_out * NN,
                       C_in, C_out, N1, N2, K1, K2, per_mode);
    }
#else
    (void)threads;
    for (int b = 0; b < B; ++b)
        conv2d_one(x + 2 * (size_t)b * C_in * NN, W, (cplx *)y + (size_t)b * C_out * NN,
                   C_in, C_out, N1, N2, K1, K2, per_mode);
#endif
    return used;
}

int oracle_spectral_conv2d_rect(const float *x, const float *W, double *y, int B, int C_in, int C_out,
                                int N1, int N2, int K1, int K2, int threads)
{
    return conv2d_batch(x, W, y, B, C_in, C_out, N1, N2, K1, K2, threads, 0);
}

/* The same with an own weight matrix per retained mode: W is [C_in, C_out, K1, K2]. */
int oracle_spectral_conv2d_permode(const float *x, const float *W, double *y, int B, int C_in, int C_out,
                                   int N1, int N2, int K1, int K2, int threads)
{
    return conv2d_batch(x, W, y, B, C_in, C_out, N1, N2, K1, K2, threads, 1);
}

/* The square case the paper evaluates (Sec. 5): N x N points, K x K modes. */
int oracle_spectral_conv2d(const float *x, const float *W, double *y,
                           int B, int C_in, int C_out, int N, int K, int threads)
{
    return oracle_spectral_conv2d_rect(x, W, y, B, C_in, C_out, N, N, K, K, threads);
}

/* The 2-D Fourier layer as FNO models apply it to real fields (Sec. 1, Sec. 2.1: R2C transform, low modes,
 * learned weights per mode, zero padding, C2R transform), in the layout of the public FNO implementations:
 * x: [B, C_in, N1, N2] float32 REAL;  y: [B, C_out, N1, N2] float64 REAL;
 * W: [C_in, C_out, 2 M1, M2] c64, an own matrix per retained mode; along the first axis the retained
 * frequencies are k1 = -M1 .. M1-1 (both low-frequency blocks of the full-length axis, index j = k1 + M1 in W),
 * along the last axis k2 = 0 .. M2-1 of the half spectrum.  2 M1 <= N1, M2 <= N2 / 2.
 *
 *   Xh[c, k1, k2] = sum_{n1, n2} x[c, n1, n2] exp(-2 pi i (k1 n1 / N1 + k2 n2 / N2))
 *   Yh[o, k1, k2] = sum_c Xh[c, k1, k2] W[c, o, k1 + M1, k2]
 *   y = C2R over the last axis of the inverse transform over the first axis of Yh (zero elsewhere), / (N1 N2)
 *
 * The C2R step is written as the full inverse of the Hermitian extension F[N1 - k1, N2 - k2] = conj F[k1, k2],
 * with the k2 = 0 column taken as the Hermitian part the C2R transform sees (its imaginary input at n2-frequency
 * zero is ignored by taking the real part of the column's inverse along the first axis). */
static void fno2d_one(const float *x, const float *W, double *y, int C_in, int C_out, int N1, int N2, int M1, int M2)
{
    size_t NN = (size_t)N1 * N2, KK = (size_t)2 * M1 * M2;
    int NL = N1 > N2 ? N1 : N2;
    cplx *img = malloc(sizeof(cplx) * NN), *line = malloc(sizeof(cplx) * NL), *scr = malloc(sizeof(cplx) * NL);
    cplx *Xh = malloc(sizeof(cplx) * C_in * KK), *Yh = malloc(sizeof(cplx) * C_out * KK);
    for (int c = 0; c < C_in; ++c) {
        for (size_t i = 0; i < NN; ++i) img[i] = (double)x[(size_t)c * NN + i];
        fft2_inplace(img, N1, N2, -1, line, scr);
        for (int j = 0; j < 2 * M1; ++j) {
            int k1 = j - M1, row = (k1 + N1) % N1;
            for (int k2 = 0; k2 < M2; ++k2) Xh[c * KK + (size_t)j * M2 + k2] = img[(size_t)row * N2 + k2];
        }
    }
    for (int o = 0; o < C_out; ++o)
        for (size_t m = 0; m < KK; ++m) {
            cplx acc = 0.0;
            for (int c = 0; c < C_in; ++c) acc += Xh[c * KK + m] * weight(W, c, o, C_out, m, KK, 1);
            Yh[o * KK + m] = acc;
        }
    double scale = 1.0 / ((double)N1 * (double)N2);
    for (int o = 0; o < C_out; ++o) {
        /* half spectrum H[row, k2], k2 <= N2/2, zero outside the retained blocks */
        for (size_t i = 0; i < NN; ++i) img[i] = 0.0;
        for (int j = 0; j < 2 * M1; ++j) {
            int row = (j - M1 + N1) % N1;
            for (int k2 = 0; k2 < M2; ++k2) img[(size_t)row * N2 + k2] = Yh[o * KK + (size_t)j * M2 + k2];
        }
        /* inverse along the first axis (complex), column by column */
        for (int k2 = 0; k2 < M2; ++k2) {
            oracle_fft(img + k2, N2, line, N1, +1, scr);
            for (int r = 0; r < N1; ++r) img[(size_t)r * N2 + k2] = line[r];
        }
        /* C2R along the last axis of every row: Hermitian extension, inverse, real part */
        for (int r = 0; r < N1; ++r) {
            cplx *rowp = img + (size_t)r * N2;
            rowp[0] = creal(rowp[0]);
            for (int k2 = 1; k2 < M2; ++k2) rowp[N2 - k2] = conj(rowp[k2]);
            oracle_fft(rowp, 1, line, N2, +1, scr);
            for (int n2 = 0; n2 < N2; ++n2) y[(size_t)o * NN + (size_t)r * N2 + n2] = creal(line[n2]) * scale;
        }
    }
    free(img); free(line); free(scr); free(Xh); free(Yh);
}

int oracle_fno2d_real(const float *x, const float *W, double *y, int B, int C_in, int C_out,
                      int N1, int N2, int M1, int M2, int threads)
{
    if (!x || !W || !y || B < 0 || C_in <= 0 || C_out <= 0 || N1 <= 0 || N2 <= 0 || M1 <= 0 || M2 <= 0 ||
        2 * M1 > N1 || 2 * M2 > N2)
        return -1;
    int used = 1;
    size_t NN = (size_t)N1 * N2;
#ifdef _OPENMP
    if (threads > 0) omp_set_num_threads(threads);
    #pragma omp parallel
    {
        #pragma omp single
        used = omp_get_num_threads();
        #pragma omp for schedule(dynamic, 1)
        for (int b = 0; b < B; ++b)
            fno2d_one(x + (size_t)b * C_in * NN, W, y + (size_t)b * C_out * NN, C_in, C_out, N1, N2, M1, M2);
    }
#else
    (void)threads;
    for (int b = 0; b < B; ++b)
        fno2d_one(x + (size_t)b * C_in * NN, W, y + (size_t)b * C_out * NN, C_in, C_out, N1, N2, M1, M2);
#endif
    return used;
}

/* Thin complex128 entry points for the pin tests (buffers interleaved doubles). */
void oracle_fft_c128(const double *in, double *out, int N, int sign)
{
    cplx *scr = malloc(sizeof(cplx) * (N > 0 ? N : 1));
    oracle_fft((const cplx *)in, 1, (cplx *)out, N, sign, scr);
    free(scr);
}
void oracle_fft_radix2_c128(const double *in, double *out, int N, int sign)
{
    cplx *scr = malloc(sizeof(cplx) * (N > 0 ? N : 1));
    oracle_fft_radix2((const cplx *)in, 1, (cplx *)out, N, sign, scr);
    free(scr);
}
void oracle_dft_direct_c128(const double *in, double *out, int N, int sign)
{
    oracle_dft_direct((const cplx *)in, 1, (cplx *)out, 1, N, sign);
}
