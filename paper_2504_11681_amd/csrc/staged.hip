// Unfused baseline: the five-stage structure the paper attributes to the PyTorch Fourier
// layer (Sec. 1 and Sec. 2.1: FFT, frequency filter copy, CGEMM, zero-pad copy, iFFT as separate
// kernels with every intermediate in global memory).  Simple, general kernels (any N up to 4096 --
// a radix-2 transform for powers of two, a direct sum otherwise --, any K, any channel count); they
// are the reference point for the fused/staged ratio.
#include "common.h"
#include "staged.h"

namespace tfno {

// ---------------------------------------------------------------------------------------------
// Full N-point transform of PC pencils per workgroup, radix-2 Stockham autosort in LDS.
// Pencil q (global index) has element n at  base(q) + n * elem_stride  with
//   base(q) = (q / inner_count) * outer_stride + (q % inner_count)      (all in complex elements).
// Last-axis transform:  inner_count = 1, outer_stride = N, elem_stride = 1.
// First-axis transform of [rows=N, cols] images: inner_count = cols, outer_stride = N*cols,
// elem_stride = cols; the PC pencils of a workgroup are then adjacent columns (coalesced).
// Only elements n < n_in are read (the rest of the input is taken as zero) and only n < n_out are
// written; input and output may use different outer strides, which gives a transform with built-in
// zero padding / truncation for the first axis of the 2-D pipeline.
// in == out is allowed when both sides use the same strides (a workgroup reads all of its pencils
// before it writes any).
// ---------------------------------------------------------------------------------------------
template <int DIR>
__global__ void __launch_bounds__(256)
k_staged_fft(const c64 *__restrict__ in, c64 *__restrict__ out, int N, int log2N, int PC,
             long long num_pencils, long long inner_count, long long in_outer_stride,
             long long out_outer_stride, long long elem_stride, int n_in, int n_out, float scale)
{
    extern __shared__ float2 lds[];
    c64 *buf0 = lds;                  // [PC][N]
    c64 *buf1 = lds + (size_t)PC * N; // [PC][N]
    c64 *tw = buf1 + (size_t)PC * N;  // [N/2] : exp(DIR * 2 pi i m / N)

    const int tid = threadIdx.x, nth = blockDim.x;
    const long long q0 = (long long)blockIdx.x * PC;

    for (int m = tid; m < N / 2; m += nth) tw[m] = cis2pi((float)(DIR * m), (float)N);

    const int total = PC * N;
    if (elem_stride == 1) {
        for (int i = tid; i < total; i += nth) {
            int j = i / N, n = i - j * N;
            long long q = q0 + j;
            if (q < num_pencils)
                buf0[j * N + n] = n < n_in ? in[(q / inner_count) * in_outer_stride + (q % inner_count) + n]
                                           : make_float2(0.f, 0.f);
        }
    } else {
        for (int i = tid; i < total; i += nth) {
            int n = i / PC, j = i - n * PC;
            long long q = q0 + j;
            if (q < num_pencils)
                buf0[j * N + n] = n < n_in ? in[(q / inner_count) * in_outer_stride + (q % inner_count) + n * elem_stride]
                                           : make_float2(0.f, 0.f);
        }
    }
    __syncthreads();

    c64 *src = buf0, *dst = buf1;
    const int half = N >> 1;
    for (int s = 0; s < log2N; ++s) {
        const int Ns = 1 << s;
        const int tw_step = half >> s;            // N / (2 Ns)
        for (int i = tid; i < PC * half; i += nth) {
            int j = i / half, t = i - j * half;
            int k = t & (Ns - 1);
            c64 a = src[j * N + t];
            c64 b = cmul(src[j * N + t + half], tw[k * tw_step]);
            int o = ((t - k) << 1) + k;           // (t / Ns) * 2 Ns + k
            dst[j * N + o] = cadd(a, b);
            dst[j * N + o + Ns] = csub(a, b);
        }
        __syncthreads();
        c64 *tmp = src; src = dst; dst = tmp;
    }

    if (elem_stride == 1) {
        for (int i = tid; i < total; i += nth) {
            int j = i / N, n = i - j * N;
            long long q = q0 + j;
            if (q < num_pencils && n < n_out) {
                c64 v = src[j * N + n];
                out[(q / inner_count) * out_outer_stride + (q % inner_count) + n] = make_float2(v.x * scale, v.y * scale);
            }
        }
    } else {
        for (int i = tid; i < total; i += nth) {
            int n = i / PC, j = i - n * PC;
            long long q = q0 + j;
            if (q < num_pencils && n < n_out) {
                c64 v = src[j * N + n];
                out[(q / inner_count) * out_outer_stride + (q % inner_count) + n * elem_stride] =
                    make_float2(v.x * scale, v.y * scale);
            }
        }
    }
}

// The same transform for lengths that are not powers of two, as the direct sum
//   out[k] = scale * sum_{n < n_in} in[n] exp(DIR 2 pi i k n / N),   k < n_out
// (n_in * n_out complex multiply-adds per pencil; addressing, zero padding, truncation and aliasing rules as above).
template <int DIR>
__global__ void __launch_bounds__(256)
k_staged_dft(const c64 *__restrict__ in, c64 *__restrict__ out, int N, int PC, long long num_pencils,
             long long inner_count, long long in_outer_stride, long long out_outer_stride, long long elem_stride,
             int n_in, int n_out, float scale)
{
    extern __shared__ float2 lds[];
    c64 *buf = lds;                   // [PC][N]
    c64 *tw = lds + (size_t)PC * N;   // [N] : exp(DIR * 2 pi i m / N)
    const int tid = threadIdx.x, nth = blockDim.x;
    const long long q0 = (long long)blockIdx.x * PC;
    for (int m = tid; m < N; m += nth) tw[m] = cis2pi((float)(DIR * m), (float)N);
    // consecutive threads take consecutive addresses: along the pencil when it is contiguous, across pencils otherwise
    const bool along = elem_stride == 1;
    for (int i = tid; i < PC * n_in; i += nth) {
        const int n = along ? i % n_in : i / PC, j = along ? i / n_in : i % PC;
        const long long q = q0 + j;
        if (q < num_pencils) buf[j * N + n] = in[(q / inner_count) * in_outer_stride + (q % inner_count) + n * elem_stride];
    }
    __syncthreads();
    for (int i = tid; i < PC * n_out; i += nth) {
        const int k = along ? i % n_out : i / PC, j = along ? i / n_out : i % PC;
        const long long q = q0 + j;
        if (q >= num_pencils) continue;
        c64 acc = make_float2(0.f, 0.f);
        int idx = 0;                  // (k n) mod N
        for (int n = 0; n < n_in; ++n) {
            acc = cmac(acc, buf[j * N + n], tw[idx]);
            idx += k;
            if (idx >= N) idx -= N;
        }
        out[(q / inner_count) * out_outer_stride + (q % inner_count) + k * elem_stride] = make_float2(acc.x * scale, acc.y * scale);
    }
}

// Frequency filter: keep rows [0,Kr) x cols [0,Kc) of every [R, Cc] image.   out: [imgs, Kr, Kc]
__global__ void __launch_bounds__(256)
k_staged_truncate(const c64 *__restrict__ in, c64 *__restrict__ out, long long imgs, int R, int Cc, int Kr, int Kc)
{
    long long total = imgs * Kr * Kc;
    for (long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (long long)gridDim.x * blockDim.x) {
        long long img = i / ((long long)Kr * Kc);
        int rem = (int)(i - img * Kr * Kc);
        int r = rem / Kc, c = rem - r * Kc;
        out[i] = in[(img * R + r) * Cc + c];
    }
}

// Zero padding: out [imgs, R, Cc] gets in [imgs, Kr, Kc] in its low corner, zeros elsewhere.
__global__ void __launch_bounds__(256)
k_staged_pad(const c64 *__restrict__ in, c64 *__restrict__ out, long long imgs, int R, int Cc, int Kr, int Kc)
{
    long long total = imgs * R * Cc;
    for (long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (long long)gridDim.x * blockDim.x) {
        long long img = i / ((long long)R * Cc);
        int rem = (int)(i - img * R * Cc);
        int r = rem / Cc, c = rem - r * Cc;
        out[i] = (r < Kr && c < Kc) ? in[(img * Kr + r) * Kc + c] : make_float2(0.f, 0.f);
    }
}

// Complex linear layer over the hidden dimension, one W for all modes (Sec. 3.1):
//   Yh[b, o, m] = sum_c Xh[b, c, m] * W[c, o],   m < M (M = K or K*K retained modes).
// grid (B * ceil(M/64), ceil(C_out/16)); block 256 = 64 modes x 4 groups of 4 outputs.
__global__ void __launch_bounds__(256)
k_staged_cgemm(const c64 *__restrict__ Xh, const c64 *__restrict__ W, c64 *__restrict__ Yh,
               int C_in, int C_out, int M, int mtiles)
{
    const long long b = blockIdx.x / mtiles;
    const int m = (blockIdx.x % mtiles) * 64 + (threadIdx.x & 63);
    const int o0 = blockIdx.y * 16 + (threadIdx.x >> 6) * 4;
    if (m >= M) return;
    c64 acc[4];
    for (int i = 0; i < 4; ++i) acc[i] = make_float2(0.f, 0.f);
    const c64 *xp = Xh + b * C_in * (long long)M + m;
    for (int c = 0; c < C_in; ++c) {
        c64 xv = xp[(long long)c * M];
        for (int i = 0; i < 4; ++i)
            if (o0 + i < C_out) acc[i] = cmac(acc[i], xv, W[(long long)c * C_out + o0 + i]);
    }
    for (int i = 0; i < 4; ++i)
        if (o0 + i < C_out) Yh[(b * C_out + o0 + i) * (long long)M + m] = acc[i];
}

// ------------------------------------------------------------------------------ host side --

static int ilog2(int n) { int l = 0; while ((1 << l) < n) ++l; return l; }

hipError_t launch_axis_fft(int dir, const c64 *in, c64 *out, int N, long long num_pencils,
                           long long inner_count, long long in_outer_stride, long long out_outer_stride,
                           long long elem_stride, int n_in, int n_out, float scale, hipStream_t s)
{
    static LdsLimitOnce fft_limit, dft_limit;
    hipError_t e = fft_limit.set({reinterpret_cast<const void *>(&k_staged_fft<-1>),
                                  reinterpret_cast<const void *>(&k_staged_fft<+1>)}, 96 * 1024);
    if (e != hipSuccess) return e;
    if (num_pencils == 0) return hipSuccess;
    int PC = 4096 / N; if (PC > 16) PC = 16; if (PC < 1) PC = 1;
    if (inner_count > 1) { while (PC > 1 && inner_count % PC) PC >>= 1; }
    if ((N & (N - 1)) != 0) {                               // not a power of two: direct sum
        e = dft_limit.set({reinterpret_cast<const void *>(&k_staged_dft<-1>),
                           reinterpret_cast<const void *>(&k_staged_dft<+1>)}, 96 * 1024);
        if (e != hipSuccess) return e;
        const size_t dlds = ((size_t)PC * N + N) * sizeof(c64);
        const long long dblocks = (num_pencils + PC - 1) / PC;
        if (dir < 0)
            hipLaunchKernelGGL(k_staged_dft<-1>, dim3((unsigned)dblocks), dim3(256), dlds, s, in, out, N, PC, num_pencils,
                               inner_count, in_outer_stride, out_outer_stride, elem_stride, n_in, n_out, scale);
        else
            hipLaunchKernelGGL(k_staged_dft<+1>, dim3((unsigned)dblocks), dim3(256), dlds, s, in, out, N, PC, num_pencils,
                               inner_count, in_outer_stride, out_outer_stride, elem_stride, n_in, n_out, scale);
        return hipGetLastError();
    }
    size_t lds = ((size_t)2 * PC * N + N / 2) * sizeof(c64);
    long long blocks = (num_pencils + PC - 1) / PC;
    int threads = 256;
    if (dir < 0)
        hipLaunchKernelGGL(k_staged_fft<-1>, dim3((unsigned)blocks), dim3(threads), lds, s, in, out, N, ilog2(N), PC,
                           num_pencils, inner_count, in_outer_stride, out_outer_stride, elem_stride, n_in, n_out, scale);
    else
        hipLaunchKernelGGL(k_staged_fft<+1>, dim3((unsigned)blocks), dim3(threads), lds, s, in, out, N, ilog2(N), PC,
                           num_pencils, inner_count, in_outer_stride, out_outer_stride, elem_stride, n_in, n_out, scale);
    return hipGetLastError();
}

static hipError_t launch_fft(int dir, const c64 *in, c64 *out, int N, long long num_pencils,
                             long long inner_count, long long outer_stride, long long elem_stride,
                             float scale, hipStream_t s)
{
    return launch_axis_fft(dir, in, out, N, num_pencils, inner_count, outer_stride, outer_stride, elem_stride, N, N, scale, s);
}

static unsigned copy_blocks(long long total)
{
    long long b = (total + 255) / 256;
    if (b > 65536 * 16) b = 65536 * 16;
    if (b < 1) b = 1;
    return (unsigned)b;
}

size_t staged_workspace_bytes(long long B, int C_in, int C_out, int N1, int N2, int K1, int K2)
{
    const size_t pts = (size_t)N1 * N2, kpts = (size_t)K1 * K2;
    // full spectrum, truncated spectrum, contracted spectrum, padded spectrum
    return sizeof(c64) * (size_t)B * ((size_t)C_in * pts + (size_t)C_in * kpts + (size_t)C_out * kpts + (size_t)C_out * pts);
}

hipError_t staged_conv(int dims, const c64 *x, const c64 *W, c64 *y, long long B, int C_in, int C_out,
                       int N1, int N2, int K1, int K2, c64 *ws, hipStream_t s)
{
    const int N = N2, K = K2;                  // the last (contiguous) axis; 1-D calls have N1 = K1 = 1
    const size_t pts = (size_t)N1 * N2, kpts = (size_t)K1 * K2;
    c64 *S = ws;                               // [B, C_in, pts]   full spectrum
    c64 *T = S + (size_t)B * C_in * pts;       // [B, C_in, kpts]  truncated
    c64 *Yh = T + (size_t)B * C_in * kpts;     // [B, C_out, kpts] contracted
    c64 *P = Yh + (size_t)B * C_out * kpts;    // [B, C_out, pts]  zero padded
    hipError_t e;
    const long long in_imgs = B * C_in, out_imgs = B * C_out;

    if (dims == 1) {
        if ((e = launch_fft(-1, x, S, N, in_imgs, 1, N, 1, 1.f, s)) != hipSuccess) return e;
        hipLaunchKernelGGL(k_staged_truncate, dim3(copy_blocks(in_imgs * K)), dim3(256), 0, s, S, T, in_imgs, 1, N, 1, K);
    } else {
        if ((e = launch_fft(-1, x, S, N, in_imgs * N1, 1, N, 1, 1.f, s)) != hipSuccess) return e;
        if ((e = launch_fft(-1, S, S, N1, in_imgs * N, N, (long long)N1 * N, N, 1.f, s)) != hipSuccess) return e;
        hipLaunchKernelGGL(k_staged_truncate, dim3(copy_blocks(in_imgs * kpts)), dim3(256), 0, s, S, T, in_imgs, N1, N, K1, K);
    }
    if ((e = hipGetLastError()) != hipSuccess) return e;

    {
        const int mtiles = (int)((kpts + 63) / 64);
        dim3 grid((unsigned)(B * mtiles), (unsigned)((C_out + 15) / 16));
        hipLaunchKernelGGL(k_staged_cgemm, grid, dim3(256), 0, s, T, W, Yh, C_in, C_out, (int)kpts, mtiles);
        if ((e = hipGetLastError()) != hipSuccess) return e;
    }

    if (dims == 1) {
        hipLaunchKernelGGL(k_staged_pad, dim3(copy_blocks(out_imgs * N)), dim3(256), 0, s, Yh, P, out_imgs, 1, N, 1, K);
        if ((e = hipGetLastError()) != hipSuccess) return e;
        return launch_fft(+1, P, y, N, out_imgs, 1, N, 1, 1.f / (float)N, s);
    }
    hipLaunchKernelGGL(k_staged_pad, dim3(copy_blocks(out_imgs * pts)), dim3(256), 0, s, Yh, P, out_imgs, N1, N, K1, K);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    if ((e = launch_fft(+1, P, P, N1, out_imgs * N, N, (long long)N1 * N, N, 1.f / (float)N1, s)) != hipSuccess) return e;
    return launch_fft(+1, P, y, N, out_imgs * N1, 1, N, 1, 1.f / (float)N, s);
}

}  // namespace tfno
