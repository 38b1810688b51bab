// Pruned transforms of long pencils, N = N1 * 256 with N1 in {8, 16} (N = 2048, 4096), for the three-kernel 1-D
// variant (pruned FFT, CGEMM over the retained modes, pruned iFFT; variant "A" of Table 2 with the truncation,
// padding and pruning of Sec. 3.3).
//
// A pencil is read as an N1 x 256 row-major array, n = 256 n1 + n2, and its spectrum indexed k = k1 + N1 k2:
//
//   X[k1 + N1 k2] = sum_{n2} w_256^(n2 k2) * [ w_N^(n2 k1) * sum_{n1} x[256 n1 + n2] w_N1^(n1 k1) ]
//
// so the first K = N1 K2 bins are, for EVERY k1, the first K2 bins of a 256-point transform: the truncation of the
// long transform becomes the truncation (and output pruning) of its 256-point rows.
//
//   stage 1  thread n2 = tid holds x[256 n1 + n2] for all n1 (coalesced 2 KiB rows), full N1-point DFT in registers,
//            twiddle w_N^(n2 k1) (per-thread constants, computed once per workgroup)
//   exchange through LDS to the row layout of the 256-point transform: 16 lanes per row k1, lane p holds
//            n2 = p + 16 j
//   stage 2  the 256-point output-pruned row transform of the short-pencil kernels (16-point DFT in registers,
//            twiddle, transpose through a 16-lane patch, pruned 16-point DFT)
//
// A sweep of the workgroup is 16 rows: one pencil of 4096 points or two of 2048.  The inverse kernel runs the
// transposed network.  Inside the truncated-spectrum buffers a pencil's K modes are stored in the order
// k1 K2 + k2 (consecutive lanes then write consecutive addresses); the contraction shares one W across all modes
// (Sec. 3.1), so any order works as long as both transforms agree.
#pragma once
#include "pruned1d_kernel.h"

namespace tfno {

template <int N1, int K2>
struct CfgLong {
    static constexpr int N = N1 * 256, K = N1 * K2;
    static constexpr int G = 16 / N1;           // pencils per sweep
    static constexpr int KH = K2 / 16;          // retained outputs per column of the 256-point transform
    static constexpr int RS = 272;              // row stride of the exchange buffer: rows g, g + 1 start 32 banks apart
    static_assert(N1 == 8 || N1 == 16, "N in {2048, 4096}");
    static_assert(K2 % 16 == 0 && KH >= 1 && KH <= 16 && (KH & (KH - 1)) == 0, "K / N1 in {16, 32, 64, 128, 256}");
};

// per-thread set-up shared by both kernels: the 256-point twiddle table and this thread's w_N^(tid k1)
template <int N1>
__device__ __forceinline__ void long_setup(c64 *TW, c64 *tw0, int tid)
{
    TW[tid] = cis2pi(-(float)((tid >> 4) * (tid & 15)), 256.f);       // [c][p]: w_256^(p c)
#pragma unroll
    for (int k1 = 1; k1 < N1; ++k1) tw0[k1] = cis2pi(-(float)(tid * k1), (float)(N1 * 256));
    tw0[0] = make_float2(1.f, 0.f);
}

// x: [npencils, N] contiguous (pencil q = b * C + c).  Xh: mode-tile major over the joint mode index b K + m.
template <int N1, int K2>
__global__ void __launch_bounds__(256, 3)
k_fwd1d_long(const c64 *__restrict__ x, c64 *__restrict__ Xh, int C, long long npencils, int K_keep)
{
    using Cf = CfgLong<N1, K2>;
    constexpr int N = Cf::N, K = Cf::K, G = Cf::G, KH = Cf::KH, RS = Cf::RS;
    // exchange buffer [16][RS]; its first 16 * 256 entries double as the 16 transpose patches of stage 2
    __shared__ __align__(16) c64 E[16 * RS];
    __shared__ c64 TW[256];
    const int tid = threadIdx.x;
    const int g = tid >> 4, p = tid & 15;                   // stage 2: row g of the sweep, lane p of the row
    c64 *patch = E + g * 256;
    c64 tw0[N1];
    long_setup<N1>(TW, tw0, tid);

    const long long nsweeps = (npencils + G - 1) / G;
    if ((long long)blockIdx.x >= nsweeps) return;           // uniform per workgroup; no barrier has been reached
    c64 v[16];
    auto load = [&](long long sweep) __attribute__((always_inline)) {
#pragma unroll
        for (int gl = 0; gl < G; ++gl) {
            long long q = sweep * G + gl;
            if (q >= npencils) q = npencils - 1;            // a valid address; the result is not stored
            const c64 *src = x + q * N + tid;
#pragma unroll
            for (int n1 = 0; n1 < N1; ++n1) v[gl * N1 + n1] = load_nt(src + 256 * n1);
        }
    };
    auto stage = [&](long long sweep, auto refill, long long next_sweep) __attribute__((always_inline)) {
        constexpr bool REFILL = decltype(refill)::value;
        c64 u[16];
#pragma unroll
        for (int gl = 0; gl < G; ++gl) RegFFT<N1, -1, 1>::run(v + gl * N1, u + gl * N1);
        __builtin_amdgcn_sched_barrier(0);
        if constexpr (REFILL) load(next_sweep);             // v is free: in flight during the rest of the sweep
        __builtin_amdgcn_sched_barrier(0);
        __syncthreads();                                    // the previous sweep's patch reads are done
#pragma unroll
        for (int i = 0; i < 16; ++i) E[i * RS + tid] = (i % N1) == 0 ? u[i] : cmul(u[i], tw0[i % N1]);
        __syncthreads();
        c64 r[16], z[16];
#pragma unroll
        for (int j = 0; j < 16; ++j) r[j] = E[g * RS + p + 16 * j];
        __syncthreads();                                    // every row has been read: the patches may overwrite E
        RegFFT<16, -1, 1>::run(r, z);
#pragma unroll
        for (int c = 0; c < 16; ++c) patch[c * 16 + (p ^ c)] = c == 0 ? z[0] : cmul(z[c], TW[c * 16 + p]);
        wave_sync();
        c64 xo[KH];
        dft_prune_out<16, KH, -1>([&](auto ppc) __attribute__((always_inline)) {
            constexpr int pp = decltype(ppc)::value;
            return patch[p * 16 + (pp ^ p)];
        }, xo);
        // row g is output k1 of pencil gl; xo[kh] is its bin k2 = p + 16 kh
        const int gl = g / N1, k1 = g % N1;
        const long long q = sweep * G + gl;
        if (q < npencils) {
            const long long b = q / C;
            const int ch = (int)(q % C);
#pragma unroll
            for (int kh = 0; kh < KH; ++kh)                // true bin k1 + N1 k2 at or past K_keep: finer truncation
                Xh[spec1d_index(b * K + k1 * K2 + p + 16 * kh, ch, C)] =
                    k1 + N1 * (p + 16 * kh) < K_keep ? xo[kh] : make_float2(0.f, 0.f);
        }
    };

    load(blockIdx.x);
    long long sweep = blockIdx.x;
    for (; sweep + gridDim.x < nsweeps; sweep += gridDim.x) stage(sweep, std::true_type{}, sweep + gridDim.x);
    stage(sweep, std::false_type{}, 0);
}

// Yh: mode-tile major (joint mode index b K + k1 K2 + k2, C channels).  y: [npencils, N] contiguous.
template <int N1, int K2>
__global__ void __launch_bounds__(256, 3)
k_inv1d_long(const c64 *__restrict__ Yh, c64 *__restrict__ y, int C, long long npencils)
{
    using Cf = CfgLong<N1, K2>;
    constexpr int N = Cf::N, K = Cf::K, G = Cf::G, KH = Cf::KH, RS = Cf::RS;
    __shared__ __align__(16) c64 E[16 * RS];
    __shared__ c64 TW[256];
    const int tid = threadIdx.x;
    const int g = tid >> 4, p = tid & 15;
    c64 *patch = E + g * 256;
    c64 tw0[N1];
    long_setup<N1>(TW, tw0, tid);

    const long long nsweeps = (npencils + G - 1) / G;
    if ((long long)blockIdx.x >= nsweeps) return;
    c64 yin[KH];
    auto load_spectrum = [&](long long sweep) __attribute__((always_inline)) {
        const int gl = g / N1, k1 = g % N1;
        long long q = sweep * G + gl;
        if (q >= npencils) q = npencils - 1;
        const long long b = q / C;
        const int ch = (int)(q % C);
#pragma unroll
        for (int kh = 0; kh < KH; ++kh) yin[kh] = Yh[spec1d_index(b * K + k1 * K2 + p + 16 * kh, ch, C)];
    };
    auto stage = [&](long long sweep, auto refill, long long next_sweep) __attribute__((always_inline)) {
        constexpr bool REFILL = decltype(refill)::value;
        // zero-padded, input-pruned 256-point inverse of row g (the stage of the short-pencil kernel)
        dft_prune_in<16, KH, +1>(yin, [&](auto ppc, c64 val) __attribute__((always_inline)) {
            constexpr int pp = decltype(ppc)::value;
            patch[p * 16 + (pp ^ p)] = val;
        });
        __builtin_amdgcn_sched_barrier(0);
        if constexpr (REFILL) load_spectrum(next_sweep);    // yin is free
        __builtin_amdgcn_sched_barrier(0);
        wave_sync();
        c64 z[16], res[16];
#pragma unroll
        for (int c = 0; c < 16; ++c) {
            c64 t = patch[c * 16 + (p ^ c)];
            if (c != 0) {
                const c64 w = TW[c * 16 + p];
                t = cmul(t, make_float2(w.x, -w.y));
            }
            z[c] = t;
        }
        RegFFT<16, +1, 1>::run(z, res);                     // res[j]: row g at n2 = p + 16 j
        __syncthreads();                                    // every patch has been read: the rows may overwrite them
#pragma unroll
        for (int j = 0; j < 16; ++j) E[g * RS + p + 16 * j] = res[j];
        __syncthreads();
        c64 u[16], o[16];
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const c64 t = E[i * RS + tid];
            const c64 w = tw0[i % N1];
            u[i] = (i % N1) == 0 ? t : cmul(t, make_float2(w.x, -w.y));
        }
        __syncthreads();                                    // E is free for the next sweep's patches
#pragma unroll
        for (int gl = 0; gl < G; ++gl) RegFFT<N1, +1, 1>::run(u + gl * N1, o + gl * N1);
#pragma unroll
        for (int gl = 0; gl < G; ++gl) {
            const long long q = sweep * G + gl;
            if (q < npencils) {
                c64 *dst = y + q * N + tid;
#pragma unroll
                for (int n1 = 0; n1 < N1; ++n1) store_nt(dst + 256 * n1, o[gl * N1 + n1]);
            }
        }
    };

    load_spectrum(blockIdx.x);
    __syncthreads();                                        // twiddle table is ready
    long long sweep = blockIdx.x;
    for (; sweep + gridDim.x < nsweeps; sweep += gridDim.x) stage(sweep, std::true_type{}, sweep + gridDim.x);
    stage(sweep, std::false_type{}, 0);
}

}  // namespace tfno
