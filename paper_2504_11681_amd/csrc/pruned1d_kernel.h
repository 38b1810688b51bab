// 1-D spectral convolution as three kernels with truncation, zero padding and butterfly pruning built into the
// transforms (Sec. 3.3) but no fusion across the contraction -- the variant the paper calls "A" in Table 2:
//
//   k_fwd1d   pencils x[b, c, :] -> the K retained bins Xh[b, c, k]                       (reads N, writes K)
//   k_cgemm_modes (fused2d_kernel.h)  Yh[b, o, k] = sum_c Xh[b, c, k] W[c, o] / N         (BF16x3 or FP32 MFMA)
//   k_inv1d   zero-padded, input-pruned inverse Yh[b, o, k] -> y[b, o, :]                  (reads K, writes N)
//
// The spectra are stored mode-tile major over the joint mode index m = b K + k ([m / 128][channel][m % 128]), the
// layout the mode CGEMM streams.  Only the truncated spectra cross global memory: 2 K / N of the tensor bytes
// extra, against the fused kernel's none; in exchange the transforms run at high occupancy and the contraction
// runs on the matrix pipe alone, which wins where the fused kernel is bound by its FP32 contraction.
//
// Pencil transform (N = 16 * LPR), as in the 2-D row stage: LPR lanes per pencil, lane p holds x[p + LPR j],
// j < 16; 16-point DFT in registers, twiddle w_N^(p k_lo), transpose through a wave-private XOR-swizzled LDS
// patch, then per column k_lo the LPR-point DFT pruned to the K/16 retained outputs.  For N = 1024 (LPR = 64) a
// wave owns a pencil, four lanes share a column (16 patch entries each) and the partial sums are added across
// the quad with DPP.
#pragma once
#include "common.h"
#include "fft_regs.h"
#include "fused1d_kernel.h"   // wave_sync

namespace tfno {

template <int N, int K>
struct CfgP1 {
    static constexpr int NT = 256;
    static constexpr int LPR = N / 16;                  // lanes per pencil
    static constexpr bool WIDE = LPR > 16;              // N = 1024: a wave per pencil, a quad per column
    static constexpr int PPS = NT / LPR;                // pencils per sweep of the workgroup
    static constexpr int KH = K / 16;                   // retained outputs per column k_lo
    static constexpr int CPL = WIDE ? 1 : 16 / LPR;     // columns per lane (narrow path)
    static constexpr int LPQ = WIDE ? LPR / 4 : LPR;    // patch entries a lane transforms per column
    static constexpr int OPL = WIDE ? (KH >= 4 ? KH / 4 : 1) : KH;   // retained bins a lane ends up with per column
    static constexpr int GS = N + (LPR < 16 ? LPR : 0); // patch stride between the pencils of a sweep
    static constexpr int NY = CPL * KH;                 // spectrum values a lane loads in the inverse kernel
    static constexpr size_t LDS_BYTES = sizeof(c64) * ((size_t)PPS * GS + N + 64);
    static_assert(N == 64 || N == 128 || N == 256 || N == 1024, "N in {64, 128, 256, 1024}");
    static_assert(K % 16 == 0 && K <= N && LPQ % KH == 0, "K / 16 must divide the transform a lane runs per column");
    static_assert(!WIDE || KH == 4 || KH == 8, "N = 1024: K in {64, 128}");
    static_assert(LDS_BYTES <= 64 * 1024, "static LDS limit");
};

template <int CTRL>
__device__ __forceinline__ float p1_quad_perm(float v)
{
    return __int_as_float(__builtin_amdgcn_mov_dpp(__float_as_int(v), CTRL, 0xf, 0xf, true));
}

// element offset of (channel c, joint mode m) in a mode-tile-major spectrum buffer with C channels
__device__ __forceinline__ long long spec1d_index(long long m, int c, int C)
{
    return ((m >> 7) * C + c) * 128 + (m & 127);
}

template <int N, int K>
struct LdsP1 {
    c64 *patch;   // this thread's pencil patch
    c64 *tw;      // [16][LPR]: w_N^(p k_lo)
    c64 *tw64;    // w_64^t (wide path)
};

template <int N, int K>
__device__ __forceinline__ LdsP1<N, K> p1_setup(unsigned char *raw, int tid)
{
    using C = CfgP1<N, K>;
    LdsP1<N, K> l;
    c64 *base = reinterpret_cast<c64 *>(raw);
    l.patch = base + (tid / C::LPR) * C::GS;
    l.tw = base + C::PPS * C::GS;
    l.tw64 = l.tw + N;
    for (int i = tid; i < N; i += C::NT) l.tw[i] = cis2pi(-(float)((i / C::LPR) * (i % C::LPR)), (float)N);
    if (tid < 64) l.tw64[tid] = cis2pi(-(float)tid, 64.f);
    return l;
}

// patch slot of entry (column c, position p)
template <int LPR>
__device__ __forceinline__ int p1_slot(int c, int p)
{
    if constexpr (LPR > 16) return c * 64 + (p ^ (4 * (c & 3)));
    else return c * LPR + (p ^ (c % LPR));
}

// ------------------------------------------------------------------------------------------------ forward
// x: [npencils, N] contiguous (pencil q = b * C + c).  Xh: mode-tile major, joint mode m = b K + k.
// REAL (both kernels): pencils of float32 values.  The forward transform of a real pencil is the complex one with a
// zero imaginary part (its first K bins are the R2C bins); bin 0 is stored halved so that the inverse kernel, which
// stores the real part of the zero-padded complex inverse, yields the C2R transform when the contraction in between
// carries the scale 2 / N.
template <int N, int K, bool REAL = false>
__global__ void __launch_bounds__(256)
k_fwd1d(const c64 *__restrict__ x, c64 *__restrict__ Xh, int C, long long npencils, int K_keep)
{
    using Cf = CfgP1<N, K>;
    constexpr int LPR = Cf::LPR, PPS = Cf::PPS, KH = Cf::KH, CPL = Cf::CPL, OPL = Cf::OPL;
    constexpr bool WIDE = Cf::WIDE;
    __shared__ __align__(16) unsigned char raw[Cf::LDS_BYTES];
    const int tid = threadIdx.x;
    const LdsP1<N, K> L = p1_setup<N, K>(raw, tid);
    const int g = tid / LPR, p = tid % LPR;
    const int kl_w = (tid & 63) >> 2, qa = tid & 3;         // wide path: column and quad position

    const long long nsweeps = (npencils + PPS - 1) / PPS;
    c64 v[16];
    auto load_pencil = [&](long long sweep) __attribute__((always_inline)) {
        long long q = sweep * PPS + g;
        if (q >= npencils) q = npencils - 1;                // a valid address; the result is not stored
        if constexpr (REAL) {
            const float *src = reinterpret_cast<const float *>(x) + q * N + p;
#pragma unroll
            for (int j = 0; j < 16; ++j) v[j] = make_float2(LPR >= 16 ? __builtin_nontemporal_load(src + LPR * j) : src[LPR * j], 0.f);
        } else {
            // (x is read once; non-temporal where the lanes of a pencil cover whole lines, so that the stream does not
            // evict the spectra the contraction reads next)
            const c64 *src = x + q * N + p;
#pragma unroll
            for (int j = 0; j < 16; ++j) v[j] = LPR >= 16 ? load_nt(src + LPR * j) : src[LPR * j];
        }
    };
    auto stage = [&](long long sweep, auto refill, long long next_sweep) __attribute__((always_inline)) {
        constexpr bool REFILL = decltype(refill)::value;
        c64 z[16];
        {
            c64 ea[8], eb[8], za[8], zo[8];
            dif_first_level<16, -1>(v, ea, eb);
            __builtin_amdgcn_sched_barrier(0);
            if constexpr (REFILL) load_pencil(next_sweep);
            __builtin_amdgcn_sched_barrier(0);
            RegFFT<8, -1, 1>::run(ea, za);
            RegFFT<8, -1, 1>::run(eb, zo);
#pragma unroll
            for (int k = 0; k < 8; ++k) { z[2 * k] = za[k]; z[2 * k + 1] = zo[k]; }
        }
        wave_sync();                                        // the previous sweep's patch reads are done
#pragma unroll
        for (int c = 0; c < 16; ++c) {
            const c64 zt = c == 0 ? z[0] : cmul(z[c], L.tw[c * LPR + p]);
            L.patch[p1_slot<LPR>(c, p)] = zt;
        }
        wave_sync();
        const long long q = sweep * PPS + g;
        const bool ok = q < npencils;
        const long long b = q / C;
        const int ch = (int)(q % C);
        if constexpr (!WIDE) {
#pragma unroll
            for (int i = 0; i < CPL; ++i) {
                const int kl = p + LPR * i;                 // kl % LPR == p
                c64 xo[KH];
                dft_prune_out<LPR, KH, -1>([&](auto ppc) __attribute__((always_inline)) {
                    constexpr int pp = decltype(ppc)::value;
                    return L.patch[kl * LPR + (pp ^ p)];
                }, xo);
                if (ok) {
#pragma unroll
                    for (int kh = 0; kh < KH; ++kh) {      // bins K_keep .. K-1: truncation finer than the kernel's K
                        c64 val = kl + 16 * kh < K_keep ? xo[kh] : make_float2(0.f, 0.f);
                        if constexpr (REAL) {
                            if (kl + 16 * kh == 0) val = make_float2(0.5f * val.x, 0.5f * val.y);
                        }
                        Xh[spec1d_index(b * K + kl + 16 * kh, ch, C)] = val;
                    }
                }
            }
        } else {
            const int swz = 4 * (kl_w & 3);
            c64 P[KH];
            dft_prune_out<16, KH, -1>([&](auto ppc) __attribute__((always_inline)) {
                constexpr int pp = decltype(ppc)::value;
                return L.patch[kl_w * 64 + ((qa + 4 * pp) ^ swz)];
            }, P);
#pragma unroll
            for (int kh = 1; kh < KH; ++kh) P[kh] = cmul(P[kh], L.tw64[qa * kh]);
            c64 R[KH / 2], O[OPL];
            {
                const bool hi = (qa & 2) != 0;
#pragma unroll
                for (int i = 0; i < KH / 2; ++i) {
                    const c64 mine = hi ? P[KH / 2 + i] : P[i], send = hi ? P[i] : P[KH / 2 + i];
                    R[i] = make_float2(mine.x + p1_quad_perm<0x4E>(send.x), mine.y + p1_quad_perm<0x4E>(send.y));
                }
            }
            {
                const bool hi = (qa & 1) != 0;
#pragma unroll
                for (int i = 0; i < OPL; ++i) {
                    const c64 mine = hi ? R[OPL + i] : R[i], send = hi ? R[i] : R[OPL + i];
                    O[i] = make_float2(mine.x + p1_quad_perm<0xB1>(send.x), mine.y + p1_quad_perm<0xB1>(send.y));
                }
            }
            if (ok) {
#pragma unroll
                for (int i = 0; i < OPL; ++i)
                {
                    const int k = kl_w + 16 * (OPL * qa + i);
                    c64 val = k < K_keep ? O[i] : make_float2(0.f, 0.f);
                    if constexpr (REAL) {
                        if (k == 0) val = make_float2(0.5f * val.x, 0.5f * val.y);
                    }
                    Xh[spec1d_index(b * K + k, ch, C)] = val;
                }
            }
        }
    };

    if ((long long)blockIdx.x >= nsweeps) return;           // uniform per workgroup; no barrier has been reached
    load_pencil(blockIdx.x);
    __syncthreads();                                        // twiddle tables are ready
    long long sweep = blockIdx.x;
    for (; sweep + gridDim.x < nsweeps; sweep += gridDim.x) stage(sweep, std::true_type{}, sweep + gridDim.x);
    stage(sweep, std::false_type{}, 0);
}

// ------------------------------------------------------------------------------------------------ inverse
// Yh: mode-tile major (joint mode m = b K + k, C channels).  y: [npencils, N] contiguous (pencil q = b * C + o).
template <int N, int K, bool REAL = false>
__global__ void __launch_bounds__(256)
k_inv1d(const c64 *__restrict__ Yh, c64 *__restrict__ y, int C, long long npencils)
{
    using Cf = CfgP1<N, K>;
    constexpr int LPR = Cf::LPR, PPS = Cf::PPS, KH = Cf::KH, CPL = Cf::CPL, NY = Cf::NY;
    constexpr bool WIDE = Cf::WIDE;
    __shared__ __align__(16) unsigned char raw[Cf::LDS_BYTES];
    const int tid = threadIdx.x;
    const LdsP1<N, K> L = p1_setup<N, K>(raw, tid);
    const int g = tid / LPR, p = tid % LPR;
    const int kl_w = (tid & 63) >> 2, qa = tid & 3;

    const long long nsweeps = (npencils + PPS - 1) / PPS;
    c64 yin[NY];                                            // [column i][kh]
    auto load_spectrum = [&](long long sweep) __attribute__((always_inline)) {
        long long q = sweep * PPS + g;
        if (q >= npencils) q = npencils - 1;
        const long long b = q / C;
        const int ch = (int)(q % C);
#pragma unroll
        for (int i = 0; i < CPL; ++i)
#pragma unroll
            for (int kh = 0; kh < KH; ++kh) {
                const int kl = WIDE ? kl_w : p + LPR * i;
                yin[i * KH + kh] = Yh[spec1d_index(b * K + kl + 16 * kh, ch, C)];
            }
    };
    auto stage = [&](long long sweep, auto refill, long long next_sweep) __attribute__((always_inline)) {
        constexpr bool REFILL = decltype(refill)::value;
        wave_sync();                                        // the previous sweep's patch reads are done
        if constexpr (!WIDE) {
#pragma unroll
            for (int i = 0; i < CPL; ++i) {
                const int kl = p + LPR * i;
                dft_prune_in<LPR, KH, +1>(yin + i * KH, [&](auto ppc, c64 val) __attribute__((always_inline)) {
                    constexpr int pp = decltype(ppc)::value;
                    L.patch[kl * LPR + (pp ^ p)] = val;
                });
            }
        } else {
            const int swz = 4 * (kl_w & 3);
            c64 t[KH];
#pragma unroll
            for (int kh = 0; kh < KH; ++kh) {
                t[kh] = yin[kh];
                if (kh != 0) {
                    const c64 w = L.tw64[qa * kh];
                    t[kh] = cmul(t[kh], make_float2(w.x, -w.y));
                }
            }
            dft_prune_in<16, KH, +1>(t, [&](auto ppc, c64 val) __attribute__((always_inline)) {
                constexpr int pp = decltype(ppc)::value;
                L.patch[kl_w * 64 + ((qa + 4 * pp) ^ swz)] = val;
            });
        }
        __builtin_amdgcn_sched_barrier(0);
        if constexpr (REFILL) load_spectrum(next_sweep);    // yin is free: in flight during the row transform
        __builtin_amdgcn_sched_barrier(0);
        wave_sync();
        c64 z[16], res[16];
#pragma unroll
        for (int c = 0; c < 16; ++c) {
            c64 t = L.patch[p1_slot<LPR>(c, p)];
            if (c != 0) {
                const c64 w = L.tw[c * LPR + p];
                t = cmul(t, make_float2(w.x, -w.y));
            }
            z[c] = t;
        }
        RegFFT<16, +1, 1>::run(z, res);
        const long long q = sweep * PPS + g;
        if (q < npencils) {
            if constexpr (REAL) {
                float *dst = reinterpret_cast<float *>(y) + q * N + p;
#pragma unroll
                for (int j = 0; j < 16; ++j) {
                    if constexpr (LPR >= 32) __builtin_nontemporal_store(res[j].x, dst + LPR * j);
                    else dst[LPR * j] = res[j].x;
                }
            } else {
                // (non-temporal only where the lanes of a pencil write whole 128-byte lines)
                c64 *dst = y + q * N + p;
#pragma unroll
                for (int j = 0; j < 16; ++j) {
                    if constexpr (LPR >= 16) store_nt(dst + LPR * j, res[j]);
                    else dst[LPR * j] = res[j];
                }
            }
        }
    };

    if ((long long)blockIdx.x >= nsweeps) return;
    load_spectrum(blockIdx.x);
    __syncthreads();                                        // twiddle tables are ready
    long long sweep = blockIdx.x;
    for (; sweep + gridDim.x < nsweeps; sweep += gridDim.x) stage(sweep, std::true_type{}, sweep + gridDim.x);
    stage(sweep, std::false_type{}, 0);
}

}  // namespace tfno
