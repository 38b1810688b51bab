// 2-D spectral convolution for gfx950 as three kernels whose only HBM intermediates are the TRUNCATED
// spectra (K x K per image instead of the K x N strips of the 2-D pipeline in Sec. 3.2 / 3.3):
//
//   k_fwd2d   one workgroup per input image x[b, c]: truncated, output-pruned 2-D forward transform
//             -> Xh[b, c, k1, k2], k1, k2 < K                           (reads N*N, writes K*K)
//   k_cgemm_modes   Yh[b, o, m] = sum_c Xh[b, c, m] * W[c, o] / N^2 over the K*K retained modes; one W for
//             all modes (Sec. 3.1), FP32 MFMA
//   k_inv2d   one workgroup per output image: zero-padded, input-pruned 2-D inverse -> y[b, o]
//
// Both transforms are separable (Sec. 3.3).  With S = N/32 the pruned first-axis transform is written as
//   X[k1] = sum_{r<S} w_N^(r k1) * F_r[k1 mod 32],   F_r = 32-point DFT of the rows n1 = r + S s, s < 32,
// so an image is processed in S passes of 32 rows: the last-axis transform of the 32 rows (truncated to K
// bins, Sec. 3.3) goes into a 32 x K LDS tile, the 32-point column transform of that tile is accumulated
// into registers with the pass twiddle, and the full N x K strip never exists anywhere.  The inverse runs
// the transposed network: spectrum in registers, per pass a twiddled 32-point inverse column transform
// into the tile and zero-padded inverse row transforms of its 32 rows.
//
// Row transform (N = 16 * LPR): LPR lanes per row, lane p holds x[p + LPR j], j < 16 (coalesced loads),
// 16-point DFT in registers, twiddle w_N^(p k_lo), transpose through a wave-private XOR-swizzled LDS patch,
// then the LPR-point DFT pruned to the K/16 retained outputs of each column k_lo (bins k_lo + 16 k_hi).
// Column transform: 4 adjacent lanes per tile column, 8-point DFT in registers, 4-point DFT across the quad
// with DPP.  All LDS accesses of the handoffs hit distinct banks per 16 lanes (the counterpart of the two
// swizzles of Sec. 4.1 / 4.2 for 8-byte accesses on wave64).
#pragma once
#include "common.h"
#include "fft_regs.h"
#include "fused1d_kernel.h"   // wave_sync, floatx16

namespace tfno {

template <int N, int K>
struct Cfg2d {
    static constexpr int NT = 256;
    static constexpr int LPR = N / 16;                          // lanes per row
    static constexpr int RPS = (NT / LPR) < 32 ? NT / LPR : 32; // rows per sweep of the workgroup
    static constexpr int ACTIVE = RPS * LPR;                    // threads that take part in the row stage
    static constexpr int RP = 32;                               // rows per pass
    static constexpr int S = N / RP;                            // passes
    static constexpr int SWEEPS = RP / RPS;
    static constexpr int NSWEEP = S * SWEEPS;
    static constexpr int KH = K / 16;                           // retained outputs per column k_lo
    static constexpr int CPL = 16 / LPR;                        // columns k_lo per lane after the transpose
    static constexpr int GS = N + (LPR < 16 ? LPR : 0);         // patch stride between the rows of a sweep
    static constexpr int TS = K + 4;                            // tile row stride (== 4 mod 16)
    static constexpr int MREP = (K + 31) / 32;                  // k1 = k' + 32 m
    static constexpr int NACC = 8 * MREP;
    static constexpr size_t LDS_BYTES = sizeof(c64) * ((size_t)RPS * GS + (size_t)RP * TS + 2 * N);
    static_assert(N == 64 || N == 128 || N == 256, "N in {64, 128, 256}");
    static_assert(K == 16 || K == 32 || K == 64, "K in {16, 32, 64}");
    static_assert(K <= N && KH <= LPR && LPR % KH == 0, "K must divide N");
    static_assert(NSWEEP % 2 == 0, "the sweep loop is unrolled by two");
    static_assert(LDS_BYTES <= 64 * 1024, "static LDS limit");
};

// value of lane (quad position PERM[q]) of the same quad
template <int CTRL>
__device__ __forceinline__ float quad_perm(float v)
{
    return __int_as_float(__builtin_amdgcn_mov_dpp(__float_as_int(v), CTRL, 0xf, 0xf, true));
}
constexpr int QP_XOR1 = 0xB1;   // [1, 0, 3, 2]
constexpr int QP_XOR2 = 0x4E;   // [2, 3, 0, 1]

// 4-point DFT across the four lanes of a quad, forward sign: lane q4 holds input q4 on entry and output
// kb = bitrev2(q4) on exit.
__device__ __forceinline__ c64 quad_dft4_fwd(c64 g, int q4)
{
    const float s2 = (q4 & 2) ? -1.f : 1.f, s1 = (q4 & 1) ? -1.f : 1.f;
    c64 t = make_float2(fmaf(s2, g.x, quad_perm<QP_XOR2>(g.x)), fmaf(s2, g.y, quad_perm<QP_XOR2>(g.y)));
    if (q4 == 3) t = make_float2(t.y, -t.x);                    // * (-i)
    return make_float2(fmaf(s1, t.x, quad_perm<QP_XOR1>(t.x)), fmaf(s1, t.y, quad_perm<QP_XOR1>(t.y)));
}
// transposed network, inverse sign: lane q4 holds input kb = bitrev2(q4) on entry and output q4 on exit.
__device__ __forceinline__ c64 quad_dft4_inv(c64 g, int q4)
{
    const float s2 = (q4 & 2) ? -1.f : 1.f, s1 = (q4 & 1) ? -1.f : 1.f;
    c64 t = make_float2(fmaf(s1, g.x, quad_perm<QP_XOR1>(g.x)), fmaf(s1, g.y, quad_perm<QP_XOR1>(g.y)));
    if (q4 == 3) t = make_float2(-t.y, t.x);                    // * (+i)
    return make_float2(fmaf(s2, t.x, quad_perm<QP_XOR2>(t.x)), fmaf(s2, t.y, quad_perm<QP_XOR2>(t.y)));
}

struct Lds2d {
    c64 *scr;    // [RPS][GS]   transpose patches, one per row of a sweep
    c64 *tile;   // [32][TS]    truncated rows of one pass
    c64 *tw;     // [16][LPR]   w_N^(p k_lo)
    c64 *twn;    // [N]         w_N^t
};

template <int N, int K>
__device__ __forceinline__ Lds2d lds_setup(unsigned char *raw, int tid)
{
    using C = Cfg2d<N, K>;
    Lds2d l;
    l.scr = reinterpret_cast<c64 *>(raw);
    l.tile = l.scr + C::RPS * C::GS;
    l.tw = l.tile + C::RP * C::TS;
    l.twn = l.tw + N;
    for (int i = tid; i < N; i += C::NT) {
        l.tw[i] = cis2pi(-(float)((i / C::LPR) * (i % C::LPR)), (float)N);
        l.twn[i] = cis2pi(-(float)i, (float)N);
    }
    return l;
}

// ------------------------------------------------------------------------------------------------ forward
template <int N, int K>
__global__ void __launch_bounds__(256)
k_fwd2d(const c64 *__restrict__ x, c64 *__restrict__ Xh)
{
    using C = Cfg2d<N, K>;
    constexpr int LPR = C::LPR, RPS = C::RPS, S = C::S, SWEEPS = C::SWEEPS, KH = C::KH, CPL = C::CPL;
    constexpr int GS = C::GS, TS = C::TS, MREP = C::MREP;
    __shared__ __align__(16) unsigned char raw[C::LDS_BYTES];
    const int tid = threadIdx.x;
    const Lds2d L = lds_setup<N, K>(raw, tid);

    const c64 *__restrict__ img = x + (long long)blockIdx.x * N * N;
    // row-stage identity
    const bool row_on = tid < C::ACTIVE;
    const int g = tid / LPR, p = tid % LPR;
    c64 *scr = L.scr + g * GS;
    // column-stage identity
    const int k2 = tid >> 2, q4 = tid & 3, kb = ((q4 & 1) << 1) | (q4 >> 1);
    const bool col_on = k2 < K;

    c64 acc[C::NACC];
#pragma unroll
    for (int i = 0; i < C::NACC; ++i) acc[i] = make_float2(0.f, 0.f);

    auto load_rows = [&](c64 *v, int sweep) __attribute__((always_inline)) {
        const int r = sweep / SWEEPS, s = (sweep % SWEEPS) * RPS + g;
        const c64 *src = img + (long long)(r + S * s) * N + p;
        if (row_on) {
#pragma unroll
            for (int j = 0; j < 16; ++j) v[j] = src[LPR * j];
        }
    };
    auto row_stage = [&](const c64 *v, int sweep) __attribute__((always_inline)) {
        if (!row_on) return;
        const int s = (sweep % SWEEPS) * RPS + g;
        c64 z[16];
        RegFFT<16, -1, 1>::run(v, z);
        wave_sync();                                        // the previous sweep's patch reads are done
#pragma unroll
        for (int kl = 0; kl < 16; ++kl) {
            const c64 zt = kl == 0 ? z[0] : cmul(z[kl], L.tw[kl * LPR + p]);
            scr[kl * LPR + (p ^ (kl % LPR))] = zt;
        }
        wave_sync();
#pragma unroll
        for (int i = 0; i < CPL; ++i) {
            const int kl = p + LPR * i;                     // kl % LPR == p
            c64 xo[KH];
            dft_prune_out<LPR, KH, -1>([&](auto ppc) __attribute__((always_inline)) {
                constexpr int pp = decltype(ppc)::value;
                return scr[kl * LPR + (pp ^ p)];
            }, xo);
#pragma unroll
            for (int kh = 0; kh < KH; ++kh) L.tile[s * TS + kl + 16 * kh] = xo[kh];
        }
    };
    auto col_stage = [&](int r) __attribute__((always_inline)) {
        if (!col_on) return;
        c64 u[8], G[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) u[j] = L.tile[(q4 + 4 * j) * TS + k2];
        RegFFT<8, -1, 1>::run(u, G);
#pragma unroll
        for (int ka = 0; ka < 8; ++ka) {
            c64 t = ka == 0 ? G[0] : cmul(G[ka], L.twn[(q4 * ka) * (N / 32)]);
            t = quad_dft4_fwd(t, q4);                       // F_r[ka + 8 kb]
#pragma unroll
            for (int m = 0; m < MREP; ++m) {
                const int k1 = ka + 8 * kb + 32 * m;
                acc[m * 8 + ka] = cmac(acc[m * 8 + ka], t, L.twn[(r * k1) & (N - 1)]);
            }
        }
    };

    c64 va[16], vb[16];
    load_rows(va, 0);
    __syncthreads();                                        // twiddle tables are ready
    for (int sweep = 0; sweep < C::NSWEEP; sweep += 2) {
        load_rows(vb, sweep + 1);
        row_stage(va, sweep);
        if constexpr (SWEEPS == 1) {
            __syncthreads();
            col_stage(sweep);
            __syncthreads();
        }
        if (sweep + 2 < C::NSWEEP) load_rows(va, sweep + 2);
        row_stage(vb, sweep + 1);
        __syncthreads();
        col_stage((sweep + 1) / SWEEPS);
        __syncthreads();
    }

    if (col_on) {
        c64 *dst = Xh + (long long)blockIdx.x * K * K + k2;
#pragma unroll
        for (int m = 0; m < MREP; ++m)
#pragma unroll
            for (int ka = 0; ka < 8; ++ka) {
                const int k1 = ka + 8 * kb + 32 * m;
                if (k1 < K) dst[k1 * K] = acc[m * 8 + ka];
            }
    }
}

// ------------------------------------------------------------------------------------------------ inverse
template <int N, int K>
__global__ void __launch_bounds__(256)
k_inv2d(const c64 *__restrict__ Yh, c64 *__restrict__ y)
{
    using C = Cfg2d<N, K>;
    constexpr int LPR = C::LPR, RPS = C::RPS, S = C::S, SWEEPS = C::SWEEPS, KH = C::KH, CPL = C::CPL;
    constexpr int GS = C::GS, TS = C::TS, MREP = C::MREP;
    __shared__ __align__(16) unsigned char raw[C::LDS_BYTES];
    const int tid = threadIdx.x;
    const Lds2d L = lds_setup<N, K>(raw, tid);

    c64 *__restrict__ img = y + (long long)blockIdx.x * N * N;
    const bool row_on = tid < C::ACTIVE;
    const int g = tid / LPR, p = tid % LPR;
    c64 *scr = L.scr + g * GS;
    const int k2 = tid >> 2, q4 = tid & 3, kb = ((q4 & 1) << 1) | (q4 >> 1);
    const bool col_on = k2 < K;

    // the retained spectrum of this image, K*K/256 (or fewer) bins per thread, for all passes
    c64 Y[C::NACC];
    {
        const c64 *src = Yh + (long long)blockIdx.x * K * K + (col_on ? k2 : 0);
#pragma unroll
        for (int m = 0; m < MREP; ++m)
#pragma unroll
            for (int ka = 0; ka < 8; ++ka) {
                const int k1 = ka + 8 * kb + 32 * m;
                const bool ok = col_on && k1 < K;
                c64 v = src[ok ? k1 * K : 0];
                Y[m * 8 + ka] = ok ? v : make_float2(0.f, 0.f);
            }
    }

    auto col_stage = [&](int r) __attribute__((always_inline)) {
        if (!col_on) return;
        c64 G[8], f[8];
#pragma unroll
        for (int ka = 0; ka < 8; ++ka) {
            c64 t = make_float2(0.f, 0.f);
#pragma unroll
            for (int m = 0; m < MREP; ++m) {
                const int k1 = ka + 8 * kb + 32 * m;
                const c64 w = L.twn[(r * k1) & (N - 1)];
                t = cmac(t, Y[m * 8 + ka], make_float2(w.x, -w.y));
            }
            t = quad_dft4_inv(t, q4);
            if (ka != 0) {
                const c64 w = L.twn[(q4 * ka) * (N / 32)];
                t = cmul(t, make_float2(w.x, -w.y));
            }
            G[ka] = t;
        }
        RegFFT<8, +1, 1>::run(G, f);
#pragma unroll
        for (int j = 0; j < 8; ++j) L.tile[(q4 + 4 * j) * TS + k2] = f[j];
    };
    // zero-padded inverse row transforms of sweep `sweep`, results left in out[]
    auto row_stage = [&](c64 *out, int sweep) __attribute__((always_inline)) {
        if (!row_on) return;
        const int s = (sweep % SWEEPS) * RPS + g;
        wave_sync();                                        // the previous sweep's patch reads are done
#pragma unroll
        for (int i = 0; i < CPL; ++i) {
            const int kl = p + LPR * i;
            c64 yin[KH];
#pragma unroll
            for (int kh = 0; kh < KH; ++kh) yin[kh] = L.tile[s * TS + kl + 16 * kh];
            dft_prune_in<LPR, KH, +1>(yin, [&](auto ppc, c64 val) __attribute__((always_inline)) {
                constexpr int pp = decltype(ppc)::value;
                scr[kl * LPR + (pp ^ p)] = val;
            });
        }
        wave_sync();
        c64 z[16];
#pragma unroll
        for (int kl = 0; kl < 16; ++kl) {
            c64 t = scr[kl * LPR + (p ^ (kl % LPR))];
            if (kl != 0) {
                const c64 w = L.tw[kl * LPR + p];
                t = cmul(t, make_float2(w.x, -w.y));
            }
            z[kl] = t;
        }
        RegFFT<16, +1, 1>::run(z, out);
    };
    auto store_rows = [&](const c64 *out, int sweep) __attribute__((always_inline)) {
        if (!row_on) return;
        const int r = sweep / SWEEPS, s = (sweep % SWEEPS) * RPS + g;
        c64 *dst = img + (long long)(r + S * s) * N + p;
#pragma unroll
        for (int j = 0; j < 16; ++j) dst[LPR * j] = out[j];
    };

    __syncthreads();                                        // twiddle tables are ready
    for (int r = 0; r < S; ++r) {
        col_stage(r);
        __syncthreads();
#pragma unroll
        for (int w = 0; w < SWEEPS; ++w) {
            c64 out[16];
            row_stage(out, r * SWEEPS + w);
            store_rows(out, r * SWEEPS + w);
        }
        __syncthreads();
    }
}

// ------------------------------------------------------------------------------------------------ CGEMM
// Yh[b, o, m] = sum_c Xh[b, c, m] * (scale * W[c, o]),  m < M (M a multiple of 64).
// One wave per (b, 32 outputs, 64 modes); v_mfma_f32_32x32x2_f32 with the two k-slots of an instruction
// carrying (re, im) of one channel: real part with A = (W.re, -W.im), imaginary part with A = (W.im, W.re).
__global__ void __launch_bounds__(256)
k_cgemm_modes(const c64 *__restrict__ Xh, const c64 *__restrict__ W, c64 *__restrict__ Yh,
              int C_in, int C_out, int M, int mblocks, float scale)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const long long b = blockIdx.x / mblocks;
    const int m0 = ((int)(blockIdx.x % mblocks) * 4 + wave) * 64;
    if (m0 >= M) return;
    const int col = lane & 31;
    const bool hi = lane >= 32;
    const int o0 = blockIdx.y * 32, o_lane = o0 + col;
    const bool o_ok = o_lane < C_out;
    const c64 *__restrict__ Xb = Xh + b * C_in * (long long)M + m0 + col;
    const c64 *__restrict__ Wl = W + (o_ok ? o_lane : 0);

    floatx16 acc_re[2], acc_im[2];
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) { acc_re[t][r] = 0.f; acc_im[t][r] = 0.f; }

    auto step = [&](int c) __attribute__((always_inline)) {
        c64 wv = Wl[(long long)c * C_out];
        if (!o_ok) wv = make_float2(0.f, 0.f);
        const float a_re = (hi ? -wv.y : wv.x) * scale, a_im = (hi ? wv.x : wv.y) * scale;
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            const c64 xv = Xb[(long long)c * M + 32 * t];
            const float bx = hi ? xv.y : xv.x;
            acc_re[t] = __builtin_amdgcn_mfma_f32_32x32x2f32(a_re, bx, acc_re[t], 0, 0, 0);
            acc_im[t] = __builtin_amdgcn_mfma_f32_32x32x2f32(a_im, bx, acc_im[t], 0, 0, 0);
        }
    };
    int c = 0;
    for (; c + 4 <= C_in; c += 4) {
#pragma unroll
        for (int u = 0; u < 4; ++u) step(c + u);
    }
    for (; c < C_in; ++c) step(c);

    c64 *__restrict__ Yb = Yh + b * C_out * (long long)M + m0 + col;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        const int o = o0 + 8 * (r / 4) + 4 * (hi ? 1 : 0) + (r % 4);
        if (o < C_out) {
#pragma unroll
            for (int t = 0; t < 2; ++t)
                Yb[(long long)o * M + 32 * t] = make_float2(acc_re[t][r], acc_im[t][r]);
        }
    }
}

}  // namespace tfno
