// 2-D spectral convolution for gfx950 as three kernels whose only HBM intermediates are the TRUNCATED
// spectra (K x K per image instead of the K x N strips of the 2-D pipeline in Sec. 3.2 / 3.3):
//
//   k_fwd2d   one workgroup per input image x[b, c]: truncated, output-pruned 2-D forward transform
//             -> Xh[b, c, k1, k2], k1, k2 < K                           (reads N*N, writes K*K)
//             stored mode-tile major, [b][m / 128][c][m % 128] with m = k1 K + k2, so that the CGEMM streams
//             one contiguous [C, 128] block per workgroup
//   k_cgemm_modes   Yh[b, o, m] = sum_c Xh[b, c, m] * W[c, o] / N^2 over the K*K retained modes; one W for
//             all modes (Sec. 3.1), FP32 MFMA
//   k_inv2d   one workgroup per output image: zero-padded, input-pruned 2-D inverse -> y[b, o]
//
// Both transforms are separable (Sec. 3.3).  With RP rows per pass (16 or 32) and S = N/RP the pruned first-axis
// transform is written as
//   X[k1] = sum_{r<S} w_N^(r k1) * F_r[k1 mod RP],   F_r = RP-point DFT of the rows n1 = r + S s, s < RP,
// so an image is processed in S passes of RP rows: the last-axis transform of these rows (truncated to K
// bins, Sec. 3.3) goes into an RP x K LDS tile, the RP-point column transform of that tile is accumulated
// into registers with the pass twiddle, and the full N x K strip never exists anywhere.  The inverse runs
// the transposed network: spectrum in registers, per pass a twiddled RP-point inverse column transform
// into the tile and zero-padded inverse row transforms of its rows.  The passes of an image can run in any
// order; workgroups start at different passes (see r_rot) because the rows of one pass map to few L2 channels.
//
// Row transform (N = 16 * LPR): LPR lanes per row, lane p holds x[p + LPR j], j < 16 (coalesced loads),
// 16-point DFT in registers, twiddle w_N^(p k_lo), transpose through a wave-private XOR-swizzled LDS patch,
// then the LPR-point DFT pruned to the K/16 retained outputs of each column k_lo (bins k_lo + 16 k_hi).
// Column transform: 4 adjacent lanes per tile column, RP/4-point DFT in registers, 4-point DFT across the quad
// with DPP.  All LDS accesses of the handoffs hit distinct banks per 16 lanes (the counterpart of the two
// swizzles of Sec. 4.1 / 4.2 for 8-byte accesses on wave64; checked with an LDS microbenchmark).
#pragma once
#include "common.h"
#include "fft_regs.h"
#include "fused1d_kernel.h"   // wave_sync, floatx16
#include "bf16x3.h"

namespace tfno {

// RP16: 16-row passes with two tile buffers (one barrier per pass) instead of 32-row passes with one buffer
template <int N, int K, bool RP16>
struct Cfg2d {
    static constexpr int NT = 256;
    static constexpr int LPR = N / 16;                          // lanes per row
    static constexpr int RP = RP16 ? 16 : 32;                   // rows per pass
    static constexpr int RPS = (NT / LPR) < RP ? NT / LPR : RP; // rows per sweep of the workgroup
    static constexpr int ACTIVE = RPS * LPR;                    // threads that take part in the row stage
    static constexpr int S = N / RP;                            // passes
    static constexpr int SWEEPS = RP / RPS;
    static constexpr int NSWEEP = S * SWEEPS;
    static constexpr int KH = K / 16;                           // retained outputs per column k_lo
    static constexpr int CPL = 16 / LPR;                        // columns k_lo per lane after the transpose
    static constexpr int GS = N + (LPR < 16 ? LPR : 0);         // patch stride between the rows of a sweep
    static constexpr int TS = K + 4;                            // tile row stride (== 4 mod 16)
    static constexpr int RPL = RP / 4;                          // tile rows per lane in the column stage
    static constexpr int MREP = (K + RP - 1) / RP;              // k1 = k' + RP m
    static constexpr int NACC = RPL * MREP;
    static constexpr int NBUF = RP == 16 ? 2 : 1;               // tile buffers (2: one barrier per pass)
    static constexpr size_t LDS_BYTES = sizeof(c64) * ((size_t)RPS * GS + (size_t)NBUF * RP * TS + 2 * N);
    static_assert(N == 64 || N == 128 || N == 256, "N in {64, 128, 256}");
    static_assert(K == 16 || K == 32 || K == 64, "K in {16, 32, 64}");
    static_assert(K <= N && KH <= LPR && LPR % KH == 0, "K must divide N");
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
    c64 *tile;   // [NBUF][RP][TS]  truncated rows of one pass
    c64 *tw;     // [16][LPR]   w_N^(p k_lo)
    c64 *twn;    // [N]         w_N^t
};

template <int N, int K, bool RP16>
__device__ __forceinline__ Lds2d lds_setup(unsigned char *raw, int tid)
{
    using C = Cfg2d<N, K, RP16>;
    Lds2d l;
    l.scr = reinterpret_cast<c64 *>(raw);
    l.tile = l.scr + C::RPS * C::GS;
    l.tw = l.tile + C::NBUF * C::RP * C::TS;
    l.twn = l.tw + N;
    for (int i = tid; i < N; i += C::NT) {
        l.tw[i] = cis2pi(-(float)((i / C::LPR) * (i % C::LPR)), (float)N);
        l.twn[i] = cis2pi(-(float)i, (float)N);
    }
    return l;
}

// ------------------------------------------------------------------------------------------------ forward
// element offset of (channel c, mode m) of batch element b in a mode-tile-major spectrum buffer
__device__ __forceinline__ long long spec_index(long long b, int c, int C, int m, int M)
{
    return ((b * (M / 128) + m / 128) * C + c) * 128 + m % 128;
}

template <int N, int K>
__global__ void __launch_bounds__(256, 3)
k_fwd2d(const c64 *__restrict__ x, c64 *__restrict__ Xh, int C_in)
{
    using C = Cfg2d<N, K, N == 256>;
    constexpr int LPR = C::LPR, RPS = C::RPS, S = C::S, SWEEPS = C::SWEEPS, KH = C::KH, CPL = C::CPL;
    constexpr int GS = C::GS, TS = C::TS, MREP = C::MREP, RP = C::RP, RPL = C::RPL, NBUF = C::NBUF;
    __shared__ __align__(16) unsigned char raw[C::LDS_BYTES];
    const int tid = threadIdx.x;
    const Lds2d L = lds_setup<N, K, C::RP == 16>(raw, tid);

    // (workgroup id = image: giving each XCD a contiguous range of images, which helps the 1-D kernels, measured
    // 5-9 % slower here)
    const unsigned image = blockIdx.x;
    const c64 *__restrict__ img = x + (long long)image * N * N;
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

    // Passes may run in any order (their contributions are summed).  The rows of one pass are N*S*8 bytes apart
    // in memory, which maps them to a fraction of the L2 channels; workgroups that share an XCD (every 8th
    // workgroup id) therefore start at different passes so that together they use all channels.
    const int r_rot = (int)(blockIdx.x >> 3);
    auto load_rows = [&](c64 *v, int sweep) __attribute__((always_inline)) {
        const int r = (sweep / SWEEPS + r_rot) & (S - 1), s = (sweep % SWEEPS) * RPS + g;
        const c64 *src = img + (long long)(r + S * s) * N + p;
        if (row_on) {
#pragma unroll
            for (int j = 0; j < 16; ++j) v[j] = load_nt(src + LPR * j);
        }
    };
    // Row transforms of the sweep held in v.  The first butterfly level consumes v, so the loads of the next
    // sweep are issued right after it and stay in flight while the rest of this sweep is computed.
    auto row_stage = [&](c64 *v, int sweep, auto refill) __attribute__((always_inline)) {
        constexpr bool REFILL = decltype(refill)::value;    // false only for the last sweep of the image
        if (!row_on) return;
        const int s = (sweep % SWEEPS) * RPS + g;
        c64 *tile = L.tile + ((sweep / SWEEPS) % NBUF) * (RP * TS);
        c64 z[16];
        {
            c64 ea[8], eb[8], za[8], zo[8];
            dif_first_level<16, -1>(v, ea, eb);
            __builtin_amdgcn_sched_barrier(0);
            if constexpr (REFILL) load_rows(v, sweep + 1);
            __builtin_amdgcn_sched_barrier(0);
            RegFFT<8, -1, 1>::run(ea, za);
            RegFFT<8, -1, 1>::run(eb, zo);
#pragma unroll
            for (int k = 0; k < 8; ++k) { z[2 * k] = za[k]; z[2 * k + 1] = zo[k]; }
        }
        // the twiddles are read eight at a time before their first use: left alone, the compiler reads, waits and
        // multiplies one at a time (15 exposed LDS round trips per sweep); all 15 at once do not fit the registers
        wave_sync();                                        // the previous sweep's patch reads are done
#pragma unroll
        for (int half = 0; half < 2; ++half) {
            c64 tw[8];
#pragma unroll
            for (int j = 0; j < 8; ++j)
                if (half + j != 0) tw[j] = L.tw[(8 * half + j) * LPR + p];
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const int kl = 8 * half + j;
                const c64 zt = kl == 0 ? z[0] : cmul(z[kl], tw[j]);
                scr[kl * LPR + (p ^ (kl % LPR))] = zt;
            }
            __builtin_amdgcn_sched_barrier(0);
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
            for (int kh = 0; kh < KH; ++kh) tile[s * TS + kl + 16 * kh] = xo[kh];
        }
    };
    // RP-point transform of the tile columns of pass `i` (rows r + S s), accumulated with the pass twiddle
    auto col_stage = [&](int i) __attribute__((always_inline)) {
        if (!col_on) return;
        const int r = (i + r_rot) & (S - 1);
        const c64 *tile = L.tile + (i % NBUF) * (RP * TS);
        c64 u[RPL], G[RPL];
#pragma unroll
        for (int j = 0; j < RPL; ++j) u[j] = tile[(q4 + 4 * j) * TS + k2];
        RegFFT<RPL, -1, 1>::run(u, G);
#pragma unroll
        for (int ka = 0; ka < RPL; ++ka) {
            c64 t = ka == 0 ? G[0] : cmul(G[ka], L.twn[(q4 * ka) * (N / RP)]);
            t = quad_dft4_fwd(t, q4);                       // F_r[ka + RPL kb]
#pragma unroll
            for (int m = 0; m < MREP; ++m) {
                const int k1 = ka + RPL * kb + RP * m;
                acc[m * RPL + ka] = cmac(acc[m * RPL + ka], t, L.twn[(r * k1) & (N - 1)]);
            }
        }
    };

    c64 v[16];
    load_rows(v, 0);
    __syncthreads();                                        // twiddle tables are ready
    // the last pass is peeled off so that every other sweep refills v unconditionally
    for (int i = 0; i < S - 1; ++i) {
#pragma unroll
        for (int w = 0; w < SWEEPS; ++w) row_stage(v, i * SWEEPS + w, std::true_type{});
        __syncthreads();
        col_stage(i);
        if constexpr (NBUF == 1) __syncthreads();           // with two tile buffers the next pass writes the other one
    }
#pragma unroll
    for (int w = 0; w < SWEEPS; ++w) {
        if (w + 1 < SWEEPS) row_stage(v, (S - 1) * SWEEPS + w, std::true_type{});
        else row_stage(v, (S - 1) * SWEEPS + w, std::false_type{});
    }
    __syncthreads();
    col_stage(S - 1);

    if (col_on) {
        const long long b = image / C_in;
        const int c = (int)(image % C_in);
#pragma unroll
        for (int m = 0; m < MREP; ++m)
#pragma unroll
            for (int ka = 0; ka < RPL; ++ka) {
                const int k1 = ka + RPL * kb + RP * m;
                if (k1 < K) Xh[spec_index(b, c, C_in, k1 * K + k2, K * K)] = acc[m * RPL + ka];
            }
    }
}

// ------------------------------------------------------------------------------------------------ inverse
template <int N, int K>
__global__ void __launch_bounds__(256, 3)
k_inv2d(const c64 *__restrict__ Yh, c64 *__restrict__ y, int C_out)
{
    using C = Cfg2d<N, K, false>;
    constexpr int LPR = C::LPR, RPS = C::RPS, S = C::S, SWEEPS = C::SWEEPS, KH = C::KH, CPL = C::CPL;
    constexpr int GS = C::GS, TS = C::TS, MREP = C::MREP, RP = C::RP, RPL = C::RPL, NBUF = C::NBUF;
    __shared__ __align__(16) unsigned char raw[C::LDS_BYTES];
    const int tid = threadIdx.x;
    const Lds2d L = lds_setup<N, K, C::RP == 16>(raw, tid);

    const unsigned image = blockIdx.x;
    c64 *__restrict__ img = y + (long long)image * N * N;
    const bool row_on = tid < C::ACTIVE;
    const int g = tid / LPR, p = tid % LPR;
    c64 *scr = L.scr + g * GS;
    const int k2 = tid >> 2, q4 = tid & 3, kb = ((q4 & 1) << 1) | (q4 >> 1);
    const bool col_on = k2 < K;

    // the retained spectrum of this image, K*K/256 (or fewer) bins per thread, for all passes
    c64 Y[C::NACC];
    {
        const long long b = image / C_out;
        const int o = (int)(image % C_out);
#pragma unroll
        for (int m = 0; m < MREP; ++m)
#pragma unroll
            for (int ka = 0; ka < RPL; ++ka) {
                const int k1 = ka + RPL * kb + RP * m;
                const bool ok = col_on && k1 < K;
                c64 v = Yh[spec_index(b, o, C_out, ok ? k1 * K + k2 : 0, K * K)];
                Y[m * RPL + ka] = ok ? v : make_float2(0.f, 0.f);
            }
    }

    const int r_rot = (int)(blockIdx.x >> 3);               // pass order rotated as in the forward kernel
    // twiddled RP-point inverse column transform of pass `i` (rows r + S s) into the tile
    auto col_stage = [&](int i) __attribute__((always_inline)) {
        if (!col_on) return;
        const int r = (i + r_rot) & (S - 1);
        c64 *tile = L.tile + (i % NBUF) * (RP * TS);
        c64 G[RPL], f[RPL];
#pragma unroll
        for (int ka = 0; ka < RPL; ++ka) {
            c64 t = make_float2(0.f, 0.f);
#pragma unroll
            for (int m = 0; m < MREP; ++m) {
                const int k1 = ka + RPL * kb + RP * m;
                const c64 w = L.twn[(r * k1) & (N - 1)];
                t = cmac(t, Y[m * RPL + ka], make_float2(w.x, -w.y));
            }
            t = quad_dft4_inv(t, q4);
            if (ka != 0) {
                const c64 w = L.twn[(q4 * ka) * (N / RP)];
                t = cmul(t, make_float2(w.x, -w.y));
            }
            G[ka] = t;
        }
        RegFFT<RPL, +1, 1>::run(G, f);
#pragma unroll
        for (int j = 0; j < RPL; ++j) tile[(q4 + 4 * j) * TS + k2] = f[j];
    };
    // zero-padded inverse row transforms of sweep `sweep`, results left in out[]
    auto row_stage = [&](c64 *out, int sweep) __attribute__((always_inline)) {
        if (!row_on) return;
        const int s = (sweep % SWEEPS) * RPS + g;
        const c64 *tile = L.tile + ((sweep / SWEEPS) % NBUF) * (RP * TS);
        wave_sync();                                        // the previous sweep's patch reads are done
#pragma unroll
        for (int i = 0; i < CPL; ++i) {
            const int kl = p + LPR * i;
            c64 yin[KH];
#pragma unroll
            for (int kh = 0; kh < KH; ++kh) yin[kh] = tile[s * TS + kl + 16 * kh];
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
        const int r = (sweep / SWEEPS + r_rot) & (S - 1), s = (sweep % SWEEPS) * RPS + g;
        c64 *dst = img + (long long)(r + S * s) * N + p;
#pragma unroll
        for (int j = 0; j < 16; ++j) store_nt(dst + LPR * j, out[j]);
    };

    __syncthreads();                                        // twiddle tables are ready
    for (int i = 0; i < S; ++i) {
        col_stage(i);
        __syncthreads();
#pragma unroll
        for (int w = 0; w < SWEEPS; ++w) {
            c64 out[16];
            row_stage(out, i * SWEEPS + w);
            store_rows(out, i * SWEEPS + w);
        }
        if constexpr (NBUF == 1) __syncthreads();           // with two tile buffers the next pass writes the other one
    }
}

// ------------------------------------------------------------------------------------------------ CGEMM
// Yh[b, o, m] = sum_c Xh[b, c, m] * (scale * W[c, o]),  m < M (M a multiple of 128), both spectra mode-tile
// major, so a tile of 128 modes of one batch element is a contiguous [C, 128] block.  A workgroup walks
// `tiles_per_wg` consecutive tiles for 64 outputs, one wave per 32 modes: every spectrum element is read once
// per 64 outputs, the stores of one tile drain under the MFMAs of the next, and the spectrum chunks are
// double buffered in registers across tile boundaries.  W (scaled) is staged in LDS 64 channels at a time.
// v_mfma_f32_32x32x2_f32 with the two k-slots of an instruction carrying (re, im) of one channel: real part
// with A = (W.re, -W.im), imaginary part with A = (W.im, W.re).
__global__ void __launch_bounds__(256, 2)
k_cgemm_modes_f32(const c64 *__restrict__ Xh, const c64 *__restrict__ W, c64 *__restrict__ Yh,
                  int C_in, int C_out, float scale, long long num_tiles, int tiles_per_wg)
{
    constexpr int U = 8;                                    // channels per register chunk
    __shared__ c64 Wl[64 * 64];                             // [channel in block][output in slab pair]
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int col = lane & 31;
    const bool hi = lane >= 32;
    const int o0 = blockIdx.y * 64;
    const long long tile0 = (long long)blockIdx.x * tiles_per_wg;
    const int ntile = (int)(num_tiles - tile0 < tiles_per_wg ? num_tiles - tile0 : tiles_per_wg);
    const int c_pad = (C_in + 2 * U - 1) / (2 * U) * (2 * U);
    const bool one_block = C_in <= 64;

    floatx16 acc_re[2], acc_im[2];

    // position of the next chunk to load: (tile, channel); channels past C_in are read from a valid address
    // and meet zero weights, tiles past the end are not loaded
    int nt = 0, nc = 0;
    auto load_next = [&](c64 *xv) __attribute__((always_inline)) {
        if (nt < ntile) {
            const c64 *src = Xh + (tile0 + nt) * C_in * 128 + 32 * wave + col;
#pragma unroll
            for (int u = 0; u < U; ++u) xv[u] = src[(nc + u < C_in ? nc + u : 0) * 128];
        }
        nc += U;
        if (nc >= c_pad) { nc = 0; ++nt; }
    };
    auto mac_chunk = [&](const c64 *xv, int cl) __attribute__((always_inline)) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const c64 w0 = Wl[(cl + u) * 64 + col], w1 = Wl[(cl + u) * 64 + 32 + col];
            const float bx = hi ? xv[u].y : xv[u].x;
            acc_re[0] = __builtin_amdgcn_mfma_f32_32x32x2f32(hi ? -w0.y : w0.x, bx, acc_re[0], 0, 0, 0);
            acc_im[0] = __builtin_amdgcn_mfma_f32_32x32x2f32(hi ? w0.x : w0.y, bx, acc_im[0], 0, 0, 0);
            acc_re[1] = __builtin_amdgcn_mfma_f32_32x32x2f32(hi ? -w1.y : w1.x, bx, acc_re[1], 0, 0, 0);
            acc_im[1] = __builtin_amdgcn_mfma_f32_32x32x2f32(hi ? w1.x : w1.y, bx, acc_im[1], 0, 0, 0);
        }
    };

    c64 xa[U], xb[U];
    load_next(xa);
    for (int t = 0; t < ntile; ++t) {
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r) { acc_re[i][r] = 0.f; acc_im[i][r] = 0.f; }
        for (int cb = 0; cb < C_in; cb += 64) {
            if (!one_block || t == 0) {
                __syncthreads();                            // the previous block of W has been consumed
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const int idx = i * 256 + tid, c = cb + idx / 64, o = o0 + idx % 64;
                    const bool ok = c < C_in && o < C_out;
                    const c64 w = W[ok ? (long long)c * C_out + o : 0];
                    Wl[idx] = ok ? make_float2(w.x * scale, w.y * scale) : make_float2(0.f, 0.f);
                }
                __syncthreads();
            }
            const int left = C_in - cb, lim = left >= 64 ? 64 : (left + 2 * U - 1) / (2 * U) * (2 * U);
#pragma unroll 1
            for (int cl = 0; cl < lim; cl += 2 * U) {
                load_next(xb);
                mac_chunk(xa, cl);
                load_next(xa);
                mac_chunk(xb, cl + U);
            }
        }
        c64 *__restrict__ Yb = Yh + (tile0 + t) * C_out * 128 + 32 * wave + col;
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int o = o0 + 32 * i + 8 * (r / 4) + 4 * (hi ? 1 : 0) + (r % 4);
                if (o < C_out) Yb[o * 128] = make_float2(acc_re[i][r], acc_im[i][r]);
            }
    }
}

// The same contraction on the BF16 matrix pipe with every FP32 operand split exactly into three BF16 terms
// and the six largest cross products accumulated in FP32 (the scheme of the wave-specialised 1-D kernel; the
// dropped products are below 2^-23 |a||b|).  v_mfma_f32_32x32x16_bf16: the 16 k-slots of an instruction are
// 8 channels x (re, im); lanes 0-31 carry channels 0-3 of the step, lanes 32-63 channels 4-7, dword d of a lane
// = (re | im << 16) of channel 4g + d.  W is staged in LDS already split, as [channel / 4][term][output][channel % 4]
// dwords (re | im << 16), so an A operand is one 16-byte LDS read plus a sign flip (real part: (W.re, -W.im))
// or a half-word swap (imaginary part: (W.im, W.re)).
__global__ void __launch_bounds__(256, 2)
k_cgemm_modes(const c64 *__restrict__ Xh, const c64 *__restrict__ W, c64 *__restrict__ Yh,
              int C_in, int C_out, float scale, long long num_tiles, int tiles_per_wg)
{
    __shared__ __align__(16) unsigned Wl[16 * 3 * 64 * 4];  // 48 KB
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int col = lane & 31, g = lane >> 5;
    const int o0 = blockIdx.y * 64;
    const long long tile0 = (long long)blockIdx.x * tiles_per_wg;
    const int ntile = (int)(num_tiles - tile0 < tiles_per_wg ? num_tiles - tile0 : tiles_per_wg);
    const int c_pad = (C_in + 31) / 32 * 32;
    const bool one_block = C_in <= 64;

    floatx16 acc_re[2], acc_im[2];

    // Position of the next 8-channel step to load: (tile, channel).  The loads are unconditional (a run-time
    // condition around a register refill turns into copies behind a full wait): channels past C_in are read from
    // channel 0 and meet zero weights, steps past the last tile re-read the first tile and are never used.  Four
    // steps (128 bytes per lane, 64 KB per CU with two workgroups) are in flight; with one the kernel waited for
    // memory most of the time (3.2 TB/s).
    // Every workgroup walks the 8-channel steps of a 64-channel block starting at a different step (the sum does
    // not care about the order): tiles are 64 KB apart, so workgroups that walk them in the same order all read
    // the same few kilobytes of every 64 KB at the same time, which maps to a fraction of the memory channels.
    const int rot = 8 * (int)(blockIdx.x & 7);
    auto rotated = [&](int c_lin) __attribute__((always_inline)) {     // c_lin: position in the padded channel order
        const int cb = c_lin & ~63, left = C_in - cb, lim = left >= 64 ? 64 : (left + 31) / 32 * 32;
        return cb + ((c_lin - cb + rot) & (lim - 1));
    };
    int nt = 0, nc = 0;
    auto load_next = [&](c64 *xv) __attribute__((always_inline)) {
        const c64 *src = Xh + (tile0 + (nt < ntile ? nt : 0)) * C_in * 128 + 32 * wave + col;
        const int c0 = rotated(nc);
#pragma unroll
        for (int d = 0; d < 4; ++d) {
            const int c = c0 + 4 * g + d;
            xv[d] = src[(c < C_in ? c : 0) * 128];
        }
        nc += 8;
        if (nc >= c_pad) { nc = 0; ++nt; }
    };
    // operand split of one step (8 channels x 32 modes of this wave)
    auto split_step = [&](const c64 *xv, uintx4 *b) __attribute__((always_inline)) {
#pragma unroll
        for (int d = 0; d < 4; ++d) {
            const Split3 re = split3(xv[d].x), im = split3(xv[d].y);
            b[0][d] = pack_bf16(re.t0, im.t0);
            b[1][d] = pack_bf16(re.t1, im.t1);
            b[2][d] = pack_bf16(re.t2, im.t2);
        }
    };
    // one step: channels cl .. cl+7 of the staged block
    auto mac_step = [&](const uintx4 *b, int cl) __attribute__((always_inline)) {
        const unsigned *wsrc = Wl + (((cl >> 2) + g) * 3 * 64 + col) * 4;
        // smallest products first: (2,0) (0,2) (1,1) (1,0) (0,1) (0,0); real and imaginary accumulators alternate
        // (the matrix pipe runs one instruction at a time, so two chains keep it busy)
        constexpr int SA[6] = {2, 0, 1, 1, 0, 0}, SB[6] = {0, 2, 1, 0, 1, 0};
#pragma unroll
        for (int sl = 0; sl < 2; ++sl) {
            uintx4 a_re[3], a_im[3];
#pragma unroll
            for (int t = 0; t < 3; ++t) {
                const uintx4 w = *reinterpret_cast<const uintx4 *>(wsrc + (t * 64 + 32 * sl) * 4);
#pragma unroll
                for (int d = 0; d < 4; ++d) {
                    a_re[t][d] = w[d] ^ 0x80000000u;
                    a_im[t][d] = __builtin_amdgcn_alignbit(w[d], w[d], 16);
                }
            }
#pragma unroll
            for (int k = 0; k < 6; ++k) {
                const bf16x8 bb = __builtin_bit_cast(bf16x8, b[SB[k]]);
                acc_re[sl] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a_re[SA[k]]), bb, acc_re[sl], 0, 0, 0);
                acc_im[sl] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a_im[SA[k]]), bb, acc_im[sl], 0, 0, 0);
            }
        }
    };

    c64 xq[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i) load_next(xq[i]);
    for (int t = 0; t < ntile; ++t) {
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r) { acc_re[i][r] = 0.f; acc_im[i][r] = 0.f; }
        for (int cb = 0; cb < C_in; cb += 64) {
            if (!one_block || t == 0) {
                __syncthreads();                            // the previous block of W has been consumed
                // all 16 loads first: one at a time, each would wait out its own L2 round trip
                c64 wq[16];
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const int idx = i * 256 + tid, c = cb + idx / 64, o = o0 + idx % 64;
                    const bool ok = c < C_in && o < C_out;
                    const c64 w = W[ok ? (long long)c * C_out + o : 0];
                    wq[i] = ok ? w : make_float2(0.f, 0.f);
                }
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const int idx = i * 256 + tid, cl = idx / 64, ol = idx % 64;
                    const Split3 re = split3(wq[i].x * scale), im = split3(wq[i].y * scale);
                    unsigned *dst = Wl + (((cl >> 2) * 3) * 64 + ol) * 4 + (cl & 3);
                    dst[0 * 64 * 4] = pack_bf16(re.t0, im.t0);
                    dst[1 * 64 * 4] = pack_bf16(re.t1, im.t1);
                    dst[2 * 64 * 4] = pack_bf16(re.t2, im.t2);
                }
                __syncthreads();
            }
            const int left = C_in - cb, lim = left >= 64 ? 64 : (left + 31) / 32 * 32;
#pragma unroll 1
            for (int cl = 0; cl < lim; cl += 32) {
                // 32 channels per turn: split all four steps, refill their registers at once (the loads then have
                // the whole contraction of the turn to arrive and are all wanted together at the next turn), contract
                uintx4 bq[4][3];
#pragma unroll
                for (int i = 0; i < 4; ++i) split_step(xq[i], bq[i]);
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int i = 0; i < 4; ++i) load_next(xq[i]);
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    mac_step(bq[i], (cl + 8 * i + rot) & (lim - 1));
                    __builtin_amdgcn_sched_barrier(0);      // keeps the W operand reads of later steps from piling up
                }
            }
        }
        c64 *__restrict__ Yb = Yh + (tile0 + t) * C_out * 128 + 32 * wave + col;
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int o = o0 + 32 * i + 8 * (r / 4) + 4 * g + (r % 4);
                if (o < C_out) Yb[o * 128] = make_float2(acc_re[i][r], acc_im[i][r]);
            }
    }
}

// The same contraction for C_in <= 8 NSTEP <= 64 (one block of W), two mode tiles per workgroup, written as
// straight-line code: all NSTEP steps of a tile live in registers (16 KB per wave), every step's registers are
// refilled with the next tile right after their operand split, and without a loop back-edge the compiler waits for
// exactly the step it needs, so a whole tile per wave (128 KB per CU) stays in flight.  The looped kernel above
// drains all loads at the top of every turn and reaches 3.2 TB/s; this one is used whenever it applies.
template <int NSTEP>
__global__ void __launch_bounds__(256, 2)
k_cgemm_modes_small(const c64 *__restrict__ Xh, const c64 *__restrict__ W, c64 *__restrict__ Yh,
                    int C_in, int C_out, float scale, long long num_tiles)
{
    constexpr int TPW = 2;
    __shared__ __align__(16) unsigned Wl[2 * NSTEP * 3 * 64 * 4];   // [channel / 4][term][output][channel % 4]
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int col = lane & 31, g = lane >> 5;
    const int o0 = blockIdx.y * 64;
    const long long tile0 = (long long)blockIdx.x * TPW;
    const int ntile = (int)(num_tiles - tile0 < TPW ? num_tiles - tile0 : TPW);

    c64 xq[NSTEP][4];
    // step i of tile t of this workgroup (a tile past the end re-reads the last one and is never used; channels past
    // C_in are read from channel 0 and meet zero weights): unconditional loads, see the looped kernel
    auto load_step = [&](int t, int i) __attribute__((always_inline)) {
        const c64 *src = Xh + (tile0 + (t < ntile ? t : ntile - 1)) * C_in * 128 + 32 * wave + col;
#pragma unroll
        for (int d = 0; d < 4; ++d) {
            const int c = 8 * i + 4 * g + d;
            xq[i][d] = src[(c < C_in ? c : 0) * 128];
        }
    };
#pragma unroll
    for (int i = 0; i < NSTEP; ++i) load_step(0, i);        // in flight while W is staged

    {
        c64 wq[2 * NSTEP];
#pragma unroll
        for (int i = 0; i < 2 * NSTEP; ++i) {
            const int idx = i * 256 + tid, c = idx / 64, o = o0 + idx % 64;
            const bool ok = c < C_in && o < C_out;
            const c64 w = W[ok ? (long long)c * C_out + o : 0];
            wq[i] = ok ? w : make_float2(0.f, 0.f);
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int i = 0; i < 2 * NSTEP; ++i) {
            const int idx = i * 256 + tid, cl = idx / 64, ol = idx % 64;
            const Split3 re = split3(wq[i].x * scale), im = split3(wq[i].y * scale);
            unsigned *dst = Wl + (((cl >> 2) * 3) * 64 + ol) * 4 + (cl & 3);
            dst[0 * 64 * 4] = pack_bf16(re.t0, im.t0);
            dst[1 * 64 * 4] = pack_bf16(re.t1, im.t1);
            dst[2 * 64 * 4] = pack_bf16(re.t2, im.t2);
        }
    }
    __syncthreads();

    floatx16 acc_re[2], acc_im[2];
    static_for<0, TPW>([&](auto tc) {
        constexpr int t = decltype(tc)::value;
        if (t < ntile) {
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int r = 0; r < 16; ++r) { acc_re[i][r] = 0.f; acc_im[i][r] = 0.f; }
            static_for<0, NSTEP>([&](auto ic) {
                constexpr int i = decltype(ic)::value;
                uintx4 b[3];
#pragma unroll
                for (int d = 0; d < 4; ++d) {
                    const Split3 re = split3(xq[i][d].x), im = split3(xq[i][d].y);
                    b[0][d] = pack_bf16(re.t0, im.t0);
                    b[1][d] = pack_bf16(re.t1, im.t1);
                    b[2][d] = pack_bf16(re.t2, im.t2);
                }
                __builtin_amdgcn_sched_barrier(0);
                if constexpr (t + 1 < TPW) load_step(t + 1, i);
                __builtin_amdgcn_sched_barrier(0);
                const unsigned *wsrc = Wl + ((2 * i + g) * 3 * 64 + col) * 4;
                // smallest products first: (2,0) (0,2) (1,1) (1,0) (0,1) (0,0)
                constexpr int SA[6] = {2, 0, 1, 1, 0, 0}, SB[6] = {0, 2, 1, 0, 1, 0};
#pragma unroll
                for (int sl = 0; sl < 2; ++sl) {
                    uintx4 a_re[3], a_im[3];
#pragma unroll
                    for (int tm = 0; tm < 3; ++tm) {
                        const uintx4 w = *reinterpret_cast<const uintx4 *>(wsrc + (tm * 64 + 32 * sl) * 4);
#pragma unroll
                        for (int d = 0; d < 4; ++d) {
                            a_re[tm][d] = w[d] ^ 0x80000000u;
                            a_im[tm][d] = __builtin_amdgcn_alignbit(w[d], w[d], 16);
                        }
                    }
#pragma unroll
                    for (int k = 0; k < 6; ++k) {
                        const bf16x8 bb = __builtin_bit_cast(bf16x8, b[SB[k]]);
                        acc_re[sl] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a_re[SA[k]]), bb, acc_re[sl], 0, 0, 0);
                        acc_im[sl] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a_im[SA[k]]), bb, acc_im[sl], 0, 0, 0);
                    }
                }
                __builtin_amdgcn_sched_barrier(0);
            });
            c64 *__restrict__ Yb = Yh + (tile0 + t) * C_out * 128 + 32 * wave + col;
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int o = o0 + 32 * i + 8 * (r / 4) + 4 * g + (r % 4);
                    if (o < C_out) Yb[o * 128] = make_float2(acc_re[i][r], acc_im[i][r]);
                }
        }
    });
}

}  // namespace tfno
