// 2-D spectral convolution for gfx950 as three kernels whose only HBM intermediates are the TRUNCATED
// spectra (K1 x K2 per image instead of the K x N strips of the 2-D pipeline in Sec. 3.2 / 3.3).  Images are
// N1 x N2 (N2 the contiguous axis); the first axis keeps its first K1 bins, the last its first K2; N (K) below
// stands for the length (mode count) of whichever axis a stage transforms.
//
//   k_fwd2d   one workgroup per input image x[b, c]: truncated, output-pruned 2-D forward transform
//             -> Xh[b, c, k1, k2], k1 < K1, k2 < K2                     (reads N1*N2, writes K1*K2)
//             stored mode-tile major, [b][m / 128][c][m % 128] with m = k1 K2 + k2, so that the CGEMM streams
//             one contiguous [C, 128] block per workgroup
//   k_cgemm_modes   (cgemm_modes_kernel.h) Yh[b, o, m] = sum_c Xh[b, c, m] * W[c, o] / (N1 N2) over the K1*K2
//             retained modes; one W for all modes (Sec. 3.1)
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
template <int N1, int N2, int K1, int K2, bool RP16>
struct Cfg2d {
    static constexpr int LPR = N2 / 16;                         // lanes per row
    static constexpr int RP = RP16 ? 16 : 32;                   // rows per pass
    static constexpr int RPS = (256 / LPR) < RP ? 256 / LPR : RP; // rows per sweep of the workgroup
    static constexpr int ACTIVE = RPS * LPR;                    // threads that take part in the row stage
    // Workgroup size: the larger of the row stage's threads and the column stage's (four lanes per column k2).  Rows
    // of 64 points keep 128 threads busy in the row stage; with 256 threads per workgroup half of every workgroup's
    // registers belonged to waves that only met the barriers, and half as many images were in flight per CU.
    static constexpr int NT = ACTIVE > 4 * K2 ? ACTIVE : 4 * K2;
    static constexpr int WG_PER_CU = 768 / NT;                  // twelve waves per CU whatever the workgroup size
    static constexpr int S = N1 / RP;                           // passes
    static constexpr int SWEEPS = RP / RPS;
    static constexpr int NSWEEP = S * SWEEPS;
    static constexpr int KH = K2 / 16;                          // retained outputs per column k_lo
    static constexpr int CPL = 16 / LPR;                        // columns k_lo per lane after the transpose
    static constexpr int GS = N2 + (LPR < 16 ? LPR : 0);        // patch stride between the rows of a sweep
    static constexpr int TS = K2 + 4;                           // tile row stride (== 4 mod 16)
    static constexpr int RPL = RP / 4;                          // tile rows per lane in the column stage
    static constexpr int MREP = (K1 + RP - 1) / RP;             // k1 = k' + RP m
    static constexpr int NACC = RPL * MREP;
    static constexpr int NBUF = RP == 16 ? 2 : 1;               // tile buffers (2: one barrier per pass)
    static constexpr size_t LDS_BYTES = sizeof(c64) * ((size_t)RPS * GS + (size_t)NBUF * RP * TS + N1 + N2);
    static_assert((N1 == 64 || N1 == 128 || N1 == 256) && (N2 == 64 || N2 == 128 || N2 == 256), "N in {64, 128, 256}");
    static_assert((K1 == 16 || K1 == 32 || K1 == 64) && (K2 == 16 || K2 == 32 || K2 == 64), "K in {16, 32, 64}");
    static_assert(K1 <= N1 && K2 <= N2 && KH <= LPR && LPR % KH == 0, "K must divide N");
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
    c64 *tw;     // [16][LPR]   w_N2^(p k_lo)
    c64 *twn;    // [N1]        w_N1^t
};

template <int N1, int N2, int K1, int K2, bool RP16>
__device__ __forceinline__ Lds2d lds_setup(unsigned char *raw, int tid)
{
    using C = Cfg2d<N1, N2, K1, K2, RP16>;
    Lds2d l;
    l.scr = reinterpret_cast<c64 *>(raw);
    l.tile = l.scr + C::RPS * C::GS;
    l.tw = l.tile + C::NBUF * C::RP * C::TS;
    l.twn = l.tw + N2;
    for (int i = tid; i < N2; i += C::NT) l.tw[i] = cis2pi(-(float)((i / C::LPR) * (i % C::LPR)), (float)N2);
    for (int i = tid; i < N1; i += C::NT) l.twn[i] = cis2pi(-(float)i, (float)N1);
    return l;
}

// ------------------------------------------------------------------------------------------------ forward
// element offset of (channel c, mode m) of batch element b in a mode-tile-major spectrum buffer
__device__ __forceinline__ long long spec_index(long long b, int c, int C, int m, int M)
{
    return ((b * (M / 128) + m / 128) * C + c) * 128 + m % 128;
}

// FNO (both kernels): the layer as FNO models apply it to real fields.  x and y are float32 images; the first axis
// keeps the frequencies k1 = -h1 .. K1-h1-1 (both low-frequency blocks; position j = k1 + h1 in the spectrum
// buffers) -- a thread's accumulator slots then stand for other frequencies of the same residue mod RP, which only
// changes the exponents of the pass twiddles --; the last axis is the R2C / C2R pair: the forward transform of a
// real row is the complex one with zero imaginary part, and the C2R inverse equals twice the real part of the
// zero-padded complex inverse once the k2 = 0 column is halved (done here, at the spectrum store).
template <int N1, int N2, int K1, int K2, bool FNO = false>
__global__ void __launch_bounds__((Cfg2d<N1, N2, K1, K2, N2 == 256>::NT), (Cfg2d<N1, N2, K1, K2, N2 == 256>::WG_PER_CU))
k_fwd2d(const c64 *__restrict__ x, c64 *__restrict__ Xh, int C_in, int K1_keep, int K2_keep, int h1)
{
    using C = Cfg2d<N1, N2, K1, K2, N2 == 256>;
    constexpr int LPR = C::LPR, RPS = C::RPS, S = C::S, SWEEPS = C::SWEEPS, KH = C::KH, CPL = C::CPL;
    constexpr int GS = C::GS, TS = C::TS, MREP = C::MREP, RP = C::RP, RPL = C::RPL, NBUF = C::NBUF;
    __shared__ __align__(16) unsigned char raw[C::LDS_BYTES];
    const int tid = threadIdx.x;
    const Lds2d L = lds_setup<N1, N2, K1, K2, C::RP == 16>(raw, tid);

    // (workgroup id = image: giving each XCD a contiguous range of images, which helps the 1-D kernels, measured
    // 5-9 % slower here)
    const unsigned image = blockIdx.x;
    using XT = std::conditional_t<FNO, float, c64>;
    const XT *__restrict__ img = reinterpret_cast<const XT *>(x) + (long long)image * N1 * N2;
    // row-stage identity
    const bool row_on = tid < C::ACTIVE;
    const int g = tid / LPR, p = tid % LPR;
    c64 *scr = L.scr + g * GS;
    // column-stage identity
    const int k2 = tid >> 2, q4 = tid & 3, kb = ((q4 & 1) << 1) | (q4 >> 1);
    const bool col_on = k2 < K2;

    c64 acc[C::NACC];
#pragma unroll
    for (int i = 0; i < C::NACC; ++i) acc[i] = make_float2(0.f, 0.f);

    // Passes may run in any order (their contributions are summed).  The rows of one pass are N2*S*8 bytes apart
    // in memory, which maps them to a fraction of the L2 channels; workgroups that share an XCD (every 8th
    // workgroup id) therefore start at different passes so that together they use all channels.
    const int r_rot = (int)(blockIdx.x >> 3);
    auto load_rows = [&](c64 *v, int sweep) __attribute__((always_inline)) {
        const int r = (sweep / SWEEPS + r_rot) & (S - 1), s = (sweep % SWEEPS) * RPS + g;
        const XT *src = img + (long long)(r + S * s) * N2 + p;
        if (row_on) {
            if constexpr (FNO) {
                // (real rows; fetching pairs of floats and swapping halves between neighbouring lanes, as the inverse
                // kernel's stores do, measured 2 - 6 % slower here: the loads are not the limit)
#pragma unroll
                for (int j = 0; j < 16; ++j)
                    v[j] = make_float2(LPR >= 16 ? __builtin_nontemporal_load(src + LPR * j) : src[LPR * j], 0.f);
            } else {
#pragma unroll
                for (int j = 0; j < 16; ++j) {
                    // (quarter-line pieces per row and instruction, LPR = 4, measured 13 % faster through the cache)
                    // (non-temporal where measured to help: 256-point rows, 312 -> 267 us on the 256 x 256 layer)
                    if constexpr (LPR >= 8) v[j] = load_nt(src + LPR * j);
                    else v[j] = src[LPR * j];
                }
            }
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
            c64 t = ka == 0 ? G[0] : cmul(G[ka], L.twn[(q4 * ka) * (N1 / RP)]);
            t = quad_dft4_fwd(t, q4);                       // F_r[ka + RPL kb]
#pragma unroll
            for (int m = 0; m < MREP; ++m) {
                // frequency of accumulator slot (ka, m); FNO: position jres + RP m of the block, frequency - h1
                const int k1 = FNO ? (ka + RPL * kb + h1) % RP + RP * m - h1 : ka + RPL * kb + RP * m;
                acc[m * RPL + ka] = cmac(acc[m * RPL + ka], t, L.twn[(r * k1) & (N1 - 1)]);
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
                // position in the block of retained first-axis modes (FNO: frequency k1 - h1)
                const int k1 = FNO ? (ka + RPL * kb + h1) % RP + RP * m : ka + RPL * kb + RP * m;
                c64 val = acc[m * RPL + ka];
                if constexpr (FNO) {
                    if (k2 == 0) val = make_float2(0.5f * val.x, 0.5f * val.y);
                }
                // (modes at or past K1_keep x K2_keep are written as zeros: truncation finer than the kernel's)
                if (k1 < K1)
                    Xh[spec_index(b, c, C_in, k1 * K2 + k2, K1 * K2)] =
                        (k1 < K1_keep && k2 < K2_keep) ? val : make_float2(0.f, 0.f);
            }
    }
}

// ------------------------------------------------------------------------------------------------ inverse
template <int N1, int N2, int K1, int K2, bool FNO = false>
__global__ void __launch_bounds__((Cfg2d<N1, N2, K1, K2, false>::NT), (Cfg2d<N1, N2, K1, K2, false>::WG_PER_CU))
k_inv2d(const c64 *__restrict__ Yh, c64 *__restrict__ y, int C_out, int h1)
{
    using C = Cfg2d<N1, N2, K1, K2, false>;
    constexpr int LPR = C::LPR, RPS = C::RPS, S = C::S, SWEEPS = C::SWEEPS, KH = C::KH, CPL = C::CPL;
    constexpr int GS = C::GS, TS = C::TS, MREP = C::MREP, RP = C::RP, RPL = C::RPL, NBUF = C::NBUF;
    __shared__ __align__(16) unsigned char raw[C::LDS_BYTES];
    const int tid = threadIdx.x;
    const Lds2d L = lds_setup<N1, N2, K1, K2, C::RP == 16>(raw, tid);

    const unsigned image = blockIdx.x;
    using XT = std::conditional_t<FNO, float, c64>;
    XT *__restrict__ img = reinterpret_cast<XT *>(y) + (long long)image * N1 * N2;
    const bool row_on = tid < C::ACTIVE;
    const int g = tid / LPR, p = tid % LPR;
    c64 *scr = L.scr + g * GS;
    const int k2 = tid >> 2, q4 = tid & 3, kb = ((q4 & 1) << 1) | (q4 >> 1);
    const bool col_on = k2 < K2;

    // the retained spectrum of this image, K1*K2/256 (or fewer) bins per thread, for all passes
    c64 Y[C::NACC];
    {
        const long long b = image / C_out;
        const int o = (int)(image % C_out);
#pragma unroll
        for (int m = 0; m < MREP; ++m)
#pragma unroll
            for (int ka = 0; ka < RPL; ++ka) {
                const int k1 = FNO ? (ka + RPL * kb + h1) % RP + RP * m : ka + RPL * kb + RP * m;   // position in the block
                const bool ok = col_on && k1 < K1;
                c64 v = Yh[spec_index(b, o, C_out, ok ? k1 * K2 + k2 : 0, K1 * K2)];
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
                const int k1 = FNO ? (ka + RPL * kb + h1) % RP + RP * m - h1 : ka + RPL * kb + RP * m;     // frequency
                const c64 w = L.twn[(r * k1) & (N1 - 1)];
                t = cmac(t, Y[m * RPL + ka], make_float2(w.x, -w.y));
            }
            t = quad_dft4_inv(t, q4);
            if (ka != 0) {
                const c64 w = L.twn[(q4 * ka) * (N1 / RP)];
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
        XT *dst = img + (long long)(r + S * s) * N2 + p;
        if constexpr (FNO) {
            // The C2R result: the real part (the scale 2 / (N1 N2) is in W).  Lane p owns the floats p + LPR j; stored one
            // by one, the LPR lanes of a row write LPR * 4 bytes per instruction (16-byte pieces for 64-point rows).
            // Instead an even lane writes the pair (p, p + 1) of segment 2u and its odd neighbour the pair of segment
            // 2u + 1, after the two have swapped the halves that belong to each other: twice the bytes per piece, whole
            // lines for 256-point rows (64 x 64 fields: inverse kernel 99 -> 84 us).
            const int odd = p & 1;
            XT *pair = dst - odd;
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const float recv = quad_perm<QP_XOR1>(odd ? out[2 * u].x : out[2 * u + 1].x);
                tfno_vf2 q;
                q.x = odd ? recv : out[2 * u].x;
                q.y = odd ? out[2 * u + 1].x : recv;
                tfno_vf2 *q2 = reinterpret_cast<tfno_vf2 *>(pair + LPR * (2 * u + odd));
                if constexpr (LPR >= 16) __builtin_nontemporal_store(q, q2);       // whole 128-byte lines
                else *q2 = q;
            }
        } else {
#pragma unroll
            for (int j = 0; j < 16; ++j) {
                // non-temporal only where the LPR lanes of a row write whole 128-byte lines: with narrower rows every
                // store instruction leaves half or quarter lines, which cost up to 40 % of the kernel time when they
                // bypass the cache that would have merged them.  (Pairing complex elements between neighbouring
                // lanes as above, 16 bytes per lane, measured no faster for 64- and 128-point rows.)
                if constexpr (LPR >= 16) store_nt(dst + LPR * j, out[j]);
                else dst[LPR * j] = out[j];
            }
        }
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

}  // namespace tfno
