// Wave-specialised fused FFT -> CGEMM -> iFFT kernel for N = 1024 (P = T = 32) on gfx950 (Sec. 4.3).
//
// Why this shape.  Measured on MI355X: FP32 MFMA and FP32 VALU instructions share one pipeline (a wave
// issuing v_mfma_f32_32x32x2_f32 and a wave issuing v_fma_f32 on the same SIMD take the SUM of their
// times), whereas BF16 MFMA runs beside VALU work at full rate.  The butterflies need the VALU, so the
// channel contraction goes to the BF16 matrix pipe with every FP32 operand split exactly into three BF16
// terms (a = a1 + a2 + a3, each the truncated top 8 significant bits of the remainder) and the six
// largest cross products accumulated in FP32; the dropped products are below 2^-23 of |a||b|, i.e. of the
// size of one FP32 rounding, so the result meets the same tolerance against the float64 oracle as an
// all-FP32 contraction.
//
//   workgroup = one batch row x 128 output channels, 512 threads = 8 waves, two per SIMD:
//     waves 0-3 ("F"): global loads and stores and the 32-point row stage of both transforms
//     waves 4-7 ("M"): the 32-point column stage of both transforms and the matrix pipe; wave m owns
//                      outputs 32m..32m+31 for all K modes
//   k-loop, 8 input channels (2 per F wave) per iteration, one workgroup barrier per iteration,
//   Z and XS double buffered:
//     F: stage A of block i+2 (32-point DFT in registers -> transposed LDS tile Z);  loads of block i+3
//     M: B operands of block i from XS (two 8-byte LDS reads per term and mode tile), 6 MFMAs
//        v_mfma_f32_32x32x16_bf16 per (mode tile, re|im);  stage B of block i+1 from Z (twiddle, column
//        DFT pruned to the Q = K/32 retained outputs, Sec. 3.3) -> 3 BF16 terms of (re, im) packed in
//        one dword -> XS;  W rows of block i+1 split meanwhile
//   MFMA k index (16 per instruction) = 8 channels x (re, im): lanes 0-31 carry channels 0-3, lanes 32-63
//   channels 4-7; within a lane dword d = (re | im << 16) of channel 4g + d.  The real part uses
//   A = (W.re, -W.im) per channel, the imaginary part A = (W.im, W.re).
//   epilogue: register r of lane l of mode tile q holds Yh[o][l%32 + 32 q] for o = 8(r/4) + 4(l/32) + r%4,
//   which is exactly what lane (half-wave l/32, column l%32) needs for the zero-padded, input-pruned column
//   transform (Sec. 3.3): the spectrum never goes through LDS.  M waves write the expanded columns to Z,
//   F waves run the 32-point inverse row stage and store, pipelined one round apart.  1/N is folded into W.
#pragma once
#include "common.h"
#include "fft_regs.h"
#include "fused1d.h"
#include "fused1d_kernel.h"
#include "bf16x3.h"


#include <type_traits>

namespace tfno {


template <int K>
struct WsCfg {
    static constexpr int N = 1024, P = 32, T = 32;
    static constexpr int Q = K / P;                 // retained outputs per column = 32-mode tiles
    static constexpr int NT = 512, NF = 4;          // F waves (and M waves)
    static constexpr int PPI = 8;                   // channels per k-loop iteration
    static constexpr int ZS = P * T;                // one pencil tile, rows XOR-swizzled instead of padded
    static constexpr int Z_BUF = NF * 2 * ZS;       // complex elements per Z buffer
    static constexpr int XS_BUF = 3 * Q * NF * 32 * 2;          // dwords per buffer: [term][q][wave][n][h]
    static constexpr size_t LDS_Z = sizeof(c64) * 2 * Z_BUF;
    static constexpr size_t LDS_XS = sizeof(unsigned) * 2 * XS_BUF;
    static constexpr size_t LDS_DYN = LDS_Z + LDS_XS;
    static constexpr size_t LDS_TW = sizeof(c64) * N;
    static_assert(K % 32 == 0 && Q >= 1 && Q <= 4, "K in {32, 64, 128}");
    static_assert(T % Q == 0, "Q must divide 32");
    static_assert(LDS_DYN + LDS_TW <= 160 * 1024, "LDS budget of one gfx950 CU");
};

template <int K, bool EVEN>
__global__ void __launch_bounds__(512)
k_fused1d_ws(Fused1dArgs a)
{
    using C = WsCfg<K>;
    constexpr int N = C::N, P = C::P, T = C::T, Q = C::Q, PPI = C::PPI, ZS = C::ZS, NT = C::NT;

    extern __shared__ __align__(16) unsigned char lds_raw[];
    c64 *Zl = reinterpret_cast<c64 *>(lds_raw);                               // [2][4 waves][2 slots][32 rows][32]
    unsigned *XS = reinterpret_cast<unsigned *>(lds_raw + C::LDS_Z);          // [2][3][Q][4][32][2]
    __shared__ c64 TW[N];                                                     // [t][p]: w_N^(t p)

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int bb = (int)xcd_contiguous(blockIdx.x, gridDim.x);
    const int o_base = blockIdx.y * 128;

    const long long bo = bb / a.inner_count, bi = bb % a.inner_count;
    const c64 *__restrict__ xb = a.x + bo * a.x_outer_stride + bi * a.x_inner_stride;
    c64 *__restrict__ yb = a.y + bo * a.y_outer_stride + bi * a.y_inner_stride;
    const int n_it = (a.C_in + PPI - 1) / PPI;
    const int h = lane >> 5, p = lane & 31;     // half-wave = pencil slot; p = t in the row stage, column in the column stage
    // Z tile element (row pp, position t) of this half-wave's pencil lives at  pp*32 + (t ^ pp):
    // a row write (lanes = consecutive t) and a column read (lanes = consecutive pp) both hit 32 distinct
    // 8-byte slots, with no padding.

    if (wave < 4) {
        // ============================================= F waves: global memory, both stages of the forward transform
        const int ztile = (wave * 2 + h) * ZS;  // this half-wave's pencil tile: only this half-wave touches it in the k-loop
        const int ja = wave * 2 + h;            // channel of this lane within the iteration's 8
        c64 v[P];

        auto load_pencil = [&](int c0) __attribute__((always_inline)) {
            const int c = c0 + ja;
            if constexpr (EVEN) {
                const c64 *src = xb + (long long)c * a.x_chan_stride + p;
#pragma unroll
                for (int jj = 0; jj < P; ++jj) v[jj] = src[T * jj];
            } else {
                const bool ok = c < a.C_in;
                const c64 *src = xb + (long long)(ok ? c : 0) * a.x_chan_stride + p;
#pragma unroll
                for (int jj = 0; jj < P; ++jj) {
                    c64 val = src[T * jj];
                    v[jj] = ok ? val : make_float2(0.f, 0.f);
                }
            }
        };
        // Row stage: 32-point transform of the slice in v, written transposed into the pencil's Z tile.  The first
        // butterfly level consumes v, so the loads of the next block are issued right after it and stay in flight
        // for a whole iteration.  The refill is a compile-time choice (`refill` is std::true_type or
        // std::false_type): a run-time condition around the loads would make v a merge of old and new values, which
        // the compiler resolves by loading into spare registers and copying them at the end of the iteration after
        // waiting for the data, and that wait exposes the whole memory latency in every iteration.
        auto row_stage = [&](auto refill, int next_c0) __attribute__((always_inline)) {
            c64 ea[P / 2], eb[P / 2], za[P / 2], zo[P / 2];
            dif_first_level<P, -1>(v, ea, eb);
            // keep the refill right here: the scheduler must not sink these loads below the butterflies
            __builtin_amdgcn_sched_barrier(0);
            if constexpr (decltype(refill)::value) load_pencil(next_c0);
            __builtin_amdgcn_sched_barrier(0);
            RegFFT<P / 2, -1, 1>::run(ea, za);
            RegFFT<P / 2, -1, 1>::run(eb, zo);
            c64 *Zt = Zl + ztile;
#pragma unroll
            for (int k = 0; k < P / 2; ++k) {
                Zt[(2 * k) * 32 + (p ^ (2 * k))] = za[k];
                Zt[(2 * k + 1) * 32 + (p ^ (2 * k + 1))] = zo[k];
            }
        };
        // Column stage of the same pencil, by the same half-wave (LDS operations of one wave complete in order, so
        // no barrier separates it from the row stage): twiddle, column transform pruned to Q outputs (Sec. 3.3),
        // exact BF16 split, into XS[xbuf].  The LDS reads are issued well ahead of their use, the column all at once
        // and the twiddles two groups ahead of the group being combined: left to itself the compiler waits after
        // every pair of reads, and 32 exposed LDS round trips cost more than all the arithmetic here.
        auto col_stage = [&](int xbuf) __attribute__((always_inline)) {
            constexpr int S = T / Q;                        // groups; group t1 holds inputs t1 + S t2
            const c64 *zcol = Zl + ztile + p * 32;          // row p of the tile = column p of the pencil
            const c64 *twp = TW + p;
            c64 zc[T], tw[T], xo[Q];
            auto read_tw = [&](auto t1c) __attribute__((always_inline)) {
                constexpr int t1 = decltype(t1c)::value;
#pragma unroll
                for (int t2 = 0; t2 < Q; ++t2)
                    if (t1 + S * t2 != 0) tw[t1 + S * t2] = twp[(t1 + S * t2) * P];
            };
#pragma unroll
            for (int tt = 0; tt < T; ++tt) zc[(tt % Q) * S + tt / Q] = zcol[((tt % Q) * S + tt / Q) ^ p];   // group order
            read_tw(std::integral_constant<int, 0>{});
            if constexpr (S > 1) read_tw(std::integral_constant<int, 1>{});
            __builtin_amdgcn_sched_barrier(0);
            static_for<0, S>([&](auto t1c) {
                constexpr int t1 = decltype(t1c)::value;
                if constexpr (t1 + 2 < S) read_tw(std::integral_constant<int, t1 + 2>{});
                c64 g[Q];
#pragma unroll
                for (int t2 = 0; t2 < Q; ++t2) {
                    const int tt = t1 + S * t2;
                    g[t2] = tt == 0 ? zc[0] : cmul(zc[tt], tw[tt]);
                }
                dft_prune_out_group<T, Q, -1, t1>(g, xo);
                __builtin_amdgcn_sched_barrier(0);
            });
            unsigned *dst = XS + xbuf * C::XS_BUF + (wave * 32 + p) * 2 + h;
#pragma unroll
            for (int q = 0; q < Q; ++q) {
                const Split3 re = split3(xo[q].x), im = split3(xo[q].y);
                dst[(0 * Q + q) * 256] = pack_bf16(re.t0, im.t0);
                dst[(1 * Q + q) * 256] = pack_bf16(re.t1, im.t1);
                dst[(2 * Q + q) * 256] = pack_bf16(re.t2, im.t2);
            }
        };
        constexpr std::true_type refill{};
        constexpr std::false_type last{};

        // Block j reaches XS[j & 1] before barrier number j + 2 (P1, P2, then one barrier per loop iteration); the
        // loads of block j + 1 are issued inside the row stage of block j.
        load_pencil(0);
        if (n_it > 1) row_stage(refill, PPI); else row_stage(last, 0);
        __syncthreads();                                    // P1: the M waves have built the twiddle table
        col_stage(0);
        __syncthreads();                                    // P2: XS[0] holds block 0
        int it = 0;
        for (; it + 2 < n_it; ++it) {                       // blocks 1 .. n_it - 2, each refilling v with its successor
            row_stage(refill, (it + 2) * PPI);
            col_stage((it + 1) & 1);
            __syncthreads();
        }
        if (it + 1 < n_it) {                                // the last block: nothing left to load
            row_stage(last, 0);
            col_stage((it + 1) & 1);
            __syncthreads();
        }
        // epilogue: stage A' of the pencil the M wave (wave + 4) left in Z[r & 1], coalesced store
        for (int r = 0; r < 16; ++r) {
            __syncthreads();                                // E_r: Z[r & 1] holds round r
            const c64 *Zt = Zl + (r & 1) * C::Z_BUF + ztile;
            c64 z[P], res[P];
#pragma unroll
            for (int pp = 0; pp < P; ++pp) z[pp] = Zt[pp * 32 + (p ^ pp)];
            RegFFT<P, +1, 1>::run(z, res);
            const int o = o_base + 32 * wave + 8 * (r / 4) + 4 * h + (r % 4);
            if (EVEN || o < a.C_out) {
                c64 *dst = yb + (long long)o * a.y_chan_stride + p;
#pragma unroll
                for (int jj = 0; jj < P; ++jj) store_nt(dst + T * jj, res[jj]);
            }
        }
        return;
    }

    // ====================================================================== M waves: column stage + matrix pipe
    const int m = wave - 4;
    const int o_lane = o_base + 32 * m + p;     // the output channel whose W this lane feeds
    const int ztile = (m * 2 + h) * ZS + p * 32;            // row p of the tile = column p of the pencil
    floatx16 acc_re[Q], acc_im[Q];
#pragma unroll
    for (int i = 0; i < Q; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) { acc_re[i][r] = 0.f; acc_im[i][r] = 0.f; }

    c64 wraw[4];                // W[c0 + 4h + d][o_lane], d < 4, of the next block
    uintx4 a_re[3], a_im[3];    // split A operands of the current block
    auto load_w = [&](int c0) __attribute__((always_inline)) {
#pragma unroll
        for (int d = 0; d < 4; ++d) {
            const int c = c0 + 4 * h + d;
            if constexpr (EVEN) {
                wraw[d] = a.W[(long long)c * a.C_out + o_lane];
            } else {
                const bool ok = c < a.C_in && o_lane < a.C_out;
                c64 val = a.W[ok ? (long long)c * a.C_out + o_lane : 0];
                wraw[d] = ok ? val : make_float2(0.f, 0.f);
            }
        }
    };
    auto split_w = [&]() __attribute__((always_inline)) {
#pragma unroll
        for (int d = 0; d < 4; ++d) {
            const Split3 re = split3(wraw[d].x * a.scale), im = split3(wraw[d].y * a.scale);
            // real part: (W.re, -W.im);  imaginary part: (W.im, W.re)
            a_re[0][d] = pack_bf16(re.t0, im.t0) ^ 0x80000000u;
            a_re[1][d] = pack_bf16(re.t1, im.t1) ^ 0x80000000u;
            a_re[2][d] = pack_bf16(re.t2, im.t2) ^ 0x80000000u;
            a_im[0][d] = pack_bf16(im.t0, re.t0);
            a_im[1][d] = pack_bf16(im.t1, re.t1);
            a_im[2][d] = pack_bf16(im.t2, re.t2);
        }
    };
    auto mfma_block = [&](int buf) __attribute__((always_inline)) {
        // lane (n = p, g = h) needs dwords [wave 2g][n][0..1] and [wave 2g+1][n][0..1] of every (term, q)
        const unsigned *src = XS + buf * C::XS_BUF + (2 * h * 32 + p) * 2;
#pragma unroll
        for (int q = 0; q < Q; ++q) {
            uintx4 b[3];
#pragma unroll
            for (int s = 0; s < 3; ++s) {
                const uint2 lo = *reinterpret_cast<const uint2 *>(src + (s * Q + q) * 256);
                const uint2 hi2 = *reinterpret_cast<const uint2 *>(src + (s * Q + q) * 256 + 64);
                b[s][0] = lo.x; b[s][1] = lo.y; b[s][2] = hi2.x; b[s][3] = hi2.y;
            }
            // smallest products first: (2,0) (0,2) (1,1) (1,0) (0,1) (0,0).  Real and imaginary accumulators
            // alternate; the matrix pipe runs one instruction at a time, so two chains already keep it busy.
            constexpr int SA[6] = {2, 0, 1, 1, 0, 0}, SB[6] = {0, 2, 1, 0, 1, 0};
#pragma unroll
            for (int k = 0; k < 6; ++k) {
                const bf16x8 bb16 = __builtin_bit_cast(bf16x8, b[SB[k]]);
                acc_re[q] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a_re[SA[k]]), bb16, acc_re[q], 0, 0, 0);
                acc_im[q] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a_im[SA[k]]), bb16, acc_im[q], 0, 0, 0);
            }
        }
    };

    // the twiddle table is only read by the column stage, so the M waves build it (accurate sincospi) while
    // the F waves already stream the first pencils; barrier P1 publishes it
    for (int i = (wave - 4) * 64 + lane; i < N; i += 256) TW[i] = cis2pi(-(float)((i / P) * (i % P)), (float)N);
    load_w(0);
    split_w();
    __syncthreads();                                        // P1
    __syncthreads();                                        // P2: XS[0] holds block 0
    for (int it = 0; it < n_it; ++it) {
        const bool more = it + 1 < n_it;
        if (more) load_w((it + 1) * PPI);
        mfma_block(it & 1);
        if (more) {
            split_w();
            __syncthreads();
        }
    }

    // ------------------------------------------------------------------ epilogue: column stage from registers
    // Register r of lane l of mode tile q holds Yh[o][p + 32 q] with o = 32 m + 8(r/4) + 4h + r%4: the Q inputs
    // lane (h, p) needs for the zero-padded, input-pruned column transform of that pencil (Sec. 3.3).
    for (int r = 0; r < 16; ++r) {
        c64 yin[Q];
        static_for<0, 16>([&](auto rc) {
            constexpr int R = decltype(rc)::value;
            if (r == R) {
#pragma unroll
                for (int q = 0; q < Q; ++q) yin[q] = make_float2(acc_re[q][R], acc_im[q][R]);
            }
        });
        c64 *zcol = Zl + (r & 1) * C::Z_BUF + ztile;
        dft_prune_in<T, Q, +1>(yin, [&](auto ttc, c64 val) __attribute__((always_inline)) {
            constexpr int tt = decltype(ttc)::value;
            if constexpr (tt == 0) zcol[p] = val;
            else {
                c64 w = TW[tt * P + p];
                zcol[tt ^ p] = cmul(val, make_float2(w.x, -w.y));
            }
        });
        __syncthreads();                                    // E_r
    }
}

template <int K>
hipError_t launch_fused1d_ws(const Fused1dArgs &a, long long batch_rows, hipStream_t s)
{
    using C = WsCfg<K>;
    static LdsLimitOnce lds_limit;
    const hipError_t e = lds_limit.set({reinterpret_cast<const void *>(&k_fused1d_ws<K, true>),
                                        reinterpret_cast<const void *>(&k_fused1d_ws<K, false>)}, (int)C::LDS_DYN);
    if (e != hipSuccess) return e;
    dim3 grid((unsigned)batch_rows, (unsigned)((a.C_out + 127) / 128));
    if (a.C_in % C::PPI == 0 && a.C_out % 128 == 0)
        hipLaunchKernelGGL((k_fused1d_ws<K, true>), grid, dim3(512), C::LDS_DYN, s, a);
    else
        hipLaunchKernelGGL((k_fused1d_ws<K, false>), grid, dim3(512), C::LDS_DYN, s, a);
    return hipGetLastError();
}

}  // namespace tfno
