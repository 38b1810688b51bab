// Fused FFT -> CGEMM -> iFFT kernel for N = 256 with two wave groups in anti-phase (Sec. 4.3), gfx950.
//
// Why another kernel.  On a SIMD the matrix pipe and the vector ALU run side by side only when DIFFERENT waves feed
// them: a wave that issues MFMAs and butterflies in turn gets the sum of both times, and a workgroup whose waves all
// sit in the same phase (transforms, barrier, contraction, barrier) leaves one of the two units idle at any moment.
// Here the eight waves of a workgroup form two groups of four, one wave of each group per SIMD, and the groups
// alternate roles from slot to slot:
//
//   workgroup = one batch row x 32 OT output channels (OT in {2, 4, 8}: up to 256 outputs, so x is read and
//               transformed once per row whatever C_out is), 512 threads
//   block     = 16 input channels (4 pencils per wave of the transforming group)
//   slot s    : group s % 2 transforms block s (loads issued two slots earlier, 16-point row DFT in registers,
//               transpose through a Z tile that the two waves of a SIMD share, 16 -> Q pruned column DFT (Sec. 3.3),
//               exact BF16 split into operand tile s % 3), while the other group contracts blocks s-2 and s-1 from
//               their operand tiles (v_mfma_f32_32x32x16_bf16, six products per tile and part, see bf16x3.h);
//               one barrier per slot.  Three operand tiles rotate: a block is written in slot b and read in slots
//               b+1 and b+2.
//   weights   : W[c][o] of the two blocks a group contracts next are fetched at the start of its transform slot,
//               BEFORE that slot's pencil loads: global loads complete in issue order, so a weight fetched after a
//               block of pencil loads would make its consumer wait for HBM.
//   epilogue  : OT rounds; in a round every slab hands 32 / OT rows of its accumulators to a spectrum tile in LDS
//               (double buffered: one barrier per round) and every wave inverts four of them: zero-padded
//               input-pruned column transform (Sec. 3.3) into a private Z tile, 16-point inverse row transform,
//               non-temporal coalesced stores.  1/N is folded into W.
//
// Host side guarantees: C_in a multiple of 32 and at least 64 (an even number >= 4 of blocks), C_out a multiple of 32.
#pragma once
#include "common.h"
#include "fft_regs.h"
#include "fused1d.h"
#include "fused1d_kernel.h"   // wave_sync, floatx16
#include "bf16x3.h"

namespace tfno {

template <int K, int OT>
struct PpCfg {
    static constexpr int N = 256, P = 16, T = 16, Q = K / P, KT = K / 32;
    static constexpr int NW = 8, NT = 512, PPW = 4, PPB = 16;
    static constexpr int TILES = OT * KT;
    static constexpr int TPW = (TILES + NW - 1) / NW;       // 32 x 32 complex tiles per wave
    static constexpr int ZROW = T + 1, ZS = P * ZROW;       // padded transpose tile of one pencil
    static constexpr int XH_BUF = 3 * (PPB / 4) * KT * 128; // dwords per operand tile: [term][channel / 4][tile][mode % 32][channel % 4]
    static constexpr int WPS = NW / OT;                     // waves that invert one slab
    static constexpr int RR = 4 * WPS;                      // rows of a slab per epilogue round
    static constexpr int ROUNDS = 32 / RR;
    static constexpr int YROW = K + 16;                     // spectrum-tile row stride: 32 dwords mod 64, so the four rows a
                                                            // wave reads land in disjoint bank halves
    static constexpr size_t LDS_ZLOOP = sizeof(c64) * 4 * PPW * ZS;
    static constexpr size_t LDS_LOOP = LDS_ZLOOP + sizeof(unsigned) * 3 * XH_BUF;
    static constexpr size_t LDS_ZEPI = sizeof(c64) * NW * PPW * ZS;
    static constexpr size_t LDS_EPI = LDS_ZEPI + sizeof(c64) * 2 * 32 * YROW;
    static constexpr size_t LDS_DYN = LDS_LOOP > LDS_EPI ? LDS_LOOP : LDS_EPI;
    static_assert(K == 32 || K == 64 || K == 128, "K in {32, 64, 128}");
    static_assert(OT == 2 || OT == 4 || OT == 8, "output slab of 64, 128 or 256 channels");
    static_assert(TPW <= KT && KT % TPW == 0, "a wave's tiles share one 32-output slab");
    static_assert(LDS_DYN + sizeof(c64) * N <= 160 * 1024, "LDS budget of one gfx950 CU");
};

template <int K, int OT>
__global__ void __launch_bounds__(512)
k_fused1d_pp(Fused1dArgs a)
{
    using C = PpCfg<K, OT>;
    constexpr int N = C::N, P = C::P, T = C::T, Q = C::Q, KT = C::KT, PPW = C::PPW, PPB = C::PPB, TPW = C::TPW;
    constexpr int ZROW = C::ZROW, ZS = C::ZS, XH_BUF = C::XH_BUF, WPS = C::WPS, RR = C::RR, YROW = C::YROW;

    extern __shared__ __align__(16) unsigned char lds_raw[];
    c64 *Zl = reinterpret_cast<c64 *>(lds_raw);                                 // k-loop [4][PPW][ZS]; epilogue [8][PPW][ZS]
    unsigned *XH = reinterpret_cast<unsigned *>(lds_raw + C::LDS_ZLOOP);        // [3][XH_BUF]
    c64 *YH = reinterpret_cast<c64 *>(lds_raw + C::LDS_ZEPI);                   // epilogue [2][32][YROW]
    __shared__ c64 TW[N];                                                       // [t][p]: w_N^(t p)

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);                  // uniform: the role branches are scalar
    const int grp = wave >> 2, wq = wave & 3;
    const int bb = (int)blockIdx.x;
    const int o_base = blockIdx.y * (32 * OT);
    const long long bo = bb / a.inner_count, bi = bb % a.inner_count;
    const c64 *__restrict__ xb = a.x + bo * a.x_outer_stride + bi * a.x_inner_stride;
    c64 *__restrict__ yb = a.y + bo * a.y_outer_stride + bi * a.y_inner_stride;

    for (int i = tid; i < N; i += C::NT) TW[i] = cis2pi(-(float)((i / P) * (i % P)), (float)N);

    // transform identity: pencil slot jw of the wave, element t of every 16-point row; column p of pencil j
    const int jw = lane / T, t = lane % T;
    c64 *Zw = Zl + wq * (PPW * ZS);
    // contraction identity
    const int tile0 = wave * TPW;
    const int ot_w = tile0 / KT, kt0 = tile0 % KT;
    const bool slab_ok = tile0 < C::TILES && o_base + 32 * ot_w < a.C_out;
    const int o_lane = slab_ok ? o_base + 32 * ot_w + (lane & 31) : 0;          // the output channel whose W this lane feeds
    const bool hi = lane >= 32;
    const int n_blk = a.C_in / PPB;
    const int k_keep = a.K_keep > 0 ? a.K_keep : K;

    floatx16 acc_re[TPW], acc_im[TPW];
#pragma unroll
    for (int i = 0; i < TPW; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) { acc_re[i][r] = 0.f; acc_im[i][r] = 0.f; }

    c64 v[P];       // the pencil slice this lane transforms next
    c64 wv[16];     // W[c][o_lane] of the two blocks contracted next: [block][4 step + d], channel 16 b + 8 step + 4 (lane / 32) + d
    __syncthreads();

    // Every global address is a wave-uniform base (scalar registers) plus a 32-bit per-lane offset that is computed
    // once: 64-bit per-lane addresses for each of the 16 + 16 loads of a slot cost more registers than the kernel has.
    const unsigned x_lane = (unsigned)(jw * (int)a.x_chan_stride + t);                  // pencil jw of the wave, element t
    const unsigned w_lane = (unsigned)(4 * (lane >> 5) * a.C_out + o_lane);             // channel 4 (lane / 32) of a step
    const unsigned y_lane = (unsigned)(jw * (int)a.y_chan_stride + t);
    auto load_pencil = [&](int b) __attribute__((always_inline)) {
        const c64 *src = xb + (long long)(PPB * b + PPW * wq) * a.x_chan_stride;       // uniform
#pragma unroll
        for (int jj = 0; jj < P; ++jj) v[jj] = src[x_lane + T * jj];
    };
    auto load_w_block = [&](c64 *dst, int b) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const c64 *row = a.W + (long long)(PPB * b + 8 * (i / 4) + (i % 4)) * a.C_out;  // uniform
            dst[i] = row[w_lane];
        }
    };
    auto put_operand = [&](unsigned *XHb, int jg, int k, c64 val) __attribute__((always_inline)) {
        unsigned *d = XHb + (jg >> 2) * (KT * 128) + (jg & 3) + (k >> 5) * 128 + (k & 31) * 4;
        const Split3 re = split3(val.x), im = split3(val.y);
        d[0 * (PPB / 4) * KT * 128] = pack_bf16(re.t0, im.t0);
        d[1 * (PPB / 4) * KT * 128] = pack_bf16(re.t1, im.t1);
        d[2 * (PPB / 4) * KT * 128] = pack_bf16(re.t2, im.t2);
    };
    // row stage: 16-point transform of the slice in v, written transposed into the Z tile
    auto stage_a = [&]() __attribute__((always_inline)) {
        c64 z[P];
        RegFFT<P, -1, 1>::run(v, z);
#pragma unroll
        for (int p = 0; p < P; ++p) Zw[jw * ZS + p * ZROW + t] = z[p];
    };
    // column stage: twiddle, 16-point transform pruned to the Q retained outputs, exact split into operand tile `buf`
    auto stage_b = [&](int buf) __attribute__((always_inline)) {
        unsigned *XHb = XH + buf * XH_BUF;
        const int j = lane / P, p = lane % P;
        const c64 *zcol = Zw + j * ZS + p * ZROW;
        c64 xo[Q];
        if constexpr (TPW <= 2) {
            c64 zc[T], tw[T];
#pragma unroll
            for (int tt = 0; tt < T; ++tt) {
                zc[tt] = zcol[tt];
                if (tt != 0) tw[tt] = TW[tt * P + p];
            }
            __builtin_amdgcn_sched_barrier(0);  // all LDS reads of the column are issued before the first use
            dft_prune_out<T, Q, -1>([&](auto ttc) __attribute__((always_inline)) {
                constexpr int tt = decltype(ttc)::value;
                if constexpr (tt == 0) return zc[0];
                else return cmul(zc[tt], tw[tt]);
            }, xo);
        } else {
            // four tiles of accumulators leave no room for a whole column: one group of Q inputs at a time
            constexpr int S = T / Q;
            static_for<0, S>([&](auto t1c) {
                constexpr int t1 = decltype(t1c)::value;
                c64 g[Q], tw[Q];
#pragma unroll
                for (int t2 = 0; t2 < Q; ++t2) {
                    g[t2] = zcol[t1 + S * t2];
                    if (t1 + S * t2 != 0) tw[t2] = TW[(t1 + S * t2) * P + p];
                }
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int t2 = 0; t2 < Q; ++t2)
                    if (t1 + S * t2 != 0) g[t2] = cmul(g[t2], tw[t2]);
                dft_prune_out_group<T, Q, -1, t1>(g, xo);
            });
        }
        const int jg = PPW * wq + j;
#pragma unroll
        for (int q = 0; q < Q; ++q) put_operand(XHb, jg, p + P * q, xo[q]);
        if (k_keep < K) {                       // truncation finer than the kernel's K: surplus bins enter as zeros
#pragma unroll
            for (int q = 0; q < Q; ++q)
                if (p + P * q >= k_keep) put_operand(XHb, jg, p + P * q, make_float2(0.f, 0.f));
        }
    };
    // contraction of one block (two 8-channel steps) from operand tile `buf` with the weights wb[8]
    auto split_w = [&](const c64 *w4, uintx4 *a_re, uintx4 *a_im) __attribute__((always_inline)) {
#pragma unroll
        for (int d = 0; d < 4; ++d) {
            const Split3 re = split3(w4[d].x * a.scale), im = split3(w4[d].y * a.scale);
            a_re[0][d] = pack_bf16(re.t0, im.t0) ^ 0x80000000u;
            a_re[1][d] = pack_bf16(re.t1, im.t1) ^ 0x80000000u;
            a_re[2][d] = pack_bf16(re.t2, im.t2) ^ 0x80000000u;
            a_im[0][d] = pack_bf16(im.t0, re.t0);
            a_im[1][d] = pack_bf16(im.t1, re.t1);
            a_im[2][d] = pack_bf16(im.t2, re.t2);
        }
    };
    // One block = 2 TPW tile-steps (8 channels x 32 modes x 32 outputs each, 12 MFMAs).  The B operands of tile-step
    // n+1 are read from LDS before the MFMAs of tile-step n are issued, so no tile-step waits for its LDS reads.
    auto read_b = [&](uintx4 *b, const unsigned *XS, int n) __attribute__((always_inline)) {
        const int s2 = n / TPW, i = n % TPW;
#pragma unroll
        for (int tm = 0; tm < 3; ++tm)
            b[tm] = *reinterpret_cast<const uintx4 *>(XS + ((tm * (PPB / 4) + 2 * s2) * KT + i) * 128);
    };
    auto mfma_tile = [&](int i, const uintx4 *b, const uintx4 *a_re, const uintx4 *a_im) __attribute__((always_inline)) {
        constexpr int SA[6] = {2, 0, 1, 1, 0, 0}, SB[6] = {0, 2, 1, 0, 1, 0};   // smallest products first
#pragma unroll
        for (int k = 0; k < 6; ++k) {
            const bf16x8 bb16 = __builtin_bit_cast(bf16x8, b[SB[k]]);
            acc_re[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a_re[SA[k]]), bb16, acc_re[i], 0, 0, 0);
            acc_im[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a_im[SA[k]]), bb16, acc_im[i], 0, 0, 0);
        }
    };
    auto mfma_block = [&](int buf, const c64 *wb) __attribute__((always_inline)) {
        const unsigned *XS = XH + buf * XH_BUF + (hi ? 1 : 0) * (KT * 128) + kt0 * 128 + (lane & 31) * 4;
        uintx4 a_re[2][3], a_im[2][3];          // operands of the two 8-channel steps
        uintx4 b[2][3];
        read_b(b[0], XS, 0);
        split_w(wb, a_re[0], a_im[0]);
        if constexpr (TPW <= 2) split_w(wb + 4, a_re[1], a_im[1]);
#pragma unroll
        for (int n = 0; n < 2 * TPW; ++n) {
            if (n + 1 < 2 * TPW) read_b(b[(n + 1) & 1], XS, n + 1);
            if constexpr (TPW > 2) {
                if (n == TPW) split_w(wb + 4, a_re[0], a_im[0]);    // four tiles: no room for both steps' operands
            }
            const int st = TPW <= 2 ? n / TPW : 0;
            mfma_tile(n % TPW, b[n & 1], a_re[st], a_im[st]);
        }
    };
    // Transform slot of block b: row stage (consumes v), the weights of the group's next contraction slot (blocks b-1
    // and b), column stage, and last the pencil loads of block b+2, which then have the whole contraction slot to
    // arrive.  Global loads complete in issue order: the weights go first so that the contraction never waits for
    // pencils.  The fences keep the compiler from moving the loads.  (The slots are peeled by hand and every choice
    // is a compile-time flag: a run-time condition around a refill of v turns into copies behind a full wait, and a
    // single loop over slots with the role chosen inside spills hundreds of registers.)
    auto fft_slot = [&](auto w_first, auto do_load, int b) __attribute__((always_inline)) {
        stage_a();
        wave_sync();
        __builtin_amdgcn_sched_barrier(0);
        if constexpr (decltype(w_first)::value) load_w_block(wv, b - 1);
        load_w_block(wv + 8, b);
        __builtin_amdgcn_sched_barrier(0);
        stage_b(b % 3);
        __builtin_amdgcn_sched_barrier(0);
        if constexpr (decltype(do_load)::value) load_pencil(b + 2);
        __builtin_amdgcn_sched_barrier(0);
    };
    // Contraction slot: blocks b0 (if `first`) and b0 + 1 (if `second`)
    auto mfma_slot = [&](auto first, auto second, int b0) __attribute__((always_inline)) {
        if (slab_ok) {
            if constexpr (decltype(first)::value) mfma_block(b0 % 3, wv);
            if constexpr (decltype(second)::value) mfma_block((b0 + 1) % 3, wv + 8);
        }
        __builtin_amdgcn_sched_barrier(0);
    };
    const std::true_type yes{};
    const std::false_type no{};

    // ------------------------------------------------------------------ k-loop: slots 0 .. n_blk
    if (grp == 0) {
        // transforms blocks 0, 2, ..; contracts {0}, {1, 2}, {3, 4}, .., {n_blk - 3, n_blk - 2}, {n_blk - 1}
        load_pencil(0);
        fft_slot(no, yes, 0);
        __syncthreads();
        mfma_slot(no, yes, -1);
        __syncthreads();
        int b = 2;
        for (; b + 2 < n_blk; b += 2) {
            fft_slot(yes, yes, b);
            __syncthreads();
            mfma_slot(yes, yes, b - 1);
            __syncthreads();
        }
        fft_slot(yes, no, b);                   // b = n_blk - 2: the group's last transform
        __syncthreads();
        c64 wx[8];
        load_w_block(wx, n_blk - 1);            // for the single block of the last slot
        __builtin_amdgcn_sched_barrier(0);
        mfma_slot(yes, yes, b - 1);
        __syncthreads();
        if (slab_ok) mfma_block((n_blk - 1) % 3, wx);
    } else {
        // transforms blocks 1, 3, ..; contracts {0, 1}, {2, 3}, .., {n_blk - 2, n_blk - 1}
        load_pencil(1);
        __syncthreads();                        // slot 0: nothing to contract yet
        fft_slot(yes, yes, 1);
        __syncthreads();
        int b = 3;
        for (; b + 2 < n_blk; b += 2) {
            mfma_slot(yes, yes, b - 3);
            __syncthreads();
            fft_slot(yes, yes, b);
            __syncthreads();
        }
        mfma_slot(yes, yes, b - 3);             // b = n_blk - 1
        __syncthreads();
        fft_slot(yes, no, b);
        __syncthreads();
        mfma_slot(yes, yes, n_blk - 2);
    }

    // ------------------------------------------------------------------ epilogue
    c64 *Ze = Zl + wave * (PPW * ZS);           // every wave has its own Z tile now
    const int slab_e = wave / WPS, row_e = 4 * (wave % WPS);    // the slab and the rows of a round that this wave inverts
    const bool store_ok = o_base + 32 * slab_e < a.C_out;
    __syncthreads();                            // the operand tiles are free: the spectrum tiles alias them
    static_for<0, C::ROUNDS>([&](auto rc) {
        constexpr int r = decltype(rc)::value;
        c64 *YHb = YH + (r & 1) * (32 * YROW);
        // Accumulator register R of lane l of tile i holds Yh[o][k], o = 8 (R / 4) + 4 (l / 32) + R % 4 of the wave's
        // slab, k = 32 (kt0 + i) + l % 32.  Round r hands over rows RR r .. RR r + RR - 1.
        if (slab_ok) {
#pragma unroll
            for (int i = 0; i < TPW; ++i) {
                c64 *dst = YHb + (ot_w * RR) * YROW + 32 * (kt0 + i) + (lane & 31);
                if constexpr (RR == 4) {
                    if ((lane >> 5) == (r & 1)) {
#pragma unroll
                        for (int x = 0; x < 4; ++x)
                            dst[x * YROW] = make_float2(acc_re[i][4 * (r / 2) + x], acc_im[i][4 * (r / 2) + x]);
                    }
                } else {
#pragma unroll
                    for (int y = 0; y < RR / 8; ++y)
#pragma unroll
                        for (int x = 0; x < 4; ++x) {
                            const int R = (RR / 8) * 4 * r + 4 * y + x;
                            dst[(8 * y + 4 * (lane >> 5) + x) * YROW] = make_float2(acc_re[i][R], acc_im[i][R]);
                        }
                }
            }
        }
        __syncthreads();
        if (store_ok) {
            // zero-padded, input-pruned column transform of the Q retained modes, conj twiddle, transposed into Ze
            const int j = lane / P, p = lane % P;
            const c64 *yrow = YHb + (slab_e * RR + row_e + j) * YROW + p;
            c64 yin[Q];
#pragma unroll
            for (int q = 0; q < Q; ++q) yin[q] = yrow[P * q];
            c64 *zcol = Ze + j * ZS + p * ZROW;
            dft_prune_in<T, Q, +1>(yin, [&](auto ttc, c64 val) __attribute__((always_inline)) {
                constexpr int tt = decltype(ttc)::value;
                if constexpr (tt == 0) zcol[0] = val;
                else {
                    c64 w = TW[tt * P + p];
                    zcol[tt] = cmul(val, make_float2(w.x, -w.y));
                }
            });
            wave_sync();
            // inverse row transform of pencil jw, store
            c64 z[P], res[P];
#pragma unroll
            for (int pp = 0; pp < P; ++pp) z[pp] = Ze[jw * ZS + pp * ZROW + t];
            RegFFT<P, +1, 1>::run(z, res);
            c64 *dst = yb + (long long)(o_base + 32 * slab_e + RR * r + row_e) * a.y_chan_stride;  // uniform
#pragma unroll
            for (int jj = 0; jj < P; ++jj) store_nt(dst + (y_lane + T * jj), res[jj]);
            wave_sync();
        }
    });
}

template <int K, int OT>
hipError_t launch_fused1d_pp(const Fused1dArgs &a, long long batch_rows, hipStream_t s)
{
    using C = PpCfg<K, OT>;
    static LdsLimitOnce lds_limit;
    const hipError_t e = lds_limit.set({reinterpret_cast<const void *>(&k_fused1d_pp<K, OT>)}, (int)C::LDS_DYN);
    if (e != hipSuccess) return e;
    dim3 grid((unsigned)batch_rows, (unsigned)((a.C_out + 32 * OT - 1) / (32 * OT)));
    hipLaunchKernelGGL((k_fused1d_pp<K, OT>), grid, dim3(C::NT), C::LDS_DYN, s, a);
    return hipGetLastError();
}

}  // namespace tfno
