// Fully fused FFT -> CGEMM -> iFFT kernel along the last (contiguous) axis (Sec. 4.3), for gfx950.
//
// Work decomposition (re-derived for wave64 / MFMA / 160 KB LDS; the idea kept from the paper is that one
// workgroup walks the hidden dimension in step with the GEMM k-loop, Sec. 2.3 / 4.1):
//
//   workgroup  = one batch row `bb` x one slab of 32*OT output channels, 256 threads (4 waves)
//   k-loop     : PPI = 256/T input channels per iteration, 64/T of them per wave.  N = P * T.
//     stage A  : thread (pencil slot jw, t) loads x[c][t + T*jj], jj < P (coalesced), P-point DFT in
//                registers, twiddle by w_N^(t p), writes column-major into the wave's PRIVATE LDS tile
//                Z[jw][p][t]  -- both transform stages of a pencil run in one wave, so the transpose needs
//                no workgroup barrier
//     stage B  : lane (pencil slot j, column p) reads Z[j][p][0..T), T-point DFT pruned to the Q = K/P
//                outputs that are retained modes k = p + P q < K (built-in truncation + output pruning,
//                Sec. 3.3), writes the planar operand tile XH[buf][c][re|im][k] (double buffered)
//     MFMA     : Yh[o][k] += W[c][o] * Xh[c][k] with v_mfma_f32_32x32x2_f32: the two k-slots of one
//                instruction carry (re, im) of ONE channel, so a complex MAC over 32 outputs x 32 modes is
//                two MFMAs (real part with A = (W.re, -W.im), imaginary part with A = (W.im, W.re)).
//                Accumulators stay in registers for the whole k-loop.  The MFMAs of iteration i sit in the
//                same basic block as the transforms of iteration i+1 so that the matrix cores run under the
//                VALU work; one workgroup barrier per iteration publishes the next XH buffer.
//   epilogue   : (a) when a wave owns a whole 32-output slab and P = 32, the accumulator layout already is
//                the stage-B' input layout (lane = column p, tile = q), so the spectrum goes from registers
//                straight into the zero-padded, input-pruned inverse transform (Sec. 3.3) with no LDS
//                handoff and no barrier; (b) otherwise accumulators -> LDS YH[o][k] per slab, then the same
//                two inverse stages.  Stage A' applies conj twiddles, P-point inverse DFT, coalesced store.
//                The 1/N scale is folded into W when it is loaded.
//
// LDS handoffs (the counterpart of the two swizzles of Sec. 4.1 / 4.2, re-derived for 4-byte banks and
// 8-byte accesses): Z rows are padded to T+1 complex so that both the write (consecutive t) and the
// transposed read (consecutive p, stride T+1) touch distinct banks; XH is planar so that an MFMA operand
// read is 32 consecutive floats per half-wave.
#pragma once
#include "common.h"
#include "fft_regs.h"
#include "fused1d.h"
#include "bf16x3.h"

namespace tfno {

typedef float floatx16 __attribute__((ext_vector_type(16)));

template <int N> struct Decomp;
template <> struct Decomp<64>   { static constexpr int P = 8,  T = 8;  };
template <> struct Decomp<128>  { static constexpr int P = 16, T = 8;  };
template <> struct Decomp<256>  { static constexpr int P = 16, T = 16; };
template <> struct Decomp<512>  { static constexpr int P = 32, T = 16; };
template <> struct Decomp<1024> { static constexpr int P = 32, T = 32; };

// BF: the contraction runs on the BF16 matrix pipe with the exact three-term operand split (bf16x3.h) instead of
// FP32 MFMA; the operand tile then holds packed BF16 terms, [term][channel / 4][mode tile][mode % 32][channel % 4].
// NW: waves per workgroup, XB: operand tile buffers.
//   NW 4, XB 2: one wave per SIMD and workgroup, operand tile double buffered, one barrier per block.
//   NW 4, XB 1: the same with a single operand tile and two barriers per block; what this buys is LDS: at K = 128 the
//               workgroup drops from 86 KB to 61 KB, so TWO workgroups share a CU and one's barriers, load waits,
//               prologue and epilogue hide under the other's work (with one wave per SIMD nothing else hides them).
//   NW 8, XB 1: two waves per SIMD in one workgroup; a block is twice as many channels; carries the 256-output slab
//               (OT = 8) at K = 128, whose accumulators alone are half of the CU's register file.
// KS: (BF16 contraction only) the 8-channel steps of a block are dealt out to KS waves per 32 x 32 tile, each with its
//     own partial accumulator; the partial sums meet in the epilogue's LDS tile.  For narrow slabs (fewer tiles than
//     waves) this puts the contraction on all waves instead of one or two that the others wait for at the barrier.
template <int N, int K, int OT, bool BF = false, int NW_ = 4, int XB_ = 2, int KS_ = 1>
struct FusedCfg {
    static constexpr int P = Decomp<N>::P, T = Decomp<N>::T;
    static constexpr int Q = K / P;                 // retained outputs per column of stage B
    static constexpr int NW = NW_, NT = 64 * NW;
    static constexpr int XB = XB_;                  // operand tile buffers
    static constexpr bool WIDE = XB == 1;           // single operand tile: two barriers per block
    static_assert(NW == 4 || XB == 1, "eight waves come with the single operand tile");
    static constexpr int RPW = 32 / NW;             // rows of a 32-output slab that a wave inverts
    static constexpr int PPW = 64 / T;              // pencils per wave per round
    static constexpr int PPI = NW * PPW;            // pencils (channels) per k-loop iteration
    static constexpr int CPL = P / T;               // stage-B columns per lane
    static constexpr int KT = (K + 31) / 32;        // 32-mode MFMA tiles
    static constexpr int KPAD = KT * 32;
    static constexpr int TILES = OT * KT;
    static constexpr int KS = KS_;                      // waves that share one tile's channel steps
    static constexpr int TPW = KS > 1 ? 1 : (TILES + NW - 1) / NW;     // 32x32 complex tiles per wave
    static constexpr bool ALLT = KS > 1 ? TILES * KS == NW : TILES % NW == 0;   // every wave owns exactly TPW tiles
    static constexpr bool DIRECT = KS == 1 && P == 32 && OT == NW && TPW == KT;   // wave w owns output slab w entirely
    static constexpr int RPA = 32 / T;              // direct epilogue: stage-B' rounds per stage-A' round
    static constexpr int ZROW = T + 1;
    static constexpr int ZS = P * ZROW + (T == 8 ? 8 - (P * ZROW) % 16 + ((P * ZROW) % 16 > 8 ? 16 : 0) : 0);
    static constexpr int YROW = K + 1;
    static constexpr int XH_BUF = BF ? 3 * (PPI / 4) * KT * 128 : PPI * 2 * KPAD;   // 4-byte words per XH buffer
    static constexpr int NWV = BF ? PPI / 2 / KS : PPI;  // W values a lane holds per iteration
    static constexpr size_t LDS_Z = sizeof(c64) * NW * PPW * ZS;
    static constexpr size_t LDS_XH = sizeof(float) * XB * XH_BUF;
    // Partial sums of a split contraction: KS copies of the epilogue tile that the inverse transform adds up as it
    // reads them, or, where only that lets a third workgroup fit the CU's LDS, ONE copy that the KS waves of a tile add
    // to in turn (a barrier per turn).
    static constexpr size_t lds_with_copies(int c)
    {
        const size_t yh = sizeof(c64) * c * 32 * YROW, xh = sizeof(float) * XB * XH_BUF;
        return sizeof(c64) * NW * PPW * ZS + (xh > yh ? xh : yh) + sizeof(c64) * N;
    }
    static constexpr bool YH_TURNS = KS > 1 && NW == 4 && lds_with_copies(KS) > 53 * 1024 && lds_with_copies(1) <= 53 * 1024;
    static constexpr int YH_COPIES = YH_TURNS ? 1 : KS;
    static constexpr size_t LDS_YH = DIRECT ? 0 : sizeof(c64) * YH_COPIES * 32 * YROW;
    static constexpr size_t LDS_TW = sizeof(c64) * N;               // twiddles w_N^(t p), laid out [t][p] (static)
    static constexpr size_t LDS_DYN = LDS_Z + (LDS_XH > LDS_YH ? LDS_XH : LDS_YH);   // dynamic part
    static constexpr size_t LDS_BYTES = LDS_DYN + LDS_TW;
    static_assert(K % P == 0 && Q >= 1 && Q <= T && T % Q == 0, "K must be a multiple of P that divides N");
    static_assert(RPW % PPW == 0, "a wave inverts RPW rows of a 32-output slab, PPW at a time");
    static_assert(!WIDE || BF, "the eight-wave kernel exists with the BF16 contraction only");
    static_assert(PPI % 8 == 0, "an iteration is a whole number of 8-channel MFMA steps");
    static_assert(TPW <= KT && KT % TPW == 0, "a wave's tiles share one 32-output slab");
    static_assert(TPW * 32 <= 128, "accumulators must fit the register file");
    static_assert(KS == 1 || (BF && TILES * KS <= NW && (PPI / 8) % KS == 0),
                  "the channel steps of a block are split over waves that would otherwise hold no tile");
    static constexpr bool FITS = LDS_BYTES <= 160 * 1024;           // LDS budget of one gfx950 CU
    // Two workgroups per CU (two waves per SIMD, 256 registers each) wherever the accumulators leave room and LDS
    // allows: left to itself the compiler takes more than 256 registers for TPW = 2 and halves the occupancy.
    // Four for the single-operand-tile form of N = 64 with one output tile (118 registers).
    // Three for N = 64 where LDS allows it and the split contraction has shrunk the weight registers (K <= 32: 174
    // registers without the bound, no spills with it; the 16-point slices of N = 256 spill about 100 bytes).
    static constexpr int MIN_WG_PER_CU = (NW == 4 && XB == 1 && P <= 8 && OT == 1 && LDS_BYTES <= 40 * 1024) ? 4
                                         : (NW == 4 && ((KS > 1 && P <= 8) || XB == 1) && LDS_BYTES <= 53 * 1024) ? 3
                                         : (NW == 4 && (TPW <= 2 || WIDE || OT == 8) && LDS_BYTES <= 80 * 1024) ? 2 : 1;
};

// KS for a slab with fewer tiles than the workgroup has waves: as many waves per tile as there are spare waves and
// 8-channel steps in a block (1 = every wave has a tile of its own anyway).  Measured on MI355X, unsplit -> split:
// B 4096, C 64, N 128, K 32: 151 -> 118 us; B 8192, C 64, N 64, K 16: 196 -> 139 us; B 8192, C 32, N 64: 97 -> 58 us;
// B 512, C 32, N 256, K 64: 15.5 -> 13.9 us; B 2048, C 32, N 512, K 64: 140 -> 131 us.
template <int N, int K, int OT, int NW = 4>
constexpr int split_steps_over_waves()
{
    using C1 = FusedCfg<N, K, OT, true, NW, NW == 8 ? 1 : 2>;
    constexpr int steps = C1::PPI / 8, spare = C1::TILES < NW ? NW / C1::TILES : 1;
    return spare < steps ? spare : steps;
}

// Orders this wave's LDS traffic (all lanes) without a workgroup barrier.
__device__ __forceinline__ void wave_sync()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// EVEN: C_in is a multiple of PPI and C_out a multiple of 32 OT, so no load or store needs a mask.
// MODE 0: fully fused.  MODE 1: FFT + CGEMM (Sec. 4.1), the accumulators leave as the truncated output spectrum
// a.Yh.  MODE 2: CGEMM + iFFT (Sec. 4.2), the operand tiles come from the truncated input spectrum a.Xh.
// REAL (MODE 0 only): the real-valued layer.  a.x and a.y point to float32 tensors (strides in floats); the forward
// transform of a real pencil is the complex one with a zero imaginary part, whose first K bins are the R2C bins;
// the C2R inverse of the zero-padded half spectrum is (2/N) Re( sum_k Y'[k] e^(+2 pi i k n / N) ) with Y'[0] = Y[0]/2,
// so bin 0 is halved on its way into the operand tile, the caller passes scale = 2/N, and only real parts are stored.
template <int N, int K, int OT, bool EVEN, bool BF, int MODE = 0, bool REAL = false, int NW = 4, int XB = 2, int KS = 1>
__global__ void __launch_bounds__((FusedCfg<N, K, OT, BF, NW, XB, KS>::NT), (FusedCfg<N, K, OT, BF, NW, XB, KS>::MIN_WG_PER_CU))
k_fused1d(Fused1dArgs a)
{
    using C = FusedCfg<N, K, OT, BF, NW, XB, KS>;
    static_assert(!C::WIDE || (MODE == 0 && !REAL), "the eight-wave kernel is the fully fused complex layer only");
    static_assert(KS == 1 || MODE != 1, "partial accumulators meet in the inverse transform's LDS tile");
    static_assert(C::FITS, "LDS budget of one gfx950 CU");
    constexpr int NWV = C::NWV;
    constexpr int P = C::P, T = C::T, Q = C::Q, PPW = C::PPW, PPI = C::PPI, CPL = C::CPL, KT = C::KT;
    constexpr int KPAD = C::KPAD, TPW = C::TPW, ZROW = C::ZROW, ZS = C::ZS, YROW = C::YROW, NT = C::NT;
    constexpr bool ALLT = C::ALLT;

    extern __shared__ __align__(16) unsigned char lds_raw[];
    c64 *Zl = reinterpret_cast<c64 *>(lds_raw);                       // [NW][PPW][ZS]
    float *XH = reinterpret_cast<float *>(lds_raw + C::LDS_Z);        // [XB][PPI][2][KPAD]
    c64 *YH = reinterpret_cast<c64 *>(lds_raw + C::LDS_Z);            // [32][YROW]   (aliases XH)
    // the twiddle table is a separate LDS object so that its reads are known not to alias the Z/XH writes
    __shared__ c64 TW[N];                                             // [T][P]: w_N^(t p)

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    // (N = 1024 only: one workgroup per CU and 1 MiB rows; with several small workgroups per CU the mapping measured
    // up to 10 % slower)
    const int bb = N == 1024 ? (int)xcd_contiguous(blockIdx.x, gridDim.x) : (int)blockIdx.x;
    const int o_base = blockIdx.y * (32 * OT);

    const long long bo = bb / a.inner_count, bi = bb % a.inner_count;
    using XT = std::conditional_t<REAL, float, c64>;        // element type of x and y in global memory
    static_assert(!REAL || MODE == 0, "the real-valued layer exists for the fully fused kernel only");
    const XT *__restrict__ xb = reinterpret_cast<const XT *>(a.x) + bo * a.x_outer_stride + bi * a.x_inner_stride;
    XT *__restrict__ yb = reinterpret_cast<XT *>(a.y) + bo * a.y_outer_stride + bi * a.y_inner_stride;
    auto widen = [](XT e) __attribute__((always_inline)) {
        if constexpr (REAL) return make_float2(e, 0.f);
        else return e;
    };
    auto fetch = [](const XT *q) __attribute__((always_inline)) {
        // (non-temporal where measured to help: the real-valued layer at N = 1024, 96 -> 88 us on the cfg3 shape; at
        // N = 256 it made no difference or cost 3 %)
        if constexpr (REAL && N == 1024) return __builtin_nontemporal_load(q);
        else return *q;
    };
    // stage-A identity of this lane; twiddles w_N^(t p) = exp(-2 pi i t p / N) live in LDS as [t][p]
    // (stage-B lanes read consecutive p: conflict-free), computed once per workgroup with accurate sincospi
    const int jw = lane / T, t = lane % T;
    const int ja = wave * PPW + jw;
    c64 *Zw = Zl + wave * (PPW * ZS);
    // (called once the first loads are on their way: the table is built while they are in flight)
    auto build_twiddles = [&]() __attribute__((always_inline)) {
        __builtin_amdgcn_sched_barrier(0);
        for (int i = tid; i < N; i += NT) TW[i] = cis2pi(-(float)((i / P) * (i % P)), (float)N);
        __syncthreads();
    };

    // MFMA tile identity of this wave: tiles tile0 .. tile0+TPW-1, all in output slab `ot_w`; with KS > 1 one tile,
    // shared with KS - 1 other waves, of which this one takes the 8-channel steps s KS + part
    const int tile0 = KS > 1 ? wave / KS : wave * TPW;
    const int part = KS > 1 ? wave % KS : 0;
    const bool has_tiles = ALLT || tile0 < C::TILES;
    const int ot_w = tile0 / KT, kt0 = tile0 % KT;
    floatx16 acc_re[TPW], acc_im[TPW];
#pragma unroll
    for (int i = 0; i < TPW; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) { acc_re[i][r] = 0.f; acc_im[i][r] = 0.f; }

    const int o_lane = o_base + 32 * ot_w + (lane & 31);   // the output channel whose W this lane feeds
    const bool hi = lane >= 32;
    const int n_it = (a.C_in + PPI - 1) / PPI;

    c64 v[P];       // the pencil slice this lane transforms next
    // W[c][o_lane] for the channels of the iteration whose MFMAs run next: all PPI of them (FP32 MFMA), or, for
    // the BF16 path, the four channels 8 s + 4 (lane / 32) + d of every 8-channel step s, at index 4 s + d
    c64 wv[NWV];
    auto wv_channel = [&](int i) __attribute__((always_inline)) {
        return BF ? 8 * ((i / 4) * KS + part) + 4 * (lane >> 5) + (i % 4) : i;
    };

    auto load_pencil = [&](int c0) __attribute__((always_inline)) {
        const int c = c0 + ja;
        if constexpr (EVEN) {
            const XT *src = xb + (long long)c * a.x_chan_stride + t;
#pragma unroll
            for (int jj = 0; jj < P; ++jj) v[jj] = widen(fetch(src + T * jj));
        } else {
            const bool ok = c < a.C_in;
            const XT *src = xb + (long long)(ok ? c : 0) * a.x_chan_stride + t;
#pragma unroll
            for (int jj = 0; jj < P; ++jj) {
                c64 val = widen(fetch(src + T * jj));
                v[jj] = ok ? val : make_float2(0.f, 0.f);
            }
        }
    };
    auto load_w = [&](c64 *dst, int c0) __attribute__((always_inline)) {
#pragma unroll
        for (int jc = 0; jc < NWV; ++jc) {
            const int c = c0 + wv_channel(jc);
            if constexpr (EVEN && ALLT) {
                dst[jc] = a.W[(long long)c * a.C_out + o_lane];
            } else {
                const bool ok = has_tiles && c < a.C_in && o_lane < a.C_out;
                c64 val = a.W[ok ? (long long)c * a.C_out + o_lane : 0];
                dst[jc] = ok ? val : make_float2(0.f, 0.f);
            }
        }
    };
    // spectrum value of (channel slot jg of the block, mode k) into an operand tile
    const int k_keep = a.K_keep > 0 ? a.K_keep : K;
    auto put_operand = [&](float *XHb, int jg, int k, c64 val) __attribute__((always_inline)) {
        if constexpr (REAL) {
            const float h = k == 0 ? 0.5f : 1.0f;           // exact: the split below sees the halved value
            val = make_float2(val.x * h, val.y * h);
        }
        if constexpr (BF) {
            unsigned *d = reinterpret_cast<unsigned *>(XHb) + (jg >> 2) * (KT * 128) + (jg & 3) + (k >> 5) * 128 + (k & 31) * 4;
            const Split3 re = split3(val.x), im = split3(val.y);
            d[0 * (PPI / 4) * KT * 128] = pack_bf16(re.t0, im.t0);
            d[1 * (PPI / 4) * KT * 128] = pack_bf16(re.t1, im.t1);
            d[2 * (PPI / 4) * KT * 128] = pack_bf16(re.t2, im.t2);
        } else {
            XHb[(jg * 2 + 0) * KPAD + k] = val.x;
            XHb[(jg * 2 + 1) * KPAD + k] = val.y;
        }
    };
    // stage A: P-point transform of the slice in v, written transposed into the wave's Z tile
    auto stage_a = [&]() __attribute__((always_inline)) {
        c64 z[P];
        RegFFT<P, -1, 1>::run(v, z);
#pragma unroll
        for (int p = 0; p < P; ++p) Zw[jw * ZS + p * ZROW + t] = z[p];
    };
    // stage B: twiddle, T-point transform pruned to the Q retained outputs of each column, into XH[buf]
    auto stage_b = [&](int buf) __attribute__((always_inline)) {
        float *XHb = XH + buf * C::XH_BUF;
#pragma unroll
        for (int cc = 0; cc < CPL; ++cc) {
            const int item = lane + 64 * cc;
            const int j = item / P, p = item % P;
            const c64 *zcol = Zw + j * ZS + p * ZROW;
            c64 xo[Q];
            if constexpr (T <= 16 && (C::TPW <= 1 || (C::WIDE && C::TPW <= 2))) {
                // all LDS reads of the column are issued before the first use: left alone, the compiler reads,
                // waits and multiplies one pair at a time (T exposed LDS round trips per column)
                c64 zc[T], tw[T];
#pragma unroll
                for (int tt = 0; tt < T; ++tt) {
                    zc[tt] = zcol[tt];
                    if (tt != 0) tw[tt] = TW[tt * P + p];
                }
                __builtin_amdgcn_sched_barrier(0);
                dft_prune_out<T, Q, -1>([&](auto ttc) __attribute__((always_inline)) {
                    constexpr int tt = decltype(ttc)::value;
                    if constexpr (tt == 0) return zc[0];
                    else return cmul(zc[tt], tw[tt]);
                }, xo);
            } else {
                dft_prune_out<T, Q, -1>([&](auto ttc) __attribute__((always_inline)) {
                    constexpr int tt = decltype(ttc)::value;
                    if constexpr (tt == 0) return zcol[0];
                    else return cmul(zcol[tt], TW[tt * P + p]);
                }, xo);
            }
            const int jg = wave * PPW + j;
#pragma unroll
            for (int q = 0; q < Q; ++q) put_operand(XHb, jg, p + P * q, xo[q]);
            // truncation finer than the kernel's K: the surplus bins enter the contraction as zeros.  (A uniform
            // branch that overwrites them; masking every value costs the full-K case 3-5 %.)
            if (k_keep < K) {
#pragma unroll
                for (int q = 0; q < Q; ++q)
                    if (p + P * q >= k_keep) put_operand(XHb, jg, p + P * q, make_float2(0.f, 0.f));
            }
        }
    };
    // complex MAC on the matrix cores (channels past C_in carry zero spectra and zero weights)
    auto mfma_block = [&](int buf) __attribute__((always_inline)) {
        const float *XHb = XH + buf * C::XH_BUF;
        if constexpr (BF) {
            // 8 channels per v_mfma_f32_32x32x16_bf16: lanes 0-31 carry channels 0-3 of the step, lanes 32-63
            // channels 4-7, dword d = (re | im << 16) of channel 4 g + d.  Six products per tile and part; the
            // accumulators of the wave's tiles are interleaved (a dependent MFMA issues about four slots later).
            const unsigned *XS = reinterpret_cast<const unsigned *>(XHb) + (hi ? 1 : 0) * (KT * 128) + kt0 * 128 + (lane & 31) * 4;
#pragma unroll
            for (int s = 0; s < PPI / 8 / KS; ++s) {
                uintx4 a_re[3], a_im[3];
#pragma unroll
                for (int d = 0; d < 4; ++d) {
                    const Split3 re = split3(wv[4 * s + d].x * a.scale), im = split3(wv[4 * s + d].y * a.scale);
                    a_re[0][d] = pack_bf16(re.t0, im.t0) ^ 0x80000000u;
                    a_re[1][d] = pack_bf16(re.t1, im.t1) ^ 0x80000000u;
                    a_re[2][d] = pack_bf16(re.t2, im.t2) ^ 0x80000000u;
                    a_im[0][d] = pack_bf16(im.t0, re.t0);
                    a_im[1][d] = pack_bf16(im.t1, re.t1);
                    a_im[2][d] = pack_bf16(im.t2, re.t2);
                }
                uintx4 b[TPW][3];
#pragma unroll
                for (int i = 0; i < TPW; ++i)
#pragma unroll
                    for (int t = 0; t < 3; ++t)
                        b[i][t] = *reinterpret_cast<const uintx4 *>(XS + ((t * (PPI / 4) + 2 * (s * KS + part)) * KT + i) * 128);
                // smallest products first: (2,0) (0,2) (1,1) (1,0) (0,1) (0,0)
                constexpr int SA[6] = {2, 0, 1, 1, 0, 0}, SB[6] = {0, 2, 1, 0, 1, 0};
#pragma unroll
                for (int k = 0; k < 6; ++k)
#pragma unroll
                    for (int i = 0; i < TPW; ++i) {
                        const bf16x8 bb16 = __builtin_bit_cast(bf16x8, b[i][SB[k]]);
                        acc_re[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a_re[SA[k]]), bb16, acc_re[i], 0, 0, 0);
                        acc_im[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a_im[SA[k]]), bb16, acc_im[i], 0, 0, 0);
                    }
            }
        } else {
#pragma unroll
            for (int jc = 0; jc < PPI; ++jc) {
                const float a_re = (hi ? -wv[jc].y : wv[jc].x) * a.scale;
                const float a_im = (hi ? wv[jc].x : wv[jc].y) * a.scale;
#pragma unroll
                for (int i = 0; i < TPW; ++i) {
                    const float bx = XHb[(jc * 2 + (hi ? 1 : 0)) * KPAD + 32 * (kt0 + i) + (lane & 31)];
                    acc_re[i] = __builtin_amdgcn_mfma_f32_32x32x2f32(a_re, bx, acc_re[i], 0, 0, 0);
                    acc_im[i] = __builtin_amdgcn_mfma_f32_32x32x2f32(a_im, bx, acc_im[i], 0, 0, 0);
                }
            }
        }
    };
    // Eight-wave kernel: the contraction of one block from the single operand tile, the weights of the whole block in
    // wv.  Global loads complete in issue order, so a wait for a weight that was fetched after a block of pencil loads
    // would also wait for those pencils (HBM latency): the weights of a block are therefore fetched at the start of
    // its stage B, BEFORE the pencil loads that are issued next, and every wait meets loads a whole phase old.
    auto mfma_block_wide = [&]() __attribute__((always_inline)) {
        const unsigned *XS = reinterpret_cast<const unsigned *>(XH) + (hi ? 1 : 0) * (KT * 128) + kt0 * 128 + (lane & 31) * 4;
        // tile-step n = (8-channel step n / TPW, tile n % TPW): its three B operands are read from LDS while the MFMAs
        // of tile-step n-1 run
        auto read_b = [&](uintx4 *b, int n) __attribute__((always_inline)) {
#pragma unroll
            for (int t = 0; t < 3; ++t)
                b[t] = *reinterpret_cast<const uintx4 *>(XS + ((t * (PPI / 4) + 2 * ((n / TPW) * KS + part)) * KT + n % TPW) * 128);
        };
        uintx4 b[2][3];
        read_b(b[0], 0);
#pragma unroll
        for (int s = 0; s < PPI / 8 / KS; ++s) {
            uintx4 a_re[3], a_im[3];
#pragma unroll
            for (int d = 0; d < 4; ++d) {
                const Split3 re = split3(wv[4 * s + d].x * a.scale), im = split3(wv[4 * s + d].y * a.scale);
                a_re[0][d] = pack_bf16(re.t0, im.t0) ^ 0x80000000u;
                a_re[1][d] = pack_bf16(re.t1, im.t1) ^ 0x80000000u;
                a_re[2][d] = pack_bf16(re.t2, im.t2) ^ 0x80000000u;
                a_im[0][d] = pack_bf16(im.t0, re.t0);
                a_im[1][d] = pack_bf16(im.t1, re.t1);
                a_im[2][d] = pack_bf16(im.t2, re.t2);
            }
            constexpr int SA[6] = {2, 0, 1, 1, 0, 0}, SB[6] = {0, 2, 1, 0, 1, 0};   // smallest products first
#pragma unroll
            for (int i = 0; i < TPW; ++i) {
                const int n = s * TPW + i;
                if (n + 1 < (PPI / 8 / KS) * TPW) read_b(b[(n + 1) & 1], n + 1);
#pragma unroll
                for (int k = 0; k < 6; ++k) {
                    const bf16x8 bb16 = __builtin_bit_cast(bf16x8, b[n & 1][SB[k]]);
                    acc_re[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a_re[SA[k]]), bb16, acc_re[i], 0, 0, 0);
                    acc_im[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a_im[SA[k]]), bb16, acc_im[i], 0, 0, 0);
                }
            }
        }
    };
    // One block of the eight-wave kernel: weights of block `it`, stage B of block `it` into the single operand tile,
    // barrier, then stage A of block it+1 (into the wave's Z tile, free again), the loads of block it+2, and the
    // contraction of block `it`; the closing barrier frees the operand tile for the next block.
    auto wide_step = [&](auto do_a, auto do_load, int it) __attribute__((always_inline)) {
        constexpr bool DO_A = decltype(do_a)::value, DO_LOAD = decltype(do_load)::value;
        // (scheduling fences: left alone, the compiler sinks stage A into the MFMA sequence and the pencil loads
        // behind the closing barrier, which leaves them one stage B to arrive instead of a whole contraction)
        load_w(wv, it * PPI);
        stage_b(0);
        wave_sync();
        __syncthreads();
        if constexpr (DO_A) { stage_a(); wave_sync(); }
        __builtin_amdgcn_sched_barrier(0);
        if constexpr (DO_LOAD) load_pencil((it + 2) * PPI);
        __builtin_amdgcn_sched_barrier(0);
        if constexpr (ALLT) mfma_block_wide();
        else if (has_tiles) mfma_block_wide();
        __builtin_amdgcn_sched_barrier(0);
        if constexpr (DO_A) __syncthreads();
    };

    // One k-loop iteration, software pipelined three deep: the MFMAs of block `it` run next to stage B of
    // block it+1 (from the Z tile written one iteration earlier) and stage A of block it+2, and the loads of
    // block it+3 are issued as soon as v is free, so they are in flight for a whole iteration.
    auto step = [&](auto do_b, auto do_a, auto do_load, int it) __attribute__((always_inline)) {
        constexpr bool DO_B = decltype(do_b)::value, DO_A = decltype(do_a)::value, DO_LOAD = decltype(do_load)::value;
        const int cur = it & 1;
        c64 wn[NWV];
        if constexpr (DO_B) load_w(wn, (it + 1) * PPI);
        if constexpr (ALLT) mfma_block(cur);
        else if (has_tiles) mfma_block(cur);
        if constexpr (DO_B) { stage_b(cur ^ 1); wave_sync(); }
        if constexpr (DO_A) { stage_a(); wave_sync(); }
        if constexpr (DO_LOAD) load_pencil((it + 3) * PPI);
        if constexpr (DO_B) {
#pragma unroll
            for (int jc = 0; jc < NWV; ++jc) wv[jc] = wn[jc];
            __syncthreads();
        }
    };
    const std::true_type yes{};
    const std::false_type no{};

    // ------------------------------------------------------------------ k-loop over input channels
    if constexpr (C::WIDE) {
        load_pencil(0);
        build_twiddles();
        stage_a();
        wave_sync();
        if (n_it > 1) load_pencil(PPI);
        int it = 0;
        for (; it + 2 < n_it; ++it) wide_step(yes, yes, it);
        if (it + 1 < n_it) { wide_step(yes, no, it); ++it; }
        wide_step(no, no, it);
    } else if constexpr (MODE != 2) {
        load_pencil(0);
        load_w(wv, 0);
        build_twiddles();
        stage_a();
        wave_sync();
        if (n_it > 1) load_pencil(PPI);
        stage_b(0);
        wave_sync();
        if (n_it > 1) {
            stage_a();
            wave_sync();
            if (n_it > 2) load_pencil(2 * PPI);
        }
        __syncthreads();
        {
            int it = 0;
            for (; it + 3 < n_it; ++it) step(yes, yes, yes, it);
            const int left = n_it - it;   // 1, 2 or 3
            if (left == 3) {
                step(yes, yes, no, it);
                step(yes, no, no, it + 1);
                step(no, no, no, it + 2);
            } else if (left == 2) {
                step(yes, no, no, it);
                step(no, no, no, it + 1);
            } else {
                step(no, no, no, it);
            }
        }
    } else {
        // CGEMM + iFFT: every thread moves K/T spectrum values per block from a.Xh into the operand tile, two
        // blocks ahead of the MFMAs (registers, then LDS); consecutive threads read consecutive modes.
        constexpr int NSV = K / T;
        static_assert(NSV * NT == PPI * K, "a block of spectrum values divides evenly over the workgroup");
        c64 sv[NSV];
        auto load_spec = [&](int c0) __attribute__((always_inline)) {
#pragma unroll
            for (int e = 0; e < NSV; ++e) {
                const int idx = tid + NT * e, k = idx % K, c = c0 + idx / K;
                const long long m = (long long)bb * K + k;
                const bool ok = EVEN || c < a.C_in;
                const c64 val = a.Xh[((m >> 7) * a.C_in + (ok ? c : 0)) * 128 + (m & 127)];
                sv[e] = ok ? val : make_float2(0.f, 0.f);
            }
        };
        auto put_spec = [&](int buf) __attribute__((always_inline)) {
#pragma unroll
            for (int e = 0; e < NSV; ++e) {
                const int idx = tid + NT * e;
                put_operand(XH + buf * C::XH_BUF, idx / K, idx % K, sv[e]);
            }
        };
        auto sstep = [&](auto do_put, auto do_load, int it) __attribute__((always_inline)) {
            constexpr bool DO_PUT = decltype(do_put)::value, DO_LOAD = decltype(do_load)::value;
            c64 wn[NWV];
            if constexpr (DO_PUT) load_w(wn, (it + 1) * PPI);
            if constexpr (ALLT) mfma_block(it & 1);
            else if (has_tiles) mfma_block(it & 1);
            if constexpr (DO_PUT) put_spec((it & 1) ^ 1);
            if constexpr (DO_LOAD) load_spec((it + 2) * PPI);
            if constexpr (DO_PUT) {
#pragma unroll
                for (int jc = 0; jc < NWV; ++jc) wv[jc] = wn[jc];
                __syncthreads();
            }
        };
        load_spec(0);
        load_w(wv, 0);
        build_twiddles();
        put_spec(0);
        if (n_it > 1) load_spec(PPI);
        __syncthreads();
        int it = 0;
        for (; it + 2 < n_it; ++it) sstep(yes, yes, it);
        if (it + 1 < n_it) { sstep(yes, no, it); ++it; }
        sstep(no, no, it);
    }
    // ------------------------------------------------------------------ epilogue
    if constexpr (MODE == 1) {
        // FFT + CGEMM: register r of lane l of tile i holds Yh[o][k] for o = 8(r/4) + 4(l/32) + r%4 of the wave's
        // slab and k = 32 (kt0 + i) + l%32; a half-wave writes 32 consecutive modes of one output channel
        if (has_tiles) {
#pragma unroll
            for (int i = 0; i < TPW; ++i) {
                const int k = 32 * (kt0 + i) + (lane & 31);
                if (k < K) {
                    const long long m = (long long)bb * K + k;
                    c64 *dst = a.Yh + (m >> 7) * a.C_out * 128 + (m & 127);
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const int o = o_base + 32 * ot_w + 8 * (r / 4) + 4 * (lane >> 5) + (r % 4);
                        if (EVEN || o < a.C_out) dst[(long long)o * 128] = make_float2(acc_re[i][r], acc_im[i][r]);
                    }
                }
            }
        }
        return;
    }
    // stage B' for Z slot `slot`, column p: zero-padded, input-pruned T-point inverse transform of the Q
    // retained modes in yin, conj twiddle, written transposed into the wave's Z tile
    auto stage_b_inv = [&](const c64 *yin, int slot, int p) __attribute__((always_inline)) {
        c64 *zcol = Zw + slot * ZS + p * ZROW;
        dft_prune_in<T, Q, +1>(yin, [&](auto ttc, c64 val) __attribute__((always_inline)) {
            constexpr int tt = decltype(ttc)::value;
            if constexpr (tt == 0) zcol[0] = val;
            else {
                c64 w = TW[tt * P + p];
                zcol[tt] = cmul(val, make_float2(w.x, -w.y));
            }
        });
    };
    // stage A' for the pencil in Z slot jw of this wave: P-point inverse transform, store
    auto ifft_store = [&](int o) __attribute__((always_inline)) {
        c64 z[P], r[P];
#pragma unroll
        for (int p = 0; p < P; ++p) z[p] = Zw[jw * ZS + p * ZROW + t];
        RegFFT<P, +1, 1>::run(z, r);
        if (EVEN || o < a.C_out) {
            XT *dst = yb + (long long)o * a.y_chan_stride + t;
#pragma unroll
            for (int jj = 0; jj < P; ++jj) {
                if constexpr (REAL) __builtin_nontemporal_store(r[jj].x, dst + T * jj);
                else store_nt(dst + T * jj, r[jj]);
            }
        }
    };

    if constexpr (C::DIRECT) {
        // Wave w owns outputs o_base + 32 w .. +31 for every mode tile.  Register r of lane l of tile q holds
        // Yh[o][p + 32 q] with p = l%32 and o = 8(r/4) + 4(l/32) + r%4: exactly the Q inputs that lane
        // (half-wave h = l/32, column p) needs for stage B' of that pencil.
        constexpr int RPA = C::RPA;
        const int p = lane & 31, h = lane >> 5;
        for (int rr = 0; rr < 16; rr += RPA) {
#pragma unroll
            for (int sub = 0; sub < RPA; ++sub) {
                const int r = rr + sub;
                c64 yin[Q];
                static_for<0, 16>([&](auto rc) {
                    constexpr int R = decltype(rc)::value;
                    if (r == R) {
#pragma unroll
                        for (int q = 0; q < Q; ++q) yin[q] = make_float2(acc_re[q][R], acc_im[q][R]);
                    }
                });
                stage_b_inv(yin, 2 * sub + h, p);
            }
            wave_sync();
            const int r2 = rr + jw / 2;
            ifft_store(o_base + 32 * wave + 8 * (r2 / 4) + 4 * (jw % 2) + (r2 % 4));
            wave_sync();
        }
    } else {
        __syncthreads();   // every wave is done reading XH, which YH aliases
        for (int ot = 0; ot < OT; ++ot) {
            // accumulator layout of the 32x32 MFMA: register r of lane l holds
            //   row (output)  8*(r/4) + 4*(l/32) + r%4,   column (mode) l%32
            if constexpr (C::YH_TURNS) {
                for (int turn = 0; turn < KS; ++turn) {
                    if (has_tiles && ot == ot_w && part == turn) {
#pragma unroll
                        for (int i = 0; i < TPW; ++i) {
                            const int k = 32 * (kt0 + i) + (lane & 31);
                            if (k < K) {
#pragma unroll
                                for (int r = 0; r < 16; ++r) {
                                    const int ol = 8 * (r / 4) + 4 * (lane >> 5) + (r % 4);
                                    c64 v2 = make_float2(acc_re[i][r], acc_im[i][r]);
                                    if (turn != 0) v2 = cadd(v2, YH[ol * YROW + k]);
                                    YH[ol * YROW + k] = v2;
                                }
                            }
                        }
                    }
                    __syncthreads();
                }
            } else {
                if (has_tiles && ot == ot_w) {
#pragma unroll
                    for (int i = 0; i < TPW; ++i) {
                        const int k = 32 * (kt0 + i) + (lane & 31);
                        if (k < K) {
#pragma unroll
                            for (int r = 0; r < 16; ++r) {
                                const int ol = 8 * (r / 4) + 4 * (lane >> 5) + (r % 4);
                                YH[(part * 32 + ol) * YROW + k] = make_float2(acc_re[i][r], acc_im[i][r]);
                            }
                        }
                    }
                }
                __syncthreads();
            }
            // wave w inverts rows RPW w .. RPW w + RPW - 1 of the slab, PPW pencils per round, in its private Z tile
            for (int rd = 0; rd < C::RPW / PPW; ++rd) {
#pragma unroll
                for (int cc = 0; cc < CPL; ++cc) {
                    const int item = lane + 64 * cc;
                    const int j = item / P, p = item % P;
                    const int ol = C::RPW * wave + rd * PPW + j;
                    c64 yin[Q];
#pragma unroll
                    for (int q = 0; q < Q; ++q) {
                        yin[q] = YH[ol * YROW + p + P * q];
#pragma unroll
                        for (int ks = 1; ks < C::YH_COPIES; ++ks) yin[q] = cadd(yin[q], YH[(ks * 32 + ol) * YROW + p + P * q]);
                    }
                    stage_b_inv(yin, j, p);
                }
                wave_sync();
                ifft_store(o_base + 32 * ot + C::RPW * wave + rd * PPW + jw);
                wave_sync();
            }
            __syncthreads();
        }
    }
}

template <int N, int K, int OT, bool BF, int MODE = 0, bool REAL = false, int NW = 4, int XB = 2, int KS = 1>
hipError_t launch_fused1d_impl(const Fused1dArgs &a, long long batch_rows, hipStream_t s)
{
    using C = FusedCfg<N, K, OT, BF, NW, XB, KS>;
    static LdsLimitOnce lds_limit;
    const hipError_t e = lds_limit.set({reinterpret_cast<const void *>(&k_fused1d<N, K, OT, true, BF, MODE, REAL, NW, XB, KS>),
                                        reinterpret_cast<const void *>(&k_fused1d<N, K, OT, false, BF, MODE, REAL, NW, XB, KS>)},
                                       (int)C::LDS_DYN);
    if (e != hipSuccess) return e;
    dim3 grid((unsigned)batch_rows, (unsigned)((a.C_out + 32 * OT - 1) / (32 * OT)));
    // unmasked kernel only when every workgroup's slab of 32 OT outputs exists in full
    if (a.C_in % C::PPI == 0 && a.C_out % (32 * OT) == 0)
        hipLaunchKernelGGL((k_fused1d<N, K, OT, true, BF, MODE, REAL, NW, XB, KS>), grid, dim3(C::NT), C::LDS_DYN, s, a);
    else
        hipLaunchKernelGGL((k_fused1d<N, K, OT, false, BF, MODE, REAL, NW, XB, KS>), grid, dim3(C::NT), C::LDS_DYN, s, a);
    return hipGetLastError();
}

// Output slab of a workgroup, in units of 32 channels: as wide as C_out needs (one workgroup then transforms the
// batch row once for all its outputs), but narrower when that would leave at least half of the 256 CUs without a
// workgroup: the extra forward transforms run on CUs that would idle (B 64, C 64, N 256: 16.0 -> 14.6 us).
inline int pick_output_tiles(int C_out, long long rows, int max_ot)
{
    int ot = C_out > 64 ? 4 : C_out > 32 ? 2 : 1;
    if (ot > max_ot) ot = max_ot;
    while (ot > 1 && rows * ((C_out + 32 * ot - 1) / (32 * ot)) * 2 <= 256) ot >>= 1;
    return ot;
}

// Real-valued layer: fully fused kernel, output slab (32 OT channels, OT <= MAXOT) chosen by C_out as for the
// complex kernel; BF16x3 contraction wherever the packed operand tile fits.
template <int N, int K, int OT>
hipError_t launch_fused1d_real_ot(const Fused1dArgs &a, long long rows, hipStream_t s)
{
    if constexpr (FusedCfg<N, K, OT, true>::FITS) {
        constexpr int KS = split_steps_over_waves<N, K, OT>();
        if (!contraction_forced_f32()) {
            if constexpr (FusedCfg<N, K, OT, true, 4, 2, KS>::FITS) return launch_fused1d_impl<N, K, OT, true, 0, true, 4, 2, KS>(a, rows, s);
            else return launch_fused1d_impl<N, K, OT, true, 0, true>(a, rows, s);
        }
    }
    return launch_fused1d_impl<N, K, OT, false, 0, true>(a, rows, s);
}
template <int N, int K, int MAXOT>
hipError_t launch_fused1d_real(const Fused1dArgs &a, long long rows, hipStream_t s)
{
    const int ot = pick_output_tiles(a.C_out, rows, MAXOT);
    if constexpr (MAXOT >= 4) {
        if (ot == 4) return launch_fused1d_real_ot<N, K, 4>(a, rows, s);
    }
    if (ot >= 2) return launch_fused1d_real_ot<N, K, 2>(a, rows, s);
    return launch_fused1d_real_ot<N, K, 1>(a, rows, s);
}

// Partially fused variant MODE (1 or 2) for every K built, workgroup slab chosen by C_out as for the fused kernel
template <int N, int K, int MODE>
hipError_t launch_partial_k(const Fused1dArgs &a, long long rows, hipStream_t s)
{
    // (the FFT + CGEMM kernel writes its accumulators straight to the spectrum: no split there)
    constexpr int KS2 = MODE == 2 ? split_steps_over_waves<N, K, 2>() : 1, KS1 = MODE == 2 ? split_steps_over_waves<N, K, 1>() : 1;
    if (a.C_out > 64) return launch_fused1d_impl<N, K, 4, true, MODE>(a, rows, s);
    if (a.C_out > 32) return launch_fused1d_impl<N, K, 2, true, MODE, false, 4, 2, KS2>(a, rows, s);
    return launch_fused1d_impl<N, K, 1, true, MODE, false, 4, 2, KS1>(a, rows, s);
}
template <int N, int MODE>
hipError_t launch_partial(int K, const Fused1dArgs &a, long long rows, hipStream_t s)
{
    switch (K) {
    case 32: return launch_partial_k<N, 32, MODE>(a, rows, s);
    case 64: return launch_partial_k<N, 64, MODE>(a, rows, s);
    case 128: return launch_partial_k<N, 128, MODE>(a, rows, s);
    default: return hipErrorInvalidValue;
    }
}

// Single-operand-tile kernels (BF16x3 contraction only): NW = 8 waves in one workgroup, or NW = 4 with two workgroups per CU
template <int N, int K, int OT, int NW = 8, int KS = 1>
hipError_t launch_fused1d_wide(const Fused1dArgs &a, long long batch_rows, hipStream_t s)
{
    static_assert(FusedCfg<N, K, OT, true, NW, 1, KS>::FITS, "LDS budget of one gfx950 CU");
    return launch_fused1d_impl<N, K, OT, true, 0, false, NW, 1, KS>(a, batch_rows, s);
}

// BF16x3 contraction unless the environment asks for FP32 MFMA (TFNO_CONTRACTION=f32)
template <int N, int K, int OT>
hipError_t launch_fused1d(const Fused1dArgs &a, long long batch_rows, hipStream_t s)
{
    // (the packed three-term operand tile is 1.5x the FP32 one; the largest shapes only fit with FP32 operands)
    if constexpr (FusedCfg<N, K, OT, true>::FITS) {
        constexpr int KS = split_steps_over_waves<N, K, OT>();
        if (!contraction_forced_f32()) {
            if constexpr (FusedCfg<N, K, OT, true, 4, 2, KS>::FITS) return launch_fused1d_impl<N, K, OT, true, 0, false, 4, 2, KS>(a, batch_rows, s);
            else return launch_fused1d_impl<N, K, OT, true>(a, batch_rows, s);
        }
    }
    return launch_fused1d_impl<N, K, OT, false>(a, batch_rows, s);
}

}  // namespace tfno
