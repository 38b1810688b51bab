// Fully fused FFT -> CGEMM -> iFFT kernel along the last (contiguous) axis (Sec. 4.3), for gfx950.
//
// Work decomposition (re-derived for wave64 / MFMA / 160 KB LDS; the idea kept from the paper is that one
// workgroup walks the hidden dimension in step with the GEMM k-loop, Sec. 2.3 / 4.1):
//
//   workgroup  = one batch row `bb` x one slab of 32*OT output channels, 256 threads (4 waves)
//   k-loop     : PPI = 256/T input channels per iteration.  N = P * T.
//     stage A  : thread (pencil j, t) loads x[c0+j][t + T*jj], jj < P (coalesced), P-point DFT in registers,
//                twiddle by w_N^(t p), writes column-major into LDS            Z[j][p][t]
//     stage B  : thread (pencil j, column p) reads Z[j][p][0..T), T-point DFT pruned to the Q = K/P outputs
//                that are retained modes k = p + P q < K (built-in truncation + output pruning, Sec. 3.3),
//                writes the planar A-operand tile                               XH[j][re|im][k]
//     MFMA     : Yh[o][k] += W[c][o] * Xh[c][k] with v_mfma_f32_32x32x2_f32: the two k-slots of one
//                instruction carry (re, im) of ONE channel, so a complex MAC over 32 outputs x 32 modes is
//                two MFMAs (real part with A = (W.re, -W.im), imaginary part with A = (W.im, W.re)).
//                Accumulators stay in registers for the whole k-loop.
//   epilogue   : per 32-output slab, accumulators -> LDS YH[o][k]; stage B' expands the K retained modes of
//                column p to T points (built-in zero padding + input pruning, Sec. 3.3), LDS Z, stage A'
//                applies conj twiddles, P-point inverse DFT, coalesced store of y.  The 1/N scale is folded
//                into W when it is loaded.
//
// LDS handoffs (the counterpart of the two swizzles of Sec. 4.1 / 4.2, re-derived for 4-byte banks and
// 8-byte accesses): Z rows are padded to T+1 complex so that both the write (consecutive t) and the
// transposed read (consecutive p, stride T+1) touch distinct banks; XH is planar so that an MFMA operand
// read is 32 consecutive floats per half-wave; YH rows are written 32 consecutive complex at a time straight
// from the MFMA accumulator layout.
#pragma once
#include "common.h"
#include "fft_regs.h"
#include "fused1d.h"

namespace tfno {

typedef float floatx16 __attribute__((ext_vector_type(16)));

template <int N> struct Decomp;
template <> struct Decomp<64>   { static constexpr int P = 8,  T = 8;  };
template <> struct Decomp<128>  { static constexpr int P = 16, T = 8;  };
template <> struct Decomp<256>  { static constexpr int P = 16, T = 16; };
template <> struct Decomp<512>  { static constexpr int P = 32, T = 16; };
template <> struct Decomp<1024> { static constexpr int P = 32, T = 32; };

template <int N, int K, int OT>
struct FusedCfg {
    static constexpr int P = Decomp<N>::P, T = Decomp<N>::T;
    static constexpr int Q = K / P;                 // retained outputs per column of stage B
    static constexpr int NT = 256, NW = 4;
    static constexpr int PPI = NT / T;              // pencils (channels) per k-loop iteration
    static constexpr int CPT = P / T;               // stage-B columns per thread
    static constexpr int KT = (K + 31) / 32;        // 32-mode MFMA tiles
    static constexpr int KPAD = KT * 32;
    static constexpr int TILES = OT * KT;
    static constexpr int TPW = (TILES + NW - 1) / NW;   // 32x32 complex tiles per wave
    static constexpr int ZROW = T + 1;
    static constexpr int ZS = P * ZROW + (T == 8 ? 8 - (P * ZROW) % 16 + ((P * ZROW) % 16 > 8 ? 16 : 0) : 0);
    static constexpr int YROW = K + 1;
    static constexpr size_t LDS_Z = sizeof(c64) * PPI * ZS;
    static constexpr size_t LDS_XH = sizeof(float) * PPI * 2 * KPAD;
    static constexpr size_t LDS_YH = sizeof(c64) * 32 * YROW;
    static constexpr size_t LDS_TW = sizeof(c64) * N;               // twiddles w_N^(t p), laid out [p][t]
    static constexpr size_t LDS_BYTES = LDS_Z + (LDS_XH > LDS_YH ? LDS_XH : LDS_YH) + LDS_TW;
    static_assert(K % P == 0 && Q >= 1 && Q <= T && T % Q == 0, "K must be a multiple of P that divides N");
    static_assert(PPI <= 32 && 32 % PPI == 0, "epilogue slabs are 32 outputs");
    static_assert(TPW <= KT && KT % TPW == 0, "a wave's tiles share one 32-output slab");
    static_assert(TPW * 32 <= 128, "accumulators must fit the register file");
};

template <int N, int K, int OT>
__global__ void __launch_bounds__(256)
k_fused1d(Fused1dArgs a)
{
    using C = FusedCfg<N, K, OT>;
    constexpr int P = C::P, T = C::T, Q = C::Q, PPI = C::PPI, CPT = C::CPT, KT = C::KT, KPAD = C::KPAD;
    constexpr int TPW = C::TPW, ZROW = C::ZROW, ZS = C::ZS, YROW = C::YROW, NT = C::NT;

    extern __shared__ __align__(16) unsigned char lds_raw[];
    c64 *Zl = reinterpret_cast<c64 *>(lds_raw);                       // [PPI][ZS]
    float *XH = reinterpret_cast<float *>(lds_raw + C::LDS_Z);        // [PPI][2][KPAD]
    c64 *YH = reinterpret_cast<c64 *>(lds_raw + C::LDS_Z);            // [32][YROW]   (aliases XH)
    const c64 *TW = reinterpret_cast<const c64 *>(lds_raw + C::LDS_BYTES - C::LDS_TW);   // [P][T]

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int bb = blockIdx.x;
    const int o_base = blockIdx.y * (32 * OT);

    const long long bo = bb / a.inner_count, bi = bb % a.inner_count;
    const c64 *__restrict__ xb = a.x + bo * a.x_outer_stride + bi * a.x_inner_stride;
    c64 *__restrict__ yb = a.y + bo * a.y_outer_stride + bi * a.y_inner_stride;

    // stage-A identity of this thread; twiddles w_N^(t p) = exp(-2 pi i t p / N) live in LDS as [p][t]
    // (consecutive t: conflict-free reads), computed once per workgroup with accurate sincospi
    const int ja = tid / T, t = tid % T;
    {
        c64 *twr = reinterpret_cast<c64 *>(lds_raw + C::LDS_BYTES - C::LDS_TW);
        for (int i = tid; i < N; i += NT) twr[i] = cis2pi(-(float)((i / T) * (i % T)), (float)N);
    }
    __syncthreads();

    // MFMA tile identity of this wave: tiles tile0 .. tile0+TPW-1, all in output slab `ot_w`
    const int tile0 = wave * TPW;
    const bool has_tiles = tile0 < C::TILES;
    const int ot_w = tile0 / KT, kt0 = tile0 % KT;
    floatx16 acc_re[TPW], acc_im[TPW];
#pragma unroll
    for (int i = 0; i < TPW; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) { acc_re[i][r] = 0.f; acc_im[i][r] = 0.f; }

    const int o_lane = o_base + 32 * ot_w + (lane & 31);   // the output channel whose W this lane feeds
    const bool hi = lane >= 32;

    // ------------------------------------------------------------------ k-loop over input channels
    c64 v[P];
    auto load_pencil = [&](int c0) {
        const int c = c0 + ja;
        if (c < a.C_in) {
            const c64 *src = xb + (long long)c * a.x_chan_stride + t;
#pragma unroll
            for (int jj = 0; jj < P; ++jj) v[jj] = src[T * jj];
        } else {
#pragma unroll
            for (int jj = 0; jj < P; ++jj) v[jj] = make_float2(0.f, 0.f);
        }
    };

    load_pencil(0);
    for (int c0 = 0; c0 < a.C_in; c0 += PPI) {
        // W rows of this iteration's channels: issued first so that their latency hides behind the
        // transforms.  Lanes 0-31 and 32-63 read the same 32 outputs (the two k-slots of the MFMA).
        c64 wv[PPI];
#pragma unroll
        for (int jc = 0; jc < PPI; ++jc) {
            wv[jc] = make_float2(0.f, 0.f);
            if (has_tiles && c0 + jc < a.C_in && o_lane < a.C_out)
                wv[jc] = a.W[(long long)(c0 + jc) * a.C_out + o_lane];
        }
        // stage A
        {
            c64 z[P];
            RegFFT<P, -1, 1>::run(v, z);
#pragma unroll
            for (int p = 0; p < P; ++p) {
                c64 zz = p == 0 ? z[0] : cmul(z[p], TW[p * T + t]);
                Zl[ja * ZS + p * ZROW + t] = zz;
            }
        }
        // v is consumed: fetch the next iteration's pencils now, in flight during stage B and the MFMAs
        if (c0 + PPI < a.C_in) load_pencil(c0 + PPI);
        __syncthreads();
        // stage B
#pragma unroll
        for (int cc = 0; cc < CPT; ++cc) {
            const int item = tid + NT * cc;
            const int j = item / P, p = item % P;
            c64 zt[T], xo[Q];
#pragma unroll
            for (int tt = 0; tt < T; ++tt) zt[tt] = Zl[j * ZS + p * ZROW + tt];
            dft_prune_out<T, Q, -1>(zt, xo);
#pragma unroll
            for (int q = 0; q < Q; ++q) {
                XH[(j * 2 + 0) * KPAD + p + P * q] = xo[q].x;
                XH[(j * 2 + 1) * KPAD + p + P * q] = xo[q].y;
            }
        }
        __syncthreads();
        // complex MAC on the matrix cores (channels past C_in carry zero spectra and zero weights)
        if (has_tiles) {
#pragma unroll
            for (int jc = 0; jc < PPI; ++jc) {
                const float a_re = (hi ? -wv[jc].y : wv[jc].x) * a.scale;
                const float a_im = (hi ? wv[jc].x : wv[jc].y) * a.scale;
#pragma unroll
                for (int i = 0; i < TPW; ++i) {
                    const float bx = XH[(jc * 2 + (hi ? 1 : 0)) * KPAD + 32 * (kt0 + i) + (lane & 31)];
                    acc_re[i] = __builtin_amdgcn_mfma_f32_32x32x2f32(a_re, bx, acc_re[i], 0, 0, 0);
                    acc_im[i] = __builtin_amdgcn_mfma_f32_32x32x2f32(a_im, bx, acc_im[i], 0, 0, 0);
                }
            }
        }
        // the next iteration's barriers order these XH reads before XH is rewritten
    }
    __syncthreads();

    // ------------------------------------------------------------------ epilogue: per 32-output slab
    for (int ot = 0; ot < OT; ++ot) {
        if (has_tiles && ot == ot_w) {
            // accumulator layout of the 32x32 MFMA: register r of lane l holds
            //   row (output)  8*(r/4) + 4*(l/32) + r%4,   column (mode) l%32
#pragma unroll
            for (int i = 0; i < TPW; ++i) {
                const int k = 32 * (kt0 + i) + (lane & 31);
                if (k < K) {
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const int ol = 8 * (r / 4) + 4 * (lane >> 5) + (r % 4);
                        YH[ol * YROW + k] = make_float2(acc_re[i][r], acc_im[i][r]);
                    }
                }
            }
        }
        __syncthreads();
        for (int it = 0; it < 32 / PPI; ++it) {
            // stage B': zero-padded, input-pruned T-point inverse transform of column p
#pragma unroll
            for (int cc = 0; cc < CPT; ++cc) {
                const int item = tid + NT * cc;
                const int j = item / P, p = item % P;
                const int ol = it * PPI + j;
                c64 yin[Q], u[T];
#pragma unroll
                for (int q = 0; q < Q; ++q) yin[q] = YH[ol * YROW + p + P * q];
                dft_prune_in<T, Q, +1>(yin, u);
#pragma unroll
                for (int tt = 0; tt < T; ++tt) Zl[j * ZS + p * ZROW + tt] = u[tt];
            }
            __syncthreads();
            // stage A': conj twiddle, P-point inverse transform, store
            {
                c64 z[P], r[P];
#pragma unroll
                for (int p = 0; p < P; ++p) {
                    c64 zz = Zl[ja * ZS + p * ZROW + t];
                    c64 w = TW[p * T + t];
                    z[p] = p == 0 ? zz : cmul(zz, make_float2(w.x, -w.y));
                }
                RegFFT<P, +1, 1>::run(z, r);
                const int o = o_base + 32 * ot + it * PPI + ja;
                if (o < a.C_out) {
                    c64 *dst = yb + (long long)o * a.y_chan_stride + t;
#pragma unroll
                    for (int jj = 0; jj < P; ++jj) dst[T * jj] = r[jj];
                }
            }
            __syncthreads();
        }
    }
}

template <int N, int K, int OT>
hipError_t launch_fused1d(const Fused1dArgs &a, long long batch_rows, hipStream_t s)
{
    using C = FusedCfg<N, K, OT>;
    static bool attr_done = false;   // benign race: every thread sets the same value
    if (!attr_done) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&k_fused1d<N, K, OT>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)C::LDS_BYTES);
        if (e != hipSuccess) return e;
        attr_done = true;
    }
    dim3 grid((unsigned)batch_rows, (unsigned)((a.C_out + 32 * OT - 1) / (32 * OT)));
    hipLaunchKernelGGL((k_fused1d<N, K, OT>), grid, dim3(256), C::LDS_BYTES, s, a);
    return hipGetLastError();
}

}  // namespace tfno
