// Per-mode contraction on the matrix pipe (the learned transformation of the Fourier layer as the FNO model defines
// it, Sec. 1 / Sec. 2.1 step 3: an own weight matrix for every retained mode):
//
//   Yh[b, o, m] = scale * sum_c Xh[b, c, m] * W[c, o, m]
//
// With a matrix per mode nothing is shared between modes, so the MFMA tile is one mode's product
// [32 batch elements x C_in] . [C_in x 32 outputs]: the batch is the M dimension.  The spectra are mode-tile major
// ([tile][channel][128 modes]), i.e. one mode's values lie 1 KB apart, so a workgroup takes EIGHT consecutive modes
// (64-byte pieces of every row it reads or writes) and goes through LDS:
//
//   workgroup = 8 modes of one tile residue x 32 batch elements x 32 outputs, 256 threads, two or three per CU
//   k-loop over 8-channel steps: the Xh and W values of the step are fetched two steps ahead, split exactly into three
//     BF16 terms (bf16x3.h; the scale is folded into W) and stored as MFMA operands
//       XS / WS [term][mode][channel / 4][batch or output][channel % 4]     (dword = re | im << 16)
//     with row strides chosen so that the stores of a wave hit 64 distinct banks and the 16-byte operand reads of a
//     quarter wave cover all banks; wave w contracts modes 2w and 2w+1: per mode three operand reads each side,
//     the sign flip / half swap that turns the stored (re, im) pairs into the real-part and imaginary-part operands
//     (A = (re, -im) and A = (im, re) against B = (re, im)), and 12 v_mfma_f32_32x32x16_bf16 (six products per part).
//   epilogue: accumulators -> LDS [batch][output][mode] in two halves of 16 batch elements -> 64-byte row stores.
//
// Built for spectra whose mode count is a multiple of 128 (every tile holds 128 modes of one batch element); other
// layouts keep the FP32 kernel of cgemm_permode_kernel.h.
#pragma once
#include "common.h"
#include "bf16x3.h"

namespace tfno {

typedef float pm_floatx16 __attribute__((ext_vector_type(16)));

struct PermodeMfma {
    static constexpr int MB = 8;                // modes per workgroup
    static constexpr int HS = 136;              // dwords between the two channel halves of a mode  (= 8 mod 64)
    static constexpr int MS = 264;              // dwords between modes                              (= 8 mod 64)
    static constexpr int TS = MB * MS;          // dwords between terms
    static constexpr int TILE = 3 * TS;         // dwords of one operand tile (25.3 KB)
    static constexpr int YROW = 9;              // c64 per (batch, output) row of the epilogue tile (8 modes + 1 pad)
    static_assert(16 * 32 * YROW * 2 <= 2 * TILE, "the epilogue tile aliases the operand tiles");
};

// FULL: 32 batch elements, 32 outputs and a multiple of 8 channels per workgroup -- no masks, and every row is
// addressed as a uniform pointer plus one lane offset.
template <bool FULL>
__global__ void __launch_bounds__(256, 2)
k_cgemm_permode_mfma(const c64 *__restrict__ Xh, const c64 *__restrict__ W, c64 *__restrict__ Yh, int C_in, int C_out,
                     int M, long long num_tiles, int TPI, float scale, int K2p, int K1a, int K2a)
{
    using P = PermodeMfma;
    constexpr int MB = P::MB, HS = P::HS, MS = P::MS, TS = P::TS;
    __shared__ __align__(16) unsigned lds[2 * P::TILE];
    unsigned *XS = lds, *WS = lds + P::TILE;
    c64 *YS = reinterpret_cast<c64 *>(lds);     // epilogue: [16 batch][32 outputs][YROW]

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    // The sixteen workgroups that share the 128-byte lines of a tile (8 modes = half a line each) get consecutive
    // places on ONE XCD, so the second half of a line is an L2 hit (workgroup ids go round-robin over the XCDs: with
    // the identity mapping neighbours sit on different L2s and every line crosses the fabric twice).
    const unsigned bx = xcd_contiguous(blockIdx.x, gridDim.x);
    const int r = (int)(bx / 16u), i0 = (int)(bx % 16u) * MB;                    // tile residue, first mode within the tile
    const long long per = (num_tiles - r + TPI - 1) / TPI;                      // tiles that hold these modes
    const long long b0 = 32LL * blockIdx.y;                                     // first of the 32 batch-like tiles
    const int o0 = 32 * (int)blockIdx.z;
    const int Ma = K1a * K2a;

    // ---- staging identity, Xh: lane = (mode pair q, channel c % 4, channel half, batch parity); wave and pass pick b / 2
    const int xq = lane & 3, xcq = (lane >> 2) & 3, xch = (lane >> 4) & 1, xbl = lane >> 5;
    // ---- staging identity, W: lane = (mode, channel c % 4, output parity); wave and pass pick channel half and o / 2
    const int wm_ = lane & 7, wcq = (lane >> 3) & 3, wol = lane >> 5;
    // the weight of this lane's mode: W is laid out for the K1a x K2a modes kept, the spectra for M = K1p K2p modes
    // (surplus modes hold zeros in Xh and read a clamped, valid weight)
    int w_mode;
    {
        const int m = (r * 128 + i0 + wm_) % M, k1 = m / K2p, k2 = m % K2p;
        w_mode = (k1 < K1a ? k1 : K1a - 1) * K2a + (k2 < K2a ? k2 : K2a - 1);
    }

    // Two steps of values are in flight (one step of MFMAs is shorter than the memory latency): set s & 1 belongs to step s.
    // Xh: pass p holds batch 2 (4 p + wave) + xbl, channel 4 xch + xcq, modes 2 xq, 2 xq + 1;
    // W: pass p holds channel 4 ((4 p + wave) % 2) + wcq, output 2 ((4 p + wave) / 2) + wol.
    // Row pointers are set up once (rows outside the problem point at a valid row and are zeroed after the load);
    // a step adds a constant to them: per-load 64-bit address arithmetic was a third of the kernel's instructions.
    constexpr int D = 2;                        // steps of values in flight (three measured no faster)
    uintx4 xr2[D][4];
    c64 wr2[D][8];
    const uintx4 *xrow[4];
    bool xok[4];
#pragma unroll
    for (int p = 0; p < 4; ++p) {
        const long long b = b0 + 2 * (4 * p + wave) + xbl;
        xok[p] = b < per;
        const long long t = r + (long long)TPI * (xok[p] ? b : 0);
        xrow[p] = reinterpret_cast<const uintx4 *>(Xh + (t * C_in + 4 * xch + xcq) * 128 + i0 + 2 * xq);
    }
    const c64 *wrow[8];
    bool wok[8];
#pragma unroll
    for (int p = 0; p < 8; ++p) {
        const int combo = 4 * p + wave, o = o0 + 2 * (combo >> 1) + wol;
        wok[p] = o < C_out;
        wrow[p] = W + ((long long)(4 * (combo & 1) + wcq) * C_out + (wok[p] ? o : 0)) * Ma + w_mode;
    }
    const long long wstep = (long long)C_out * Ma;      // one channel further in W
    const bool c_even = C_in % 8 == 0;                  // no channel masks needed
    // FULL: batch 2 (4 p + wave) + xbl = 8 p + 2 wave + xbl; channel 4 (wave % 2) + wcq, output 4 p + 2 (wave / 2) + wol
    const int bstride = TPI * C_in * 64;                                        // uintx4 between batch elements
    const uintx4 *xbase = reinterpret_cast<const uintx4 *>(Xh + ((r + (long long)TPI * b0) * C_in) * 128 + i0) + 2 * wave * bstride;
    const c64 *wbase = W + ((long long)(4 * (wave & 1)) * C_out + o0 + 2 * (wave >> 1)) * Ma;
    const unsigned xlane = (unsigned)((xbl * TPI * C_in + 4 * xch + xcq) * 64 + xq);
    const unsigned wlane = (unsigned)((wcq * C_out + wol) * Ma + w_mode);
    auto fetch = [&](uintx4 *xr, c64 *wr, int c0) __attribute__((always_inline)) {
        if constexpr (FULL) {
            const uintx4 *xs = xbase + c0 * 64;
            const c64 *ws = wbase + (size_t)c0 * (size_t)wstep;
#pragma unroll
            for (int p = 0; p < 4; ++p) xr[p] = xs[xlane + (unsigned)(8 * p * bstride)];
#pragma unroll
            for (int p = 0; p < 8; ++p) wr[p] = ws[wlane + (unsigned)(4 * p * Ma)];
        } else {
            const bool cx = c_even || c0 + 4 * xch + xcq < C_in;
#pragma unroll
            for (int p = 0; p < 4; ++p) {
                const uintx4 v = xrow[p][cx ? (long long)c0 * 64 : 0];          // 64 uintx4 = 128 c64 per channel
                xr[p] = (cx && xok[p]) ? v : uintx4{0u, 0u, 0u, 0u};
            }
#pragma unroll
            for (int p = 0; p < 8; ++p) {
                const bool cw = c_even || c0 + 4 * ((4 * p + wave) & 1) + wcq < C_in;
                const c64 v = wrow[p][cw ? c0 * wstep : 0];
                wr[p] = (cw && wok[p]) ? v : make_float2(0.f, 0.f);
            }
        }
    };
    auto put3 = [&](unsigned *d, float re_, float im_) __attribute__((always_inline)) {
        const Split3 re = split3(re_), im = split3(im_);
        d[0] = pack_bf16(re.t0, im.t0);
        d[TS] = pack_bf16(re.t1, im.t1);
        d[2 * TS] = pack_bf16(re.t2, im.t2);
    };
    auto stage = [&](const uintx4 *xr, const c64 *wr) __attribute__((always_inline)) {
#pragma unroll
        for (int p = 0; p < 4; ++p) {
            unsigned *d = XS + (2 * xq) * MS + xch * HS + (2 * (4 * p + wave) + xbl) * 4 + xcq;
            put3(d, __uint_as_float(xr[p][0]), __uint_as_float(xr[p][1]));
            put3(d + MS, __uint_as_float(xr[p][2]), __uint_as_float(xr[p][3]));
        }
#pragma unroll
        for (int p = 0; p < 8; ++p) {
            const int combo = 4 * p + wave;
            unsigned *d = WS + wm_ * MS + (combo & 1) * HS + (2 * (combo >> 1) + wol) * 4 + wcq;
            put3(d, wr[p].x * scale, wr[p].y * scale);
        }
    };

    pm_floatx16 acc_re[2], acc_im[2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int k = 0; k < 16; ++k) { acc_re[i][k] = 0.f; acc_im[i][k] = 0.f; }

    const int n_steps = (C_in + 7) / 8;
#pragma unroll
    for (int e = 0; e < D; ++e) fetch(xr2[e], wr2[e], 8 * (e < n_steps ? e : n_steps - 1));
    // (steps in pairs so that the register set of a step is a compile-time choice; past the end a fetch repeats the
    // last step and is dropped)
    for (int s2 = 0; s2 < n_steps; s2 += D) {
#pragma unroll
      for (int e = 0; e < D; ++e) {
        const int s = s2 + e;
        if (s >= n_steps) break;
        stage(xr2[e], wr2[e]);
        __builtin_amdgcn_sched_barrier(0);
        fetch(xr2[e], wr2[e], 8 * (s + D < n_steps ? s + D : n_steps - 1));
        __builtin_amdgcn_sched_barrier(0);
        __syncthreads();
        const unsigned *xa = XS + (lane >> 5) * HS + (lane & 31) * 4, *wb = WS + (lane >> 5) * HS + (lane & 31) * 4;
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int m = 2 * wave + i;
            uintx4 a_re[3], a_im[3], b[3];
#pragma unroll
            for (int t = 0; t < 3; ++t) {
                const uintx4 v = *reinterpret_cast<const uintx4 *>(xa + t * TS + m * MS);
                b[t] = *reinterpret_cast<const uintx4 *>(wb + t * TS + m * MS);
#pragma unroll
                for (int d = 0; d < 4; ++d) {
                    a_re[t][d] = v[d] ^ 0x80000000u;                    // (re, -im)
                    a_im[t][d] = __builtin_amdgcn_alignbit(v[d], v[d], 16);   // (im, re)
                }
            }
            constexpr int SA[6] = {2, 0, 1, 1, 0, 0}, SB[6] = {0, 2, 1, 0, 1, 0};   // smallest products first
#pragma unroll
            for (int k = 0; k < 6; ++k) {
                const bf16x8 bb16 = __builtin_bit_cast(bf16x8, b[SB[k]]);
                acc_re[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a_re[SA[k]]), bb16, acc_re[i], 0, 0, 0);
                acc_im[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a_im[SA[k]]), bb16, acc_im[i], 0, 0, 0);
            }
        }
        __syncthreads();
      }
    }

    // ---- epilogue.  Register R of lane l of tile i holds Yh for batch 8 (R / 4) + 4 (l / 32) + R % 4, output l % 32,
    // mode 2 wave + i.  Two halves of 16 batch elements go through LDS so that every (batch, output) row leaves as
    // 64 contiguous bytes.
#pragma unroll
    for (int hb = 0; hb < 2; ++hb) {
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int R = 8 * hb; R < 8 * hb + 8; ++R) {
                const int bl = 8 * ((R / 4) & 1) + 4 * (lane >> 5) + (R % 4);       // batch within the half
                YS[(bl * 32 + (lane & 31)) * P::YROW + 2 * wave + i] = make_float2(acc_re[i][R], acc_im[i][R]);
            }
        __syncthreads();
#pragma unroll
        for (int p = 0; p < 4; ++p) {
            const int row = 128 * p + (tid >> 1), half = tid & 1;       // row = (batch within the half, output); 4 modes per thread
            const int bl = row >> 5, o = o0 + (row & 31);
            const long long b = b0 + 16 * hb + bl;
            if (b < per && o < C_out) {
                const c64 *src = YS + row * P::YROW + 4 * half;
                const c64 y0 = src[0], y1 = src[1], y2 = src[2], y3 = src[3];
                uintx4 *dst = reinterpret_cast<uintx4 *>(Yh + ((r + (long long)TPI * b) * C_out + o) * 128 + i0 + 4 * half);
                dst[0] = uintx4{__float_as_uint(y0.x), __float_as_uint(y0.y), __float_as_uint(y1.x), __float_as_uint(y1.y)};
                dst[1] = uintx4{__float_as_uint(y2.x), __float_as_uint(y2.y), __float_as_uint(y3.x), __float_as_uint(y3.y)};
            }
        }
        __syncthreads();
    }
}

}  // namespace tfno
