// Contraction over the hidden dimension with an own weight matrix per retained mode (the learned transformation of
// the Fourier layer as the FNO model defines it, Sec. 1 / Sec. 2.1 step 3; Sec. 3.1 treats the case of one shared
// matrix, which the MFMA kernels of cgemm_modes_kernel.h cover):
//
//   Yh[b, o, m] = scale * sum_c Xh[b, c, m] * W[c, o, m]
//
// on spectra in the mode-tile-major layout ([tile][channel][128 modes]).  There is no matrix shared between modes,
// so nothing maps onto an MFMA tile without gathering one mode's values across the batch; the kernel instead keeps
// a thread per mode (all global accesses are 128 consecutive modes of one channel: coalesced for Xh, W and Yh) and
// reuses registers: a thread accumulates BT batch elements x OT outputs, so every W value loaded is used BT times
// and every Xh value OT times.  Tiles t with the same t % TPI hold the same modes (TPI = tiles per batch element,
// or 1 when several batch elements share a tile), which is what lets one W value serve BT tiles.
// W is [C_in, C_out, K1a, K2a] for the modes actually kept; the spectra may be laid out for more (see below).
#pragma once
#include "common.h"

namespace tfno {

template <int BT, int OT>
__global__ void __launch_bounds__(256, 2)
k_cgemm_permode(const c64 *__restrict__ Xh, const c64 *__restrict__ W, c64 *__restrict__ Yh, int C_in, int C_out,
                int M, long long num_tiles, int TPI, float scale, int K2p, int K1a, int K2a)
{
    const int tid = threadIdx.x, i = tid & 127, half = tid >> 7;
    const int r = (int)(blockIdx.x % (unsigned)TPI);
    const long long grp = blockIdx.x / (unsigned)TPI;
    const int m = (r * 128 + i) % M;                        // the mode this thread owns in every tile it visits
    // The spectra are laid out for K1p x K2p modes (M = K1p K2p, the built kernel sizes), W for the K1a x K2a modes
    // actually kept.  Surplus modes hold zeros in Xh; they read a clamped (valid) weight.
    const int k1 = m / K2p, k2 = m % K2p;
    const int Ma = K1a * K2a;
    const int wm = (k1 < K1a ? k1 : K1a - 1) * K2a + (k2 < K2a ? k2 : K2a - 1);
    const int o0 = ((int)blockIdx.y * 2 + half) * OT;

    const c64 *xp[BT];
    bool tv[BT];
#pragma unroll
    for (int bi = 0; bi < BT; ++bi) {
        const long long t = r + (long long)TPI * (grp * BT + bi);
        tv[bi] = t < num_tiles;
        xp[bi] = Xh + ((tv[bi] ? t : r) * C_in) * 128 + i;   // tile r exists and holds the same modes
    }
    const c64 *wp[OT];
#pragma unroll
    for (int oi = 0; oi < OT; ++oi) {
        const int o = o0 + oi < C_out ? o0 + oi : C_out - 1;
        wp[oi] = W + (long long)o * Ma + wm;
    }
    const long long wstep = (long long)C_out * Ma;

    c64 acc[BT][OT];
#pragma unroll
    for (int bi = 0; bi < BT; ++bi)
#pragma unroll
        for (int oi = 0; oi < OT; ++oi) acc[bi][oi] = make_float2(0.f, 0.f);

#pragma unroll 2
    for (int c = 0; c < C_in; ++c) {
        c64 xv[BT], wv[OT];
#pragma unroll
        for (int oi = 0; oi < OT; ++oi) wv[oi] = wp[oi][c * wstep];
#pragma unroll
        for (int bi = 0; bi < BT; ++bi) xv[bi] = xp[bi][(long long)c * 128];
#pragma unroll
        for (int bi = 0; bi < BT; ++bi)
#pragma unroll
            for (int oi = 0; oi < OT; ++oi) acc[bi][oi] = cmac(acc[bi][oi], xv[bi], wv[oi]);
    }

#pragma unroll
    for (int bi = 0; bi < BT; ++bi) {
        if (!tv[bi]) continue;
        const long long t = r + (long long)TPI * (grp * BT + bi);
        c64 *yp = Yh + (t * C_out) * 128 + i;
#pragma unroll
        for (int oi = 0; oi < OT; ++oi)
            if (o0 + oi < C_out) yp[(long long)(o0 + oi) * 128] = make_float2(acc[bi][oi].x * scale, acc[bi][oi].y * scale);
    }
}

}  // namespace tfno
