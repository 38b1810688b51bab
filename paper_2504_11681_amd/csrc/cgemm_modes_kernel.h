// Complex GEMM over the retained modes of a truncated spectrum in mode-tile-major layout (the contraction step of
// Sec. 3.1 with one W shared by every mode), used between the 2-D image kernels and by the unfused 1-D variants.
#pragma once
#include "common.h"
#include "fft_regs.h"         // static_for
#include "fused1d_kernel.h"   // wave_sync, floatx16
#include "bf16x3.h"

namespace tfno {

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

// The same contraction with ALL of W resident in LDS, for 64 < C_in <= 128 (96 KB as three BF16 terms): the looped
// kernel above restages a 64-channel block of W twice per mode tile, with the L2 round trip of its loads and four
// barriers exposed every time, which is half of its run time at C_in = 128.  Here eight waves share one copy of W,
// staged once; after that no wave meets a barrier: wave w walks the 32 modes 32 (w % 4) of tiles tile0 + 2 t + w / 4,
// its loads four 8-channel steps ahead across tile boundaries.
__global__ void __launch_bounds__(512)
k_cgemm_modes_resident(const c64 *__restrict__ Xh, const c64 *__restrict__ W, c64 *__restrict__ Yh,
                       int C_in, int C_out, float scale, long long num_tiles, int pairs_per_wg)
{
    extern __shared__ __align__(16) unsigned Wres[];        // [channel / 4][term][output][channel % 4], c_pad channels
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int col = lane & 31, g = lane >> 5;
    const int o0 = blockIdx.y * 64;
    const long long tile0 = (long long)blockIdx.x * 2 * pairs_per_wg;
    const int c_pad = (C_in + 31) / 32 * 32;
    // tiles of this wave: tile0 + 2 t + wave / 4, t < nt_w
    const long long first = tile0 + (wave >> 2);
    const int nt_w = first >= num_tiles ? 0 : (int)((num_tiles - first + 1) / 2 < pairs_per_wg ? (num_tiles - first + 1) / 2 : pairs_per_wg);

    const int rot = 8 * (int)(blockIdx.x & 7);              // see the looped kernel: spreads the memory channels
    auto rotated = [&](int c_lin) __attribute__((always_inline)) {
        const int cb = c_lin & ~63, left = C_in - cb, lim = left >= 64 ? 64 : (left + 31) / 32 * 32;
        return cb + ((c_lin - cb + rot) & (lim - 1));
    };
    int nt = 0, nc = 0;
    auto load_next = [&](c64 *xv) __attribute__((always_inline)) {
        // (past this wave's last tile the first one is read again and never used; a wave without tiles reads tile 0)
        const long long ti = nt_w > 0 ? first + 2 * (nt < nt_w ? nt : 0) : 0;
        const c64 *src = Xh + ti * C_in * 128 + 32 * (wave & 3) + col;
        const int c0 = rotated(nc);
#pragma unroll
        for (int d = 0; d < 4; ++d) {
            const int c = c0 + 4 * g + d;
            xv[d] = src[(c < C_in ? c : 0) * 128];
        }
        nc += 8;
        if (nc >= c_pad) { nc = 0; ++nt; }
    };
    c64 xq[4][4];
    {
        // W first: its staging is on every wave's critical path, the first steps of X are not
        c64 wq[16];
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const int idx = i * 512 + tid, c = idx / 64, o = o0 + idx % 64;
            const bool ok = c < C_in && o < C_out;
            const c64 w = W[ok ? (long long)c * C_out + o : 0];
            wq[i] = ok ? w : make_float2(0.f, 0.f);
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int i = 0; i < 4; ++i) load_next(xq[i]);       // in flight while W is staged
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const int idx = i * 512 + tid, cl = idx / 64, ol = idx % 64;
            if (cl < c_pad) {
                const Split3 re = split3(wq[i].x * scale), im = split3(wq[i].y * scale);
                unsigned *dst = Wres + (((cl >> 2) * 3) * 64 + ol) * 4 + (cl & 3);
                dst[0 * 64 * 4] = pack_bf16(re.t0, im.t0);
                dst[1 * 64 * 4] = pack_bf16(re.t1, im.t1);
                dst[2 * 64 * 4] = pack_bf16(re.t2, im.t2);
            }
        }
    }
    __syncthreads();                                        // the only barrier: W is resident

    // W operands of a step: [output half][term], read one step ahead of their MFMAs (the LDS round trip of six
    // 16-byte reads would otherwise sit between every step's split and its MFMAs)
    const int nsteps = c_pad / 8;
    uintx4 wbuf[2][2][3];
    auto read_w = [&](uintx4 (*w)[3], int step) __attribute__((always_inline)) {
        const int c0 = rotated(8 * step);
        const unsigned *wsrc = Wres + (((c0 >> 2) + g) * 3 * 64 + col) * 4;
#pragma unroll
        for (int sl = 0; sl < 2; ++sl)
#pragma unroll
            for (int tm = 0; tm < 3; ++tm) w[sl][tm] = *reinterpret_cast<const uintx4 *>(wsrc + (tm * 64 + 32 * sl) * 4);
    };
    read_w(wbuf[0], 0);

    floatx16 acc_re[2], acc_im[2];
    for (int t = 0; t < nt_w; ++t) {
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r) { acc_re[i][r] = 0.f; acc_im[i][r] = 0.f; }
#pragma unroll 1
        for (int s4 = 0; s4 < nsteps; s4 += 4) {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                uintx4 b[3];
#pragma unroll
                for (int d = 0; d < 4; ++d) {
                    const Split3 re = split3(xq[i][d].x), im = split3(xq[i][d].y);
                    b[0][d] = pack_bf16(re.t0, im.t0);
                    b[1][d] = pack_bf16(re.t1, im.t1);
                    b[2][d] = pack_bf16(re.t2, im.t2);
                }
                __builtin_amdgcn_sched_barrier(0);
                load_next(xq[i]);                           // four steps ahead
                read_w(wbuf[(i + 1) & 1], s4 + i + 1 < nsteps ? s4 + i + 1 : 0);
                __builtin_amdgcn_sched_barrier(0);
                constexpr int SA[6] = {2, 0, 1, 1, 0, 0}, SB[6] = {0, 2, 1, 0, 1, 0};   // smallest products first
#pragma unroll
                for (int sl = 0; sl < 2; ++sl) {
                    uintx4 a_re[3], a_im[3];
#pragma unroll
                    for (int tm = 0; tm < 3; ++tm)
#pragma unroll
                        for (int d = 0; d < 4; ++d) {
                            const unsigned w = wbuf[i & 1][sl][tm][d];
                            a_re[tm][d] = w ^ 0x80000000u;
                            a_im[tm][d] = __builtin_amdgcn_alignbit(w, w, 16);
                        }
#pragma unroll
                    for (int k = 0; k < 6; ++k) {
                        const bf16x8 bb = __builtin_bit_cast(bf16x8, b[SB[k]]);
                        acc_re[sl] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a_re[SA[k]]), bb, acc_re[sl], 0, 0, 0);
                        acc_im[sl] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a_im[SA[k]]), bb, acc_im[sl], 0, 0, 0);
                    }
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        c64 *__restrict__ Yb = Yh + (first + 2 * t) * C_out * 128 + 32 * (wave & 3) + col;
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
    {
        // W first: its staging is on every wave's critical path, the first tile of X is not
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
        for (int i = 0; i < NSTEP; ++i) load_step(0, i);    // in flight while W is staged
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
