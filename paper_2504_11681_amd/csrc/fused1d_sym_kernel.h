// Fused FFT -> CGEMM -> iFFT kernel for N = 1024 with eight symmetric waves (Sec. 4.3), gfx950.
//
//   workgroup = one batch row x 128 output channels, 512 threads = 8 waves, two per SIMD.
//   Every wave does the same work, so the VALU load of the transforms is spread evenly:
//     k-loop, 8 input channels per iteration (one pencil per wave), one barrier per iteration:
//       row stage of block i+1: a whole wave owns a pencil, lane p holds x[p + 64 j], j < 16 (512-byte coalesced
//         loads); 16-point DFT in registers, twiddle w_N^(p k_lo), transpose through a wave-private XOR-swizzled
//         LDS patch, then four lanes per column k_lo: 16-point DFT of every fourth patch entry pruned to the
//         K/16 retained outputs (Sec. 3.3), twiddle w_64^(a k_hi), sum over the quad with DPP; the retained bins
//         k = k_lo + 16 k_hi are split exactly into three BF16 terms and written as MFMA operands to XS
//         (double buffered).  The first butterfly level frees the load registers, so the loads of block i+2 are
//         issued right after it and stay in flight for a whole iteration.
//       contraction of block i: wave w owns outputs 32 (w/2) .. +31 and K/64 of the K/32 mode tiles;
//         v_mfma_f32_32x32x16_bf16 on operands split into three BF16 terms, six products per tile and part
//         (FP32-accurate, see bf16x3.h); four independent accumulators are interleaved because a dependent MFMA
//         can only issue about four issue slots after its predecessor.
//       Every wave runs the contraction first, then the transforms of the next block: the contraction does not
//       depend on the loads in flight, so the transforms wait for them as late as possible.
//     epilogue, 16 rounds of 8 output pencils (one per wave), one barrier per round: accumulators -> LDS (mode
//       order), twiddled zero-padded input-pruned column transform (Sec. 3.3) into the patch, 16-point inverse
//       row transform, 512-byte coalesced stores.  1/N is folded into W.
//   MFMA k index (16 per instruction) = 8 channels x (re, im): lanes 0-31 carry channels 0-3, lanes 32-63
//   channels 4-7; dword d of a lane = (re | im << 16) of channel 4g + d.  Real part: A = (W.re, -W.im), imaginary
//   part: A = (W.im, W.re).  Accumulator register r of lane l holds output 8(r/4) + 4(l/32) + r%4, mode l%32.
#pragma once
#include "common.h"
#include "fft_regs.h"
#include "fused1d.h"
#include "fused1d_kernel.h"   // wave_sync, floatx16
#include "bf16x3.h"

namespace tfno {

template <int K>
struct SymCfg {
    static constexpr int N = 1024, NT = 512, NW = 8, PPI = 8;
    static constexpr int KH = K / 16;               // retained k_hi per column k_lo
    static constexpr int KT = K / 32;               // 32-mode tiles
    static constexpr int TPW = KT / 2;              // mode tiles per wave
    static constexpr int OPL = KH / 4;              // retained bins per lane after the quad reduction
    static constexpr int PATCH = 16 * 64;           // complex elements of one wave's transpose patch
    static constexpr int XT = K == 128 ? 144 : 160; // dwords between mode tiles of the operand buffer (128 + pad, see row_stage)
    static constexpr int XS_BUF = 3 * 2 * KT * XT;  // dwords per operand buffer: [term][g][tile][d][n]
    static constexpr int YH_BUF = 8 * K;            // complex elements per spectrum buffer: [pencil][mode]
    static constexpr size_t LDS_PATCH = sizeof(c64) * NW * PATCH;
    static constexpr size_t LDS_XS = sizeof(unsigned) * 2 * XS_BUF;
    static constexpr size_t LDS_YH = sizeof(c64) * 2 * YH_BUF;
    static constexpr size_t LDS_DYN = LDS_PATCH + (LDS_XS > LDS_YH ? LDS_XS : LDS_YH);
    static_assert(K == 64 || K == 128, "K in {64, 128}");
    static_assert(LDS_DYN + sizeof(c64) * (N + 64) <= 160 * 1024, "LDS budget of one gfx950 CU");
};

template <int CTRL>
__device__ __forceinline__ float sym_quad_perm(float v)
{
    return __int_as_float(__builtin_amdgcn_mov_dpp(__float_as_int(v), CTRL, 0xf, 0xf, true));
}

// EVEN: C_in is a multiple of 8 and C_out a multiple of 128 (no masks).  DEEP: the number of 8-channel blocks
// is even and at least four; the k-loop then keeps two blocks of loads in flight per wave.
// REAL: the real-valued layer.  a.x and a.y point to float32 tensors (strides in floats); the forward transform of
// a real pencil is the complex one with a zero imaginary part, whose first K bins are the R2C bins; the C2R inverse of
// the zero-padded half spectrum is (2/N) Re( sum_k Y'[k] e^(+2 pi i k n / N) ) with Y'[0] = Y[0]/2, so bin 0 is halved
// on its way into the operand tile, the caller passes scale = 2/N, and only real parts are stored.
template <int K, bool EVEN, bool DEEP, bool REAL = false>
__global__ void __launch_bounds__(512)
k_fused1d_sym(Fused1dArgs a)
{
    using C = SymCfg<K>;
    constexpr int N = C::N, KH = C::KH, KT = C::KT, TPW = C::TPW, OPL = C::OPL, PPI = C::PPI;

    extern __shared__ __align__(16) unsigned char lds_raw[];
    c64 *patch_all = reinterpret_cast<c64 *>(lds_raw);                          // [8 waves][16][64]
    unsigned *XS = reinterpret_cast<unsigned *>(lds_raw + C::LDS_PATCH);         // [2][3][2][KT][32][4]
    c64 *YH = reinterpret_cast<c64 *>(lds_raw + C::LDS_PATCH);                   // [2][8][K]  (aliases XS)
    __shared__ c64 TW[N];                                                        // [k_lo][p]: w_N^(p k_lo)
    __shared__ c64 TW64[64];                                                     // w_64^t

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int bb = (int)xcd_contiguous(blockIdx.x, gridDim.x);
    const int o_base = blockIdx.y * 128;
    const long long bo = bb / a.inner_count, bi = bb % a.inner_count;
    const c64 *__restrict__ xb = a.x + bo * a.x_outer_stride + bi * a.x_inner_stride;
    c64 *__restrict__ yb = a.y + bo * a.y_outer_stride + bi * a.y_inner_stride;
    const float *__restrict__ xbr = reinterpret_cast<const float *>(a.x) + bo * a.x_outer_stride + bi * a.x_inner_stride;
    float *__restrict__ ybr = reinterpret_cast<float *>(a.y) + bo * a.y_outer_stride + bi * a.y_inner_stride;
    const int n_it = (a.C_in + PPI - 1) / PPI;
    c64 *patch = patch_all + wave * C::PATCH;
    const int p = lane;                                 // row-stage identity
    const int kl = lane >> 2, qa = lane & 3;            // column-stage identity: column k_lo, quad position
    // patch entry (k_lo, p) lives at k_lo*64 + (p ^ 4(k_lo & 7)): a half wave of the column stage reads rows k_lo = 0..7
    // at positions qa + 4 p', which the swizzle spreads over all 32 eight-byte bank pairs (with k_lo & 3 rows k_lo and
    // k_lo + 4 met in one pair)
    const int swz = 4 * (kl & 7);
    const int g = lane >> 5, nn = lane & 31;            // MFMA identity
    const int slab = wave >> 1;                         // 32-output slab of this wave
    const int tile0 = (wave & 1) * TPW;                 // first mode tile of this wave
    const int o_lane = o_base + 32 * slab + nn;         // the output channel whose W this lane feeds

    floatx16 acc_re[TPW], acc_im[TPW];
#pragma unroll
    for (int i = 0; i < TPW; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) { acc_re[i][r] = 0.f; acc_im[i][r] = 0.f; }

    c64 va[16], vb[16];         // the next two pencils of this wave: block b lives in buffer b & 1
    c64 wraw[4];                // W[c0 + 4g + d][o_lane], d < 4, of the next block
    uintx4 a_re[3], a_im[3];    // split A operands of the current block

    auto load_pencil = [&](c64 *v, int c0) __attribute__((always_inline)) {
        const int c = c0 + wave;
        if constexpr (REAL) {
            const bool ok = EVEN || c < a.C_in;
            const float *src = xbr + (long long)(ok ? c : 0) * a.x_chan_stride + p;
#pragma unroll
            for (int j = 0; j < 16; ++j) {
                const float val = __builtin_nontemporal_load(src + 64 * j);
                v[j] = make_float2(ok ? val : 0.f, 0.f);
            }
        } else if constexpr (EVEN) {
            const c64 *src = xb + (long long)c * a.x_chan_stride + p;
#pragma unroll
            for (int j = 0; j < 16; ++j) v[j] = load_nt(src + 64 * j);
        } else {
            const bool ok = c < a.C_in;
            const c64 *src = xb + (long long)(ok ? c : 0) * a.x_chan_stride + p;
#pragma unroll
            for (int j = 0; j < 16; ++j) {
                c64 val = load_nt(src + 64 * j);
                v[j] = ok ? val : make_float2(0.f, 0.f);
            }
        }
    };
    auto load_w = [&](int c0) __attribute__((always_inline)) {
#pragma unroll
        for (int d = 0; d < 4; ++d) {
            const int c = c0 + 4 * g + d;
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
            a_re[0][d] = pack_bf16(re.t0, im.t0) ^ 0x80000000u;
            a_re[1][d] = pack_bf16(re.t1, im.t1) ^ 0x80000000u;
            a_re[2][d] = pack_bf16(re.t2, im.t2) ^ 0x80000000u;
            a_im[0][d] = pack_bf16(im.t0, re.t0);
            a_im[1][d] = pack_bf16(im.t1, re.t1);
            a_im[2][d] = pack_bf16(im.t2, re.t2);
        }
    };
    // Forward transform of the pencil in v, pruned to the K retained bins, into operand buffer `buf`.
    // REFILL, DEEP: v is reloaded with block refill_c0, two blocks ahead, as soon as its transform has left the
    // registers (after the patch writes): two blocks of loads per wave, 128 KB per CU, are then in flight, which
    // the loaded HBM latency needs; one block (64 KB) leaves the k-loop waiting for memory.
    // REFILL, not DEEP: v is reloaded with the next block right after the first butterfly level.
    auto row_stage = [&](c64 *v, int buf, auto refill, int refill_c0, auto &&hook) __attribute__((always_inline)) {
        constexpr bool REFILL = decltype(refill)::value;
        hook(std::integral_constant<int, 0>{});
        {
            c64 ea[8], eb[8], za[8], zo[8];
            dif_first_level<16, -1>(v, ea, eb);
            if constexpr (REFILL && !DEEP) {
                __builtin_amdgcn_sched_barrier(0);
                load_pencil(v, refill_c0);
                __builtin_amdgcn_sched_barrier(0);
            }
            RegFFT<8, -1, 1>::run(ea, za);
            RegFFT<8, -1, 1>::run(eb, zo);
            hook(std::integral_constant<int, 10>{});
            wave_sync();                                    // the previous pencil's patch reads are done
            hook(std::integral_constant<int, 1>{});
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                const int c0 = 2 * k, c1 = 2 * k + 1;       // z[2k] = za[k], z[2k+1] = zo[k]
                const c64 t0 = c0 == 0 ? za[0] : cmul(za[k], TW[c0 * 64 + p]);
                const c64 t1 = cmul(zo[k], TW[c1 * 64 + p]);
                patch[c0 * 64 + (p ^ (4 * (c0 & 7)))] = t0;
                patch[c1 * 64 + (p ^ (4 * (c1 & 7)))] = t1;
            }
        }
        hook(std::integral_constant<int, 11>{});
        if constexpr (REFILL && DEEP) {
            __builtin_amdgcn_sched_barrier(0);
            load_pencil(v, refill_c0);
            __builtin_amdgcn_sched_barrier(0);
        }
        wave_sync();
        hook(std::integral_constant<int, 2>{});
        // lane (k_lo, qa): entries p = qa + 4 p', p' < 16, of column k_lo
        c64 P[KH];
        dft_prune_out<16, KH, -1>([&](auto ppc) __attribute__((always_inline)) {
            constexpr int pp = decltype(ppc)::value;
            return patch[kl * 64 + ((qa + 4 * pp) ^ swz)];
        }, P);
#pragma unroll
        for (int kh = 1; kh < KH; ++kh) P[kh] = cmul(P[kh], TW64[qa * kh]);
        // sum over the quad; lane qa keeps bins k_hi = OPL qa + i
        c64 R[KH / 2], O[OPL];
        {
            const bool hi = (qa & 2) != 0;
#pragma unroll
            for (int i = 0; i < KH / 2; ++i) {
                const c64 mine = hi ? P[KH / 2 + i] : P[i], send = hi ? P[i] : P[KH / 2 + i];
                R[i] = make_float2(mine.x + sym_quad_perm<0x4E>(send.x), mine.y + sym_quad_perm<0x4E>(send.y));
            }
        }
        {
            const bool hi = (qa & 1) != 0;
#pragma unroll
            for (int i = 0; i < OPL; ++i) {
                const c64 mine = hi ? R[OPL + i] : R[i], send = hi ? R[i] : R[OPL + i];
                O[i] = make_float2(mine.x + sym_quad_perm<0xB1>(send.x), mine.y + sym_quad_perm<0xB1>(send.y));
            }
        }
        // bin k = k_lo + 16 (OPL qa + i)  ->  XS[buf][term][wave / 4][k / 32][wave % 4][k % 32]
        // Planar in the channel slot d = wave % 4: a wave stores ONE slot of every mode, so with the slot innermost
        // ([n][d]) its 64 dword stores could reach 16 banks only.  Here lane (k_lo, qa) stores at position k_lo (+ 16)
        // of tile qa (K = 128) or qa / 2 (K = 64); the tile stride of 128 + 16 (K = 128) or 128 + 32 (K = 64) dwords
        // turns (k_lo, qa) into 64 different banks.
        unsigned *dst = XS + buf * C::XS_BUF + (wave >> 2) * (KT * C::XT) + (wave & 3) * 32;
        if constexpr (REAL) {
            if (lane == 0) O[0] = make_float2(0.5f * O[0].x, 0.5f * O[0].y);    // bin 0 (k_lo = 0, qa = 0, i = 0)
        }
#pragma unroll
        for (int i = 0; i < OPL; ++i) {
            const int k = kl + 16 * (OPL * qa + i);
            const Split3 re = split3(O[i].x), im = split3(O[i].y);
            unsigned *d = dst + (k >> 5) * C::XT + (k & 31);
            d[0 * 2 * KT * C::XT] = pack_bf16(re.t0, im.t0);
            d[1 * 2 * KT * C::XT] = pack_bf16(re.t1, im.t1);
            d[2 * 2 * KT * C::XT] = pack_bf16(re.t2, im.t2);
        }
        hook(std::integral_constant<int, 12>{});
    };
    auto mfma_block = [&](int buf) __attribute__((always_inline)) {
        const unsigned *src = XS + buf * C::XS_BUF + (g * KT + tile0) * C::XT + nn;
        uintx4 b[TPW][3];
#pragma unroll
        for (int i = 0; i < TPW; ++i)
#pragma unroll
            for (int t = 0; t < 3; ++t) {
                const unsigned *q = src + t * 2 * KT * C::XT + i * C::XT;
                b[i][t] = uintx4{q[0], q[32], q[64], q[96]};    // the four channel slots of mode nn
            }
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
    };
    // one k-loop iteration: contraction of block `it`, row stage of block it + 1 (held in v), W of block it + 1.
    // The 12 TPW MFMAs of the block are spread over the three stretches of the row stage (between its wave-level LDS
    // synchronisations) and interleaved with its vector instructions by an explicit pattern: a wave that issues the
    // contraction and then the transforms pays the sum of both, and both waves of a SIMD reach the contraction
    // together after the barrier, so without the pattern the matrix pipe runs while the vector ALU idles and vice
    // versa.  (Contraction first: it does not depend on the loads in flight, so the row stage, which starts by
    // waiting for them, still meets them as late as possible.)
    auto no_hook = [](auto) __attribute__((always_inline)) {};
    auto body = [&](int it, c64 *v, auto refill) __attribute__((always_inline)) {
        load_w((it + 1) * PPI);
        const unsigned *src = XS + (it & 1) * C::XS_BUF + (g * KT + tile0) * C::XT + nn;
        uintx4 b[TPW][3];
        constexpr int SA[6] = {2, 0, 1, 1, 0, 0}, SB[6] = {0, 2, 1, 0, 1, 0};      // smallest products first
        auto products = [&](int k0, int k1) __attribute__((always_inline)) {
#pragma unroll
            for (int k = k0; k < k1; ++k)
#pragma unroll
                for (int i = 0; i < TPW; ++i) {
                    const bf16x8 bb16 = __builtin_bit_cast(bf16x8, b[i][SB[k]]);
                    acc_re[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a_re[SA[k]]), bb16, acc_re[i], 0, 0, 0);
                    acc_im[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a_im[SA[k]]), bb16, acc_im[i], 0, 0, 0);
                }
        };
        auto pattern = [&](auto mfmas, auto valu_per_mfma) __attribute__((always_inline)) {
            static_for<0, decltype(mfmas)::value>([&](auto) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x002, decltype(valu_per_mfma)::value, 0);
            });
        };
        row_stage(v, (it + 1) & 1, refill, (it + (DEEP ? 3 : 2)) * PPI, [&](auto rc) __attribute__((always_inline)) {
            constexpr int R = decltype(rc)::value;
            if constexpr (R == 0) {
#pragma unroll
                for (int i = 0; i < TPW; ++i)
#pragma unroll
                    for (int t = 0; t < 3; ++t) {
                        const unsigned *q = src + t * 2 * KT * C::XT + i * C::XT;
                        b[i][t] = uintx4{q[0], q[32], q[64], q[96]};        // the four channel slots of mode nn
                    }
                products(0, 2);
            } else if constexpr (R == 10) {
                pattern(std::integral_constant<int, 4 * TPW>{}, std::integral_constant<int, 20>{});
            } else if constexpr (R == 1) {
                products(2, 3);
            } else if constexpr (R == 11) {
                pattern(std::integral_constant<int, 2 * TPW>{}, std::integral_constant<int, 20>{});
            } else if constexpr (R == 2) {
                products(3, 6);
            } else if constexpr (R == 12) {
                pattern(std::integral_constant<int, 6 * TPW>{}, std::integral_constant<int, 18>{});
            }
        });
        split_w();
        __syncthreads();
    };
    const std::true_type yes{};
    const std::false_type no{};

    // ------------------------------------------------------------------ k-loop over input channels
    load_pencil(va, 0);
    if constexpr (DEEP) load_pencil(vb, PPI);
    load_w(0);
    // the twiddle tables are built while the first loads are in flight
    __builtin_amdgcn_sched_barrier(0);
    for (int i = tid; i < N; i += C::NT) TW[i] = cis2pi(-(float)((i >> 6) * (i & 63)), (float)N);
    if (tid < 64) TW64[tid] = cis2pi(-(float)tid, 64.f);
    __syncthreads();                                        // twiddle tables are ready
    if constexpr (DEEP) {
        row_stage(va, 0, yes, 2 * PPI, no_hook);
    } else {
        if (n_it > 1) row_stage(va, 0, yes, PPI, no_hook);
        else row_stage(va, 0, no, 0, no_hook);
    }
    split_w();
    __syncthreads();                                        // XS[0] holds block 0
    if constexpr (DEEP) {
        // iteration `it` transforms block it + 1 (buffer (it + 1) & 1) and refills that buffer with block it + 3
        int it = 0;
        for (; it + 4 < n_it; it += 2) {
            body(it, vb, yes);
            body(it + 1, va, yes);
        }
        body(it, vb, yes);          // it = n_it - 4: block n_it - 3, refill with the last block
        body(it + 1, va, no);       // block n_it - 2
        body(it + 2, vb, no);       // block n_it - 1
        mfma_block((it + 3) & 1);
    } else {
        int it = 0;
        for (; it + 2 < n_it; ++it) body(it, va, yes);
        if (it + 1 < n_it) { body(it, va, no); ++it; }
        mfma_block(it & 1);
    }

    // ------------------------------------------------------------------ epilogue
    __syncthreads();                                        // every wave is done reading XS, which YH aliases
    for (int r = 0; r < 16; ++r) {
        // spectra of this round's 8 output pencils (slot 2 slab + l/32), in mode order
        {
            c64 *dst = YH + (r & 1) * C::YH_BUF + (2 * slab + g) * K + 32 * tile0 + nn;
            static_for<0, 16>([&](auto rc) {
                constexpr int R = decltype(rc)::value;
                if (r == R) {
#pragma unroll
                    for (int i = 0; i < TPW; ++i) dst[32 * i] = make_float2(acc_re[i][R], acc_im[i][R]);
                }
            });
        }
        __syncthreads();
        // wave w inverts pencil slot w: output 32 (w/2) + 8 (r/4) + 4 (w%2) + r%4
        const c64 *Yp = YH + (r & 1) * C::YH_BUF + wave * K;
        c64 yin[KH];
#pragma unroll
        for (int kh = 0; kh < KH; ++kh) {
            c64 t = Yp[kl + 16 * kh];
            if (kh != 0) {
                const c64 w = TW64[qa * kh];
                t = cmul(t, make_float2(w.x, -w.y));
            }
            yin[kh] = t;
        }
        wave_sync();                                        // the previous pencil's patch reads are done
        dft_prune_in<16, KH, +1>(yin, [&](auto ppc, c64 val) __attribute__((always_inline)) {
            constexpr int pp = decltype(ppc)::value;
            patch[kl * 64 + ((qa + 4 * pp) ^ swz)] = val;
        });
        wave_sync();
        c64 z[16], res[16];
#pragma unroll
        for (int c = 0; c < 16; ++c) {
            c64 t = patch[c * 64 + (p ^ (4 * (c & 7)))];
            if (c != 0) {
                const c64 w = TW[c * 64 + p];
                t = cmul(t, make_float2(w.x, -w.y));
            }
            z[c] = t;
        }
        RegFFT<16, +1, 1>::run(z, res);
        const int o = o_base + 32 * (wave >> 1) + 8 * (r / 4) + 4 * (wave & 1) + (r % 4);
        if (EVEN || o < a.C_out) {
            if constexpr (REAL) {
                float *dst = ybr + (long long)o * a.y_chan_stride + p;
#pragma unroll
                for (int j = 0; j < 16; ++j) __builtin_nontemporal_store(res[j].x, dst + 64 * j);
            } else {
                c64 *dst = yb + (long long)o * a.y_chan_stride + p;
#pragma unroll
                for (int j = 0; j < 16; ++j) store_nt(dst + 64 * j, res[j]);
            }
        }
    }
}

template <int K, bool REAL = false>
hipError_t launch_fused1d_sym(const Fused1dArgs &a, long long batch_rows, hipStream_t s)
{
    using C = SymCfg<K>;
    static LdsLimitOnce lds_limit;
    const hipError_t e = lds_limit.set({reinterpret_cast<const void *>(&k_fused1d_sym<K, true, true, REAL>),
                                        reinterpret_cast<const void *>(&k_fused1d_sym<K, true, false, REAL>),
                                        reinterpret_cast<const void *>(&k_fused1d_sym<K, false, false, REAL>)},
                                       (int)C::LDS_DYN);
    if (e != hipSuccess) return e;
    dim3 grid((unsigned)batch_rows, (unsigned)((a.C_out + 127) / 128));
    const bool even = a.C_in % C::PPI == 0 && a.C_out % 128 == 0;
    const int n_it = (a.C_in + C::PPI - 1) / C::PPI;
    if (even && n_it % 2 == 0 && n_it >= 4)
        hipLaunchKernelGGL((k_fused1d_sym<K, true, true, REAL>), grid, dim3(512), C::LDS_DYN, s, a);
    else if (even)
        hipLaunchKernelGGL((k_fused1d_sym<K, true, false, REAL>), grid, dim3(512), C::LDS_DYN, s, a);
    else
        hipLaunchKernelGGL((k_fused1d_sym<K, false, false, REAL>), grid, dim3(512), C::LDS_DYN, s, a);
    return hipGetLastError();
}

}  // namespace tfno
