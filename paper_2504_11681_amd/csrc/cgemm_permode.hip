// Launcher of the per-mode-weight contraction.
#include "cgemm_permode_kernel.h"
#include "cgemm_permode_mfma_kernel.h"
#include "fused1d.h"
#include "fused2d.h"

namespace tfno {

hipError_t cgemm_permode_launch(const c64 *Xh, const c64 *W, c64 *Yh, int C_in, int C_out, int M, long long num_tiles,
                                int TPI, float scale, int K2p, int K1a, int K2a, hipStream_t s)
{
    if (num_tiles <= 0) return hipSuccess;
    if (TPI < 1 || M < 1 || (long long)TPI * 128 > (long long)M + 127) return hipErrorInvalidValue;
    if (K2p < 1 || M % K2p != 0 || K1a < 1 || K1a > M / K2p || K2a < 1 || K2a > K2p) return hipErrorInvalidValue;
    const long long per = (num_tiles + TPI - 1) / TPI;      // tiles that hold the same modes
    // Matrix-pipe kernel: whole 128-mode tiles per batch element, enough channels and batch elements to fill its
    // 32 x 32 x 8-channel tiles; everything else (and TFNO_CONTRACTION=f32) keeps the FP32 kernel.
    if (M % 128 == 0 && TPI == M / 128 && C_in >= 16 && C_out >= 16 && per >= 16 && !contraction_forced_f32() &&
        (per + 31) / 32 <= 65535 && (C_out + 31) / 32 <= 65535) {
        const dim3 grid((unsigned)(TPI * 16), (unsigned)((per + 31) / 32), (unsigned)((C_out + 31) / 32));
        // without masks where every tile is full and the extents a workgroup addresses with 32-bit offsets (32 batch
        // elements of Xh, all of W) stay below 2^31 bytes
        const bool fits32 = 32LL * TPI * C_in * 1024 < (1LL << 31) && (long long)C_in * C_out * K1a * K2a * 8 < (1LL << 31);
        if (per % 32 == 0 && C_out % 32 == 0 && C_in % 8 == 0 && fits32)
            hipLaunchKernelGGL(k_cgemm_permode_mfma<true>, grid, dim3(256), 0, s, Xh, W, Yh, C_in, C_out, M, num_tiles, TPI, scale, K2p, K1a, K2a);
        else
            hipLaunchKernelGGL(k_cgemm_permode_mfma<false>, grid, dim3(256), 0, s, Xh, W, Yh, C_in, C_out, M, num_tiles, TPI, scale, K2p, K1a, K2a);
        return hipGetLastError();
    }
    constexpr int OT = 8;
    const unsigned gy = (unsigned)((C_out + 2 * OT - 1) / (2 * OT));
    if (per >= 8) {
        const dim3 grid((unsigned)(TPI * ((per + 7) / 8)), gy);
        hipLaunchKernelGGL((k_cgemm_permode<8, OT>), grid, dim3(256), 0, s, Xh, W, Yh, C_in, C_out, M, num_tiles, TPI, scale, K2p, K1a, K2a);
    } else {
        const dim3 grid((unsigned)(TPI * ((per + 1) / 2)), gy);
        hipLaunchKernelGGL((k_cgemm_permode<2, OT>), grid, dim3(256), 0, s, Xh, W, Yh, C_in, C_out, M, num_tiles, TPI, scale, K2p, K1a, K2a);
    }
    return hipGetLastError();
}

}  // namespace tfno
