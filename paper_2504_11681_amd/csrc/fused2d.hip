// Mode CGEMM instantiations and the launcher of the 2-D pipeline (the image kernels live in fused2d_n*.hip).
#include "cgemm_modes_kernel.h"
#include "fused2d.h"
#include "fused1d.h"

namespace tfno {

bool fused2d_supported(int N1, int N2, int K1, int K2)
{
    auto n_ok = [](int n) { return n == 64 || n == 128 || n == 256; };
    auto k_ok = [](int k) { return k == 16 || k == 32 || k == 64; };
    return n_ok(N1) && n_ok(N2) && k_ok(K1) && k_ok(K2);
}

size_t fused2d_workspace_bytes(long long B, int C_in, int C_out, int K1, int K2)
{
    return sizeof(c64) * (size_t)B * K1 * K2 * ((size_t)C_in + C_out);
}

hipError_t cgemm_modes_launch(const c64 *Xh, const c64 *W, c64 *Yh, int C_in, int C_out, float scale, long long tiles,
                              hipStream_t s)
{
    if (!contraction_forced_f32() && C_in <= 64) {
        // one block of W: the straight-line kernel, two mode tiles per workgroup
        const dim3 g2((unsigned)((tiles + 1) / 2), (unsigned)((C_out + 63) / 64));
        if (C_in <= 32)
            hipLaunchKernelGGL(k_cgemm_modes_small<4>, g2, dim3(256), 0, s, Xh, W, Yh, C_in, C_out, scale, tiles);
        else
            hipLaunchKernelGGL(k_cgemm_modes_small<8>, g2, dim3(256), 0, s, Xh, W, Yh, C_in, C_out, scale, tiles);
        return hipGetLastError();
    }
    if (!contraction_forced_f32() && C_in <= 128) {
        // all of W resident in LDS, eight waves, two mode tiles at a time; about one workgroup per CU
        const int c_pad = (C_in + 31) / 32 * 32, lds = c_pad * 3 * 64 * 4;
        static LdsLimitOnce lds_limit;
        const hipError_t e = lds_limit.set({reinterpret_cast<const void *>(&k_cgemm_modes_resident)}, 128 * 3 * 64 * 4);
        if (e != hipSuccess) return e;
        const long long pairs = (tiles + 1) / 2, gy = (C_out + 63) / 64;
        long long ppw = pairs * gy / 256;
        ppw = ppw < 1 ? 1 : ppw > 16 ? 16 : ppw;
        const dim3 gr((unsigned)((pairs + ppw - 1) / ppw), (unsigned)gy);
        hipLaunchKernelGGL(k_cgemm_modes_resident, gr, dim3(512), lds, s, Xh, W, Yh, C_in, C_out, scale, tiles, (int)ppw);
        return hipGetLastError();
    }
    // about two workgroups per CU, each walking several mode tiles
    const int tpw = tiles >= 1024 ? (int)(tiles / 512 > 16 ? 16 : tiles / 512) : 1;
    const dim3 ggrid((unsigned)((tiles + tpw - 1) / tpw), (unsigned)((C_out + 63) / 64));
    if (contraction_forced_f32())
        hipLaunchKernelGGL(k_cgemm_modes_f32, ggrid, dim3(256), 0, s, Xh, W, Yh, C_in, C_out, scale, tiles, tpw);
    else
        hipLaunchKernelGGL(k_cgemm_modes, ggrid, dim3(256), 0, s, Xh, W, Yh, C_in, C_out, scale, tiles, tpw);
    return hipGetLastError();
}

hipError_t fused2d_images(int dir, const c64 *in, c64 *out, long long images, int C, int N1, int N2, int K1, int K2,
                          int k1_keep, int k2_keep, bool fno, int h1, hipStream_t s)
{
    if (!fused2d_supported(N1, N2, K1, K2) || (fno && (h1 < 0 || h1 > K1))) return hipErrorInvalidValue;
    auto run = fno ? (N1 == 64 ? fused2d_fno_images_n64 : N1 == 128 ? fused2d_fno_images_n128 : fused2d_fno_images_n256)
                   : (N1 == 64 ? fused2d_images_n64 : N1 == 128 ? fused2d_images_n128 : fused2d_images_n256);
    return run(dir, in, out, images, C, N2, K1, K2, k1_keep, k2_keep, fno ? h1 : 0, s);
}

hipError_t fused2d_launch(const c64 *x, const c64 *W, c64 *y, long long B, int C_in, int C_out, int N1, int N2,
                          int K1, int K2, int k1_keep, int k2_keep, c64 *ws, hipStream_t s)
{
    const int M = K1 * K2;                                  // a multiple of 128
    c64 *Xh = ws, *Yh = ws + (size_t)B * C_in * M;
    hipError_t e = fused2d_images(-1, x, Xh, B * C_in, C_in, N1, N2, K1, K2, k1_keep, k2_keep, false, 0, s);
    if (e != hipSuccess) return e;
    e = cgemm_modes_launch(Xh, W, Yh, C_in, C_out, 1.0f / ((float)N1 * (float)N2), B * (M / 128), s);
    if (e != hipSuccess) return e;
    return fused2d_images(+1, Yh, y, B * C_out, C_out, N1, N2, K1, K2, K1, K2, false, 0, s);
}

}  // namespace tfno
