// Instantiations and launcher of the 2-D kernels.
#include "fused2d_kernel.h"
#include "fused2d.h"
#include "fused1d.h"

namespace tfno {

bool fused2d_supported(int N, int K)
{
    return (N == 64 || N == 128 || N == 256) && (K == 16 || K == 32 || K == 64) && K <= N;
}

size_t fused2d_workspace_bytes(long long B, int C_in, int C_out, int K)
{
    return sizeof(c64) * (size_t)B * K * K * ((size_t)C_in + C_out);
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
    // about two workgroups per CU, each walking several mode tiles
    const int tpw = tiles >= 1024 ? (int)(tiles / 512 > 16 ? 16 : tiles / 512) : 1;
    const dim3 ggrid((unsigned)((tiles + tpw - 1) / tpw), (unsigned)((C_out + 63) / 64));
    if (contraction_forced_f32())
        hipLaunchKernelGGL(k_cgemm_modes_f32, ggrid, dim3(256), 0, s, Xh, W, Yh, C_in, C_out, scale, tiles, tpw);
    else
        hipLaunchKernelGGL(k_cgemm_modes, ggrid, dim3(256), 0, s, Xh, W, Yh, C_in, C_out, scale, tiles, tpw);
    return hipGetLastError();
}

template <int N, int K>
static hipError_t launch_nk(const c64 *x, const c64 *W, c64 *y, long long B, int C_in, int C_out, c64 *ws,
                            hipStream_t s)
{
    const int M = K * K;
    c64 *Xh = ws, *Yh = ws + (size_t)B * C_in * M;
    hipLaunchKernelGGL((k_fwd2d<N, K>), dim3((unsigned)(B * C_in)), dim3(256), 0, s, x, Xh, C_in);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    if ((e = cgemm_modes_launch(Xh, W, Yh, C_in, C_out, 1.0f / ((float)N * (float)N), B * (M / 128), s)) != hipSuccess)
        return e;
    hipLaunchKernelGGL((k_inv2d<N, K>), dim3((unsigned)(B * C_out)), dim3(256), 0, s, (const c64 *)Yh, y, C_out);
    return hipGetLastError();
}

template <int N>
static hipError_t launch_n(int K, const c64 *x, const c64 *W, c64 *y, long long B, int C_in, int C_out, c64 *ws,
                           hipStream_t s)
{
    switch (K) {
    case 16: return launch_nk<N, 16>(x, W, y, B, C_in, C_out, ws, s);
    case 32: return launch_nk<N, 32>(x, W, y, B, C_in, C_out, ws, s);
    case 64: return launch_nk<N, 64>(x, W, y, B, C_in, C_out, ws, s);
    default: return hipErrorInvalidValue;
    }
}

hipError_t fused2d_launch(const c64 *x, const c64 *W, c64 *y, long long B, int C_in, int C_out, int N, int K,
                          c64 *ws, hipStream_t s)
{
    if (!fused2d_supported(N, K)) return hipErrorInvalidValue;
    switch (N) {
    case 64: return launch_n<64>(K, x, W, y, B, C_in, C_out, ws, s);
    case 128: return launch_n<128>(K, x, W, y, B, C_in, C_out, ws, s);
    case 256: return launch_n<256>(K, x, W, y, B, C_in, C_out, ws, s);
    default: return hipErrorInvalidValue;
    }
}

}  // namespace tfno
