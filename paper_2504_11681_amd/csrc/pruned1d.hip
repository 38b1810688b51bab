// Instantiations and launcher of the unfused 1-D variant with pruned transforms.
#include "pruned1d_kernel.h"
#include "pruned1d_long_kernel.h"
#include "fused2d.h"          // cgemm_modes_launch
#include "pruned1d.h"

namespace tfno {

bool pruned1d_supported(int N, int K)
{
    if (K < 16 || K % 16 != 0 || K > N) return false;
    const int KH = K / 16;
    if (N == 1024) return KH == 4 || KH == 8;
    if (N == 2048 || N == 4096) {
        // long pencils: N1 = N / 256 rows of 256 points, each keeping K / N1 bins
        const int N1 = N / 256;
        if (K % N1) return false;
        const int K2 = K / N1;
        return K2 == 16 || K2 == 32 || K2 == 64 || K2 == 128 || K2 == 256;
    }
    if (N != 64 && N != 128 && N != 256) return false;
    const int LPR = N / 16;
    return (KH & (KH - 1)) == 0 && KH <= LPR;
}

static long long mode_tiles(long long B, int K) { return (B * K + 127) / 128; }

// Grid of a grid-stride transform kernel: as many workgroups as the chip holds at once (asked of the runtime once per
// kernel), then trimmed so that every workgroup runs the same number of sweeps.  A fixed grid of 1024 ran the N = 1024
// kernels (three workgroups per CU, 768 at once) as one full round plus a round of 256 workgroups on an empty chip.
template <auto Kern>
static unsigned balanced_grid(long long sweeps, int threads)
{
    static std::once_flag once;
    static long long slots = 0;
    std::call_once(once, [&] {
        int per_cu = 0, dev = 0, cus = 0;
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, Kern, threads, 0) != hipSuccess || per_cu < 1) per_cu = 2;
        if (hipGetDevice(&dev) != hipSuccess ||
            hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1)
            cus = 256;
        slots = (long long)per_cu * cus;
    });
    if (sweeps <= slots) return (unsigned)sweeps;
    const long long rounds = (sweeps + slots - 1) / slots;
    return (unsigned)((sweeps + rounds - 1) / rounds);
}

size_t pruned1d_workspace_bytes(long long B, int C_in, int C_out, int K)
{
    return sizeof(c64) * (size_t)mode_tiles(B, K) * 128 * ((size_t)C_in + C_out);
}

size_t pruned1d_spectrum_elems(long long B, int C, int K) { return (size_t)mode_tiles(B, K) * 128 * (size_t)C; }

template <int N, int K, bool REAL = false>
static hipError_t launch_nk(int stages, const c64 *x, const c64 *W, c64 *y, c64 *Xh, c64 *Yh, long long B, int C_in,
                            int C_out, int K_keep, hipStream_t s)
{
    using Cf = CfgP1<N, K>;
    const long long tiles = mode_tiles(B, K);
    const long long pin = B * C_in, pout = B * C_out;
    const long long sin = (pin + Cf::PPS - 1) / Cf::PPS, sout = (pout + Cf::PPS - 1) / Cf::PPS;
    // a few sweeps per workgroup amortise the twiddle tables and keep a prefetch in flight
    // (measured: the forward kernels gain 2 - 4 % and the real-valued inverse 13 % from the balanced grid; the complex
    // inverse kernels, which write twice the bytes, lose 4 % and keep the fixed grid)
    const unsigned gin = balanced_grid<&k_fwd1d<N, K, REAL>>(sin, 256);
    const unsigned gout = REAL ? balanced_grid<&k_inv1d<N, K, REAL>>(sout, 256) : (unsigned)(sout < 1024 ? sout : 1024);
    hipError_t e = hipSuccess;
    if (stages & PRUNED_FWD) {
        hipLaunchKernelGGL((k_fwd1d<N, K, REAL>), dim3(gin), dim3(256), 0, s, x, Xh, C_in, pin, K_keep);
        if ((e = hipGetLastError()) != hipSuccess) return e;
    }
    if (stages & PRUNED_GEMM)
        if ((e = cgemm_modes_launch(Xh, W, Yh, C_in, C_out, 1.0f / (float)N, tiles, s)) != hipSuccess) return e;
    if (stages & PRUNED_INV) {
        hipLaunchKernelGGL((k_inv1d<N, K, REAL>), dim3(gout), dim3(256), 0, s, (const c64 *)Yh, y, C_out, pout);
        e = hipGetLastError();
    }
    return e;
}

template <int N1, int K2>
static hipError_t launch_long(int stages, const c64 *x, const c64 *W, c64 *y, c64 *Xh, c64 *Yh, long long B, int C_in,
                              int C_out, int K_keep, hipStream_t s)
{
    using Cf = CfgLong<N1, K2>;
    const long long tiles = mode_tiles(B, Cf::K);
    const long long pin = B * C_in, pout = B * C_out;
    const long long sin = (pin + Cf::G - 1) / Cf::G, sout = (pout + Cf::G - 1) / Cf::G;
    const unsigned gin = balanced_grid<&k_fwd1d_long<N1, K2>>(sin, 256), gout = (unsigned)(sout < 2048 ? sout : 2048);
    hipError_t e = hipSuccess;
    if (stages & PRUNED_FWD) {
        hipLaunchKernelGGL((k_fwd1d_long<N1, K2>), dim3(gin), dim3(256), 0, s, x, Xh, C_in, pin, K_keep);
        if ((e = hipGetLastError()) != hipSuccess) return e;
    }
    if (stages & PRUNED_GEMM)
        if ((e = cgemm_modes_launch(Xh, W, Yh, C_in, C_out, 1.0f / (float)Cf::N, tiles, s)) != hipSuccess) return e;
    if (stages & PRUNED_INV) {
        hipLaunchKernelGGL((k_inv1d_long<N1, K2>), dim3(gout), dim3(256), 0, s, (const c64 *)Yh, y, C_out, pout);
        e = hipGetLastError();
    }
    return e;
}

template <int N1>
static hipError_t launch_long_n(int K2, int stages, const c64 *x, const c64 *W, c64 *y, c64 *Xh, c64 *Yh, long long B,
                                int C_in, int C_out, int K_keep, hipStream_t s)
{
    switch (K2) {
    case 16: return launch_long<N1, 16>(stages, x, W, y, Xh, Yh, B, C_in, C_out, K_keep, s);
    case 32: return launch_long<N1, 32>(stages, x, W, y, Xh, Yh, B, C_in, C_out, K_keep, s);
    case 64: return launch_long<N1, 64>(stages, x, W, y, Xh, Yh, B, C_in, C_out, K_keep, s);
    case 128: return launch_long<N1, 128>(stages, x, W, y, Xh, Yh, B, C_in, C_out, K_keep, s);
    case 256: return launch_long<N1, 256>(stages, x, W, y, Xh, Yh, B, C_in, C_out, K_keep, s);
    default: return hipErrorInvalidValue;
    }
}

template <int N, bool REAL = false>
static hipError_t launch_n(int K, int stages, const c64 *x, const c64 *W, c64 *y, c64 *Xh, c64 *Yh, long long B,
                           int C_in, int C_out, int K_keep, hipStream_t s)
{
    constexpr int LPR = N / 16;
    switch (K) {
    case 16: return launch_nk<N, 16, REAL>(stages, x, W, y, Xh, Yh, B, C_in, C_out, K_keep, s);
    case 32: if constexpr (LPR >= 2) return launch_nk<N, 32, REAL>(stages, x, W, y, Xh, Yh, B, C_in, C_out, K_keep, s); break;
    case 64: if constexpr (LPR >= 4) return launch_nk<N, 64, REAL>(stages, x, W, y, Xh, Yh, B, C_in, C_out, K_keep, s); break;
    case 128: if constexpr (LPR >= 8) return launch_nk<N, 128, REAL>(stages, x, W, y, Xh, Yh, B, C_in, C_out, K_keep, s); break;
    case 256: if constexpr (LPR >= 16) return launch_nk<N, 256, REAL>(stages, x, W, y, Xh, Yh, B, C_in, C_out, K_keep, s); break;
    default: break;
    }
    return hipErrorInvalidValue;
}

hipError_t pruned1d_stages(int stages, const c64 *x, const c64 *W, c64 *y, c64 *Xh, c64 *Yh, long long B, int C_in,
                           int C_out, int N, int K, int K_keep, hipStream_t s)
{
    if (!pruned1d_supported(N, K) || K_keep < 1 || K_keep > K) return hipErrorInvalidValue;
    switch (N) {
    case 64: return launch_n<64>(K, stages, x, W, y, Xh, Yh, B, C_in, C_out, K_keep, s);
    case 128: return launch_n<128>(K, stages, x, W, y, Xh, Yh, B, C_in, C_out, K_keep, s);
    case 256: return launch_n<256>(K, stages, x, W, y, Xh, Yh, B, C_in, C_out, K_keep, s);
    case 1024:
        if (K == 64) return launch_nk<1024, 64>(stages, x, W, y, Xh, Yh, B, C_in, C_out, K_keep, s);
        return launch_nk<1024, 128>(stages, x, W, y, Xh, Yh, B, C_in, C_out, K_keep, s);
    case 2048: return launch_long_n<8>(K / 8, stages, x, W, y, Xh, Yh, B, C_in, C_out, K_keep, s);
    case 4096: return launch_long_n<16>(K / 16, stages, x, W, y, Xh, Yh, B, C_in, C_out, K_keep, s);
    default: return hipErrorInvalidValue;
    }
}

hipError_t pruned1d_real_stages(int stages, const float *x, float *y, c64 *Xh, c64 *Yh, long long B, int C_in, int C_out,
                                int N, int K, int K_keep, hipStream_t s)
{
    if (!pruned1d_supported(N, K) || N > 1024 || K_keep < 1 || K_keep > K || (stages & PRUNED_GEMM))
        return hipErrorInvalidValue;
    const c64 *xc = reinterpret_cast<const c64 *>(x);
    c64 *yc = reinterpret_cast<c64 *>(y);
    switch (N) {
    case 64: return launch_n<64, true>(K, stages, xc, nullptr, yc, Xh, Yh, B, C_in, C_out, K_keep, s);
    case 128: return launch_n<128, true>(K, stages, xc, nullptr, yc, Xh, Yh, B, C_in, C_out, K_keep, s);
    case 256: return launch_n<256, true>(K, stages, xc, nullptr, yc, Xh, Yh, B, C_in, C_out, K_keep, s);
    case 1024:
        if (K == 64) return launch_nk<1024, 64, true>(stages, xc, nullptr, yc, Xh, Yh, B, C_in, C_out, K_keep, s);
        return launch_nk<1024, 128, true>(stages, xc, nullptr, yc, Xh, Yh, B, C_in, C_out, K_keep, s);
    default: return hipErrorInvalidValue;
    }
}

hipError_t pruned1d_launch(const c64 *x, const c64 *W, c64 *y, long long B, int C_in, int C_out, int N, int K,
                           int K_keep, c64 *ws, hipStream_t s)
{
    return pruned1d_stages(PRUNED_FWD | PRUNED_GEMM | PRUNED_INV, x, W, y, ws, ws + pruned1d_spectrum_elems(B, C_in, K),
                           B, C_in, C_out, N, K, K_keep, s);
}

}  // namespace tfno
