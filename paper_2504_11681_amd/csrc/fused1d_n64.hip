// Fused-kernel instantiations for N = 64 (one translation unit per N so they build in parallel).
#include "fused1d_kernel.h"

namespace tfno {

hipError_t fused1d_launch_n64(int K, const Fused1dArgs &a, long long rows, hipStream_t s)
{
    switch (K) {
    case 8:
        if (a.C_out > 64) return launch_fused1d<64, 8, 4>(a, rows, s);
        if (a.C_out > 32) return launch_fused1d<64, 8, 2>(a, rows, s);
        return launch_fused1d<64, 8, 1>(a, rows, s);
    case 16:
        if (a.C_out > 64) return launch_fused1d<64, 16, 4>(a, rows, s);
        if (a.C_out > 32) return launch_fused1d<64, 16, 2>(a, rows, s);
        return launch_fused1d<64, 16, 1>(a, rows, s);
    case 32:
        if (a.C_out > 64) return launch_fused1d<64, 32, 4>(a, rows, s);
        if (a.C_out > 32) return launch_fused1d<64, 32, 2>(a, rows, s);
        return launch_fused1d<64, 32, 1>(a, rows, s);
    case 64:
        if (a.C_out > 64) return launch_fused1d<64, 64, 4>(a, rows, s);
        if (a.C_out > 32) return launch_fused1d<64, 64, 2>(a, rows, s);
        return launch_fused1d<64, 64, 1>(a, rows, s);
    default: return hipErrorInvalidValue;
    }
}

}  // namespace tfno
