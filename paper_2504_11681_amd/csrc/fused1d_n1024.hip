// Fused-kernel instantiations for N = 1024 (one translation unit per N so they build in parallel).
#include "fused1d_kernel.h"

namespace tfno {

hipError_t fused1d_launch_n1024(int K, const Fused1dArgs &a, long long rows, hipStream_t s)
{
    switch (K) {
    case 32:
        if (a.C_out > 64) return launch_fused1d<1024, 32, 4>(a, rows, s);
        if (a.C_out > 32) return launch_fused1d<1024, 32, 2>(a, rows, s);
        return launch_fused1d<1024, 32, 1>(a, rows, s);
    case 64:
        if (a.C_out > 64) return launch_fused1d<1024, 64, 4>(a, rows, s);
        if (a.C_out > 32) return launch_fused1d<1024, 64, 2>(a, rows, s);
        return launch_fused1d<1024, 64, 1>(a, rows, s);
    case 128:
        if (a.C_out > 64) return launch_fused1d<1024, 128, 4>(a, rows, s);
        if (a.C_out > 32) return launch_fused1d<1024, 128, 2>(a, rows, s);
        return launch_fused1d<1024, 128, 1>(a, rows, s);
    case 256:
        if (a.C_out > 32) return launch_fused1d<1024, 256, 2>(a, rows, s);
        return launch_fused1d<1024, 256, 1>(a, rows, s);
    default: return hipErrorInvalidValue;
    }
}

}  // namespace tfno
