// Real-valued layer: fused-kernel instantiations for N = 512.
#include "fused1d_kernel.h"

namespace tfno {

hipError_t fused1d_real_launch_n512(int K, const Fused1dArgs &a, long long rows, hipStream_t s)
{
    switch (K) {
    case 32: return launch_fused1d_real<512, 32, 4>(a, rows, s);
    case 64: return launch_fused1d_real<512, 64, 4>(a, rows, s);
    case 128: return launch_fused1d_real<512, 128, 4>(a, rows, s);
    case 256: return launch_fused1d_real<512, 256, 2>(a, rows, s);
    default: return hipErrorInvalidValue;
    }
}

}  // namespace tfno
