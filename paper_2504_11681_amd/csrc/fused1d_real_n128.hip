// Real-valued layer: fused-kernel instantiations for N = 128.
#include "fused1d_kernel.h"

namespace tfno {

hipError_t fused1d_real_launch_n128(int K, const Fused1dArgs &a, long long rows, hipStream_t s)
{
    switch (K) {
    case 16: return launch_fused1d_real<128, 16, 4>(a, rows, s);
    case 32: return launch_fused1d_real<128, 32, 4>(a, rows, s);
    case 64: return launch_fused1d_real<128, 64, 4>(a, rows, s);
    default: return hipErrorInvalidValue;
    }
}

}  // namespace tfno
