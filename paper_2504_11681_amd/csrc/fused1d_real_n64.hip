// Real-valued layer: fused-kernel instantiations for N = 64.
#include "fused1d_kernel.h"

namespace tfno {

hipError_t fused1d_real_launch_n64(int K, const Fused1dArgs &a, long long rows, hipStream_t s)
{
    switch (K) {
    case 8: return launch_fused1d_real<64, 8, 4>(a, rows, s);
    case 16: return launch_fused1d_real<64, 16, 4>(a, rows, s);
    case 32: return launch_fused1d_real<64, 32, 4>(a, rows, s);
    default: return hipErrorInvalidValue;
    }
}

}  // namespace tfno
