// Partially fused variant CGEMM + iFFT (Sec. 4.2): instantiations for N = 256.
#include "fused1d_kernel.h"

namespace tfno {

hipError_t fused1d_gemmifft_launch_n256(int K, const Fused1dArgs &a, long long rows, hipStream_t s)
{
    return launch_partial<256, 2>(K, a, rows, s);
}

}  // namespace tfno
