// Symmetric-wave fused-kernel instantiations (N = 1024).
#include "fused1d_sym_kernel.h"

namespace tfno {

hipError_t fused1d_sym_launch(int N, int K, const Fused1dArgs &a, long long rows, hipStream_t s)
{
    if (N != 1024) return hipErrorInvalidValue;
    switch (K) {
    case 64: return launch_fused1d_sym<64>(a, rows, s);
    case 128: return launch_fused1d_sym<128>(a, rows, s);
    default: return hipErrorInvalidValue;
    }
}

bool fused1d_sym_supported(int N, int K) { return N == 1024 && (K == 64 || K == 128); }

// the real-valued layer (float32 x and y) on the same kernel
hipError_t fused1d_sym_real_launch(int N, int K, const Fused1dArgs &a, long long rows, hipStream_t s)
{
    if (N != 1024) return hipErrorInvalidValue;
    switch (K) {
    case 64: return launch_fused1d_sym<64, true>(a, rows, s);
    case 128: return launch_fused1d_sym<128, true>(a, rows, s);
    default: return hipErrorInvalidValue;
    }
}

}  // namespace tfno
