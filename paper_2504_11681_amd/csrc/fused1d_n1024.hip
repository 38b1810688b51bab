// Fused-kernel instantiations for N = 1024 (one translation unit per N so they build in parallel).
#include "fused1d_kernel.h"

namespace tfno {

hipError_t fused1d_launch_n1024(int K, const Fused1dArgs &a, long long rows, hipStream_t s)
{
    switch (K) {
    case 32:
        switch (pick_output_tiles(a.C_out, rows, 4)) {
        case 4: return launch_fused1d<1024, 32, 4>(a, rows, s);
        case 2: return launch_fused1d<1024, 32, 2>(a, rows, s);
        default: return launch_fused1d<1024, 32, 1>(a, rows, s);
        }
    case 64:
        switch (pick_output_tiles(a.C_out, rows, 4)) {
        case 4: return launch_fused1d<1024, 64, 4>(a, rows, s);
        case 2: return launch_fused1d<1024, 64, 2>(a, rows, s);
        default: return launch_fused1d<1024, 64, 1>(a, rows, s);
        }
    case 128:
        switch (pick_output_tiles(a.C_out, rows, 4)) {
        case 4: return launch_fused1d<1024, 128, 4>(a, rows, s);
        case 2: return launch_fused1d<1024, 128, 2>(a, rows, s);
        default: return launch_fused1d<1024, 128, 1>(a, rows, s);
        }
    case 256:
        if (pick_output_tiles(a.C_out, rows, 2) == 2) return launch_fused1d<1024, 256, 2>(a, rows, s);
        return launch_fused1d<1024, 256, 1>(a, rows, s);
    default: return hipErrorInvalidValue;
    }
}

}  // namespace tfno
