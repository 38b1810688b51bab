// Fused-kernel instantiations for N = 128 (one translation unit per N so they build in parallel).
#include "fused1d_kernel.h"

namespace tfno {

hipError_t fused1d_launch_n128(int K, const Fused1dArgs &a, long long rows, hipStream_t s)
{
    switch (K) {
    case 16:
        switch (pick_output_tiles(a.C_out, rows, 4)) {
        case 4: return launch_fused1d<128, 16, 4>(a, rows, s);
        case 2: return launch_fused1d<128, 16, 2>(a, rows, s);
        default: return launch_fused1d<128, 16, 1>(a, rows, s);
        }
    case 32:
        switch (pick_output_tiles(a.C_out, rows, 4)) {
        case 4: return launch_fused1d<128, 32, 4>(a, rows, s);
        case 2: return launch_fused1d<128, 32, 2>(a, rows, s);
        default: return launch_fused1d<128, 32, 1>(a, rows, s);
        }
    case 64:
        switch (pick_output_tiles(a.C_out, rows, 4)) {
        case 4: return launch_fused1d<128, 64, 4>(a, rows, s);
        case 2: return launch_fused1d<128, 64, 2>(a, rows, s);
        default: return launch_fused1d<128, 64, 1>(a, rows, s);
        }
    case 128:
        switch (pick_output_tiles(a.C_out, rows, 4)) {
        case 4: return launch_fused1d<128, 128, 4>(a, rows, s);
        case 2: return launch_fused1d<128, 128, 2>(a, rows, s);
        default: return launch_fused1d<128, 128, 1>(a, rows, s);
        }
    default: return hipErrorInvalidValue;
    }
}

}  // namespace tfno
