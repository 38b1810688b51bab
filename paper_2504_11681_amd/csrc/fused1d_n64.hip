// Fused-kernel instantiations for N = 64 (one translation unit per N so they build in parallel).
#include "fused1d_kernel.h"

namespace tfno {

hipError_t fused1d_launch_n64(int K, const Fused1dArgs &a, long long rows, hipStream_t s)
{
    switch (K) {
    case 8:
        switch (pick_output_tiles(a.C_out, rows, 4)) {
        case 4: return launch_fused1d<64, 8, 4>(a, rows, s);
        case 2: return launch_fused1d<64, 8, 2>(a, rows, s);
        default: return launch_fused1d<64, 8, 1>(a, rows, s);
        }
    case 16:
        switch (pick_output_tiles(a.C_out, rows, 4)) {
        case 4: return launch_fused1d<64, 16, 4>(a, rows, s);
        case 2: return launch_fused1d<64, 16, 2>(a, rows, s);
        default: return launch_fused1d<64, 16, 1>(a, rows, s);
        }
    case 32:
        switch (pick_output_tiles(a.C_out, rows, 4)) {
        case 4: return launch_fused1d<64, 32, 4>(a, rows, s);
        case 2: return launch_fused1d<64, 32, 2>(a, rows, s);
        default: return launch_fused1d<64, 32, 1>(a, rows, s);
        }
    case 64:
        switch (pick_output_tiles(a.C_out, rows, 4)) {
        case 4: return launch_fused1d<64, 64, 4>(a, rows, s);
        case 2: return launch_fused1d<64, 64, 2>(a, rows, s);
        default: return launch_fused1d<64, 64, 1>(a, rows, s);
        }
    default: return hipErrorInvalidValue;
    }
}

}  // namespace tfno
