// Fused-kernel instantiations for N = 128 (one translation unit per N so they build in parallel).
#include "fused1d_kernel.h"

namespace tfno {

hipError_t fused1d_launch_n128(int K, const Fused1dArgs &a, long long rows, hipStream_t s)
{
    // K >= 64 with more batch rows than CUs: the single-operand-tile form of the kernel, whose LDS lets two workgroups
    // share a CU (65 against 89 KB at K = 64); a batch row is only C_in / 32 blocks long here, so a workgroup is mostly
    // pipeline fill and drain and needs a neighbour to overlap with.
    if (rows > 256 && !contraction_forced_f32() && !generic_kernels_forced()) {
        if (K == 64) {
            if (a.C_out > 64) return launch_fused1d_wide<128, 64, 4, 4>(a, rows, s);
            if (a.C_out > 32) return launch_fused1d_wide<128, 64, 2, 4>(a, rows, s);
            return launch_fused1d_wide<128, 64, 1, 4, split_steps_over_waves<128, 64, 1>()>(a, rows, s);
        }
    }
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
