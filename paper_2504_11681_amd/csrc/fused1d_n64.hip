// Fused-kernel instantiations for N = 64 (one translation unit per N so they build in parallel).
#include "fused1d_kernel.h"

namespace tfno {

hipError_t fused1d_launch_n64(int K, const Fused1dArgs &a, long long rows, hipStream_t s)
{
    // More than 64 outputs, K <= 32, more than two batch rows per CU: the single-operand-tile form takes 145 - 149
    // registers against 202 for the double-buffered one, so three workgroups share a CU (B 4096, C 128: 167 -> 163 us;
    // C 96: 139 -> 125 us).  (With at most 64 outputs the split contraction already gets the double-buffered form
    // there.)
    if (rows > 512 && a.C_out > 64 && !contraction_forced_f32() && !generic_kernels_forced()) {
        if (K == 8) return launch_fused1d_wide<64, 8, 4, 4>(a, rows, s);
        if (K == 16) return launch_fused1d_wide<64, 16, 4, 4>(a, rows, s);
        if (K == 32) return launch_fused1d_wide<64, 32, 4, 4>(a, rows, s);
    }
    // At most 32 outputs, K <= 32, more than three batch rows per CU: the single-operand-tile form with the split
    // contraction takes 118 registers and 31 KB of LDS, so FOUR workgroups share a CU (B 8192, C 32: 57 -> 55 us;
    // B 16384, C 16: 89 -> 76 us).  With 33 - 64 outputs it gains 1 - 3 % on whole channel blocks and loses as much on
    // masked ones, and stays on the double-buffered form.
    if (rows > 768 && a.C_out <= 32 && !contraction_forced_f32() && !generic_kernels_forced()) {
        if (K == 8) return launch_fused1d_wide<64, 8, 1, 4, split_steps_over_waves<64, 8, 1>()>(a, rows, s);
        if (K == 16) return launch_fused1d_wide<64, 16, 1, 4, split_steps_over_waves<64, 16, 1>()>(a, rows, s);
        if (K == 32) return launch_fused1d_wide<64, 32, 1, 4, split_steps_over_waves<64, 32, 1>()>(a, rows, s);
    }
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
