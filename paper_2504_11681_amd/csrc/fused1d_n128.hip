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
    // K <= 32, 33 .. 64 outputs, more than two batch rows per CU: the single operand tile again, here because it lets
    // THREE workgroups share a CU: 52 KB of LDS once the two partial sums of the split contraction are added in turns
    // into one epilogue tile, 156 registers.  B 4096, C 64: 117 -> 110 us (K = 32), 116 -> 106 us (K = 16); C 48:
    // 102 -> 92 us.  With 32 outputs (four partial sums, three extra barriers) it measured slower (54 -> 59 us), and
    // at B = 512 there is no third workgroup to place (16.3 -> 17.0 us).
    // (... except for a single, half-empty block of input channels: B 8192, C 16: 90 -> 78 us)
    if (rows > 512 && a.C_out <= 32 && a.C_in <= 16 && !contraction_forced_f32() && !generic_kernels_forced()) {
        if (K == 32) return launch_fused1d_wide<128, 32, 1, 4, split_steps_over_waves<128, 32, 1>()>(a, rows, s);
        if (K == 16) return launch_fused1d_wide<128, 16, 1, 4, split_steps_over_waves<128, 16, 1>()>(a, rows, s);
    }
    if (rows > 512 && a.C_out > 32 && a.C_out <= 64 && !contraction_forced_f32() && !generic_kernels_forced()) {
        if (K == 32) return launch_fused1d_wide<128, 32, 2, 4, split_steps_over_waves<128, 32, 2>()>(a, rows, s);
        if (K == 16) return launch_fused1d_wide<128, 16, 2, 4, split_steps_over_waves<128, 16, 2>()>(a, rows, s);
    }
    // ... and with more than 64 outputs and whole channel blocks (159 registers; the masked instantiation spills):
    // B 2048, C 128: 131 -> 124 us (K = 32), 128 -> 122 us (K = 16); B 1024, C 256: 197 -> 187 us.
    if (rows > 512 && a.C_out > 64 && a.C_in % 32 == 0 && a.C_out % 128 == 0 && !contraction_forced_f32() && !generic_kernels_forced()) {
        if (K == 16) return launch_fused1d_wide<128, 16, 4, 4>(a, rows, s);
        if (K == 32) return launch_fused1d_wide<128, 32, 4, 4>(a, rows, s);
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
