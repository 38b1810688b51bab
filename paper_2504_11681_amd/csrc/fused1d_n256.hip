// Fused-kernel instantiations for N = 256 (one translation unit per N so they build in parallel).
#include "fused1d_kernel.h"

namespace tfno {

// Kernel choice for N = 256, measured on MI355X over the hidden-dimension sweep (B = 512):
//   K = 128, C_out <= 128, more batch rows than CUs: four waves with a single operand tile, two workgroups per CU
//       (C = 128: 80 us against 93 us for the double-buffered kernel that fits one workgroup per CU; C = 64: 34
//       against 40 us; C = 32: 16 against 21 us);
//   C_out > 128: one workgroup covers 256 outputs, so x is read and transformed once per batch row: the two-group
//       kernel for K = 32 and 64 where the channel counts are whole blocks (130 / 160 us against 155 / 185 us for two
//       128-output workgroups per row), the eight-wave kernel otherwise and for K = 128 (247 against 299 us);
//   at most 256 workgroups of 32 (K <= 64: or 64) outputs: the eight-wave kernel with those slabs;
//   everything else: the four-wave double-buffered kernel, two workgroups per CU wherever its LDS allows.
// TFNO_KERNEL=generic keeps the four-wave double-buffered kernel everywhere (A/B measurements).
template <int K>
static hipError_t launch_special_n256(const Fused1dArgs &a, long long rows, hipStream_t s, bool *done)
{
    *done = true;
    // (a 256-output workgroup per batch row needs about as many rows as CUs: B = 128, C = 256: 59 / 94 us at K = 64 / 128
    // against 53 / 74 us for the four-wave kernel's 128-output slabs, B = 64: 58 / 93 against 43 / 51 us; B = 256:
    // 80 / 117 against 89 / 148 us)
    if (a.C_out > 128 && rows >= 192) {
        if constexpr (K != 128) {
            if (a.inner_count == 1 && fused1d_pp_supported(256, K, a.C_in, a.C_out)) return fused1d_pp_launch(256, K, a, rows, s);
        }
        return launch_fused1d_wide<256, K, 8>(a, rows, s);
    }
    // Batches that give at most one workgroup per CU are bound by the latency of one workgroup: eight waves with
    // 32-output slabs halve the pencil blocks each wave transforms (B = 64, C = 64: 14.6 -> 12.3 us at K = 64,
    // 13.6 -> 11.7 at K = 32, 14.7 -> 13.2 at K = 128; B = 64, C = 128: 23.2 -> 20.0 us); with 64-output slabs they
    // still win at K <= 64 (B = 64, C = 256: 42.7 -> 36.9 us; B = 128, C = 128: 25.4 -> 23.9 us).  With more
    // workgroups than CUs the four-wave kernel's two workgroups per CU are faster (B = 256, C = 64: 17.9 against 26.2 us).
    // One or two 32-output slabs are only KT or 2 KT tiles: the 8-channel steps of a block are dealt out to the waves
    // that would otherwise wait for the one or two waves holding tiles (cfg2: 12.9 -> 11.4 us in the same run;
    // B = 64, C = 256: 38.0 -> 34.9 us).
    constexpr int KS1 = split_steps_over_waves<256, K, 1, 8>(), KS2 = split_steps_over_waves<256, K, 2, 8>();
    if (rows * ((a.C_out + 31) / 32) <= 256) return launch_fused1d_wide<256, K, 1, 8, KS1>(a, rows, s);
    if constexpr (K != 128) {
        if (rows * ((a.C_out + 63) / 64) <= 256) return launch_fused1d_wide<256, K, 2, 8, KS2>(a, rows, s);
    }
    // K <= 64 with more than four batch rows per CU: the single operand tile leaves room for THREE workgroups per CU
    // (49 KB of LDS, 163 - 168 registers) where the instantiation does not spill: whole channel blocks, and at
    // K = 64 at most 64 outputs (B 2048: C 64 / 128 at K = 32 106 -> 100 / 208 -> 200 us, C 32 / 64 at K = 64
    // 58 -> 53 / 110 -> 108 us; with spills, C 128 at K = 64 236 -> 282 us and masked C 48 91 -> 99 us, not used).
    if constexpr (K != 128) {
        const int ot = a.C_out > 64 ? 4 : a.C_out > 32 ? 2 : 1;
        if (rows > 1024 && a.C_in % 16 == 0 && a.C_out % (32 * ot) == 0 && (K == 32 || ot <= 2)) {
            if (ot == 4) return launch_fused1d_wide<256, K, 4, 4, split_steps_over_waves<256, K, 4>()>(a, rows, s);
            if (ot == 2) return launch_fused1d_wide<256, K, 2, 4, split_steps_over_waves<256, K, 2>()>(a, rows, s);
            return launch_fused1d_wide<256, K, 1, 4, split_steps_over_waves<256, K, 1>()>(a, rows, s);
        }
    }
    if constexpr (K == 128) {
        // (two workgroups per CU need more batch rows than CUs; below that the double-buffered kernel's single
        // barrier per block is the better deal)
        if (rows > 256) {
            if (a.C_out > 64) return launch_fused1d_wide<256, K, 4, 4>(a, rows, s);
            if (a.C_out > 32) return launch_fused1d_wide<256, K, 2, 4>(a, rows, s);
            return launch_fused1d_wide<256, K, 1, 4>(a, rows, s);
        }
    }
    *done = false;
    return hipSuccess;
}

hipError_t fused1d_launch_n256(int K, const Fused1dArgs &a, long long rows, hipStream_t s)
{
    if (!contraction_forced_f32() && !generic_kernels_forced()) {
        bool done = false;
        hipError_t e = hipSuccess;
        switch (K) {
        case 32: e = launch_special_n256<32>(a, rows, s, &done); break;
        case 64: e = launch_special_n256<64>(a, rows, s, &done); break;
        case 128: e = launch_special_n256<128>(a, rows, s, &done); break;
        default: break;
        }
        if (done) return e;
    }
    switch (K) {
    case 16:
        switch (pick_output_tiles(a.C_out, rows, 4)) {
        case 4: return launch_fused1d<256, 16, 4>(a, rows, s);
        case 2: return launch_fused1d<256, 16, 2>(a, rows, s);
        default: return launch_fused1d<256, 16, 1>(a, rows, s);
        }
    case 32:
        switch (pick_output_tiles(a.C_out, rows, 4)) {
        case 4: return launch_fused1d<256, 32, 4>(a, rows, s);
        case 2: return launch_fused1d<256, 32, 2>(a, rows, s);
        default: return launch_fused1d<256, 32, 1>(a, rows, s);
        }
    case 64:
        switch (pick_output_tiles(a.C_out, rows, 4)) {
        case 4: return launch_fused1d<256, 64, 4>(a, rows, s);
        case 2: return launch_fused1d<256, 64, 2>(a, rows, s);
        default: return launch_fused1d<256, 64, 1>(a, rows, s);
        }
    case 128:
        switch (pick_output_tiles(a.C_out, rows, 4)) {
        case 4: return launch_fused1d<256, 128, 4>(a, rows, s);
        case 2: return launch_fused1d<256, 128, 2>(a, rows, s);
        default: return launch_fused1d<256, 128, 1>(a, rows, s);
        }
    case 256:
        if (pick_output_tiles(a.C_out, rows, 2) == 2) return launch_fused1d<256, 256, 2>(a, rows, s);
        return launch_fused1d<256, 256, 1>(a, rows, s);
    default: return hipErrorInvalidValue;
    }
}

}  // namespace tfno
