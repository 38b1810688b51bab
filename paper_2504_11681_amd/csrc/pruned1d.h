// Host-visible interface of the unfused 1-D variant with pruned transforms (three kernels).
#pragma once
#include "common.h"

namespace tfno {

// N in {64, 128, 256} with K a multiple of 16 such that K/16 divides N/16, N = 1024 with K in {64, 128}, or
// N in {2048, 4096} with K / (N / 256) in {16, 32, 64, 128, 256}.
bool pruned1d_supported(int N, int K);
// Workspace for the truncated spectra of input and output, padded to whole 128-mode tiles.
size_t pruned1d_workspace_bytes(long long B, int C_in, int C_out, int K);
// K_keep (1 .. K): bins K_keep .. K-1 of the forward transform are written as zeros, which truncates to K_keep modes.
hipError_t pruned1d_launch(const c64 *x, const c64 *W, c64 *y, long long B, int C_in, int C_out, int N, int K,
                           int K_keep, c64 *ws, hipStream_t s);
// Single stages for the partially fused variants: stages is a mask of PRUNED_FWD (x -> Xh), PRUNED_GEMM
// (Xh -> Yh, scaled by 1/N) and PRUNED_INV (Yh -> y); Xh holds ceil(B K / 128) * 128 * C_in elements, Yh the same
// with C_out.
enum { PRUNED_FWD = 1, PRUNED_GEMM = 2, PRUNED_INV = 4 };
size_t pruned1d_spectrum_elems(long long B, int C, int K);
hipError_t pruned1d_stages(int stages, const c64 *x, const c64 *W, c64 *y, c64 *Xh, c64 *Yh, long long B, int C_in,
                           int C_out, int N, int K, int K_keep, hipStream_t s);

// Real pencils (x, y float32; N <= 1024): PRUNED_FWD writes the R2C bins with bin 0 halved, PRUNED_INV stores the real
// part of the zero-padded inverse; the contraction between them (not run here) carries the scale 2 / N.
hipError_t pruned1d_real_stages(int stages, const float *x, float *y, c64 *Xh, c64 *Yh, long long B, int C_in, int C_out,
                                int N, int K, int K_keep, hipStream_t s);

}  // namespace tfno
