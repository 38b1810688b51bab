// Host-visible interface of the 2-D kernels (truncated-spectrum pipeline).
#pragma once
#include "common.h"

namespace tfno {

// True when the image kernels exist for (N, K): N in {64, 128, 256}, K in {16, 32, 64}, K <= N.
bool fused2d_supported(int N, int K);
// Workspace for Xh[B, C_in, K, K] and Yh[B, C_out, K, K].
size_t fused2d_workspace_bytes(long long B, int C_in, int C_out, int K);
// Enqueues forward transform, mode CGEMM and inverse transform on stream s.
hipError_t fused2d_launch(const c64 *x, const c64 *W, c64 *y, long long B, int C_in, int C_out, int N, int K,
                          c64 *ws, hipStream_t s);

// Yh = Xh . (scale W) over `tiles` tiles of 128 modes; both spectra mode-tile major ([tile][channel][128]).
hipError_t cgemm_modes_launch(const c64 *Xh, const c64 *W, c64 *Yh, int C_in, int C_out, float scale, long long tiles,
                              hipStream_t s);

}  // namespace tfno
