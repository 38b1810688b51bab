// Host-visible interface of the 2-D kernels (truncated-spectrum pipeline).
#pragma once
#include "common.h"

namespace tfno {

// True when the image kernels exist for N1 x N2 images keeping K1 x K2 modes: N1, N2 in {64, 128, 256},
// K1, K2 in {16, 32, 64}.
bool fused2d_supported(int N1, int N2, int K1, int K2);
// Workspace for Xh[B, C_in, K1, K2] and Yh[B, C_out, K1, K2].
size_t fused2d_workspace_bytes(long long B, int C_in, int C_out, int K1, int K2);
// Enqueues forward transform, mode CGEMM and inverse transform on stream s.
hipError_t fused2d_launch(const c64 *x, const c64 *W, c64 *y, long long B, int C_in, int C_out, int N1, int N2,
                          int K1, int K2, int k1_keep, int k2_keep, c64 *ws, hipStream_t s);
// One of the two image kernels: dir < 0 forward x[images, N1, N2] -> Xh (C = C_in), dir > 0 inverse Yh -> y (C = C_out).
// k1_keep, k2_keep (forward only): modes at or past them are written as zeros.
// fno: the real-field variants (x, y float32 images; first-axis frequencies -h1 .. K1-h1-1 at positions 0 .. K1-1;
// R2C / C2R along the last axis, the caller's contraction carries the scale 2 / (N1 N2)); h1 is ignored otherwise.
hipError_t fused2d_images(int dir, const c64 *in, c64 *out, long long images, int C, int N1, int N2, int K1, int K2,
                          int k1_keep, int k2_keep, bool fno, int h1, hipStream_t s);
// The two image kernels for one first-axis length (one translation unit each; fused2d_fno_*: the real-field variants).
#define TFNO_DECLARE_IMAGES(name)                                                                                     \
    hipError_t name(int dir, const c64 *in, c64 *out, long long images, int C, int N2, int K1, int K2, int k1_keep, \
                    int k2_keep, int h1, hipStream_t s)
TFNO_DECLARE_IMAGES(fused2d_images_n64);
TFNO_DECLARE_IMAGES(fused2d_images_n128);
TFNO_DECLARE_IMAGES(fused2d_images_n256);
TFNO_DECLARE_IMAGES(fused2d_fno_images_n64);
TFNO_DECLARE_IMAGES(fused2d_fno_images_n128);
TFNO_DECLARE_IMAGES(fused2d_fno_images_n256);
#undef TFNO_DECLARE_IMAGES

// Yh = Xh . (scale W) over `tiles` tiles of 128 modes; both spectra mode-tile major ([tile][channel][128]).
hipError_t cgemm_modes_launch(const c64 *Xh, const c64 *W, c64 *Yh, int C_in, int C_out, float scale, long long tiles,
                              hipStream_t s);

// Yh[t][o][i] = scale * sum_c Xh[t][c][i] * W[c][o][k1][k2] with an own weight matrix per mode; tile t, lane i holds
// mode m = ((t % TPI) * 128 + i) % M = k1 K2p + k2 of the M = K1p K2p modes the spectra are laid out for, W is
// [C_in, C_out, K1a, K2a] for the modes kept (K1a <= K1p, K2a <= K2p; the surplus modes of Xh hold zeros).
hipError_t cgemm_permode_launch(const c64 *Xh, const c64 *W, c64 *Yh, int C_in, int C_out, int M, long long num_tiles,
                                int TPI, float scale, int K2p, int K1a, int K2a, hipStream_t s);

}  // namespace tfno
