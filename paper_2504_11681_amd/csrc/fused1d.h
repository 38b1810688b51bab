// Host-visible interface of the fused last-axis kernel family.
#pragma once
#include "common.h"

namespace tfno {

// One "batch row" bb of the launch is the pair (bb / inner_count, bb % inner_count); its input pencils
// start at x + outer*x_outer_stride + inner*x_inner_stride + c*x_chan_stride (complex elements) and are
// contiguous along the transformed axis.  Plain 1-D: inner_count = 1.  Middle stage of the 2-D pipeline:
// outer = batch element, inner = retained row of the first axis.
struct Fused1dArgs {
    const c64 *x;
    const c64 *W;
    c64 *y;
    int C_in, C_out;
    long long inner_count;
    long long x_outer_stride, x_inner_stride, x_chan_stride;
    long long y_outer_stride, y_inner_stride, y_chan_stride;
    float scale;    // folded into W (1/N for 1-D; the 2-D pipeline passes its full 1/N^2 here)
    int K_keep;     // modes actually kept, 1 <= K_keep <= K (0 = all K): bins K_keep .. K-1 of the kernel's K enter
                    // the contraction as zeros, which is how mode counts between the built K are served
    // Partially fused variants only (inner_count = 1): truncated spectra in the mode-tile-major layout of the
    // unfused pruned variant, joint mode m = row * K + k at ((m / 128) * C + c) * 128 + m % 128.
    const c64 *Xh;  // read instead of x by the CGEMM + iFFT kernel
    c64 *Yh;        // written instead of y by the FFT + CGEMM kernel
};

// Returns true when a fused kernel exists for (N, K).
bool fused1d_supported(int N, int K);
// Enqueues the fused kernel; hipErrorInvalidValue when (N, K) is unsupported.
hipError_t fused1d_launch(int N, int K, const Fused1dArgs &a, long long batch_rows, hipStream_t s);

// True when the environment asks for FP32-MFMA contractions only (TFNO_CONTRACTION=f32).
bool contraction_forced_f32();
// True when the environment asks for the four-wave double-buffered kernel everywhere (TFNO_KERNEL=generic).
bool generic_kernels_forced();

// Wave-specialised variant (BF16x3 split contraction on the matrix pipe beside the VALU transforms).
bool fused1d_ws_supported(int N, int K);
hipError_t fused1d_ws_launch(int N, int K, const Fused1dArgs &a, long long rows, hipStream_t s);

// Symmetric-wave variant (every wave runs transforms and contraction; BF16x3 split contraction).
bool fused1d_sym_supported(int N, int K);
hipError_t fused1d_sym_launch(int N, int K, const Fused1dArgs &a, long long rows, hipStream_t s);
hipError_t fused1d_sym_real_launch(int N, int K, const Fused1dArgs &a, long long rows, hipStream_t s);

// Two-group variant for N = 256 (eight waves, the groups alternate between transforms and contraction; 256 outputs
// per workgroup): whole 32-channel blocks only, 128 < C_out, K in {32, 64}.
bool fused1d_pp_supported(int N, int K, int C_in, int C_out);
hipError_t fused1d_pp_launch(int N, int K, const Fused1dArgs &a, long long rows, hipStream_t s);

// Partially fused variants (Sec. 4.1 and 4.2): mode 1 = FFT + CGEMM in one kernel, writes the truncated output
// spectrum a.Yh; mode 2 = CGEMM + iFFT in one kernel, reads the truncated input spectrum a.Xh.  Built for
// N in {128, 256}, K in {32, 64, 128}; the contraction always runs on the BF16 matrix pipe.
bool fused1d_partial_supported(int N, int K);
// Real-valued layer (a.x, a.y: float32 tensors, strides in floats; a.scale = 2 / N): the fused kernel's shapes with
// K <= N / 2.
bool fused1d_real_supported(int N, int K);
hipError_t fused1d_real_launch(int N, int K, const Fused1dArgs &a, long long rows, hipStream_t s);
hipError_t fused1d_real_launch_n64(int K, const Fused1dArgs &a, long long rows, hipStream_t s);
hipError_t fused1d_real_launch_n128(int K, const Fused1dArgs &a, long long rows, hipStream_t s);
hipError_t fused1d_real_launch_n256(int K, const Fused1dArgs &a, long long rows, hipStream_t s);
hipError_t fused1d_real_launch_n512(int K, const Fused1dArgs &a, long long rows, hipStream_t s);
hipError_t fused1d_real_launch_n1024(int K, const Fused1dArgs &a, long long rows, hipStream_t s);
hipError_t fused1d_partial_launch(int mode, int N, int K, const Fused1dArgs &a, long long rows, hipStream_t s);
hipError_t fused1d_fftgemm_launch_n128(int K, const Fused1dArgs &a, long long rows, hipStream_t s);
hipError_t fused1d_fftgemm_launch_n256(int K, const Fused1dArgs &a, long long rows, hipStream_t s);
hipError_t fused1d_gemmifft_launch_n128(int K, const Fused1dArgs &a, long long rows, hipStream_t s);
hipError_t fused1d_gemmifft_launch_n256(int K, const Fused1dArgs &a, long long rows, hipStream_t s);

// Per-N dispatchers, one translation unit each.
hipError_t fused1d_launch_n64(int K, const Fused1dArgs &a, long long rows, hipStream_t s);
hipError_t fused1d_launch_n128(int K, const Fused1dArgs &a, long long rows, hipStream_t s);
hipError_t fused1d_launch_n256(int K, const Fused1dArgs &a, long long rows, hipStream_t s);
hipError_t fused1d_launch_n512(int K, const Fused1dArgs &a, long long rows, hipStream_t s);
hipError_t fused1d_launch_n1024(int K, const Fused1dArgs &a, long long rows, hipStream_t s);

}  // namespace tfno
