#pragma once
#include "common.h"
namespace tfno {
size_t staged_workspace_bytes(long long B, int C_in, int C_out, int N1, int N2, int K1, int K2);
// Generic radix-2 LDS transform of strided pencils with optional built-in zero padding (n_in < N) and
// truncation (n_out < N); see the kernel comment in staged.hip for the addressing.
hipError_t launch_axis_fft(int dir, const c64 *in, c64 *out, int N, long long num_pencils,
                           long long inner_count, long long in_outer_stride, long long out_outer_stride,
                           long long elem_stride, int n_in, int n_out, float scale, hipStream_t s);
// N1 x N2 points keeping K1 x K2 modes; 1-D calls pass N1 = K1 = 1.
hipError_t staged_conv(int dims, const c64 *x, const c64 *W, c64 *y, long long B, int C_in, int C_out,
                       int N1, int N2, int K1, int K2, c64 *ws, hipStream_t s);
}
