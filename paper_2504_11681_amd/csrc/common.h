// Shared device/host helpers for the tfno HIP library (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace tfno {

#define TFNO_HD __host__ __device__ __forceinline__

typedef float2 c64;   // interleaved complex64: x = re, y = im

TFNO_HD c64 cadd(c64 a, c64 b) { return make_float2(a.x + b.x, a.y + b.y); }
TFNO_HD c64 csub(c64 a, c64 b) { return make_float2(a.x - b.x, a.y - b.y); }
// a * b  (two multiplies + two fused multiply-adds)
TFNO_HD c64 cmul(c64 a, c64 b)
{
    return make_float2(fmaf(a.x, b.x, -(a.y * b.y)), fmaf(a.x, b.y, a.y * b.x));
}
// acc + a * b
TFNO_HD c64 cmac(c64 acc, c64 a, c64 b)
{
    float re = fmaf(a.x, b.x, acc.x);
    re = fmaf(-a.y, b.y, re);
    float im = fmaf(a.x, b.y, acc.y);
    im = fmaf(a.y, b.x, im);
    return make_float2(re, im);
}
// exp(2 pi i * num / den) with one accurate sincospi evaluation
__device__ __forceinline__ c64 cis2pi(float num, float den)
{
    float s, c;
    sincospif(2.0f * num / den, &s, &c);
    return make_float2(c, s);
}

}  // namespace tfno
