// Shared device/host helpers for the tfno HIP library (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <initializer_list>
#include <mutex>

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
// Streaming (non-temporal) store for an output tensor that the kernel writes exactly once: the line is not kept in
// the 256 MB last-level cache, whose write-back of a previous launch's dirty output otherwise lands in the read
// phase of the next launch (symmetric N = 1024 kernel at the sustained clock: 125 us with plain stores, 112 us with
// these).
typedef float tfno_vf2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ void store_nt(c64 *p, c64 v)
{
    tfno_vf2 t;
    t.x = v.x;
    t.y = v.y;
    __builtin_nontemporal_store(t, reinterpret_cast<tfno_vf2 *>(p));
}

// The same hint for an input that is read exactly once (the symmetric N = 1024 kernel gains 2 % from it, the other
// kernels nothing, so only that one uses it).
__device__ __forceinline__ c64 load_nt(const c64 *p)
{
    const tfno_vf2 t = __builtin_nontemporal_load(reinterpret_cast<const tfno_vf2 *>(p));
    return make_float2(t.x, t.y);
}

// Workgroup ids are dealt round-robin to the 8 XCDs (id % 8).  This maps a launch index to a work item so that the
// workgroups resident on one XCD own a CONTIGUOUS range of items instead of every eighth one.  With items that are
// 0.5-1 MiB apart in memory (batch rows, images), every eighth item shares the address bits that select the
// memory channel group, so each XCD would talk to a fraction of the channels and the XCDs finish the write phase up
// to 10 us apart (production 1-D shape: 105 us -> 99 us with this mapping).  It pays for the N = 1024 kernels (one
// workgroup per CU, 1 MiB per batch row); the kernels that keep several smaller workgroups per CU (N = 256, the
// 2-D image kernels) measured 5-10 % slower with it and keep the identity mapping.
__device__ __forceinline__ unsigned xcd_contiguous(unsigned id, unsigned n)
{
    const unsigned q = n >> 3, r = n & 7, x = id & 7;
    return x * q + (x < r ? x : r) + (id >> 3);
}

// Raises the dynamic-LDS limit of a launch site's kernels exactly once per process, whichever host thread gets
// there first (std::call_once); later calls return the result of that one attempt.
struct LdsLimitOnce {
    std::once_flag flag;
    hipError_t result = hipSuccess;
    hipError_t set(std::initializer_list<const void *> kernels, int bytes)
    {
        std::call_once(flag, [&] {
            for (const void *k : kernels) {
                result = hipFuncSetAttribute(k, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
                if (result != hipSuccess) return;
            }
        });
        return result;
    }
};

// exp(2 pi i * num / den) with one accurate sincospi evaluation
__device__ __forceinline__ c64 cis2pi(float num, float den)
{
    float s, c;
    sincospif(2.0f * num / den, &s, &c);
    return make_float2(c, s);
}

}  // namespace tfno
