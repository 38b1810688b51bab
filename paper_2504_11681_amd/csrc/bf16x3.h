// Exact FP32 -> 3 x BF16 operand split for contractions on the BF16 matrix pipe with FP32 accuracy.
#pragma once
#include "common.h"

namespace tfno {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef unsigned int uintx4 __attribute__((ext_vector_type(4)));

// Exact 3-way split of an FP32 value into BF16-representable terms (truncation: hi bits of the remainder).
struct Split3 { float t0, t1, t2; };
__device__ __forceinline__ Split3 split3(float a)
{
    Split3 s;
    s.t0 = __uint_as_float(__float_as_uint(a) & 0xffff0000u);
    float r = a - s.t0;
    s.t1 = __uint_as_float(__float_as_uint(r) & 0xffff0000u);
    s.t2 = r - s.t1;     // at most 8 significant bits left: exactly a BF16 value
    return s;
}
// dword with BF16(lo) in bits 0-15 and BF16(hi) in bits 16-31 (operands already BF16-representable or truncated)
__device__ __forceinline__ unsigned pack_bf16(float lo, float hi)
{
    return __builtin_amdgcn_perm(__float_as_uint(hi), __float_as_uint(lo), 0x07060302u);
}

}  // namespace tfno
