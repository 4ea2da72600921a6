// Internal: the two divisions of the quantizer without the long IEEE division sequence.
//
// The quantizer is defined in IEEE binary32 operations (scale = f16((mx - mn) / qmax), inv = 1 / scale),
// and its results have to be bit-exact.  Both divisions have a tiny operand set, so cheaper sequences
// can be checked against the real division for every possible operand; cocktail_selftest_arithmetic
// does that on the device, and a test runs it.
#pragma once
#include <hip/hip_runtime.h>

namespace cocktail {

// r / qmax for qmax in {3, 15, 255} and 0 <= r <= 131008 (the largest difference of two fp16 values):
// multiply by the rounded reciprocal, then one correction step with the exact remainder.
// The result goes through an empty asm statement: the quantizer rounds it to fp16 next, and without
// the barrier the compiler merges the last fma with that conversion into one instruction that rounds
// once (fp32 product-sum straight to fp16), which differs from binary32-then-fp16 at fp16 ties.
template <int QMAX>
__device__ __forceinline__ float div_by_qmax(float r) {
#pragma clang fp contract(off)
  constexpr float c = 1.0f / float(QMAX);   // rounded to nearest at compile time
  const float q0 = r * c;
  const float rem = __builtin_fmaf(-q0, float(QMAX), r);
  float q = __builtin_fmaf(rem, c, q0);
  asm volatile("" : "+v"(q));
  return q;
}

// 1 / x for x = any positive finite fp16 value: hardware reciprocal (1 ulp) plus one Newton step.
__device__ __forceinline__ float recip_of_fp16_value(float x) {
#pragma clang fp contract(off)
  const float y = __builtin_amdgcn_rcpf(x);
  const float e = __builtin_fmaf(-x, y, 1.0f);
  return __builtin_fmaf(e, y, y);
}

}  // namespace cocktail
