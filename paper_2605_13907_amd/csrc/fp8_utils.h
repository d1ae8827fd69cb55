// Device helpers of the FP8-E4M3 kernels: conversions and a correctly rounded division by a per-row scale.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ais {
namespace dev {

typedef float f32x2v __attribute__((ext_vector_type(2)));
constexpr float kE4M3Max = 448.f;

__device__ __forceinline__ float clamp448(float q) { return __builtin_amdgcn_fmed3f(q, -kE4M3Max, kE4M3Max); }

// two fp32 -> two E4M3 codes in the low 16 bits (round to nearest even; inputs clamped, so no overflow case)
__device__ __forceinline__ uint32_t to_e4m3x2(float a, float b) {
  return (uint32_t)__builtin_amdgcn_cvt_pk_fp8_f32(clamp448(a), clamp448(b), 0, false) & 0xffffu;
}
__device__ __forceinline__ f32x2v from_e4m3x2(uint32_t w) { return __builtin_amdgcn_cvt_pk_f32_fp8((int)w, false); }

__device__ __forceinline__ float scale_of(float amax) {
  const float s = amax / kE4M3Max;
  return s > 0.f ? s : 1.f;
}

// x / s, correctly rounded, for many x and one s.  With r = RN(1 / s) (one true division per row):
//   q0 = RN(x r)                       within about 1.5 ulp of the quotient
//   q1 = RN(q0 + (x - q0 s) r)         a faithful quotient (error below one ulp); the residual in an fma
//   q  = RN(q1 + (x - q1 s) r)         the residual of a faithful quotient is exact in an fma, and with a
//                                      correctly rounded reciprocal this last step yields the correctly
//                                      rounded quotient (Markstein's theorem on division by fma correction)
// The theorem excludes a divisor whose significand is all ones, and the argument needs r and the residuals
// to stay clear of overflow and the subnormal range: those rows take the true division.  The quotient's
// sign is copied from x, so that -0 stays -0.
struct RowDivider {
  float s, r;
  bool slow;
};
__device__ __forceinline__ RowDivider make_divider(float s) {
  const uint32_t bits = __float_as_uint(s);
  const int expo = (int)((bits >> 23) & 0xffu) - 127;
  RowDivider d;
  d.s = s;
  d.r = 1.0f / s;
  d.slow = ((bits & 0x7fffffu) == 0x7fffffu) || expo < -60 || expo > 60;
  return d;
}
// SLOW is a compile-time choice so that the loops that call this stay free of control flow; kernels branch
// once per row on d.slow and run one of two copies of their loop.
template <bool SLOW>
__device__ __forceinline__ float divide(float x, const RowDivider& d) {
  if (SLOW) return x / d.s;
  const float q0 = x * d.r;
  const float q1 = __builtin_fmaf(__builtin_fmaf(-q0, d.s, x), d.r, q0);
  const float q = __builtin_fmaf(__builtin_fmaf(-q1, d.s, x), d.r, q1);
  return __builtin_copysignf(q, x);
}

}  // namespace dev
}  // namespace ais
