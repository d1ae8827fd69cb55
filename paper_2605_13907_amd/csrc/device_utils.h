// Device-side helpers shared by the sweep kernels: 16-byte vector access to bf16 / fp32 rows,
// wavefront reductions, and the running (max, sum) state of the streaming log-sum-exp.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ais {
namespace dev {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef uint16_t bf16_t;   // raw storage of a bfloat16

constexpr float kNegHuge = -3.0e38f;   // initial running maximum: a finite stand-in for -inf keeps (max - max) free of NaN
// Value of an element that is excluded from a soft-max sum (the sampled token's own term, positions past the end of a
// row): it never raises a maximum above the finite running one and adds exactly 2^(-inf) = 0.  A huge finite value
// would not do: for a lane that has seen nothing else the new maximum is the rounded product x * scale, the fma that
// forms x * scale - max keeps the product exact, and what is left of that rounding is astronomically large there.
constexpr float kMasked = -__builtin_inff();

__device__ __forceinline__ float exp2_fast(float x) { return __builtin_amdgcn_exp2f(x); }
__device__ __forceinline__ float log2_fast(float x) { return __builtin_amdgcn_logf(x); }

// log(1 + s * 2^e) for s >= 0, in fp64, without overflow when e is large (a sampled token thousands of units
// below the row maximum makes s * 2^e exceed the range of a double, while its logarithm is an ordinary number).
// Beyond 2^64 the "1 +" is below fp64 resolution and the logarithm is taken directly; the fp32 log2 of s there
// costs a relative 1e-7 of a result that is at least 44.
__device__ __forceinline__ double log1p_scaled(float s, double e) {
  const double l2 = e + (double)log2_fast(s);      // log2 of the ratio; -inf when s == 0
  if (l2 > 64.0) return l2 * 0.6931471805599453;
  return s > 0.f ? log1p((double)s * exp2(e)) : 0.0;   // here e <= 64 + 149: 2^e is finite
}

__device__ __forceinline__ u32x4 load_stream(const u32x4* p) { return __builtin_nontemporal_load(p); }
__device__ __forceinline__ void store_stream(u32x4* p, u32x4 v) { __builtin_nontemporal_store(v, p); }

template <typename T> struct Vec;
template <> struct Vec<bf16_t> {
  static constexpr int N = 8;
  static __device__ __forceinline__ void unpack(u32x4 q, float* x) {
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      x[2 * k] = __uint_as_float(q[k] << 16);
      x[2 * k + 1] = __uint_as_float(q[k] & 0xffff0000u);
    }
  }
  static __device__ __forceinline__ u32x4 pack(const float* x) {   // round to nearest even
    u32x4 q;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      f32x2 f = {x[2 * k], x[2 * k + 1]};
      q[k] = __builtin_bit_cast(uint32_t, __builtin_convertvector(f, bf16x2));
    }
    return q;
  }
  // q with element `sub` replaced by v (rounded to nearest even)
  static __device__ __forceinline__ u32x4 put(u32x4 q, int sub, float v) {
    const uint32_t h = __builtin_bit_cast(uint16_t, static_cast<__bf16>(v));
    const uint32_t keep = (sub & 1) ? 0x0000ffffu : 0xffff0000u;
    const uint32_t bits = (sub & 1) ? (h << 16) : h;
#pragma unroll
    for (int w = 0; w < 4; ++w)
      if (w == (sub >> 1)) q[w] = (q[w] & keep) | bits;
    return q;
  }
  static __device__ __forceinline__ float load1(const bf16_t* p) { return __uint_as_float(uint32_t(*p) << 16); }
  static __device__ __forceinline__ void store1(bf16_t* p, float v) {
    *p = __builtin_bit_cast(uint16_t, static_cast<__bf16>(v));
  }
};
template <> struct Vec<float> {
  static constexpr int N = 4;
  static __device__ __forceinline__ void unpack(u32x4 q, float* x) {
#pragma unroll
    for (int k = 0; k < 4; ++k) x[k] = __uint_as_float(q[k]);
  }
  static __device__ __forceinline__ u32x4 pack(const float* x) {
    u32x4 q;
#pragma unroll
    for (int k = 0; k < 4; ++k) q[k] = __float_as_uint(x[k]);
    return q;
  }
  static __device__ __forceinline__ u32x4 put(u32x4 q, int sub, float v) {
#pragma unroll
    for (int w = 0; w < 4; ++w)
      if (w == sub) q[w] = __float_as_uint(v);
    return q;
  }
  static __device__ __forceinline__ float load1(const float* p) { return *p; }
  static __device__ __forceinline__ void store1(float* p, float v) { *p = v; }
};

// ---- wavefront reductions ----------------------------------------------------------------------
// Lane exchange inside a row of 16 lanes goes through DPP (no LDS traffic); the two steps across
// rows use ds_bpermute via __shfl_xor.
template <int CTRL>
__device__ __forceinline__ float dpp_move(float v) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xf, 0xf, true));
}
constexpr int kDppQuadXor1 = 0xB1;      // quad_perm [1,0,3,2]
constexpr int kDppQuadXor2 = 0x4E;      // quad_perm [2,3,0,1]
constexpr int kDppRowHalfMirror = 0x141;
constexpr int kDppRowMirror = 0x140;

// Running log-sum-exp state in base 2: the row's sum of 2^(t_v) equals s * 2^m.
struct MaxSum {
  float m, s;
};
__device__ __forceinline__ MaxSum merge(MaxSum a, MaxSum b) {
  float m = fmaxf(a.m, b.m);
  return {m, a.s * exp2_fast(a.m - m) + b.s * exp2_fast(b.m - m)};
}
template <int CTRL>
__device__ __forceinline__ MaxSum merge_dpp(MaxSum a) {
  return merge(a, MaxSum{dpp_move<CTRL>(a.m), dpp_move<CTRL>(a.s)});
}
__device__ __forceinline__ MaxSum wave_merge(MaxSum a) {
  a = merge_dpp<kDppQuadXor1>(a);
  a = merge_dpp<kDppQuadXor2>(a);
  a = merge_dpp<kDppRowHalfMirror>(a);
  a = merge_dpp<kDppRowMirror>(a);
  a = merge(a, MaxSum{__shfl_xor(a.m, 16), __shfl_xor(a.s, 16)});
  a = merge(a, MaxSum{__shfl_xor(a.m, 32), __shfl_xor(a.s, 32)});
  return a;
}

// Folds `n` unpacked logits into the running state with one rescale of the old sum.
template <int n>
__device__ __forceinline__ void accumulate(const float* x, float scale, MaxSum& st) {
  float cm = x[0];
#pragma unroll
  for (int k = 1; k < n; ++k) cm = fmaxf(cm, x[k]);
  const float mn = fmaxf(st.m, cm * scale);
  float acc0 = st.s * exp2_fast(st.m - mn), acc1 = 0.f;
#pragma unroll
  for (int k = 0; k < n; k += 2) {
    acc0 += exp2_fast(__builtin_fmaf(x[k], scale, -mn));
    if (k + 1 < n) acc1 += exp2_fast(__builtin_fmaf(x[k + 1], scale, -mn));
  }
  st.m = mn;
  st.s = acc0 + acc1;
}


// Wavefront-wide maximum, same exchange pattern as wave_merge.
__device__ __forceinline__ float wave_max(float v) {
  v = fmaxf(v, dpp_move<kDppQuadXor1>(v));
  v = fmaxf(v, dpp_move<kDppQuadXor2>(v));
  v = fmaxf(v, dpp_move<kDppRowHalfMirror>(v));
  v = fmaxf(v, dpp_move<kDppRowMirror>(v));
  v = fmaxf(v, __shfl_xor(v, 16));
  v = fmaxf(v, __shfl_xor(v, 32));
  return v;
}

// Wavefront-wide sum, same exchange pattern; every lane holds the result.
__device__ __forceinline__ float wave_sum(float v) {
  v += dpp_move<kDppQuadXor1>(v);
  v += dpp_move<kDppQuadXor2>(v);
  v += dpp_move<kDppRowHalfMirror>(v);
  v += dpp_move<kDppRowMirror>(v);
  v += __shfl_xor(v, 16);
  v += __shfl_xor(v, 32);
  return v;
}

}  // namespace dev
}  // namespace ais
