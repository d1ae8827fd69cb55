// FP8-E4M3 per-row quantisation of logits: the rollout-side perturbation (Sec. 2.1; Eq. 1 with the E4M3
// value grid, q_max = 448, in place of the integer grid; per-row scale s = max|z| / 448).
//
//   fp8_quantize_kernel          z -> (codes, s)        read 2 * e * V (two passes over the row), write V
//   fp8_dequantize_kernel        (codes, s) -> z_r      read V, write e * V
//   fp8_rollout_logprob_kernel   z, y -> log softmax(z_r)[y] without materialising codes or z_r
//
// gfx950's conversion instructions implement the OCP E4M3 format (round to nearest even); inputs are
// clamped to +-448 first, so the conversion never sees an overflow.  The arithmetic that decides a code is
// fp32: s = max|z| / 448 and q = z / s, both correctly rounded divisions (q through the per-row divider of
// fp8_utils.h).  Rows that fit the register file take the single-read kernels of fp8_rows.hip.
#include "ais_internal.h"
#include "device_utils.h"
#include "fp8_utils.h"

#include <type_traits>

namespace ais {
namespace {

using namespace dev;

// Row abs-max -> scale, shared by the workgroup through LDS.
template <typename T, bool VEC>
__device__ __forceinline__ float row_scale(const T* zr, int vocab, float* lds) {
  constexpr int N = Vec<T>::N;
  const int tid = threadIdx.x;
  const int nvec = VEC ? vocab / N : 0;
  float amax = 0.f;
  if (VEC) {
    const u32x4* zv = reinterpret_cast<const u32x4*>(zr);
    for (int i = tid; i < nvec; i += kSweepThreads) {
      float x[N];
      Vec<T>::unpack(zv[i], x);      // cached load: the row is read again right away
#pragma unroll
      for (int k = 0; k < N; ++k) amax = fmaxf(amax, fabsf(x[k]));
    }
  }
  for (int v = nvec * N + tid; v < vocab; v += kSweepThreads) amax = fmaxf(amax, fabsf(Vec<T>::load1(zr + v)));
  amax = wave_max(amax);
  if ((tid & 63) == 0) lds[tid >> 6] = amax;
  __syncthreads();
  amax = fmaxf(fmaxf(lds[0], lds[1]), fmaxf(lds[2], lds[3]));
  return scale_of(amax);
}

template <typename T, bool VEC>
__global__ __launch_bounds__(kSweepThreads) void fp8_quantize_kernel(const T* __restrict__ logits, long long row_stride,
                                                                     int vocab, unsigned char* __restrict__ codes,
                                                                     long long codes_stride,
                                                                     float* __restrict__ scale_out) {
  constexpr int N = Vec<T>::N;
  __shared__ float lds[kSweepThreads / 64];
  const long long row = blockIdx.x;
  const int tid = threadIdx.x;
  const T* zr = logits + row * row_stride;
  unsigned char* cr = codes + row * codes_stride;
  const float s = row_scale<T, VEC>(zr, vocab, lds);
  if (tid == 0) scale_out[row] = s;
  const RowDivider d = make_divider(s);
  const int nvec = VEC ? vocab / N : 0;
  auto encode = [&](auto slow) {
    constexpr bool SLOW = decltype(slow)::value;
    if (VEC) {
      const u32x4* zv = reinterpret_cast<const u32x4*>(zr);
      for (int i = tid; i < nvec; i += kSweepThreads) {
        float x[N];
        Vec<T>::unpack(load_stream(zv + i), x);
        uint32_t w[N / 4];
#pragma unroll
        for (int k = 0; k < N / 4; ++k)
          w[k] = to_e4m3x2(divide<SLOW>(x[4 * k], d), divide<SLOW>(x[4 * k + 1], d)) |
                 (to_e4m3x2(divide<SLOW>(x[4 * k + 2], d), divide<SLOW>(x[4 * k + 3], d)) << 16);
        if (N == 8) {
          uint2 o = {w[0], w[N / 4 - 1]};
          *reinterpret_cast<uint2*>(cr + (long long)i * N) = o;
        } else {
          *reinterpret_cast<uint32_t*>(cr + (long long)i * N) = w[0];
        }
      }
    }
    for (int v = nvec * N + tid; v < vocab; v += kSweepThreads)
      cr[v] = (unsigned char)(to_e4m3x2(divide<SLOW>(Vec<T>::load1(zr + v), d), 0.f) & 0xffu);
  };
  if (d.slow) encode(std::true_type{}); else encode(std::false_type{});
}

template <typename T, bool VEC>
__global__ __launch_bounds__(kSweepThreads) void fp8_dequantize_kernel(const unsigned char* __restrict__ codes,
                                                                       long long codes_stride,
                                                                       const float* __restrict__ scale, int vocab,
                                                                       T* __restrict__ out, long long out_stride) {
  constexpr int N = Vec<T>::N;
  const long long row = blockIdx.x;
  const int tid = threadIdx.x;
  const unsigned char* cr = codes + row * codes_stride;
  T* orow = out + row * out_stride;
  const float s = scale[row];
  const int nvec = VEC ? vocab / N : 0;
  if (VEC) {
    u32x4* ov = reinterpret_cast<u32x4*>(orow);
    for (int i = tid; i < nvec; i += kSweepThreads) {
      uint32_t w[2];
      if (N == 8) {
        const uint2 c = *reinterpret_cast<const uint2*>(cr + (long long)i * N);
        w[0] = c.x;
        w[1] = c.y;
      } else {
        w[0] = *reinterpret_cast<const uint32_t*>(cr + (long long)i * N);
        w[1] = 0;
      }
      float x[N];
#pragma unroll
      for (int k = 0; k < N / 4; ++k) {
        const f32x2v lo = from_e4m3x2(w[k] & 0xffffu), hi = from_e4m3x2(w[k] >> 16);
        x[4 * k] = lo[0] * s;
        x[4 * k + 1] = lo[1] * s;
        x[4 * k + 2] = hi[0] * s;
        x[4 * k + 3] = hi[1] * s;
      }
      store_stream(ov + i, Vec<T>::pack(x));
    }
  }
  for (int v = nvec * N + tid; v < vocab; v += kSweepThreads) Vec<T>::store1(orow + v, from_e4m3x2(cr[v])[0] * s);
}

// log softmax(z_r)[y] with z_r = s * e4m3(z / s): abs-max pass, then a streaming log-sum-exp over the
// round-tripped values.
template <typename T, bool VEC>
__global__ __launch_bounds__(kSweepThreads) void fp8_rollout_logprob_kernel(
    const T* __restrict__ logits, long long row_stride, int vocab, const int* __restrict__ token_ids,
    const unsigned char* __restrict__ valid, float* __restrict__ logp_out, int* __restrict__ status) {
  constexpr int N = Vec<T>::N;
  __shared__ float lds[kSweepThreads / 64];
  __shared__ MaxSum lds_ms[kSweepThreads / 64];
  const long long row = blockIdx.x;
  const int tid = threadIdx.x;
  if (valid != nullptr && valid[row] == 0) {
    if (tid == 0) logp_out[row] = 0.f;
    return;
  }
  const T* zr = logits + row * row_stride;
  const float s = row_scale<T, VEC>(zr, vocab, lds);
  const RowDivider d = make_divider(s);
  const int nvec = VEC ? vocab / N : 0;
  MaxSum st{kNegHuge, 0.f};
  // the round-tripped logit is s * decode(code): the row scale is folded into the exponent's multiplier (s > 0,
  // so the running maximum can be taken over the decoded values)
  const float scale = s * kLog2e;
  auto sweep = [&](auto slow) {
    constexpr bool SLOW = decltype(slow)::value;
    if (VEC) {
      const u32x4* zv = reinterpret_cast<const u32x4*>(zr);
      for (int i = tid; i < nvec; i += kSweepThreads) {
        float x[N];
        Vec<T>::unpack(load_stream(zv + i), x);
#pragma unroll
        for (int k = 0; k < N; k += 2) {
          const f32x2v r = from_e4m3x2(to_e4m3x2(divide<SLOW>(x[k], d), divide<SLOW>(x[k + 1], d)));
          x[k] = r[0];
          x[k + 1] = r[1];
        }
        accumulate<N>(x, scale, st);
      }
    }
    for (int v = nvec * N + tid; v < vocab; v += kSweepThreads) {
      float x = from_e4m3x2(to_e4m3x2(divide<SLOW>(Vec<T>::load1(zr + v), d), 0.f))[0];
      accumulate<1>(&x, scale, st);
    }
  };
  if (d.slow) sweep(std::true_type{}); else sweep(std::false_type{});
  st = wave_merge(st);
  if ((tid & 63) == 0) lds_ms[tid >> 6] = st;
  __syncthreads();
  if (tid == 0) {
    MaxSum t = lds_ms[0];
#pragma unroll
    for (int w = 1; w < kSweepThreads / 64; ++w) t = merge(t, lds_ms[w]);
    const int y = token_ids[row];
    if (y >= 0 && y < vocab) {
      const float zy = from_e4m3x2(to_e4m3x2(Vec<T>::load1(zr + y) / s, 0.f))[0] * s;
      logp_out[row] = zy - (t.m + log2_fast(t.s)) * kLn2;
    } else {
      logp_out[row] = 0.f;
      atomicOr(status, AIS_STATUS_BAD_TOKEN);
    }
  }
}

bool aligned(const void* p, long long stride_bytes, int a) {
  return reinterpret_cast<uintptr_t>(p) % a == 0 && stride_bytes % a == 0;
}

}  // namespace

int launch_fp8_quantize(ais_ctx* ctx, const void* logits, ais_dtype dtype, long long n_rows, int vocab,
                        long long row_stride, unsigned char* codes, long long codes_stride, float* scale_out) {
  if (n_rows == 0) return AIS_OK;
  dim3 grid((unsigned)n_rows), block(kSweepThreads);
  ScopedTimer timer(ctx, AIS_K_FP8_QUANT);
  if (try_fp8_quantize_table(ctx, logits, dtype, n_rows, vocab, row_stride, codes, codes_stride, scale_out))
    return hip_fail(ctx, hipGetLastError());      // bf16 row held in registers, codes from a per-row table
  if (try_fp8_quantize_rows(ctx, logits, dtype, n_rows, vocab, row_stride, codes, codes_stride, scale_out))
    return hip_fail(ctx, hipGetLastError());      // row held in registers: one read of the logits
  if (dtype == AIS_BF16) {
    const bf16_t* z = static_cast<const bf16_t*>(logits);
    if (aligned(z, row_stride * 2, 16) && aligned(codes, codes_stride, 8))
      fp8_quantize_kernel<bf16_t, true><<<grid, block, 0, ctx->stream>>>(z, row_stride, vocab, codes, codes_stride, scale_out);
    else
      fp8_quantize_kernel<bf16_t, false><<<grid, block, 0, ctx->stream>>>(z, row_stride, vocab, codes, codes_stride, scale_out);
  } else {
    const float* z = static_cast<const float*>(logits);
    if (aligned(z, row_stride * 4, 16) && aligned(codes, codes_stride, 4))
      fp8_quantize_kernel<float, true><<<grid, block, 0, ctx->stream>>>(z, row_stride, vocab, codes, codes_stride, scale_out);
    else
      fp8_quantize_kernel<float, false><<<grid, block, 0, ctx->stream>>>(z, row_stride, vocab, codes, codes_stride, scale_out);
  }
  return hip_fail(ctx, hipGetLastError());
}

int launch_fp8_dequantize(ais_ctx* ctx, const unsigned char* codes, long long codes_stride, const float* scale,
                          long long n_rows, int vocab, void* out, ais_dtype dtype, long long out_stride) {
  if (n_rows == 0) return AIS_OK;
  dim3 grid((unsigned)n_rows), block(kSweepThreads);
  ScopedTimer timer(ctx, AIS_K_FP8_DEQUANT);
  if (try_fp8_dequantize_burst(ctx, codes, codes_stride, scale, n_rows, vocab, out, dtype, out_stride))
    return hip_fail(ctx, hipGetLastError());
  if (dtype == AIS_BF16) {
    bf16_t* o = static_cast<bf16_t*>(out);
    if (aligned(o, out_stride * 2, 16) && aligned(codes, codes_stride, 8))
      fp8_dequantize_kernel<bf16_t, true><<<grid, block, 0, ctx->stream>>>(codes, codes_stride, scale, vocab, o, out_stride);
    else
      fp8_dequantize_kernel<bf16_t, false><<<grid, block, 0, ctx->stream>>>(codes, codes_stride, scale, vocab, o, out_stride);
  } else {
    float* o = static_cast<float*>(out);
    if (aligned(o, out_stride * 4, 16) && aligned(codes, codes_stride, 4))
      fp8_dequantize_kernel<float, true><<<grid, block, 0, ctx->stream>>>(codes, codes_stride, scale, vocab, o, out_stride);
    else
      fp8_dequantize_kernel<float, false><<<grid, block, 0, ctx->stream>>>(codes, codes_stride, scale, vocab, o, out_stride);
  }
  return hip_fail(ctx, hipGetLastError());
}

int launch_fp8_rollout_logprob(ais_ctx* ctx, const void* logits, ais_dtype dtype, long long n_rows, int vocab,
                               long long row_stride, const int* token_ids, const unsigned char* valid,
                               float* logp_out) {
  if (n_rows == 0) return AIS_OK;
  dim3 grid((unsigned)n_rows), block(kSweepThreads);
  ScopedTimer timer(ctx, AIS_K_FP8_LOGPROB);
  if (try_fp8_rollout_logprob_table(ctx, logits, dtype, n_rows, vocab, row_stride, token_ids, valid, logp_out))
    return hip_fail(ctx, hipGetLastError());      // bf16 row read once, terms of the sum from a per-row table
  if (dtype == AIS_BF16) {
    const bf16_t* z = static_cast<const bf16_t*>(logits);
    if (aligned(z, row_stride * 2, 16))
      fp8_rollout_logprob_kernel<bf16_t, true><<<grid, block, 0, ctx->stream>>>(z, row_stride, vocab, token_ids, valid, logp_out, ctx->status_dev);
    else
      fp8_rollout_logprob_kernel<bf16_t, false><<<grid, block, 0, ctx->stream>>>(z, row_stride, vocab, token_ids, valid, logp_out, ctx->status_dev);
  } else {
    const float* z = static_cast<const float*>(logits);
    if (aligned(z, row_stride * 4, 16))
      fp8_rollout_logprob_kernel<float, true><<<grid, block, 0, ctx->stream>>>(z, row_stride, vocab, token_ids, valid, logp_out, ctx->status_dev);
    else
      fp8_rollout_logprob_kernel<float, false><<<grid, block, 0, ctx->stream>>>(z, row_stride, vocab, token_ids, valid, logp_out, ctx->status_dev);
  }
  return hip_fail(ctx, hipGetLastError());
}

}  // namespace ais
