// Register-resident FP8-E4M3 quantisation: the row is read from HBM once and held in the register file of
// one compute unit (1,024 threads x NV 16-byte vectors per lane) between the abs-max reduction that fixes
// the scale and the pass that encodes with it.  Same results as the streaming two-pass kernel in fp8.hip,
// which remains the route for rows that do not fit or are not 16-byte aligned.  (The fused rollout log-prob
// stays a streaming kernel: its second pass is bound by arithmetic, and a workgroup that owns a whole compute
// unit cannot overlap that arithmetic with another row's loads; measured slower than two streaming passes.)
#include "ais_internal.h"
#include "device_utils.h"
#include "fp8_utils.h"

#include <type_traits>

namespace ais {
namespace {

using namespace dev;

constexpr int kRowThreads = 1024;
constexpr int kRowWaves = kRowThreads / 64;

// Loads the row, returns its scale (abs-max / 448) to every thread.  q[] and xt hold the row afterwards.
template <typename T, int NV>
__device__ __forceinline__ float load_row_and_scale(const T* zr, int vocab, u32x4 (&q)[NV], float& xt, float* lds) {
  constexpr int N = Vec<T>::N;
  const int tid = threadIdx.x;
  const int nvec = vocab / N;
  const int tail = vocab - nvec * N;
  const u32x4* zv = reinterpret_cast<const u32x4*>(zr);
  const u32x4 zero = {0u, 0u, 0u, 0u};
#pragma unroll
  for (int k = 0; k < NV; ++k) {
    const int i = tid + k * kRowThreads;
    q[k] = (i < nvec) ? load_stream(zv + i) : zero;
  }
  xt = (tid < tail) ? Vec<T>::load1(zr + nvec * N + tid) : 0.f;
  float amax = fabsf(xt);
#pragma unroll
  for (int k = 0; k < NV; ++k) {
    float x[N];
    Vec<T>::unpack(q[k], x);
#pragma unroll
    for (int j = 0; j < N; ++j) amax = fmaxf(amax, fabsf(x[j]));
    __builtin_amdgcn_sched_barrier(0);
  }
  amax = wave_max(amax);
  if ((tid & 63) == 0) lds[tid >> 6] = amax;
  __syncthreads();
  amax = lds[0];
#pragma unroll
  for (int w = 1; w < kRowWaves; ++w) amax = fmaxf(amax, lds[w]);
  const float s = scale_of(amax);
  // Keep the row packed until the scale is known: the empty asm, which names the scale as an input, stops
  // the compiler from unpacking every vector ahead of the reduction (twice the registers for bf16).
#pragma unroll
  for (int k = 0; k < NV; ++k) asm volatile("" : "+v"(q[k]) : "v"(s));
  return s;
}

template <typename T, int NV>
__global__ __launch_bounds__(kRowThreads) void fp8_quantize_row_kernel(const T* __restrict__ logits,
                                                                       long long row_stride, int vocab,
                                                                       unsigned char* __restrict__ codes,
                                                                       long long codes_stride,
                                                                       float* __restrict__ scale_out) {
  constexpr int N = Vec<T>::N;
  __shared__ float lds[kRowWaves];
  const long long row = blockIdx.x;
  const int tid = threadIdx.x;
  const T* zr = logits + row * row_stride;
  unsigned char* cr = codes + row * codes_stride;
  const int nvec = vocab / N;
  const int tail = vocab - nvec * N;
  u32x4 q[NV];
  float xt;
  const float s = load_row_and_scale<T, NV>(zr, vocab, q, xt, lds);
  if (tid == 0) scale_out[row] = s;
  const RowDivider d = make_divider(s);
  auto encode = [&](auto slow) {
    constexpr bool SLOW = decltype(slow)::value;
#pragma unroll
    for (int k = 0; k < NV; ++k) {
      const int i = tid + k * kRowThreads;
      float x[N];
      Vec<T>::unpack(q[k], x);
      uint32_t w[N / 4];
#pragma unroll
      for (int j = 0; j < N / 4; ++j)
        w[j] = to_e4m3x2(divide<SLOW>(x[4 * j], d), divide<SLOW>(x[4 * j + 1], d)) |
               (to_e4m3x2(divide<SLOW>(x[4 * j + 2], d), divide<SLOW>(x[4 * j + 3], d)) << 16);
      if (i < nvec) {
        if (N == 8) {
          uint2 o = {w[0], w[N / 4 - 1]};
          *reinterpret_cast<uint2*>(cr + (long long)i * N) = o;
        } else {
          *reinterpret_cast<uint32_t*>(cr + (long long)i * N) = w[0];
        }
      }
      __builtin_amdgcn_sched_barrier(0);
    }
    if (tid < tail) cr[nvec * N + tid] = (unsigned char)(to_e4m3x2(divide<SLOW>(xt, d), 0.f) & 0xffu);
  };
  if (d.slow) encode(std::true_type{}); else encode(std::false_type{});
}

template <typename T>
int vectors_per_lane(const void* z, int vocab, long long row_stride) {
  constexpr int N = Vec<T>::N;
  const bool ok16 = reinterpret_cast<uintptr_t>(z) % 16 == 0 && (row_stride * (long long)sizeof(T)) % 16 == 0;
  const int need = (vocab / N + kRowThreads - 1) / kRowThreads;
  return (ok16 && need <= 24) ? (need < 1 ? 1 : need) : 0;
}

#define AIS_ROW_DISPATCH(NEED, CALL)          \
  if (NEED <= 4) { CALL(4) }                  \
  else if (NEED <= 8) { CALL(8) }             \
  else if (NEED <= 12) { CALL(12) }           \
  else if (NEED <= 16) { CALL(16) }           \
  else if (NEED <= 20) { CALL(20) }           \
  else { CALL(24) }

}  // namespace

// Returns true when the register-resident kernel was launched, false when the row does not qualify.
bool try_fp8_quantize_rows(ais_ctx* ctx, const void* logits, ais_dtype dtype, long long n_rows, int vocab,
                           long long row_stride, unsigned char* codes, long long codes_stride, float* scale_out) {
  const int store_align = dtype == AIS_BF16 ? 8 : 4;
  if (reinterpret_cast<uintptr_t>(codes) % store_align != 0 || codes_stride % store_align != 0) return false;
  dim3 grid((unsigned)n_rows), block(kRowThreads);
  if (dtype == AIS_BF16) {
    const int need = vectors_per_lane<bf16_t>(logits, vocab, row_stride);
    if (need == 0) return false;
    const bf16_t* z = static_cast<const bf16_t*>(logits);
#define CALL(NVAL) fp8_quantize_row_kernel<bf16_t, NVAL><<<grid, block, 0, ctx->stream>>>(z, row_stride, vocab, codes, codes_stride, scale_out);
    AIS_ROW_DISPATCH(need, CALL)
#undef CALL
  } else {
    const int need = vectors_per_lane<float>(logits, vocab, row_stride);
    if (need == 0) return false;
    const float* z = static_cast<const float*>(logits);
#define CALL(NVAL) fp8_quantize_row_kernel<float, NVAL><<<grid, block, 0, ctx->stream>>>(z, row_stride, vocab, codes, codes_stride, scale_out);
    AIS_ROW_DISPATCH(need, CALL)
#undef CALL
  }
  return true;
}

}  // namespace ais
