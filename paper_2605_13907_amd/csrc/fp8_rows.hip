// The FP8-E4M3 kernels that give one workgroup of 1,024 threads a whole row: the register-resident quantisation
// and the burst form of the dequantisation (further down).
//
// Register-resident FP8-E4M3 quantisation: the row is read from HBM once and held in the register file of
// one compute unit (1,024 threads x NV 16-byte vectors per lane) between the abs-max reduction that fixes
// the scale and the pass that encodes with it.  Rows of 25 to 33 vectors per lane keep their last 9 vectors
// per lane in LDS, filled by direct global -> LDS copies.  Same results as the streaming two-pass kernel in
// fp8.hip, which remains the route for rows that do not fit or are not 16-byte aligned.  (The fused rollout log-prob
// stays a streaming kernel: its second pass costs 18 vector instructions per element, about 18 us per row on one
// compute unit, and a workgroup that owns the whole unit cannot overlap that arithmetic with another row's loads:
// the register-resident form took 4.6 ms on 41,643 rows of 151,936 where two streaming passes take 3.6 ms.)
#include "ais_internal.h"
#include "device_utils.h"
#include "fp8_utils.h"

#include <type_traits>

namespace ais {
namespace {

using namespace dev;

constexpr int kRowThreads = 1024;
constexpr int kRowWaves = kRowThreads / 64;
constexpr int kSlotBytes = kRowThreads * 16;      // one LDS slot: a 16-byte vector per lane
constexpr int kLdsSlots = 9;                      // 144 KiB of the 160 KiB of a compute unit

typedef __attribute__((address_space(3))) void* lds_ptr;
typedef const __attribute__((address_space(1))) void* glb_ptr;

// Loads the row, returns its scale (abs-max / 448) to every thread.  q[] (vectors 0 .. NV - 1 of the lane), the
// LDS slots lrow (vectors NV .. NV + NL - 1, 16 bytes at index 1024 (k - NV) + tid) and xt hold the row afterwards.
// KFULL: the caller promises that the row has more than KFULL * 1024 vectors, so vectors 0 .. KFULL - 1 of every
// lane exist and are loaded without a bounds branch.
template <typename T, int NV, int NL, int KFULL>
__device__ __forceinline__ float load_row_and_scale(const T* zr, int vocab, u32x4 (&q)[NV], u32x4* lrow, float& xt,
                                                    float* lds) {
  constexpr int N = Vec<T>::N;
  const int tid = threadIdx.x;
  const int nvec = vocab / N;
  const int tail = vocab - nvec * N;
  const u32x4* zv = reinterpret_cast<const u32x4*>(zr);
  const u32x4 zero = {0u, 0u, 0u, 0u};
#pragma unroll
  for (int k = 0; k < NV; ++k) {
    const int i = tid + k * kRowThreads;
    if (k < KFULL) q[k] = load_stream(zv + i);
    else q[k] = (i < nvec) ? load_stream(zv + i) : zero;
  }
  if (NL > 0) {
    // lane i of a wavefront deposits its 16 bytes at the wavefront's base + 16 i: the slot layout; lanes past the
    // end of the row re-read its last vector (a valid address) and are masked where the slots are read
    int tid0 = tid;
    asm volatile("" : "+v"(tid0));
#pragma unroll
    for (int k = 0; k < NL; ++k) {
      const int i = min(tid0 + (NV + k) * kRowThreads, nvec - 1);
      __builtin_amdgcn_global_load_lds((glb_ptr)(zv + i), (lds_ptr)(lrow + k * kRowThreads + (tid0 & ~63)), 16, 0,
                                       2 /* non-temporal */);
      __builtin_amdgcn_sched_barrier(0);
    }
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
  if (NL > 0) {
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");     // the copies into the slots have landed
    int tid1 = tid;
    asm volatile("" : "+v"(tid1));
#pragma unroll
    for (int k = 0; k < NL; ++k) {
      // every slot holds data (lanes past the end of the row hold a copy of its last vector, which changes no
      // maximum); read without a branch, so that the reads stay in this order
      float x[N];
      Vec<T>::unpack(lrow[k * kRowThreads + tid1], x);
#pragma unroll
      for (int j = 0; j < N; ++j) amax = fmaxf(amax, fabsf(x[j]));
      __builtin_amdgcn_sched_barrier(0);
    }
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

template <typename T, int NV, int NL, int KFULL>
__global__ __launch_bounds__(kRowThreads) void fp8_quantize_row_kernel(const T* __restrict__ logits,
                                                                       long long row_stride, int vocab,
                                                                       unsigned char* __restrict__ codes,
                                                                       long long codes_stride,
                                                                       float* __restrict__ scale_out) {
  constexpr int N = Vec<T>::N;
  __shared__ float lds[kRowWaves];
  extern __shared__ __align__(16) unsigned char lds_slots[];
  u32x4* lrow = reinterpret_cast<u32x4*>(lds_slots);
  const long long row = blockIdx.x;
  const int tid = threadIdx.x;
  const T* zr = logits + row * row_stride;
  unsigned char* cr = codes + row * codes_stride;
  const int nvec = vocab / N;
  const int tail = vocab - nvec * N;
  u32x4 q[NV];
  float xt;
  const float s = load_row_and_scale<T, NV, NL, KFULL>(zr, vocab, q, lrow, xt, lds);
  if (tid == 0) scale_out[row] = s;
  const RowDivider d = make_divider(s);
  // vector indices from an opaque copy of the thread index, so that no per-vector offset stays alive from the loads
  int tid2 = tid;
  asm volatile("" : "+v"(tid2));
  auto encode = [&](auto slow) {
    constexpr bool SLOW = decltype(slow)::value;
    auto encode_vector = [&](u32x4 v, int i) {
      float x[N];
      Vec<T>::unpack(v, x);
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
    };
#pragma unroll
    for (int k = 0; k < NV; ++k) {
      encode_vector(q[k], tid2 + k * kRowThreads);
      __builtin_amdgcn_sched_barrier(0);
    }
    if (NL > 0) {
#pragma unroll
      for (int k = 0; k < NL; ++k) {
        encode_vector(lrow[k * kRowThreads + tid2], tid2 + (NV + k) * kRowThreads);
        __builtin_amdgcn_sched_barrier(0);
      }
    }
    if (tid < tail) cr[nvec * N + tid] = (unsigned char)(to_e4m3x2(divide<SLOW>(xt, d), 0.f) & 0xffu);
  };
  if (d.slow) encode(std::true_type{}); else encode(std::false_type{});
}

// ---- dequantise, burst form ------------------------------------------------------------------------------------
// out[n, v] = decode(code[n, v]) * scale[n].  One workgroup of 1,024 threads per row; every lane loads all of its
// code chunks (N codes each, N = elements of a 16-byte output vector), decodes them into output vectors held in
// registers, and only then issues all of its stores: the long same-direction bursts that a read+write stream needs
// on this device (see dlogits_burst_kernel).  Rows wider than NV * 1,024 vectors take NSEG such bursts, one after
// the other.  Vectors 0 .. KFULL - 1 of every lane are certain to exist.
template <typename T, int NV, int NSEG, int KFULL>
__global__ __launch_bounds__(kRowThreads) void fp8_dequantize_burst_kernel(const unsigned char* __restrict__ codes,
                                                                           long long codes_stride,
                                                                           const float* __restrict__ scale, int vocab,
                                                                           T* __restrict__ out, long long out_stride) {
  constexpr int N = Vec<T>::N;
  typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
  const long long row = blockIdx.x;
  const int tid = threadIdx.x;
  const unsigned char* cr = codes + row * codes_stride;
  T* orow = out + row * out_stride;
  u32x4* ov = reinterpret_cast<u32x4*>(orow);
  const float s = scale[row];
  const int nvec = vocab / N;
  const int tail = vocab - nvec * N;
#pragma unroll
  for (int seg = 0; seg < NSEG; ++seg) {
    uint32_t w[NV][N / 4];
#pragma unroll
    for (int k = 0; k < NV; ++k) {
      const int i = tid + (seg * NV + k) * kRowThreads;
      if (seg * NV + k < KFULL || i < nvec) {
        if (N == 8) {
          const u32x2 c = __builtin_nontemporal_load(reinterpret_cast<const u32x2*>(cr + (long long)i * N));
          w[k][0] = c[0];
          w[k][N / 4 - 1] = c[1];
        } else {
          w[k][0] = __builtin_nontemporal_load(reinterpret_cast<const uint32_t*>(cr + (long long)i * N));
        }
      } else {
#pragma unroll
        for (int j = 0; j < N / 4; ++j) w[k][j] = 0u;
      }
    }
    u32x4 q[NV];
#pragma unroll
    for (int k = 0; k < NV; ++k) {                // in order of arrival
      float x[N];
#pragma unroll
      for (int j = 0; j < N / 4; ++j) {
        const f32x2v lo = from_e4m3x2(w[k][j] & 0xffffu), hi = from_e4m3x2(w[k][j] >> 16);
        x[4 * j] = lo[0] * s;
        x[4 * j + 1] = lo[1] * s;
        x[4 * j + 2] = hi[0] * s;
        x[4 * j + 3] = hi[1] * s;
      }
      q[k] = Vec<T>::pack(x);
      __builtin_amdgcn_sched_barrier(0);
    }
    // every vector is made opaque here: no store can be issued before the last load has returned
#pragma unroll
    for (int k = 0; k < NV; ++k) asm volatile("" : "+v"(q[k]));
#pragma unroll
    for (int k = 0; k < NV; ++k) {
      const int i = tid + (seg * NV + k) * kRowThreads;
      if (seg * NV + k < KFULL || i < nvec) store_stream(ov + i, q[k]);
    }
  }
  if (tid < tail) Vec<T>::store1(orow + nvec * N + tid, from_e4m3x2(cr[nvec * N + tid])[0] * s);
}

template <typename T>
int vectors_per_lane(const void* z, int vocab, long long row_stride) {
  constexpr int N = Vec<T>::N;
  const bool ok16 = reinterpret_cast<uintptr_t>(z) % 16 == 0 && (row_stride * (long long)sizeof(T)) % 16 == 0;
  const int need = (vocab / N + kRowThreads - 1) / kRowThreads;
  return (ok16 && need <= 24 + kLdsSlots) ? (need < 1 ? 1 : need) : 0;
}

template <typename T, int NV, int NL, int KFULL>
bool launch_rows(ais_ctx* ctx, const T* z, long long n_rows, int vocab, long long row_stride, unsigned char* codes,
                 long long codes_stride, float* scale_out) {
  auto kernel = fp8_quantize_row_kernel<T, NV, NL, KFULL>;
  if (NL > 0) {
    static std::once_flag once[kMaxDevices];               // the attribute belongs to the function on one device
    static bool ok[kMaxDevices];
    if (!allow_dynamic_lds(ctx, reinterpret_cast<const void*>(kernel), NL * kSlotBytes, once, ok))
      return false;                                // the caller falls back to the streaming kernel
  }
  kernel<<<dim3((unsigned)n_rows), dim3(kRowThreads), NL * kSlotBytes, ctx->stream>>>(z, row_stride, vocab, codes,
                                                                                       codes_stride, scale_out);
  return true;
}

template <typename T>
bool dispatch_rows(ais_ctx* ctx, int need, const T* z, long long n_rows, int vocab, long long row_stride,
                   unsigned char* codes, long long codes_stride, float* scale_out) {
// PREV: the widest row of the previous class; a row that reaches this one has more than PREV * 1024 vectors
#define AIS_ROW_CASE(PREV, NEED, NVAL, NLVAL) \
  if (need <= NEED)                           \
    return launch_rows<T, NVAL, NLVAL, PREV>(ctx, z, n_rows, vocab, row_stride, codes, codes_stride, scale_out);
  AIS_ROW_CASE(0, 4, 4, 0)
  AIS_ROW_CASE(4, 8, 8, 0)
  AIS_ROW_CASE(8, 12, 12, 0)
  AIS_ROW_CASE(12, 16, 16, 0)
  AIS_ROW_CASE(16, 20, 20, 0)
  AIS_ROW_CASE(20, 24, 24, 0)
  AIS_ROW_CASE(24, 27, 18, kLdsSlots)
  AIS_ROW_CASE(27, 31, 22, kLdsSlots)
  AIS_ROW_CASE(31, 33, 24, kLdsSlots)
#undef AIS_ROW_CASE
  return false;
}

}  // namespace

// Returns true when the register-resident kernel was launched, false when the row does not qualify.
bool try_fp8_quantize_rows(ais_ctx* ctx, const void* logits, ais_dtype dtype, long long n_rows, int vocab,
                           long long row_stride, unsigned char* codes, long long codes_stride, float* scale_out) {
  const int store_align = dtype == AIS_BF16 ? 8 : 4;
  if (reinterpret_cast<uintptr_t>(codes) % store_align != 0 || codes_stride % store_align != 0) return false;
  if (dtype == AIS_BF16) {
    const int need = vectors_per_lane<bf16_t>(logits, vocab, row_stride);
    if (need == 0) return false;
    return dispatch_rows<bf16_t>(ctx, need, static_cast<const bf16_t*>(logits), n_rows, vocab, row_stride, codes,
                                 codes_stride, scale_out);
  }
  const int need = vectors_per_lane<float>(logits, vocab, row_stride);
  if (need == 0) return false;
  return dispatch_rows<float>(ctx, need, static_cast<const float*>(logits), n_rows, vocab, row_stride, codes,
                              codes_stride, scale_out);
}

// Returns true when the burst kernel was launched, false when the rows do not qualify (alignment, or wider than
// 48 output vectors per lane); the caller then runs the streaming kernel.
bool try_fp8_dequantize_burst(ais_ctx* ctx, const unsigned char* codes, long long codes_stride, const float* scale,
                              long long n_rows, int vocab, void* out, ais_dtype dtype, long long out_stride) {
  const int esize = dtype == AIS_BF16 ? 2 : 4;
  const int n = 16 / esize;                          // elements of an output vector = codes of a chunk
  if (reinterpret_cast<uintptr_t>(out) % 16 != 0 || (out_stride * esize) % 16 != 0) return false;
  if (reinterpret_cast<uintptr_t>(codes) % n != 0 || codes_stride % n != 0) return false;
  const int need = (vocab / n + kRowThreads - 1) / kRowThreads;
  dim3 grid((unsigned)n_rows), block(kRowThreads);
  // (vectors that surely exist, vectors per lane and burst, bursts): a row reaches a class only if it is wider than
  // the class before it
#define AIS_DEQ_CASE(KFULL, NVAL, NSEG)                                                                        \
  if (need <= NVAL * NSEG) {                                                                                   \
    if (dtype == AIS_BF16)                                                                                     \
      fp8_dequantize_burst_kernel<bf16_t, NVAL, NSEG, KFULL><<<grid, block, 0, ctx->stream>>>(                 \
          codes, codes_stride, scale, vocab, static_cast<bf16_t*>(out), out_stride);                           \
    else                                                                                                       \
      fp8_dequantize_burst_kernel<float, NVAL, NSEG, KFULL><<<grid, block, 0, ctx->stream>>>(                  \
          codes, codes_stride, scale, vocab, static_cast<float*>(out), out_stride);                            \
    return true;                                                                                               \
  }
  AIS_DEQ_CASE(0, 4, 1)
  AIS_DEQ_CASE(4, 8, 1)
  AIS_DEQ_CASE(8, 12, 1)
  AIS_DEQ_CASE(12, 16, 1)
  AIS_DEQ_CASE(16, 19, 1)
  AIS_DEQ_CASE(19, 20, 1)
  AIS_DEQ_CASE(20, 16, 2)
  AIS_DEQ_CASE(32, 16, 3)
#undef AIS_DEQ_CASE
  return false;
}

}  // namespace ais
