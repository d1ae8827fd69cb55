// The two vocabulary sweeps of the path, and a plain copy kernel used as a bandwidth yardstick.
//
//   token_logprob_kernel   one pass over a logits row with a running (max, sum) pair:
//                          lse = log sum_v exp(z_v / T), logp = z_y / T - lse, the latter evaluated as
//                          -log1p(sum_{v != y} exp((z_v - z_y) / T))
//                          (Alg. 1, "Compute full-precision log-probs")
//   dlogits_kernel         second pass: dz_v = g (softmax_v - 1[v = y]) / T, written in the logits'
//                          dtype (gradient of Eq. 19 through the log-softmax; g is the row's coefficient)
//
// Both are bound by HBM bandwidth: nothing here is a contraction, so no matrix cores.  One workgroup
// of 256 threads (4 wavefronts of 64) owns one row, so a row's partial results never leave its
// compute unit; consecutive lanes read consecutive 16-byte vectors (8 bf16 or 4 fp32 logits), i.e.
// each wavefront load instruction covers 1 KiB of contiguous memory.  Logits are read and written
// with streaming (non-temporal) accesses: a batch is tens of GB and nothing survives in cache
// between the two sweeps.
#include "ais_internal.h"

namespace ais {
namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef uint16_t bf16_t;   // raw storage of a bfloat16

constexpr float kNegHuge = -3.0e38f;   // finite stand-in for -inf: keeps (max - max) free of NaN

__device__ __forceinline__ float exp2_fast(float x) { return __builtin_amdgcn_exp2f(x); }
__device__ __forceinline__ float log2_fast(float x) { return __builtin_amdgcn_logf(x); }

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

// ---- sweep 1: token log-probability --------------------------------------------------------------
// grid.x = n_rows, block = kSweepThreads.  VEC: 16-byte vector path (row base and pitch 16-byte aligned).
template <typename T, bool VEC, int UNROLL>
__global__ __launch_bounds__(kSweepThreads) void token_logprob_kernel(
    const T* __restrict__ logits, long long row_stride, int vocab, const int* __restrict__ token_ids,
    const unsigned char* __restrict__ valid, float inv_temperature, float* __restrict__ logp_out,
    float* __restrict__ lse_out, int* __restrict__ status) {
  constexpr int N = Vec<T>::N;
  const long long row = blockIdx.x;
  const int tid = threadIdx.x;
  if (valid != nullptr && valid[row] == 0) {      // not evaluated: neither the row nor its token is read
    if (tid == 0) {
      logp_out[row] = 0.f;
      lse_out[row] = 0.f;
    }
    return;
  }
  const T* zr = logits + row * row_stride;
  const float scale = inv_temperature * kLog2e;   // 2^(z * scale) = exp(z / T)

  // The sampled token's own term is kept out of the running sum: with S_o = sum over the other tokens,
  // logp = -log1p(S_o / e^{z_y/T}) keeps its relative accuracy when the row is sharply peaked (p_y -> 1),
  // where z_y/T - lse would cancel.  Its logit is loaded first so that the latency hides behind the sweep.
  const int y = token_ids[row];
  const bool y_ok = (y >= 0) && (y < vocab);
  const float zy = y_ok ? Vec<T>::load1(zr + y) : 0.f;
  const int nvec = VEC ? vocab / N : 0;
  // vector index at which this thread meets the sampled token, or a value no index ever takes
  const int yvec = (y_ok && y < nvec * N && (y / N) % kSweepThreads == tid) ? y / N : -(1 << 30);
  const int ysub = y % N;

  MaxSum st{kNegHuge, 0.f};
  if (VEC) {
    const u32x4* zv = reinterpret_cast<const u32x4*>(zr);
    int i = tid;
    for (; i + (UNROLL - 1) * kSweepThreads < nvec; i += UNROLL * kSweepThreads) {
      u32x4 q[UNROLL];
#pragma unroll
      for (int u = 0; u < UNROLL; ++u) q[u] = load_stream(zv + i + u * kSweepThreads);
      float x[UNROLL * N];
#pragma unroll
      for (int u = 0; u < UNROLL; ++u) Vec<T>::unpack(q[u], x + u * N);
      if ((unsigned)(yvec - i) < (unsigned)(UNROLL * kSweepThreads)) {   // rare: once per row, one lane
        const int hit = ((yvec - i) / kSweepThreads) * N + ysub;
#pragma unroll
        for (int k = 0; k < UNROLL * N; ++k)
          if (k == hit) x[k] = kNegHuge;
      }
      accumulate<UNROLL * N>(x, scale, st);
    }
    for (; i < nvec; i += kSweepThreads) {
      float x[N];
      Vec<T>::unpack(load_stream(zv + i), x);
      if (i == yvec) {
#pragma unroll
        for (int k = 0; k < N; ++k)
          if (k == ysub) x[k] = kNegHuge;
      }
      accumulate<N>(x, scale, st);
    }
  }
  for (int v = nvec * N + tid; v < vocab; v += kSweepThreads) {   // ragged tail, or the whole row when !VEC
    float x = (y_ok && v == y) ? kNegHuge : Vec<T>::load1(zr + v);
    accumulate<1>(&x, scale, st);
  }

  st = wave_merge(st);
  __shared__ MaxSum lds[kSweepThreads / 64];
  if ((tid & 63) == 0) lds[tid >> 6] = st;
  __syncthreads();
  if (tid == 0) {
    MaxSum t = lds[0];
#pragma unroll
    for (int w = 1; w < kSweepThreads / 64; ++w) t = merge(t, lds[w]);
    if (y_ok) {
      // once per row, in fp64: r = S_o / e^{z_y/T};  logp = -log1p(r);  lse = z_y/T + log1p(r)
      const double ty = (double)zy * (double)scale;
      const double r = (double)t.s * exp2((double)t.m - ty);
      const double l1p = log1p(r);
      logp_out[row] = (float)(-l1p);
      lse_out[row] = (float)((double)zy * (double)inv_temperature + l1p);
    } else {
      lse_out[row] = (t.m + log2_fast(t.s)) * kLn2;
      logp_out[row] = 0.f;
      atomicOr(status, AIS_STATUS_BAD_TOKEN);
    }
  }
}

// ---- sweep 2: gradient w.r.t. the logits -------------------------------------------------------------
// dz[v] = c * (2^(z_v * scale - lse * log2e) - 1[v = y]) with c = g / T.  Rows with g == 0 (not evaluated,
// zero advantage, or clipped away) are filled with zeros without being read.  In-place operation is safe:
// every element is read and written by the same thread, once.
template <typename T, bool VEC, int UNROLL>
__global__ __launch_bounds__(kSweepThreads) void dlogits_kernel(
    const T* logits, long long row_stride, int vocab, const int* __restrict__ token_ids,
    const float* __restrict__ g, const float* __restrict__ lse, const float* __restrict__ logp,
    float inv_temperature, T* dlogits) {
  constexpr int N = Vec<T>::N;
  const long long row = blockIdx.x;
  const int tid = threadIdx.x;
  const T* zr = logits + row * row_stride;
  T* dr = dlogits + row * row_stride;
  const float gn = g[row];
  const int nvec = VEC ? vocab / N : 0;

  if (gn == 0.f) {
    if (VEC) {
      u32x4* dv = reinterpret_cast<u32x4*>(dr);
      const u32x4 zero = {0u, 0u, 0u, 0u};
      for (int i = tid; i < nvec; i += kSweepThreads) store_stream(dv + i, zero);
    }
    for (int v = nvec * N + tid; v < vocab; v += kSweepThreads) Vec<T>::store1(dr + v, 0.f);
    return;
  }

  const float scale = inv_temperature * kLog2e;
  const float shift = -lse[row] * kLog2e;
  const float c = gn * inv_temperature;
  int y = token_ids[row];
  if (y < 0 || y >= vocab) y = -1;               // flagged by the first sweep; no one-hot term
  const int yvec = (VEC && y >= 0 && y < nvec * N) ? y / N : -1;
  const int ylane = y - yvec * N;
  // the sampled token's element is c (p_y - 1) = c expm1(logp): no cancellation when p_y is close to 1
  const float dzy = c * expm1f(logp[row]);

  if (VEC) {
    const u32x4* zv = reinterpret_cast<const u32x4*>(zr);
    u32x4* dv = reinterpret_cast<u32x4*>(dr);
    int i = tid;
    for (; i + (UNROLL - 1) * kSweepThreads < nvec; i += UNROLL * kSweepThreads) {
      u32x4 q[UNROLL];
#pragma unroll
      for (int u = 0; u < UNROLL; ++u) q[u] = load_stream(zv + i + u * kSweepThreads);
#pragma unroll
      for (int u = 0; u < UNROLL; ++u) {
        float x[N];
        Vec<T>::unpack(q[u], x);
#pragma unroll
        for (int k = 0; k < N; ++k) x[k] = c * exp2_fast(__builtin_fmaf(x[k], scale, shift));
        if (i + u * kSweepThreads == yvec) {
#pragma unroll
          for (int k = 0; k < N; ++k)
            if (k == ylane) x[k] = dzy;
        }
        store_stream(dv + i + u * kSweepThreads, Vec<T>::pack(x));
      }
    }
    for (; i < nvec; i += kSweepThreads) {
      float x[N];
      Vec<T>::unpack(load_stream(zv + i), x);
#pragma unroll
      for (int k = 0; k < N; ++k) x[k] = c * exp2_fast(__builtin_fmaf(x[k], scale, shift));
      if (i == yvec) {
#pragma unroll
        for (int k = 0; k < N; ++k)
          if (k == ylane) x[k] = dzy;
      }
      store_stream(dv + i, Vec<T>::pack(x));
    }
  }
  for (int v = nvec * N + tid; v < vocab; v += kSweepThreads) {
    float p = c * exp2_fast(__builtin_fmaf(Vec<T>::load1(zr + v), scale, shift));
    if (v == y) p = dzy;
    Vec<T>::store1(dr + v, p);
  }
}

// ---- plain copy ------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void copy_kernel(u32x4* __restrict__ dst, const u32x4* __restrict__ src,
                                                   long long nvec) {
  const long long stride = (long long)gridDim.x * blockDim.x;
  for (long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x; i < nvec; i += stride)
    store_stream(dst + i, load_stream(src + i));
}

bool vec_ok(const void* base, long long row_stride, size_t esize) {
  return (reinterpret_cast<uintptr_t>(base) % 16 == 0) && ((row_stride * (long long)esize) % 16 == 0);
}

constexpr int kUnroll = 4;

}  // namespace

int launch_token_logprob(ais_ctx* ctx, const void* logits, ais_dtype dtype, long long n_rows, int vocab,
                         long long row_stride, const int* token_ids, const unsigned char* valid,
                         float inv_temperature, float* logp_out, float* lse_out) {
  if (n_rows == 0) return AIS_OK;
  dim3 grid((unsigned)n_rows), block(kSweepThreads);
  ScopedTimer timer(ctx, AIS_K_LOGPROB);
  if (dtype == AIS_BF16) {
    const bf16_t* z = static_cast<const bf16_t*>(logits);
    if (vec_ok(z, row_stride, 2))
      token_logprob_kernel<bf16_t, true, kUnroll><<<grid, block, 0, ctx->stream>>>(
          z, row_stride, vocab, token_ids, valid, inv_temperature, logp_out, lse_out, ctx->status_dev);
    else
      token_logprob_kernel<bf16_t, false, 1><<<grid, block, 0, ctx->stream>>>(
          z, row_stride, vocab, token_ids, valid, inv_temperature, logp_out, lse_out, ctx->status_dev);
  } else {
    const float* z = static_cast<const float*>(logits);
    if (vec_ok(z, row_stride, 4))
      token_logprob_kernel<float, true, kUnroll><<<grid, block, 0, ctx->stream>>>(
          z, row_stride, vocab, token_ids, valid, inv_temperature, logp_out, lse_out, ctx->status_dev);
    else
      token_logprob_kernel<float, false, 1><<<grid, block, 0, ctx->stream>>>(
          z, row_stride, vocab, token_ids, valid, inv_temperature, logp_out, lse_out, ctx->status_dev);
  }
  return hip_fail(ctx, hipGetLastError());
}

int launch_dlogits(ais_ctx* ctx, const void* logits, ais_dtype dtype, long long n_rows, int vocab,
                   long long row_stride, const int* token_ids, const float* g, const float* lse,
                   const float* logp, float inv_temperature, void* dlogits) {
  if (n_rows == 0) return AIS_OK;
  dim3 grid((unsigned)n_rows), block(kSweepThreads);
  ScopedTimer timer(ctx, AIS_K_DLOGITS);
  if (dtype == AIS_BF16) {
    const bf16_t* z = static_cast<const bf16_t*>(logits);
    bf16_t* dz = static_cast<bf16_t*>(dlogits);
    if (vec_ok(z, row_stride, 2) && vec_ok(dz, row_stride, 2))
      dlogits_kernel<bf16_t, true, kUnroll><<<grid, block, 0, ctx->stream>>>(z, row_stride, vocab, token_ids, g,
                                                                            lse, logp, inv_temperature, dz);
    else
      dlogits_kernel<bf16_t, false, 1><<<grid, block, 0, ctx->stream>>>(z, row_stride, vocab, token_ids, g, lse,
                                                                       logp, inv_temperature, dz);
  } else {
    const float* z = static_cast<const float*>(logits);
    float* dz = static_cast<float*>(dlogits);
    if (vec_ok(z, row_stride, 4) && vec_ok(dz, row_stride, 4))
      dlogits_kernel<float, true, kUnroll><<<grid, block, 0, ctx->stream>>>(z, row_stride, vocab, token_ids, g, lse,
                                                                          logp, inv_temperature, dz);
    else
      dlogits_kernel<float, false, 1><<<grid, block, 0, ctx->stream>>>(z, row_stride, vocab, token_ids, g, lse,
                                                                      logp, inv_temperature, dz);
  }
  return hip_fail(ctx, hipGetLastError());
}

int launch_copy(ais_ctx* ctx, void* dst, const void* src, long long bytes) {
  if (bytes == 0) return AIS_OK;
  const long long nvec = bytes / 16;
  long long blocks = (nvec + 255) / 256;
  if (blocks > 256 * 64) blocks = 256 * 64;   // 64 workgroups per compute unit, grid-stride beyond that
  ScopedTimer timer(ctx, AIS_K_COPY);
  copy_kernel<<<dim3((unsigned)blocks), dim3(256), 0, ctx->stream>>>(static_cast<u32x4*>(dst),
                                                                     static_cast<const u32x4*>(src), nvec);
  return hip_fail(ctx, hipGetLastError());
}

}  // namespace ais
