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
#include "device_utils.h"

namespace ais {
namespace {

using namespace dev;

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
    const float* __restrict__ g, const unsigned char* __restrict__ valid, const float* __restrict__ lse,
    const float* __restrict__ logp, float inv_temperature, T* dlogits) {
  constexpr int N = Vec<T>::N;
  const long long row = blockIdx.x;
  const int tid = threadIdx.x;
  const T* zr = logits + row * row_stride;
  T* dr = dlogits + row * row_stride;
  // g == nullptr: unit coefficient on evaluated rows, i.e. the unscaled direction softmax - onehot
  const float gn = g != nullptr ? g[row] : ((valid == nullptr || valid[row] != 0) ? 1.f : 0.f);
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
  const float c = g != nullptr ? gn * inv_temperature : gn;
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

// 16-byte loads in flight per lane and loop iteration (build-time tunables)
#ifndef AIS_LOGPROB_UNROLL
#define AIS_LOGPROB_UNROLL 4
#endif
#ifndef AIS_DLOGITS_UNROLL
#define AIS_DLOGITS_UNROLL 4
#endif
constexpr int kUnrollFwd = AIS_LOGPROB_UNROLL;
constexpr int kUnrollBwd = AIS_DLOGITS_UNROLL;

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
      token_logprob_kernel<bf16_t, true, kUnrollFwd><<<grid, block, 0, ctx->stream>>>(
          z, row_stride, vocab, token_ids, valid, inv_temperature, logp_out, lse_out, ctx->status_dev);
    else
      token_logprob_kernel<bf16_t, false, 1><<<grid, block, 0, ctx->stream>>>(
          z, row_stride, vocab, token_ids, valid, inv_temperature, logp_out, lse_out, ctx->status_dev);
  } else {
    const float* z = static_cast<const float*>(logits);
    if (vec_ok(z, row_stride, 4))
      token_logprob_kernel<float, true, kUnrollFwd><<<grid, block, 0, ctx->stream>>>(
          z, row_stride, vocab, token_ids, valid, inv_temperature, logp_out, lse_out, ctx->status_dev);
    else
      token_logprob_kernel<float, false, 1><<<grid, block, 0, ctx->stream>>>(
          z, row_stride, vocab, token_ids, valid, inv_temperature, logp_out, lse_out, ctx->status_dev);
  }
  return hip_fail(ctx, hipGetLastError());
}

int launch_dlogits(ais_ctx* ctx, const void* logits, ais_dtype dtype, long long n_rows, int vocab,
                   long long row_stride, const int* token_ids, const float* g, const unsigned char* valid,
                   const float* lse, const float* logp, float inv_temperature, void* dlogits) {
  if (n_rows == 0) return AIS_OK;
  dim3 grid((unsigned)n_rows), block(kSweepThreads);
  ScopedTimer timer(ctx, AIS_K_DLOGITS);
  if (dtype == AIS_BF16) {
    const bf16_t* z = static_cast<const bf16_t*>(logits);
    bf16_t* dz = static_cast<bf16_t*>(dlogits);
    if (vec_ok(z, row_stride, 2) && vec_ok(dz, row_stride, 2))
      dlogits_kernel<bf16_t, true, kUnrollBwd><<<grid, block, 0, ctx->stream>>>(z, row_stride, vocab, token_ids, g,
                                                                            valid, lse, logp, inv_temperature, dz);
    else
      dlogits_kernel<bf16_t, false, 1><<<grid, block, 0, ctx->stream>>>(z, row_stride, vocab, token_ids, g, valid, lse,
                                                                       logp, inv_temperature, dz);
  } else {
    const float* z = static_cast<const float*>(logits);
    float* dz = static_cast<float*>(dlogits);
    if (vec_ok(z, row_stride, 4) && vec_ok(dz, row_stride, 4))
      dlogits_kernel<float, true, kUnrollBwd><<<grid, block, 0, ctx->stream>>>(z, row_stride, vocab, token_ids, g, valid, lse,
                                                                          logp, inv_temperature, dz);
    else
      dlogits_kernel<float, false, 1><<<grid, block, 0, ctx->stream>>>(z, row_stride, vocab, token_ids, g, valid, lse,
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
