// The two vocabulary sweeps of the path, and a plain copy kernel used as a bandwidth yardstick.
//
//   token_logprob_kernel   one pass over a logits row with a running (max, sum) pair:
//                          lse = log sum_v exp(z_v / T), logp = z_y / T - lse, the latter evaluated as
//                          -log1p(sum_{v != y} exp((z_v - z_y) / T))
//                          (Alg. 1, "Compute full-precision log-probs")
//   dlogits_burst_kernel   second pass: dz_v = g (softmax_v - 1[v = y]) / T, written in the logits'
//                          dtype (gradient of Eq. 19 through the log-softmax; g is the row's coefficient)
//
// Both are bound by HBM bandwidth: nothing here is a contraction, so no matrix cores.  One workgroup
// owns one row (256 threads in the read-only sweep, 1,024 in the read+write sweep), so a row's partial
// results never leave its compute unit; consecutive lanes access consecutive 16-byte vectors (8 bf16 or
// 4 fp32 logits), i.e. each wavefront memory instruction covers 1 KiB of contiguous memory.  Logits are
// read and written with streaming (non-temporal) accesses: a batch is tens of GB and nothing survives in
// cache between the two sweeps (a temporal load costs the read-only sweep 11 % of its bandwidth).
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
          if (k == hit) x[k] = kMasked;
      }
      accumulate<UNROLL * N>(x, scale, st);
    }
    for (; i < nvec; i += kSweepThreads) {
      float x[N];
      Vec<T>::unpack(load_stream(zv + i), x);
      if (i == yvec) {
#pragma unroll
        for (int k = 0; k < N; ++k)
          if (k == ysub) x[k] = kMasked;
      }
      accumulate<N>(x, scale, st);
    }
  }
  for (int v = nvec * N + tid; v < vocab; v += kSweepThreads) {   // ragged tail, or the whole row when !VEC
    float x = (y_ok && v == y) ? kMasked : Vec<T>::load1(zr + v);
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
      const double l1p = log1p_scaled(t.s, (double)t.m - ty);
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
//
// Element-wise form: the route for rows that are not 16-byte aligned.  grid.x = n_rows, block = kSweepThreads.
template <typename T>
__global__ __launch_bounds__(kSweepThreads) void dlogits_elementwise_kernel(
    const T* logits, long long row_stride, int vocab, const int* __restrict__ token_ids,
    const float* __restrict__ g, const unsigned char* __restrict__ valid, const float* __restrict__ lse,
    const float* __restrict__ logp, float inv_temperature, T* dlogits) {
  const long long row = blockIdx.x;
  const int tid = threadIdx.x;
  const T* zr = logits + row * row_stride;
  T* dr = dlogits + row * row_stride;
  // g == nullptr: unit coefficient on evaluated rows, i.e. the unscaled direction softmax - onehot
  const float gn = g != nullptr ? g[row] : ((valid == nullptr || valid[row] != 0) ? 1.f : 0.f);
  if (gn == 0.f) {
    for (int v = tid; v < vocab; v += kSweepThreads) Vec<T>::store1(dr + v, 0.f);
    return;
  }
  const float scale = inv_temperature * kLog2e;
  const float shift = -lse[row] * kLog2e;
  const float c = g != nullptr ? gn * inv_temperature : gn;
  int y = token_ids[row];
  if (y < 0 || y >= vocab) y = -1;               // flagged by the first sweep; no one-hot term
  // the sampled token's element is c (p_y - 1) = c expm1(logp): no cancellation when p_y is close to 1
  const float dzy = c * expm1f(logp[row]);
  for (int v = tid; v < vocab; v += kSweepThreads) {
    float p = c * exp2_fast(__builtin_fmaf(Vec<T>::load1(zr + v), scale, shift));
    if (v == y) p = dzy;
    Vec<T>::store1(dr + v, p);
  }
}

// Burst form: the route for 16-byte aligned rows.  A workgroup of 1,024 threads owns the row; every wavefront
// issues all of its loads (up to NV 16-byte vectors per lane, i.e. up to NV KiB per wavefront), transforms
// the vectors in place as they arrive, and only when its last load has landed issues all of its stores.
// Measured on MI355X, a read+write stream shaped this way (long load bursts followed by long store bursts,
// all wavefronts of a compute unit in step because they start together) sustains 5.8-6.0 TB/s where a loop
// that stores each vector as soon as it is computed, and every plain copy variant, saturate at 5.2-5.3 TB/s.
// grid.x = 8 * ceil(n_rows / 8), block = kBurstThreads.  Requires 16-byte aligned rows.  Rows wider than NV * 1024 vectors
// are processed in consecutive segments (there is no dependence between segments: lse is an input).
constexpr int kBurstThreads = 1024;

// NSEG > 0 promises that the row fits NSEG segments, which are then unrolled: the loop-free form is ~3 %
// faster than the same code inside a run-time loop.  NSEG = 0: run-time loop over as many segments as needed.
// KFULL promises that the row has more than KFULL * 1024 vectors: vectors 0 .. KFULL - 1 of every lane exist and
// are loaded and stored without a bounds branch (1.5 % faster at 19 vectors per lane).
template <typename T, int NV, int NSEG, int KFULL>
__global__ __launch_bounds__(kBurstThreads) void dlogits_burst_kernel(
    const T* logits, long long row_stride, int vocab, const int* __restrict__ token_ids,
    const float* __restrict__ g, const unsigned char* __restrict__ valid, const float* __restrict__ lse,
    const float* __restrict__ logp, float inv_temperature, T* dlogits, long long n_rows) {
  constexpr int N = Vec<T>::N;
  // Workgroups are dealt to the 8 XCDs round-robin by their index; every XCD walks a contiguous range of rows
  // (grid.x = 8 * ceil(n_rows / 8)).  Against rows dealt round-robin this is neutral on a batch of full rows
  // and 1-3 % faster where zero-filled rows mix with read+write rows.
  const long long rows_per_xcd = gridDim.x >> 3;
  const long long row = (long long)(blockIdx.x & 7) * rows_per_xcd + (blockIdx.x >> 3);
  if (row >= n_rows) return;
  const int tid = threadIdx.x;
  const T* zr = logits + row * row_stride;
  T* dr = dlogits + row * row_stride;
  const u32x4* zv = reinterpret_cast<const u32x4*>(zr);
  u32x4* dv = reinterpret_cast<u32x4*>(dr);
  const int nvec = vocab / N;
  const int tail = vocab - nvec * N;     // < N elements, one per thread for the first `tail` threads
  const float gn = g != nullptr ? g[row] : ((valid == nullptr || valid[row] != 0) ? 1.f : 0.f);

  if (gn == 0.f) {
    const u32x4 zero = {0u, 0u, 0u, 0u};
    for (int i = tid; i < nvec; i += kBurstThreads) store_stream(dv + i, zero);
    if (tid < tail) Vec<T>::store1(dr + nvec * N + tid, 0.f);
    return;
  }

  const float scale = inv_temperature * kLog2e;
  const float shift = -lse[row] * kLog2e;
  const float c = g != nullptr ? gn * inv_temperature : gn;
  int y = token_ids[row];
  if (y < 0 || y >= vocab) y = -1;               // flagged by the first sweep; no one-hot term
  // The sampled token's element is c (p_y - 1) = c expm1(logp): no cancellation when p_y is close to 1.  The
  // lane that holds it patches its packed output register before the store burst.
  const int yvec = (y >= 0 && y < nvec * N && (y / N) % kBurstThreads == tid) ? y / N : -1;
  const float dzy = c * expm1f(logp[row]);

  const int n_base = NSEG > 0 ? NSEG * NV * kBurstThreads : nvec;
  constexpr int kUnrollSegments = NSEG > 0 ? NSEG : 1;
#pragma unroll kUnrollSegments
  for (int base = 0; base < n_base; base += NV * kBurstThreads) {
    u32x4 q[NV];
#pragma unroll
    for (int k = 0; k < NV; ++k) {
      const int i = base + tid + k * kBurstThreads;
      if (NSEG > 0 && base / kBurstThreads + k < KFULL) q[k] = load_stream(zv + i);
      else q[k] = (i < nvec) ? load_stream(zv + i) : u32x4{0u, 0u, 0u, 0u};
    }
#pragma unroll
    for (int k = 0; k < NV; ++k) {                // in place, in order of arrival
      float x[N];
      Vec<T>::unpack(q[k], x);
#pragma unroll
      for (int j = 0; j < N; ++j) x[j] = c * exp2_fast(__builtin_fmaf(x[j], scale, shift));
      q[k] = Vec<T>::pack(x);
      __builtin_amdgcn_sched_barrier(0);
    }
    // every vector is made opaque here: no store can be issued before the last load has returned
#pragma unroll
    for (int k = 0; k < NV; ++k) asm volatile("" : "+v"(q[k]));
    if ((unsigned)(yvec - base - tid) < (unsigned)(NV * kBurstThreads)) {   // one lane, once per row
      const int hit = (yvec - base - tid) / kBurstThreads;
#pragma unroll
      for (int k = 0; k < NV; ++k)
        if (k == hit) q[k] = Vec<T>::put(q[k], y % N, dzy);
    }
#pragma unroll
    for (int k = 0; k < NV; ++k) {
      const int i = base + tid + k * kBurstThreads;
      if ((NSEG > 0 && base / kBurstThreads + k < KFULL) || i < nvec) store_stream(dv + i, q[k]);
    }
  }
  if (tid < tail) {
    const int v = nvec * N + tid;
    Vec<T>::store1(dr + v, v == y ? dzy : c * exp2_fast(__builtin_fmaf(Vec<T>::load1(zr + v), scale, shift)));
  }
}

template <typename T>
void launch_dlogits_burst(ais_ctx* ctx, const T* z, long long n_rows, int vocab, long long row_stride,
                          const int* token_ids, const float* g, const unsigned char* valid, const float* lse,
                          const float* logp, float inv_t, T* dz) {
  const int need = (vocab / Vec<T>::N + kBurstThreads - 1) / kBurstThreads;
  dim3 grid((unsigned)(((n_rows + 7) / 8) * 8)), block(kBurstThreads);
  // (vectors that surely exist, vectors per lane and burst, bursts): a row reaches a class only if it is wider than
  // the class before it, which is what the first figure states
#define AIS_BURST_CASE(KFULL, NVAL, NSEG)                                                                  \
  dlogits_burst_kernel<T, NVAL, NSEG, KFULL><<<grid, block, 0, ctx->stream>>>(z, row_stride, vocab, token_ids, \
                                                                              g, valid, lse, logp, inv_t, dz, n_rows)
  if (need <= 4) AIS_BURST_CASE(0, 4, 1);
  else if (need <= 8) AIS_BURST_CASE(4, 8, 1);
  else if (need <= 12) AIS_BURST_CASE(8, 12, 1);
  else if (need <= 13) AIS_BURST_CASE(12, 13, 1);
  else if (need <= 14) AIS_BURST_CASE(13, 14, 1);
  else if (need <= 15) AIS_BURST_CASE(14, 15, 1);
  else if (need <= 16) AIS_BURST_CASE(15, 16, 1);
  else if (need <= 17) AIS_BURST_CASE(16, 17, 1);
  else if (need <= 18) AIS_BURST_CASE(17, 18, 1);
  else if (need <= 19) AIS_BURST_CASE(18, 19, 1);
  else if (need <= 20) AIS_BURST_CASE(19, 20, 1);
  else if (need <= 32) AIS_BURST_CASE(20, 16, 2);   // wider rows: two or three bursts of 16 vectors per lane
  else if (need <= 48) AIS_BURST_CASE(32, 16, 3);
  else AIS_BURST_CASE(0, 16, 0);
#undef AIS_BURST_CASE
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

// 16-byte loads in flight per lane and loop iteration of the log-prob sweep (build-time tunable)
#ifndef AIS_LOGPROB_UNROLL
#define AIS_LOGPROB_UNROLL 4
#endif
constexpr int kUnrollFwd = AIS_LOGPROB_UNROLL;

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
      launch_dlogits_burst<bf16_t>(ctx, z, n_rows, vocab, row_stride, token_ids, g, valid, lse, logp,
                                   inv_temperature, dz);
    else
      dlogits_elementwise_kernel<bf16_t><<<grid, block, 0, ctx->stream>>>(z, row_stride, vocab, token_ids, g, valid,
                                                                         lse, logp, inv_temperature, dz);
  } else {
    const float* z = static_cast<const float*>(logits);
    float* dz = static_cast<float*>(dlogits);
    if (vec_ok(z, row_stride, 4) && vec_ok(dz, row_stride, 4))
      launch_dlogits_burst<float>(ctx, z, n_rows, vocab, row_stride, token_ids, g, valid, lse, logp,
                                  inv_temperature, dz);
    else
      dlogits_elementwise_kernel<float><<<grid, block, 0, ctx->stream>>>(z, row_stride, vocab, token_ids, g, valid,
                                                                        lse, logp, inv_temperature, dz);
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
