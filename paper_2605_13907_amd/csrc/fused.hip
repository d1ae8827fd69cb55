// One-sweep variant of the two vocabulary passes: each logits row is read from HBM once, kept in the
// register file of one compute unit while its log-sum-exp is formed, and written back as the unscaled
// gradient direction  s[n, v] = softmax(z_n / T)_v - 1[v = y_n].
//
// The mixing coefficient alpha (Eq. 17) depends on every row of the batch, so the final gradient of
// Eq. 19 cannot be written in the same sweep that computes the log-probs; but alpha enters that gradient
// only through one scalar per row: dz[n, :] = g_n * s[n, :].  Emitting s and, after the diagnostics, the
// per-row scale g_n lets the consumer (the LM-head backward) fold g_n into its own operands, and the path
// moves 2 * e * V bytes per token instead of 3 * e * V.
//
// A 151,936-wide bf16 row is 297 KiB; a CDNA4 compute unit has 512 KiB of vector registers.  One
// workgroup of 1,024 threads (16 wavefronts, 4 per SIMD, up to 128 registers per lane) holds the row as
// NV 16-byte vectors per lane.  All NV loads of a lane are issued back to back, so the whole row is in
// flight at once and memory latency is paid once per row.  Rows wider than 24 vectors per lane keep their
// last 9 vectors per lane in LDS (144 KiB of the compute unit's 160), which are filled by direct
// global -> LDS copies and never pass through registers on the way in: up to 33 vectors per lane, 270,336
// bf16 elements.  Rows wider than that fall back to the two-pass kernels.
#include "ais_internal.h"
#include "device_utils.h"

namespace ais {
namespace {

using namespace dev;

constexpr int kRowThreads = 1024;
constexpr int kRowWaves = kRowThreads / 64;

// A vector of excluded elements (-inf in the row's type), for lanes past the end of the row.
template <typename T> __device__ __forceinline__ u32x4 masked_fill();
template <> __device__ __forceinline__ u32x4 masked_fill<bf16_t>() {
  return u32x4{0xff80ff80u, 0xff80ff80u, 0xff80ff80u, 0xff80ff80u};
}
template <> __device__ __forceinline__ u32x4 masked_fill<float>() {
  return u32x4{0xff800000u, 0xff800000u, 0xff800000u, 0xff800000u};
}

// q with its element `sub` excluded (replaced by -inf in the row's type).
template <typename T> __device__ __forceinline__ u32x4 patch_masked(u32x4 q, int sub);
template <> __device__ __forceinline__ u32x4 patch_masked<bf16_t>(u32x4 q, int sub) {
  const uint32_t keep = (sub & 1) ? 0x0000ffffu : 0xffff0000u;
  const uint32_t put = (sub & 1) ? 0xff800000u : 0x0000ff80u;
#pragma unroll
  for (int w = 0; w < 4; ++w)
    if (w == (sub >> 1)) q[w] = (q[w] & keep) | put;
  return q;
}
template <> __device__ __forceinline__ u32x4 patch_masked<float>(u32x4 q, int sub) {
#pragma unroll
  for (int w = 0; w < 4; ++w)
    if (w == sub) q[w] = 0xff800000u;
  return q;
}

typedef __attribute__((address_space(3))) void* lds_ptr;
typedef const __attribute__((address_space(1))) void* glb_ptr;

// grid.x = n_rows, block = kRowThreads.  Requires 16-byte aligned rows and
// KFULL * kRowThreads < vocab / N <= (NV + NL) * kRowThreads: vectors 0 .. KFULL - 1 of every lane exist and are
// loaded and stored without a bounds branch.
// Vector k of a lane (elements N * (tid + 1024 k) ..) lives in register q[k] for k < NV and in LDS slot k - NV
// (16 bytes at byte offset 16 * (1024 (k - NV) + tid) of the dynamic LDS) for NV <= k < NV + NL.
template <typename T, int NV, int NL, int KFULL>
__global__ __launch_bounds__(kRowThreads) void fused_logprob_softmax_kernel(
    const T* logits, long long row_stride, int vocab, const int* __restrict__ token_ids,
    const unsigned char* __restrict__ valid, float inv_temperature, float* __restrict__ logp_out,
    float* __restrict__ lse_out, T* sgrad, int* __restrict__ status) {
  constexpr int N = Vec<T>::N;
  __shared__ MaxSum lds[kRowWaves];
  __shared__ float lds_row[2];          // shift (= -lse * log2e) and the sampled token's element
  extern __shared__ __align__(16) unsigned char lds_slots[];
  u32x4* lrow = reinterpret_cast<u32x4*>(lds_slots);
  const long long row = blockIdx.x;
  const int tid = threadIdx.x;
  const T* zr = logits + row * row_stride;
  T* sr = sgrad + row * row_stride;
  const int nvec = vocab / N;
  const int tail = vocab - nvec * N;    // < N elements, one per thread for the first `tail` threads
  u32x4* sv = reinterpret_cast<u32x4*>(sr);

  if (valid != nullptr && valid[row] == 0) {     // not evaluated: no read, zero direction
    if (tid == 0) {
      logp_out[row] = 0.f;
      lse_out[row] = 0.f;
    }
    const u32x4 zero = {0u, 0u, 0u, 0u};
#pragma unroll
    for (int k = 0; k < NV + NL; ++k) {
      const int i = tid + k * kRowThreads;
      if (i < nvec) store_stream(sv + i, zero);
    }
    if (tid < tail) Vec<T>::store1(sr + nvec * N + tid, 0.f);
    return;
  }

  // ---- phase 1: the whole row into registers ----
  const u32x4* zv = reinterpret_cast<const u32x4*>(zr);
  u32x4 q[NV];
#pragma unroll
  for (int k = 0; k < NV; ++k) {
    const int i = tid + k * kRowThreads;
    if (k < KFULL) q[k] = load_stream(zv + i);       // the launcher promises nvec > KFULL * kRowThreads
    else q[k] = (i < nvec) ? load_stream(zv + i) : masked_fill<T>();
  }
  // the LDS slots: lane i of a wavefront deposits its 16 bytes at the wavefront's base + 16 i, which is the
  // slot layout; lanes past the end of the row re-read its last vector (a valid address) and are masked later
  if (NL > 0) {
    int tid0 = tid;                                   // opaque copies keep the per-vector offsets short-lived
    asm volatile("" : "+v"(tid0));
#pragma unroll
    for (int k = 0; k < NL; ++k) {
      const int i = min(tid0 + (NV + k) * kRowThreads, nvec - 1);
      __builtin_amdgcn_global_load_lds((glb_ptr)(zv + i), (lds_ptr)(lrow + k * kRowThreads + (tid0 & ~63)), 16, 0,
                                       2 /* non-temporal */);
      __builtin_amdgcn_sched_barrier(0);
    }
  }
  float xt = (tid < tail) ? Vec<T>::load1(zr + nvec * N + tid) : kMasked;

  const float scale = inv_temperature * kLog2e;
  const int y = token_ids[row];
  const bool y_ok = (y >= 0) && (y < vocab);
  const float zy = y_ok ? Vec<T>::load1(zr + y) : 0.f;
  // where this thread holds the sampled token: vector slot k and lane element, or the tail register
  const int yv = (y_ok && y < nvec * N) ? y / N : -1;
  const int yk = (yv >= 0 && yv % kRowThreads == tid) ? yv / kRowThreads : -1;
  const int ysub = y % N;
  const bool y_in_tail = y_ok && y >= nvec * N && (y - nvec * N) == tid;

  // The sampled token's own term is kept out of the running sum (see token_logprob_kernel).  Its element
  // is overwritten, in the packed registers, by -inf: one lane of one wavefront takes this branch, the sweeps
  // below stay free of control flow.
  if (yk >= 0 && yk < NV) {
#pragma unroll
    for (int k = 0; k < NV; ++k)
      if (k == yk) q[k] = patch_masked<T>(q[k], ysub);
  }
  if (y_in_tail) xt = kMasked;

  // ---- phase 1: running (max, sum) over the row, one vector at a time ----
  MaxSum st{kNegHuge, 0.f};
#pragma unroll
  for (int k = 0; k < NV; ++k) {
    float x[N];
    Vec<T>::unpack(q[k], x);
    accumulate<N>(x, scale, st);
    __builtin_amdgcn_sched_barrier(0);   // keeps the unpacked values of one vector short-lived
  }
  if (NL > 0) {
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");     // the copies into the slots have landed
    if (yk >= NV) {                                        // the sampled token lies in a slot of this lane
      u32x4* p = lrow + (yk - NV) * kRowThreads + tid;
      *p = patch_masked<T>(*p, ysub);
    }
    int tid1 = tid;
    asm volatile("" : "+v"(tid1));
#pragma unroll
    for (int k = 0; k < NL; ++k) {
      const int i = tid1 + (NV + k) * kRowThreads;
      // every slot holds data (lanes past the end of the row hold a copy of its last vector); read without a
      // branch, so that the reads stay in this order, and mask afterwards where the row can end
      const u32x4 v = lrow[k * kRowThreads + tid1];
      float x[N];
      Vec<T>::unpack(v, x);
      if (NV + k >= KFULL) {
#pragma unroll
        for (int j = 0; j < N; ++j) x[j] = (i < nvec) ? x[j] : kMasked;
      }
      accumulate<N>(x, scale, st);
      __builtin_amdgcn_sched_barrier(0);
    }
  }
  accumulate<1>(&xt, scale, st);
  st = wave_merge(st);
  if ((tid & 63) == 0) lds[tid >> 6] = st;
  __syncthreads();
  if (tid == 0) {
    MaxSum t = lds[0];
#pragma unroll
    for (int w = 1; w < kRowWaves; ++w) t = merge(t, lds[w]);
    float lse, logp;
    if (y_ok) {
      const double l1p = log1p_scaled(t.s, (double)t.m - (double)zy * (double)scale);
      logp = (float)(-l1p);
      lse = (float)((double)zy * (double)inv_temperature + l1p);
    } else {
      lse = (t.m + log2_fast(t.s)) * kLn2;
      logp = 0.f;
      atomicOr(status, AIS_STATUS_BAD_TOKEN);
    }
    logp_out[row] = logp;
    lse_out[row] = lse;
    lds_row[0] = -lse * kLog2e;
    lds_row[1] = expm1f(logp);            // p_y - 1 without cancellation
  }
  __syncthreads();
  const float shift = lds_row[0];
  const float sy = lds_row[1];
  // The row stays in registers in its packed form: the empty asm, which names the shift as an input, makes
  // each vector opaque until the reduction is done, so that neither the unpacked fp32 values of phase 1 are
  // kept alive nor the unpacking of phase 2 is hoisted above the barrier (either costs a multiple of the
  // registers).
#pragma unroll
  for (int k = 0; k < NV; ++k) asm volatile("" : "+v"(q[k]) : "v"(shift));

  // ---- phase 2: softmax from the registers (the patched element comes out as 0) ----
  // The vector indices are recomputed from an opaque copy of the thread index: otherwise the compiler keeps the
  // byte offset of every vector alive from the loads to these stores, one more register per vector.
  int tid2 = tid;
  asm volatile("" : "+v"(tid2));
#pragma unroll
  for (int k = 0; k < NV; ++k) {
    const int i = tid2 + k * kRowThreads;
    float x[N];
    Vec<T>::unpack(q[k], x);
#pragma unroll
    for (int j = 0; j < N; ++j) x[j] = exp2_fast(__builtin_fmaf(x[j], scale, shift));
    if (k < KFULL || i < nvec) store_stream(sv + i, Vec<T>::pack(x));
    __builtin_amdgcn_sched_barrier(0);
  }
  if (NL > 0) {
#pragma unroll
    for (int k = 0; k < NL; ++k) {
      const int i = tid2 + (NV + k) * kRowThreads;
      float x[N];
      Vec<T>::unpack(lrow[k * kRowThreads + tid2], x);
#pragma unroll
      for (int j = 0; j < N; ++j) x[j] = exp2_fast(__builtin_fmaf(x[j], scale, shift));
      if (i < nvec) store_stream(sv + i, Vec<T>::pack(x));
      __builtin_amdgcn_sched_barrier(0);
    }
  }
  if (tid < tail) Vec<T>::store1(sr + nvec * N + tid, exp2_fast(__builtin_fmaf(xt, scale, shift)));
  // the sampled token's element p_y - 1, by the lane that owns it, after its vector store has completed
  if (yk >= 0 || y_in_tail) {
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    Vec<T>::store1(sr + y, sy);
  }
}

constexpr int kSlotBytes = kRowThreads * 16;      // one LDS slot: a 16-byte vector per lane
constexpr int kLdsSlots = 9;                      // 144 KiB of the 160 KiB of a compute unit

template <typename T, int NV, int NL, int KFULL>
int launch_nv(ais_ctx* ctx, const T* z, long long n_rows, int vocab, long long row_stride, const int* token_ids,
              const unsigned char* valid, float inv_t, float* logp, float* lse, T* sgrad) {
  auto kernel = fused_logprob_softmax_kernel<T, NV, NL, KFULL>;
  if (NL > 0) {
    static std::once_flag once[kMaxDevices];               // the attribute belongs to the function on one device
    static bool ok[kMaxDevices];
    if (!allow_dynamic_lds(ctx, reinterpret_cast<const void*>(kernel), NL * kSlotBytes, once, ok))
      return hip_fail(ctx, hipErrorInvalidValue);
  }
  kernel<<<dim3((unsigned)n_rows), dim3(kRowThreads), NL * kSlotBytes, ctx->stream>>>(
      z, row_stride, vocab, token_ids, valid, inv_t, logp, lse, sgrad, ctx->status_dev);
  return AIS_OK;
}

// Vectors per lane needed for a row, or 0 when the row cannot be held (too wide, or not 16-byte aligned).
template <typename T>
int vectors_per_lane(const void* z, const void* s, int vocab, long long row_stride) {
  constexpr int N = Vec<T>::N;
  const bool ok16 = reinterpret_cast<uintptr_t>(z) % 16 == 0 && reinterpret_cast<uintptr_t>(s) % 16 == 0 &&
                    (row_stride * (long long)sizeof(T)) % 16 == 0;
  const int need = (vocab / N + kRowThreads - 1) / kRowThreads;
  return (ok16 && need <= 24 + kLdsSlots) ? (need < 1 ? 1 : need) : 0;
}

template <typename T>
int launch_typed(ais_ctx* ctx, int need, const void* logits, long long n_rows, int vocab, long long row_stride,
                 const int* token_ids, const unsigned char* valid, float inv_t, float* logp, float* lse,
                 void* sgrad) {
  const T* z = static_cast<const T*>(logits);
  T* s = static_cast<T*>(sgrad);
  // NV is a compile-time constant (the row lives in named registers); sizes near the register limit get an
  // exact instantiation so that common vocabularies (e.g. 151,936 -> 19 vectors per lane) do not spill
  // PREV: the widest row of the previous class; a row that reaches this one has more than PREV * 1024 vectors
#define AIS_FUSED_CASE(PREV, NEED, NVAL, NLVAL)                                                         \
  if (need <= NEED)                                                                                     \
    return launch_nv<T, NVAL, NLVAL, PREV>(ctx, z, n_rows, vocab, row_stride, token_ids, valid, inv_t, \
                                           logp, lse, s);
  AIS_FUSED_CASE(0, 4, 4, 0)
  AIS_FUSED_CASE(4, 8, 8, 0)
  AIS_FUSED_CASE(8, 12, 12, 0)
  AIS_FUSED_CASE(12, 16, 16, 0)
  AIS_FUSED_CASE(16, 17, 17, 0)
  AIS_FUSED_CASE(17, 18, 18, 0)
  AIS_FUSED_CASE(18, 19, 19, 0)
  AIS_FUSED_CASE(19, 20, 20, 0)
  AIS_FUSED_CASE(20, 21, 21, 0)
  AIS_FUSED_CASE(21, 22, 22, 0)
  AIS_FUSED_CASE(22, 23, 23, 0)
  AIS_FUSED_CASE(23, 24, 24, 0)
  AIS_FUSED_CASE(24, 27, 18, kLdsSlots)
  AIS_FUSED_CASE(27, 29, 20, kLdsSlots)
  AIS_FUSED_CASE(29, 31, 22, kLdsSlots)
  AIS_FUSED_CASE(31, 33, 24, kLdsSlots)
#undef AIS_FUSED_CASE
  return AIS_ERR_SIZE;                            // not reached: vectors_per_lane() bounds `need`
}

}  // namespace

// Sets *used_registers to false (and launches nothing) when the row does not fit the register file or is
// not 16-byte aligned; the caller then runs the two-pass kernels.
int launch_fused_logprob_softmax(ais_ctx* ctx, const void* logits, ais_dtype dtype, long long n_rows, int vocab,
                                 long long row_stride, const int* token_ids, const unsigned char* valid,
                                 float inv_temperature, float* logp_out, float* lse_out, void* sgrad,
                                 bool* used_registers) {
  const int need = dtype == AIS_BF16 ? vectors_per_lane<bf16_t>(logits, sgrad, vocab, row_stride)
                                     : vectors_per_lane<float>(logits, sgrad, vocab, row_stride);
  *used_registers = need > 0;
  if (need == 0 || n_rows == 0) return AIS_OK;
  ScopedTimer timer(ctx, AIS_K_FUSED);
  const int rc = dtype == AIS_BF16
                     ? launch_typed<bf16_t>(ctx, need, logits, n_rows, vocab, row_stride, token_ids, valid,
                                            inv_temperature, logp_out, lse_out, sgrad)
                     : launch_typed<float>(ctx, need, logits, n_rows, vocab, row_stride, token_ids, valid,
                                           inv_temperature, logp_out, lse_out, sgrad);
  if (rc != AIS_OK) return rc;
  return hip_fail(ctx, hipGetLastError());
}

}  // namespace ais
