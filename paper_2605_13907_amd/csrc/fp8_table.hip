// FP8-E4M3 per-row quantisation and rollout log-prob for bf16 logits by table lookup.
//
// A bf16 logit has 15 magnitude bits, and only the 20 binades below the row's abs-max can give a non-zero E4M3
// code (the quotient z / s of anything smaller lies below 2^-10, half the smallest E4M3 value).  So a row has at
// most 2,560 distinct magnitudes that matter, against 150,000 elements: once the row's scale s = max|z| / 448 is
// known (Eq. 1 with the E4M3 grid, Sec. 2.1), the workgroup evaluates
//     code(m) = e4m3(RN(m / s))            true fp32 division, then the hardware conversion (round to nearest even)
// once per magnitude m into a table in LDS, and every element then costs a table read instead of a correctly rounded
// division and a conversion.  The arithmetic that decides a code is exactly the plain definition's; it is only
// done once per distinct input.  For the rollout log-prob the table holds exp(z_r(m) - max_v z_r) for both signs
// directly, so the sweep over the row needs no division, no conversion and no exponential at all.
//
// One workgroup of 1,024 threads per row; the row is read from HBM once and waits in registers (up to 24 16-byte
// vectors per lane, 196,608 logits; 23 for the log-prob, which parks up to 8 more per lane in LDS: 253,952 logits)
// while the table is built.  Wider, unaligned or fp32 rows take the kernels of fp8_rows.hip / fp8.hip.
#include "ais_internal.h"
#include "device_utils.h"
#include "fp8_utils.h"

namespace ais {
namespace {

using namespace dev;

constexpr int kRowThreads = 1024;
constexpr int kRowWaves = kRowThreads / 64;
constexpr int kTabEntries = 2560;             // 20 binades x 128 significands, ending at the row's abs-max
constexpr int kTabStride = 4096;              // floats between the two sign halves of the log-prob table
constexpr int kSlotBytes = kRowThreads * 16;  // one 16-byte vector per thread
typedef uint16_t u16x2 __attribute__((ext_vector_type(2)));
typedef __attribute__((address_space(3))) void* lds_ptr;
typedef const __attribute__((address_space(1))) void* glb_ptr;

// Copies vector min(tid + k * 1024, nvec - 1) of the row at zv into LDS slot `slot` (16 bytes per thread at index
// tid): lane i of a wavefront deposits its 16 bytes at the wavefront's base + 16 i.  nvec >= 1.
__device__ __forceinline__ void copy_to_slot(const u32x4* zv, int nvec, int k, u32x4* slot, int tid) {
  const int i = min(tid + k * kRowThreads, nvec - 1);
  __builtin_amdgcn_global_load_lds((glb_ptr)(zv + (unsigned)i), (lds_ptr)(slot + (tid & ~63)), 16, 0,
                                   2 /* non-temporal */);
}

__device__ __forceinline__ float bf16_bits_to_float(int bits) { return __uint_as_float((uint32_t)bits << 16); }

// E4M3 code of q (saturating, round to nearest even) and the value of a code.
__device__ __forceinline__ uint32_t code_of(float q) { return to_e4m3x2(q, 0.f) & 0xffu; }
__device__ __forceinline__ float value_of(uint32_t code) { return from_e4m3x2(code)[0]; }

// Issues the loads of a row: q[k] is vector tid + 1024 k of the row (slots past the end hold zeros), xt the ragged
// tail (one element for the first `tail` threads).  KFULL: vectors 0 .. KFULL - 1 of every lane are certain to exist.
template <int NV, int KFULL>
__device__ __forceinline__ void issue_row(const bf16_t* zr, int vocab, u32x4 (&q)[NV], float& xt) {
  const int tid = threadIdx.x;
  const int nvec = vocab / 8;
  const int tail = vocab - nvec * 8;
  const u32x4* zv = reinterpret_cast<const u32x4*>(zr);
  const u32x4 zero = {0u, 0u, 0u, 0u};
#pragma unroll
  for (int k = 0; k < NV; ++k) {
    const int i = tid + k * kRowThreads;
    if (k < KFULL) q[k] = load_stream(zv + i);
    else q[k] = (i < nvec) ? load_stream(zv + i) : zero;
  }
  xt = (tid < tail) ? Vec<bf16_t>::load1(zr + nvec * 8 + tid) : 0.f;
}

// Largest and smallest element of the row held in q[], the NL LDS slots at lrow (slot j: 16 bytes per thread at index
// 1024 j + tid; every slot holds vectors of the row, possibly repeated ones) and xt, returned to every thread.
// `lds`: 2 * kRowWaves floats.
template <int NV, int NL = 0>
__device__ __forceinline__ void row_minmax(u32x4 (&q)[NV], float xt, float* lds, float& zmax, float& zmin,
                                           const u32x4* lrow = nullptr) {
  const int tid = threadIdx.x;
  float hi = xt, lo = xt;
  auto fold = [&](const u32x4& v) {
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      // the word itself stands for its upper logit: as an fp32 it is that logit with 16 more significand bits, which
      // order it among equals only (they are cut off at the end); a NaN loses every comparison either way
      const float a = __uint_as_float(v[w] << 16), b = __uint_as_float(v[w]);
      hi = fmaxf(hi, fmaxf(a, b));
      lo = fminf(lo, fminf(a, b));
    }
  };
#pragma unroll
  for (int k = 0; k < NV; ++k) {
    fold(q[k]);
    __builtin_amdgcn_sched_barrier(0);
  }
  if (NL > 0) {
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");       // the copies into the slots have landed
    int t1 = tid;
    asm volatile("" : "+v"(t1));
#pragma unroll
    for (int j = 0; j < NL; ++j) {
      fold(lrow[j * kRowThreads + t1]);
      __builtin_amdgcn_sched_barrier(0);
    }
  }
  hi = wave_max(hi);
  lo = -wave_max(-lo);
  if ((tid & 63) == 0) {
    lds[tid >> 6] = hi;
    lds[kRowWaves + (tid >> 6)] = lo;
  }
  __syncthreads();
  hi = lds[0];
  lo = lds[kRowWaves];
#pragma unroll
  for (int w = 1; w < kRowWaves; ++w) {
    hi = fmaxf(hi, lds[w]);
    lo = fminf(lo, lds[kRowWaves + w]);
  }
  zmax = __uint_as_float(__float_as_uint(hi) & 0xffff0000u);
  zmin = __uint_as_float(__float_as_uint(lo) & 0xffff0000u);
  // keep the row packed until the scale is known (the empty asm names the reduction result as an input)
#pragma unroll
  for (int k = 0; k < NV; ++k) asm volatile("" : "+v"(q[k]) : "v"(zmax));
}

// Table index of a bf16 magnitude (15 bits): magnitudes below the table's first entry share it (their code is 0,
// as is the first entry's), and nothing finite lies above the last entry, the row's abs-max; a NaN's payload does,
// and is held inside the table.
__device__ __forceinline__ int table_index(uint32_t mag, int base) {
  return min(max((int)mag - base, 0), kTabEntries - 1);
}

// ---- quantise ----------------------------------------------------------------------------------------------
// Persistent grid, one workgroup per compute unit, rows dealt round-robin; the registers of a vector whose codes have
// been written are reloaded at once with the same vector of the workgroup's next row (see the log-prob kernel below
// for why).
template <int NV, int KFULL>
__global__ __launch_bounds__(kRowThreads) void fp8_quantize_table_kernel(const bf16_t* __restrict__ logits,
                                                                         long long row_stride, int vocab,
                                                                         unsigned char* __restrict__ codes,
                                                                         long long codes_stride,
                                                                         float* __restrict__ scale_out,
                                                                         long long n_rows) {
  __shared__ float lds[2 * kRowWaves];
  __shared__ unsigned char table[kTabEntries];
  const int tid = threadIdx.x;
  const int nvec = vocab / 8;
  const int tail = vocab - nvec * 8;
  long long row = blockIdx.x;
  if (row >= n_rows) return;
  u32x4 q[NV];
  float xt;
  issue_row<NV, KFULL>(logits + row * row_stride, vocab, q, xt);
  for (; row < n_rows; row += gridDim.x) {
    unsigned char* cr = codes + row * codes_stride;
    // after its last row a workgroup fetches that row once more (into registers nobody reads again): the loop
    // body stays free of conditions, which keeps the reloaded registers the very ones that were just read
    const long long next = row + gridDim.x < n_rows ? row + gridDim.x : row;
    const u32x4* zn = reinterpret_cast<const u32x4*>(logits + next * row_stride);
    float zmax, zmin;
    row_minmax<NV>(q, xt, lds, zmax, zmin);
    const float amax = fmaxf(zmax, -zmin);
    const float s = scale_of(amax);
    if (tid == 0) scale_out[row] = s;
    // entry i belongs to the bf16 magnitude with bits base + i; the last entry is the abs-max itself
    const int base = (int)(__float_as_uint(amax) >> 16) - (kTabEntries - 1);
    for (int i = tid; i < kTabEntries; i += kRowThreads) {
      const int bits = base + i;
      table[i] = (unsigned char)code_of(bits > 0 ? bf16_bits_to_float(bits) / s : 0.f);
    }
    __syncthreads();
    auto code2 = [&](uint32_t w) -> uint32_t {           // two logits -> two codes in the low 16 bits
      const uint32_t c0 = table[table_index(w & 0x7fffu, base)];
      const uint32_t c1 = table[table_index((w >> 16) & 0x7fffu, base)];
      // the sign of the logit is the sign of the code, zero included
      return c0 | (c1 << 8) | ((w >> 8) & 0x80u) | ((w >> 16) & 0x8000u);
    };
#pragma unroll
    for (int k = 0; k < NV; ++k) {
      // the slot's index comes from a fresh opaque copy of the thread index: otherwise every slot's load and store
      // offsets are computed once, ahead of the row loop, and stay alive in four registers per slot
      int tk = tid;
      asm volatile("" : "+v"(tk));
      __builtin_assume(tk >= 0 && tk < kRowThreads);
      const int i = tk + k * kRowThreads;
      uint2 o;
      o.x = code2(q[k][0]) | (code2(q[k][1]) << 16);
      asm volatile("" : "+v"(o.x));                      // four table reads in flight at a time: fewer registers
      __builtin_amdgcn_sched_barrier(0);
      o.y = code2(q[k][2]) | (code2(q[k][3]) << 16);
      asm volatile("" : "+v"(o.y));                      // the codes are formed here, before the registers are reused
      __builtin_amdgcn_sched_barrier(0);
      if (k < KFULL || i < nvec) *reinterpret_cast<uint2*>(cr + (long long)i * 8) = o;
      // (i >= 0 and nvec >= 1, so the clamped index is a valid vector of the row)
      q[k] = load_stream(zn + (unsigned)(k < KFULL ? i : min(i, nvec - 1)));
      __builtin_amdgcn_sched_barrier(0);
    }
    if (tid < tail) {
      cr[nvec * 8 + tid] = (unsigned char)(code2(__float_as_uint(xt) >> 16) & 0xffu);
      xt = Vec<bf16_t>::load1(reinterpret_cast<const bf16_t*>(zn) + nvec * 8 + tid);
    }
    __syncthreads();                                     // everyone has finished reading the table
  }
}

// ---- rollout log-prob ----------------------------------------------------------------------------------------
// logp[n] = z_r[y] - log sum_v exp(z_r[v]) with z_r = s * value(code(z / s)).  The table holds, for every
// magnitude and both signs, 2^(log2e (z_r - max_v z_r)): the row's largest term is exactly 1.
//
// A row (297 KiB at 151,936 logits) fills most of a compute unit's register file, so only one can be resident, and a
// workgroup that loaded, reduced and summed one row after the other would leave the memory system idle while it
// computes.  The grid is therefore persistent (one workgroup per compute unit, rows dealt round-robin), and the
// registers of the vector that the sum has just consumed are reloaded at once with the same vector of the
// workgroup's next row: by the time the sum is finished the next row is on its way or has landed.
//
// Rows beyond 23 vectors per lane park vectors 23 .. 23 + NL - 1 of every lane in LDS slots (16 KiB each, filled by
// direct global -> LDS copies); a slot is refilled with the next row's vector by the thread that has just read its
// 16 bytes of it, so no thread ever waits for another.  With slots the two sign halves of the table are interleaved
// (8 bytes per magnitude, 20 KiB) instead of 16 KiB apart (32 KiB), which is what lets 8 slots fit beside it.
template <bool INTERLEAVED>
struct LogprobTable {
  static constexpr int kFloats = INTERLEAVED ? 2 * kTabEntries : 2 * kTabStride;
  // positions (in floats) of magnitude i's positive and negative entry
  static __device__ __forceinline__ int pos(int i) { return INTERLEAVED ? 2 * i : i; }
  static __device__ __forceinline__ int neg(int i) { return INTERLEAVED ? 2 * i + 1 : kTabStride + i; }
  // Byte offsets into the table of the two logits of a word, formed on both 16-bit halves at once: magnitude
  // minus base, saturating at 0 (smaller magnitudes share the first entry: their code is 0, as is its) and held
  // below the table's end (only a NaN's payload lies above the abs-max), times the entry pitch, plus the sign's part.
  static __device__ __forceinline__ uint32_t offsets(uint32_t w, uint32_t base2) {
    u16x2 t = __builtin_bit_cast(u16x2, w & 0x7fff7fffu);
    t = __builtin_elementwise_sub_sat(t, __builtin_bit_cast(u16x2, base2));
    t = __builtin_elementwise_min(t, u16x2{kTabEntries - 1, kTabEntries - 1});
    if (INTERLEAVED) {
      static_assert((kTabEntries - 1) * 8 + 4 < 0x10000, "an offset must fit a 16-bit half");
      t = t << 3;
      return __builtin_bit_cast(uint32_t, t) | ((w >> 13) & 0x00040004u);     // sign bit -> byte 4 of the entry
    }
    static_assert(kTabStride * 4 == 0x4000, "the sign bit of a half is moved to this bit of its offset");
    t = t << 2;
    return __builtin_bit_cast(uint32_t, t) | ((w >> 1) & 0x40004000u);
  }
};

template <int NV, int KFULL, int NL>
__global__ __launch_bounds__(kRowThreads) void fp8_rollout_logprob_table_kernel(
    const bf16_t* __restrict__ logits, long long row_stride, int vocab, const int* __restrict__ token_ids,
    const unsigned char* __restrict__ valid, float* __restrict__ logp_out, int* __restrict__ status,
    long long n_rows) {
  typedef LogprobTable<(NL > 0)> Tab;
  __shared__ float lds_mm[2 * kRowWaves];
  __shared__ float lds_sum[kRowWaves];
  __shared__ float table[Tab::kFloats];                    // kTabEntries magnitudes x 2 signs in use
  extern __shared__ __align__(16) unsigned char lds_slots[];
  u32x4* lrow = reinterpret_cast<u32x4*>(lds_slots);       // NL slots
  static_assert(NL == 0 || KFULL == NV, "rows that need slots fill every register vector");
  const int tid = threadIdx.x;
  const int nvec = vocab / 8;
  const int tail = vocab - nvec * 8;
  // this workgroup's next evaluated row at or after `r`; rows that are not evaluated get their 0 on the way
  auto next_row = [&](long long r) -> long long {
    for (; r < n_rows; r += gridDim.x) {
      if (valid == nullptr || valid[r] != 0) break;        // uniform
      if (tid == 0) logp_out[r] = 0.f;
    }
    return r;
  };
  long long row = next_row(blockIdx.x);
  if (row >= n_rows) return;
  u32x4 q[NV];
  float xt;
  issue_row<NV, KFULL>(logits + row * row_stride, vocab, q, xt);
  if (NL > 0) {
    int t0 = tid;
    asm volatile("" : "+v"(t0));
#pragma unroll
    for (int j = 0; j < NL; ++j) {
      copy_to_slot(reinterpret_cast<const u32x4*>(logits + row * row_stride), nvec, NV + j, lrow + j * kRowThreads, t0);
      __builtin_amdgcn_sched_barrier(0);
    }
  }
  while (row < n_rows) {
    const bf16_t* zr = logits + row * row_stride;
    const long long next = next_row(row + gridDim.x);
    // after its last row a workgroup fetches that row once more (into registers nobody reads again): the loop
    // body stays free of conditions, which keeps the reloaded registers the very ones that were just read
    const u32x4* zn = reinterpret_cast<const u32x4*>(logits + (next < n_rows ? next : row) * row_stride);
    // the sampled token's logit: asked for before the prefetches below, which it would otherwise queue behind
    const int y = token_ids[row];
    const bool y_ok = y >= 0 && y < vocab;
    const float zy_raw = (tid == 0 && y_ok) ? Vec<bf16_t>::load1(zr + y) : 0.f;

    float zmax, zmin;
    row_minmax<NV, NL>(q, xt, lds_mm, zmax, zmin, lrow);
    const float amax = fmaxf(zmax, -zmin);
    const float s = scale_of(amax);
    const float scale = s * kLog2e;                        // z_r * log2e = value(code) * scale
    // quantisation is monotone: the largest round-tripped logit is that of the largest logit
    const float top = value_of(code_of(zmax / s)) * scale;
    // entry i belongs to the bf16 magnitude with bits base + i; the abs-max is the last entry or an earlier one
    const int base = max((int)(__float_as_uint(amax) >> 16) - (kTabEntries - 1), 0);
    for (int i = tid; i < kTabEntries; i += kRowThreads) {
      const float v = value_of(code_of(bf16_bits_to_float(base + i) / s));
      table[Tab::pos(i)] = exp2_fast(__builtin_fmaf(v, scale, -top));
      table[Tab::neg(i)] = exp2_fast(__builtin_fmaf(-v, scale, -top));
    }
    __syncthreads();
    const uint32_t base2 = (uint32_t)base * 0x00010001u;
    auto at = [&](uint32_t byte_offset) -> float {
      return *reinterpret_cast<const float*>(reinterpret_cast<const unsigned char*>(table) + byte_offset);
    };
    auto term = [&](uint32_t h) -> float { return at(Tab::offsets(h, base2) & 0xffffu); };   // h: one bf16, low half
    // sum of the eight terms of one vector
    auto vector_sum = [&](const u32x4& v) -> float {
      float part = 0.f;
#pragma unroll
      for (int w = 0; w < 4; ++w) {
        const uint32_t o = Tab::offsets(v[w], base2);
        part += at(o & 0xffffu);
        part += at(o >> 16);
        if (w == 1) {
          asm volatile("" : "+v"(part));                   // the sum so far is formed here, not deferred
          __builtin_amdgcn_sched_barrier(0);               // four table reads in flight at a time: fewer registers
        }
      }
      asm volatile("" : "+v"(part));
      __builtin_amdgcn_sched_barrier(0);
      return part;
    };
    float acc0 = 0.f;
#pragma unroll
    for (int k = 0; k < NV; ++k) {
      const float part = vector_sum(q[k]);
      // slots past the end of the row hold zeros, which would count as logits of 0; the slot's index comes from a
      // fresh opaque copy of the thread index, so that no per-slot offset is kept alive across the row loop
      int tk = tid;
      asm volatile("" : "+v"(tk));
      __builtin_assume(tk >= 0 && tk < kRowThreads);
      const int i = tk + k * kRowThreads;
      const bool exists = k < KFULL || i < nvec;
      acc0 += exists ? part : 0.f;
      // this vector is done with: its registers take the same vector of the next row (a slot past the end of the
      // row takes a copy of the row's last vector, which changes neither maximum nor minimum and is never summed)
      // (i >= 0 and nvec >= 1, so the clamped index is a valid vector of the row; uniform row base + 32-bit offset)
      q[k] = load_stream(zn + (unsigned)(k < KFULL ? i : min(i, nvec - 1)));
      __builtin_amdgcn_sched_barrier(0);
    }
#pragma unroll
    for (int j = 0; j < NL; ++j) {
      int tk = tid;
      asm volatile("" : "+v"(tk));
      __builtin_assume(tk >= 0 && tk < kRowThreads);
      u32x4* slot = lrow + j * kRowThreads;
      const float part = vector_sum(slot[tk]);             // (the terms have been read out of LDS: `part` is formed)
      acc0 += (tk + (NV + j) * kRowThreads < nvec) ? part : 0.f;
      // the thread's 16 bytes of the slot are free: they take the next row's vector
      copy_to_slot(zn, nvec, NV + j, slot, tk);
      __builtin_amdgcn_sched_barrier(0);
    }
    if (tid < tail) {
      acc0 += term(__float_as_uint(xt) >> 16);
      xt = Vec<bf16_t>::load1(reinterpret_cast<const bf16_t*>(zn) + nvec * 8 + tid);
    }
    const float acc = wave_sum(acc0);
    if ((tid & 63) == 0) lds_sum[tid >> 6] = acc;
    // also: everyone has finished reading the table.  With slots the barrier is written out: a workgroup fence would
    // wait for the copies of the next row that are on their way into the slots, which is what they are there to avoid
    // (nothing reads a slot before row_minmax has waited for them).
    if (NL > 0) asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
    else __syncthreads();
    if (tid == 0) {
      float sum = lds_sum[0];
#pragma unroll
      for (int w = 1; w < kRowWaves; ++w) sum += lds_sum[w];
      if (y_ok) {
        const float zy = value_of(code_of(zy_raw / s)) * s;
        logp_out[row] = zy - (top + log2_fast(sum)) * kLn2;
      } else {
        logp_out[row] = 0.f;
        atomicOr(status, AIS_STATUS_BAD_TOKEN);
      }
    }
    row = next;
  }
  // copies of the row fetched once more may still be on their way into the slots
  if (NL > 0) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
}

// Vectors per lane of a 16-byte aligned bf16 row, or 0 when the row does not qualify for these kernels.
int table_vectors_per_lane(const void* z, int vocab, long long row_stride, int most) {
  const bool ok16 = reinterpret_cast<uintptr_t>(z) % 16 == 0 && (row_stride * 2) % 16 == 0;
  const int need = (vocab / 8 + kRowThreads - 1) / kRowThreads;
  return (ok16 && need >= 1 && need <= most) ? need : 0;     // at least one whole vector per row
}

}  // namespace

// PREV: the widest row of the previous class; a row that reaches a class has more than PREV * 1024 vectors
#define AIS_TABLE_CASES(CASE) CASE(0, 4) CASE(4, 8) CASE(8, 12) CASE(12, 16) CASE(16, 18) CASE(18, 19) CASE(19, 20)

// Returns true when the table kernel was launched, false when the rows do not qualify (not bf16, not 16-byte
// aligned, wider than 24 vectors per lane, or codes not 8-byte aligned).
bool try_fp8_quantize_table(ais_ctx* ctx, const void* logits, ais_dtype dtype, long long n_rows, int vocab,
                            long long row_stride, unsigned char* codes, long long codes_stride, float* scale_out) {
  if (dtype != AIS_BF16) return false;
  if (reinterpret_cast<uintptr_t>(codes) % 8 != 0 || codes_stride % 8 != 0) return false;
  const int need = table_vectors_per_lane(logits, vocab, row_stride, 24);
  if (need == 0) return false;
  const bf16_t* z = static_cast<const bf16_t*>(logits);
  // persistent: one workgroup per compute unit (a workgroup's registers leave room for no second one)
  dim3 grid((unsigned)(n_rows < ctx->n_cus ? n_rows : ctx->n_cus)), block(kRowThreads);
#define AIS_CASE(PREV, NVAL)                                                                                  \
  if (need <= NVAL) {                                                                                         \
    fp8_quantize_table_kernel<NVAL, PREV><<<grid, block, 0, ctx->stream>>>(z, row_stride, vocab, codes,       \
                                                                           codes_stride, scale_out, n_rows);  \
    return true;                                                                                              \
  }
  AIS_TABLE_CASES(AIS_CASE)
  AIS_CASE(20, 24)
#undef AIS_CASE
  return false;
}

bool try_fp8_rollout_logprob_table(ais_ctx* ctx, const void* logits, ais_dtype dtype, long long n_rows, int vocab,
                                   long long row_stride, const int* token_ids, const unsigned char* valid,
                                   float* logp_out) {
  if (dtype != AIS_BF16) return false;
  // 23 vectors per lane in registers, 8 more in LDS slots beside the table
  const int need = table_vectors_per_lane(logits, vocab, row_stride, 23 + 8);
  if (need == 0) return false;
  const bf16_t* z = static_cast<const bf16_t*>(logits);
  // persistent: one workgroup per compute unit (a workgroup's registers and table leave room for no second one)
  dim3 grid((unsigned)(n_rows < ctx->n_cus ? n_rows : ctx->n_cus)), block(kRowThreads);
#define AIS_CASE(PREV, NVAL)                                                                                        \
  if (need <= NVAL) {                                                                                               \
    fp8_rollout_logprob_table_kernel<NVAL, PREV, 0><<<grid, block, 0, ctx->stream>>>(                               \
        z, row_stride, vocab, token_ids, valid, logp_out, ctx->status_dev, n_rows);                                 \
    return true;                                                                                                    \
  }
  AIS_TABLE_CASES(AIS_CASE)
  AIS_CASE(20, 21)
  AIS_CASE(21, 22)
  AIS_CASE(22, 23)
#undef AIS_CASE
#define AIS_CASE(NEED, NLVAL)                                                                                       \
  if (need <= NEED) {                                                                                               \
    auto kernel = fp8_rollout_logprob_table_kernel<23, 23, NLVAL>;                                                  \
    static std::once_flag once[kMaxDevices];               /* the attribute belongs to the function on one device */ \
    static bool ok[kMaxDevices];                                                                                    \
    if (!allow_dynamic_lds(ctx, reinterpret_cast<const void*>(kernel), NLVAL * kSlotBytes, once, ok))              \
      return false;                                        /* the caller falls back to the streaming kernel */     \
    kernel<<<grid, block, NLVAL * kSlotBytes, ctx->stream>>>(z, row_stride, vocab, token_ids, valid, logp_out,      \
                                                             ctx->status_dev, n_rows);                              \
    return true;                                                                                                    \
  }
  AIS_CASE(27, 4)
  AIS_CASE(31, 8)
#undef AIS_CASE
  return false;
}

}  // namespace ais
