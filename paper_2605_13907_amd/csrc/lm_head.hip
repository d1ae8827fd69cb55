// Token log-probabilities straight from the final hidden states and the output-embedding matrix:
// the [rows x vocab] logits are produced tile by tile on the matrix cores and folded into a running
// (max, sum) per token while they are still in the accumulators, so they never reach memory.
//
//   z[t, v] = sum_d H[t, d] W[v, d],   logp_t = z[t, y_t] / T - log sum_v exp(z[t, v] / T)
//
// This is a dense contraction (2 * rows * vocab * d_model flops against (rows + vocab) * d_model inputs),
// bound by the MFMA rate, unlike the sweeps over materialised logits, which are bound by HBM.
//
// Layout of the work.  The product is taken transposed, C^T[v, t] = W H^T, with v_mfma_f32_32x32x16_bf16:
// a lane of the wavefront then owns one *token* column of every 32x32 tile and 16 vocabulary entries of
// it, so the running softmax state of a token lives in one lane's registers and the reduction over the
// vocabulary needs no cross-lane traffic until the very end.  A 512-thread workgroup (8 wavefronts,
// 2 along the vocabulary x 4 along the tokens, 128 x 64 outputs each) computes 256 vocabulary entries x
// 256 tokens per tile, stepping through d_model 64 at a time: both operand slices (2 x 32 KiB) are staged
// through LDS with an XOR swizzle of the 16-byte chunks so that the fragment reads are free of bank
// conflicts, double-buffered so that one barrier per step suffices, and the global loads of the next
// step are in flight while the 32 MFMAs of the current one run.  A workgroup owns one block of 256
// tokens and a contiguous chunk of vocabulary tiles; per token and chunk it emits a partial (max, sum),
// and a small second kernel merges the partials and subtracts.  Workgroups are numbered so that those
// resident on one XCD (which share an L2) work on a few token blocks x a few vocabulary chunks at the
// same time, and therefore share both operands.
#include "ais_internal.h"
#include "device_utils.h"

namespace ais {
namespace {

using namespace dev;

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kLmThreads = 512;
constexpr int kLmTileV = 256;      // vocabulary entries per tile
constexpr int kLmTileT = 256;      // tokens per tile
constexpr int kLmTileK = 64;       // d_model elements per step
constexpr int kLmWaveV = 128;      // per wavefront: 4 MFMA tiles along the vocabulary
constexpr int kLmWaveT = 64;       //                2 along the tokens
constexpr int kLmOperandBytes = kLmTileV * kLmTileK * 2;            // 32 KiB: one operand slice
constexpr int kLmStageBytes = 2 * kLmOperandBytes;                   // W slice then H slice
constexpr int kLmLdsBytes = 2 * kLmStageBytes;                       // double buffer: 128 KiB

// Byte offset of 16-byte chunk `c` (0..7) of row `row` inside one operand slice.  A row is 128 bytes; the
// chunk index is XORed with bits 1..3 of the row so that 16 consecutive rows read at the same logical
// chunk touch 16 different 16-byte bank groups.
__device__ __forceinline__ int lds_chunk_offset(int row, int c) { return row * 128 + ((c ^ ((row >> 1) & 7)) << 4); }

__device__ __forceinline__ bf16x8 as_bf16x8(u32x4 q) { return __builtin_bit_cast(bf16x8, q); }

// One workgroup: token block `tb`, vocabulary tiles [vt0, vt1).  KTAIL: d_model is not a multiple of the
// 64-element step, so the last step's chunks past the end are replaced by zeros.
template <bool KTAIL>
__global__ __launch_bounds__(kLmThreads) void lm_head_partial_kernel(
    const bf16_t* __restrict__ hidden, long long ld_h, const bf16_t* __restrict__ weight, long long ld_w,
    int n_rows, int d_model, int vocab, const int* __restrict__ token_ids, const unsigned char* __restrict__ valid,
    float scale, int n_items, int n_chunks, int tiles_per_chunk, int n_vtiles, float* __restrict__ part_m,
    float* __restrict__ part_s, float* __restrict__ zy_out) {
  extern __shared__ __align__(16) unsigned char lds[];
  // Workgroups are dealt to the 8 XCDs round-robin; give every XCD a contiguous range of work items.
  const int per_xcd = gridDim.x >> 3;
  const int item = (int)(blockIdx.x & 7) * per_xcd + (int)(blockIdx.x >> 3);
  if (item >= n_items) return;                                  // uniform for the workgroup
  const int tb = item / n_chunks, ch = item - tb * n_chunks;
  const int vt0 = ch * tiles_per_chunk;
  const int vt1 = min(n_vtiles, vt0 + tiles_per_chunk);
  const int t0 = tb * kLmTileT;

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int wv = wave & 1, wt = wave >> 1;                      // position of the wavefront in the tile
  const int half = lane >> 5, col = lane & 31;

  // ---- global -> LDS staging: thread owns chunk c of rows r0 + 64 i of both operand slices
  const int c = tid & 7, r0 = tid >> 3;
  const bf16_t* hp[4];
  const bf16_t* wp[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int trow = min(t0 + r0 + 64 * i, n_rows - 1);         // rows past the end repeat the last one; discarded later
    hp[i] = hidden + (long long)trow * ld_h + c * 8;
  }
  auto point_w = [&](int vt) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int vrow = min(vt * kLmTileV + r0 + 64 * i, vocab - 1);
      wp[i] = weight + (long long)vrow * ld_w + c * 8;
    }
  };
  const int st_off = lds_chunk_offset(r0, c);                   // + 8 KiB per i: 64 rows further down
  u32x4 sw[4], sh[4];
  const u32x4 zero4 = {0u, 0u, 0u, 0u};
  (void)zero4;
  auto fetch = [&](int k0) {
    if (KTAIL) {
      // d_model is a multiple of 8: a chunk is wholly inside or wholly outside; outside chunks re-read the
      // row's first chunk (a valid address) and are zeroed
      const bool in = k0 + c * 8 < d_model;
      const int k = in ? k0 : -c * 8;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const u32x4 w = *reinterpret_cast<const u32x4*>(wp[i] + k);
        const u32x4 h = *reinterpret_cast<const u32x4*>(hp[i] + k);
        sw[i] = in ? w : zero4;
        sh[i] = in ? h : zero4;
      }
    } else {
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        sw[i] = *reinterpret_cast<const u32x4*>(wp[i] + k0);
        sh[i] = *reinterpret_cast<const u32x4*>(hp[i] + k0);
      }
    }
  };
  auto stage = [&](int buf) {
    unsigned char* base = lds + buf * kLmStageBytes + st_off;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      *reinterpret_cast<u32x4*>(base + i * 8192) = sw[i];
      *reinterpret_cast<u32x4*>(base + kLmOperandBytes + i * 8192) = sh[i];
    }
  };

  // ---- LDS -> MFMA fragments: lane reads row (32-row tile base + col), chunk 2 kk + half
  int frag_off[4];
#pragma unroll
  for (int kk = 0; kk < 4; ++kk) frag_off[kk] = lds_chunk_offset(col, 2 * kk + half);
  const int a_base = wv * kLmWaveV * 128;                          // W rows of this wavefront
  const int b_base = kLmOperandBytes + wt * kLmWaveT * 128;        // H rows of this wavefront

  f32x16 acc[4][2];
  auto clear_acc = [&]() {
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
  };
  // Fragments of step kk + 1 are requested before the MFMAs of step kk are issued; the scheduling barriers keep
  // the compiler from hoisting all four steps' reads to the top (96 more live registers).
  auto read_frags = [&](const unsigned char* base, int kk, bf16x8 (&a)[4], bf16x8 (&b)[2]) {
#pragma unroll
    for (int i = 0; i < 4; ++i)
      a[i] = as_bf16x8(*reinterpret_cast<const u32x4*>(base + a_base + i * 4096 + frag_off[kk]));
#pragma unroll
    for (int j = 0; j < 2; ++j)
      b[j] = as_bf16x8(*reinterpret_cast<const u32x4*>(base + b_base + j * 4096 + frag_off[kk]));
  };
  auto multiply = [&](int buf) {
    const unsigned char* base = lds + buf * kLmStageBytes;
    bf16x8 a[2][4], b[2][2];
    read_frags(base, 0, a[0], b[0]);
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
      if (kk < 3) read_frags(base, kk + 1, a[(kk + 1) & 1], b[(kk + 1) & 1]);
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[kk & 1][i], b[kk & 1][j], acc[i][j], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
    }
  };

  // ---- per-lane softmax state of its two token columns, in the base-2 domain (x * scale)
  float run_m[2] = {kNegHuge, kNegHuge}, run_s[2] = {0.f, 0.f};
  int tok[2], y[2];
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    tok[j] = t0 + wt * kLmWaveT + j * 32 + col;
    y[j] = -1;
    if (tok[j] < n_rows && (valid == nullptr || valid[tok[j]] != 0)) {
      const int id = token_ids[tok[j]];
      y[j] = (id >= 0 && id < vocab) ? id : -1;
    }
  }
  // accumulator element v of MFMA tile i holds vocabulary entry  vbase + 32 i + 8 (v / 4) + 4 half + v % 4
  auto fold_tile = [&](int vt) {
    const int vbase = vt * kLmTileV + wv * kLmWaveV;
    if (vt * kLmTileV + kLmTileV > vocab) {                      // uniform: only the last tile of the vocabulary
      // entries past the end of the vocabulary become -inf: they never win the max (which starts from a
      // finite value) and add exp2(-inf) = 0 to the sum
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const bool in = vbase + 32 * i + 8 * (v >> 2) + 4 * half + (v & 3) < vocab;
#pragma unroll
          for (int j = 0; j < 2; ++j) acc[i][j][v] = in ? acc[i][j][v] : -__builtin_inff();
        }
    }
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      float tmax = kNegHuge;
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) tmax = fmaxf(tmax, acc[i][j][v]);
      const float m_new = fmaxf(run_m[j], tmax * scale);         // finite: run_m is, and -inf never wins
      float sum = 0.f;
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) sum += exp2_fast(fmaf(acc[i][j][v], scale, -m_new));
      run_s[j] = fmaf(run_s[j], exp2_fast(run_m[j] - m_new), sum);
      run_m[j] = m_new;
      // the sampled token's own logit: held by exactly one lane of one wavefront of one workgroup
      const int rel = y[j] - vbase;
      if ((unsigned)rel < (unsigned)kLmWaveV && ((rel >> 2) & 1) == half) {
        const int idx = (rel >> 5) * 16 + ((rel & 31) >> 3) * 4 + (rel & 3);
        float zy = 0.f;
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
          for (int v = 0; v < 16; ++v) zy = (i * 16 + v == idx) ? acc[i][j][v] : zy;
        zy_out[tok[j]] = zy;
      }
    }
  };

  // ---- main loop over (vocabulary tile, d_model step), flattened so that the prefetch crosses tiles
  const int n_ksteps = (d_model + kLmTileK - 1) / kLmTileK;
  int vt = vt0, kt = 0, buf = 0;
  point_w(vt);
  fetch(0);
  clear_acc();
  for (;;) {
    stage(buf);
    __syncthreads();
    int nkt = kt + 1, nvt = vt;
    if (nkt == n_ksteps) { nkt = 0; nvt = vt + 1; }
    const bool more = nvt < vt1;
    if (more) {
      if (nkt == 0) point_w(nvt);
      fetch(nkt * kLmTileK);
    }
    multiply(buf);
    if (kt == n_ksteps - 1) {
      fold_tile(vt);
      clear_acc();
    }
    if (!more) break;
    kt = nkt;
    vt = nvt;
    buf ^= 1;
  }

  // ---- merge the two lane halves, then the two wavefronts along the vocabulary, and emit the partial
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    const float om = __shfl_xor(run_m[j], 32), os = __shfl_xor(run_s[j], 32);
    const float m = fmaxf(run_m[j], om);
    run_s[j] = run_s[j] * exp2_fast(run_m[j] - m) + os * exp2_fast(om - m);
    run_m[j] = m;
  }
  __syncthreads();                                              // everyone is done with the staging buffers
  float* xm = reinterpret_cast<float*>(lds);                    // [4 token groups][64 tokens] max, then sum
  float* xs = xm + 256;
  if (wv == 1 && half == 0) {
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      xm[wt * 64 + j * 32 + col] = run_m[j];
      xs[wt * 64 + j * 32 + col] = run_s[j];
    }
  }
  __syncthreads();
  if (wv == 0 && half == 0) {
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const float om = xm[wt * 64 + j * 32 + col], os = xs[wt * 64 + j * 32 + col];
      const float m = fmaxf(run_m[j], om);
      const float s = run_s[j] * exp2_fast(run_m[j] - m) + os * exp2_fast(om - m);
      if (tok[j] < n_rows) {
        part_m[(long long)ch * n_rows + tok[j]] = m;
        part_s[(long long)ch * n_rows + tok[j]] = s;
      }
    }
  }
}

// lse and log-prob from the per-chunk partials.  One thread per token.
__global__ __launch_bounds__(256) void lm_head_merge_kernel(const float* __restrict__ part_m,
                                                            const float* __restrict__ part_s,
                                                            const float* __restrict__ zy, int n_rows, int n_chunks,
                                                            int vocab, const int* __restrict__ token_ids,
                                                            const unsigned char* __restrict__ valid,
                                                            float inv_temperature, float* __restrict__ logp_out,
                                                            float* __restrict__ lse_out, int* __restrict__ status) {
  const int n = blockIdx.x * 256 + threadIdx.x;
  if (n >= n_rows) return;
  if (valid != nullptr && valid[n] == 0) {
    logp_out[n] = 0.f;
    lse_out[n] = 0.f;
    return;
  }
  float m = kNegHuge;
  for (int k = 0; k < n_chunks; ++k) m = fmaxf(m, part_m[(long long)k * n_rows + n]);
  double s = 0.0;
  for (int k = 0; k < n_chunks; ++k)
    s += (double)part_s[(long long)k * n_rows + n] * (double)exp2_fast(part_m[(long long)k * n_rows + n] - m);
  const double lse = ((double)m + log2(s)) * 0.6931471805599453;
  lse_out[n] = (float)lse;
  const int id = token_ids[n];
  if (id >= 0 && id < vocab) {
    logp_out[n] = (float)((double)zy[n] * (double)inv_temperature - lse);
  } else {
    logp_out[n] = 0.f;
    atomicOr(status, AIS_STATUS_BAD_TOKEN);
  }
}

}  // namespace

// Splits the vocabulary tiles into equal chunks so that (token blocks x chunks) work items of equal size
// fill the compute units in as few rounds as possible.
LmHeadPlan lm_head_plan(long long n_rows, int vocab, int n_cus) {
  LmHeadPlan p;
  p.n_tblocks = (int)((n_rows + kLmTileT - 1) / kLmTileT);
  p.n_vtiles = (vocab + kLmTileV - 1) / kLmTileV;
  long long best = -1;
  p.tiles_per_chunk = p.n_vtiles;
  p.n_chunks = 1;
  for (int chunks = 1; chunks <= p.n_vtiles && chunks <= 64; ++chunks) {
    const int tpc = (p.n_vtiles + chunks - 1) / chunks;
    const int real = (p.n_vtiles + tpc - 1) / tpc;
    const long long items = (long long)p.n_tblocks * real;
    const long long rounds = (items + n_cus - 1) / n_cus;
    const long long cost = rounds * (tpc + 1);            // + 1: set-up and tear-down of a work item, in tile units
    if (best < 0 || cost < best) {
      best = cost;
      p.tiles_per_chunk = tpc;
      p.n_chunks = real;
    }
  }
  return p;
}

int launch_lm_head_logprob(ais_ctx* ctx, const void* hidden, long long ld_h, const void* weight, long long ld_w,
                           long long n_rows, int d_model, int vocab, const int* token_ids,
                           const unsigned char* valid, float inv_temperature, const LmHeadPlan& plan,
                           float* part_m, float* part_s, float* zy, float* logp_out, float* lse_out) {
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(lm_head_partial_kernel<false>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, kLmLdsBytes);
    if (e == hipSuccess)
      e = hipFuncSetAttribute(reinterpret_cast<const void*>(lm_head_partial_kernel<true>),
                              hipFuncAttributeMaxDynamicSharedMemorySize, kLmLdsBytes);
    if (e != hipSuccess) return hip_fail(ctx, e);
    attr_set = true;
  }
  const int n_items = plan.n_tblocks * plan.n_chunks;
  const int grid = ((n_items + 7) / 8) * 8;
  {
    ScopedTimer timer(ctx, AIS_K_LM_HEAD);
    auto kernel = (d_model % kLmTileK != 0) ? lm_head_partial_kernel<true> : lm_head_partial_kernel<false>;
    kernel<<<grid, kLmThreads, kLmLdsBytes, ctx->stream>>>(
        static_cast<const bf16_t*>(hidden), ld_h, static_cast<const bf16_t*>(weight), ld_w, (int)n_rows, d_model,
        vocab, token_ids, valid, inv_temperature * kLog2e, n_items, plan.n_chunks, plan.tiles_per_chunk,
        plan.n_vtiles, part_m, part_s, zy);
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return hip_fail(ctx, e);
  lm_head_merge_kernel<<<(unsigned)((n_rows + 255) / 256), 256, 0, ctx->stream>>>(
      part_m, part_s, zy, (int)n_rows, plan.n_chunks, vocab, token_ids, valid, inv_temperature, logp_out, lse_out,
      ctx->status_dev);
  return hip_fail(ctx, hipGetLastError());
}

}  // namespace ais
