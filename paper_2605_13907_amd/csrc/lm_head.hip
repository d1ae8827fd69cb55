// Token log-probabilities straight from the final hidden states and the output-embedding matrix:
// the [rows x vocab] logits are produced tile by tile on the matrix cores and folded into a running
// (max, sum) per token while they are still in the accumulators, so they never reach memory.
//
//   z[t, v] = sum_d H[t, d] W[v, d],   logp_t = z[t, y_t] / T - log sum_v exp(z[t, v] / T)
//
// This is a dense contraction (2 * rows * vocab * d_model flops against (rows + vocab) * d_model inputs),
// a matrix-core kernel, unlike the sweeps over materialised logits, which are bound by HBM.
//
// Layout of the work.  The product is taken transposed, C^T[v, t] = W H^T, with v_mfma_f32_32x32x16_bf16:
// a lane of the wavefront then owns one *token* column of every 32x32 tile and 16 vocabulary entries of
// it, so the running softmax state of a token lives in one lane's registers and the reduction over the
// vocabulary needs no cross-lane traffic until the very end.  A 512-thread workgroup (8 wavefronts,
// 2 along the vocabulary x 4 along the tokens, 128 x 64 outputs each) computes 256 vocabulary entries x
// 256 tokens per tile.  It owns one block of 256 tokens and a contiguous chunk of vocabulary tiles; per
// token and chunk it emits a partial (max, sum), and a small second kernel merges the partials and
// subtracts.  Workgroups are numbered so that those resident on one XCD (which share an L2) work on a few
// token blocks x all vocabulary chunks at the same time, and therefore share both operands.
//
// Three kernels do the tile arithmetic.  The streaming kernels copy operand slices from global memory straight into
// LDS and interleave copies, LDS reads and MFMAs one by one: slices of 64 elements of d_model in two buffers when
// d_model is a multiple of 64 (a row of a slice is then a whole 128-byte line: half the L2 requests of 64-byte
// rows for the same bytes), slices of 32 elements in a ring of four stages when it is a multiple of 32; the
// register-staged kernel accepts any d_model that is a multiple of 8.  All keep the operand slices in LDS with an
// XOR swizzle of their 16-byte chunks, which makes the fragment reads free of bank conflicts (measured: none).
//
// What bounds it.  With 256 x 256 tiles every MFMA needs 256 bytes from L2 and, with 128 x 64 outputs per wavefront,
// 768 bytes of fragments from LDS; under a sustained run with real (toggling) data the part is also power-limited
// (the shader clock settles near 1.7 GHz instead of 2.4).  Measured at the Qwen3-8B shape on one device: 41.0-41.5 ms
// with 64-element slices (1.25-1.26 PFLOP/s), 43.4 ms with 32-element slices; the same kernel with the copies left
// out (wrong results, timing only) 34.3 ms, with every copy fetching a slice that is already in L2 39.1 ms; the
// library GEMM that materialises the logits 34.5 ms (1.50 PFLOP/s).
#include "ais_internal.h"
#include "device_utils.h"

#include <type_traits>

namespace ais {
namespace {

using namespace dev;

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kLmThreads = 512;
constexpr int kLmTileV = 256;      // vocabulary entries per tile
constexpr int kLmTileT = 256;      // tokens per tile
constexpr int kLmTileK = 64;       // d_model elements per step of the register-staged kernel
constexpr int kLmWaveV = 128;      // per wavefront: 4 MFMA tiles along the vocabulary
constexpr int kLmWaveT = 64;       //                2 along the tokens
// Token blocks that walk the vocabulary chunks together (see LmItem::init).  1 = token block major: the workgroups
// resident on an XCD share a few hidden-state blocks and sit on all chunks of the vocabulary.  Measured at 41,643
// rows x 151,936 x 4,096: 43.9 ms; groups of 2 / 4 / 8 / 16 / 32 token blocks on the same chunk (more sharing of the
// output-embedding tiles, less of the hidden-state block, which a work item re-reads for every vocabulary tile):
// 44.3 / 47.4 / 47.5 / 50.1 / 52.9 ms.
constexpr int kLmTokenBlockGroup = 1;
__device__ __forceinline__ bf16x8 as_bf16x8(u32x4 q) { return __builtin_bit_cast(bf16x8, q); }


// ---- pieces shared by the two kernels ---------------------------------------------------------------------

// Decomposition of the evaluated rows into work items, decided on the device once their number is known
// (lm_head_setup_kernel): n_tblocks blocks of 256 evaluated rows x n_chunks chunks of tiles_per_chunk
// vocabulary tiles, per_xcd work items for each of the 8 XCDs.
struct LmDevPlan {
  int n_eval, n_tblocks, n_chunks, tiles_per_chunk, per_xcd, n_items, tb_group;
};

// Splits n_vtiles vocabulary tiles into equal chunks so that (token blocks x chunks) equal work items fill the
// compute units in as few rounds as possible.  Workgroups are bound to XCDs by their index, so what counts is
// the rounds of the busiest XCD (n_cus / 8 units each).  At most max_items items, at most 64 chunks.
__host__ __device__ inline void lm_choose_chunks(int n_tblocks, int n_vtiles, int n_cus, long long max_items,
                                                 int* n_chunks, int* tiles_per_chunk) {
  const int cus_per_xcd = n_cus >= 8 ? n_cus / 8 : 1;
  long long best = -1;
  *n_chunks = 1;
  *tiles_per_chunk = n_vtiles;
  for (int chunks = 1; chunks <= n_vtiles && chunks <= 64; ++chunks) {
    const int tpc = (n_vtiles + chunks - 1) / chunks;
    const int real = (n_vtiles + tpc - 1) / tpc;
    const long long items = (long long)n_tblocks * real;
    if (items > max_items && chunks > 1) continue;
    const long long per_xcd = (items + 7) / 8;
    const long long rounds = (per_xcd + cus_per_xcd - 1) / cus_per_xcd;
    const long long cost = rounds * (tpc + 1);            // + 1: set-up and tear-down of a work item, in tile units
    if (best < 0 || cost < best) {
      best = cost;
      *tiles_per_chunk = tpc;
      *n_chunks = real;
    }
  }
}

// The rows to evaluate.  With a mask, `index` lists the evaluated rows in order (built by
// lm_head_setup_kernel); without one, every row is evaluated.
struct LmRows {
  const int* index;
  int n_rows;
  // source row of evaluated position p (positions past the end repeat the last one; their results are discarded)
  __device__ __forceinline__ int row(int p, int n_eval) const {
    p = min(p, n_eval - 1);
    return index != nullptr ? index[p] : p;
  }
};

// Which part of the problem this workgroup owns, and where the thread sits in its tile.
struct LmItem {
  int tb, ch, vt0, vt1, t0, n_eval, n_chunks;
  int lane, wave, wv, wt, half, col;
  __device__ __forceinline__ bool init(const LmDevPlan* __restrict__ plan, int n_vtiles) {
    // Workgroups are dealt to the 8 XCDs round-robin; every XCD takes a contiguous, equally long range of work
    // items (token block major): its resident workgroups then share a few token blocks' hidden-state slices and
    // each other's vocabulary tiles through the L2.
    const int xcd = blockIdx.x & 7, local = blockIdx.x >> 3;
    const int item = xcd * plan->per_xcd + local;
    if (local >= plan->per_xcd || item >= plan->n_items) return false;   // uniform for the workgroup
    n_eval = plan->n_eval;
    n_chunks = plan->n_chunks;
    const int tiles_per_chunk = plan->tiles_per_chunk;
    // items are ordered group by group of tb_group token blocks, chunk by chunk inside a group, token block by
    // token block inside a chunk: the workgroups resident on an XCD then sit on tb_group token blocks x a few chunks
    const int group = plan->tb_group, per_group = group * n_chunks;
    const int g = item / per_group, j = item - g * per_group;
    const int gsize = min(group, plan->n_tblocks - g * group);     // the last group may be smaller
    ch = j / gsize;
    tb = g * group + (j - ch * gsize);
    vt0 = ch * tiles_per_chunk;
    vt1 = min(n_vtiles, vt0 + tiles_per_chunk);
    t0 = tb * kLmTileT;
    lane = threadIdx.x & 63;
    wave = threadIdx.x >> 6;
    wv = wave & 1;                                               // position of the wavefront in the tile
    wt = wave >> 1;
    half = lane >> 5;
    col = lane & 31;
    return true;
  }
};

typedef f32x16 LmAcc[4][2];

__device__ __forceinline__ void lm_clear(LmAcc& acc) {
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
}

// Per-lane soft-max state of the lane's two token columns, in the base-2 domain (logit * scale).
struct LmSoftmax {
  float run_m[2], run_s[2];
  int tok[2], y[2];
  // tok[j]: evaluated position of the lane's token column j; y[j]: its sampled token, -1 if there is none to find
  __device__ __forceinline__ void init(const LmItem& it, const LmRows& rows, int vocab,
                                       const int* __restrict__ token_ids) {
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      run_m[j] = kNegHuge;
      run_s[j] = 0.f;
      tok[j] = it.t0 + it.wt * kLmWaveT + j * 32 + it.col;
      y[j] = -1;
      if (tok[j] < it.n_eval) {
        const int id = token_ids[rows.row(tok[j], it.n_eval)];
        y[j] = (id >= 0 && id < vocab) ? id : -1;
      }
    }
  }
  // Folds the finished tile `vt` into the running state.  Accumulator element v of MFMA tile i holds
  // vocabulary entry  vbase + 32 i + 8 (v / 4) + 4 half + v % 4  of token column j.
  __device__ __forceinline__ void fold(LmAcc& acc, const LmItem& it, int vt, int vocab, float scale,
                                       float* __restrict__ zy_out) {
    const int vbase = vt * kLmTileV + it.wv * kLmWaveV;
    if (vt * kLmTileV + kLmTileV > vocab) {                      // uniform: only the last tile of the vocabulary
      // entries past the end of the vocabulary become -inf: they never win the max (which starts from a
      // finite value) and add exp2(-inf) = 0 to the sum
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const bool in = vbase + 32 * i + 8 * (v >> 2) + 4 * it.half + (v & 3) < vocab;
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
      if ((unsigned)rel < (unsigned)kLmWaveV && ((rel >> 2) & 1) == it.half) {
        const int idx = (rel >> 5) * 16 + ((rel & 31) >> 3) * 4 + (rel & 3);
        float zy = 0.f;
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
          for (int v = 0; v < 16; ++v) zy = (i * 16 + v == idx) ? acc[i][j][v] : zy;
        zy_out[tok[j]] = zy;
        // the kernels count their outstanding global->LDS copies; this rare store must not be among them
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
      }
    }
  }
  // Merges the two lane halves, then the two wavefronts along the vocabulary (through `xch`, 2 KiB of LDS that
  // no one uses any more), and writes the chunk's partial (max, sum) of every token of the block.
  __device__ __forceinline__ void finish(const LmItem& it, float* xch, int n_rows, float* __restrict__ part_m,
                                         float* __restrict__ part_s) {
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const float om = __shfl_xor(run_m[j], 32), os = __shfl_xor(run_s[j], 32);
      const float m = fmaxf(run_m[j], om);
      run_s[j] = run_s[j] * exp2_fast(run_m[j] - m) + os * exp2_fast(om - m);
      run_m[j] = m;
    }
    __syncthreads();                                            // everyone is done with the staging buffers
    float* xm = xch;                                            // [4 token groups][64 tokens] max, then sum
    float* xs = xch + 256;
    if (it.wv == 1 && it.half == 0) {
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        xm[it.wt * 64 + j * 32 + it.col] = run_m[j];
        xs[it.wt * 64 + j * 32 + it.col] = run_s[j];
      }
    }
    __syncthreads();
    if (it.wv == 0 && it.half == 0) {
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const float om = xm[it.wt * 64 + j * 32 + it.col], os = xs[it.wt * 64 + j * 32 + it.col];
        const float m = fmaxf(run_m[j], om);
        const float s = run_s[j] * exp2_fast(run_m[j] - m) + os * exp2_fast(om - m);
        if (tok[j] < it.n_eval) {
          part_m[(long long)it.ch * n_rows + tok[j]] = m;
          part_s[(long long)it.ch * n_rows + tok[j]] = s;
        }
      }
    }
  }
};

// What the gradient variant of the streaming kernel needs besides the operands: per-row lse, log-prob and
// coefficient (inputs), and the block of dlogits it writes: rows x a chunk of the vocabulary, bf16, row-major.
struct LmGradArgs {
  const float* lse;        // [n_rows]  log sum_v exp(z / T), as written by the log-prob call
  const float* logp;       // [n_rows]  log-prob of the sampled token
  const float* coeff;      // [n_rows]  d loss / d (row's log-prob) times 1 / T; 0 on rows without gradient
  bf16_t* ds;              // [n_rows, ds_stride]  coeff (softmax - onehot) over this chunk of the vocabulary
  long long ds_stride;     // elements, a multiple of 4
  int y_off;               // first vocabulary entry of the chunk: token ids are global, tile indices local
  int compact;             // != 0: row p of ds belongs to the p-th listed row (LmRows::index), not to source row p
};

// Per-lane state of the gradient variant: for each of the lane's two token columns the row it writes to, the
// sampled token's position inside the chunk, -lse in the base-2 domain, the coefficient and the sampled token's
// own element coeff (p_y - 1) = coeff expm1(logp), which would cancel if it were formed from p_y.
struct LmGrad {
  long long row[2];
  int y[2];
  float shift[2], c[2], dy[2];
  __device__ __forceinline__ void init(const LmItem& it, const LmRows& rows, int vocab,
                                       const int* __restrict__ token_ids, const LmGradArgs& ga) {
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const int tok = it.t0 + it.wt * kLmWaveT + j * 32 + it.col;
      row[j] = -1;
      y[j] = -1;
      shift[j] = 0.f;
      c[j] = 0.f;
      dy[j] = 0.f;
      if (tok < it.n_eval) {
        const int r = rows.row(tok, it.n_eval);
        row[j] = ga.compact ? tok : r;
        c[j] = ga.coeff[r];
        if (c[j] != 0.f) {                  // rows without gradient: lse may be 0 there, and nothing is exponentiated
          const int id = token_ids[r] - ga.y_off;
          y[j] = (id >= 0 && id < vocab) ? id : -1;
          shift[j] = -ga.lse[r] * kLog2e;
          dy[j] = c[j] * expm1f(ga.logp[r]);
        }
      }
    }
  }
  // Writes the finished tile `vt`.  Accumulator element v of MFMA tile i holds vocabulary entry
  // vbase + 32 i + 8 (v / 4) + 4 half + v % 4 of token column j: four consecutive entries per (i, v / 4), 8 bytes.
  __device__ __forceinline__ void emit(const LmAcc& acc, const LmItem& it, int vt, int vocab, float scale,
                                       const LmGradArgs& ga) {
    const int vbase = vt * kLmTileV + it.wv * kLmWaveV;
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      if (row[j] < 0) continue;
      bf16_t* out = ga.ds + row[j] * ga.ds_stride;
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int v0 = vbase + 32 * i + 8 * q + 4 * it.half;
          if (v0 >= vocab) continue;
          float x[4];
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            x[e] = c[j] != 0.f ? c[j] * exp2_fast(fmaf(acc[i][j][4 * q + e], scale, shift[j])) : 0.f;
            if (v0 + e == y[j]) x[e] = dy[j];
          }
          if (v0 + 3 < vocab) {
            f32x2 lo = {x[0], x[1]}, hi = {x[2], x[3]};
            uint2 w = {__builtin_bit_cast(uint32_t, __builtin_convertvector(lo, bf16x2)),
                       __builtin_bit_cast(uint32_t, __builtin_convertvector(hi, bf16x2))};
            *reinterpret_cast<uint2*>(out + v0) = w;
          } else {
#pragma unroll
            for (int e = 0; e < 4; ++e)
              if (v0 + e < vocab) Vec<bf16_t>::store1(out + v0 + e, x[e]);
          }
        }
    }
    // the kernel counts its outstanding global->LDS copies; these stores must not be among them
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  }
};

typedef __attribute__((address_space(3))) void* lds_ptr;
typedef const __attribute__((address_space(1))) void* glb_ptr;

// ---- streaming kernel: d_model a multiple of 32 ---------------------------------------------------------------
// Steps of 32 elements of d_model; the two operand slices of a step (2 x 16 KiB) go from global memory straight
// into one of NS LDS stages (global_load_lds_dwordx4: lane i of a wavefront deposits its 16 bytes at base + 16 i,
// so the swizzle is applied by choosing which chunk each lane fetches).  The copies of step s + NS - 1 are issued
// during the second half of step s, NS - 2 steps before they are awaited, so the memory pipe stays busy across
// step boundaries.  One barrier per step, in its middle: it publishes step s + 1 (every wavefront has waited for
// its own copies) and retires step s - 1 (every wavefront has read what it needs), whose stage the new copies
// overwrite.  The instruction stream is pinned: each LDS read and each copy sits in the shadow of an MFMA, the
// fragments of step s + 1 are read during the second half of step s, and two MFMAs whose operands are already
// in registers are issued just before the barrier, so the matrix cores have work while the wavefronts gather.
constexpr int kStK = 32;
constexpr int kStOperandBytes = kLmTileV * kStK * 2;             // 16 KiB
constexpr int kStStageBytes = 2 * kStOperandBytes;               // 32 KiB

// 16-byte chunk c (0..3) of row `row` of a slice with 64-byte rows: XOR with bits 2..3 of the row makes 16
// consecutive rows, read at one logical chunk, cover all 16 bank groups.
__device__ __forceinline__ int st_chunk_offset(int row, int c) { return row * 64 + ((c ^ ((row >> 2) & 3)) << 4); }

// GRAD = false: every finished tile is folded into the running soft-max state (log-prob call).  GRAD = true: every
// finished tile is written out as coeff (softmax - onehot) in bf16, lse being an input (gradient call).
template <int NS, bool GRAD>
__global__ __launch_bounds__(kLmThreads) void lm_head_stream_kernel(
    const bf16_t* __restrict__ hidden, long long ld_h, const bf16_t* __restrict__ weight, long long ld_w,
    LmRows rows, const LmDevPlan* __restrict__ plan, int d_model, int vocab, const int* __restrict__ token_ids,
    float scale, int n_vtiles, float* __restrict__ part_m, float* __restrict__ part_s,
    float* __restrict__ zy_out, LmGradArgs ga) {
  extern __shared__ __align__(16) unsigned char lds[];
  LmItem it;
  if (!it.init(plan, n_vtiles)) return;
  const int n_rows = rows.n_rows;
  const int lane = it.lane, wave = it.wave;

  // ---- copies: wavefront w moves rows 16 w .. 16 w + 15 (+ 128 j) of each slice; a lane sits at chunk position
  // lane & 3 of row lane >> 2 and therefore fetches logical chunk (lane & 3) ^ ((row >> 2) & 3)
  const int crow = 16 * wave + (lane >> 2);
  const int cchunk = (lane & 3) ^ ((lane >> 4) & 3);
  const bf16_t* hp[2];
  const bf16_t* wp[2];
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    const int trow = rows.row(it.t0 + crow + 128 * j, it.n_eval);
    hp[j] = hidden + (long long)trow * ld_h + cchunk * 8;
  }
  auto point_w = [&](int vt) {
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const int vrow = min(vt * kLmTileV + crow + 128 * j, vocab - 1);
      wp[j] = weight + (long long)vrow * ld_w + cchunk * 8;
    }
  };
  const int n_ksteps = d_model / kStK;
  const int n_steps = (it.vt1 - it.vt0) * n_ksteps;
  // cursor of the next step to be copied
  int c_step = 0, c_kt = 0, c_vt = it.vt0;
  point_w(c_vt);
  // One of the four copy instructions (W rows, H rows, W rows + 128, H rows + 128) that bring the cursor's step
  // into LDS stage `stage`; the fourth advances the cursor.  They are issued one at a time between MFMAs: a
  // wavefront stalls while the memory pipe accepts a copy, and spreading them keeps those stalls short and out
  // of phase across wavefronts.  Once the cursor has reached the last step it stays there: the copies issued
  // after that re-fetch the last step into stages nobody reads any more, which keeps the number of outstanding
  // copies (and therefore the wait) the same in every step and the loop free of branches.
  auto copy_part = [&](int stage, int q) {
    unsigned char* base = lds + stage * kStStageBytes + wave * 1024 + (q >> 1) * 8192;
    const int k0 = c_kt * kStK;
    if ((q & 1) == 0)
      __builtin_amdgcn_global_load_lds((glb_ptr)(wp[q >> 1] + k0), (lds_ptr)base, 16, 0, 0);
    else
      __builtin_amdgcn_global_load_lds((glb_ptr)(hp[q >> 1] + k0), (lds_ptr)(base + kStOperandBytes), 16, 0, 0);
    if (q == 3 && c_step + 1 < n_steps) {
      ++c_step;
      if (++c_kt == n_ksteps) {
        c_kt = 0;
        ++c_vt;
        point_w(c_vt);
      }
    }
  };

  // ---- fragments: lane reads row (32-row tile base + col), chunk 2 kk + half of a 64-byte row
  int frag_off[2];
#pragma unroll
  for (int kk = 0; kk < 2; ++kk) frag_off[kk] = st_chunk_offset(it.col, 2 * kk + it.half);
  const int a_base = it.wv * kLmWaveV * 64;
  const int b_base = kStOperandBytes + it.wt * kLmWaveT * 64;
  // One fragment read.  The eight MFMAs of a half-step run in the order (a0,b0) (a0,b1) (a1,b0) (a1,b1) (a2,b0) ..., so
  // the fragments are needed, and therefore read, in the order a0 b0 b1 a1 a2 a3 (r = 0..5).
  auto read_frag = [&](int step, int kk, int r, bf16x8 (&a)[4], bf16x8 (&b)[2]) {
    const unsigned char* base = lds + (step % NS) * kStStageBytes + frag_off[kk];
    if (r == 1 || r == 2)
      b[r - 1] = as_bf16x8(*reinterpret_cast<const u32x4*>(base + b_base + (r - 1) * 2048));
    else {
      const int i = r == 0 ? 0 : r - 2;
      a[i] = as_bf16x8(*reinterpret_cast<const u32x4*>(base + a_base + i * 2048));
    }
  };
  auto read_frags = [&](int step, int kk, bf16x8 (&a)[4], bf16x8 (&b)[2]) {
#pragma unroll
    for (int r = 0; r < 6; ++r) read_frag(step, kk, r, a, b);
  };

  LmAcc acc;
  lm_clear(acc);
  // MFMAs first .. last - 1 (of 8) of one half-step
  auto mfma_range = [&](const bf16x8 (&a)[4], const bf16x8 (&b)[2], int first, int last) {
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j)
        if (2 * i + j >= first && 2 * i + j < last)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
  };
  LmSoftmax sm;
  LmGrad gr;
  if (GRAD) gr.init(it, rows, vocab, token_ids, ga);
  else sm.init(it, rows, vocab, token_ids);
  auto tile_done = [&](int tile) {
    if (GRAD) gr.emit(acc, it, tile, vocab, scale, ga);
    else sm.fold(acc, it, tile, vocab, scale, zy_out);
  };

  // Every wavefront issues 4 copies per step and they complete in order: waiting until at most 4 * younger
  // are outstanding means the step before the `younger` most recent ones has landed.
  static_assert(NS >= 3 && NS <= 5, "the waits below are written for 3 to 5 stages");
  auto wait_all_but = [](auto younger) {
    constexpr int Y = decltype(younger)::value;
    if (Y == 3) asm volatile("s_waitcnt vmcnt(12)" ::: "memory");
    else if (Y == 2) asm volatile("s_waitcnt vmcnt(8)" ::: "memory");
    else if (Y == 1) asm volatile("s_waitcnt vmcnt(4)" ::: "memory");
    else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  };
#define AIS_PIN __builtin_amdgcn_sched_barrier(0)
  bf16x8 a0[4], b0[2], a1[4], b1[2];
  int vt = it.vt0, kt = 0;
  // First part of a step: the eight MFMAs of its first 16 elements, one read of the second 16 elements'
  // fragments in the shadow of each; then the first two MFMAs of the second half, which give the matrix cores
  // work while the wavefronts gather at the barrier.  The barrier publishes the next step (every wavefront
  // has waited for its own copies of it) and retires the previous one.
  // Which fragment reads follow MFMA q of a half-step: two after each of the first two, one after the next two,
  // so that the last read is four MFMAs old when the next half-step begins.
  auto reads_after = [&](int q, int step, int kk, bf16x8 (&a)[4], bf16x8 (&b)[2]) {
    if (q == 0) { read_frag(step, kk, 0, a, b); read_frag(step, kk, 1, a, b); }
    if (q == 1) { read_frag(step, kk, 2, a, b); read_frag(step, kk, 3, a, b); }
    if (q == 2) read_frag(step, kk, 4, a, b);
    if (q == 3) read_frag(step, kk, 5, a, b);
  };
  auto first_part = [&](int s) {
#pragma unroll
    for (int q = 0; q < 8; ++q) {
      mfma_range(a0, b0, q, q + 1);
      AIS_PIN;
      reads_after(q, s, 1, a1, b1);
      AIS_PIN;
    }
    mfma_range(a1, b1, 0, 2);
    AIS_PIN;
    // Outstanding copies, oldest first: step s + 1, then NS - 3 younger steps.  Wait for the former, then meet.
    // Written as one opaque instruction pair: a workgroup-scope fence here would make the compiler wait for
    // every outstanding copy, which is exactly what the extra stages are there to avoid.  The LDS reads issued
    // above need not be complete at the barrier: the stage they read is not overwritten before the next one.
    if (NS - 3 == 2) asm volatile("s_waitcnt vmcnt(8)\n\ts_barrier" ::: "memory");
    else if (NS - 3 == 1) asm volatile("s_waitcnt vmcnt(4)\n\ts_barrier" ::: "memory");
    else asm volatile("s_waitcnt vmcnt(0)\n\ts_barrier" ::: "memory");
    AIS_PIN;
  };

  // ---- prologue: NS - 1 steps in flight, step 0 published
#pragma unroll
  for (int st = 0; st < NS - 1; ++st)
#pragma unroll
    for (int q = 0; q < 4; ++q) copy_part(st, q);
  wait_all_but(std::integral_constant<int, NS - 2>{});
  __syncthreads();
  read_frags(0, 0, a0, b0);
  first_part(0);
  // ---- steady state: the rest of step s, with the reads of step s + 1 and the copies of step s + NS - 1 (into
  // the stage step s - 1 has left) in the shadows, then the first part of step s + 1
  for (int s = 0; s + 1 < n_steps; ++s) {
    const int stage = (s + NS - 1) % NS;
#pragma unroll
    for (int q = 2; q < 8; ++q) {
      mfma_range(a1, b1, q, q + 1);
      AIS_PIN;
      reads_after(q - 2, s + 1, 0, a0, b0);
      AIS_PIN;
      if (q >= 4) copy_part(stage, q - 4);
      AIS_PIN;
    }
    if (++kt == n_ksteps) {
      tile_done(vt);
      lm_clear(acc);
      kt = 0;
      ++vt;
    }
    first_part(s + 1);
  }
#undef AIS_PIN
  mfma_range(a1, b1, 2, 8);
  tile_done(vt);
  // copies of the last steps may still be in flight, and they land in LDS that finish() is about to reuse
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  if (!GRAD) sm.finish(it, reinterpret_cast<float*>(lds), n_rows, part_m, part_s);
}

// ---- streaming kernel with 64-element steps: d_model a multiple of 64 -------------------------------------------
// The same arithmetic on slices of 64 elements of d_model: a row of a slice is then a whole 128-byte line, so a copy
// instruction of a wavefront asks L2 for 8 full lines instead of 16 half lines (half the requests for the same
// bytes).  Two buffers of 64 KiB (W slice, H slice, 128-byte rows, chunks swizzled as in lds_chunk_offset below).  A
// step has four sub-steps of 16 elements; the fragments of a sub-step are read during the one before it.  One
// barrier per step, after the second MFMA of its last sub-step: every wavefront has then issued all its reads of
// the step's buffer and has waited for its own copies of the next step, so the barrier publishes the next step and
// frees the buffer; the copies of the step after next go into it at once (four in the rest of this step, four in the
// first sub-step of the next), a whole step before they are awaited.
constexpr int kS64K = 64;
constexpr int kS64OperandBytes = kLmTileV * kS64K * 2;           // 32 KiB
constexpr int kS64BufferBytes = 2 * kS64OperandBytes;            // 64 KiB
constexpr int kS64LdsBytes = 2 * kS64BufferBytes;                // 128 KiB

__device__ __forceinline__ int s64_chunk_offset(int row, int c) { return row * 128 + ((c ^ ((row >> 1) & 7)) << 4); }

template <bool GRAD>
__global__ __launch_bounds__(kLmThreads) void lm_head_stream64_kernel(
    const bf16_t* __restrict__ hidden, long long ld_h, const bf16_t* __restrict__ weight, long long ld_w,
    LmRows rows, const LmDevPlan* __restrict__ plan, int d_model, int vocab, const int* __restrict__ token_ids,
    float scale, int n_vtiles, float* __restrict__ part_m, float* __restrict__ part_s,
    float* __restrict__ zy_out, LmGradArgs ga) {
  extern __shared__ __align__(16) unsigned char lds[];
  LmItem it;
  if (!it.init(plan, n_vtiles)) return;
  const int n_rows = rows.n_rows;
  const int lane = it.lane, wave = it.wave;

  // ---- copies: wavefront w moves rows 8 w .. 8 w + 7 (+ 64 j, j = 0..3) of each slice; a lane sits at chunk
  // position lane & 7 of row lane >> 3 and therefore fetches logical chunk (lane & 7) ^ ((row >> 1) & 7), which is
  // the same for the four rows 64 apart
  const int crow = 8 * wave + (lane >> 3);
  const int cchunk = (lane & 7) ^ ((crow >> 1) & 7);
  const bf16_t* hp[4];
  const bf16_t* wp[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int trow = rows.row(it.t0 + crow + 64 * j, it.n_eval);
    hp[j] = hidden + (long long)trow * ld_h + cchunk * 8;
  }
  auto point_w = [&](int vt) {
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int vrow = min(vt * kLmTileV + crow + 64 * j, vocab - 1);
      wp[j] = weight + (long long)vrow * ld_w + cchunk * 8;
    }
  };
  const int n_ksteps = d_model / kS64K;
  const int n_steps = (it.vt1 - it.vt0) * n_ksteps;
  // cursor of the step being copied
  int c_step = 0, c_kt = 0, c_vt = it.vt0;
  point_w(c_vt);
  // One of the eight copy instructions (W rows, H rows, then the same 64, 128 and 192 rows further) that bring the
  // cursor's step into buffer `buf`; the eighth advances the cursor.  Once the cursor has reached the last step it
  // stays there: the copies issued after that re-fetch the last step into a buffer nobody reads any more, which
  // keeps the loop free of branches.
  auto copy_part = [&](int buf, int q) {
    unsigned char* base = lds + buf * kS64BufferBytes + (8 * wave + 64 * (q >> 1)) * 128;
    const int k0 = c_kt * kS64K;
    if ((q & 1) == 0)
      __builtin_amdgcn_global_load_lds((glb_ptr)(wp[q >> 1] + k0), (lds_ptr)base, 16, 0, 0);
    else
      __builtin_amdgcn_global_load_lds((glb_ptr)(hp[q >> 1] + k0), (lds_ptr)(base + kS64OperandBytes), 16, 0, 0);
    if (q == 7 && c_step + 1 < n_steps) {
      ++c_step;
      if (++c_kt == n_ksteps) {
        c_kt = 0;
        ++c_vt;
        point_w(c_vt);
      }
    }
  };

  // ---- fragments: lane reads row (32-row tile base + col), chunk 2 kk + half of a 128-byte row
  int frag_off[4];
#pragma unroll
  for (int kk = 0; kk < 4; ++kk) frag_off[kk] = s64_chunk_offset(it.col, 2 * kk + it.half);
  const int a_base = it.wv * kLmWaveV * 128;
  const int b_base = kS64OperandBytes + it.wt * kLmWaveT * 128;
  // One fragment read, in the order the MFMAs need them: a0 b0 b1 a1 a2 a3 (r = 0..5).
  auto read_frag = [&](int step, int kk, int r, bf16x8 (&a)[4], bf16x8 (&b)[2]) {
    const unsigned char* base = lds + (step & 1) * kS64BufferBytes + frag_off[kk];
    if (r == 1 || r == 2)
      b[r - 1] = as_bf16x8(*reinterpret_cast<const u32x4*>(base + b_base + (r - 1) * 4096));
    else {
      const int i = r == 0 ? 0 : r - 2;
      a[i] = as_bf16x8(*reinterpret_cast<const u32x4*>(base + a_base + i * 4096));
    }
  };
  // Which fragment reads follow MFMA q of a sub-step: two after each of the first two, one after the next two.
  auto reads_after = [&](int q, int step, int kk, bf16x8 (&a)[4], bf16x8 (&b)[2]) {
    if (q == 0) { read_frag(step, kk, 0, a, b); read_frag(step, kk, 1, a, b); }
    if (q == 1) { read_frag(step, kk, 2, a, b); read_frag(step, kk, 3, a, b); }
    if (q == 2) read_frag(step, kk, 4, a, b);
    if (q == 3) read_frag(step, kk, 5, a, b);
  };

  LmAcc acc;
  lm_clear(acc);
  auto mfma_one = [&](const bf16x8 (&a)[4], const bf16x8 (&b)[2], int q) {
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j)
        if (2 * i + j == q) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
  };
  LmSoftmax sm;
  LmGrad gr;
  if (GRAD) gr.init(it, rows, vocab, token_ids, ga);
  else sm.init(it, rows, vocab, token_ids);
  auto tile_done = [&](int tile) {
    if (GRAD) gr.emit(acc, it, tile, vocab, scale, ga);
    else sm.fold(acc, it, tile, vocab, scale, zy_out);
  };

#define AIS_PIN __builtin_amdgcn_sched_barrier(0)
  // Copies of the step after next issued in the rest of a step, right after its barrier (the others follow in the
  // first sub-step of the next step), and MFMAs of the last sub-step issued before the barrier.  Measured at 41,643
  // rows x 151,936 x 4,096 on one device: (4, 2) 41.0 ms; (6, 2) 41.1; (0, 2) 42.0; (4, 4) 40.7; (6, 1) 40.7.
  constexpr int kTailCopies = 4;
  constexpr int kPB = 2;
  static_assert(kPB >= 1 && kPB <= 4, "four MFMAs after the barrier carry the reads of the next sub-step");
  static_assert(kTailCopies >= 0 && kTailCopies <= 8 - kPB && (kTailCopies % 2) == 0, "one copy per MFMA of the tail");
  bf16x8 a0[4], b0[2], a1[4], b1[2];
  int vt = it.vt0, kt = 0;
  // ---- prologue: step 0 and the first half of step 1's copies in flight, step 0 published
#pragma unroll
  for (int q = 0; q < 8; ++q) copy_part(0, q);
#pragma unroll
  for (int q = 0; q < kTailCopies; ++q) copy_part(1, q);
  // copies complete in order: step 0 has landed
  if (kTailCopies == 6) asm volatile("s_waitcnt vmcnt(6)" ::: "memory");
  else if (kTailCopies == 4) asm volatile("s_waitcnt vmcnt(4)" ::: "memory");
  else if (kTailCopies == 2) asm volatile("s_waitcnt vmcnt(2)" ::: "memory");
  else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();
#pragma unroll
  for (int r = 0; r < 6; ++r) read_frag(0, 0, r, a0, b0);
  for (int s = 0; s < n_steps; ++s) {
    // sub-step 0, with the second half of the next step's copies
#pragma unroll
    for (int q = 0; q < 8; ++q) {
      mfma_one(a0, b0, q);
      AIS_PIN;
      reads_after(q, s, 1, a1, b1);
      AIS_PIN;
      if (q < 8 - kTailCopies) copy_part((s + 1) & 1, kTailCopies + q);
      AIS_PIN;
    }
#pragma unroll
    for (int q = 0; q < 8; ++q) {
      mfma_one(a1, b1, q);
      AIS_PIN;
      reads_after(q, s, 2, a0, b0);
      AIS_PIN;
    }
#pragma unroll
    for (int q = 0; q < 8; ++q) {
      mfma_one(a0, b0, q);
      AIS_PIN;
      reads_after(q, s, 3, a1, b1);
      AIS_PIN;
    }
    // last sub-step: two MFMAs give the matrix cores work while the wavefronts gather; then this wavefront's copies
    // of step s + 1 must have landed (all of them: nothing younger is in flight) and everyone meets.  Written as one
    // opaque instruction pair, like the barrier of the 32-element kernel.
#pragma unroll
    for (int q = 0; q < kPB; ++q) mfma_one(a1, b1, q);
    AIS_PIN;
    asm volatile("s_waitcnt vmcnt(0)\n\ts_barrier" ::: "memory");
    AIS_PIN;
#pragma unroll
    for (int q = kPB; q < 8; ++q) {
      mfma_one(a1, b1, q);
      AIS_PIN;
      reads_after(q - kPB, s + 1, 0, a0, b0);
      AIS_PIN;
      if (q >= 8 - kTailCopies) copy_part(s & 1, q - (8 - kTailCopies));
      AIS_PIN;
    }
    if (++kt == n_ksteps) {
      tile_done(vt);
      lm_clear(acc);
      kt = 0;
      ++vt;
    }
  }
#undef AIS_PIN
  // copies of the last steps may still be in flight, and they land in LDS that finish() is about to reuse
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  if (!GRAD) sm.finish(it, reinterpret_cast<float*>(lds), n_rows, part_m, part_s);
}

// ---- register-staged kernel: any d_model that is a multiple of 8 ---------------------------------------------
// Steps of 64 elements; the last step's chunks past the end of d_model must become zeros, so the slices are
// loaded into registers before the arithmetic of a step and written to the other of two LDS buffers in the
// middle of it.
constexpr int kLmOperandBytes = kLmTileV * kLmTileK * 2;            // 32 KiB: one operand slice
constexpr int kLmStageBytes = 2 * kLmOperandBytes;                   // W slice then H slice
constexpr int kLmLdsBytes = 2 * kLmStageBytes;                       // double buffer: 128 KiB

// Byte offset of 16-byte chunk `c` (0..7) of row `row` inside one operand slice.  A row is 128 bytes; the
// chunk index is XORed with bits 1..3 of the row so that 16 consecutive rows read at the same logical
// chunk touch 16 different 16-byte bank groups.
__device__ __forceinline__ int lds_chunk_offset(int row, int c) { return row * 128 + ((c ^ ((row >> 1) & 7)) << 4); }

__global__ __launch_bounds__(kLmThreads) void lm_head_staged_kernel(
    const bf16_t* __restrict__ hidden, long long ld_h, const bf16_t* __restrict__ weight, long long ld_w,
    LmRows rows, const LmDevPlan* __restrict__ plan, int d_model, int vocab, const int* __restrict__ token_ids,
    float scale, int n_vtiles, float* __restrict__ part_m, float* __restrict__ part_s,
    float* __restrict__ zy_out) {
  extern __shared__ __align__(16) unsigned char lds[];
  LmItem it;
  if (!it.init(plan, n_vtiles)) return;
  const int n_rows = rows.n_rows;
  const int tid = threadIdx.x;

  // ---- global -> registers -> LDS: thread owns chunk c of rows r0 + 64 i of both operand slices
  const int c = tid & 7, r0 = tid >> 3;
  const bf16_t* hp[4];
  const bf16_t* wp[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int trow = rows.row(it.t0 + r0 + 64 * i, it.n_eval);
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
  auto fetch = [&](int k0) {
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
  for (int kk = 0; kk < 4; ++kk) frag_off[kk] = lds_chunk_offset(it.col, 2 * kk + it.half);
  const int a_base = it.wv * kLmWaveV * 128;                       // W rows of this wavefront
  const int b_base = kLmOperandBytes + it.wt * kLmWaveT * 128;     // H rows of this wavefront

  LmAcc acc;
  lm_clear(acc);
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
  // The 32 MFMAs of one step.  `mid` runs between the second and the third group of eight: the place where
  // the next step's slices are written to the other LDS buffer, so that neither the load latency nor the LDS
  // writes stall the matrix cores.
  auto multiply = [&](int buf, auto&& mid) {
    const unsigned char* base = lds + buf * kLmStageBytes;
    bf16x8 a[2][4], b[2][2];
    read_frags(base, 0, a[0], b[0]);
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
      if (kk < 3) read_frags(base, kk + 1, a[(kk + 1) & 1], b[(kk + 1) & 1]);
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[kk & 1][i], b[kk & 1][j], acc[i][j], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
      if (kk == 1) {
        mid();
        __builtin_amdgcn_sched_barrier(0);
      }
    }
  };

  LmSoftmax sm;
  sm.init(it, rows, vocab, token_ids);

  // ---- main loop over (vocabulary tile, d_model step), flattened so that the prefetch crosses tiles
  const int n_ksteps = (d_model + kLmTileK - 1) / kLmTileK;
  int vt = it.vt0, kt = 0, buf = 0;
  point_w(vt);
  fetch(0);
  stage(0);
  __syncthreads();
  for (;;) {
    int nkt = kt + 1, nvt = vt;
    if (nkt == n_ksteps) { nkt = 0; nvt = vt + 1; }
    const bool more = nvt < it.vt1;
    if (more) {
      if (nkt == 0) point_w(nvt);
      fetch(nkt * kLmTileK);
    }
    multiply(buf, [&]() { if (more) stage(buf ^ 1); });
    if (kt == n_ksteps - 1) {
      sm.fold(acc, it, vt, vocab, scale, zy_out);
      lm_clear(acc);
    }
    if (!more) break;
    // one barrier per step: the other buffer is complete, and everyone has finished reading this one
    // before the next step's `mid` overwrites it
    __syncthreads();
    kt = nkt;
    vt = nvt;
    buf ^= 1;
  }
  sm.finish(it, reinterpret_cast<float*>(lds), n_rows, part_m, part_s);
}

// One workgroup, before the main kernel.  With a mask it lists the rows to evaluate (index[p] = p-th row with
// valid != 0, pos[n] = position of row n in that list or -1; each thread owns a contiguous run of rows); in
// both cases thread 0 then decides the decomposition for the number of evaluated rows.
// n_cap >= 0: the list holds at most n_cap rows; further rows are dropped (pos = -1) and reported in *status.
__global__ __launch_bounds__(1024) void lm_head_setup_kernel(const unsigned char* __restrict__ valid, int n_rows,
                                                             int n_vtiles, int n_cus, int max_items, int tb_group,
                                                             int* __restrict__ index, int* __restrict__ pos,
                                                             LmDevPlan* __restrict__ plan, int n_cap = -1,
                                                             int* __restrict__ status = nullptr) {
  __shared__ int run_start[1024];
  __shared__ int total;
  const int tid = threadIdx.x;
  if (valid != nullptr) {
    const int per = (n_rows + 1023) / 1024;
    const int r0 = min(n_rows, tid * per), r1 = min(n_rows, r0 + per);
    int cnt = 0;
    for (int n = r0; n < r1; ++n) cnt += valid[n] != 0;
    run_start[tid] = cnt;
    __syncthreads();
    if (tid == 0) {
      int run = 0;
      for (int t = 0; t < 1024; ++t) {
        const int c = run_start[t];
        run_start[t] = run;
        run += c;
      }
      total = run;
    }
    __syncthreads();
    const int cap = n_cap >= 0 ? n_cap : n_rows;
    int p = run_start[tid];
    for (int n = r0; n < r1; ++n) {
      if (valid[n] != 0) {
        if (p < cap) {
          index[p] = n;
          pos[n] = p;
        } else {
          pos[n] = -1;
        }
        ++p;
      } else {
        pos[n] = -1;
      }
    }
    if (tid == 0 && total > cap) {
      total = cap;
      if (status != nullptr) atomicOr(status, AIS_STATUS_LIVE_OVERFLOW);
    }
    // (total is read below by thread 0 only)
  } else if (tid == 0) {
    total = n_rows;
  }
  if (tid == 0) {
    LmDevPlan d;
    d.n_eval = total;
    d.n_tblocks = (total + kLmTileT - 1) / kLmTileT;
    lm_choose_chunks(d.n_tblocks, n_vtiles, n_cus, max_items, &d.n_chunks, &d.tiles_per_chunk);
    d.n_items = d.n_tblocks * d.n_chunks;
    d.per_xcd = (d.n_items + 7) / 8;
    d.tb_group = max(1, min(tb_group, d.n_tblocks));
    *plan = d;
  }
}

// lse and log-prob from the per-chunk partials.  One thread per row; partials are stored by evaluated position.
__global__ __launch_bounds__(256) void lm_head_merge_kernel(const float* __restrict__ part_m,
                                                            const float* __restrict__ part_s,
                                                            const float* __restrict__ zy, int n_rows,
                                                            const LmDevPlan* __restrict__ plan, int vocab,
                                                            const int* __restrict__ token_ids,
                                                            const int* __restrict__ pos,
                                                            float inv_temperature, float* __restrict__ logp_out,
                                                            float* __restrict__ lse_out, int* __restrict__ status) {
  const int n = blockIdx.x * 256 + threadIdx.x;
  if (n >= n_rows) return;
  const int n_chunks = plan->n_chunks;
  const int p = pos != nullptr ? pos[n] : n;
  if (p < 0) {
    logp_out[n] = 0.f;
    lse_out[n] = 0.f;
    return;
  }
  float m = kNegHuge;
  for (int k = 0; k < n_chunks; ++k) m = fmaxf(m, part_m[(long long)k * n_rows + p]);
  double s = 0.0;
  for (int k = 0; k < n_chunks; ++k)
    s += (double)part_s[(long long)k * n_rows + p] * (double)exp2_fast(part_m[(long long)k * n_rows + p] - m);
  const double lse = ((double)m + log2(s)) * 0.6931471805599453;
  lse_out[n] = (float)lse;
  const int id = token_ids[n];
  if (id >= 0 && id < vocab) {
    logp_out[n] = (float)((double)zy[p] * (double)inv_temperature - lse);
  } else {
    logp_out[n] = 0.f;
    atomicOr(status, AIS_STATUS_BAD_TOKEN);
  }
}

// ---- rows that take part in the gradient call, gathered ------------------------------------------------------
__global__ __launch_bounds__(256) void lm_live_mask_kernel(const float* __restrict__ coeff, int n_rows,
                                                           unsigned char* __restrict__ mask) {
  const int n = blockIdx.x * 256 + threadIdx.x;
  if (n < n_rows) mask[n] = coeff[n] != 0.f;
}

// out[p, :] = hidden[index[p], :] for the listed rows, zeros for p in [n_eval, n_cap).  One workgroup per row.
__global__ __launch_bounds__(256) void lm_gather_rows_kernel(const bf16_t* __restrict__ hidden, long long ld_h,
                                                             const int* __restrict__ index,
                                                             const LmDevPlan* __restrict__ plan, int d_model,
                                                             bf16_t* __restrict__ out) {
  const int p = blockIdx.x;
  const bool live = p < plan->n_eval;
  const u32x4* src = reinterpret_cast<const u32x4*>(hidden + (live ? (long long)index[p] * ld_h : 0));
  u32x4* dst = reinterpret_cast<u32x4*>(out + (long long)p * d_model);
  const u32x4 zero = {0u, 0u, 0u, 0u};
  for (int c = threadIdx.x; c < d_model / 8; c += 256) dst[c] = live ? src[c] : zero;
}

// Rows [n_eval, n_cap) of a chunk of dlogits are nobody's: zeros, so that the two GEMMs can run over n_cap rows.
__global__ __launch_bounds__(256) void lm_zero_tail_rows_kernel(bf16_t* __restrict__ ds, long long ds_stride,
                                                                int width, const LmDevPlan* __restrict__ plan) {
  const int p = plan->n_eval + blockIdx.x;                      // the grid covers n_cap rows; only the tail works
  if (p >= (int)gridDim.x) return;
  bf16_t* row = ds + (long long)p * ds_stride;
  for (int v = threadIdx.x; v < width; v += 256) row[v] = 0;
}

// dhidden[n, :] = gathered[pos[n], :] for the listed rows, zeros for the others.  One workgroup per row.
__global__ __launch_bounds__(256) void lm_scatter_rows_kernel(const float* __restrict__ gathered,
                                                              const int* __restrict__ pos, int d_model,
                                                              float* __restrict__ out) {
  const int n = blockIdx.x;
  const int p = pos[n];
  const float4* src = reinterpret_cast<const float4*>(gathered + (long long)(p < 0 ? 0 : p) * d_model);
  float4* dst = reinterpret_cast<float4*>(out + (long long)n * d_model);
  for (int c = threadIdx.x; c < d_model / 4; c += 256) dst[c] = p < 0 ? make_float4(0.f, 0.f, 0.f, 0.f) : src[c];
}

}  // namespace

// Worst case of the decomposition (every row evaluated): sizes the grid and the workspace.
LmHeadPlan lm_head_plan(long long n_rows, int vocab, int n_cus) {
  LmHeadPlan p;
  p.n_tblocks = (int)((n_rows + kLmTileT - 1) / kLmTileT);
  p.n_vtiles = (vocab + kLmTileV - 1) / kLmTileV;
  lm_choose_chunks(p.n_tblocks, p.n_vtiles, n_cus, 1LL << 40, &p.n_chunks, &p.tiles_per_chunk);
  p.max_chunks = p.n_vtiles < 64 ? p.n_vtiles : 64;
  return p;
}

#ifndef AIS_LM_STAGES
#define AIS_LM_STAGES 4
#endif

int launch_lm_head_logprob(ais_ctx* ctx, const void* hidden, long long ld_h, const void* weight, long long ld_w,
                           long long n_rows, int d_model, int vocab, const int* token_ids,
                           const unsigned char* valid, float inv_temperature, const LmHeadPlan& plan,
                           float* part_m, float* part_s, float* zy, int* row_index, int* row_pos, void* dev_plan,
                           float* logp_out, float* lse_out) {
  constexpr int kStreamLds = AIS_LM_STAGES * kStStageBytes;
  static std::once_flag once_stream[kMaxDevices], once_s64[kMaxDevices], once_staged[kMaxDevices];   // per function and device
  static bool ok_stream[kMaxDevices], ok_s64[kMaxDevices], ok_staged[kMaxDevices];
  if (!allow_dynamic_lds(ctx, reinterpret_cast<const void*>(lm_head_stream_kernel<AIS_LM_STAGES, false>), kStreamLds,
                         once_stream, ok_stream) ||
      !allow_dynamic_lds(ctx, reinterpret_cast<const void*>(lm_head_stream64_kernel<false>), kS64LdsBytes, once_s64,
                         ok_s64) ||
      !allow_dynamic_lds(ctx, reinterpret_cast<const void*>(lm_head_staged_kernel), kLmLdsBytes, once_staged,
                         ok_staged))
    return hip_fail(ctx, hipErrorInvalidValue);
  // The grid covers the work items of the worst case; with fewer evaluated rows the device-side plan may use
  // more, shorter chunks, but never more items than that, and the workgroups left over leave at once.
  const int max_items = ((plan.n_tblocks * plan.n_chunks + 7) / 8) * 8;
  LmDevPlan* dplan = static_cast<LmDevPlan*>(dev_plan);
  lm_head_setup_kernel<<<1, 1024, 0, ctx->stream>>>(valid, (int)n_rows, plan.n_vtiles, ctx->n_cus, max_items,
                                                    kLmTokenBlockGroup, row_index, row_pos, dplan);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return hip_fail(ctx, e);
  LmRows rows{valid != nullptr ? row_index : nullptr, (int)n_rows};
  {
    ScopedTimer timer(ctx, AIS_K_LM_HEAD);
    if (d_model % kS64K == 0)
      lm_head_stream64_kernel<false><<<max_items, kLmThreads, kS64LdsBytes, ctx->stream>>>(
          static_cast<const bf16_t*>(hidden), ld_h, static_cast<const bf16_t*>(weight), ld_w, rows, dplan, d_model,
          vocab, token_ids, inv_temperature * kLog2e, plan.n_vtiles, part_m, part_s, zy, LmGradArgs{});
    else if (d_model % kStK == 0)
      lm_head_stream_kernel<AIS_LM_STAGES, false><<<max_items, kLmThreads, kStreamLds, ctx->stream>>>(
          static_cast<const bf16_t*>(hidden), ld_h, static_cast<const bf16_t*>(weight), ld_w, rows, dplan, d_model,
          vocab, token_ids, inv_temperature * kLog2e, plan.n_vtiles, part_m, part_s, zy, LmGradArgs{});
    else
      lm_head_staged_kernel<<<max_items, kLmThreads, kLmLdsBytes, ctx->stream>>>(
          static_cast<const bf16_t*>(hidden), ld_h, static_cast<const bf16_t*>(weight), ld_w, rows, dplan, d_model,
          vocab, token_ids, inv_temperature * kLog2e, plan.n_vtiles, part_m, part_s, zy);
  }
  e = hipGetLastError();
  if (e != hipSuccess) return hip_fail(ctx, e);
  lm_head_merge_kernel<<<(unsigned)((n_rows + 255) / 256), 256, 0, ctx->stream>>>(
      part_m, part_s, zy, (int)n_rows, dplan, vocab, token_ids, valid != nullptr ? row_pos : nullptr,
      inv_temperature, logp_out, lse_out, ctx->status_dev);
  return hip_fail(ctx, hipGetLastError());
}

// dlogits of one chunk of the vocabulary, from hidden states and the chunk's rows of the output embedding, into
// ds[n_rows, ds_stride] (bf16).  `weight` points at the chunk's first row, `vocab` is the chunk's width, `y_off` its
// first vocabulary entry.  Every row is processed (rows whose coefficient is 0 come out as zeros).
// With a list (live_mask != nullptr: the rows with a gradient, at most n_cap of them) row p of ds belongs to the p-th
// listed row and rows up to n_cap - 1 are written (zeros past the end of the list).
int launch_lm_head_dlogits_chunk(ais_ctx* ctx, const void* hidden, long long ld_h, const void* weight,
                                 long long ld_w, long long n_rows, int d_model, int vocab, int y_off,
                                 const int* token_ids, const float* lse, const float* logp, const float* coeff,
                                 float inv_temperature, void* dev_plan, void* ds, long long ds_stride,
                                 const unsigned char* live_mask, int* row_index, int* row_pos, int n_cap) {
  constexpr int kStreamLds = AIS_LM_STAGES * kStStageBytes;
  static std::once_flag once[kMaxDevices], once64[kMaxDevices];
  static bool ok[kMaxDevices], ok64[kMaxDevices];
  if (!allow_dynamic_lds(ctx, reinterpret_cast<const void*>(lm_head_stream_kernel<AIS_LM_STAGES, true>), kStreamLds,
                         once, ok) ||
      !allow_dynamic_lds(ctx, reinterpret_cast<const void*>(lm_head_stream64_kernel<true>), kS64LdsBytes, once64, ok64))
    return hip_fail(ctx, hipErrorInvalidValue);
  const LmHeadPlan plan = lm_head_plan(n_rows, vocab, ctx->n_cus);
  const int max_items = ((plan.n_tblocks * plan.n_chunks + 7) / 8) * 8;
  LmDevPlan* dplan = static_cast<LmDevPlan*>(dev_plan);
  lm_head_setup_kernel<<<1, 1024, 0, ctx->stream>>>(live_mask, (int)n_rows, plan.n_vtiles, ctx->n_cus, max_items,
                                                    kLmTokenBlockGroup, row_index, row_pos, dplan,
                                                    live_mask != nullptr ? n_cap : -1, ctx->status_dev);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return hip_fail(ctx, e);
  LmRows rows{live_mask != nullptr ? row_index : nullptr, (int)n_rows};
  LmGradArgs ga{lse, logp, coeff, static_cast<bf16_t*>(ds), ds_stride, y_off, live_mask != nullptr ? 1 : 0};
  {
    ScopedTimer timer(ctx, AIS_K_LM_HEAD_GRAD);
    if (d_model % kS64K == 0)
      lm_head_stream64_kernel<true><<<max_items, kLmThreads, kS64LdsBytes, ctx->stream>>>(
          static_cast<const bf16_t*>(hidden), ld_h, static_cast<const bf16_t*>(weight), ld_w, rows, dplan, d_model,
          vocab, token_ids, inv_temperature * kLog2e, plan.n_vtiles, nullptr, nullptr, nullptr, ga);
    else
      lm_head_stream_kernel<AIS_LM_STAGES, true><<<max_items, kLmThreads, kStreamLds, ctx->stream>>>(
          static_cast<const bf16_t*>(hidden), ld_h, static_cast<const bf16_t*>(weight), ld_w, rows, dplan, d_model,
          vocab, token_ids, inv_temperature * kLog2e, plan.n_vtiles, nullptr, nullptr, nullptr, ga);
  }
  e = hipGetLastError();
  if (e != hipSuccess) return hip_fail(ctx, e);
  if (live_mask != nullptr && n_cap > 0)
    lm_zero_tail_rows_kernel<<<(unsigned)n_cap, 256, 0, ctx->stream>>>(static_cast<bf16_t*>(ds), ds_stride, vocab,
                                                                       dplan);
  return hip_fail(ctx, hipGetLastError());
}

int launch_lm_live_mask(ais_ctx* ctx, const float* coeff, long long n_rows, unsigned char* mask) {
  lm_live_mask_kernel<<<(unsigned)((n_rows + 255) / 256), 256, 0, ctx->stream>>>(coeff, (int)n_rows, mask);
  return hip_fail(ctx, hipGetLastError());
}

// The list and the plan for `n_rows` rows with the mask, once (the chunk launches rebuild the plan for their width).
int launch_lm_gather_rows(ais_ctx* ctx, const void* hidden, long long ld_h, long long n_rows, int d_model,
                          const unsigned char* live_mask, int* row_index, int* row_pos, void* dev_plan, int n_cap,
                          void* gathered) {
  LmDevPlan* dplan = static_cast<LmDevPlan*>(dev_plan);
  lm_head_setup_kernel<<<1, 1024, 0, ctx->stream>>>(live_mask, (int)n_rows, 1, ctx->n_cus, 1 << 30,
                                                    kLmTokenBlockGroup, row_index, row_pos, dplan, n_cap,
                                                    ctx->status_dev);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return hip_fail(ctx, e);
  lm_gather_rows_kernel<<<(unsigned)n_cap, 256, 0, ctx->stream>>>(static_cast<const bf16_t*>(hidden), ld_h, row_index,
                                                                  dplan, d_model, static_cast<bf16_t*>(gathered));
  return hip_fail(ctx, hipGetLastError());
}

int launch_lm_scatter_rows(ais_ctx* ctx, const float* gathered, const int* row_pos, long long n_rows, int d_model,
                           float* out) {
  lm_scatter_rows_kernel<<<(unsigned)n_rows, 256, 0, ctx->stream>>>(gathered, row_pos, d_model, out);
  return hip_fail(ctx, hipGetLastError());
}

}  // namespace ais
