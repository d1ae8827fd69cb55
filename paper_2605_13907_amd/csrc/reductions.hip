// Per-row scalar work and the batch-wide reductions of the path.
//
// The batch is a set of variable-length segments (responses) of rows, some rows masked out.  A small
// plan kernel cuts every response into tiles of kTileRows rows; level 1 reduces one tile per workgroup
// (lane shuffles, then one exchange through LDS) to a partial; level 2, run by whichever workgroup of the
// same launch finishes last, folds the partials of each response in order, forms the group-relative
// advantages (Eq. 3) and the batch moments, and evaluates the three diagnostics and the mixing coefficient
// (Eq. 12-17).  Everything is accumulated in fp64 in a fixed order (no floating point atomics), so results
// are bit-reproducible from run to run; spreads are carried as pairwise-merged (count, mean, squared
// deviations) triples, never as differences of power sums.  These kernels move a few bytes per row (about a
// megabyte per batch) and are latency-bound; the time of the path is in the two sweeps.
#include "ais_internal.h"

namespace ais {
namespace {

__device__ __forceinline__ long long clampll(long long v, long long lo, long long hi) {
  return v < lo ? lo : (v > hi ? hi : v);
}

// Row range of response i, forced into [0, n_rows] and non-negative length whatever cu_rows holds.
__device__ __forceinline__ void response_rows(const long long* cu_rows, int i, long long n_rows, long long& lo,
                                              long long& hi) {
  lo = clampll(cu_rows[i], 0, n_rows);
  hi = clampll(cu_rows[i + 1], lo, n_rows);
}

// ---- plan: tile_off[i] = first tile of response i, tile_off[n_resp] = number of tiles -------------------
// One workgroup.  Each thread owns a contiguous chunk of responses; thread 0 scans the 256 chunk totals.
__global__ __launch_bounds__(kTileThreads) void plan_kernel(const long long* __restrict__ cu_rows, int n_resp,
                                                            long long n_rows, int* __restrict__ tile_off,
                                                            int max_tiles, int* __restrict__ status,
                                                            int* __restrict__ ticket) {
  __shared__ long long chunk_sum[kTileThreads];
  const int tid = threadIdx.x;
  if (tid == 0) *ticket = 0;         // counts the finished workgroups of each reduction kernel that follows
  const int per = (n_resp + kTileThreads - 1) / kTileThreads;
  const int i0 = min(n_resp, tid * per), i1 = min(n_resp, i0 + per);
  long long sum = 0;
  bool bad = false;
  for (int i = i0; i < i1; ++i) {
    long long lo, hi;
    response_rows(cu_rows, i, n_rows, lo, hi);
    bad |= (cu_rows[i] != lo) || (cu_rows[i + 1] != hi);
    sum += (hi - lo + kTileRows - 1) / kTileRows;
  }
  if (tid == 0 && n_resp > 0) bad |= (cu_rows[0] != 0) || (cu_rows[n_resp] != n_rows);
  chunk_sum[tid] = sum;
  __syncthreads();
  if (tid == 0) {
    long long run = 0;
    for (int t = 0; t < kTileThreads; ++t) {
      long long s = chunk_sum[t];
      chunk_sum[t] = run;
      run += s;
    }
    if (run > max_tiles) bad = true;             // cannot happen when cu_rows is a partition of the rows
    tile_off[n_resp] = (int)clampll(run, 0, max_tiles);
  }
  __syncthreads();
  long long run = chunk_sum[tid];
  for (int i = i0; i < i1; ++i) {
    long long lo, hi;
    response_rows(cu_rows, i, n_rows, lo, hi);
    tile_off[i] = (int)clampll(run, 0, max_tiles);
    run += (hi - lo + kTileRows - 1) / kTileRows;
  }
  if (bad) atomicOr(status, AIS_STATUS_BAD_CU);
}

// Response that owns tile b: the last i with tile_off[i] <= b.
__device__ __forceinline__ int find_response(const int* __restrict__ tile_off, int n_resp, int b) {
  int lo = 0, hi = n_resp;          // invariant: tile_off[lo] <= b < tile_off[hi]
  while (hi - lo > 1) {
    int mid = (lo + hi) >> 1;
    if (tile_off[mid] <= b) lo = mid; else hi = mid;
  }
  return lo;
}

constexpr int kWaves = kTileThreads / 64;

// Sum over a wavefront by lane shuffles, in a fixed tree order; lane 0 holds the result.  No barrier is involved:
// these kernels are latency-bound and a workgroup barrier per tree level was most of their time.
template <typename V>
__device__ __forceinline__ V wave_sum(V v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_down(v, off);
  return v;
}

// Workgroup-wide sum: wavefront sums, then the kWaves partials through LDS in index order.  `lds` holds kWaves
// values; the result is valid in every thread.  Must be called by all threads of the workgroup.
template <typename V>
__device__ __forceinline__ V block_sum(V v, V* lds) {
  v = wave_sum(v);
  if ((threadIdx.x & 63) == 0) lds[threadIdx.x >> 6] = v;
  __syncthreads();
  V r = lds[0];
#pragma unroll
  for (int w = 1; w < kWaves; ++w) r += lds[w];
  __syncthreads();
  return r;
}

// Count, mean and sum of squared deviations from the mean of a set of values.  Sets are merged pairwise (the
// update of Chan, Golub and LeVeque): the error of the spread scales with the spread itself, not with the mean, and
// a set of equal values has spread exactly 0 however it was split.
struct Moments {
  double n, mean, m2;
};

__device__ __forceinline__ Moments merge(const Moments& a, const Moments& b) {
  if (b.n == 0.0) return a;
  if (a.n == 0.0) return b;
  const double n = a.n + b.n, delta = b.mean - a.mean;
  Moments r;
  r.n = n;
  r.mean = a.mean + delta * (b.n / n);
  r.m2 = a.m2 + b.m2 + delta * delta * (a.n * b.n / n);
  return r;
}

__device__ __forceinline__ void push(Moments& m, double x) {
  m.n += 1.0;
  const double delta = x - m.mean;
  m.mean += delta / m.n;
  m.m2 += delta * (x - m.mean);
}

__device__ __forceinline__ Moments wave_merge(Moments m) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) {
    const Moments o{__shfl_down(m.n, off), __shfl_down(m.mean, off), __shfl_down(m.m2, off)};
    m = merge(m, o);       // lanes whose partner is beyond the wavefront merge rubbish; lane 0 never depends on them
  }
  return m;
}

// One workgroup-wide reduction of everything a level of the diagnostics needs, with a single barrier pair: NM sets
// of moments, ND plain sums and NI integer sums.  `lds_d` holds (3 NM + ND) kWaves doubles, `lds_i` NI kWaves
// integers.  Results replace the arguments and are valid in every thread.  Must be called by all threads.
template <int NM, int ND, int NI>
__device__ __forceinline__ void block_reduce(Moments (&m)[NM], double (&d)[ND], long long (&c)[NI], double* lds_d,
                                             long long* lds_i) {
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
#pragma unroll
  for (int k = 0; k < NM; ++k) m[k] = wave_merge(m[k]);
#pragma unroll
  for (int k = 0; k < ND; ++k) d[k] = wave_sum(d[k]);
#pragma unroll
  for (int k = 0; k < NI; ++k) c[k] = wave_sum(c[k]);
  if (lane == 0) {
#pragma unroll
    for (int k = 0; k < NM; ++k) {
      lds_d[(3 * k + 0) * kWaves + w] = m[k].n;
      lds_d[(3 * k + 1) * kWaves + w] = m[k].mean;
      lds_d[(3 * k + 2) * kWaves + w] = m[k].m2;
    }
#pragma unroll
    for (int k = 0; k < ND; ++k) lds_d[(3 * NM + k) * kWaves + w] = d[k];
#pragma unroll
    for (int k = 0; k < NI; ++k) lds_i[k * kWaves + w] = c[k];
  }
  __syncthreads();
#pragma unroll
  for (int k = 0; k < NM; ++k) {
    Moments r{lds_d[(3 * k + 0) * kWaves], lds_d[(3 * k + 1) * kWaves], lds_d[(3 * k + 2) * kWaves]};
#pragma unroll
    for (int v = 1; v < kWaves; ++v)
      r = merge(r, Moments{lds_d[(3 * k + 0) * kWaves + v], lds_d[(3 * k + 1) * kWaves + v],
                           lds_d[(3 * k + 2) * kWaves + v]});
    m[k] = r;
  }
#pragma unroll
  for (int k = 0; k < ND; ++k) {
    double r = lds_d[(3 * NM + k) * kWaves];
#pragma unroll
    for (int v = 1; v < kWaves; ++v) r += lds_d[(3 * NM + k) * kWaves + v];
    d[k] = r;
  }
#pragma unroll
  for (int k = 0; k < NI; ++k) {
    long long r = lds_i[k * kWaves];
#pragma unroll
    for (int v = 1; v < kWaves; ++v) r += lds_i[k * kWaves + v];
    c[k] = r;
  }
  __syncthreads();
}

// True in exactly one workgroup of the grid: the one that finishes last.  Every workgroup calls this once,
// after its own results are written; the caller's writes are made visible device-wide before the ticket is
// taken, and the last workgroup sees all of them.  Level 2 of each reduction runs in that workgroup, which
// saves a kernel launch per reduction; the order in which level 2 folds the partials does not depend on which
// workgroup happens to be last, so results stay bit-reproducible.
__device__ __forceinline__ bool last_workgroup(int* ticket) {
  __shared__ int s_last;
  __syncthreads();                           // this workgroup's result has been written by thread 0
  if (threadIdx.x == 0) {
    __threadfence();
    s_last = (atomicAdd(ticket, 1) == (int)gridDim.x - 1);
    if (s_last) *ticket = 0;                 // every other workgroup has taken its ticket: ready for the next launch
  }
  __syncthreads();
  const bool last = s_last != 0;
  if (last) __threadfence();
  return last;
}

// ---- level 2: responses -> advantages, batch moments, diagnostics, alpha --------------------------------------
// Runs in the last workgroup of diag_reduce_kernel.  `partial` is volatile: it was written by other
// workgroups of the same launch and must be read from memory, not from a cache line or register of this one.
__device__ void diag_final(const volatile DiagPartial* partial, const int* __restrict__ tile_off, int n_resp,
                           int group_size, const float* __restrict__ rewards, const ais_params& p,
                           float* __restrict__ adv_out, int* __restrict__ count_out, ais_diag* __restrict__ diag_out,
                           const int* __restrict__ status, double* lds_d, long long* lds_i) {
  Moments mw{0, 0, 0}, ma{0, 0, 0}, maw{0, 0, 0};     // of w_bar, of A and of A w_bar over the valid rows of the batch
  double sabs = 0, sd = 0, sdp = 0;
  long long cnt = 0, nclip = 0;
  for (int i = threadIdx.x; i < n_resp; i += kTileThreads) {
    // fold this response's tiles in order
    Moments r{0, 0, 0};
    long long r_cnt = 0;
    for (int t = tile_off[i]; t < tile_off[i + 1]; ++t) {
      const long long c = partial[t].cnt;
      r = merge(r, Moments{(double)c, partial[t].mean_w, partial[t].m2_w});
      sabs += partial[t].sabs;
      sd += partial[t].sd;
      sdp += partial[t].sdp;
      r_cnt += c;
      nclip += partial[t].nclip;
    }
    // group-relative advantage (Eq. 3): reward minus the mean over the G responses of the prompt
    const int g0 = (i / group_size) * group_size;
    double mean = 0;
    for (int j = 0; j < group_size; ++j) mean += (double)rewards[g0 + j];
    mean /= group_size;
    double a = (double)rewards[i] - mean;
    if (p.adv_mode == 1) {
      double var = 0;
      for (int j = 0; j < group_size; ++j) {
        const double e = (double)rewards[g0 + j] - mean;
        var += e * e;
      }
      const double den = sqrt(var / group_size) + (double)p.eps_std;
      a = den > 0.0 ? a / den : 0.0;     // eps_std = 0 and equal rewards: 0 / 0, read as 0
    }
    const float a32 = (float)a;
    adv_out[i] = a32;
    count_out[i] = (int)r_cnt;
    a = (double)a32;                     // the advantage every later step sees is the stored fp32 value
    // token-level moments of A and A w_bar: A is constant over the response's rows, so the response's rows
    // have mean A mean(w_bar) and squared deviations A^2 m2(w_bar)
    cnt += r_cnt;
    mw = merge(mw, r);
    ma = merge(ma, Moments{r.n, a, 0.0});
    maw = merge(maw, Moments{r.n, a * r.mean, a * a * r.m2});
  }
  {
    Moments m[3] = {mw, ma, maw};
    double d[3] = {sabs, sd, sdp};
    long long c[2] = {cnt, nclip};
    block_reduce(m, d, c, lds_d, lds_i);
    mw = m[0]; ma = m[1]; maw = m[2];
    sabs = d[0]; sd = d[1]; sdp = d[2];
    cnt = c[0]; nclip = c[1];
  }
  if (threadIdx.x != 0) return;

  ais_diag d;
  d.n_valid = cnt;
  d.status = *status;
  d.reserved = 0;
  if (cnt == 0) {
    d.mean_w = d.var_w = d.cv2 = d.dbar = d.std_a = d.std_aw = d.dsigma = 0.0;
    d.ess_ratio = 1.0; d.alpha_ess = 1.0; d.alpha_mis = 0.0; d.alpha_var = 0.0; d.clip_frac = 0.0;
    d.alpha = 0.0; d.kl_roll_train = 0.0; d.mean_abs_dp = 0.0;
  } else {
    const double N = (double)cnt;
    d.mean_w = mw.mean;
    d.var_w = mw.m2 / N;
    // every truncated ratio underflowed to 0: CV^2 is 0 / 0; read as 0 (equal weights), like the empty batch
    const double cv = d.mean_w > 0.0 ? sqrt(d.var_w) / d.mean_w : 0.0;    // std / mean: mean^2 alone may underflow
    d.cv2 = cv * cv;
    d.ess_ratio = 1.0 / (1.0 + d.cv2);
    d.alpha_ess = 1.0 / sqrt(1.0 + d.cv2);                    // Eq. 12
    d.dbar = sabs / N;                                        // Eq. 13
    d.alpha_mis = fmin(1.0, d.dbar / (double)p.delta);        // Eq. 14
    d.std_a = sqrt(ma.m2 / N);
    d.std_aw = sqrt(maw.m2 / N);
    // Eq. 15; with eps_std = 0 and all advantages equal the ratio is 0 / 0: nothing to amplify, read as 0
    const double den = d.std_a + (double)p.eps_std;
    d.dsigma = den > 0.0 ? d.std_aw / den : 0.0;
    d.alpha_var = fmax(0.0, (d.dsigma - (double)p.gamma) / (double)p.gamma);   // Eq. 16
    const double rel = fmin(1.0, fmax(0.0, d.alpha_ess - (double)p.beta_var * d.alpha_var));
    d.alpha = rel * d.alpha_mis;                              // Eq. 17
    d.clip_frac = (double)nclip / N;
    d.kl_roll_train = -sd / N;       // tokens were drawn from pi_roll: mean of log pi_roll - log pi_train
    d.mean_abs_dp = sdp / N;
  }
  if (p.alpha_override >= 0.f) d.alpha = (double)p.alpha_override;
  *diag_out = d;
}

// ---- level 1: one tile of one response -> DiagPartial; level 2 in the last workgroup ------------------------
__global__ __launch_bounds__(kTileThreads) void diag_reduce_kernel(
    const float* __restrict__ logp_train, const float* __restrict__ logp_roll,
    const unsigned char* __restrict__ valid, long long n_rows, const long long* __restrict__ cu_rows, int n_resp,
    const int* __restrict__ tile_off, DiagPartial* partial, int group_size, const float* __restrict__ rewards,
    ais_params p, float* __restrict__ adv_out, int* __restrict__ count_out, ais_diag* __restrict__ diag_out,
    const int* __restrict__ status, int* ticket) {
  __shared__ double lds_d[12 * kWaves];          // three sets of moments and three sums per wavefront
  __shared__ long long lds_i[2 * kWaves];
  const int b = blockIdx.x;
  if (b < tile_off[n_resp]) {                        // uniform for the workgroup; the others only take a ticket
    const int i = find_response(tile_off, n_resp, b);
    long long lo, hi;
    response_rows(cu_rows, i, n_rows, lo, hi);
    const long long r0 = lo + (long long)(b - tile_off[i]) * kTileRows;
    const long long r1 = min(hi, r0 + kTileRows);
    const double lnC = log((double)p.C);
    Moments mw{0, 0, 0};
    double sabs = 0, sd = 0, sdp = 0;
    long long cnt = 0, nclip = 0;
    for (long long n = r0 + threadIdx.x; n < r1; n += kTileThreads) {
      if (valid != nullptr && valid[n] == 0) continue;
      const double lt = (double)logp_train[n], lr = (double)logp_roll[n];
      const double d = lt - lr;                                            // log rho (Alg. 1, sampler-trainer ratio)
      const double w = exp(fmin(d, lnC));                                  // w_bar = min(rho, C) (Eq. 10)
      push(mw, w);
      sabs += fabs(d);
      sd += d;
      sdp += fabs(exp(lt) - exp(lr));
      cnt += 1;
      nclip += (d > lnC) ? 1 : 0;
    }
    Moments m[1] = {mw};
    double d[3] = {sabs, sd, sdp};
    long long c[2] = {cnt, nclip};
    block_reduce(m, d, c, lds_d, lds_i);
    DiagPartial t;
    t.mean_w = m[0].mean;
    t.m2_w = m[0].m2;
    t.sabs = d[0];
    t.sd = d[1];
    t.sdp = d[2];
    t.cnt = c[0];
    t.nclip = c[1];
    if (threadIdx.x == 0) partial[b] = t;
  }
  // ---- level 2, in the workgroup that finishes last ----
  if (last_workgroup(ticket))
    diag_final(partial, tile_off, n_resp, group_size, rewards, p, adv_out, count_out, diag_out, status, lds_d, lds_i);
}

// ---- per-row coefficient of the gradient, rectification weight, loss ------------------------------------------------
__device__ void loss_final(const volatile double* partial, int n_tiles, double* __restrict__ loss_out, double* lds_d) {
  double acc = 0;
  for (int t = threadIdx.x; t < n_tiles; t += kTileThreads) acc += partial[t];
  acc = block_sum(acc, lds_d);
  if (threadIdx.x == 0) *loss_out = acc;
}

__global__ __launch_bounds__(kTileThreads) void row_coeff_kernel(
    const float* __restrict__ logp_train, const float* __restrict__ logp_roll, const float* __restrict__ logp_old,
    const float* __restrict__ logp_ref, const unsigned char* __restrict__ valid, long long n_rows,
    const long long* __restrict__ cu_rows, int n_resp, const float* __restrict__ adv,
    const int* __restrict__ count, const ais_diag* __restrict__ diag, ais_params p,
    const int* __restrict__ tile_off, double* partial, float* __restrict__ g_out,
    float* __restrict__ wtilde_out, float g_scale, double* __restrict__ loss_out, int* ticket) {
  __shared__ double lds_d[kWaves];
  const int b = blockIdx.x;
  if (b < tile_off[n_resp]) {                        // uniform for the workgroup; the others only take a ticket
    const int i = find_response(tile_off, n_resp, b);
    long long lo, hi;
    response_rows(cu_rows, i, n_rows, lo, hi);
    const long long r0 = lo + (long long)(b - tile_off[i]) * kTileRows;
    const long long r1 = min(hi, r0 + kTileRows);
    const double alpha = diag->alpha;
    const double a = (double)adv[i];
    const int cnt = count[i];
    const double wgt = cnt > 0 ? 1.0 / ((double)n_resp * (double)cnt) : 0.0;   // 1/G and 1/|o_i| of Eq. 19 over all prompts
    const double lnC = log((double)p.C);
    const double lo_clip = 1.0 - (double)p.clip_eps, hi_clip = 1.0 + (double)p.clip_eps;
    const bool kl = (logp_ref != nullptr) && (p.beta_kl > 0.f);
    double acc = 0;
    for (long long n = r0 + threadIdx.x; n < r1; n += kTileThreads) {
      float g = 0.f, wt = 0.f;
      if (valid == nullptr || valid[n] != 0) {
        const double lt = (double)logp_train[n];
        // the sampler-trainer ratio is taken at the checkpoint that generated the rollout (Alg. 1, "Sampler-Trainer
        // ratio"; Sec. 3.2: the two ratios are orthogonal), the old-new ratio between that checkpoint and theta
        const double l_old = logp_old != nullptr ? (double)logp_old[n] : lt;
        const double wbar = exp(fmin(l_old - (double)logp_roll[n], lnC));
        const double wtilde = 1.0 + alpha * (wbar - 1.0);                       // Eq. 18 / Alg. 1 rectification weight
        const double rho_on = logp_old != nullptr ? exp(lt - l_old) : 1.0;
        const double clipped = fmin(fmax(rho_on, lo_clip), hi_clip);
        // the unclipped branch is the minimum (ties included) iff the ratio has not left the trust
        // region on the side the advantage pushes towards
        const bool active = (a >= 0.0) ? (rho_on <= hi_clip) : (rho_on >= lo_clip);
        const double s = active ? rho_on * a : clipped * a;
        double obj = wtilde * s;
        double dobj = active ? wtilde * a * rho_on : 0.0;
        if (kl) {
          const double q = (double)logp_ref[n] - lt;
          const double eq = exp(q);
          obj -= (double)p.beta_kl * (eq - q - 1.0);
          dobj -= (double)p.beta_kl * (1.0 - eq);
        }
        acc -= wgt * obj;
        g = (float)(wgt * dobj * (double)g_scale);
        wt = (float)wtilde;
      }
      g_out[n] = g;
      if (wtilde_out != nullptr) wtilde_out[n] = wt;
    }
    acc = block_sum(acc, lds_d);
    if (threadIdx.x == 0) partial[b] = acc;
  }
  if (last_workgroup(ticket)) loss_final(partial, tile_off[n_resp], loss_out, lds_d);
}

}  // namespace

WorkspaceLayout workspace_layout(long long n_rows, int n_resp) {
  auto up = [](size_t v) { return (v + 255) & ~size_t(255); };
  WorkspaceLayout w;
  w.max_tiles = (int)((n_rows + kTileRows - 1) / kTileRows) + n_resp;
  w.tile_off = 0;                      // int [n_resp + 1] followed by the ticket counter
  w.partial = up(w.tile_off + sizeof(int) * (size_t)(n_resp + 2));
  w.g = up(w.partial + sizeof(DiagPartial) * (size_t)w.max_tiles);
  w.total = up(w.g + sizeof(float) * (size_t)n_rows);
  return w;
}

int launch_plan(ais_ctx* ctx, const long long* cu_rows, int n_resp, long long n_rows, int* tile_off,
                int max_tiles) {
  plan_kernel<<<1, kTileThreads, 0, ctx->stream>>>(cu_rows, n_resp, n_rows, tile_off, max_tiles, ctx->status_dev,
                                                   tile_off + n_resp + 1);
  return hip_fail(ctx, hipGetLastError());
}

int launch_diagnostics(ais_ctx* ctx, const float* logp_train, const float* logp_roll, const unsigned char* valid,
                       long long n_rows, const long long* cu_rows, int n_resp, int group_size,
                       const float* rewards, const ais_params& p, int* tile_off, int max_tiles,
                       DiagPartial* partial, float* adv_out, int* count_out, ais_diag* diag_out) {
  diag_reduce_kernel<<<max_tiles, kTileThreads, 0, ctx->stream>>>(logp_train, logp_roll, valid, n_rows, cu_rows,
                                                                  n_resp, tile_off, partial, group_size, rewards, p,
                                                                  adv_out, count_out, diag_out, ctx->status_dev,
                                                                  tile_off + n_resp + 1);
  return hip_fail(ctx, hipGetLastError());
}

int launch_row_coeff(ais_ctx* ctx, const float* logp_train, const float* logp_roll, const float* logp_old,
                     const float* logp_ref, const unsigned char* valid, long long n_rows,
                     const long long* cu_rows, int n_resp, const float* adv, const int* count,
                     const ais_diag* diag, const ais_params& p, int* tile_off, int max_tiles,
                     double* partial, float* g_out, float* wtilde_out, double* loss_out, float g_scale) {
  row_coeff_kernel<<<max_tiles, kTileThreads, 0, ctx->stream>>>(logp_train, logp_roll, logp_old, logp_ref, valid,
                                                                n_rows, cu_rows, n_resp, adv, count, diag, p,
                                                                tile_off, partial, g_out, wtilde_out, g_scale,
                                                                loss_out, tile_off + n_resp + 1);
  return hip_fail(ctx, hipGetLastError());
}

}  // namespace ais
