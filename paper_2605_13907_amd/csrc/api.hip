// The C entry points: host-side argument checks, workspace, launches.  See include/ais.h for the contract.
#include <algorithm>
#include <cmath>
#include <cstring>
#include <mutex>
#include <new>

#include <rocblas/rocblas.h>

#include "ais_internal.h"

// Scratch memory of ais_diagnostics_static: every GPU the library runs on holds its own copy of this array, at its
// own address, until the process ends.  In host code the name is only a handle for hipGetSymbolAddress, never an
// address: each device's address is looked up once, in ais_create, and kept; kernels receive that pointer.
static __device__ __align__(256) unsigned char scratch[AIS_STATIC_SCRATCH_BYTES];

namespace ais {

int hip_fail(ais_ctx* ctx, hipError_t e) {
  if (e == hipSuccess) return AIS_OK;
  if (ctx != nullptr) ctx->last_hip_error = (int)e;
  return AIS_ERR_HIP;
}

int ensure_workspace(ais_ctx* ctx, size_t bytes) {
  if (bytes <= ctx->ws_bytes) return AIS_OK;
  ctx->plan.valid = false;             // the tiling lived in the block that is about to be replaced
  // growing is rare (first call at a new size); it waits for queued work that may still use the old block
  hipError_t e = hipStreamSynchronize(ctx->stream);
  if (e != hipSuccess) return hip_fail(ctx, e);
  if (ctx->ws != nullptr) {
    (void)hipFree(ctx->ws);
    ctx->ws = nullptr;
    ctx->ws_bytes = 0;
  }
  const size_t want = bytes + bytes / 4;
  e = hipMalloc(&ctx->ws, want);
  if (e != hipSuccess) {
    ctx->last_hip_error = (int)e;
    (void)hipGetLastError();
    return AIS_ERR_NOMEM;
  }
  ctx->ws_bytes = want;
  return AIS_OK;
}

ScopedTimer::ScopedTimer(ais_ctx* c, int which) : ctx(c) {
  if (!ctx->profiling) return;
  ais_ctx::Timed t;
  t.which = which;
  hipEvent_t* ev[2] = {&t.start, &t.stop};
  for (auto* e : ev) {
    if (!ctx->pool.empty()) {
      *e = ctx->pool.back();
      ctx->pool.pop_back();
    } else if (hipEventCreate(e) != hipSuccess) {
      return;
    }
  }
  (void)hipEventRecord(t.start, ctx->stream);
  ctx->timed.push_back(t);
  idx = (int)ctx->timed.size() - 1;
}
ScopedTimer::~ScopedTimer() {
  if (idx >= 0) (void)hipEventRecord(ctx->timed[idx].stop, ctx->stream);
}

namespace {

// Clears an output with a kernel: a caller may be recording the stream into a graph, where memset nodes are avoided.
__global__ __launch_bounds__(256) void zero_fill_kernel(float* __restrict__ out, size_t n) {
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) out[i] = 0.f;
}

struct DeviceGuard {
  int prev = -1;
  bool ok = true;
  explicit DeviceGuard(int dev) {
    if (hipGetDevice(&prev) != hipSuccess) prev = -1;
    if (prev != dev) ok = (hipSetDevice(dev) == hipSuccess);
  }
  ~DeviceGuard() {
    if (prev >= 0) (void)hipSetDevice(prev);
  }
};

int check_logits(const void* logits, ais_dtype dtype, long long n_rows, long long vocab, long long row_stride) {
  if (dtype != AIS_BF16 && dtype != AIS_F32) return AIS_ERR_DTYPE;
  if (n_rows < 0 || n_rows > 0x7fffffffLL - 8) return AIS_ERR_SIZE;   // grids are rounded up to a multiple of 8 rows
  if (vocab < 1 || vocab > 0x7fffffffLL - 8) return AIS_ERR_SIZE;
  if (row_stride < vocab) return AIS_ERR_STRIDE;
  if (n_rows > 0 && logits == nullptr) return AIS_ERR_NULL;
  const size_t esize = dtype == AIS_BF16 ? 2 : 4;
  if (reinterpret_cast<uintptr_t>(logits) % esize != 0) return AIS_ERR_ALIGN;
  return AIS_OK;
}

int check_params(const ais_params* p) {
  if (p == nullptr) return AIS_ERR_NULL;
  auto fin = [](float v) { return std::isfinite(v); };
  if (!fin(p->C) || p->C < 1.f) return AIS_ERR_PARAM;
  if (!fin(p->delta) || p->delta <= 0.f) return AIS_ERR_PARAM;
  if (!fin(p->gamma) || p->gamma <= 0.f) return AIS_ERR_PARAM;
  if (!fin(p->eps_std) || p->eps_std < 0.f) return AIS_ERR_PARAM;
  if (!fin(p->beta_var) || p->beta_var < 0.f) return AIS_ERR_PARAM;
  if (!fin(p->clip_eps) || p->clip_eps < 0.f || p->clip_eps >= 1.f) return AIS_ERR_PARAM;
  if (p->adv_mode != 0 && p->adv_mode != 1) return AIS_ERR_PARAM;
  if (std::isnan(p->alpha_override) || p->alpha_override > 1.f) return AIS_ERR_PARAM;
  if (!fin(p->inv_temperature) || p->inv_temperature <= 0.f) return AIS_ERR_PARAM;
  if (!fin(p->beta_kl) || p->beta_kl < 0.f) return AIS_ERR_PARAM;
  return AIS_OK;
}

int check_batch(long long n_rows, int n_resp, int group_size) {
  if (n_rows < 0 || n_rows > 0x7fffffffLL) return AIS_ERR_SIZE;
  if (n_resp < 1 || n_resp > (1 << 24)) return AIS_ERR_SIZE;
  if (group_size < 1) return AIS_ERR_SIZE;
  if (n_resp % group_size != 0) return AIS_ERR_GROUP;
  return AIS_OK;
}

// Address of the current device's copy of the static scratch array; looked up once per device.  The caller has
// made `device` current.
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {};

int static_scratch_address(int device, void** out) {
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (g_scratch_ptr[device] == nullptr) {
    void* ptr = nullptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || ptr == nullptr) {
      (void)hipGetLastError();
      return AIS_ERR_HIP;
    }
    g_scratch_ptr[device] = ptr;
  }
  *out = g_scratch_ptr[device];
  return AIS_OK;
}

// Launches the plan kernel unless the tiling the last ais_diagnostics call left in the workspace is the one wanted.
int plan_for_step(ais_ctx* ctx, const long long* cu_rows, int n_resp, long long n_rows, int* tile_off, int max_tiles) {
  const ais_ctx::Plan& k = ctx->plan;
  if (k.valid && k.cu_rows == cu_rows && k.n_rows == n_rows && k.n_resp == n_resp && k.stream == ctx->stream)
    return AIS_OK;
  ctx->plan.valid = false;
  return launch_plan(ctx, cu_rows, n_resp, n_rows, tile_off, max_tiles);
}

int check_diagnostics_args(const float* logp_train, const float* logp_roll, long long n_rows,
                           const long long* cu_rows, int n_resp, int group_size, const float* rewards,
                           const ais_params* params, const float* adv_out, const int* count_out,
                           const ais_diag* diag_out) {
  int rc = check_batch(n_rows, n_resp, group_size);
  if (rc != AIS_OK) return rc;
  rc = check_params(params);
  if (rc != AIS_OK) return rc;
  if (cu_rows == nullptr || rewards == nullptr || adv_out == nullptr || count_out == nullptr ||
      diag_out == nullptr)
    return AIS_ERR_NULL;
  if (n_rows > 0 && (logp_train == nullptr || logp_roll == nullptr)) return AIS_ERR_NULL;
  return AIS_OK;
}

}  // namespace
}  // namespace ais

using namespace ais;

extern "C" {

int ais_version(void) { return 1000; }

void ais_params_default(ais_params* p) {
  if (p == nullptr) return;
  p->C = 5.0f;
  p->delta = 0.02f;
  p->gamma = 1.2f;
  p->eps_std = 1e-6f;
  p->beta_var = 1.0f;
  p->clip_eps = 0.2f;
  p->adv_mode = 0;
  p->alpha_override = -1.0f;
  p->inv_temperature = 1.0f;
  p->beta_kl = 0.0f;
}

const char* ais_strerror(int err) {
  switch (err) {
    case AIS_OK: return "ok";
    case AIS_ERR_NULL: return "a required pointer is NULL";
    case AIS_ERR_SIZE: return "a size is negative, zero or too large";
    case AIS_ERR_STRIDE: return "row_stride is smaller than vocab";
    case AIS_ERR_ALIGN: return "a pointer is not aligned to its element type";
    case AIS_ERR_PARAM: return "a hyper-parameter is outside its domain";
    case AIS_ERR_GROUP: return "n_resp is not a multiple of group_size";
    case AIS_ERR_DTYPE: return "unknown logits dtype";
    case AIS_ERR_HIP: return "a HIP runtime call failed";
    case AIS_ERR_NOMEM: return "workspace allocation failed";
    case AIS_ERR_SCRATCH: return "the batch needs more than the static scratch array holds";
    default: return "unknown error";
  }
}

int ais_create(ais_ctx** out, int device, void* hip_stream) {
  if (out == nullptr) return AIS_ERR_NULL;
  *out = nullptr;
  int n_dev = 0;
  if (hipGetDeviceCount(&n_dev) != hipSuccess || device < 0 || device >= n_dev) {
    (void)hipGetLastError();
    return AIS_ERR_HIP;
  }
  if (device >= kMaxDevices) return AIS_ERR_SIZE;   // per-device launch attributes are cached in fixed tables
  ais_ctx* ctx = new (std::nothrow) ais_ctx;
  if (ctx == nullptr) return AIS_ERR_NOMEM;
  ctx->device = device;
  ctx->stream = static_cast<hipStream_t>(hip_stream);
  DeviceGuard guard(device);
  hipError_t e = guard.ok ? hipMalloc(reinterpret_cast<void**>(&ctx->status_dev), 256) : hipErrorInvalidDevice;
  if (e == hipSuccess) e = hipMemset(ctx->status_dev, 0, 256);
  if (e != hipSuccess) {
    (void)hipGetLastError();
    delete ctx;
    return AIS_ERR_HIP;
  }
  int cus = 0;
  if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, device) == hipSuccess && cus > 0)
    ctx->n_cus = cus;
  else
    (void)hipGetLastError();
  int rc = ensure_workspace(ctx, 1 << 20);
  if (rc == AIS_OK) rc = guard.ok ? static_scratch_address(device, &ctx->static_scratch) : AIS_ERR_HIP;
  if (rc != AIS_OK) {
    if (ctx->ws != nullptr) (void)hipFree(ctx->ws);
    (void)hipFree(ctx->status_dev);
    delete ctx;
    return rc;
  }
  *out = ctx;
  return AIS_OK;
}

int ais_destroy(ais_ctx* ctx) {
  if (ctx == nullptr) return AIS_OK;
  DeviceGuard guard(ctx->device);
  (void)hipStreamSynchronize(ctx->stream);
  for (auto& t : ctx->timed) {
    (void)hipEventDestroy(t.start);
    (void)hipEventDestroy(t.stop);
  }
  for (auto& e : ctx->pool) (void)hipEventDestroy(e);
  if (ctx->blas != nullptr) (void)rocblas_destroy_handle(static_cast<rocblas_handle>(ctx->blas));
  if (ctx->ws != nullptr) (void)hipFree(ctx->ws);
  if (ctx->status_dev != nullptr) (void)hipFree(ctx->status_dev);
  delete ctx;
  return AIS_OK;
}

int ais_set_stream(ais_ctx* ctx, void* hip_stream) {
  if (ctx == nullptr) return AIS_ERR_NULL;
  ctx->stream = static_cast<hipStream_t>(hip_stream);
  return AIS_OK;
}

int ais_last_hip_error(const ais_ctx* ctx) { return ctx == nullptr ? 0 : ctx->last_hip_error; }

int ais_status(ais_ctx* ctx, int* host_out, int clear) {
  if (ctx == nullptr || host_out == nullptr) return AIS_ERR_NULL;
  DeviceGuard guard(ctx->device);
  hipError_t e = hipStreamSynchronize(ctx->stream);
  if (e == hipSuccess) e = hipMemcpy(host_out, ctx->status_dev, sizeof(int), hipMemcpyDeviceToHost);
  if (e == hipSuccess && clear) e = hipMemset(ctx->status_dev, 0, sizeof(int));
  return hip_fail(ctx, e);
}

int ais_token_logprob(ais_ctx* ctx, const void* logits, ais_dtype dtype, long long n_rows, long long vocab,
                      long long row_stride, const int* token_ids, const unsigned char* valid,
                      float inv_temperature, float* logp_out, float* lse_out) {
  int rc = check_logits(logits, dtype, n_rows, vocab, row_stride);
  if (rc != AIS_OK) return rc;
  if (n_rows > 0 && (token_ids == nullptr || logp_out == nullptr || lse_out == nullptr)) return AIS_ERR_NULL;
  if (!std::isfinite(inv_temperature) || inv_temperature <= 0.f) return AIS_ERR_PARAM;
  if (ctx == nullptr) return AIS_ERR_NULL;
  DeviceGuard guard(ctx->device);
  return launch_token_logprob(ctx, logits, dtype, n_rows, (int)vocab, row_stride, token_ids, valid,
                              inv_temperature, logp_out, lse_out);
}

int ais_diagnostics(ais_ctx* ctx, const float* logp_train, const float* logp_roll, const unsigned char* valid,
                    long long n_rows, const long long* cu_rows, int n_resp, int group_size,
                    const float* rewards, const ais_params* params, float* adv_out, int* count_out,
                    ais_diag* diag_out) {
  int rc = check_diagnostics_args(logp_train, logp_roll, n_rows, cu_rows, n_resp, group_size, rewards, params, adv_out,
                                  count_out, diag_out);
  if (rc != AIS_OK) return rc;
  if (ctx == nullptr) return AIS_ERR_NULL;
  DeviceGuard guard(ctx->device);
  const WorkspaceLayout w = workspace_layout(n_rows, n_resp);
  rc = ensure_workspace(ctx, w.total);
  if (rc != AIS_OK) return rc;
  char* ws = static_cast<char*>(ctx->ws);
  int* tile_off = reinterpret_cast<int*>(ws + w.tile_off);
  ctx->plan.valid = false;
  rc = launch_plan(ctx, cu_rows, n_resp, n_rows, tile_off, w.max_tiles);
  if (rc != AIS_OK) return rc;
  rc = launch_diagnostics(ctx, logp_train, logp_roll, valid, n_rows, cu_rows, n_resp, group_size, rewards, *params,
                          tile_off, w.max_tiles, reinterpret_cast<DiagPartial*>(ws + w.partial), adv_out, count_out,
                          diag_out);
  if (rc != AIS_OK) return rc;
  // the tiling stays in the workspace for the calls that complete this step
  ctx->plan.cu_rows = cu_rows;
  ctx->plan.n_rows = n_rows;
  ctx->plan.n_resp = n_resp;
  ctx->plan.stream = ctx->stream;
  ctx->plan.valid = true;
  return AIS_OK;
}

int ais_diagnostics_static(ais_ctx* ctx, const float* logp_train, const float* logp_roll,
                           const unsigned char* valid, long long n_rows, const long long* cu_rows, int n_resp,
                           int group_size, const float* rewards, const ais_params* params, float* adv_out,
                           int* count_out, ais_diag* diag_out) {
  int rc = check_diagnostics_args(logp_train, logp_roll, n_rows, cu_rows, n_resp, group_size, rewards, params, adv_out,
                                  count_out, diag_out);
  if (rc != AIS_OK) return rc;
  // what the two kernels need: the tiling with its ticket counter, and one partial per tile (not the per-row
  // coefficients of the gradient call, which come after them in the layout)
  const WorkspaceLayout w = workspace_layout(n_rows, n_resp);
  if (w.g > (size_t)AIS_STATIC_SCRATCH_BYTES) return AIS_ERR_SCRATCH;
  if (ctx == nullptr) return AIS_ERR_NULL;
  if (ctx->static_scratch == nullptr) return AIS_ERR_HIP;
  DeviceGuard guard(ctx->device);
  char* ws = static_cast<char*>(ctx->static_scratch);     // this device's address of the array, never its name
  int* tile_off = reinterpret_cast<int*>(ws + w.tile_off);
  // the plan kernel writes every tile_off entry this call reads and zeroes the ticket counter; every partial that
  // level 2 reads is written by level 1 of the same launch: nothing of an earlier call's contents is used
  rc = launch_plan(ctx, cu_rows, n_resp, n_rows, tile_off, w.max_tiles);
  if (rc != AIS_OK) return rc;
  return launch_diagnostics(ctx, logp_train, logp_roll, valid, n_rows, cu_rows, n_resp, group_size, rewards, *params,
                            tile_off, w.max_tiles, reinterpret_cast<DiagPartial*>(ws + w.partial), adv_out, count_out,
                            diag_out);
}

int ais_grpo_loss_grad(ais_ctx* ctx, const void* logits, ais_dtype dtype, long long n_rows, long long vocab,
                       long long row_stride, const int* token_ids, const unsigned char* valid,
                       const long long* cu_rows, int n_resp, const float* logp_train, const float* lse,
                       const float* logp_roll, const float* logp_old, const float* logp_ref, const float* adv,
                       const int* count, const ais_diag* diag, const ais_params* params, float* wtilde_out,
                       double* loss_out, void* dlogits) {
  int rc = check_logits(logits, dtype, n_rows, vocab, row_stride);
  if (rc != AIS_OK) return rc;
  rc = check_batch(n_rows, n_resp, 1);
  if (rc != AIS_OK) return rc;
  rc = check_params(params);
  if (rc != AIS_OK) return rc;
  if (cu_rows == nullptr || adv == nullptr || count == nullptr || diag == nullptr || loss_out == nullptr)
    return AIS_ERR_NULL;
  if (n_rows > 0 && (token_ids == nullptr || logp_train == nullptr || lse == nullptr || logp_roll == nullptr ||
                     dlogits == nullptr))
    return AIS_ERR_NULL;
  if (reinterpret_cast<uintptr_t>(dlogits) % (dtype == AIS_BF16 ? 2 : 4) != 0) return AIS_ERR_ALIGN;
  if (ctx == nullptr) return AIS_ERR_NULL;
  DeviceGuard guard(ctx->device);
  const WorkspaceLayout w = workspace_layout(n_rows, n_resp);
  rc = ensure_workspace(ctx, w.total);
  if (rc != AIS_OK) return rc;
  char* ws = static_cast<char*>(ctx->ws);
  int* tile_off = reinterpret_cast<int*>(ws + w.tile_off);
  float* g = reinterpret_cast<float*>(ws + w.g);
  rc = plan_for_step(ctx, cu_rows, n_resp, n_rows, tile_off, w.max_tiles);
  if (rc != AIS_OK) return rc;
  rc = launch_row_coeff(ctx, logp_train, logp_roll, logp_old, logp_ref, valid, n_rows, cu_rows, n_resp, adv, count,
                        diag, *params, tile_off, w.max_tiles, reinterpret_cast<double*>(ws + w.partial), g,
                        wtilde_out, loss_out, 1.0f);
  if (rc != AIS_OK) return rc;
  return launch_dlogits(ctx, logits, dtype, n_rows, (int)vocab, row_stride, token_ids, g, nullptr, lse, logp_train,
                        params->inv_temperature, dlogits);
}

int ais_token_logprob_softmax_grad(ais_ctx* ctx, const void* logits, ais_dtype dtype, long long n_rows,
                                   long long vocab, long long row_stride, const int* token_ids,
                                   const unsigned char* valid, float inv_temperature, float* logp_out,
                                   float* lse_out, void* sgrad_out) {
  int rc = check_logits(logits, dtype, n_rows, vocab, row_stride);
  if (rc != AIS_OK) return rc;
  if (n_rows > 0 && (token_ids == nullptr || logp_out == nullptr || lse_out == nullptr || sgrad_out == nullptr))
    return AIS_ERR_NULL;
  if (reinterpret_cast<uintptr_t>(sgrad_out) % (dtype == AIS_BF16 ? 2 : 4) != 0) return AIS_ERR_ALIGN;
  if (!std::isfinite(inv_temperature) || inv_temperature <= 0.f) return AIS_ERR_PARAM;
  if (ctx == nullptr) return AIS_ERR_NULL;
  DeviceGuard guard(ctx->device);
  bool used = false;
  rc = launch_fused_logprob_softmax(ctx, logits, dtype, n_rows, (int)vocab, row_stride, token_ids, valid,
                                    inv_temperature, logp_out, lse_out, sgrad_out, &used);
  if (rc != AIS_OK || used) return rc;
  // the row does not fit the register file: two passes (log-probs, then the direction with unit coefficient)
  rc = launch_token_logprob(ctx, logits, dtype, n_rows, (int)vocab, row_stride, token_ids, valid, inv_temperature,
                            logp_out, lse_out);
  if (rc != AIS_OK) return rc;
  return launch_dlogits(ctx, logits, dtype, n_rows, (int)vocab, row_stride, token_ids, nullptr, valid, lse_out,
                        logp_out, inv_temperature, sgrad_out);
}

int ais_grpo_row_scale(ais_ctx* ctx, const float* logp_train, const float* logp_roll, const float* logp_old,
                       const float* logp_ref, const unsigned char* valid, long long n_rows,
                       const long long* cu_rows, int n_resp, const float* adv, const int* count,
                       const ais_diag* diag, const ais_params* params, float* wtilde_out, double* loss_out,
                       float* g_out) {
  int rc = check_batch(n_rows, n_resp, 1);
  if (rc != AIS_OK) return rc;
  rc = check_params(params);
  if (rc != AIS_OK) return rc;
  if (cu_rows == nullptr || adv == nullptr || count == nullptr || diag == nullptr || loss_out == nullptr)
    return AIS_ERR_NULL;
  if (n_rows > 0 && (logp_train == nullptr || logp_roll == nullptr || g_out == nullptr)) return AIS_ERR_NULL;
  if (ctx == nullptr) return AIS_ERR_NULL;
  DeviceGuard guard(ctx->device);
  const WorkspaceLayout w = workspace_layout(n_rows, n_resp);
  rc = ensure_workspace(ctx, w.total);
  if (rc != AIS_OK) return rc;
  char* ws = static_cast<char*>(ctx->ws);
  int* tile_off = reinterpret_cast<int*>(ws + w.tile_off);
  rc = plan_for_step(ctx, cu_rows, n_resp, n_rows, tile_off, w.max_tiles);
  if (rc != AIS_OK) return rc;
  return launch_row_coeff(ctx, logp_train, logp_roll, logp_old, logp_ref, valid, n_rows, cu_rows, n_resp, adv, count,
                          diag, *params, tile_off, w.max_tiles, reinterpret_cast<double*>(ws + w.partial), g_out,
                          wtilde_out, loss_out, params->inv_temperature);
}

int ais_fp8_quantize_rows(ais_ctx* ctx, const void* logits, ais_dtype dtype, long long n_rows, long long vocab,
                          long long row_stride, unsigned char* codes_out, long long codes_stride,
                          float* scale_out) {
  int rc = check_logits(logits, dtype, n_rows, vocab, row_stride);
  if (rc != AIS_OK) return rc;
  if (codes_stride < vocab) return AIS_ERR_STRIDE;
  if (n_rows > 0 && (codes_out == nullptr || scale_out == nullptr)) return AIS_ERR_NULL;
  if (ctx == nullptr) return AIS_ERR_NULL;
  DeviceGuard guard(ctx->device);
  return launch_fp8_quantize(ctx, logits, dtype, n_rows, (int)vocab, row_stride, codes_out, codes_stride,
                             scale_out);
}

int ais_fp8_dequantize_rows(ais_ctx* ctx, const unsigned char* codes, long long codes_stride, const float* scale,
                            long long n_rows, long long vocab, void* out, ais_dtype out_dtype,
                            long long out_stride) {
  int rc = check_logits(out, out_dtype, n_rows, vocab, out_stride);
  if (rc != AIS_OK) return rc;
  if (codes_stride < vocab) return AIS_ERR_STRIDE;
  if (n_rows > 0 && (codes == nullptr || scale == nullptr)) return AIS_ERR_NULL;
  if (ctx == nullptr) return AIS_ERR_NULL;
  DeviceGuard guard(ctx->device);
  return launch_fp8_dequantize(ctx, codes, codes_stride, scale, n_rows, (int)vocab, out, out_dtype, out_stride);
}

int ais_fp8_rollout_logprob(ais_ctx* ctx, const void* logits, ais_dtype dtype, long long n_rows, long long vocab,
                            long long row_stride, const int* token_ids, const unsigned char* valid,
                            float* logp_roll_out) {
  int rc = check_logits(logits, dtype, n_rows, vocab, row_stride);
  if (rc != AIS_OK) return rc;
  if (n_rows > 0 && (token_ids == nullptr || logp_roll_out == nullptr)) return AIS_ERR_NULL;
  if (ctx == nullptr) return AIS_ERR_NULL;
  DeviceGuard guard(ctx->device);
  return launch_fp8_rollout_logprob(ctx, logits, dtype, n_rows, (int)vocab, row_stride, token_ids, valid,
                                    logp_roll_out);
}

int ais_lm_head_logprob(ais_ctx* ctx, const void* hidden, long long hidden_stride, const void* weight,
                        long long weight_stride, ais_dtype dtype, long long n_rows, long long d_model,
                        long long vocab, const int* token_ids, const unsigned char* valid, float inv_temperature,
                        float* logp_out, float* lse_out) {
  if (dtype != AIS_BF16) return AIS_ERR_DTYPE;
  if (n_rows < 0 || n_rows > 0x7fffffffLL - 256) return AIS_ERR_SIZE;
  if (vocab < 1 || vocab > 0x7fffffffLL - 256) return AIS_ERR_SIZE;
  if (d_model < 8 || d_model > (1 << 20) || d_model % 8 != 0) return AIS_ERR_SIZE;
  if (hidden_stride < d_model || weight_stride < d_model) return AIS_ERR_STRIDE;
  if (weight == nullptr) return AIS_ERR_NULL;
  if (n_rows > 0 && (hidden == nullptr || token_ids == nullptr || logp_out == nullptr || lse_out == nullptr))
    return AIS_ERR_NULL;
  if (reinterpret_cast<uintptr_t>(hidden) % 16 != 0 || reinterpret_cast<uintptr_t>(weight) % 16 != 0 ||
      hidden_stride % 8 != 0 || weight_stride % 8 != 0)
    return AIS_ERR_ALIGN;
  if (!std::isfinite(inv_temperature) || inv_temperature <= 0.f) return AIS_ERR_PARAM;
  if (ctx == nullptr) return AIS_ERR_NULL;
  if (n_rows == 0) return AIS_OK;
  DeviceGuard guard(ctx->device);
  const LmHeadPlan plan = lm_head_plan(n_rows, (int)vocab, ctx->n_cus);
  // workspace: per-chunk partial (max, sum) and the sampled token's logit of every evaluated position, the list
  // of evaluated rows, its inverse, and the device-side decomposition
  const size_t per = sizeof(float) * (size_t)n_rows;
  int rc = ensure_workspace(ctx, per * (2 * (size_t)plan.max_chunks + 3) + 256);
  if (rc != AIS_OK) return rc;
  ctx->plan.valid = false;             // this call's partials overwrite whatever tiling the workspace held
  float* part_m = static_cast<float*>(ctx->ws);
  float* part_s = part_m + (size_t)plan.max_chunks * (size_t)n_rows;
  float* zy = part_s + (size_t)plan.max_chunks * (size_t)n_rows;
  int* row_index = reinterpret_cast<int*>(zy + n_rows);
  int* row_pos = row_index + n_rows;
  void* dev_plan = row_pos + n_rows;
  return launch_lm_head_logprob(ctx, hidden, hidden_stride, weight, weight_stride, n_rows, (int)d_model, (int)vocab,
                                token_ids, valid, inv_temperature, plan, part_m, part_s, zy, row_index, row_pos,
                                dev_plan, logp_out, lse_out);
}

int ais_lm_head_grad(ais_ctx* ctx, const void* hidden, long long hidden_stride, const void* weight,
                     long long weight_stride, ais_dtype dtype, long long n_rows, long long d_model, long long vocab,
                     const int* token_ids, const float* lse, const float* logp, const float* coeff,
                     float inv_temperature, long long chunk_vocab, long long n_live_max, float* dhidden_out,
                     float* dweight_out) {
  if (dtype != AIS_BF16) return AIS_ERR_DTYPE;
  if (n_rows < 0 || n_rows > 0x7fffffffLL - 256) return AIS_ERR_SIZE;
  if (vocab < 1 || vocab > 0x7fffffffLL - 256) return AIS_ERR_SIZE;
  if (d_model < 32 || d_model > (1 << 20) || d_model % 32 != 0) return AIS_ERR_SIZE;
  if (chunk_vocab == 0) chunk_vocab = 8192;
  if (chunk_vocab < 256 || chunk_vocab > (1 << 24) || chunk_vocab % 256 != 0) return AIS_ERR_SIZE;
  if (hidden_stride < d_model || weight_stride < d_model) return AIS_ERR_STRIDE;
  if (weight == nullptr || dweight_out == nullptr) return AIS_ERR_NULL;
  if (n_rows > 0 && (hidden == nullptr || token_ids == nullptr || lse == nullptr || logp == nullptr ||
                     coeff == nullptr || dhidden_out == nullptr))
    return AIS_ERR_NULL;
  if (reinterpret_cast<uintptr_t>(hidden) % 16 != 0 || reinterpret_cast<uintptr_t>(weight) % 16 != 0 ||
      hidden_stride % 8 != 0 || weight_stride % 8 != 0 || reinterpret_cast<uintptr_t>(dhidden_out) % 4 != 0 ||
      reinterpret_cast<uintptr_t>(dweight_out) % 4 != 0)
    return AIS_ERR_ALIGN;
  if (!std::isfinite(inv_temperature) || inv_temperature <= 0.f) return AIS_ERR_PARAM;
  if (ctx == nullptr) return AIS_ERR_NULL;
  DeviceGuard guard(ctx->device);
  if (n_rows == 0) {                   // no rows: the embedding gradient is zero, there is no hidden-state gradient
    const size_t n = (size_t)vocab * (size_t)d_model;
    const unsigned blocks = (unsigned)std::min<size_t>((n + 255) / 256, (size_t)ctx->n_cus * 8);
    zero_fill_kernel<<<blocks, 256, 0, ctx->stream>>>(dweight_out, n);
    return hip_fail(ctx, hipGetLastError());
  }
  if (chunk_vocab > ((vocab + 255) / 256) * 256) chunk_vocab = ((vocab + 255) / 256) * 256;
  const bool gather = n_live_max >= 0 && n_live_max < n_rows;
  const long long m_rows = gather ? n_live_max : n_rows;       // rows that the recomputation and the GEMMs cover
  if (m_rows == 0) {                    // the caller vouches that no row has a gradient
    zero_fill_kernel<<<(unsigned)std::min<size_t>(((size_t)vocab * d_model + 255) / 256, (size_t)ctx->n_cus * 8), 256, 0,
                       ctx->stream>>>(dweight_out, (size_t)vocab * (size_t)d_model);
    zero_fill_kernel<<<(unsigned)std::min<size_t>(((size_t)n_rows * d_model + 255) / 256, (size_t)ctx->n_cus * 8), 256, 0,
                       ctx->stream>>>(dhidden_out, (size_t)n_rows * (size_t)d_model);
    return hip_fail(ctx, hipGetLastError());
  }
  // workspace: the chunk's dlogits, the device-side decomposition of the recompute kernel and, with a row list, the
  // mask, the list, its inverse, the gathered hidden states and their gradient
  auto up = [](size_t b) { return (b + 255) & ~size_t(255); };
  const size_t ds_bytes = up((size_t)m_rows * (size_t)chunk_vocab * 2);
  const size_t plan_bytes = 256;
  const size_t mask_bytes = gather ? up((size_t)n_rows) : 0;
  const size_t list_bytes = gather ? up((size_t)n_rows * 4) : 0;
  const size_t hg_bytes = gather ? up((size_t)m_rows * (size_t)d_model * 2) : 0;
  const size_t dhg_bytes = gather ? up((size_t)m_rows * (size_t)d_model * 4) : 0;
  int rc = ensure_workspace(ctx, ds_bytes + plan_bytes + mask_bytes + 2 * list_bytes + hg_bytes + dhg_bytes);
  if (rc != AIS_OK) return rc;
  ctx->plan.valid = false;             // the chunk's dlogits overwrite whatever tiling the workspace held
  char* ds = static_cast<char*>(ctx->ws);
  void* dev_plan = ds + ds_bytes;
  unsigned char* live_mask = gather ? reinterpret_cast<unsigned char*>(ds + ds_bytes + plan_bytes) : nullptr;
  int* row_index = gather ? reinterpret_cast<int*>(ds + ds_bytes + plan_bytes + mask_bytes) : nullptr;
  int* row_pos = gather ? reinterpret_cast<int*>(ds + ds_bytes + plan_bytes + mask_bytes + list_bytes) : nullptr;
  char* h_gathered = ds + ds_bytes + plan_bytes + mask_bytes + 2 * list_bytes;
  float* dh_gathered = reinterpret_cast<float*>(h_gathered + hg_bytes);
  if (gather) {
    rc = launch_lm_live_mask(ctx, coeff, n_rows, live_mask);
    if (rc == AIS_OK)
      rc = launch_lm_gather_rows(ctx, hidden, hidden_stride, n_rows, (int)d_model, live_mask, row_index, row_pos, dev_plan,
                                 (int)m_rows, h_gathered);
    if (rc != AIS_OK) return rc;
  }
  // operands of the two GEMMs: the hidden states they read and the gradient they write, with their pitches
  const void* h_gemm = gather ? static_cast<const void*>(h_gathered) : hidden;
  const long long h_gemm_stride = gather ? d_model : hidden_stride;
  float* dh_gemm = gather ? dh_gathered : dhidden_out;
  if (ctx->blas == nullptr) {
    rocblas_handle h = nullptr;
    if (rocblas_create_handle(&h) != rocblas_status_success) return AIS_ERR_HIP;
    ctx->blas = h;
  }
  rocblas_handle blas = static_cast<rocblas_handle>(ctx->blas);
  if (rocblas_set_stream(blas, ctx->stream) != rocblas_status_success) return AIS_ERR_HIP;
  if (rocblas_set_pointer_mode(blas, rocblas_pointer_mode_host) != rocblas_status_success) return AIS_ERR_HIP;
  const float one = 1.f, zero = 0.f;
  const char* w_base = static_cast<const char*>(weight);
  for (long long v0 = 0; v0 < vocab; v0 += chunk_vocab) {
    const int width = (int)std::min<long long>(chunk_vocab, vocab - v0);
    const void* w_chunk = w_base + (size_t)v0 * (size_t)weight_stride * 2;
    rc = launch_lm_head_dlogits_chunk(ctx, hidden, hidden_stride, w_chunk, weight_stride, n_rows, (int)d_model, width,
                                      (int)v0, token_ids, lse, logp, coeff, inv_temperature, dev_plan, ds,
                                      chunk_vocab, live_mask, row_index, row_pos, (int)m_rows);
    if (rc != AIS_OK) return rc;
    // The library is column-major; a row-major [r, c] matrix with pitch p is its column-major [c, r] transpose
    // with leading dimension p.
    // dhidden[m_rows, D] (+)= ds[m_rows, width] weight_chunk[width, D]:   C^T[D, m_rows] = W_c^T[D, width] ds^T[width, m_rows]
    rocblas_status st = rocblas_gemm_ex(
        blas, rocblas_operation_none, rocblas_operation_none, (rocblas_int)d_model, (rocblas_int)m_rows, width, &one,
        w_chunk, rocblas_datatype_bf16_r, (rocblas_int)weight_stride, ds, rocblas_datatype_bf16_r,
        (rocblas_int)chunk_vocab, v0 == 0 ? &zero : &one, dh_gemm, rocblas_datatype_f32_r, (rocblas_int)d_model,
        dh_gemm, rocblas_datatype_f32_r, (rocblas_int)d_model, rocblas_datatype_f32_r, rocblas_gemm_algo_standard,
        0, 0);
    if (st != rocblas_status_success) return AIS_ERR_HIP;
    // dweight_chunk[width, D] = ds^T[width, m_rows] hidden[m_rows, D]:   C^T[D, width] = H^T[D, m_rows] ds[m_rows, width]
    float* dw_chunk = dweight_out + (size_t)v0 * (size_t)d_model;
    st = rocblas_gemm_ex(blas, rocblas_operation_none, rocblas_operation_transpose, (rocblas_int)d_model, width,
                         (rocblas_int)m_rows, &one, h_gemm, rocblas_datatype_bf16_r, (rocblas_int)h_gemm_stride, ds,
                         rocblas_datatype_bf16_r, (rocblas_int)chunk_vocab, &zero, dw_chunk, rocblas_datatype_f32_r,
                         (rocblas_int)d_model, dw_chunk, rocblas_datatype_f32_r, (rocblas_int)d_model,
                         rocblas_datatype_f32_r, rocblas_gemm_algo_standard, 0, 0);
    if (st != rocblas_status_success) return AIS_ERR_HIP;
  }
  if (gather) return launch_lm_scatter_rows(ctx, dh_gathered, row_pos, n_rows, (int)d_model, dhidden_out);
  return AIS_OK;
}

int ais_profile(ais_ctx* ctx, int enable) {
  if (ctx == nullptr) return AIS_ERR_NULL;
  DeviceGuard guard(ctx->device);
  hipError_t e = hipStreamSynchronize(ctx->stream);
  for (auto& t : ctx->timed) {
    ctx->pool.push_back(t.start);
    ctx->pool.push_back(t.stop);
  }
  ctx->timed.clear();
  ctx->profiling = enable != 0;
  return hip_fail(ctx, e);
}

int ais_profile_read(ais_ctx* ctx, int which, float* total_ms, int* launches) {
  if (ctx == nullptr || total_ms == nullptr || launches == nullptr) return AIS_ERR_NULL;
  if (which < 0 || which >= AIS_K_COUNT_) return AIS_ERR_SIZE;
  DeviceGuard guard(ctx->device);
  hipError_t e = hipStreamSynchronize(ctx->stream);
  if (e != hipSuccess) return hip_fail(ctx, e);
  float total = 0.f;
  int n = 0;
  for (auto& t : ctx->timed) {
    if (t.which != which) continue;
    float ms = 0.f;
    e = hipEventElapsedTime(&ms, t.start, t.stop);
    if (e != hipSuccess) return hip_fail(ctx, e);
    total += ms;
    ++n;
  }
  *total_ms = total;
  *launches = n;
  return AIS_OK;
}

int ais_copy(ais_ctx* ctx, void* dst, const void* src, long long bytes) {
  if (bytes < 0 || bytes % 16 != 0) return AIS_ERR_SIZE;
  if (bytes > 0 && (dst == nullptr || src == nullptr)) return AIS_ERR_NULL;
  if (reinterpret_cast<uintptr_t>(dst) % 16 != 0 || reinterpret_cast<uintptr_t>(src) % 16 != 0) return AIS_ERR_ALIGN;
  if (ctx == nullptr) return AIS_ERR_NULL;
  DeviceGuard guard(ctx->device);
  return launch_copy(ctx, dst, src, bytes);
}

}  // extern "C"
