// Internal declarations shared by the translation units of the library (not installed).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <mutex>
#include <vector>

#include "ais.h"

namespace ais {

constexpr int kSweepThreads = 256;     // one workgroup (4 wavefronts) streams one logits row
constexpr int kTileThreads = 256;      // workgroup of the per-row scalar kernels
constexpr int kTileRows = 1024;        // rows of one response handled by one such workgroup
constexpr int kMaxDevices = 64;        // device indices a context may be created on
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

// Per-tile partial results of the diagnostics reduction (level 1 -> level 2).  The spread of w_bar travels as
// (count, mean, sum of squared deviations from the mean), merged pairwise: a variance never comes out of the
// difference of two large sums.
struct DiagPartial {
  double mean_w;  // mean of w_bar over the tile's valid rows
  double m2_w;    // sum of (w_bar - mean_w)^2
  double sabs;    // sum of |log pi_train - log pi_roll|
  double sd;      // sum of (log pi_train - log pi_roll)
  double sdp;     // sum of |pi_train - pi_roll|
  long long cnt;  // valid rows
  long long nclip;  // rows with rho > C
};

// Byte offsets of the regions of the context workspace for a call with (n_rows, n_resp).
struct WorkspaceLayout {
  size_t tile_off;   // int [n_resp + 2]   first tile of each response, total, and the ticket counter
  size_t partial;    // DiagPartial [max_tiles]  (reused as double [max_tiles] by the loss)
  size_t g;          // float [n_rows]     per-row gradient coefficient
  size_t total;
  int max_tiles;
};
WorkspaceLayout workspace_layout(long long n_rows, int n_resp);

// Decomposition of the hidden-state read-out when every row is evaluated: token blocks x chunks of vocabulary
// tiles.  The decomposition actually used is decided on the device from the number of evaluated rows.
struct LmHeadPlan {
  int n_tblocks;        // blocks of 256 tokens
  int n_vtiles;         // tiles of 256 vocabulary entries
  int n_chunks;         // contiguous chunks the tiles are split into
  int tiles_per_chunk;  // tiles of every chunk but possibly the last
  int max_chunks;       // most chunks the device-side decision can use (sizes the workspace)
};
LmHeadPlan lm_head_plan(long long n_rows, int vocab, int n_cus);

}  // namespace ais

struct ais_ctx {
  int device = 0;
  hipStream_t stream = nullptr;
  void* ws = nullptr;
  size_t ws_bytes = 0;
  int* status_dev = nullptr;
  int n_cus = 256;               // compute units of the device
  int last_hip_error = 0;
  bool profiling = false;
  struct Timed { hipEvent_t start, stop; int which; };
  std::vector<Timed> timed;      // events of measured launches
  std::vector<hipEvent_t> pool;  // recycled events
  // The row tiling that the last ais_diagnostics call left in the workspace (tile_off and a ticket counter that is
  // back at zero).  The calls that follow it in a step reuse the tiling instead of launching the plan kernel again
  // when they name the same cu_rows array, sizes and stream; anything else that writes the workspace clears it.
  struct Plan {
    const long long* cu_rows = nullptr;
    long long n_rows = -1;
    int n_resp = -1;
    hipStream_t stream = nullptr;
    bool valid = false;
  } plan;
  void* static_scratch = nullptr;   // address, on this context's device, of the library's static scratch array
  void* blas = nullptr;             // rocblas_handle of the two plain GEMMs of ais_lm_head_grad, created on first use
};

namespace ais {

int ensure_workspace(ais_ctx* ctx, size_t bytes);
int hip_fail(ais_ctx* ctx, hipError_t e);

// Raises the dynamic-LDS limit of kernel `fn` to `bytes` on the context's device, once per (kernel, device): `once`
// and `ok` are the caller's function-local tables of kMaxDevices entries.  False if the runtime refuses.
inline bool allow_dynamic_lds(ais_ctx* ctx, const void* fn, int bytes, std::once_flag* once, bool* ok) {
  std::call_once(once[ctx->device], [&] {
    ok[ctx->device] = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, bytes) == hipSuccess;
    if (!ok[ctx->device]) (void)hipGetLastError();
  });
  return ok[ctx->device];
}

// Brackets one launch with events when profiling is on.
struct ScopedTimer {
  ais_ctx* ctx;
  int idx = -1;
  ScopedTimer(ais_ctx* c, int which);
  ~ScopedTimer();
};

// Launchers (each checks nothing: arguments were validated by the entry point).
int launch_token_logprob(ais_ctx* ctx, const void* logits, ais_dtype dtype, long long n_rows, int vocab,
                         long long row_stride, const int* token_ids, const unsigned char* valid,
                         float inv_temperature, float* logp_out, float* lse_out);
int launch_dlogits(ais_ctx* ctx, const void* logits, ais_dtype dtype, long long n_rows, int vocab,
                   long long row_stride, const int* token_ids, const float* g, const unsigned char* valid,
                   const float* lse, const float* logp, float inv_temperature, void* dlogits);
int launch_fused_logprob_softmax(ais_ctx* ctx, const void* logits, ais_dtype dtype, long long n_rows, int vocab,
                                 long long row_stride, const int* token_ids, const unsigned char* valid,
                                 float inv_temperature, float* logp_out, float* lse_out, void* sgrad,
                                 bool* used_registers);
int launch_plan(ais_ctx* ctx, const long long* cu_rows, int n_resp, long long n_rows, int* tile_off, int max_tiles);
int launch_diagnostics(ais_ctx* ctx, const float* logp_train, const float* logp_roll, const unsigned char* valid,
                       long long n_rows, const long long* cu_rows, int n_resp, int group_size,
                       const float* rewards, const ais_params& p, int* tile_off, int max_tiles,
                       DiagPartial* partial, float* adv_out, int* count_out, ais_diag* diag_out);
int launch_row_coeff(ais_ctx* ctx, const float* logp_train, const float* logp_roll, const float* logp_old,
                     const float* logp_ref, const unsigned char* valid, long long n_rows,
                     const long long* cu_rows, int n_resp, const float* adv, const int* count,
                     const ais_diag* diag, const ais_params& p, int* tile_off, int max_tiles,
                     double* partial, float* g_out, float* wtilde_out, double* loss_out, float g_scale);
int launch_copy(ais_ctx* ctx, void* dst, const void* src, long long bytes);
int launch_fp8_quantize(ais_ctx* ctx, const void* logits, ais_dtype dtype, long long n_rows, int vocab,
                        long long row_stride, unsigned char* codes, long long codes_stride, float* scale_out);
bool try_fp8_quantize_rows(ais_ctx* ctx, const void* logits, ais_dtype dtype, long long n_rows, int vocab,
                           long long row_stride, unsigned char* codes, long long codes_stride, float* scale_out);
int launch_fp8_dequantize(ais_ctx* ctx, const unsigned char* codes, long long codes_stride, const float* scale,
                          long long n_rows, int vocab, void* out, ais_dtype dtype, long long out_stride);
bool try_fp8_dequantize_burst(ais_ctx* ctx, const unsigned char* codes, long long codes_stride, const float* scale,
                              long long n_rows, int vocab, void* out, ais_dtype dtype, long long out_stride);
bool try_fp8_quantize_table(ais_ctx* ctx, const void* logits, ais_dtype dtype, long long n_rows, int vocab,
                            long long row_stride, unsigned char* codes, long long codes_stride, float* scale_out);
bool try_fp8_rollout_logprob_table(ais_ctx* ctx, const void* logits, ais_dtype dtype, long long n_rows, int vocab,
                                   long long row_stride, const int* token_ids, const unsigned char* valid,
                                   float* logp_out);
int launch_fp8_rollout_logprob(ais_ctx* ctx, const void* logits, ais_dtype dtype, long long n_rows, int vocab,
                               long long row_stride, const int* token_ids, const unsigned char* valid,
                               float* logp_out);

int launch_lm_head_dlogits_chunk(ais_ctx* ctx, const void* hidden, long long ld_h, const void* weight,
                                 long long ld_w, long long n_rows, int d_model, int vocab, int y_off,
                                 const int* token_ids, const float* lse, const float* logp, const float* coeff,
                                 float inv_temperature, void* dev_plan, void* ds, long long ds_stride,
                                 const unsigned char* live_mask, int* row_index, int* row_pos, int n_cap);
int launch_lm_live_mask(ais_ctx* ctx, const float* coeff, long long n_rows, unsigned char* mask);
int launch_lm_gather_rows(ais_ctx* ctx, const void* hidden, long long ld_h, long long n_rows, int d_model,
                          const unsigned char* live_mask, int* row_index, int* row_pos, void* dev_plan, int n_cap,
                          void* gathered);
int launch_lm_scatter_rows(ais_ctx* ctx, const float* gathered, const int* row_pos, long long n_rows, int d_model,
                           float* out);
int launch_lm_head_logprob(ais_ctx* ctx, const void* hidden, long long ld_h, const void* weight, long long ld_w,
                           long long n_rows, int d_model, int vocab, const int* token_ids,
                           const unsigned char* valid, float inv_temperature, const LmHeadPlan& plan,
                           float* part_m, float* part_s, float* zy, int* row_index, int* row_pos, void* dev_plan,
                           float* logp_out, float* lse_out);

}  // namespace ais
