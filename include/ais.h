/*
 * ais.h — C ABI of the AIS-GRPO hot path on one AMD MI355X (gfx950).
 *
 * The library evaluates, for one batch of rollouts, the part of an AIS-GRPO
 * training step that lies between the trainer's forward pass and its backward
 * pass (Alg. 1, "Adaptive Coefficient Estimation", "Advantage Rectification"
 * and the objective of Eq. 19):
 *
 *   ais_token_logprob    log pi_train(o_t) for every evaluated token, from the
 *                        full-vocabulary trainer logits
 *   ais_diagnostics      sampler-trainer ratios, the three diagnostics
 *                        (Eq. 12, 14, 16), the mixing coefficient alpha
 *                        (Eq. 17), group-relative advantages (Eq. 3)
 *   ais_grpo_loss_grad   rectification weights (Eq. 18), the AIS-GRPO loss
 *                        (Eq. 19, negated) and its gradient w.r.t. the logits
 *
 * Conventions that hold for every call
 *   Memory     Every array argument is DEVICE memory owned by the caller on the
 *              context's GPU, unless its comment says "host".  Nothing is kept
 *              after a call returns; the context owns only a small reduction
 *              workspace.  Outputs must not overlap inputs unless stated.
 *   Order      Calls enqueue work on the context's HIP stream and return
 *              without waiting for it.  Results are ready when that stream
 *              reaches the point of the call.  Calls on one context must not
 *              overlap in time (they share its workspace); different contexts
 *              are independent.
 *   Workspace  The workspace grows when a call needs more than any call before
 *              it (more rows or responses): that call waits for the stream and
 *              allocates device memory.  Calls at sizes seen before allocate
 *              nothing and can be recorded into a HIP graph; run one call at
 *              the largest size before capturing.
 *   Layout     Logits are row-major [n_rows, vocab] with a row pitch of
 *              row_stride elements.  One row is one token position.  Response
 *              i owns rows [cu_rows[i], cu_rows[i+1]); cu_rows[0] = 0,
 *              cu_rows[n_resp] = n_rows, non-decreasing.  Prompt p owns the
 *              group_size consecutive responses starting at p * group_size.
 *              valid[n] != 0 marks a row whose token is evaluated (a generated,
 *              non-padding position; for masked-diffusion rollouts a masked
 *              position).  valid == NULL means all rows.
 *   Errors     Functions return 0 on success or a negative ais_error.
 *              Arguments are checked on the host before anything is launched;
 *              a failing call launches nothing.  Faults that only the device
 *              can see (a token id outside [0, vocab) on an evaluated row,
 *              cu_rows that is not a partition of the rows) never cause an
 *              out-of-range access: the row is computed as if it had no token
 *              (its logp is 0), and a bit is set in the context's status word
 *              (ais_status) and in ais_diag.status.
 *   Degenerate n_rows = 0, no valid row at all, a response without valid rows,
 *              all rewards equal: not errors; outputs are 0 and alpha = 0.
 */
#ifndef AIS_H_
#define AIS_H_

#ifdef __cplusplus
extern "C" {
#endif

typedef struct ais_ctx ais_ctx;

typedef enum ais_dtype { AIS_BF16 = 0, AIS_F32 = 1 } ais_dtype;

typedef enum ais_error {
  AIS_OK = 0,
  AIS_ERR_NULL = -1,    /* a required pointer is NULL                                  */
  AIS_ERR_SIZE = -2,    /* a negative or zero size where one is not allowed, or > limit  */
  AIS_ERR_STRIDE = -3,  /* row_stride < vocab                                          */
  AIS_ERR_ALIGN = -4,   /* a pointer is not aligned to its element type                */
  AIS_ERR_PARAM = -5,   /* a hyper-parameter outside its domain                        */
  AIS_ERR_GROUP = -6,   /* n_resp is not a positive multiple of group_size             */
  AIS_ERR_DTYPE = -7,   /* unknown ais_dtype                                           */
  AIS_ERR_HIP = -8,     /* a HIP runtime call failed (see ais_last_hip_error)          */
  AIS_ERR_NOMEM = -9,   /* workspace allocation failed                                 */
  AIS_ERR_SCRATCH = -10 /* the batch needs more than the static scratch array holds    */
} ais_error;

/* Bits of the device status word. */
#define AIS_STATUS_BAD_TOKEN 1   /* evaluated row with token id outside [0, vocab)     */
#define AIS_STATUS_BAD_CU    2   /* cu_rows not a non-decreasing partition of the rows */
#define AIS_STATUS_LIVE_OVERFLOW 4 /* ais_lm_head_grad: more rows with a gradient than n_live_max */

/* Hyper-parameters.  ais_params_default() fills in the paper's values:
 * C, delta, gamma, eps_std from App. "AIS hyperparameters"; clip_eps from the
 * hyper-parameter table of App. "RL Training Setup". */
typedef struct ais_params {
  float C;               /* 5.0   truncation of the importance ratio, >= 1 (Eq. 10)            */
  float delta;           /* 0.02  saturation threshold of alpha_mis, > 0 (Eq. 14)              */
  float gamma;           /* 1.2   variance tolerance of alpha_var, > 0 (Eq. 16)                */
  float eps_std;         /* 1e-6  stabiliser in the variance-amplification ratio (Eq. 15)      */
  float beta_var;        /* 1.0   beta of Eq. 17; the paper prints no value                    */
  float clip_eps;        /* 0.2   PPO clipping range of Eq. 19, in [0, 1)                      */
  int   adv_mode;        /* 0: A = r - mean(group) (Eq. 3);  1: divided by (pstd(group)+eps)  */
  float alpha_override;  /* < 0: adaptive alpha (Eq. 17); in [0,1]: forced (0 = plain GRPO,
                            1 = token-level truncated importance sampling, Eq. 8)              */
  float inv_temperature; /* 1.0   logits are multiplied by this before the softmax, > 0        */
  float beta_kl;         /* 0.0   weight of the KL term of Eq. 19 (needs logp_ref), >= 0       */
} ais_params;

/* Written by ais_diagnostics into DEVICE memory; statistics are over the valid
 * rows of the batch (population moments, A broadcast to the tokens of its response). */
typedef struct ais_diag {
  long long n_valid;     /* number of valid rows                                               */
  double mean_w, var_w;  /* mean and population variance of w_bar = min(rho, C)                */
  double cv2;            /* squared coefficient of variation of w_bar (0 if every w_bar is 0)  */
  double ess_ratio;      /* 1 / (1 + cv2)                                                      */
  double dbar;           /* mean |log pi_train - log pi_roll|            (Eq. 13)              */
  double std_a, std_aw;  /* population std of A and of A * w_bar                               */
  double dsigma;         /* std_aw / (std_a + eps_std)                    (Eq. 15)             */
  double alpha_ess;      /* (1 + cv2)^(-1/2)                              (Eq. 12)             */
  double alpha_mis;      /* min(1, dbar / delta)                          (Eq. 14)             */
  double alpha_var;      /* max(0, (dsigma - gamma) / gamma)              (Eq. 16)             */
  double alpha;          /* clip(alpha_ess - beta_var alpha_var, 0, 1) alpha_mis (Eq. 17),
                            or alpha_override                                                  */
  double clip_frac;      /* share of valid rows with rho > C                                   */
  double kl_roll_train;  /* mean(log pi_roll - log pi_train) over the sampled tokens: the estimate
                            of KL(pi_roll || pi_train) plotted in Sec. 3.1's training-dynamics figure */
  double mean_abs_dp;    /* mean |pi_train(x_t) - pi_roll(x_t)|, the E|Delta p| of the same figure   */
  int status;            /* the context's status word at the time of the call                 */
  int reserved;
} ais_diag;

/* ---- context ------------------------------------------------------------------------------ */

/* Creates a context on GPU `device` that launches on `hip_stream` (a hipStream_t; NULL = the
 * default stream).  *out is host memory.  Allocates a small device workspace.  Device indices
 * of 64 and above are rejected with AIS_ERR_SIZE. */
int ais_create(ais_ctx** out, int device, void* hip_stream);
/* Waits for the context's stream, frees the workspace.  NULL is allowed. */
int ais_destroy(ais_ctx* ctx);
/* Changes the stream later calls launch on. */
int ais_set_stream(ais_ctx* ctx, void* hip_stream);
/* Writes the paper's defaults into *p (host memory). */
void ais_params_default(ais_params* p);
/* Static, NUL-terminated description of an ais_error. */
const char* ais_strerror(int err);
/* hipError_t of the last failing HIP call on this context (0 if none). */
int ais_last_hip_error(const ais_ctx* ctx);
/* Waits for the stream, copies the device status word to *host_out, and clears it if `clear`. */
int ais_status(ais_ctx* ctx, int* host_out, int clear);
/* Library version, major * 1000 + minor. */
int ais_version(void);

/* ---- the three calls of the path ------------------------------------------------------------ */

/* log pi_train(o_t): one streaming pass over each valid row (Alg. 1, "Compute full-precision
 * log-probs ... for all generated tokens").
 *   logits      [n_rows, row_stride] of `dtype`; read once; rows with valid == 0 are not read
 *   token_ids   [n_rows] sampled token per row; ignored (never read) where valid == 0
 *   logp_out    [n_rows] fp32  inv_temperature * z[n, y_n] - lse_n;  0 where valid == 0
 *   lse_out     [n_rows] fp32  log sum_v exp(inv_temperature * z[n, v]);  0 where valid == 0
 * Any vocab >= 1 and any row_stride >= vocab are accepted; 16-byte vector loads are used when
 * the base pointer and the row pitch allow it, an element-wise path otherwise.
 * Errors: NULL logits/token_ids/logp_out/lse_out (with n_rows > 0), n_rows < 0, vocab < 1,
 * vocab >= 2^31, row_stride < vocab, inv_temperature <= 0 or not finite, unknown dtype,
 * logits not aligned to its element size. */
int ais_token_logprob(ais_ctx* ctx, const void* logits, ais_dtype dtype, long long n_rows,
                      long long vocab, long long row_stride, const int* token_ids,
                      const unsigned char* valid, float inv_temperature, float* logp_out,
                      float* lse_out);

/* Ratios, diagnostics and alpha (Alg. 1, "Sampler-Trainer ratio" to "Bilateral gating";
 * Eq. 7, 10, 12-17), plus the group-relative advantages (Eq. 3).
 *   logp_train, logp_roll  [n_rows] fp32
 *   cu_rows     [n_resp + 1] int64 row offsets of the responses
 *   rewards     [n_resp] fp32
 *   adv_out     [n_resp] fp32   A_i
 *   count_out   [n_resp] int32  |o_i| = number of valid rows of response i
 *   diag_out    one ais_diag in device memory
 * Errors: NULL pointers (valid may be NULL), n_rows < 0, n_resp < 1, group_size < 1,
 * n_resp % group_size != 0, C < 1, delta <= 0, gamma <= 0, eps_std < 0, alpha_override > 1,
 * adv_mode not in {0, 1}. */
int ais_diagnostics(ais_ctx* ctx, const float* logp_train, const float* logp_roll,
                    const unsigned char* valid, long long n_rows, const long long* cu_rows,
                    int n_resp, int group_size, const float* rewards, const ais_params* params,
                    float* adv_out, int* count_out, ais_diag* diag_out);

/* ais_diagnostics for callers that cannot allocate device memory: code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc.  Same arguments, same kernels and bit-identical results; the row tiling,
 * the ticket counter and the per-tile partials live in a static device array of AIS_STATIC_SCRATCH_BYTES that every
 * GPU the library runs on holds until the process ends, so the call allocates nothing, frees nothing and never
 * waits for the stream, whatever sizes came before.
 *   Limit      56 * (ceil(n_rows / 1024) + n_resp) + 4 * (n_resp + 2) bytes, each part rounded up to 256, must fit
 *              the array: e.g. 18 million rows in 512 responses, or 1 million rows in 16,000 responses.  Beyond
 *              that the call returns AIS_ERR_SCRATCH and launches nothing.
 *   Sharing    every call on one GPU, from any context, uses that GPU's one array (the kernels overwrite what they
 *              read, so earlier contents do not matter): calls that overlap in time on one GPU race, also across
 *              contexts and streams.  The row tiling it leaves behind is not reused by the calls that follow.
 * Errors: as ais_diagnostics, plus AIS_ERR_SCRATCH. */
#define AIS_STATIC_SCRATCH_BYTES (1 << 20)
int ais_diagnostics_static(ais_ctx* ctx, const float* logp_train, const float* logp_roll,
                           const unsigned char* valid, long long n_rows, const long long* cu_rows,
                           int n_resp, int group_size, const float* rewards, const ais_params* params,
                           float* adv_out, int* count_out, ais_diag* diag_out);

/* Loss and gradient (Alg. 1, "Advantage Rectification" and "Policy Update"; Eq. 18, 19).
 * The two ratios of Sec. 3.2 are kept apart: the sampler-trainer ratio is taken at the checkpoint theta_old that
 * generated the rollout, the old-new ratio between theta_old and the current parameters.  With
 * l_old = logp_old (logp_train if logp_old is NULL), w_bar = min(exp(l_old - logp_roll), C),
 * w_tilde = 1 + alpha (w_bar - 1) and rho_on = exp(logp_train - l_old) (1 if logp_old is NULL):
 *   loss = -(1/n_resp) sum_i (1/|o_i|) sum_{valid t in i}
 *              [ w_tilde min(rho_on A_i, clip(rho_on, 1 -+ clip_eps) A_i) - beta_kl k3_t ]
 *   dlogits[n, v] = g_n * inv_temperature * (softmax(inv_temperature z_n)_v - 1[v = y_n])
 * where g_n is the derivative of that row's term w.r.t. its log-probability (zero when the
 * clipped branch is the minimum), alpha / w_tilde / A being constants, and
 * k3 = exp(q) - q - 1, q = logp_ref - logp_train (used only if logp_ref != NULL and beta_kl > 0).
 *   logits, token_ids, valid, cu_rows   as above (the same arrays given to the first two calls)
 *   logp_train, lse   outputs of ais_token_logprob on the current logits;  adv, count, diag  outputs of
 *               ais_diagnostics (which, when logp_old is given, was fed logp_old as its logp_train: the
 *               diagnostics of Alg. 1 are taken at theta_old)
 *   logp_old, logp_ref   [n_rows] fp32 or NULL
 *   cu_rows     when this is the array (same pointer, sizes and stream) that the last ais_diagnostics call on the
 *               context was given, the row tiling that call left in the workspace is reused: the array must still
 *               hold the same values, and a HIP graph should capture the calls of a step together
 *   wtilde_out  [n_rows] fp32 (0 where valid == 0); may be NULL
 *   loss_out    one double in device memory
 *   dlogits     [n_rows, row_stride] of `dtype`, same pitch as logits; every element of the
 *               first `vocab` columns is written (0 on rows without gradient); bf16 results
 *               are rounded to nearest even.  May be the same buffer as `logits` (in place).
 * Errors: as for the first two calls. */
int ais_grpo_loss_grad(ais_ctx* ctx, const void* logits, ais_dtype dtype, long long n_rows,
                       long long vocab, long long row_stride, const int* token_ids,
                       const unsigned char* valid, const long long* cu_rows, int n_resp,
                       const float* logp_train, const float* lse, const float* logp_roll,
                       const float* logp_old, const float* logp_ref, const float* adv,
                       const int* count, const ais_diag* diag, const ais_params* params,
                       float* wtilde_out, double* loss_out, void* dlogits);

/* ---- one-sweep variant: unscaled gradient direction plus a per-row scale -------------------------- */

/* The mixing coefficient alpha enters the gradient of Eq. 19 only through one scalar per row:
 * dlogits[n, :] = g[n] * s[n, :] with s[n, v] = softmax(inv_temperature z_n)_v - 1[v = y_n].  This pair of
 * calls emits s in the same sweep that computes the log-probs, and g after the diagnostics, so that each
 * logits row is read from HBM once (2 e V bytes per token in total instead of 3 e V); a consumer such as
 * the LM-head backward folds g[n] into its own operands.
 *
 * ais_token_logprob_softmax_grad: as ais_token_logprob, and additionally
 *   sgrad_out  [n_rows, row_stride] of `dtype`: s on evaluated rows, 0 on the others; may be the same
 *              buffer as `logits` (in place).  Rows are held in the register file and LDS of one compute
 *              unit (up to 270,336 bf16 or 135,168 fp32 elements, 16-byte aligned); wider or unaligned
 *              rows are processed in two passes with the same results.
 * ais_grpo_row_scale: as ais_grpo_loss_grad without the logits; writes
 *   g_out      [n_rows] fp32: the derivative of the loss w.r.t. the row's log-probability times
 *              inv_temperature (0 on rows not evaluated or clipped away), so that g_out[n] * s[n, :] equals
 *              the dlogits of ais_grpo_loss_grad up to rounding
 *   wtilde_out, loss_out as in ais_grpo_loss_grad. */
int ais_token_logprob_softmax_grad(ais_ctx* ctx, const void* logits, ais_dtype dtype, long long n_rows,
                                   long long vocab, long long row_stride, const int* token_ids,
                                   const unsigned char* valid, float inv_temperature, float* logp_out,
                                   float* lse_out, void* sgrad_out);
int ais_grpo_row_scale(ais_ctx* ctx, const float* logp_train, const float* logp_roll, const float* logp_old,
                       const float* logp_ref, const unsigned char* valid, long long n_rows,
                       const long long* cu_rows, int n_resp, const float* adv, const int* count,
                       const ais_diag* diag, const ais_params* params, float* wtilde_out,
                       double* loss_out, float* g_out);

/* ---- the rollout-side FP8 perturbation (input generation on the device) ------------------------ */

/* Per-row FP8-E4M3 quantisation of logits: the symmetric scaling of Eq. 1 with the E4M3 value grid
 * (Sec. 2.1; OCP "fn" format, largest magnitude 448) in place of the integer grid:
 *   s_n = max_v |z[n, v]| / 448  (1 for an all-zero row),  code[n, v] = e4m3(z[n, v] / s_n)
 * rounded to nearest, ties to even, saturating; both divisions are correctly rounded fp32.
 *   codes_out  [n_rows, codes_stride] bytes, the first `vocab` of each row are written
 *   scale_out  [n_rows] fp32
 * Errors: as ais_token_logprob, plus codes_stride < vocab (AIS_ERR_STRIDE). */
int ais_fp8_quantize_rows(ais_ctx* ctx, const void* logits, ais_dtype dtype, long long n_rows,
                          long long vocab, long long row_stride, unsigned char* codes_out,
                          long long codes_stride, float* scale_out);

/* The other half of Eq. 1's round trip (Sec. 2.1): the rollout engine's view of the logits,
 *   out[n, v] = s_n * value(code[n, v])  in fp32, stored as `out_dtype` (bf16: rounded to nearest even).
 * Errors: NULL pointers, sizes, strides < vocab, unknown dtype, misaligned out. */
int ais_fp8_dequantize_rows(ais_ctx* ctx, const unsigned char* codes, long long codes_stride,
                            const float* scale, long long n_rows, long long vocab, void* out,
                            ais_dtype out_dtype, long long out_stride);

/* The rollout policy's log-probability of the sampled tokens under that perturbation:
 * logp_roll_out[n] = log softmax(z_r[n, :])[y_n] with z_r = dequantise(quantise(z)), computed without
 * materialising codes or z_r; 0 where valid == 0.  This is what the FP8 sampler would report for the
 * ratio of Alg. 1 ("Sampler-Trainer ratio").  Errors: as ais_token_logprob. */
int ais_fp8_rollout_logprob(ais_ctx* ctx, const void* logits, ais_dtype dtype, long long n_rows,
                            long long vocab, long long row_stride, const int* token_ids,
                            const unsigned char* valid, float* logp_roll_out);

/* ---- log-probabilities without materialised logits ------------------------------------------- */

/* log pi_train(o_t) (Alg. 1, "Compute full-precision log-probs ... for all generated tokens") taken
 * straight from the last hidden states and the output-embedding matrix of the policy:
 *   z[n, v] = sum_d hidden[n, d] * weight[v, d]   (bf16 inputs, fp32 accumulation on the matrix cores)
 *   logp_out[n] = inv_temperature * z[n, y_n] - lse_n,  lse_n = log sum_v exp(inv_temperature * z[n, v])
 * The [n_rows, vocab] logits are folded into a running (max, sum) per token as they are produced and
 * are never written to memory.
 *   hidden      [n_rows, hidden_stride] device, bf16; the first d_model entries of each row are read;
 *               rows with valid == 0 are neither read nor evaluated (the evaluated rows are gathered
 *               into blocks of 256, so the cost follows their number)
 *   weight      [vocab, weight_stride]  device, bf16; row v is the output embedding of token v
 *   token_ids   [n_rows] device; ignored where valid == 0
 *   logp_out, lse_out  [n_rows] device fp32; 0 where valid == 0; a row whose token id is outside
 *               [0, vocab) gets logp 0, its lse, and AIS_STATUS_BAD_TOKEN in the status word
 * Uses the context workspace (2 * chunks + 3 words per row, chunks <= 64); nothing is retained.
 * Errors: dtype other than AIS_BF16 (AIS_ERR_DTYPE); n_rows < 0, vocab < 1, d_model < 8 or not a
 * multiple of 8 (AIS_ERR_SIZE); a stride < d_model (AIS_ERR_STRIDE); NULL pointers; hidden or weight
 * not 16-byte aligned or a stride not a multiple of 8 elements (AIS_ERR_ALIGN); inv_temperature
 * <= 0 or not finite (AIS_ERR_PARAM). */
int ais_lm_head_logprob(ais_ctx* ctx, const void* hidden, long long hidden_stride, const void* weight,
                        long long weight_stride, ais_dtype dtype, long long n_rows, long long d_model,
                        long long vocab, const int* token_ids, const unsigned char* valid,
                        float inv_temperature, float* logp_out, float* lse_out);

/* Gradient of the loss with respect to the last hidden states and the output-embedding matrix, again without
 * materialised logits (Alg. 1, "Policy Update": the gradient of Eq. 19 reaches the model through the read-out).
 * With z = hidden weight^T, p = softmax(inv_temperature z) and the per-row coefficient c (zero where a row has
 * no gradient: not evaluated, zero advantage, clipped away):
 *   dlogits[n, v]  = c[n] (p[n, v] - 1[v = y_n])                      (never stored as a whole)
 *   dhidden[n, :]  = sum_v dlogits[n, v] weight[v, :]
 *   dweight[v, :]  = sum_n dlogits[n, v] hidden[n, :]
 * The vocabulary is walked in chunks: the logits of a chunk are recomputed on the matrix cores from the operands,
 * turned into dlogits (bf16) with the row's lse, and consumed at once by two library GEMMs (rocBLAS, fp32
 * accumulation and output); only [n_rows, chunk_vocab] dlogits exist at any time.
 *   hidden, weight, token_ids, dtype, strides   as for ais_lm_head_logprob; d_model a multiple of 32
 *   lse, logp   [n_rows] fp32, outputs of ais_lm_head_logprob for the same operands and temperature
 *   coeff       [n_rows] fp32, as written by ais_grpo_row_scale (its g_out: it carries inv_temperature)
 *   chunk_vocab vocabulary entries per chunk, a multiple of 256; 0 selects 8192.  The context workspace grows to
 *               2 * n_rows * chunk_vocab bytes.
 *   n_live_max  negative, or >= n_rows: every row goes through the recomputation and the GEMMs.  Otherwise a bound
 *               that the caller vouches for on the number of rows with coeff != 0 (for a masked-diffusion batch:
 *               the number of evaluated positions, which its loader knows): those rows are gathered on the device
 *               and recomputation and GEMMs run over n_live_max rows only, so the cost follows the rows that have
 *               a gradient.  If there are more such rows than n_live_max, the surplus rows are left out (their
 *               dhidden is 0 and they do not enter dweight) and AIS_STATUS_LIVE_OVERFLOW is set; nothing is read
 *               or written out of range.  The workspace then holds 2 n_live_max (chunk_vocab + 3 d_model) bytes
 *               and 9 bytes per row.
 *   dhidden_out [n_rows, d_model] fp32, contiguous; dweight_out [vocab, d_model] fp32, contiguous; both are
 *               overwritten.
 * Errors: as ais_lm_head_logprob; d_model not a multiple of 32 or chunk_vocab not a multiple of 256
 * (AIS_ERR_SIZE); a failing library call (AIS_ERR_HIP). */
int ais_lm_head_grad(ais_ctx* ctx, const void* hidden, long long hidden_stride, const void* weight,
                     long long weight_stride, ais_dtype dtype, long long n_rows, long long d_model,
                     long long vocab, const int* token_ids, const float* lse, const float* logp,
                     const float* coeff, float inv_temperature, long long chunk_vocab, long long n_live_max,
                     float* dhidden_out, float* dweight_out);

/* ---- measurement helpers -------------------------------------------------------------------- */

/* Kernels whose device time can be read back. */
typedef enum ais_kernel {
  AIS_K_LOGPROB = 0, AIS_K_DLOGITS = 1, AIS_K_COPY = 2, AIS_K_FP8_QUANT = 3, AIS_K_FP8_DEQUANT = 4,
  AIS_K_FP8_LOGPROB = 5, AIS_K_FUSED = 6, AIS_K_LM_HEAD = 7, AIS_K_LM_HEAD_GRAD = 8, AIS_K_COUNT_ = 9
} ais_kernel;

/* With `enable` != 0 every launch of the kernels above is bracketed by HIP events on the
 * context's stream; enabling also clears what was gathered before. */
int ais_profile(ais_ctx* ctx, int enable);
/* Waits for the stream; *total_ms (host) = summed event time of kernel `which`, *launches (host)
 * = number of launches measured since profiling was enabled. */
int ais_profile_read(ais_ctx* ctx, int which, float* total_ms, int* launches);
/* Plain device-to-device copy kernel of `bytes` bytes (a multiple of 16, both pointers 16-byte
 * aligned): the yardstick for achievable HBM bandwidth and for scaling hardware counters. */
int ais_copy(ais_ctx* ctx, void* dst, const void* src, long long bytes);

#ifdef __cplusplus
}
#endif
#endif /* AIS_H_ */
