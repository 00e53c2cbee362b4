/*
 * jd_verify.h - C ABI of the batched verification head of Judge Decoding
 * (arXiv 2501.19309) for AMD MI355X (gfx950).
 *
 * One call verifies, for B independent sequences, M drafted tokens against the
 * target model's final-layer embeddings of the M+1 positions [s_L, c_1, ..., c_M]
 * (Fig. 4, right):
 *
 *   1. LM head: L[b,r,:] = (x[b,r,:] . W_lm) / T, p_{r+1} = softmax(L[b,r,:])   (Sec. 3.1, Eq. 2)
 *   2. draft probabilities q_{j+1}[c_{j+1}] from the draft tensor                 (Sec. 3.1, Eq. 3)
 *   3. standard test   z_stand[j] = ( eps_j * q[c] < p[c] )                       (Sec. 3.1, Eq. 4)
 *      (or, under JD_RULE_TOPK, c among the top_k most probable tokens of p       Sec. 5)
 *   4. judge test      z_judge[j] = ( w_judge . e[b,j+1,:] + bias > logit(delta) )
 *      i.e. sigmoid(f_judge(e)) > delta on the embedding of the judged token      (Sec. 4.1; App. B.1)
 *   5. z = z_stand OR z_judge                                                     (Sec. 4.1, "Inference")
 *   6. accept_len = number of leading ones of z                                   (Eq. 4; App. B.2, Fig. 8)
 *   7. next_token: inverse-CDF draw from norm(max(0, p - q)) of the first rejected
 *      position, or from p_{M+1} when all M were accepted                         (Sec. 3.1, after Eq. 4)
 *
 * Index convention (0-based): slot j holds the paper's c_{j+1}, q_{j+1}, eps_{j+1};
 * its standard test reads LM-head row j, its judge test reads embedding row j+1.
 *
 * All tensor arguments are DEVICE pointers owned by the caller and only borrowed:
 * w_judge (and the weight scales) for the lifetime of the context, W_lm for the lifetime of the
 * context if it is fp32 and only until create returns otherwise, everything else for the call.
 * Tensors are dense, row-major, last index contiguous.  Work is enqueued on the
 * caller's HIP stream and NOT synchronised; outputs are valid once the stream has
 * reached the end of the call.  jd_verify_create makes config.device the calling
 * thread's current device; for every later call on the context the calling thread's
 * current device must be that device and the stream must belong to it (the library does
 * not switch devices on the caller's behalf).  A context is not thread-safe; distinct
 * contexts are independent.  No function throws; every function returns 0 (JD_OK) or a negative
 * JD_ERR_* code, and jd_verify_strerror() names it.
 */
#ifndef JD_VERIFY_H
#define JD_VERIFY_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* ---- error codes ---------------------------------------------------------------- */
#define JD_OK                     0
#define JD_ERR_INVALID_ARG       -1   /* NULL pointer, bad enum, delta outside [0.5,1], T <= 0 ...   */
#define JD_ERR_SHAPE             -2   /* B/M beyond the context's maxima, M > 63, d % 8 != 0 ...      */
#define JD_ERR_UNSUPPORTED_DTYPE -3   /* dtype combination the kernels do not cover                   */
#define JD_ERR_OOM               -4   /* workspace allocation failed                                  */
#define JD_ERR_HIP               -5   /* a HIP runtime call failed (no device, launch failure)        */

/* ---- enums ----------------------------------------------------------------------- */
#define JD_F32   0                    /* IEEE binary32                                                */
#define JD_BF16  1                    /* bfloat16, 2 bytes                                            */
#define JD_FP8_E4M3 2                 /* W_lm only: OCP FP8 E4M3 ("e4m3fn") codes, 1 byte, with one   */
                                      /* fp32 scale per vocabulary entry (jd_verify_create_scaled);   */
                                      /* the paper runs its targets with 8-bit weights (Table 1)      */
#define JD_INT8  3                    /* W_lm only: two's-complement 8-bit integers, 1 byte, with one */
                                      /* fp32 scale per vocabulary entry (weight-only quantisation    */
                                      /* with per-output-channel scales; jd_verify_create_scaled)     */

#define JD_W_VD  0                    /* W_lm stored [V][d]: row v = vocabulary entry v (checkpoint)  */
#define JD_W_DV  1                    /* W_lm stored [d][V]                                           */

#define JD_DRAFT_LOGITS 0             /* draft tensor = fp32 logits; q = softmax at temperature 1     */
#define JD_DRAFT_PROBS  1             /* draft tensor = the probability vectors q_i themselves        */

#define JD_MODE_JUDGE    0            /* z = z_stand OR z_judge (Sec. 4.1)                            */
#define JD_MODE_STANDARD 1            /* z = z_stand (plain speculative sampling, Eq. 4)              */

#define JD_RULE_SAMPLING 0            /* z_stand by Eq. 4; new token by inverse CDF (residual / bonus) */
#define JD_RULE_TOPK     1            /* z_stand = c is among the top_k most probable tokens of p      */
                                      /* (Sec. 5 training-free baseline; top_k = 1 is the greedy      */
                                      /* matching of Sec. 3.2); new token = argmax p, lowest id on ties */

#define JD_RESAMPLE_RESIDUAL 0        /* replacement drawn from norm(max(0, p - q))                   */
#define JD_RESAMPLE_TARGET   1        /* replacement drawn from p itself (literal Sec. 3.1 wording)   */

/* per-sequence status bits written to d_status */
#define JD_STATUS_BAD_TOKEN     1u    /* a draft token id outside [0,V): that slot is rejected        */
#define JD_STATUS_NAN           2u    /* NaN met in target logits, a draft row or a judge logit       */
#define JD_STATUS_ZERO_RESIDUAL 4u    /* max(0,p-q) had no mass; next_token was drawn from p instead  */

/* kernels whose durations jd_verify_profile_end() reports */
#define JD_K_LMHEAD    0              /* LM-head contraction + per-tile softmax partials              */
#define JD_K_DRAFTSTAT 1              /* draft-logit row statistics                                   */
#define JD_K_ACCEPT    2              /* second softmax pass, judge, the two accept tests per slot    */
#define JD_K_SAMPLER   3              /* mask OR, ballot, accepted prefix, inverse-CDF sampler        */
#define JD_NUM_KERNELS 4

typedef struct jd_verify_ctx jd_verify_ctx;   /* opaque, owned by the library */

typedef struct {
  int32_t d, V;                 /* hidden size, vocabulary size                                       */
  int32_t max_B, max_M;         /* workspace is sized for these; 1 <= max_M <= 63                     */
  int32_t w_dtype, emb_dtype;   /* JD_F32 | JD_BF16, equal; or w_dtype JD_FP8_E4M3 | JD_INT8 with emb_dtype JD_BF16 */
                                /* (w_judge always has emb_dtype)                                      */
  int32_t w_layout;             /* JD_W_VD | JD_W_DV                                                  */
  int32_t draft_kind;           /* JD_DRAFT_LOGITS | JD_DRAFT_PROBS                                   */
  int32_t mode;                 /* JD_MODE_JUDGE | JD_MODE_STANDARD                                   */
  float   temperature;          /* target softmax temperature T > 0                                   */
  float   delta;                /* judge threshold in [0.5, 1]; 1 never accepts (reduces to Eq. 4)    */
  float   judge_bias;           /* scalar added to w_judge . e                                        */
  int32_t device;               /* HIP device ordinal                                                 */
  int32_t rule;                 /* JD_RULE_SAMPLING | JD_RULE_TOPK                                    */
  int32_t top_k;                /* 1 <= top_k <= V, read only under JD_RULE_TOPK                      */
  int32_t resample;             /* JD_RESAMPLE_RESIDUAL | JD_RESAMPLE_TARGET (JD_RULE_SAMPLING only)  */
} jd_verify_config;

typedef struct {                /* device pointers; the first three are required, NULL skips the rest */
  int32_t*  d_accept_len;       /* [B]        m*: accepted draft tokens, 0..M                         */
  int32_t*  d_next_token;       /* [B]        replacement (m* < M) or bonus (m* == M) token           */
  uint32_t* d_status;           /* [B]        JD_STATUS_* bits                                        */
  uint8_t*  d_z_stand;          /* [B, M]     per-slot standard test, not prefix-conditioned          */
  uint8_t*  d_z_judge;          /* [B, M]     per-slot judge test                                     */
  float*    d_p_at_draft;       /* [B, M]     p_{j+1}[c_{j+1}]                                        */
  float*    d_q_at_draft;       /* [B, M]     q_{j+1}[c_{j+1}]                                        */
  float*    d_judge_logit;      /* [B, M]     w_judge . e[b, j+1] + bias                              */
  float*    d_row_max;          /* [B, M+1]   max_v L[b,r,v]                                          */
  float*    d_row_sumexp;       /* [B, M+1]   sum_v exp(L[b,r,v] - max)                               */
  float*    d_probs;            /* [B, M+1, V] full softmax (debug / parity; costs an extra pass)     */
} jd_verify_outputs;

/*
 * Create a context (Sec. 3.1 / 4.1 fix the operands: W_lm, f_judge, delta).
 * Validates cfg, selects the device, allocates the workspace (fp32 logits
 * [max_B*(max_M+1), V], reduction partials) and, for bf16 weights, builds a private
 * copy of W_lm re-tiled into MFMA operand order (one extra W_lm-sized allocation,
 * one-time cost).  d_w_judge must stay valid and unchanged until destroy.  d_W_lm likewise for
 * JD_F32 weights, which are read in place by every call; for JD_BF16 / JD_FP8_E4M3 / JD_INT8 the
 * library works from its own copies only, create has finished reading d_W_lm when it returns, and
 * the caller may release or overwrite it then (a 405B-sized head need not be held twice).
 * Errors: INVALID_ARG, SHAPE, UNSUPPORTED_DTYPE (checked before any HIP call), OOM, HIP (also when
 * cfg->device is not a gfx950 device: the library holds code for that architecture only).
 * On error *out_ctx is set to NULL; jd_verify_last_error_detail() says which runtime call failed.
 */
int jd_verify_create(const jd_verify_config* cfg, const void* d_W_lm, const void* d_w_judge,
                     jd_verify_ctx** out_ctx);

/*
 * Same as jd_verify_create for quantised weights (w_dtype JD_FP8_E4M3 or JD_INT8; the paper's targets run
 * with 8-bit weights, Table 1 / App. B.3): the effective LM head is W[v,:] = d_w_scale[v] * decode(code[v,:]).
 *   d_w_scale   [V] fp32 device pointer, borrowed for the lifetime of the context (every call reads it);
 *               NULL means all ones.
 *               Must be NULL for JD_F32 / JD_BF16 weights (INVALID_ARG otherwise).
 * The library builds a re-tiled copy of the codes (V*d bytes) and, for max_B*(max_M+1) > 176, a second one in the
 * fragment order of the 352-row kernel (another V*d bytes).  No bf16 copy is held: every kernel turns the codes into
 * bf16 exactly, in registers, on their way to the matrix cores.
 * d must be a multiple of 16.  Other errors as jd_verify_create.
 */
int jd_verify_create_scaled(const jd_verify_config* cfg, const void* d_W_lm, const float* d_w_scale,
                            const void* d_w_judge, jd_verify_ctx** out_ctx);

/*
 * Verify one batch (steps 1-7 above).  1 <= B <= max_B, 1 <= M <= max_M.
 *   d_emb          [B, M+1, d]   LM-head input, emb_dtype
 *   d_emb_judge    [B, M+1, d]   judge input (the paper's judge reads the embedding before the
 *                                final RMS norm, Sec. 4.1); NULL means use d_emb.  Row 0 is unused.
 *   d_draft_tokens [B, M]        int32 ids in [0, V)
 *   d_draft        [B, draft_rows, V] fp32 logits or probabilities (per draft_kind)
 *   draft_rows     M or M+1 (a trailing row is ignored)
 *   d_uniforms     [B, M+1]      fp32 in [0,1): M accept draws eps, then the sampler draw
 *   out            struct of device output pointers (see above)
 *   hip_stream     hipStream_t to enqueue on (NULL = the default stream)
 * Never allocates, never synchronises, never reads tensor contents on the host.
 * Errors: INVALID_ARG (NULL ctx / required pointer), SHAPE, HIP.
 */
int jd_verify_run(jd_verify_ctx* ctx, int32_t B, int32_t M,
                  const void* d_emb, const void* d_emb_judge,
                  const int32_t* d_draft_tokens, const float* d_draft, int32_t draft_rows,
                  const float* d_uniforms, const jd_verify_outputs* out, void* hip_stream);

/*
 * The same call in the paper's own wiring (Sec. 4.1, "Model design and training": the judge is
 * trained on the target's last embedding BEFORE the final RMS normalisation, the LM head reads
 * it after).  The caller hands over the pre-norm hidden states once; the library normalises them
 * for the LM head and feeds them as they are to the judge:
 *   x[r, k] = round( h[r, k] * gamma[k] / sqrt(mean_k(h[r, k]^2) + rms_eps) )
 * computed in float64 and rounded once, to nearest even, to emb_dtype (the rounded tensor is what
 * the LM head multiplies; it lives in the context's workspace and is overwritten by every call).
 *   d_hidden       [B, M+1, d]   pre-norm hidden states, emb_dtype; also the judge input
 *   d_gamma        [d]           gain of the normalisation, emb_dtype
 *   rms_eps        >= 0, finite  added to the mean square
 * Everything else, and the error behaviour, as for jd_verify_run; INVALID_ARG also for a NULL
 * d_gamma or an rms_eps that is negative or not finite.
 */
int jd_verify_run_prenorm(jd_verify_ctx* ctx, int32_t B, int32_t M,
                          const void* d_hidden, const void* d_gamma, double rms_eps,
                          const int32_t* d_draft_tokens, const float* d_draft, int32_t draft_rows,
                          const float* d_uniforms, const jd_verify_outputs* out, void* hip_stream);

/*
 * The step after a verify call (Sec. 3.1, end of the paragraph after Eq. 4: the accepted tokens and
 * the one new token are added to the context), stream-ordered so that a decode loop needs no host
 * synchronisation between calls.  For each sequence b, with n = d_accept_len[b] in [0, M]:
 *   d_token_buf[b, len .. len+n-1] = d_draft_tokens[b, 0 .. n-1];  d_token_buf[b, len+n] = d_next_token[b];
 *   d_lengths[b] = len + n + 1,                         where len = d_lengths[b] before the call.
 * Tokens that would land at or beyond `cap` are dropped and the length saturates at cap; an
 * accept_len outside [0, M] is clamped into it.
 *   d_draft_tokens [B, M] int32, d_accept_len [B] int32, d_next_token [B] int32  (inputs, device)
 *   d_token_buf    [B, cap] int32, d_lengths [B] int32                          (updated in place, device)
 * Stateless: needs no context, allocates nothing, does not synchronise.
 * Errors: INVALID_ARG (NULL pointer), SHAPE (B < 1, M < 1, cap < 1), HIP.
 */
int jd_verify_append_tokens(int32_t B, int32_t M, const int32_t* d_draft_tokens, const int32_t* d_accept_len,
                            const int32_t* d_next_token, int32_t* d_token_buf, int32_t cap, int32_t* d_lengths,
                            void* hip_stream);

/*
 * jd_verify_run for callers that cannot allocate device memory: code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc.  No context: the workspace that jd_verify_create would allocate
 * (fp32 logits [B*(M+1), V rounded up to 64], reduction partials, row statistics, sampler chunk masses) lives in
 * a static device array of JD_NOALLOC_SCRATCH_BYTES bytes inside the library, which every device that loads
 * the library holds until the process ends.  The call allocates and frees nothing, on the device or through
 * any library, and does not synchronise.
 *   cfg            as for jd_verify_create; w_dtype and emb_dtype must both be JD_F32, the one weight type the
 *                  LM head multiplies in place from the caller's tensor (bf16 and 8-bit weights run from a
 *                  re-tiled copy that only a context can hold: UNSUPPORTED_DTYPE).  max_B / max_M only bound
 *                  B and M here; cfg->device must be the calling thread's current device (INVALID_ARG).
 *   d_W_lm, d_w_judge   device pointers as for jd_verify_create, borrowed for the call only
 *   everything else as for jd_verify_run.
 * Limit: the workspace of the call must fit the array - roughly 4 * B*(M+1) * (V+63)/64*64 bytes plus 256 KiB,
 * e.g. 26 rows at V = 128256, or 704 rows at V = 5000; beyond it the call returns JD_ERR_SHAPE and
 * jd_verify_last_error_detail() gives the two sizes.  Nothing in the array needs to start at zero: every
 * kernel writes what later kernels of the same call read.  All calls on one device share that device's
 * array, so two calls that overlap in time on one device (two streams, two threads) race; calls on one
 * stream, or otherwise ordered, are safe, and so are calls on different devices.  The first call on a device
 * looks up the array's device address (hipGetSymbolAddress); make that call, or create any context on the
 * device, before capturing.  Errors otherwise as for jd_verify_create (host-side checks) and jd_verify_run.
 */
#define JD_NOALLOC_SCRATCH_BYTES (16u << 20)
int jd_verify_run_noalloc(const jd_verify_config* cfg, const void* d_W_lm, const void* d_w_judge,
                          int32_t B, int32_t M, const void* d_emb, const void* d_emb_judge,
                          const int32_t* d_draft_tokens, const float* d_draft, int32_t draft_rows,
                          const float* d_uniforms, const jd_verify_outputs* out, void* hip_stream);

/* Free the workspace and the context.  destroy(NULL) is a no-op returning JD_OK.
 * Caller memory is never freed. */
int jd_verify_destroy(jd_verify_ctx* ctx);

/* Static, NUL-terminated description of an error code. */
const char* jd_verify_strerror(int code);

/* For JD_ERR_HIP / JD_ERR_OOM: which HIP call failed last in the calling thread and what the
 * runtime said ("" if none yet).  Thread-local storage owned by the library, overwritten by the
 * next failure in the same thread. */
const char* jd_verify_last_error_detail(void);

/*
 * Per-kernel timing with HIP events on the stream passed to jd_verify_run.
 * profile_begin arms the context: each of the next max_calls runs records an event
 * before and after every kernel group.  profile_end synchronises on those events,
 * writes the mean duration in milliseconds of each JD_K_* group into
 * avg_ms[JD_NUM_KERNELS] (host pointer) and the number of profiled runs into *n_calls
 * (host pointer), and disarms the context.  Errors: INVALID_ARG, HIP.
 */
int jd_verify_profile_begin(jd_verify_ctx* ctx, int32_t max_calls);
int jd_verify_profile_end(jd_verify_ctx* ctx, float* avg_ms, int32_t* n_calls);

/*
 * Introspection (host pointers): bytes of device memory the context allocated
 * (workspace + re-tiled weights), and the vocabulary stride of the fp32 logits scratch.
 */
int jd_verify_workspace_bytes(const jd_verify_ctx* ctx, uint64_t* out_bytes);

/* Host-only validation of a config, exactly the checks create performs before touching
 * the device.  Lets callers (and CPU-only tests) probe argument errors without a GPU. */
int jd_verify_validate_config(const jd_verify_config* cfg);

/*
 * Two measurements of the device itself, for reading roofline fractions (the bound the north-star
 * targets are stated against: HBM for the B = 1 shapes, the matrix cores for the batched one).  Not
 * part of verification.  Both make `device` current, allocate and free their own buffers, run on the
 * default stream and synchronise; out_* are host pointers.
 *   jd_verify_probe_mfma_bf16: TFLOP/s that a loop of nothing but independent
 *       v_mfma_f32_16x16x32_bf16 sustains on all compute units (no memory traffic), i.e. what
 *       the matrix cores deliver at the clock the board grants them.  operand_mode 0: all-zero
 *       operands; 1: values spread like N(0,1), as embeddings and weights are (lower: the power
 *       drawn, hence the clock, depends on the data); 2: the same N(0,1)-like loop on the other bf16
 *       shape, v_mfma_f32_32x32x16_bf16 (the comparison behind the kernels' 16 x 16 tiles).
 *   jd_verify_probe_hbm_read: GB/s of a pure streaming read (128-bit non-temporal loads, grid stride) of a
 *       zero-filled buffer of `bytes` bytes, 1 MiB <= bytes <= 64 GiB (use >= 2 GiB: smaller buffers
 *       measure the last-level cache).  jd_verify_probe_hbm_read_plain: the same kernel with plain (temporal)
 *       loads, which reach about an eighth less on this chip - the reason the library reads everything it reads
 *       once per launch non-temporally.
 * Errors: INVALID_ARG (NULL pointer, mode, size), OOM, HIP.
 */
int jd_verify_probe_mfma_bf16(int32_t device, int32_t operand_mode, double* out_tflops);
int jd_verify_probe_hbm_read(int32_t device, uint64_t bytes, double* out_gbs);
int jd_verify_probe_hbm_read_plain(int32_t device, uint64_t bytes, double* out_gbs);

#ifdef __cplusplus
}
#endif
#endif /* JD_VERIFY_H */
