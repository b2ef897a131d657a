/*
 * atts.h -- C ABI of the ATTS verification + conformal hot path for AMD MI355X (gfx950).
 *
 * The library implements, as hand-written HIP kernels, the data-parallel part of
 * "ATTS: Asynchronous Test-Time Scaling via Conformal Prediction":
 *
 *   atts_score_drafts      the "Verification" stage of the three-stage rejection sampling
 *                          pipeline: the target model teacher-forces m = K draft
 *                          continuations that share one prompt prefix and turns the
 *                          per-token log-probabilities into one unnormalised conformity
 *                          score per draft (Sec. "Q2", paragraph "Online Calibration",
 *                          the equation defining s = -l(X, Y)).
 *   atts_calibrate_online  "Online Calibration": the calibration multiset grows by the
 *                          scores of newly pre-sampled outputs.
 *   atts_classify_ordinal  the marginal conformal p-value of Eq. "p-value" /
 *                          Proposition 1 for each test score, the accept rule p > alpha of
 *                          Eq. "prediction_set", generalised to several ascending levels
 *                          (ordinal classes), and the classic conformal quantile of
 *                          Eq. "quantile".
 *
 * Conventions
 *   - Every function returns an int32_t status: ATTS_OK (0) or a negative ATTS_ERR_*.
 *     atts_last_error_string() gives the detail for the calling thread's last failure.
 *     No exception crosses this boundary.
 *   - "dev" pointers are device (HBM) addresses on the current HIP device; "host"
 *     pointers are ordinary host memory.  The caller owns every buffer it passes in.
 *     The library owns only what its opaque handles hold.
 *   - hip_stream is a hipStream_t passed as void* (NULL = the default stream).  All
 *     device work is enqueued on that stream and the call returns without
 *     synchronising.  Argument errors that can be detected on the host are reported
 *     before anything is enqueued.
 *   - Matrices are row-major.  Weight matrices are [out_features, in_features].
 *   - There is no CPU fallback: every entry point needs a gfx950 device.
 */
#ifndef ATTS_H
#define ATTS_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define ATTS_OK                 0
#define ATTS_ERR_INVALID_ARG   (-1)  /* NULL pointer, value out of range                   */
#define ATTS_ERR_SHAPE         (-2)  /* model / call shape the kernels do not support      */
#define ATTS_ERR_WORKSPACE     (-3)  /* workspace missing, misaligned or too small         */
#define ATTS_ERR_CAPACITY      (-4)  /* calibration set would exceed its capacity          */
#define ATTS_ERR_HIP           (-5)  /* a HIP runtime call failed                          */

#define ATTS_DTYPE_F32   0   /* matrices and activations in fp32 (fp32 MFMA)              */
#define ATTS_DTYPE_BF16  1   /* matrices and activations in bf16, fp32 accumulation       */

#define ATTS_SCORE_MEAN_NLL 0   /* s_k = -(1/T_k) sum_t log q_t(y_t | ...)  (log-perplexity) */
#define ATTS_SCORE_SUM_NLL  1   /* s_k = -sum_t log q_t(y_t | ...)                           */

#define ATTS_MAX_ALPHAS 8

typedef struct atts_model atts_model;   /* opaque: target-model description + weight pointers */
typedef struct atts_calib atts_calib;   /* opaque: online calibration multiset (device)       */

/* Target model q_t: a pre-norm decoder with RMSNorm, rotate-half rotary embedding,
 * grouped-query causal attention, SwiGLU feed-forward, untied LM head, no biases.
 * (The paper leaves the architecture to the served model; this is the family of the
 * targets it evaluates.) */
typedef struct {
    int32_t n_layers;
    int32_t d_model;
    int32_t n_q_heads;
    int32_t n_kv_heads;     /* divides n_q_heads                                       */
    int32_t head_dim;       /* even, <= 256                                            */
    int32_t d_ffn;
    int32_t vocab;
    int32_t dtype;          /* ATTS_DTYPE_*: element type of every matrix below        */
    float   rope_theta;
    float   rms_eps;
} atts_model_desc;

/* Device pointers, BORROWED: they must stay valid while the model handle is used.
 * The per-layer entries are HOST arrays of n_layers device pointers (copied at create).
 * Norm gains are always fp32 vectors; matrices have element type desc.dtype. */
typedef struct {
    const void*        tok_embed;   /* dev [vocab, d_model]                              */
    const float*       final_norm;  /* dev [d_model]                                     */
    const void*        lm_head;     /* dev [vocab, d_model]                              */
    const float* const* attn_norm;  /* host[L] -> dev [d_model]                          */
    const void*  const* wqkv;       /* host[L] -> dev [(n_q + 2 n_kv) head_dim, d_model] : q | k | v rows */
    const void*  const* wo;         /* host[L] -> dev [d_model, n_q head_dim]            */
    const float* const* ffn_norm;   /* host[L] -> dev [d_model]                          */
    const void*  const* w_gate_up;  /* host[L] -> dev [2 d_ffn, d_model] : gate rows, then up rows */
    const void*  const* w_down;     /* host[L] -> dev [d_model, d_ffn]                   */
} atts_weights;

/* Text of the calling thread's most recent error ("" if none).  Never NULL. */
const char* atts_last_error_string(void);

/* ------------------------------------------------------------------------------------
 * Target model handle
 * ---------------------------------------------------------------------------------- */

/* Validates the description (ATTS_ERR_INVALID_ARG / ATTS_ERR_SHAPE) and records the weight
 * pointers.  Allocates a 4-byte device error flag; no weights are copied. */
int32_t atts_model_create(const atts_model_desc* desc, const atts_weights* weights, atts_model** out);
int32_t atts_model_destroy(atts_model* model);

/* Bytes of device workspace atts_score_drafts needs for a prefix of P tokens and K drafts
 * of at most T_max tokens. */
int32_t atts_workspace_bytes(const atts_model* model, int32_t P, int32_t K, int32_t T_max, size_t* out_bytes);

/* Verification ("How to perform rejection sampling via conformal prediction", paragraph
 * "Verification"; score: Sec. "Q2", "Online Calibration").
 *
 * Runs the target model once over the token tree  prefix -> K drafts  (each draft row
 * attends to the whole prefix and causally to its own draft; the prefix is computed once
 * and shared) and returns, for draft k and token t < len_k,
 *     token_logprobs[k, t] = log q_t(y^k_t | x_0..x_{P-1}, y^k_0..y^k_{t-1})
 * (y^k_0 is predicted from the last prefix position) and the conformity score
 *     scores[k] = -(1/len_k) sum_t token_logprobs[k, t]      (ATTS_SCORE_MEAN_NLL)
 *               = -          sum_t token_logprobs[k, t]      (ATTS_SCORE_SUM_NLL).
 * The [K T_max, vocab] logit matrix is never materialised.
 *
 *   prefix_ids      dev int32 [P], P >= 1
 *   draft_ids       dev int32 [K, T_max] row-major
 *   draft_lens      dev int32 [K], each in [1, T_max]; NULL = every draft has T_max tokens.
 *                   Positions t >= len_k are padding: their ids are ignored and their
 *                   token_logprobs are written as 0.
 *   token_logprobs  dev float [K, T_max], or NULL if only the scores are wanted
 *   scores          dev float [K]
 *   workspace       dev, 256-byte aligned, >= atts_workspace_bytes(...) bytes; contents
 *                   are scratch (nothing is kept between calls)
 *
 * A token id outside [0, vocab) (among the non-padding ids) does not fault: it is read as
 * id 0 and sets the model's sticky device error flag, see atts_model_check.
 * Results are bit-reproducible run to run: no floating-point atomics anywhere; calls with few rows through the model,
 * whose narrow projections split their inner dimension over workgroups, add the partial sums in a fixed order.
 * Host-detectable errors: NULL model/ids/scores, P < 1, K < 1, T_max < 1, bad score_mode,
 * P + T_max > 1048576 -> ATTS_ERR_INVALID_ARG; workspace -> ATTS_ERR_WORKSPACE. */
int32_t atts_score_drafts(const atts_model* model,
                          const int32_t* prefix_ids, int32_t P,
                          const int32_t* draft_ids, const int32_t* draft_lens,
                          int32_t K, int32_t T_max, int32_t score_mode,
                          float* token_logprobs, float* scores,
                          void* workspace, size_t workspace_bytes, void* hip_stream);

/* ------------------------------------------------------------------------------------
 * Prefix handle: a prompt prefix prefilled once and reused across turns
 *
 * In the turn loop of the method (Sec. "How to perform rejection sampling via conformal prediction": sampling,
 * verification, continuation, repeated) every turn's drafts continue the same context, and an accepted
 * continuation becomes part of it; the serving engine the paper builds on keeps that context's keys and values
 * instead of recomputing them.  The handle holds, per layer, the keys (after RoPE) and values of the prefix rows
 * in the layouts the attention kernels read, plus the hidden state of the last row (the state that predicts the
 * first token of every draft).
 *
 *   atts_prefix_create          an empty prefix that can grow to `capacity` rows (allocates device memory:
 *                               2 L capacity n_kv head_dim elements of the model dtype)
 *   atts_prefix_extend          runs the target model over n more tokens that continue the prefix (plain causal
 *                               attention over the cached rows and themselves) and appends their keys / values;
 *                               the first call on an empty handle is the prefill of the prompt.  ids dev int32 [n].
 *                               Workspace as atts_prefix_extend_workspace_bytes says (scratch, nothing kept).
 *                               ATTS_ERR_CAPACITY if length + n > capacity (nothing is changed).
 *   atts_score_drafts_cached    atts_score_drafts with the handle in place of (prefix_ids, P): only the K T_max
 *                               draft rows go through the model; same outputs, same workspace size as
 *                               atts_workspace_bytes(model, length, K, T_max).  The handle is not modified.
 *   atts_prefix_length / reset  rows held / forget them (capacity and memory are kept)
 * The handle borrows the model (which must outlive it).  Calls that touch one handle must be ordered (one stream,
 * or externally synchronised).  Out-of-range token ids behave as in atts_score_drafts.
 * ---------------------------------------------------------------------------------- */
typedef struct atts_prefix atts_prefix;
int32_t atts_prefix_create(const atts_model* model, int32_t capacity, atts_prefix** out);
int32_t atts_prefix_destroy(atts_prefix* prefix);
int32_t atts_prefix_length(const atts_prefix* prefix, int32_t* out_rows);
int32_t atts_prefix_reset(atts_prefix* prefix);
int32_t atts_prefix_extend_workspace_bytes(const atts_prefix* prefix, int32_t n, size_t* out_bytes);
int32_t atts_prefix_extend(atts_prefix* prefix, const int32_t* ids, int32_t n, void* workspace, size_t workspace_bytes,
                           void* hip_stream);
int32_t atts_score_drafts_cached(const atts_prefix* prefix, const int32_t* draft_ids, const int32_t* draft_lens, int32_t K,
                                 int32_t T_max, int32_t score_mode, float* token_logprobs, float* scores, void* workspace,
                                 size_t workspace_bytes, void* hip_stream);

/* Target-model continuation of rejected candidates (Sec. "How to perform rejection sampling via conformal
 * prediction", paragraph "Target Model Sampling"): each of the K candidates keeps its draft as a prefix and the
 * target model generates n_new more tokens for it.  Decoding is greedy: out_ids[k][t] is the first arg max of the
 * target's next-token logits given prefix + draft k + out_ids[k][0 .. t - 1].  All K candidates advance together,
 * one row per candidate and step (the weight-streaming regime); their keys / values share the cached prefix.
 *   prefix      handle holding the shared context (length >= 1); not modified
 *   draft_ids   dev int32 [K, T] row-major, the rejected drafts
 *   draft_lens  dev int32 [K], each in [1, T] (values outside are read as clamped): candidate k continues after
 *               its first draft_lens[k] tokens, the rest of its row is padding; NULL = every draft has T tokens
 *   eos_id      >= 0: the end-of-sequence token; once a candidate has produced it, all its later out_ids are
 *               eos_id too (its rows keep going through the model with the others, their results are dropped);
 *               < 0: no such token
 *   out_ids     dev int32 [K, n_new] row-major
 *   workspace   dev, 256-byte aligned, >= atts_continue_workspace_bytes(prefix, K, T, n_new) bytes; scratch
 * 1 <= K <= 768, T >= 1, n_new >= 1, length + T + n_new <= 1048576.  Out-of-range ids as in atts_score_drafts.
 * When a head's row (head_dim elements of the model dtype) is not a power-of-two number of 16-byte pieces, the
 * decoding steps use a general attention kernel that holds one score per key in LDS: contexts beyond about 13,000
 * keys are then refused with ATTS_ERR_SHAPE. */
int32_t atts_continue_workspace_bytes(const atts_prefix* prefix, int32_t K, int32_t T, int32_t n_new, size_t* out_bytes);
int32_t atts_continue_greedy(const atts_prefix* prefix, const int32_t* draft_ids, const int32_t* draft_lens, int32_t K, int32_t T,
                             int32_t n_new, int32_t eos_id, int32_t* out_ids, void* workspace, size_t workspace_bytes,
                             void* hip_stream);
/* The same continuation with sampling instead of the arg max: out_ids[k][t] is drawn from
 * softmax(logits / temperature) by inverse CDF with the caller's uniform uniforms[k][t] in [0, 1): the first index v
 * (vocabulary order) whose cumulative probability reaches the uniform.  The random numbers are inputs, so a call
 * is a deterministic function of its arguments.  temperature > 0; uniforms dev float [K, n_new]. */
int32_t atts_continue_sample(const atts_prefix* prefix, const int32_t* draft_ids, const int32_t* draft_lens, int32_t K, int32_t T,
                             int32_t n_new, int32_t eos_id, float temperature, const float* uniforms, int32_t* out_ids,
                             void* workspace, size_t workspace_bytes, void* hip_stream);

/* Synchronises hip_stream, copies the sticky device error flag to *host_flag (0 = clean,
 * 1 = some token id was out of range since the last check) and clears it. */
int32_t atts_model_check(const atts_model* model, void* hip_stream, int32_t* host_flag);

/* ------------------------------------------------------------------------------------
 * Stand-alone stages of the scoring path (same kernels atts_score_drafts launches)
 * ---------------------------------------------------------------------------------- */

/* Fused LM head: lp[b] = z_b[target_b] - log sum_v exp(z_b[v]),  z_b = W x_b, without ever
 * storing z ("Verification": the logits of the target model are reduced to the log-
 * probability of the drafted token on the fly).
 *   x dev [B, d] (dtype), w dev [V, d] (dtype), targets dev int32 [B] in [0, V),
 *   logprobs dev float [B]; workspace >= atts_lmhead_workspace_bytes(B, V). */
int32_t atts_lmhead_workspace_bytes(int32_t B, int32_t V, size_t* out_bytes);
int32_t atts_lmhead_logprobs(int32_t dtype, const void* x, const void* w, const int32_t* targets,
                             int32_t B, int32_t d, int32_t V, float* logprobs,
                             void* workspace, size_t workspace_bytes, void* hip_stream);

/* atts_lmhead_logprobs for callers that cannot allocate device memory or bring a workspace (code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc): same arguments without the workspace, same kernels,
 * same results bit for bit.  The per-row partials live in a 16 MiB device array that is part of the library's code
 * object (every GPU the library runs on holds its own copy until the process ends); the call allocates nothing.
 * Limit: atts_lmhead_workspace_bytes(B, V) <= 16 MiB (about 880 rows at a 152,064-token vocabulary, 134,000 rows at
 * 1,000 tokens); beyond it ATTS_ERR_WORKSPACE is returned before anything is enqueued.  Every call on one GPU uses
 * that GPU's one array: calls that overlap in time on the same GPU (different streams or threads) race; order
 * them.  Nothing in the array has to be cleared between calls (every partial a call reads it has written). */
int32_t atts_lmhead_logprobs_static(int32_t dtype, const void* x, const void* w, const int32_t* targets,
                                    int32_t B, int32_t d, int32_t V, float* logprobs, void* hip_stream);

/* C[M, N] (fp32) = A[M, Kdim] . W[N, Kdim]^T  -- the MFMA GEMM every projection uses
 * (scoring is the compute-bound part of the method, Sec. "Q1").  Kdim * sizeof(dtype) must
 * be a multiple of 16 bytes. */
int32_t atts_gemm_nt(int32_t dtype, const void* a, const void* w, float* c,
                     int32_t M, int32_t N, int32_t Kdim, void* hip_stream);

/* Shared-prefix (token-tree) attention over rows  [prefix (P) | draft 0 (T) | ... | draft K-1 (T)].
 * Row r attends to prefix rows <= r, and, if it is a draft row, to all P prefix rows plus the
 * rows of its own draft up to itself ("shared-prefix mechanism", Introduction).
 *   qkv dev [R, (n_q + 2 n_kv) hd] (dtype), q and k already rotated; out dev [R, n_q hd] (dtype);
 *   workspace: >= atts_attention_workspace_bytes(...) (holds the transposed V). */
int32_t atts_attention_workspace_bytes(int32_t dtype, int32_t R, int32_t n_kv, int32_t hd, size_t* out_bytes);
int32_t atts_attention_shared_prefix(int32_t dtype, const void* qkv, void* out,
                                     int32_t P, int32_t K, int32_t T,
                                     int32_t n_q, int32_t n_kv, int32_t hd,
                                     void* workspace, size_t workspace_bytes, void* hip_stream);

/* ------------------------------------------------------------------------------------
 * Stage timing of atts_score_drafts (measurement aid, off by default, not thread-safe)
 *
 * While enabled, every kernel launch of atts_score_drafts is bracketed by a pair of HIP events
 * recorded on the caller's stream and attributed to one of the stages below (the steps of the
 * "Verification" forward pass).  atts_profile_read waits for the recorded events and returns
 * the accumulated device time and launch count of a stage since the last atts_profile_enable.
 * ---------------------------------------------------------------------------------- */
#define ATTS_STAGE_EMBED        0   /* embedding gather + rotary table                      */
#define ATTS_STAGE_NORM         1   /* the 2 L RMSNorms                                     */
#define ATTS_STAGE_GEMM_QKV     2
#define ATTS_STAGE_ROPE         3   /* rotary embedding (+ V transpose)                     */
#define ATTS_STAGE_ATTENTION    4   /* shared-prefix attention                              */
#define ATTS_STAGE_GEMM_O       5   /* output projection + residual                         */
#define ATTS_STAGE_GEMM_GATE_UP 6   /* gate/up projection + SiLU*up                         */
#define ATTS_STAGE_GEMM_DOWN    7   /* down projection + residual                           */
#define ATTS_STAGE_GATHER_NORM  8   /* scoring-row gather + final norm                      */
#define ATTS_STAGE_LMHEAD       9   /* fused LM head log-softmax-gather GEMM                */
#define ATTS_STAGE_REDUCE      10   /* partial combine + score reduction                    */
#define ATTS_STAGE_CALIB_SORT  11   /* atts_calibrate_online: sorting the new batch         */
#define ATTS_STAGE_CALIB_MERGE 12   /* atts_calibrate_online: merge into the resident array */
#define ATTS_STAGE_CLASSIFY    13   /* atts_classify_ordinal, atts_classify_conditional     */
#define ATTS_STAGE_COUNT       14

/* on != 0: start recording (clears earlier records); on == 0: stop and drop the records. */
int32_t atts_profile_enable(int32_t on);
/* total_ms / launches: accumulated over the launches of `stage` recorded so far (either may be NULL). */
int32_t atts_profile_read(int32_t stage, double* total_ms, int64_t* launches);

/* ------------------------------------------------------------------------------------
 * Online conformal calibration and ordinal classification
 * ---------------------------------------------------------------------------------- */

/* Creates an empty calibration multiset that can hold up to `capacity` scores
 * (1 <= capacity <= 2^30).  Allocates its device storage (about 16 bytes per score). */
int32_t atts_calib_create(int64_t capacity, atts_calib** out);
int32_t atts_calib_destroy(atts_calib* calib);
/* Number of scores currently in the multiset (host-side bookkeeping, exact). */
int32_t atts_calib_size(const atts_calib* calib, int64_t* out_n);
/* Empties the multiset (no device work). */
int32_t atts_calib_reset(atts_calib* calib);

/* Online calibration: D_cal <- D_cal U {new_scores}.
 *   new_scores dev float [n_new], n_new >= 0 (0 is a no-op).
 * ATTS_ERR_CAPACITY if size + n_new > capacity (nothing is changed).
 * The multiset is kept in sorted order on the device.  +-inf are ordinary values, -0 == +0,
 * a NaN calibration score is kept (it counts in N) but never compares ">=" to anything.
 * Calls on one handle must be ordered (one stream, or externally synchronised). */
int32_t atts_calibrate_online(atts_calib* calib, const float* new_scores, int64_t n_new, void* hip_stream);

/* Marginal conformal p-value ranks and ordinal classes for M test scores against the
 * multiset as it stands (N = its size, N >= 1):
 *     ranks[i]    = #{ j : test_scores[i] <= cal_j }                 (Eq. "p-value" numerator - 1)
 *     pvalues[i]  = (ranks[i] + 1) / (N + 1)                         (Eq. "p-value")
 *     r_l         = floor(alphas[l] * (N + 1))   in binary64          (p <= alpha_l  <=>  ranks + 1 <= r_l)
 *     classes[i]  = #{ l : ranks[i] + 1 <= r_l }                     (0 = accept: p > every alpha;
 *                                                                     with two levels 1 = resample,
 *                                                                     2 = target fallback)
 *     thresholds[l] = the (N + 1 - r_l)-th smallest calibration score (Eq. "quantile"),
 *                     +inf if r_l = 0, -inf if r_l > N; ranks[i] + 1 <= r_l  <=>  test > thresholds[l]
 * A NaN test score gets rank 0 (the smallest p-value).
 *   test_scores dev float [M] (M >= 0); alphas HOST double [n_alpha], non-decreasing, each in
 *   (0, 1), 1 <= n_alpha <= ATTS_MAX_ALPHAS; ranks dev int32 [M]; pvalues dev float [M] or
 *   NULL; classes dev uint8 [M]; thresholds dev float [n_alpha] or NULL.
 * ranks == NULL (then pvalues must be NULL too) asks for the decisions only: the classes are then taken from
 * the equivalent comparison of each score with the thresholds (same classes, bit for bit, no search per
 * score). */
int32_t atts_classify_ordinal(const atts_calib* calib, const float* test_scores, int64_t M,
                              const double* alphas, int32_t n_alpha,
                              int32_t* ranks, float* pvalues, uint8_t* classes, float* thresholds,
                              void* hip_stream);

/* Conditional coverage (Sec. "Q2", paragraph "Online Calibration", last sentence; Proposition 2): the candidates of
 * every input are ranked against the calibration scores of the SAME input only.  For input x (0 <= x < n_inputs)
 * with m_x = cal_offsets[x + 1] - cal_offsets[x] own calibration scores and its candidates
 * t in [test_offsets[x], test_offsets[x + 1]):
 *     ranks[t]   = #{ j in input x : test_scores[t] <= cal_scores[j] }
 *     pvalues[t] = (ranks[t] + 1) / (m_x + 1)
 *     r_l        = floor(alphas[l] * (m_x + 1))   in binary64
 *     classes[t] = #{ l : ranks[t] + 1 <= r_l }
 * i.e. atts_classify_ordinal's rule with the input's own m_x scores as the calibration set (an input without
 * calibration scores accepts everything: p = 1).  NaN, -0 and +-inf behave as there.  No handle: the scores
 * need not be sorted and nothing is kept.
 *   cal_scores dev float [cal_offsets[n_inputs]]; test_scores dev float [test_offsets[n_inputs]];
 *   cal_offsets, test_offsets dev int64 [n_inputs + 1], non-decreasing, first entry 0 (read by the kernel only:
 *   a decreasing pair is treated as an empty range); alphas HOST double [n_alpha] as for atts_classify_ordinal;
 *   ranks dev int32, pvalues dev float or NULL, classes dev uint8: one entry per test score.
 * One wavefront per input: meant for many small sets (tens to a few thousand scores each). */
int32_t atts_classify_conditional(const float* cal_scores, const int64_t* cal_offsets, const float* test_scores,
                                  const int64_t* test_offsets, int64_t n_inputs, const double* alphas, int32_t n_alpha,
                                  int32_t* ranks, float* pvalues, uint8_t* classes, void* hip_stream);

/* Copies the multiset, in ascending order (NaNs first), to out dev float [size]. */
int32_t atts_calib_export(const atts_calib* calib, float* out, void* hip_stream);

/* Restores a multiset that atts_calib_export wrote (checkpoint / resume of "Online Calibration"): the handle's
 * contents are REPLACED by scores dev float [n], which must be in the order atts_calib_export produces (ascending,
 * NaNs first, by the comparison rules above; -0 and +0 in any order).  n >= 0 (0 empties the handle).  The order
 * is the caller's promise and is not verified (device data); unsorted input gives wrong ranks, never a fault.
 * Ranks, classes and thresholds after an import equal those of the handle that was exported, bit for bit.
 * ATTS_ERR_CAPACITY if n > capacity (nothing is changed). */
int32_t atts_calib_import(atts_calib* calib, const float* scores, int64_t n, void* hip_stream);

/* ------------------------------------------------------------------------------------
 * The classic, synchronous pipeline (Sec. "Preliminary", "Classic Setup"): the design the
 * asynchronous rule is measured against.  Built as the comparator for the asynchronous
 * arithmetic intensity r = T_c / (T_m + T_s) of Sec. "Q1": none of the three steps can run
 * for an input before ALL m of its candidates have been scored.
 *
 *   atts_classic_normalize        Eq. "softmax": scores[i, k] = exp(-nll[i, k]) / sum_j exp(-nll[i, j]), the share of
 *                                 candidate k in the likelihood of the m candidates of input i (nll = the unnormalised
 *                                 score atts_score_drafts returns; larger share = more likely).  fp32; a NaN loss makes
 *                                 every score of its input NaN.  nll, scores dev float [n_inputs, m] row-major; m >= 1.
 *   atts_classic_threshold        Eq. "quantile": tau[0] = the k-th smallest of ALL n_scores normalised calibration
 *                                 scores, k = ceil((N + 1)(1 - alpha)) = N + 1 - floor(alpha (N + 1)) with the floor of
 *                                 one binary64 product (+inf if k > N): a global sort of the set.  cal_scores dev float
 *                                 [n_scores] (read only), 1 <= n_scores <= 2^30; alpha in (0, 1); tau dev float [1];
 *                                 workspace dev, 256-byte aligned, >= atts_classic_workspace_bytes(n_scores), scratch.
 *   atts_classic_prediction_sets  Eq. "pred_set": member[i] = 1 if scores[i] >= tau[0] else 0 (ties with the threshold
 *                                 are members; a NaN score is not).  scores dev float [count], tau dev float [1] (read
 *                                 on the device, so the three calls chain on one stream without a host round trip),
 *                                 member dev uint8 [count].
 * Host-detectable errors (NULLs, sizes, alpha, workspace) are reported before anything is enqueued.
 * ---------------------------------------------------------------------------------- */
int32_t atts_classic_workspace_bytes(int64_t n_scores, size_t* out_bytes);
int32_t atts_classic_normalize(const float* nll, int64_t n_inputs, int32_t m, float* scores, void* hip_stream);
int32_t atts_classic_threshold(const float* cal_scores, int64_t n_scores, double alpha, float* tau, void* workspace,
                               size_t workspace_bytes, void* hip_stream);
int32_t atts_classic_prediction_sets(const float* scores, int64_t count, const float* tau, uint8_t* member, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* ATTS_H */
