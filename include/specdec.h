/*
 * specdec.h -- C ABI of the MI355X (gfx950) draft-verify-correct round of
 * speculative decoding with adaptive candidate length (SpecDec++).
 *
 * The library implements Algorithm 2 of the paper (Sec. 4.3) with Algorithm 1's
 * verify / correct tail (Appendix C) as hand-written HIP kernels.  PyTorch (or
 * any other allocator) only provides device memory for the weights; every step
 * of the path runs in this library's kernels on `hip_stream`.
 *
 * Conventions
 *   - "DEVICE" pointers are HIP device pointers owned by the caller and must stay
 *     alive and unchanged while a context that was given them exists.
 *   - "HOST" pointers are ordinary host memory, read or written before return.
 *   - Matrices are row-major [out, in]; dtype is SD_F32 or SD_BF16 for every
 *     tensor of one model (weights, activations and KV cache share it).
 *   - Every function returns an sd_status; 0 is success, negative is an error.
 *     Nothing throws or aborts.  Host out-parameters are written only on SD_OK.
 *     On an error the sequences' committed state (tokens, lengths) is unchanged.
 *   - Calls on one context must not overlap; calls on different contexts may come
 *     from different threads.  Use one GPU per process (the device that is current
 *     when sd_create runs must be current in every later call on that context; the
 *     permission to use more than 64 KB of LDS is set once per process, by a
 *     kernel's first launch).
 */
#ifndef SPECDEC_H
#define SPECDEC_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef int32_t sd_status;
enum {
  SD_OK = 0,
  SD_EINVAL = -1,     /* null pointer, bad shape, unsupported dtype or size        */
  SD_ENOMEM = -2,     /* device or host allocation failed                          */
  SD_ERANGE = -3,     /* sequence would overflow max_seq, or a token id >= vocab   */
  SD_ENONFINITE = -4, /* a kernel saw NaN/Inf logits (sticky until sd_prefill)      */
  SD_EDEVICE = -5     /* a HIP call failed                                          */
};
enum { SD_F32 = 0, SD_BF16 = 1 };

#define SD_MAX_K 32          /* largest supported k_max                           */
#define SD_MAX_HEAD_LAYERS 8

/* Llama-style decoder (the paper's model family, Sec. 5.1): token embedding,
 * n_layers x [RMSNorm, q|k|v projection, rotary embedding (rotate-half pairing),
 * causal grouped-query attention, output projection, residual, RMSNorm, SwiGLU MLP,
 * residual], final RMSNorm, LM head.  All pointers DEVICE. */
typedef struct {
  int32_t n_layers, d_model, n_heads, n_kv_heads, head_dim, d_ffn, vocab, dtype;
  float rope_theta, rms_eps;
  const void *tok_emb;             /* [vocab, d_model]                                 */
  const void *lm_head;             /* [vocab, d_model]                                 */
  const void *final_norm;          /* [d_model]                                        */
  const void *const *wqkv;         /* HOST array[n_layers] of DEVICE [(Hq+2Hkv)*hd, d] (q rows, k rows, v rows) */
  const void *const *wo;           /* HOST array[n_layers] of DEVICE [d, Hq*hd]        */
  const void *const *w_gate_up;    /* HOST array[n_layers] of DEVICE [2*d_ffn, d] (gate rows, then up rows) */
  const void *const *w_down;       /* HOST array[n_layers] of DEVICE [d, d_ffn]        */
  const void *const *norm_attn;    /* HOST array[n_layers] of DEVICE [d]               */
  const void *const *norm_mlp;     /* HOST array[n_layers] of DEVICE [d]               */
} sd_model;

/* Acceptance-prediction head f_theta (Eq. 3; "(D+1)-layer ResNet with SiLU",
 * Sec. 5.1): z <- SiLU(W_j z + b_j) for j < n_layers-1 (z <- z + SiLU(..) when
 * `residual` and the layer is square), then one linear layer to a single logit;
 * the library applies the sigmoid.  Input: the draft's final-RMSNorm output for
 * the last ingested token.  dims[0] must equal the draft's d_model and
 * dims[n_layers] must be 1.  May be NULL in sd_create: then the predicted
 * acceptance is 1 and only k_max, EOS and cache capacity end the draft loop. */
typedef struct {
  int32_t n_layers;                /* 1..SD_MAX_HEAD_LAYERS                            */
  const int32_t *dims;             /* HOST array[n_layers+1]                           */
  int32_t residual;
  int32_t dtype;                   /* must equal the draft model's dtype               */
  const void *const *W;            /* HOST array[n_layers] of DEVICE [dims[j+1], dims[j]] */
  const void *const *b;            /* HOST array[n_layers] of DEVICE [dims[j+1]]       */
} sd_head;

typedef struct {
  int32_t batch;                   /* sequences decoded together (>= 1)                */
  int32_t max_seq;                 /* KV-cache capacity per sequence, in tokens: a multiple
                                      of 64, at most 32768 (bf16) or 12288 (fp32 models) */
  int32_t k_max;                   /* cap on candidates per round (Sec. 5.1), 1..SD_MAX_K */
  void *hip_stream;                /* hipStream_t all work is enqueued on (NULL = default) */
} sd_config;

/* Per-call decoding parameters: threshold h of the stop rule (stop when
 * 1 - prod p_hat > h, Sec. 4.3), softmax temperature (Appendix D.1 uses 1),
 * greedy mode (Sec. 4.1), optional EOS (manual stop, Sec. 4.2 footnote), top-k warping
 * of both models' distributions before the softmax (the paper's inference setting is
 * top-k = 50, Appendix D.1; every logit >= the k-th largest of its row is kept; 0 = full
 * vocabulary), and the Philox seed.  Uniforms are Philox4x32-10 with key = seed and counter
 * (slot i, round index, sequence id, stream), stream 0 = draft sample,
 * 1 = accept test r_i, 2 = residual / bonus sample;
 * u = (word0 >> 8) * 2^-24. */
typedef struct {
  float h;
  float temperature;
  int32_t greedy;
  int32_t eos_id;                  /* < 0: none                                        */
  uint64_t seed;
  int32_t top_k;                   /* 0: off                                           */
  int32_t reserved;                /* must be 0                                        */
} sd_params;

/* Result of one round for one sequence (Algorithm 2's return): K candidates were
 * drawn, the first n_accepted were kept, and tokens[0..n_new) = y_1..y_n, y'. */
typedef struct {
  int32_t K, n_accepted, n_new;
  int32_t tokens[SD_MAX_K + 1];
  int32_t cand[SD_MAX_K];          /* y_1..y_K as drawn                                */
  float p_hat;                     /* cumulative predicted acceptance at the stop      */
} sd_round_out;

/* Counters of Sec. 3.2 (N_draft + N_target = N + N_discarded for whole rounds)
 * and measured phase times, summed over the rounds of the call. */
typedef struct {
  int64_t N, N_draft, N_target, N_discarded, rounds;
  double t_draft_s, t_target_s, t_accept_s, t_total_s;
} sd_stats;

typedef struct sd_ctx sd_ctx;

/* Build a context: copies the model descriptions, allocates both KV caches,
 * the stored draft rows q_1..q_K, the target rows p_1..p_{K+1} and all scratch on
 * the current HIP device.  `head` may be NULL.  SD_EINVAL for inconsistent shapes
 * (vocab mismatch between the models, head_dim not in {64,128} for bf16, ...). */
sd_status sd_create(sd_ctx **out, const sd_model *target, const sd_model *draft,
                    const sd_head *head, const sd_config *cfg);
sd_status sd_destroy(sd_ctx *ctx);

/* Reset sequence `seq` to the prompt (HOST ids, n_prompt >= 1): runs both models
 * over prompt[0 .. n_prompt-1) so that each cache holds every finalised token but
 * the last, which the first round ingests.  Resets the sequence's round index to
 * 0 and clears the sticky non-finite flag.  SD_ERANGE if n_prompt + 2 > max_seq
 * or an id is outside [0, vocab). */
sd_status sd_prefill(sd_ctx *ctx, int32_t seq, const int32_t *prompt_host, int32_t n_prompt);

/* One draft-verify-correct round for every sequence of the batch (Algorithm 2):
 * adaptive draft loop with the head's stop rule, one target pass over the K+1
 * positions, accept / residual resample, KV rollback.  out_per_seq: HOST
 * array[batch].  The candidate cap of a sequence is min(k_max, max_seq - P - 1);
 * SD_ERANGE if that is < 1 for any sequence (nothing is changed). */
sd_status specdec_round(sd_ctx *ctx, const sd_params *params, sd_round_out *out_per_seq);

/* Rounds until every sequence has max_new_tokens new tokens (or emitted EOS).  A
 * round may overshoot; outputs are truncated to max_new_tokens and N counts kept
 * tokens only.  out_tokens_host: HOST [batch, max_new_tokens]; out_lens: HOST
 * [batch]; stats may be NULL. */
sd_status specdec_generate(sd_ctx *ctx, const sd_params *params, int32_t max_new_tokens,
                           int32_t *out_tokens_host, int32_t *out_lens, sd_stats *stats);

/* The accept / residual-resample step on its own (Algorithm 1's tail, Appendix C):
 * for each sequence b with K_b = K_per_seq_dev[b] candidates cand_dev[b, 0..K_b),
 * n_out_dev[b] = number accepted, tok_out_dev[b] = y', accept_flags_dev[b, i] =
 * outcome of the (i+1)-th accept test taken on its own (0 for i >= K_b).
 * p_logits_dev: DEVICE fp32 [B, Kmax+1, V]; q_logits_dev: DEVICE fp32 [B, Kmax, V];
 * cand_dev: DEVICE int32 [B, Kmax]; K_per_seq_dev: DEVICE int32 [B];
 * outputs DEVICE int32 [B], int32 [B], uint8 [B, Kmax].  `stats_ws_dev` is DEVICE
 * scratch of sd_accept_workspace_bytes(B, Kmax) bytes, 16-byte aligned.  Enqueued on
 * `hip_stream`; does not synchronise.
 * The device arrays are the caller's and cannot be checked on the host without a
 * synchronisation, so the kernels make them safe instead: a K_b outside [0, Kmax]
 * is clamped into it, and a candidate id outside [0, V) counts as rejected (its flag
 * is 0, n_out stops before it, y' is the residual sample of that position).  The
 * int32 at byte offset B * (2 * Kmax + 1) * 16 of the workspace is the call's status
 * word: 0 when every input was in range, bit 0 set when a K_b was clamped, bit 1 when
 * a candidate id was out of range (valid once the stream has reached the end of the
 * call). */
sd_status sd_accept_resample(const float *p_logits_dev, const float *q_logits_dev,
                             const int32_t *cand_dev, const int32_t *K_per_seq_dev,
                             int32_t B, int32_t Kmax, int32_t V, const sd_params *params,
                             int32_t round_idx, void *stats_ws_dev, void *hip_stream,
                             int32_t *n_out_dev, int32_t *tok_out_dev, uint8_t *accept_flags_dev);
int64_t sd_accept_workspace_bytes(int32_t B, int32_t Kmax);

/* sd_accept_resample for callers that cannot allocate device memory (code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc): the same step
 * with the row statistics kept in a device array that is part of the library image
 * (SD_ACCEPT_STATIC_MAX_BATCH * (2 * SD_MAX_K + 1) * 16 + 16 bytes = 66 576 bytes per
 * GPU, held until the process ends) instead of a caller's workspace.  Same arguments,
 * same kernels and same results as sd_accept_resample; B > SD_ACCEPT_STATIC_MAX_BATCH
 * is SD_ERANGE.  The call allocates nothing, frees nothing and does not synchronise.
 * If status_word_dev_out is not NULL it receives the DEVICE address of the call's
 * status word (see sd_accept_resample).  Every call on a GPU shares that GPU's array:
 * calls that overlap on one GPU (different streams, different threads) race; calls on
 * one stream are ordered and each overwrites what the last one left. */
#define SD_ACCEPT_STATIC_MAX_BATCH 64
sd_status sd_accept_resample_static(const float *p_logits_dev, const float *q_logits_dev,
                                    const int32_t *cand_dev, const int32_t *K_per_seq_dev,
                                    int32_t B, int32_t Kmax, int32_t V, const sd_params *params,
                                    int32_t round_idx, void *hip_stream,
                                    int32_t *n_out_dev, int32_t *tok_out_dev,
                                    uint8_t *accept_flags_dev, int32_t **status_word_dev_out);

/* Phase times of the most recent specdec_round / round of specdec_generate on this
 * context, measured with HIP events on the context's stream (the decomposition of
 * Sec. 3.2 / Eq. 1 needs per-forward times): seconds[0] = the draft loop, [1] = the
 * target pass over the K+1 positions, [2] = accept / resample + commit.  HOST array of
 * 3.  target_rows (may be NULL) receives the activation rows that target pass carried
 * (K+1 for one sequence; the packed row slots of a batch).  Zeros before the first round. */
sd_status sd_last_round_times(sd_ctx *ctx, double *seconds, int32_t *target_rows);

/* Teacher-forced forward for parity checks and timing: ingest `n` tokens (HOST
 * ids) of sequence `seq` into model `which` (0 = target, 1 = draft) at cache
 * positions start .. start+n-1 (start <= that cache's current length; later
 * positions are discarded first) and copy the n rows of fp32 logits [n, vocab]
 * (and, if non-NULL, the final-RMSNorm hidden rows [n, d_model] as fp32) to HOST.
 * n <= 32.  Leaves the cache length at start + n. */
sd_status sd_forward(sd_ctx *ctx, int32_t which, int32_t seq, int32_t start, const int32_t *tokens_host,
                     int32_t n, float *logits_host, float *hidden_host);

/* Introspection of sequence state (HOST outs, any may be NULL): P = finalised
 * tokens, cache lengths of target and draft, round index. */
sd_status sd_seq_state(sd_ctx *ctx, int32_t seq, int32_t *P, int32_t *kv_len_target,
                       int32_t *kv_len_draft, int32_t *round_idx);

/* The fp32 rows the last round used (for decision replay): copies q_logits
 * [K, vocab], p_logits [K+1, vocab] and the head's K-1 sigmoid outputs of
 * sequence `seq` to HOST buffers (any may be NULL). */
sd_status sd_last_round_rows(sd_ctx *ctx, int32_t seq, float *q_logits_host, float *p_logits_host,
                             float *head_s_host);

/* Per-launch timing of the weight-streaming GEMM kernels of the target pass.
 * sd_profile_enable(ctx, every) brackets the GEMM launches of every `every`-th
 * target layer (and the LM head) with HIP events from then on (0 = off); the sampled
 * layers move on by one with every pass (pass p samples the layers l with
 * (l + p) % every == 0), so a run of passes covers all of them.
 * sd_profile_read waits for the context's stream, then sums, since the last read, the
 * sampled launches' streamed weight
 * bytes and durations per matrix kind (0 qkv, 1 o, 2 gate_up, 3 down, 4 lm_head):
 * HOST arrays of 5. */
sd_status sd_profile_enable(sd_ctx *ctx, int32_t every);
sd_status sd_profile_read(sd_ctx *ctx, int64_t *launches, double *seconds, double *weight_bytes);

/* The weight-streaming skinny GEMM on its own (the kernel the target pass over
 * M = K+1 rows and the M = 1 draft steps spend their time in; Algorithm 2's
 * "compute in parallel" step): Y[m, n] = sum_k X[m, k] * W[n, k], fp32 out.
 * W: DEVICE [N, K] and X: DEVICE [M, K], both `dtype`; Y: DEVICE fp32 [M, N]; ws: DEVICE
 * scratch of sd_gemm_workspace_bytes(...) bytes (per-K-slice partial sums, added in
 * slice order).  1 <= M <= 160; for SD_BF16, K % 128 == 0 and N % 16 == 0, pointers
 * 16-byte aligned (more than 17 rows are handed to the tiled kernel below; up to 8 rows with
 * K >= 2048 (K % 8 == 0), and 9 .. 17 rows with K % 512 == 0, go through kernels that stream whole
 * 1 KB pieces of single weight rows and take any N >= 1).  Enqueued on `hip_stream`; does not
 * synchronise. */
sd_status sd_gemm_skinny(int32_t dtype, const void *W_dev, const void *X_dev, int32_t M, int32_t N, int32_t K,
                         float *Y_dev, void *ws_dev, void *hip_stream);

/* The gated activation of a decoder layer's MLP as both forward passes of Algorithm 2 compute it:
 *   act[m, f] = silu(sum_k X[m, k] W[f, k]) * (sum_k X[m, k] W[ffn + f, k]),   silu(z) = z / (1 + exp(-z)),
 * W: DEVICE [2 ffn, K] = [gate; up] and X: DEVICE [M, K], both `dtype`; act: DEVICE [M, ffn] in `dtype`.
 * Two ways to the same result, both rounding once, to `dtype`, at the end:
 *   mode 1: ONE launch, the row-stripe GEMM with the activation in its final sweep; ws is not used.  Possible
 *           (sd_mlp_act_is_fused returns 1) for SD_BF16, M <= 8, K >= 2048, K % 8 == 0, when a workgroup can hold a
 *           row range of gate and one of up (always for K <= 8192: up to four 2048-wide stripes per row), and for
 *           9 <= M <= 17 with K % 512 == 0; SD_EINVAL elsewhere.
 *   mode 0: sd_gemm_skinny's product followed by an activation kernel; ws is DEVICE scratch of
 *           sd_gemm_workspace_bytes(dtype, M, 2 ffn, K) bytes.
 *   mode -1: what the forward passes do: mode 1 where it is possible, else mode 0.
 * 1 <= M <= 160 and sd_gemm_skinny's shape rules with N = 2 ffn; SD_EINVAL / SD_EDEVICE otherwise.
 * Enqueued on `hip_stream`; does not synchronise. */
int32_t sd_mlp_act_is_fused(int32_t dtype, int32_t M, int32_t ffn, int32_t K);
sd_status sd_mlp_act(int32_t dtype, const void *W_gate_up_dev, const void *X_dev, int32_t M, int32_t ffn, int32_t K,
                     void *act_dev, void *ws_dev, int32_t mode, void *hip_stream);

/* The first step of a decoder layer's attention as both forward passes of Algorithm 2 compute it, on M rows:
 *   [q; k; v][m] = W X[m],  W: DEVICE [(n_heads + 2 n_kv_heads) head_dim, K] = q rows, k rows, v rows;
 *   q and k take the rotary embedding at row_pos[m]: the pair (v[i], v[i + head_dim/2]) of every head is turned by
 *   the angle whose cosine and sine are cos_sin[row_pos[m]][i][0..1] (DEVICE fp32 [max_seq][head_dim/2][2]);
 *   q -> q_out [M][n_heads head_dim], k -> k_cache[row_seq[m]][kv head][row_pos[m]][:] of a
 *   [n_seq][n_kv_heads][max_seq][head_dim] array, v -> v_cache[row_seq[m]][kv head][:][row_pos[m]] of a
 *   [n_seq][n_kv_heads][head_dim][max_seq] array (values are kept transposed), all in `dtype`.
 * row_seq, row_pos: DEVICE int32 [M]; a row with row_seq[m] < 0 writes nothing; the caller guarantees
 * 0 <= row_pos[m] < max_seq and that row_seq[m] indexes the caches.  X: DEVICE [M, K] in `dtype`.
 *   mode 1: ONE launch: the row-stripe GEMM walks the rows of W so that both rows of a rotary pair land in one
 *           wavefront, and its final sweep rotates and writes q and the cache entries; ws is not used.  Possible
 *           (sd_qkv_rope_is_fused returns 1) for SD_BF16 and head_dim a power of two, with M <= 8, K >= 2048,
 *           K % 8 == 0, or with 9 <= M <= 17, K % 512 == 0; SD_EINVAL elsewhere.
 *   mode 0: sd_gemm_skinny's product followed by a rotary + append kernel; ws is DEVICE scratch of
 *           sd_gemm_workspace_bytes(dtype, M, N, K) bytes, N = (n_heads + 2 n_kv_heads) head_dim.
 *   mode -1: what the forward passes do: mode 1 where it is possible, else mode 0.
 * Both modes round once, to `dtype`, at the end, and give the same bits.  1 <= M <= 160 and sd_gemm_skinny's
 * shape rules; SD_EINVAL / SD_EDEVICE otherwise.  Enqueued on `hip_stream`; does not synchronise. */
int32_t sd_qkv_rope_is_fused(int32_t dtype, int32_t M, int32_t n_heads, int32_t n_kv_heads, int32_t head_dim,
                             int32_t K);
sd_status sd_qkv_rope(int32_t dtype, const void *W_qkv_dev, const void *X_dev, int32_t M, int32_t n_heads,
                      int32_t n_kv_heads, int32_t head_dim, int32_t K, const int32_t *row_seq_dev,
                      const int32_t *row_pos_dev, const float *cos_sin_dev, void *q_out_dev, void *k_cache_dev,
                      void *v_cache_dev, int32_t max_seq, void *ws_dev, int32_t mode, void *hip_stream);

/* ---- Training of the acceptance-prediction head (Sec. 4.4) ---------------------------
 *
 * sd_head_examples builds the training examples of one (prompt, response) pair with the
 * context's two models: `tokens` (HOST) holds n_prompt prompt tokens followed by the N
 * tokens X_1..X_N of a target response (e.g. the output of specdec_generate, which is
 * distributed as the target's own samples).  Teacher-forced on X it computes, for every i,
 * Y_i ~ q_i (uniform of (slot i, example, sequence 0, stream 3)) and the target
 * P_i = min(1, p_i(Y_i)/q_i(Y_i)) under `temperature` / `top_k`; mixes tokens
 * (Z_i = X_i when the uniform of (slot i, example, 0, stream 4) < r, else Y_i; mask_i = 1
 * where Z_i = Y_i: the tokens that carry a loss); and runs the draft over (prompt, Z) to get
 * E_i, its final (post-RMSNorm) embedding of Z_i.
 * E_dev: DEVICE fp32 [N, d_draft]; P_dev: DEVICE fp32 [N]; mask_dev: DEVICE int32 [N];
 * Y_host, Z_host: HOST int32 [N], may be null.  Needs n_prompt + N + 2 <= max_seq.
 * Uses sequence slot `seq` and leaves it inactive: sd_prefill it again before decoding.
 * Synchronises the stream. */
sd_status sd_head_examples(sd_ctx *ctx, int32_t seq, const int32_t *tokens_host, int32_t n_prompt, int32_t N, float r,
                           uint64_t seed, int32_t example, float temperature, int32_t top_k, float *E_dev,
                           float *P_dev, int32_t *mask_dev, int32_t *Y_host, int32_t *Z_host);

/* A trainer owns fp32 copies of a head's weights (initialised from `init`, whose arrays are
 * DEVICE memory in init->dtype), their gradients and Adam moments, and activation buffers
 * for batches of up to n_max <= 4096 rows.  Work is enqueued on `hip_stream`. */
typedef struct sd_trainer sd_trainer;
sd_status sd_trainer_create(sd_trainer **out, const sd_head *init, int32_t n_max, void *hip_stream);
sd_status sd_trainer_destroy(sd_trainer *tr);

/* One step on a batch of n examples (E: DEVICE fp32 [n, dims[0]], P: DEVICE fp32 [n], mask:
 * DEVICE int32 [n]): forward, the weighted BCE of Sec. 4.4 averaged over the n_m masked rows
 *   (1/n_m) sum_{mask} -w_acc P log P_hat - w_rej (1 - P) log(1 - P_hat),   P_hat = sigmoid(f(E)),
 * its gradient for every W_j, b_j, and, when apply != 0, one Adam update (bias-corrected, no
 * weight decay) with the given lr / beta1 / beta2 / eps.  loss_host (HOST, may be null)
 * receives the loss before the update; passing it synchronises the stream. */
sd_status sd_trainer_step(sd_trainer *tr, const float *E_dev, const float *P_dev, const int32_t *mask_dev, int32_t n,
                          float w_acc, float w_rej, float lr, float beta1, float beta2, float eps, int32_t apply,
                          float *loss_host);
/* logits_dev[i] = f_theta(E_i) with the current weights (DEVICE fp32 [n]). */
sd_status sd_trainer_predict(sd_trainer *tr, const float *E_dev, int32_t n, float *logits_dev);
/* Copy layer `layer`'s W (what = 0), b (1), last gradient of W (2) or of b (3) to HOST fp32. */
sd_status sd_trainer_read(sd_trainer *tr, int32_t layer, int32_t what, float *host);
/* Write the current weights, converted to `dtype`, into caller-owned DEVICE arrays laid out
 * like sd_head.W / sd_head.b (so that a head for sd_create can be built from them). */
sd_status sd_trainer_export(sd_trainer *tr, int32_t dtype, void *const *W_out_dev, void *const *b_out_dev);

/* The tiled GEMM of the prompt pass and of wide (batched) target passes: both models ingest
 * the prefix before the first round of Algorithm 2, and with hundreds of rows per weight the
 * product is bound by the matrix cores, not by the weight stream.  Y[m, n] = sum_k X[m, k] *
 * W[n, k], bf16 in, fp32 out.  W: DEVICE bf16 [N, K]; X: DEVICE bf16 [M, K]; Y: DEVICE fp32
 * [M, N]; ws: DEVICE scratch of sd_gemm_tile_workspace_bytes(M, N, K) bytes (0 for large M: may
 * then be null; for M <= 192 the product may be split along K to fill the chip and the slices
 * are added in slice order).  1 <= M <= 1024, K % 32 == 0, N % 4 == 0, pointers 16-byte
 * aligned; SD_EINVAL / SD_EDEVICE otherwise.  Enqueued on `hip_stream`; does not synchronise. */
int64_t sd_gemm_tile_workspace_bytes(int32_t M, int32_t N, int32_t K);
sd_status sd_gemm_tile(const void *W_dev, const void *X_dev, int32_t M, int32_t N, int32_t K, float *Y_dev,
                       void *workspace_dev, void *hip_stream);
int64_t sd_gemm_workspace_bytes(int32_t dtype, int32_t M, int32_t N, int32_t K);

const char *sd_strerror(sd_status s);
const char *sd_version(void);

#ifdef __cplusplus
}
#endif
#endif /* SPECDEC_H */
