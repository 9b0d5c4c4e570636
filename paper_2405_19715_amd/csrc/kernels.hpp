// Host-side launchers of the HIP kernels.  Every launcher validates the shapes the
// kernel and its grid assume and returns hipErrorInvalidValue instead of launching
// when they do not hold.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace sd {

enum { DT_F32 = 0, DT_BF16 = 1 };
constexpr int MAX_ROWS = 160;          // most activation rows a round's forward call carries (streaming GEMM)
constexpr int MAX_PREFILL_ROWS = 1024; // most rows of one prompt-pass chunk (tiled GEMM, elementwise kernels)

// ---------------------------------------------------------------- skinny GEMM
// part[s, m, n] = sum over the s-th K-slice of X[m, :] * W[n, :]   (fp32)
// W: [N, K] row-major in dtype; X: [M, K] rows (row stride ldx elements) in dtype,
// optionally gathered through xrow (device int32 [M], may be null).
// The number of K-slices is gemm_splits(dtype, M, N, K); consumers add the slices
// in slice order.  bf16 products: up to 8 rows with K >= 2048 go through the row-stripe kernel (vector-ALU dot
// products on whole 1 KB row pieces: the access pattern that reads HBM fastest), 9 .. 17 rows with K a multiple of
// 512 through its matrix-core sibling (gemm_mstripe.hip), more rows through the tiled kernel (launch_gemm_tile),
// which reads every weight once however many rows there are, the rest (up to 16 rows) through the MFMA streaming kernel.
int gemm_splits(int dtype, int M, int N, int K);
hipError_t launch_gemm(hipStream_t st, int dtype, const void* W, const void* X, int ldx, const int* xrow,
                       float* part, int M, int N, int K);

// act[m, f] = silu(X[m, :] . W[f, :]) * (X[m, :] . W[ffn + f, :]) in bf16, W = [gate; up] = [2 ffn, K]: the
// row-stripe kernel with the MLP's activation in its final sweep (no partial sums, no activation launch).
// Possible where gemm_silu_fused says so: bf16, up to 8 rows, K >= 2048 with a stripe count that leaves room for a
// gate and an up range in one workgroup (always for K <= 8192), or 9 .. 17 rows with K a multiple of 512;
// launch_gemm_silu returns
// hipErrorInvalidValue elsewhere.  Same sums, same rounding as launch_gemm + launch_silu_mul on such a shape.
// With `ssq` (device, [M][ssq_n]: per-workgroup sums of squares of the UNSCALED input rows, as launch_gemm_resid
// leaves them) both sums are multiplied by r_m = rsqrt(sum_i ssq[m][i] / d_in + eps) first: the RMSNorm factor the
// producer of X left out.
bool gemm_silu_fused(int dtype, int M, int ffn, int K);
hipError_t launch_gemm_silu(hipStream_t st, int dtype, const void* W, const void* X, int ldx, const int* xrow,
                            void* act, int M, int ffn, int K, const float* ssq = nullptr, int ssq_n = 0, int d_in = 0,
                            float eps = 0.f);

// x[m, n] += X[m, :] . W[n, :] (the residual stream, fp32); xg[m, n] = bf16(x[m, n] * gain[n]); ssq[m][g] = sum of
// x[m, n]^2 over the columns of workgroup g, g < gemm_resid_groups(...): the residual add and the RMSNorm that
// follows a projection, minus the per-row factor rsqrt(mean(x^2) + eps), which the consumer of xg applies to
// its own sums (launch_gemm_silu with `ssq`).  Row-stripe kernel with one slice only: gemm_resid_groups returns
// 0 where that does not apply, and launch_gemm_resid hipErrorInvalidValue.
// launch_gemm with one slice whose sums are multiplied by the rows' RMSNorm factors from `ssq` (see
// launch_gemm_silu): for the product that follows a launch_gemm_resid.  Row-stripe shapes only (gemm_scaled_ok).
bool gemm_scaled_ok(int dtype, int M, int N, int K);
hipError_t launch_gemm_scaled(hipStream_t st, int dtype, const void* W, const void* X, int ldx, const int* xrow,
                              float* part, int M, int N, int K, const float* ssq, int ssq_n, int d_in, float eps);
int gemm_resid_groups(int dtype, int M, int N, int K);
// The q|k|v product of a decoder layer (W = [q rows; k rows; v rows], (Hq + 2 Hkv) hd rows of K) that also does
// what follows it: rotary embedding of q and k at row_pos[m], q -> qbuf [M, Hq hd], k -> kcache[seq, kvh, pos, :],
// v -> vcache[seq, kvh, :, pos]; rows with row_seq[m] < 0 write nothing.  With `ssq` the sums first take the rows'
// RMSNorm factors as in launch_gemm_scaled.  Row-stripe shapes with a power-of-two head dimension only
// (gemm_rope_fused); elsewhere launch_gemm + launch_rope_kv do the same in two launches.
bool gemm_rope_fused(int dtype, int M, int Hq, int Hkv, int hd, int K);
hipError_t launch_gemm_rope(hipStream_t st, int dtype, const void* W, const void* X, int ldx, int M, int Hq, int Hkv,
                            int hd, int K, const int32_t* row_seq, const int32_t* row_pos, const float* cos_sin,
                            void* qbuf, void* kcache, void* vcache, int max_seq, const float* ssq, int ssq_n, int d_in,
                            float eps);
hipError_t launch_gemm_resid(hipStream_t st, int dtype, const void* W, const void* X, int ldx, const int* xrow,
                             float* x, const void* gain, void* xg, float* ssq, int M, int N, int K);
// A hidden layer of the acceptance head in one launch: z_out[m, n] = silu(X[m, :] . W[n, :] + bias[n]) (+ z_in[row, n]
// with row = z_rows ? z_rows[m] : m when z_in is set; needs N == K), in bf16.  Same sums and roundings as launch_gemm
// + launch_head_act on such a shape.  Row-stripe shapes with one slice only (gemm_head_fused).
bool gemm_head_fused(int dtype, int M, int N, int K);
hipError_t launch_gemm_head(hipStream_t st, int dtype, const void* W, const void* X, int ldx, const int* xrow,
                            const void* bias, const void* z_in, const int* z_rows, void* z_out, int M, int N, int K);

// ---------------------------------------------------------------- tiled GEMM (prompt pass, wide target passes)
// C[s, m, n] = sum over the s-th K-slice of X[m, k] * W[n, k], bf16 in, fp32 out [S][M][N] with
// S = gemm_tile_splits(M, N, K) (1 for large M); X rows optionally gathered through xrow.
// Any M >= 1; K % 32 == 0, N % 4 == 0, ldx % 8 == 0, 16-byte aligned pointers.
int gemm_tile_splits(int M, int N, int K);
hipError_t launch_gemm_tile(hipStream_t st, const void* W, const void* X, int ldx, const int* xrow, float* C,
                            int M, int N, int K);

// ---------------------------------------------------------------- row plans
struct RowPlan {           // device arrays, one entry per activation row
  int32_t* seq;            // sequence of the row, -1 = padding row
  int32_t* pos;            // absolute position of the row's token
  int32_t* tok;            // token id
  int32_t* gseq;           // per row group: the sequence its rows belong to, -1 = no live row
  int32_t* gend;           // per row group: largest pos + 1 over its live rows (keys to attend)
};

// ---------------------------------------------------------------- elementwise
// `ssq` is scratch for per-block sums of squares: MAX_PREFILL_ROWS * NORM_MAX_BLOCKS floats.
constexpr int NORM_MAX_BLOCKS = 64;    // d <= 65536
// x[m,:] = E[tok[m],:]; xn[m,:] = rmsnorm(x[m,:]) * g
hipError_t launch_embed_norm(hipStream_t st, int dtype, const void* emb, const void* g, float eps,
                             const int32_t* tok, float* x, void* xn, float* ssq, int M, int d, int vocab);
// x[m,:] += sum_s part[s,m,:]; xn[m,:] = rmsnorm(x[m,:]) * g
hipError_t launch_add_norm(hipStream_t st, int dtype, const float* part, int S, const void* g, float eps,
                           float* x, void* xn, float* ssq, int M, int d);
// q,k,v = sum_s part[s,m,:]; rotary embedding on q,k at pos[m]; q -> qbuf [M, Hq*hd];
// k -> kcache[seq, kvh, pos, :]; v -> vcache[seq, kvh, :, pos] (transposed), rows with seq < 0 skipped
hipError_t launch_rope_kv(hipStream_t st, int dtype, const float* part, int S, const RowPlan& rows,
                          const float* cos_sin, void* qbuf, void* kcache, void* vcache, int M, int Hq,
                          int Hkv, int hd, int max_seq);
// act[m,f] = silu(sum_s part[s,m,f]) * (sum_s part[s,m,ffn+f])
hipError_t launch_silu_mul(hipStream_t st, int dtype, const float* part, int S, void* act, int M, int ffn);
// out[(m / RS) * ld_group + (m % RS) * ld_row + n] = sum_s part[s,m,n]     (fp32 logits rows);
// with dst (device int32 [M]) row m goes to out[dst[m] * ld_row + n] instead, dst[m] < 0 drops it
hipError_t launch_reduce_rows(hipStream_t st, const float* part, int S, float* out, int RS, int64_t ld_group,
                              int64_t ld_row, int M, int N, const int32_t* dst = nullptr);
// z_out[m,:] = silu(sum_s part + b) (+ z_in when residual)       (acceptance head hidden layer)
hipError_t launch_head_act(hipStream_t st, int dtype, const float* part, int S, const void* bias,
                           const void* z_in, const int* z_in_rows, void* z_out, int residual, int M, int n);

// ---------------------------------------------------------------- attention
// out[m, h*hd:(h+1)*hd] = softmax_j<=pos[m]( q[m,h,:] . K[seq,kvh,j,:] / sqrt(hd) ) V
// Rows come in groups of RS consecutive rows that belong to one sequence (padding
// rows have seq < 0).  `scratch` holds split partials: attn_scratch_floats(...) floats.
// max_kv_len: upper bound on pos + 1 over all rows (sizes the grid).
// full = true (prompt pass, bf16 only): every wavefront walks all the key blocks its query
// tiles may see and writes finished outputs; no partials, `scratch` unused, M up to
// MAX_PREFILL_ROWS.  Otherwise M <= MAX_ROWS.
size_t attn_scratch_floats(int M, int Hq, int hd, int max_seq);
hipError_t launch_attention(hipStream_t st, int dtype, const void* qbuf, const void* kcache,
                            const void* vcache, const RowPlan& rows, void* out, float* scratch, int M,
                            int RS, int Hq, int Hkv, int hd, int max_seq, int max_kv_len, bool full = false);

// ---------------------------------------------------------------- sampling / accept
struct SeqState {          // device arrays, one entry per sequence unless noted
  int32_t* P;              // finalised tokens
  int32_t* kv_t;           // target cache length
  int32_t* kv_d;           // draft cache length
  int32_t* K;              // candidates drawn so far this round
  int32_t* kcap;           // candidate cap of this round
  int32_t* stopped;        // draft loop ended
  float* p_hat;            // cumulative predicted acceptance
  int32_t* cand;           // [B, 32] y_1..y_K
  int32_t* n_acc;          // accepted candidates
  int32_t* y_new;          // correction / bonus token
  int32_t* tokens;         // [B, max_seq] finalised tokens
  float* head_s;           // [B, 32] head outputs used this round
  uint8_t* flags;          // [B, 32] accept-test outcomes
  int32_t* round;          // round index
  int32_t* last_row;       // activation row holding the sequence's newest token
  int32_t* err;            // [1] sticky: non-finite logits seen
  int32_t* active;         // 0: the sequence sits this round out (finished)
};

struct DecodeParams { float h, temperature; int greedy, eos_id; uint64_t seed; int top_k; };

hipError_t launch_begin_round(hipStream_t st, const SeqState& s, int B, int k_max, int max_seq);
hipError_t launch_plan_draft(hipStream_t st, const SeqState& s, const RowPlan& rows, int B, int step,
                             int max_seq);
// rs = row slots per sequence (>= largest K of the round + 1)
hipError_t launch_plan_verify(hipStream_t st, const SeqState& s, const RowPlan& rows, int B, int rs,
                              int max_seq);
// Ragged target pass: sequence b takes ceil((K_b + 1) / RS) groups of RS row slots, packed one
// sequence after another (n_groups in all, counted by the caller from the same K_b); dst[m] = row of
// the [B, k_max + 1, V] logits array that slot m feeds, or -1 for a padding slot.
hipError_t launch_plan_verify_ragged(hipStream_t st, const SeqState& s, const RowPlan& rows, int B, int RS,
                                     int n_groups, int k_max, int max_seq, int32_t* dst);
// draw y_i from the draft logits row, update p_hat with the head's logit, apply the stop rule
// host_flags (may be null): B words in host-mapped coherent memory; word b becomes (tick << 1) | stopped_b when the
// kernel ends, also for a sequence that had stopped before (tick < 2^30)
hipError_t launch_sample_stop(hipStream_t st, int dtype, const SeqState& s, const float* q_logits,
                              int64_t ld_seq, const void* z, const int* z_rows, int z_dim, const void* w_last,
                              const void* b_last, int have_head, const DecodeParams& p, int B, int V,
                              int step, int32_t* host_flags = nullptr, uint32_t tick = 0);
// softmax statistics of the live rows of the target logits [B, Kmax + 1, V] (row j of sequence b
// is live when j <= K[b]) and the draft logits [B, Kmax, V] (live when j < K[b]), in one launch:
// stats[row] = {max, sum exp((l-max)/T), argmax, top-k threshold}.  With top_k > 0 only logits >=
// the row's k-th largest enter the sum and the threshold is that value (else -inf).
// K[b] outside [0, Kmax] is clamped, a candidate id outside [0, V) counts as rejected; `bad` (device int32,
// may be null) is set to 0 by launch_row_stats and gets bit 0 (a clamped K) / bit 1 (a candidate id out of
// range) from launch_accept, which must follow it on the same stream.
hipError_t launch_row_stats(hipStream_t st, const float* p_logits, const float* q_logits, int Kmax,
                            const int32_t* K, int B, int V, float temperature, int top_k, float* p_stats,
                            float* q_stats, int32_t* err, int32_t* bad = nullptr);
// accept tests, n, and the residual / bonus sample y' for every sequence
hipError_t launch_accept(hipStream_t st, const float* p_logits, const float* q_logits, const float* p_stats,
                         const float* q_stats, const int32_t* cand, int cand_ld, const int32_t* K,
                         const int32_t* round, int round_const, const DecodeParams& p, int B, int Kmax,
                         int V, int32_t* n_out, int32_t* tok_out, uint8_t* flags, int flags_ld,
                         int32_t* bad = nullptr);
// training targets of the acceptance head (Sec. 4.4): for row i of p / q [n, V], Y_i ~ q_i with the
// uniform of (slot0 + i, example, 0, stream 3) and P_i = min(1, p_i(Y_i) / q_i(Y_i))
hipError_t launch_labels(hipStream_t st, const float* p_logits, const float* q_logits, int n, int V,
                         float temperature, int top_k, uint64_t seed, int slot0, int example, int32_t* Y, float* P);
// token mixing: Z_i = X_i when u(i + 1, example, 0, stream 4) < r, else Y_i (mask_i = 1)
hipError_t launch_mix(hipStream_t st, const int32_t* X, const int32_t* Y, int n, float r, uint64_t seed,
                      int example, int32_t* Z, int32_t* mask);
// append y_1..y_n, y' to the token history and roll both cache lengths back
// and pack {K, n, y', p_hat, cand[32], P, kv_t, kv_d, err} (40 ints per sequence) for the host
hipError_t launch_commit(hipStream_t st, const SeqState& s, int32_t* result, int B, int max_seq);
constexpr int RESULT_INTS = 40;

// y[i] = (float) x[i] for n elements of `dtype`
hipError_t launch_to_f32(hipStream_t st, int dtype, const void* x, float* y, size_t n);

}  // namespace sd
