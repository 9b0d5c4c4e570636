// Host side of the library: the context (KV caches, workspaces, device-resident
// sequence state), the Llama-style forward as a fixed kernel sequence, the round of
// Algorithm 2 (adaptive draft loop, target pass over K+1 rows, accept / resample,
// KV rollback), the generation loop with the counters of Sec. 3.2, and the C ABI.
#include "../../include/specdec.h"

#include "kernels.hpp"

#include <chrono>
#include <cmath>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <new>
#include <vector>

using namespace sd;

namespace {

constexpr int PREFILL_CHUNK = 32;
constexpr int CAND_LD = 32;

#define SD_HIP(call)                                  \
  do {                                                \
    hipError_t e_ = (call);                           \
    if (e_ != hipSuccess) return map_hip(e_);         \
  } while (0)

sd_status map_hip(hipError_t e) {
  if (e == hipErrorOutOfMemory) return SD_ENOMEM;
  if (e == hipErrorInvalidValue) return SD_EINVAL;
  return SD_EDEVICE;
}

struct ModelRt {
  sd_model m{};
  std::vector<const void*> wqkv, wo, wgu, wdown, na, nm;
  char* kcache = nullptr;        // [layer][batch][Hkv][max_seq][hd]
  char* vcache = nullptr;        // [layer][batch][Hkv][hd][max_seq]
  size_t layer_bytes = 0;
  float* cos_sin = nullptr;      // [max_seq][hd/2][2]
  int esz = 4;
  int n_q() const { return m.n_heads * m.head_dim; }
  int n_kv() const { return m.n_kv_heads * m.head_dim; }
};

struct HeadRt {
  bool present = false;
  int n_layers = 0, residual = 0, dtype = 0;
  std::vector<int> dims;
  std::vector<const void*> W, b;
};

struct ProfSample { hipEvent_t a, b; int kind; double bytes; };

}  // namespace

struct sd_ctx {
  sd_config cfg{};
  hipStream_t st = nullptr;
  ModelRt target, draft;
  HeadRt head;
  int B = 1, max_rows = 0;
  int prefill_rows = 0;          // rows of one prompt-pass chunk of a bf16 model (tiled GEMM path)

  // activations (sized for the wider model)
  float* x = nullptr;
  void *xn = nullptr, *qbuf = nullptr, *attn = nullptr, *act = nullptr, *hz[2] = {nullptr, nullptr};
  float *part = nullptr, *attn_scratch = nullptr, *ssq = nullptr;
  float *q_logits = nullptr, *p_logits = nullptr, *fw_logits = nullptr, *stats = nullptr;
  float* fw_logits2 = nullptr;     // second [32, V] logits buffer, allocated by the first sd_head_examples call
  int32_t* lm_dst = nullptr;       // [MAX_ROWS] logits row of every slot of a ragged target pass
  int32_t* ex_ints = nullptr;      // X, Y, Z, mask staging of sd_head_examples: 4 * max_seq ints
  RowPlan rows{};
  SeqState s{};
  int32_t* result = nullptr;       // device, [B, RESULT_INTS]
  int32_t* pinned = nullptr;       // host, pinned staging
  int32_t* hflags = nullptr;       // host, pinned and coherent: [B] stop flags the draft step's last kernel writes itself
  int32_t* hflags_dev = nullptr;   // the same memory as the device addresses it
  uint32_t tick = 0;               // draft steps issued so far: tags the flag words
  size_t pinned_ints = 0;
  std::vector<void*> allocs;

  // host mirrors of committed state
  std::vector<int> P, kv_t, kv_d, round, active;

  hipEvent_t ev[4]{};
  double last_phase_s[3]{};       // draft loop, target pass, accept + commit of the most recent round
  int last_rows = 0;              // row slots of the most recent target pass
  int prof_every = 0;
  int prof_pass = 0;              // profiled target passes since sd_profile_enable: rotates the sampled layers
  std::vector<ProfSample> prof_pool;
  size_t prof_used = 0;
  int64_t prof_launches[5]{};
  double prof_seconds[5]{}, prof_bytes[5]{};
};

namespace {

sd_status dev_alloc(sd_ctx* c, void** p, size_t bytes, bool zero = false) {
  *p = nullptr;
  if (bytes == 0) bytes = 16;
  hipError_t e = hipMalloc(p, bytes);
  if (e != hipSuccess) { (void)hipGetLastError(); return SD_ENOMEM; }
  c->allocs.push_back(*p);
  if (zero) SD_HIP(hipMemsetAsync(*p, 0, bytes, c->st));
  return SD_OK;
}

bool model_ok(const sd_model* m) {
  if (!m) return false;
  if (m->n_layers < 1 || m->d_model < 1 || m->n_heads < 1 || m->n_kv_heads < 1 || m->head_dim < 2 || m->d_ffn < 1 ||
      m->vocab < 1)
    return false;
  if (m->n_heads % m->n_kv_heads != 0 || (m->head_dim & 1)) return false;
  if (m->dtype != SD_F32 && m->dtype != SD_BF16) return false;
  if (!m->tok_emb || !m->lm_head || !m->final_norm || !m->wqkv || !m->wo || !m->w_gate_up || !m->w_down ||
      !m->norm_attn || !m->norm_mlp)
    return false;
  for (int l = 0; l < m->n_layers; ++l)
    if (!m->wqkv[l] || !m->wo[l] || !m->w_gate_up[l] || !m->w_down[l] || !m->norm_attn[l] || !m->norm_mlp[l])
      return false;
  if (m->dtype == SD_BF16) {
    // the bf16 kernels stream 128-element K steps and 16-row output tiles
    const int nq = m->n_heads * m->head_dim, nkv = m->n_kv_heads * m->head_dim;
    if (m->d_model % 128 || nq % 128 || m->d_ffn % 128 || (nq + 2 * nkv) % 16 || m->vocab % 16) return false;
    if (m->head_dim != 64 && m->head_dim != 128) return false;
  } else {
    if (m->head_dim != 32 && m->head_dim != 64 && m->head_dim != 128) return false;
  }
  return true;
}

void copy_model(ModelRt& rt, const sd_model* m) {
  rt.m = *m;
  const int L = m->n_layers;
  rt.wqkv.assign(m->wqkv, m->wqkv + L);
  rt.wo.assign(m->wo, m->wo + L);
  rt.wgu.assign(m->w_gate_up, m->w_gate_up + L);
  rt.wdown.assign(m->w_down, m->w_down + L);
  rt.na.assign(m->norm_attn, m->norm_attn + L);
  rt.nm.assign(m->norm_mlp, m->norm_mlp + L);
  rt.m.wqkv = rt.wqkv.data();
  rt.m.wo = rt.wo.data();
  rt.m.w_gate_up = rt.wgu.data();
  rt.m.w_down = rt.wdown.data();
  rt.m.norm_attn = rt.na.data();
  rt.m.norm_mlp = rt.nm.data();
  rt.esz = m->dtype == SD_BF16 ? 2 : 4;
}

sd_status alloc_model(sd_ctx* c, ModelRt& rt) {
  const sd_model& m = rt.m;
  rt.layer_bytes = (size_t)c->B * m.n_kv_heads * c->cfg.max_seq * m.head_dim * rt.esz;
  sd_status s;
  // caches start zeroed: the attention kernel multiplies masked probabilities (0) with
  // whatever sits beyond a sequence's length, which must therefore be finite
  if ((s = dev_alloc(c, (void**)&rt.kcache, rt.layer_bytes * m.n_layers, true)) != SD_OK) return s;
  if ((s = dev_alloc(c, (void**)&rt.vcache, rt.layer_bytes * m.n_layers, true)) != SD_OK) return s;
  const int half = m.head_dim / 2;
  std::vector<float> tab((size_t)c->cfg.max_seq * half * 2);
  for (int pos = 0; pos < c->cfg.max_seq; ++pos)
    for (int i = 0; i < half; ++i) {
      const double ang = (double)pos * std::pow((double)m.rope_theta, -2.0 * i / m.head_dim);
      tab[((size_t)pos * half + i) * 2] = (float)std::cos(ang);
      tab[((size_t)pos * half + i) * 2 + 1] = (float)std::sin(ang);
    }
  if ((s = dev_alloc(c, (void**)&rt.cos_sin, tab.size() * sizeof(float))) != SD_OK) return s;
  SD_HIP(hipMemcpy(rt.cos_sin, tab.data(), tab.size() * sizeof(float), hipMemcpyHostToDevice));
  return SD_OK;
}

size_t part_floats_for(int dtype, int max_rows, int N, int K) {
  size_t best = 0;
  for (int M = 1; M <= std::min(max_rows, (int)MAX_ROWS); ++M) {
    const size_t v = (size_t)gemm_splits(dtype, M, N, K) * M * N;
    if (v > best) best = v;
  }
  return best;
}

size_t part_floats(const sd_ctx* c) {
  size_t best = 0;
  for (const ModelRt* rt : {&c->target, &c->draft}) {
    const sd_model& m = rt->m;
    const int shapes[5][2] = {{rt->n_q() + 2 * rt->n_kv(), m.d_model}, {m.d_model, rt->n_q()},
                              {2 * m.d_ffn, m.d_model},               {m.d_model, m.d_ffn},
                              {m.vocab, m.d_model}};
    for (auto& sh : shapes) best = std::max(best, part_floats_for(m.dtype, c->max_rows, sh[0], sh[1]));
    // the prompt pass of a bf16 model: up to prefill_rows rows through the tiled kernel
    if (m.dtype == SD_BF16)
      for (int i = 0; i < 4; ++i)
        for (int M = MAX_ROWS + 1; M <= c->prefill_rows; ++M)
          best = std::max(best, (size_t)gemm_splits(m.dtype, M, shapes[i][0], shapes[i][1]) * M * shapes[i][0]);
  }
  if (c->head.present)
    for (int j = 0; j + 1 < c->head.n_layers; ++j)
      best = std::max(best, part_floats_for(c->head.dtype, c->B, c->head.dims[j + 1], c->head.dims[j]));
  return best;
}

// ---- profiling of the target pass's GEMM launches
ProfSample* prof_begin(sd_ctx* c, int kind, double bytes) {
  if (c->prof_used == c->prof_pool.size()) {
    ProfSample ps{};
    if (hipEventCreate(&ps.a) != hipSuccess || hipEventCreate(&ps.b) != hipSuccess) return nullptr;
    c->prof_pool.push_back(ps);
  }
  ProfSample* ps = &c->prof_pool[c->prof_used++];
  ps->kind = kind;
  ps->bytes = bytes;
  (void)hipEventRecord(ps->a, c->st);
  return ps;
}

// Reading the timers is kept out of the rounds (an elapsed-time query costs the host microseconds, 40 of them
// a good part of a millisecond): samples pile up in the pool until sd_profile_read, or until the pool is large.
constexpr size_t PROF_POOL_SOFT_MAX = 8192;
void prof_collect(sd_ctx* c) {      // stream must be idle
  for (size_t i = 0; i < c->prof_used; ++i) {
    ProfSample& ps = c->prof_pool[i];
    float ms = 0.f;
    if (hipEventElapsedTime(&ms, ps.a, ps.b) == hipSuccess) {
      c->prof_launches[ps.kind] += 1;
      c->prof_seconds[ps.kind] += ms * 1e-3;
      c->prof_bytes[ps.kind] += ps.bytes;
    }
  }
  c->prof_used = 0;
}

// One GEMM, optionally bracketed by events.
sd_status gemm(sd_ctx* c, const ModelRt& rt, const void* W, const void* X, int ldx, const int* xrow, int M, int N,
               int K, int prof_kind, float* out = nullptr) {
  ProfSample* ps = prof_kind >= 0 ? prof_begin(c, prof_kind, (double)N * K * rt.esz) : nullptr;
  SD_HIP(launch_gemm(c->st, rt.m.dtype, W, X, ldx, xrow, out ? out : c->part, M, N, K));
  if (ps) (void)hipEventRecord(ps->b, c->st);
  return SD_OK;
}

// The decoder over the rows of c->rows (M rows in groups of RS).  Leaves the
// final-RMSNorm rows in c->xn.  If logits_out != null, runs the LM head over n_lm rows
// (gathered through lm_rows when non-null); LM row i = (group i / lm_rs, slot i % lm_rs) goes
// to logits_out[group * ld_group + slot * ld_row + v].
// tile = true (prompt pass of a bf16 model, one row group of more than 32 rows): M may reach
// c->prefill_rows; the GEMMs then go through the tiled kernel (launch_gemm picks it by M) and
// attention through its unsplit variant.
sd_status forward(sd_ctx* c, ModelRt& rt, int M, int RS, int max_kv_len, const int* lm_rows, int n_lm,
                  float* logits_out, int lm_rs, int64_t ld_group, int64_t ld_row, bool profile, bool tile = false,
                  const int32_t* lm_dst = nullptr) {
  const sd_model& m = rt.m;
  const int dt = m.dtype, d = m.d_model, nq = rt.n_q(), nkv = rt.n_kv();
  hipStream_t st = c->st;
  if (tile && (dt != SD_BF16 || RS != M || logits_out)) return SD_EINVAL;
  if (!tile && M > MAX_ROWS) return SD_EINVAL;
  auto mm = [&](const void* W, const void* X, int ldx, int N, int K, int prof_kind) -> sd_status {
    return gemm(c, rt, W, X, ldx, nullptr, M, N, K, prof_kind);
  };
  auto slices = [&](int N, int K) { return gemm_splits(dt, M, N, K); };
  const bool fuse_act = gemm_silu_fused(dt, M, m.d_ffn, d);     // gate|up GEMM writes silu(gate) * up itself
  const int res_groups = fuse_act ? gemm_resid_groups(dt, M, d, nq) : 0;   // > 0: residual + norm ride on the o projection
  const int down_groups = gemm_scaled_ok(dt, M, nq + 2 * nkv, d) ? gemm_resid_groups(dt, M, d, m.d_ffn) : 0;   // and on down
  const bool rope_fused = !tile && gemm_rope_fused(dt, M, m.n_heads, m.n_kv_heads, m.head_dim, d);
  int in_groups = 0;            // > 0: xn = x * gain without the rows' norm factors; their sums of squares sit in c->ssq
  SD_HIP(launch_embed_norm(st, dt, m.tok_emb, rt.na[0], m.rms_eps, c->rows.tok, c->x, c->xn, c->ssq, M, d, m.vocab));
  for (int l = 0; l < m.n_layers; ++l) {
    const bool pr = profile && c->prof_every > 0 && ((l + c->prof_pass) % c->prof_every) == 0;
    sd_status s;
    void* kc = rt.kcache + (size_t)l * rt.layer_bytes;
    void* vc = rt.vcache + (size_t)l * rt.layer_bytes;
    if (rope_fused) {             // q|k|v product, rotary embedding and KV append in one launch
      ProfSample* ps = pr ? prof_begin(c, 0, (double)(nq + 2 * nkv) * d * rt.esz) : nullptr;
      SD_HIP(launch_gemm_rope(st, dt, rt.wqkv[l], c->xn, d, M, m.n_heads, m.n_kv_heads, m.head_dim, d, c->rows.seq,
                              c->rows.pos, rt.cos_sin, c->qbuf, kc, vc, c->cfg.max_seq,
                              in_groups > 0 ? c->ssq : nullptr, in_groups, d, m.rms_eps));
      if (ps) (void)hipEventRecord(ps->b, st);
    } else {
      if (in_groups > 0) {        // the rows of xn still lack their RMSNorm factor (previous layer's down projection)
        ProfSample* ps = pr ? prof_begin(c, 0, (double)(nq + 2 * nkv) * d * rt.esz) : nullptr;
        SD_HIP(launch_gemm_scaled(st, dt, rt.wqkv[l], c->xn, d, nullptr, c->part, M, nq + 2 * nkv, d, c->ssq, in_groups,
                                  d, m.rms_eps));
        if (ps) (void)hipEventRecord(ps->b, st);
      } else if ((s = mm(rt.wqkv[l], c->xn, d, nq + 2 * nkv, d, pr ? 0 : -1)) != SD_OK) {
        return s;
      }
      SD_HIP(launch_rope_kv(st, dt, c->part, slices(nq + 2 * nkv, d), c->rows, rt.cos_sin, c->qbuf, kc, vc,
                            M, m.n_heads, m.n_kv_heads, m.head_dim, c->cfg.max_seq));
    }
    SD_HIP(launch_attention(st, dt, c->qbuf, kc, vc, c->rows, c->attn, c->attn_scratch, M, RS, m.n_heads,
                            m.n_kv_heads, m.head_dim, c->cfg.max_seq, max_kv_len, tile));
    if (res_groups > 0) {
      // the output projection adds itself to the residual rows and leaves x * gain for the MLP, whose first
      // product applies the rows' RMSNorm factors to its sums: no launch between the two products
      ProfSample* ps = pr ? prof_begin(c, 1, (double)d * nq * rt.esz) : nullptr;
      SD_HIP(launch_gemm_resid(st, dt, rt.wo[l], c->attn, nq, nullptr, c->x, rt.nm[l], c->xn, c->ssq, M, d, nq));
      if (ps) (void)hipEventRecord(ps->b, st);
    } else {
      if ((s = mm(rt.wo[l], c->attn, nq, d, nq, pr ? 1 : -1)) != SD_OK) return s;
      SD_HIP(launch_add_norm(st, dt, c->part, slices(d, nq), rt.nm[l], m.rms_eps, c->x, c->xn, c->ssq, M, d));
    }
    if (fuse_act) {
      ProfSample* ps = pr ? prof_begin(c, 2, 2.0 * m.d_ffn * d * rt.esz) : nullptr;
      SD_HIP(launch_gemm_silu(st, dt, rt.wgu[l], c->xn, d, nullptr, c->act, M, m.d_ffn, d,
                              res_groups > 0 ? c->ssq : nullptr, res_groups, d, m.rms_eps));
      if (ps) (void)hipEventRecord(ps->b, st);
    } else {
      if ((s = mm(rt.wgu[l], c->xn, d, 2 * m.d_ffn, d, pr ? 2 : -1)) != SD_OK) return s;
      SD_HIP(launch_silu_mul(st, dt, c->part, slices(2 * m.d_ffn, d), c->act, M, m.d_ffn));
    }
    const void* g_next = (l + 1 < m.n_layers) ? rt.na[l + 1] : m.final_norm;
    if (down_groups > 0 && l + 1 < m.n_layers) {
      // same for the MLP's output: the down projection adds itself to the residual rows, the next layer's q|k|v
      // product applies the norm factors (the last layer keeps the separate kernel: its rows feed the LM head)
      ProfSample* ps = pr ? prof_begin(c, 3, (double)d * m.d_ffn * rt.esz) : nullptr;
      SD_HIP(launch_gemm_resid(st, dt, rt.wdown[l], c->act, m.d_ffn, nullptr, c->x, g_next, c->xn, c->ssq, M, d,
                               m.d_ffn));
      if (ps) (void)hipEventRecord(ps->b, st);
      in_groups = down_groups;
    } else {
      if ((s = mm(rt.wdown[l], c->act, m.d_ffn, d, m.d_ffn, pr ? 3 : -1)) != SD_OK) return s;
      SD_HIP(launch_add_norm(st, dt, c->part, slices(d, m.d_ffn), g_next, m.rms_eps, c->x, c->xn, c->ssq, M, d));
      in_groups = 0;
    }
  }
  if (logits_out) {
    sd_status s;
    // one slice whose rows land back to back in the logits array (one sequence): the product writes them itself
    const int S = gemm_splits(dt, n_lm, m.vocab, d);
    const bool direct = S == 1 && !lm_dst && ld_row == m.vocab && n_lm <= lm_rs && m.vocab % 4 == 0;
    if ((s = gemm(c, rt, m.lm_head, c->xn, d, lm_rows, n_lm, m.vocab, d, profile && c->prof_every > 0 ? 4 : -1,
                  direct ? logits_out : nullptr)) != SD_OK)
      return s;
    if (!direct)
      SD_HIP(launch_reduce_rows(st, c->part, S, logits_out, lm_rs, ld_group, ld_row, n_lm, m.vocab, lm_dst));
  }
  if (profile && c->prof_every > 0) ++c->prof_pass;        // the next pass samples the layers one further
  return SD_OK;
}

// Acceptance head's hidden layers on the newest row of every sequence; returns the
// buffer / row map / width the last (linear) layer reads.
sd_status head_hidden(sd_ctx* c, const void** z, const int** z_rows, int* z_dim) {
  const HeadRt& h = c->head;
  const void* cur = c->xn;
  const int* cur_rows = c->s.last_row;
  for (int j = 0; j + 1 < h.n_layers; ++j) {
    const int K = h.dims[j], N = h.dims[j + 1];
    void* out = c->hz[j & 1];
    const bool skip = h.residual && N == K;
    if (gemm_head_fused(h.dtype, c->B, N, K)) {        // bias, SiLU and the skip connection ride on the product
      SD_HIP(launch_gemm_head(c->st, h.dtype, h.W[j], cur, K, cur_rows, h.b[j], skip ? cur : nullptr, cur_rows, out,
                              c->B, N, K));
    } else {
      SD_HIP(launch_gemm(c->st, h.dtype, h.W[j], cur, K, cur_rows, c->part, c->B, N, K));
      SD_HIP(launch_head_act(c->st, h.dtype, c->part, gemm_splits(h.dtype, c->B, N, K), h.b[j], cur, cur_rows, out,
                             skip ? 1 : 0, c->B, N));
    }
    cur = out;
    cur_rows = nullptr;
  }
  *z = cur;
  *z_rows = cur_rows;
  *z_dim = h.dims[h.n_layers - 1];
  return SD_OK;
}

// Host-planned rows (prefill and teacher-forced forward): tokens at consecutive
// positions of one sequence.
sd_status plan_host_rows(sd_ctx* c, int seq, int start, const int32_t* toks, int n) {
  int32_t* h = c->pinned;
  for (int i = 0; i < n; ++i) {
    h[i] = seq;
    h[MAX_PREFILL_ROWS + i] = start + i;
    h[2 * MAX_PREFILL_ROWS + i] = toks[i];
  }
  SD_HIP(hipMemcpyAsync(c->rows.seq, h, n * sizeof(int32_t), hipMemcpyHostToDevice, c->st));
  SD_HIP(hipMemcpyAsync(c->rows.pos, h + MAX_PREFILL_ROWS, n * sizeof(int32_t), hipMemcpyHostToDevice, c->st));
  SD_HIP(hipMemcpyAsync(c->rows.tok, h + 2 * MAX_PREFILL_ROWS, n * sizeof(int32_t), hipMemcpyHostToDevice, c->st));
  h[3 * MAX_PREFILL_ROWS] = seq;                 // one row group: the whole chunk
  h[3 * MAX_PREFILL_ROWS + 1] = start + n;
  SD_HIP(hipMemcpyAsync(c->rows.gseq, h + 3 * MAX_PREFILL_ROWS, sizeof(int32_t), hipMemcpyHostToDevice, c->st));
  SD_HIP(hipMemcpyAsync(c->rows.gend, h + 3 * MAX_PREFILL_ROWS + 1, sizeof(int32_t), hipMemcpyHostToDevice, c->st));
  return SD_OK;
}

sd_status set_dev_int(sd_ctx* c, int32_t* arr, int idx, int32_t v) {
  SD_HIP(hipMemcpy(arr + idx, &v, sizeof(v), hipMemcpyHostToDevice));
  return SD_OK;
}

float bf16_to_float(uint16_t h) {
  uint32_t u = (uint32_t)h << 16;
  float f;
  std::memcpy(&f, &u, 4);
  return f;
}

DecodeParams to_dp(const sd_params* p) {
  return DecodeParams{p->h, p->temperature, p->greedy, p->eos_id, p->seed, p->top_k};
}

bool params_ok(const sd_params* p) {
  return p && p->temperature > 0.f && std::isfinite(p->temperature) && !std::isnan(p->h) && p->top_k >= 0 &&
         p->reserved == 0;
}

}  // namespace

// =============================================================================== C ABI
#pragma GCC visibility push(default)
extern "C" {

const char* sd_strerror(sd_status s) {
  switch (s) {
    case SD_OK: return "ok";
    case SD_EINVAL: return "invalid argument";
    case SD_ENOMEM: return "out of memory";
    case SD_ERANGE: return "sequence or token id out of range";
    case SD_ENONFINITE: return "non-finite logits";
    case SD_EDEVICE: return "HIP error";
    default: return "unknown status";
  }
}

const char* sd_version(void) { return "specdec-gfx950 0.1"; }

sd_status sd_destroy(sd_ctx* c) {
  if (!c) return SD_EINVAL;
  (void)hipStreamSynchronize(c->st);
  for (void* p : c->allocs) (void)hipFree(p);
  if (c->pinned) (void)hipHostFree(c->pinned);
  if (c->hflags) (void)hipHostFree(c->hflags);
  for (auto& e : c->ev)
    if (e) (void)hipEventDestroy(e);
  for (auto& ps : c->prof_pool) {
    (void)hipEventDestroy(ps.a);
    (void)hipEventDestroy(ps.b);
  }
  delete c;
  return SD_OK;
}

sd_status sd_create(sd_ctx** out, const sd_model* target, const sd_model* draft, const sd_head* head,
                    const sd_config* cfg) {
  if (!out || !cfg) return SD_EINVAL;
  *out = nullptr;
  if (!model_ok(target) || !model_ok(draft)) return SD_EINVAL;
  if (target->vocab != draft->vocab) return SD_EINVAL;
  if (cfg->batch < 1 || cfg->k_max < 1 || cfg->k_max > SD_MAX_K || cfg->max_seq < 64 || cfg->max_seq % 64 != 0)
    return SD_EINVAL;
  if (cfg->batch * (cfg->k_max + 1) > MAX_ROWS) return SD_EINVAL;
  // what the attention kernels take: 512 key blocks of 64 (bf16); a prefix of scores in 64 KB of LDS (fp32)
  for (const sd_model* m : {target, draft})
    if (cfg->max_seq > (m->dtype == SD_BF16 ? 32768 : 12288)) return SD_EINVAL;
  if (head) {
    if (head->n_layers < 1 || head->n_layers > SD_MAX_HEAD_LAYERS || !head->dims || !head->W || !head->b)
      return SD_EINVAL;
    if (head->dims[0] != draft->d_model || head->dims[head->n_layers] != 1 || head->dtype != draft->dtype)
      return SD_EINVAL;
    for (int j = 0; j < head->n_layers; ++j) {
      if (!head->W[j] || !head->b[j] || head->dims[j] < 1) return SD_EINVAL;
      if (head->dtype == SD_BF16 && j + 1 < head->n_layers && (head->dims[j] % 128 || head->dims[j + 1] % 16))
        return SD_EINVAL;
    }
  }
  sd_ctx* c = new (std::nothrow) sd_ctx();
  if (!c) return SD_ENOMEM;
  c->cfg = *cfg;
  c->st = (hipStream_t)cfg->hip_stream;
  c->B = cfg->batch;
  const bool any_bf16 = target->dtype == SD_BF16 || draft->dtype == SD_BF16;
  c->prefill_rows = any_bf16 ? std::min((int)MAX_PREFILL_ROWS, cfg->max_seq) : PREFILL_CHUNK;
  c->max_rows = std::max(std::max(PREFILL_CHUNK, c->prefill_rows), std::max(c->B * (cfg->k_max + 1), 2 * c->B));
  copy_model(c->target, target);
  copy_model(c->draft, draft);
  if (head) {
    c->head.present = true;
    c->head.n_layers = head->n_layers;
    c->head.residual = head->residual;
    c->head.dtype = head->dtype;
    c->head.dims.assign(head->dims, head->dims + head->n_layers + 1);
    c->head.W.assign(head->W, head->W + head->n_layers);
    c->head.b.assign(head->b, head->b + head->n_layers);
  }
  sd_status s = SD_OK;
  auto fail = [&](sd_status e) { sd_destroy(c); return e; };
  if ((s = alloc_model(c, c->target)) != SD_OK) return fail(s);
  if ((s = alloc_model(c, c->draft)) != SD_OK) return fail(s);

  const int R = c->max_rows, B = c->B, V = target->vocab;
  const int dmax = std::max(target->d_model, draft->d_model);
  const int nqmax = std::max(c->target.n_q(), c->draft.n_q());
  const int ffmax = std::max(target->d_ffn, draft->d_ffn);
  size_t hzmax = 16;
  if (head)
    for (int j = 1; j < head->n_layers; ++j) hzmax = std::max(hzmax, (size_t)head->dims[j]);
  size_t attn_fl = 16;
  for (const ModelRt* rt : {&c->target, &c->draft})
    if (rt->m.dtype == SD_BF16)
      attn_fl = std::max(attn_fl, attn_scratch_floats(std::min(R, (int)MAX_ROWS), rt->m.n_heads, rt->m.head_dim, cfg->max_seq));

#define SD_ALLOC(ptr, bytes, zero)                                              \
  if ((s = dev_alloc(c, (void**)&(ptr), (bytes), (zero))) != SD_OK) return fail(s)
  SD_ALLOC(c->x, (size_t)R * dmax * 4, true);
  SD_ALLOC(c->xn, (size_t)R * dmax * 4, true);
  SD_ALLOC(c->qbuf, (size_t)R * nqmax * 4, true);
  SD_ALLOC(c->attn, (size_t)R * nqmax * 4, true);
  SD_ALLOC(c->act, (size_t)R * ffmax * 4, true);
  SD_ALLOC(c->hz[0], (size_t)B * hzmax * 4, true);
  SD_ALLOC(c->hz[1], (size_t)B * hzmax * 4, true);
  SD_ALLOC(c->part, part_floats(c) * 4, false);
  SD_ALLOC(c->attn_scratch, attn_fl * 4, false);
  SD_ALLOC(c->ssq, (size_t)MAX_PREFILL_ROWS * NORM_MAX_BLOCKS * 4, true);
  SD_ALLOC(c->q_logits, (size_t)B * cfg->k_max * V * 4, true);
  SD_ALLOC(c->p_logits, (size_t)B * (cfg->k_max + 1) * V * 4, true);
  SD_ALLOC(c->fw_logits, (size_t)PREFILL_CHUNK * V * 4, true);
  SD_ALLOC(c->stats, (size_t)B * (2 * cfg->k_max + 1) * 4 * 4, true);
  SD_ALLOC(c->rows.seq, MAX_PREFILL_ROWS * 4, true);
  SD_ALLOC(c->rows.pos, MAX_PREFILL_ROWS * 4, true);
  SD_ALLOC(c->rows.tok, MAX_PREFILL_ROWS * 4, true);
  SD_ALLOC(c->rows.gseq, MAX_PREFILL_ROWS * 4, true);
  SD_ALLOC(c->rows.gend, MAX_PREFILL_ROWS * 4, true);
  SD_ALLOC(c->s.P, B * 4, true);
  SD_ALLOC(c->s.kv_t, B * 4, true);
  SD_ALLOC(c->s.kv_d, B * 4, true);
  SD_ALLOC(c->s.K, B * 4, true);
  SD_ALLOC(c->s.kcap, B * 4, true);
  SD_ALLOC(c->s.stopped, B * 4, true);
  SD_ALLOC(c->s.p_hat, B * 4, true);
  SD_ALLOC(c->s.cand, B * CAND_LD * 4, true);
  SD_ALLOC(c->s.n_acc, B * 4, true);
  SD_ALLOC(c->s.y_new, B * 4, true);
  SD_ALLOC(c->s.tokens, (size_t)B * cfg->max_seq * 4, true);
  SD_ALLOC(c->s.head_s, B * CAND_LD * 4, true);
  SD_ALLOC(c->s.flags, B * CAND_LD, true);
  SD_ALLOC(c->s.round, B * 4, true);
  SD_ALLOC(c->s.last_row, B * 4, true);
  SD_ALLOC(c->s.err, 16, true);
  SD_ALLOC(c->s.active, B * 4, true);
  SD_ALLOC(c->result, (size_t)B * RESULT_INTS * 4, true);
  SD_ALLOC(c->lm_dst, MAX_ROWS * 4, true);
#undef SD_ALLOC
  c->pinned_ints = std::max<size_t>(3 * MAX_PREFILL_ROWS + 2, (size_t)B * RESULT_INTS) + 64;
  if (hipHostMalloc((void**)&c->pinned, c->pinned_ints * 4, hipHostMallocDefault) != hipSuccess) return fail(SD_ENOMEM);
  if (hipHostMalloc((void**)&c->hflags, (size_t)B * 4, hipHostMallocCoherent | hipHostMallocMapped) != hipSuccess)
    return fail(SD_ENOMEM);
  std::memset(c->hflags, 0, (size_t)B * 4);
  if (hipHostGetDevicePointer((void**)&c->hflags_dev, c->hflags, 0) != hipSuccess) return fail(SD_EDEVICE);
  for (auto& e : c->ev)
    if (hipEventCreate(&e) != hipSuccess) return fail(SD_EDEVICE);
  c->P.assign(B, 0);
  c->kv_t.assign(B, 0);
  c->kv_d.assign(B, 0);
  c->round.assign(B, 0);
  c->active.assign(B, 0);
  if (hipStreamSynchronize(c->st) != hipSuccess) return fail(SD_EDEVICE);
  *out = c;
  return SD_OK;
}

sd_status sd_prefill(sd_ctx* c, int32_t seq, const int32_t* prompt, int32_t n) {
  if (!c || !prompt || seq < 0 || seq >= c->B || n < 1) return SD_EINVAL;
  if (n + 2 > c->cfg.max_seq) return SD_ERANGE;
  for (int i = 0; i < n; ++i)
    if (prompt[i] < 0 || prompt[i] >= c->target.m.vocab) return SD_ERANGE;
  SD_HIP(hipStreamSynchronize(c->st));
  SD_HIP(hipMemcpy(c->s.tokens + (size_t)seq * c->cfg.max_seq, prompt, n * sizeof(int32_t), hipMemcpyHostToDevice));
  sd_status s;
  for (ModelRt* rt : {&c->target, &c->draft}) {
    // bf16 models take the prompt in chunks of up to prefill_rows rows through the tiled
    // GEMM (bound by the matrix cores); fp32 (tiny) models in 32-row chunks
    const bool bf16 = rt->m.dtype == SD_BF16;
    const int chunk = bf16 ? c->prefill_rows : PREFILL_CHUNK;
    for (int start = 0; start < n - 1; start += chunk) {
      const int m = std::min(chunk, n - 1 - start);
      const bool tile = bf16 && m > PREFILL_CHUNK;     // a short chunk is weight-bound: streaming kernel
      if ((s = plan_host_rows(c, seq, start, prompt + start, m)) != SD_OK) return s;
      if ((s = forward(c, *rt, m, m, start + m, nullptr, 0, nullptr, 1, 0, 0, false, tile)) != SD_OK) return s;
      SD_HIP(hipStreamSynchronize(c->st));
    }
  }
  if ((s = set_dev_int(c, c->s.P, seq, n)) != SD_OK) return s;
  if ((s = set_dev_int(c, c->s.kv_t, seq, n - 1)) != SD_OK) return s;
  if ((s = set_dev_int(c, c->s.kv_d, seq, n - 1)) != SD_OK) return s;
  if ((s = set_dev_int(c, c->s.round, seq, 0)) != SD_OK) return s;
  if ((s = set_dev_int(c, c->s.active, seq, 1)) != SD_OK) return s;
  if ((s = set_dev_int(c, c->s.err, 0, 0)) != SD_OK) return s;
  c->P[seq] = n;
  c->kv_t[seq] = c->kv_d[seq] = n - 1;
  c->round[seq] = 0;
  c->active[seq] = 1;
  return SD_OK;
}

// Stop flags of the draft step tagged `tick` into c->pinned[0..B).  The flag words arrive in host memory when the
// step's last kernel ends; the wait is a bounded watch of those words (a step takes milliseconds), and if they do not
// show within the bound (a runtime that does not make such stores visible before a synchronisation, a failed
// launch) the stream is synchronised and the flags are copied from the device instead, so a wrong answer is not possible.
static sd_status wait_stop_flags(sd_ctx* c, uint32_t tick) {
  const int B = c->B;
  volatile const int32_t* hf = c->hflags;
  const auto t0 = std::chrono::steady_clock::now();
  for (uint32_t spins = 0;; ++spins) {
    bool ready = true;
    for (int b = 0; b < B; ++b) ready = ready && ((uint32_t)hf[b] >> 1) == tick;
    if (ready) {
      for (int b = 0; b < B; ++b) c->pinned[b] = hf[b] & 1;
      return SD_OK;
    }
    if ((spins & 0x3ff) == 0x3ff &&
        std::chrono::duration<double>(std::chrono::steady_clock::now() - t0).count() > 0.25)
      break;
  }
  SD_HIP(hipMemcpyAsync(c->pinned, c->s.stopped, B * sizeof(int32_t), hipMemcpyDeviceToHost, c->st));
  SD_HIP(hipStreamSynchronize(c->st));
  return SD_OK;
}

static sd_status round_impl(sd_ctx* c, const sd_params* params, sd_round_out* out, sd_stats* stats) {
  const int B = c->B, k_max = c->cfg.k_max, max_seq = c->cfg.max_seq, V = c->target.m.vocab;
  int maxP = 0, n_active = 0;
  for (int b = 0; b < B; ++b) {
    if (!c->active[b]) continue;
    ++n_active;
    if (c->P[b] < 1) return SD_EINVAL;                       // not prefilled
    if (std::min(k_max, max_seq - c->P[b] - 1) < 1) return SD_ERANGE;
    maxP = std::max(maxP, c->P[b]);
  }
  if (n_active == 0) return SD_EINVAL;
  const DecodeParams dp = to_dp(params);
  hipStream_t st = c->st;
  sd_status s;

  SD_HIP(launch_begin_round(st, c->s, B, k_max, max_seq));
  SD_HIP(hipEventRecord(c->ev[0], st));
  // ---- adaptive draft loop (Algorithm 2's first block)
  int k_round = k_max;                      // largest K of the round = draft steps taken
  std::vector<int> k_seq(B, 0);             // per-sequence K as the stop flags reveal it (0: not yet stopped)
  for (int step = 1; step <= k_max; ++step) {
    SD_HIP(launch_plan_draft(st, c->s, c->rows, B, step, max_seq));
    const int kv_bound = std::min(max_seq, maxP + step);
    if ((s = forward(c, c->draft, 2 * B, 2, kv_bound, c->s.last_row, B, c->q_logits + (size_t)(step - 1) * V, 1,
                     (int64_t)k_max * V, V, false)) != SD_OK)
      return s;
    const void* z = nullptr;
    const int* z_rows = nullptr;
    int z_dim = 0;
    const bool use_head = c->head.present && step > 1;
    if (use_head && (s = head_hidden(c, &z, &z_rows, &z_dim)) != SD_OK) return s;
    // the step's last kernel writes every sequence's stop flag, tagged with the step's number, into coherent host
    // memory: the host watches that word instead of draining the stream through a copy and a synchronisation
    const uint32_t tick = (++c->tick) & 0x3fffffffu;
    SD_HIP(launch_sample_stop(st, c->draft.m.dtype, c->s, c->q_logits, (int64_t)k_max * V, z, z_rows, z_dim,
                              use_head ? c->head.W[c->head.n_layers - 1] : nullptr,
                              use_head ? c->head.b[c->head.n_layers - 1] : nullptr, use_head ? 1 : 0, dp, B, V,
                              step, c->hflags_dev, tick));
    if (step < k_max) {
      if ((s = wait_stop_flags(c, tick)) != SD_OK) return s;
      bool all = true;
      for (int b = 0; b < B; ++b) {
        all = all && c->pinned[b] != 0;
        if (c->pinned[b] != 0 && k_seq[b] == 0 && c->active[b]) k_seq[b] = step;
      }
      if (all) {
        k_round = step;
        break;
      }
    }
  }
  SD_HIP(hipEventRecord(c->ev[1], st));
  // ---- target pass over the K+1 positions (row slots sized by this round's largest K)
  // One sequence: its K+1 rows are one group.  Several: K differs between sequences, so each takes
  // ceil((K_b+1)/4) groups of 4 row slots, packed, instead of max_b(K_b)+1 slots each; the GEMMs then
  // carry sum_b (K_b+1) rows plus at most 3 padding rows per sequence.
  const int rs = k_round + 1;
  constexpr int RAGGED_RS = 4;
  int n_groups = 0;
  for (int b = 0; b < B; ++b)
    if (c->active[b]) n_groups += ((k_seq[b] ? k_seq[b] : k_round) + RAGGED_RS) / RAGGED_RS;
  if (B > 1 && n_groups * RAGGED_RS < B * rs && n_groups * RAGGED_RS <= MAX_ROWS) {
    const int Mv = n_groups * RAGGED_RS;
    c->last_rows = Mv;
    SD_HIP(launch_plan_verify_ragged(st, c->s, c->rows, B, RAGGED_RS, n_groups, k_max, max_seq, c->lm_dst));
    if ((s = forward(c, c->target, Mv, RAGGED_RS, std::min(max_seq, maxP + k_round), nullptr, Mv, c->p_logits,
                     RAGGED_RS, 0, V, true, false, c->lm_dst)) != SD_OK)
      return s;
  } else {
    const int Mv = B * rs;
    c->last_rows = Mv;
    SD_HIP(launch_plan_verify(st, c->s, c->rows, B, rs, max_seq));
    if ((s = forward(c, c->target, Mv, rs, std::min(max_seq, maxP + k_round), nullptr, Mv, c->p_logits, rs,
                     (int64_t)(k_max + 1) * V, V, true)) != SD_OK)
      return s;
  }
  SD_HIP(hipEventRecord(c->ev[2], st));
  // ---- accept / residual resample, commit, rollback
  float* p_stats = c->stats;
  float* q_stats = c->stats + (size_t)B * (k_max + 1) * 4;
  SD_HIP(launch_row_stats(st, c->p_logits, c->q_logits, k_max, c->s.K, B, V, dp.temperature, dp.top_k, p_stats, q_stats,
                          c->s.err));
  SD_HIP(launch_accept(st, c->p_logits, c->q_logits, p_stats, q_stats, c->s.cand, CAND_LD, c->s.K, c->s.round, 0, dp,
                       B, k_max, V, c->s.n_acc, c->s.y_new, c->s.flags, CAND_LD));
  SD_HIP(launch_commit(st, c->s, c->result, B, max_seq));
  SD_HIP(hipEventRecord(c->ev[3], st));
  SD_HIP(hipMemcpyAsync(c->pinned, c->result, (size_t)B * RESULT_INTS * sizeof(int32_t), hipMemcpyDeviceToHost, st));
  SD_HIP(hipStreamSynchronize(st));
  if (c->prof_used > PROF_POOL_SOFT_MAX) prof_collect(c);

  bool nonfinite = false;
  for (int b = 0; b < B; ++b) {
    const int32_t* r = c->pinned + (size_t)b * RESULT_INTS;
    nonfinite = nonfinite || r[39] != 0;
    if (c->active[b]) {
      c->P[b] = r[36];
      c->kv_t[b] = r[37];
      c->kv_d[b] = r[38];
      c->round[b] += 1;
    }
    if (out) {
      sd_round_out& o = out[b];
      std::memset(&o, 0, sizeof(o));
      if (!c->active[b]) continue;
      o.K = r[0];
      o.n_accepted = r[1];
      o.n_new = r[1] + 1;
      for (int i = 0; i < o.n_accepted; ++i) o.tokens[i] = r[4 + i];
      o.tokens[o.n_accepted] = r[2];
      for (int i = 0; i < SD_MAX_K; ++i) o.cand[i] = r[4 + i];
      std::memcpy(&o.p_hat, &r[3], 4);
    }
  }
  for (int k = 0; k < 3; ++k) {
    float ms = 0.f;
    c->last_phase_s[k] = hipEventElapsedTime(&ms, c->ev[k], c->ev[k + 1]) == hipSuccess ? ms * 1e-3 : 0.0;
  }
  if (stats) {
    stats->t_draft_s += c->last_phase_s[0];
    stats->t_target_s += c->last_phase_s[1];
    stats->t_accept_s += c->last_phase_s[2];
  }
  return nonfinite ? SD_ENONFINITE : SD_OK;
}

sd_status specdec_round(sd_ctx* c, const sd_params* params, sd_round_out* out) {
  if (!c || !out || !params_ok(params)) return SD_EINVAL;
  return round_impl(c, params, out, nullptr);
}

sd_status specdec_generate(sd_ctx* c, const sd_params* params, int32_t max_new, int32_t* out_tokens, int32_t* out_lens,
                           sd_stats* stats) {
  if (!c || !out_tokens || !out_lens || !params_ok(params) || max_new < 1) return SD_EINVAL;
  const int B = c->B;
  std::vector<sd_round_out> ro(B);
  std::vector<int> len(B, 0);
  std::vector<int32_t> toks((size_t)B * max_new, 0);
  std::vector<int> was_active(c->active);
  sd_stats st{};
  const auto t0 = std::chrono::steady_clock::now();
  sd_status rc = SD_OK;
  for (;;) {
    bool any = false;
    for (int b = 0; b < B; ++b) any = any || c->active[b];
    if (!any) break;
    rc = round_impl(c, params, ro.data(), &st);
    if (rc != SD_OK) break;
    st.rounds += 1;
    for (int b = 0; b < B; ++b) {
      if (!c->active[b]) continue;
      const sd_round_out& o = ro[b];
      int n_new = o.n_new;
      bool finished = false;
      if (params->eos_id >= 0)
        for (int i = 0; i < n_new; ++i)
          if (o.tokens[i] == params->eos_id) { n_new = i + 1; finished = true; break; }
      const int keep = std::min(n_new, max_new - len[b]);
      for (int i = 0; i < keep; ++i) toks[(size_t)b * max_new + len[b] + i] = o.tokens[i];
      len[b] += keep;
      st.N += keep;
      st.N_draft += o.K;
      st.N_target += 1;
      st.N_discarded += o.K - o.n_accepted;
      if (finished || len[b] >= max_new) {
        c->active[b] = 0;
        sd_status e = set_dev_int(c, c->s.active, b, 0);
        if (e != SD_OK) { rc = e; break; }
      }
    }
    if (rc != SD_OK) break;
  }
  st.t_total_s = std::chrono::duration<double>(std::chrono::steady_clock::now() - t0).count();
  // sequences that were live on entry stay usable for further calls
  for (int b = 0; b < B; ++b)
    if (was_active[b] && !c->active[b]) {
      c->active[b] = 1;
      (void)set_dev_int(c, c->s.active, b, 1);
    }
  if (rc != SD_OK) return rc;
  std::memcpy(out_tokens, toks.data(), toks.size() * sizeof(int32_t));
  for (int b = 0; b < B; ++b) out_lens[b] = len[b];
  if (stats) *stats = st;
  return SD_OK;
}

int64_t sd_accept_workspace_bytes(int32_t B, int32_t Kmax) {
  if (B < 1 || Kmax < 1) return 0;
  return (int64_t)B * (2 * Kmax + 1) * 16 + 16;
}

static sd_status accept_resample_on(const float* p_logits, const float* q_logits, const int32_t* cand,
                                    const int32_t* K, int32_t B, int32_t Kmax, int32_t V, const sd_params* params,
                                    int32_t round_idx, void* ws, hipStream_t st, int32_t* n_out, int32_t* tok_out,
                                    uint8_t* flags) {
  const DecodeParams dp = to_dp(params);
  float* p_stats = (float*)ws;
  float* q_stats = p_stats + (size_t)B * (Kmax + 1) * 4;
  int32_t* oob = (int32_t*)(p_stats + (size_t)B * (2 * Kmax + 1) * 4);      // the status word behind the statistics
  SD_HIP(launch_row_stats(st, p_logits, q_logits, Kmax, K, B, V, dp.temperature, dp.top_k, p_stats, q_stats, nullptr, oob));
  SD_HIP(launch_accept(st, p_logits, q_logits, p_stats, q_stats, cand, Kmax, K, nullptr, round_idx, dp, B, Kmax, V,
                       n_out, tok_out, flags, Kmax, oob));
  return SD_OK;
}

sd_status sd_accept_resample(const float* p_logits, const float* q_logits, const int32_t* cand, const int32_t* K,
                             int32_t B, int32_t Kmax, int32_t V, const sd_params* params, int32_t round_idx,
                             void* ws, void* hip_stream, int32_t* n_out, int32_t* tok_out, uint8_t* flags) {
  if (!p_logits || !q_logits || !cand || !K || !ws || !n_out || !tok_out || !flags || !params_ok(params))
    return SD_EINVAL;
  if (B < 1 || Kmax < 1 || Kmax > SD_MAX_K || V < 1) return SD_EINVAL;
  if (reinterpret_cast<uintptr_t>(ws) & 15) return SD_EINVAL;
  return accept_resample_on(p_logits, q_logits, cand, K, B, Kmax, V, params, round_idx, ws, (hipStream_t)hip_stream,
                            n_out, tok_out, flags);
}

// ---- the same step for callers that cannot allocate: the row statistics live in a file-scope device array.
// Every GPU holds its own copy of the array at its own address; the address is looked up once per device.
namespace {
constexpr int STATIC_ACCEPT_MAX_B = SD_ACCEPT_STATIC_MAX_BATCH;
constexpr size_t STATIC_ACCEPT_BYTES = (size_t)STATIC_ACCEPT_MAX_B * (2 * SD_MAX_K + 1) * 16 + 16;
constexpr int MAX_DEVICES = 64;
}  // namespace
static __device__ __align__(256) unsigned char scratch[STATIC_ACCEPT_BYTES];

static sd_status static_scratch_ptr(void** out) {
  static std::mutex mu;
  static void* ptr_of_device[MAX_DEVICES] = {};
  int dev = -1;
  SD_HIP(hipGetDevice(&dev));
  if (dev < 0 || dev >= MAX_DEVICES) return SD_EDEVICE;
  std::lock_guard<std::mutex> lock(mu);
  if (!ptr_of_device[dev]) {
    void* p = nullptr;
    SD_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
    if (!p) return SD_EDEVICE;
    ptr_of_device[dev] = p;
  }
  *out = ptr_of_device[dev];
  return SD_OK;
}

sd_status sd_accept_resample_static(const float* p_logits, const float* q_logits, const int32_t* cand,
                                    const int32_t* K, int32_t B, int32_t Kmax, int32_t V, const sd_params* params,
                                    int32_t round_idx, void* hip_stream, int32_t* n_out, int32_t* tok_out,
                                    uint8_t* flags, int32_t** status_word_dev) {
  if (!p_logits || !q_logits || !cand || !K || !n_out || !tok_out || !flags || !params_ok(params)) return SD_EINVAL;
  if (B < 1 || Kmax < 1 || Kmax > SD_MAX_K || V < 1) return SD_EINVAL;
  if (B > STATIC_ACCEPT_MAX_B) return SD_ERANGE;            // beyond the static array: use sd_accept_resample
  void* ws = nullptr;
  sd_status s = static_scratch_ptr(&ws);
  if (s != SD_OK) return s;
  if (status_word_dev) *status_word_dev = (int32_t*)((float*)ws + (size_t)B * (2 * Kmax + 1) * 4);
  // nothing in the array has to start at zero: every statistic a call reads it has written before, and the status
  // word is cleared by the first kernel
  return accept_resample_on(p_logits, q_logits, cand, K, B, Kmax, V, params, round_idx, ws, (hipStream_t)hip_stream,
                            n_out, tok_out, flags);
}

sd_status sd_forward(sd_ctx* c, int32_t which, int32_t seq, int32_t start, const int32_t* tokens, int32_t n,
                     float* logits_host, float* hidden_host) {
  if (!c || !tokens || (which != 0 && which != 1) || seq < 0 || seq >= c->B || n < 1 || n > PREFILL_CHUNK || start < 0)
    return SD_EINVAL;
  ModelRt& rt = which == 0 ? c->target : c->draft;
  std::vector<int>& kv = which == 0 ? c->kv_t : c->kv_d;
  if (start > kv[seq]) return SD_EINVAL;
  if (start + n > c->cfg.max_seq) return SD_ERANGE;
  for (int i = 0; i < n; ++i)
    if (tokens[i] < 0 || tokens[i] >= rt.m.vocab) return SD_ERANGE;
  sd_status s;
  SD_HIP(hipStreamSynchronize(c->st));
  if ((s = plan_host_rows(c, seq, start, tokens, n)) != SD_OK) return s;
  const int V = rt.m.vocab, d = rt.m.d_model;
  if ((s = forward(c, rt, n, n, start + n, nullptr, n, logits_host ? c->fw_logits : nullptr, n, 0, V, false)) != SD_OK)
    return s;
  SD_HIP(hipStreamSynchronize(c->st));
  if (logits_host) SD_HIP(hipMemcpy(logits_host, c->fw_logits, (size_t)n * V * 4, hipMemcpyDeviceToHost));
  if (hidden_host) {
    if (rt.m.dtype == SD_F32) {
      SD_HIP(hipMemcpy(hidden_host, c->xn, (size_t)n * d * 4, hipMemcpyDeviceToHost));
    } else {
      std::vector<uint16_t> tmp((size_t)n * d);
      SD_HIP(hipMemcpy(tmp.data(), c->xn, tmp.size() * 2, hipMemcpyDeviceToHost));
      for (size_t i = 0; i < tmp.size(); ++i) hidden_host[i] = bf16_to_float(tmp[i]);
    }
  }
  kv[seq] = start + n;
  return set_dev_int(c, which == 0 ? c->s.kv_t : c->s.kv_d, seq, start + n);
}

// Training examples of the acceptance head for one (prompt, response) pair (Sec. 4.4).
sd_status sd_head_examples(sd_ctx* c, int32_t seq, const int32_t* tokens, int32_t n_prompt, int32_t N, float r,
                           uint64_t seed, int32_t example, float temperature, int32_t top_k, float* E_dev,
                           float* P_dev, int32_t* mask_dev, int32_t* Y_host, int32_t* Z_host) {
  if (!c || !tokens || !E_dev || !P_dev || !mask_dev || seq < 0 || seq >= c->B || n_prompt < 1 || N < 1 ||
      !(r >= 0.f && r <= 1.f) || !(temperature > 0.f) || top_k < 0)
    return SD_EINVAL;
  if (n_prompt + N + 2 > c->cfg.max_seq) return SD_ERANGE;
  const int V = c->target.m.vocab, d = c->draft.m.d_model, ms = c->cfg.max_seq;
  if (c->draft.m.vocab != V) return SD_EINVAL;
  for (int i = 0; i < n_prompt + N; ++i)
    if (tokens[i] < 0 || tokens[i] >= V) return SD_ERANGE;
  sd_status s;
  if (!c->fw_logits2 && (s = dev_alloc(c, (void**)&c->fw_logits2, (size_t)PREFILL_CHUNK * V * 4, true)) != SD_OK) return s;
  if (!c->ex_ints && (s = dev_alloc(c, (void**)&c->ex_ints, (size_t)4 * ms * 4, true)) != SD_OK) return s;
  int32_t *Xd = c->ex_ints, *Yd = Xd + ms, *Zd = Yd + ms;
  hipStream_t st = c->st;
  // both caches take the prompt (positions 0 .. n_prompt - 2)
  if ((s = sd_prefill(c, seq, tokens, n_prompt)) != SD_OK) return s;
  SD_HIP(hipMemcpyAsync(Xd, tokens + n_prompt, (size_t)N * 4, hipMemcpyHostToDevice, st));
  // pass 1, teacher-forced on the response X: row of position n_prompt - 1 + j predicts X_{j+1}
  for (int j0 = 0; j0 < N; j0 += PREFILL_CHUNK) {
    const int m = std::min(PREFILL_CHUNK, N - j0), start = n_prompt - 1 + j0;
    SD_HIP(hipStreamSynchronize(st));                  // the pinned row plan is reused
    if ((s = plan_host_rows(c, seq, start, tokens + start, m)) != SD_OK) return s;
    if ((s = forward(c, c->target, m, m, start + m, nullptr, m, c->fw_logits, m, 0, V, false)) != SD_OK) return s;
    if ((s = forward(c, c->draft, m, m, start + m, nullptr, m, c->fw_logits2, m, 0, V, false)) != SD_OK) return s;
    SD_HIP(launch_labels(st, c->fw_logits, c->fw_logits2, m, V, temperature, top_k, seed, j0 + 1, example, Yd + j0,
                         P_dev + j0));
  }
  SD_HIP(launch_mix(st, Xd, Yd, N, r, seed, example, Zd, mask_dev));
  std::vector<int32_t> z(N + 1);
  z[0] = tokens[n_prompt - 1];
  SD_HIP(hipStreamSynchronize(st));
  SD_HIP(hipMemcpy(z.data() + 1, Zd, (size_t)N * 4, hipMemcpyDeviceToHost));
  if (Y_host) SD_HIP(hipMemcpy(Y_host, Yd, (size_t)N * 4, hipMemcpyDeviceToHost));
  if (Z_host) memcpy(Z_host, z.data() + 1, (size_t)N * 4);
  // pass 2, draft only, on the mixed sequence: the row whose input token is Z_i gives E_i
  for (int j0 = 0; j0 < N + 1; j0 += PREFILL_CHUNK) {
    const int m = std::min(PREFILL_CHUNK, N + 1 - j0), start = n_prompt - 1 + j0;
    SD_HIP(hipStreamSynchronize(st));
    if ((s = plan_host_rows(c, seq, start, z.data() + j0, m)) != SD_OK) return s;
    if ((s = forward(c, c->draft, m, m, start + m, nullptr, 0, nullptr, 1, 0, 0, false)) != SD_OK) return s;
    // rows of this chunk are Z_{j0} .. (row 0 of the first chunk is the last prompt token: skipped)
    const int skip = j0 == 0 ? 1 : 0;
    if (m - skip > 0)
      SD_HIP(launch_to_f32(st, c->draft.m.dtype, (const char*)c->xn + (size_t)skip * d * c->draft.esz,
                           E_dev + (size_t)(j0 - 1 + skip) * d, (size_t)(m - skip) * d));
  }
  SD_HIP(hipStreamSynchronize(st));
  // the caches now hold a training sequence: the slot must be prefilled again before it decodes
  c->active[seq] = 0;
  return set_dev_int(c, c->s.active, seq, 0);
}

sd_status sd_seq_state(sd_ctx* c, int32_t seq, int32_t* P, int32_t* kv_t, int32_t* kv_d, int32_t* round_idx) {
  if (!c || seq < 0 || seq >= c->B) return SD_EINVAL;
  if (P) *P = c->P[seq];
  if (kv_t) *kv_t = c->kv_t[seq];
  if (kv_d) *kv_d = c->kv_d[seq];
  if (round_idx) *round_idx = c->round[seq];
  return SD_OK;
}

sd_status sd_last_round_times(sd_ctx* c, double* seconds, int32_t* target_rows) {
  if (!c || !seconds) return SD_EINVAL;
  for (int k = 0; k < 3; ++k) seconds[k] = c->last_phase_s[k];
  if (target_rows) *target_rows = c->last_rows;
  return SD_OK;
}

sd_status sd_last_round_rows(sd_ctx* c, int32_t seq, float* q_host, float* p_host, float* head_s_host) {
  if (!c || seq < 0 || seq >= c->B) return SD_EINVAL;
  SD_HIP(hipStreamSynchronize(c->st));
  int32_t K = 0;
  SD_HIP(hipMemcpy(&K, c->s.K + seq, 4, hipMemcpyDeviceToHost));
  const int V = c->target.m.vocab, k_max = c->cfg.k_max;
  if (K < 1 || K > k_max) return SD_EINVAL;
  if (q_host)
    SD_HIP(hipMemcpy(q_host, c->q_logits + (size_t)seq * k_max * V, (size_t)K * V * 4, hipMemcpyDeviceToHost));
  if (p_host)
    SD_HIP(hipMemcpy(p_host, c->p_logits + (size_t)seq * (k_max + 1) * V, (size_t)(K + 1) * V * 4,
                     hipMemcpyDeviceToHost));
  if (head_s_host && K > 1)
    SD_HIP(hipMemcpy(head_s_host, c->s.head_s + (size_t)seq * CAND_LD, (size_t)(K - 1) * 4, hipMemcpyDeviceToHost));
  return SD_OK;
}

sd_status sd_profile_enable(sd_ctx* c, int32_t every) {
  if (!c || every < 0) return SD_EINVAL;
  c->prof_every = every;
  c->prof_pass = 0;
  return SD_OK;
}

sd_status sd_profile_read(sd_ctx* c, int64_t* launches, double* seconds, double* bytes) {
  if (!c || !launches || !seconds || !bytes) return SD_EINVAL;
  SD_HIP(hipStreamSynchronize(c->st));
  prof_collect(c);
  for (int k = 0; k < 5; ++k) {
    launches[k] = c->prof_launches[k];
    seconds[k] = c->prof_seconds[k];
    bytes[k] = c->prof_bytes[k];
    c->prof_launches[k] = 0;
    c->prof_seconds[k] = 0;
    c->prof_bytes[k] = 0;
  }
  return SD_OK;
}

int64_t sd_gemm_workspace_bytes(int32_t dtype, int32_t M, int32_t N, int32_t K) {
  if ((dtype != SD_F32 && dtype != SD_BF16) || M < 1 || M > MAX_ROWS || N < 1 || K < 1) return 0;
  return (int64_t)gemm_splits(dtype, M, N, K) * M * N * 4;
}

sd_status sd_gemm_skinny(int32_t dtype, const void* W, const void* X, int32_t M, int32_t N, int32_t K, float* Y,
                         void* ws, void* hip_stream) {
  if (!W || !X || !Y || !ws || (dtype != SD_F32 && dtype != SD_BF16)) return SD_EINVAL;
  hipStream_t st = (hipStream_t)hip_stream;
  SD_HIP(launch_gemm(st, dtype, W, X, K, nullptr, (float*)ws, M, N, K));
  SD_HIP(launch_reduce_rows(st, (const float*)ws, gemm_splits(dtype, M, N, K), Y, M, 0, N, M, N));
  return SD_OK;
}

int32_t sd_mlp_act_is_fused(int32_t dtype, int32_t M, int32_t ffn, int32_t K) {
  if ((dtype != SD_F32 && dtype != SD_BF16) || M < 1 || M > MAX_ROWS || ffn < 1 || K < 1) return 0;
  return gemm_silu_fused(dtype, M, ffn, K) ? 1 : 0;
}

sd_status sd_mlp_act(int32_t dtype, const void* W_gate_up, const void* X, int32_t M, int32_t ffn, int32_t K,
                     void* act, void* ws, int32_t mode, void* hip_stream) {
  if (!W_gate_up || !X || !act || (dtype != SD_F32 && dtype != SD_BF16) || M < 1 || M > MAX_ROWS || ffn < 1 || K < 1 ||
      mode < -1 || mode > 1)
    return SD_EINVAL;
  hipStream_t st = (hipStream_t)hip_stream;
  const bool can = gemm_silu_fused(dtype, M, ffn, K);
  if (mode == 1 && !can) return SD_EINVAL;
  if (mode != 0 && can) {
    SD_HIP(launch_gemm_silu(st, dtype, W_gate_up, X, K, nullptr, act, M, ffn, K));
    return SD_OK;
  }
  if (!ws) return SD_EINVAL;
  SD_HIP(launch_gemm(st, dtype, W_gate_up, X, K, nullptr, (float*)ws, M, 2 * ffn, K));
  SD_HIP(launch_silu_mul(st, dtype, (const float*)ws, gemm_splits(dtype, M, 2 * ffn, K), act, M, ffn));
  return SD_OK;
}

int32_t sd_qkv_rope_is_fused(int32_t dtype, int32_t M, int32_t n_heads, int32_t n_kv_heads, int32_t head_dim,
                             int32_t K) {
  if ((dtype != SD_F32 && dtype != SD_BF16) || M < 1 || M > MAX_ROWS || n_heads < 1 || n_kv_heads < 1 ||
      head_dim < 2 || K < 1)
    return 0;
  return gemm_rope_fused(dtype, M, n_heads, n_kv_heads, head_dim, K) ? 1 : 0;
}

sd_status sd_qkv_rope(int32_t dtype, const void* W_qkv, const void* X, int32_t M, int32_t n_heads, int32_t n_kv_heads,
                      int32_t head_dim, int32_t K, const int32_t* row_seq, const int32_t* row_pos,
                      const float* cos_sin, void* q_out, void* k_cache, void* v_cache, int32_t max_seq, void* ws,
                      int32_t mode, void* hip_stream) {
  if (!W_qkv || !X || !row_seq || !row_pos || !cos_sin || !q_out || !k_cache || !v_cache ||
      (dtype != SD_F32 && dtype != SD_BF16) || M < 1 || M > MAX_ROWS || n_heads < 1 || n_kv_heads < 1 ||
      head_dim < 2 || (head_dim & 1) || K < 1 || max_seq < 1 || mode < -1 || mode > 1)
    return SD_EINVAL;
  hipStream_t st = (hipStream_t)hip_stream;
  const bool can = gemm_rope_fused(dtype, M, n_heads, n_kv_heads, head_dim, K);
  if (mode == 1 && !can) return SD_EINVAL;
  if (mode != 0 && can) {
    SD_HIP(launch_gemm_rope(st, dtype, W_qkv, X, K, M, n_heads, n_kv_heads, head_dim, K, row_seq, row_pos, cos_sin,
                            q_out, k_cache, v_cache, max_seq, nullptr, 0, 0, 0.f));
    return SD_OK;
  }
  if (!ws) return SD_EINVAL;
  const int N = (n_heads + 2 * n_kv_heads) * head_dim;
  SD_HIP(launch_gemm(st, dtype, W_qkv, X, K, nullptr, (float*)ws, M, N, K));
  RowPlan rows{};
  rows.seq = const_cast<int32_t*>(row_seq);
  rows.pos = const_cast<int32_t*>(row_pos);
  SD_HIP(launch_rope_kv(st, dtype, (const float*)ws, gemm_splits(dtype, M, N, K), rows, cos_sin, q_out, k_cache,
                        v_cache, M, n_heads, n_kv_heads, head_dim, max_seq));
  return SD_OK;
}

int64_t sd_gemm_tile_workspace_bytes(int32_t M, int32_t N, int32_t K) {
  if (M < 1 || M > MAX_PREFILL_ROWS || N < 1 || K < 32 || K % 32 != 0) return -1;
  const int S = gemm_tile_splits(M, N, K);
  return S > 1 ? (int64_t)S * M * N * 4 : 0;
}

sd_status sd_gemm_tile(const void* W, const void* X, int32_t M, int32_t N, int32_t K, float* Y, void* ws,
                       void* hip_stream) {
  if (!W || !X || !Y || M < 1 || M > MAX_PREFILL_ROWS || N < 1 || K < 32 || K % 32 != 0) return SD_EINVAL;
  hipStream_t st = (hipStream_t)hip_stream;
  const int S = gemm_tile_splits(M, N, K);
  if (S > 1 && !ws) return SD_EINVAL;
  SD_HIP(launch_gemm_tile(st, W, X, K, nullptr, S > 1 ? (float*)ws : Y, M, N, K));
  if (S > 1) SD_HIP(launch_reduce_rows(st, (const float*)ws, S, Y, M, 0, N, M, N));
  return SD_OK;
}

}  // extern "C"
#pragma GCC visibility pop
