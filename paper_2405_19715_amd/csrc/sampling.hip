// Device-resident control of a round (Algorithm 2): row plans for the draft steps
// and the target pass, the draft sample + acceptance-head stop rule, the softmax /
// accept / residual-resample step (Algorithm 1's tail, Appendix C), and the commit
// that appends the new tokens and rolls both KV caches back.
//
// A sample from non-negative weights f with one uniform u is the inverse CDF in
// index order: the first v whose running sum exceeds u * total.  The running sum
// is taken in a fixed order (each of 16 wavefronts owns a contiguous range and walks it in
// rows of 256 elements, a row's sum is an inclusive lane scan, row totals and wavefront
// totals are added in order), so a draw never depends on scheduling.  The weights of a
// softmax row are 2^((l - max) log2(e) / T) on the hardware's exp2 (row_weight).
#include "common.hpp"
#include "kernels.hpp"

namespace sd {

namespace {

constexpr int SB = 1024;            // threads of the vocab-wide kernels
constexpr int CAND_LD = 32;         // row stride of the per-sequence candidate arrays
constexpr int RES_LD = 40;          // ints per sequence in the packed round result
constexpr float LOG2E = 1.44269504088896340736f;

struct ArgMax { float v; int i; };

__device__ __forceinline__ ArgMax better(ArgMax a, ArgMax b) {
  return (b.v > a.v || (b.v == a.v && b.i < a.i)) ? b : a;      // ties go to the lowest id
}

// Block-wide argmax (lowest index among equal maxima).  sh: SB/64 floats + SB/64 ints.
__device__ ArgMax block_argmax(ArgMax a, float* shv, int* shi) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    ArgMax b{__shfl_xor(a.v, o, WAVE), __shfl_xor(a.i, o, WAVE)};
    a = better(a, b);
  }
  const int w = threadIdx.x >> 6, nw = blockDim.x >> 6;
  if ((threadIdx.x & 63) == 0) { shv[w] = a.v; shi[w] = a.i; }
  __syncthreads();
  ArgMax r{shv[0], shi[0]};
  for (int k = 1; k < nw; ++k) r = better(r, ArgMax{shv[k], shi[k]});
  __syncthreads();
  return r;
}

// Monotone map float -> uint32 (larger float, larger key).
__device__ __forceinline__ uint32_t order_key(float x) {
  const uint32_t u = __float_as_uint(x);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
__device__ __forceinline__ float key_to_float(uint32_t k) {
  return __uint_as_float((k & 0x80000000u) ? (k & 0x7fffffffu) : ~k);
}

// The k-th largest of l[0..V) (1 <= k <= V), found bit by bit on the order keys: 32 block-wide
// counts of "key >= candidate".  Top-k warping keeps l[v] >= it.  A row of up to 32 elements per
// thread (V = 32000 with 1024 threads) is read once into registers and every count is a compare
// whose lane mask is popcounted; longer rows are re-read from L2 in every pass.  sh: SB/64 ints.
__device__ float block_kth_largest(const float* __restrict__ l, int V, int k, int* sh) {
  constexpr int NK = 32;
  uint32_t t = 0;
  const int w = threadIdx.x >> 6, nw = blockDim.x >> 6;
  const bool in_regs = V <= NK * (int)blockDim.x;
  uint32_t key[NK];
  if (in_regs) {
#pragma unroll
    for (int u = 0; u < NK; ++u) {
      const int v = u * blockDim.x + threadIdx.x;
      key[u] = v < V ? order_key(l[v]) : 0u;         // 0 is below every candidate (a candidate has a bit set)
    }
  }
  for (int bit = 31; bit >= 0; --bit) {
    const uint32_t cand = t | (1u << bit);
    int c = 0;
    if (in_regs) {
#pragma unroll
      for (int u = 0; u < NK; ++u) c += __popcll(__ballot(key[u] >= cand));      // wave-uniform
    } else {
      for (int v = threadIdx.x; v < V; v += blockDim.x) c += order_key(l[v]) >= cand ? 1 : 0;
#pragma unroll
      for (int o = 32; o > 0; o >>= 1) c += __shfl_xor(c, o, WAVE);
    }
    if ((threadIdx.x & 63) == 0) sh[w] = c;
    __syncthreads();
    int tot = 0;
    for (int i = 0; i < nw; ++i) tot += sh[i];
    __syncthreads();
    if (tot >= k) t = cand;
  }
  return key_to_float(t);
}

// Inverse-CDF draw over v in [0, V) with weight f(v) >= 0; returns -1 when the total
// mass is not positive.  sh_w: SB/64 floats, sh_res: 1 int.
//
// The cumulative sum runs in index order, but it is not formed left to right by one
// thread: wavefront w owns the contiguous range [w CW, (w+1) CW), walks it in rows of 256
// elements (lane l holds elements 4l .. 4l+3 of a row, so every load is coalesced), and
// a row's total is the last lane of an inclusive lane scan.  Pass 1 gives every
// wavefront its total; the wavefront whose range contains u * S repeats its walk with
// exactly the same additions to find the row, the lane and the element.
template <typename F>
__device__ int block_sample(F f, int V, float u, float* sh_w, int* sh_res) {
  const int t = threadIdx.x, lane = t & 63, w = t >> 6;
  constexpr int NW = SB / 64;
  constexpr int NR = 8;                                         // rows evaluated together (V = 32000: a wavefront's whole range)
  const int CW = (((V + NW - 1) / NW) + 255) & ~255;            // elements per wavefront, whole rows
  const int beg = min(w * CW, V), end = min(beg + CW, V);
  // NR rows from c0 on: all weights are fetched before the first scan (the loads of a row do not
  // wait for the scan of the row before); per row the lane sum ls, the inclusive lane scan and the total
  auto rows_scan = [&](int c0, float (*fv)[4], float* ls, float* incl, float* tot) {
#pragma unroll
    for (int r = 0; r < NR; ++r)
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const int v = c0 + r * 256 + 4 * lane + e;
        fv[r][e] = v < end ? f(v) : 0.f;
      }
#pragma unroll
    for (int r = 0; r < NR; ++r) {
      float a = 0.f;
#pragma unroll
      for (int e = 0; e < 4; ++e) a += fv[r][e];
      ls[r] = a;
#pragma unroll
      for (int o = 1; o < 64; o <<= 1) {
        const float n = __shfl_up(a, o, WAVE);
        if (lane >= o) a += n;
      }
      incl[r] = a;
      tot[r] = __shfl(a, 63, WAVE);
    }
  };
  float cw = 0.f;
  for (int c0 = beg; c0 < end; c0 += NR * 256) {
    float fv[NR][4], ls[NR], incl[NR], tot[NR];
    rows_scan(c0, fv, ls, incl, tot);
#pragma unroll
    for (int r = 0; r < NR; ++r)
      if (c0 + r * 256 < end) cw += tot[r];
  }
  if (lane == 0) sh_w[w] = cw;
  if (t == 0) *sh_res = -1;
  __syncthreads();
  float off = 0.f, total = 0.f;
  for (int k = 0; k < NW; ++k) {
    if (k == w) off = total;
    total += sh_w[k];
  }
  if (!(total > 0.f)) return -1;                                // uniform: every thread sees the same total
  const float target = u * total;
  if (off <= target && target < off + cw) {                     // wave-uniform
    float run = 0.f;
    bool found = false;
    for (int c0 = beg; c0 < end && !found; c0 += NR * 256) {
      float fv[NR][4], ls[NR], incl[NR], tot[NR];
      rows_scan(c0, fv, ls, incl, tot);
#pragma unroll
      for (int r = 0; r < NR; ++r) {
        if (found || c0 + r * 256 >= end) continue;
        if (off + (run + tot[r]) > target) {
          const unsigned long long m = __ballot(off + (run + incl[r]) > target);
          if (lane == __ffsll((long long)m) - 1) {
            float acc = run + (incl[r] - ls[r]);
            int pick = -1, last_pos = -1;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
              acc += fv[r][e];
              if (fv[r][e] > 0.f) last_pos = c0 + r * 256 + 4 * lane + e;
              if (pick < 0 && off + acc > target) pick = c0 + r * 256 + 4 * lane + e;
            }
            *sh_res = pick >= 0 ? pick : last_pos;
          }
          found = true;
        } else {
          run += tot[r];
        }
      }
    }
  }
  __syncthreads();
  int res = *sh_res;
  if (res < 0) {                      // rounding left no bucket: largest v with mass
    int best = -1;
    for (int v = t; v < V; v += SB)
      if (f(v) > 0.f) best = v;
    __syncthreads();
    atomicMax(sh_res, best);
    __syncthreads();
    res = *sh_res;
  }
  return res;
}

// ------------------------------------------------------------------ logits rows held in registers
// A row of up to 32768 16-byte-aligned elements is read once, into the registers of one 1024-thread workgroup, in
// the layout of the inverse-CDF walk: wavefront w owns the contiguous range [w CW, (w + 1) CW), lane l holds elements
// 4 l .. 4 l + 3 of each of its 256-element rows, so a load instruction covers 1 KB.  Statistics (block maximum
// first, then one weight per element) and the draw work on those registers.
constexpr int NR = 8;                                  // 256-element rows per wavefront
constexpr int REG_V_MAX = (SB / 64) * NR * 256;        // 32768: a row fits the registers of one workgroup

struct RowStat { float mx, sum, thr; int arg; };

// The weight of a logit x in a row with maximum mx: exp((x - mx) / T) as 2^((x - mx) k), k = log2(e) / T, on the
// hardware's exp2 (1 ulp; results below 2^-126 are flushed to 0).  The product's rounding adds a relative error of
// at most 2^-24 |(x - mx) k| ln 2: 4e-8 per unit of distance below the maximum, i.e. the weights that carry the
// sum are as exact as expf's, and three instructions replace the library routine's fifteen (a workgroup per row is
// bound by its CU's vector ALUs as much as by memory).  Every place that needs a row's weights calls this, so the
// statistics, the residual and the draw see the same bits.
__device__ __forceinline__ float row_weight(float x, float mx, float k) { return __builtin_amdgcn_exp2f((x - mx) * k); }

// Row l[0..V) into x, sampling layout (V a multiple of 4, l 16-byte aligned).  Elements beyond the wavefront's
// range get PAD: far below any logit (it never wins a maximum, its weight is 0) and finite, so nothing after the
// load needs to know which elements are real.
constexpr float PAD = -1.0e30f;
template <bool STREAM>
__device__ __forceinline__ void load_row_regs(const float* __restrict__ l, int beg, int end, int lane, float (&x)[NR][4]) {
  typedef float f32x4 __attribute__((ext_vector_type(4)));
#pragma unroll
  for (int r = 0; r < NR; ++r) {
    const int v0 = beg + r * 256 + 4 * lane;           // beg, end and v0 are multiples of 4
    x[r][0] = x[r][1] = x[r][2] = x[r][3] = PAD;
    if (v0 < end) {                                    // STREAM: first and only read from HBM, non-temporal
      const f32x4* src = reinterpret_cast<const f32x4*>(l + v0);
      const f32x4 t = STREAM ? __builtin_nontemporal_load(src) : *src;
      x[r][0] = t.x;
      x[r][1] = t.y;
      x[r][2] = t.z;
      x[r][3] = t.w;
    }
  }
}

// Statistics of the row held in x (maximum with the lowest index among equals, top-k threshold, sum of the kept
// weights) and, in place, x <- the weights of the kept elements, 0 elsewhere.  sh_i: SB / 64 + 1 ints.
template <bool TOPK>
__device__ __forceinline__ RowStat row_stat_regs(float (&x)[NR][4], int beg, int lane, float k, int top_k, bool& bad,
                                                 float* sh_w, int* sh_i) {
  float m = x[0][0], lo = x[0][0];
#pragma unroll
  for (int r = 0; r < NR; ++r) {
    m = fmaxf(fmaxf(m, x[r][0]), fmaxf(x[r][1], fmaxf(x[r][2], x[r][3])));
    lo = fminf(fminf(lo, x[r][0]), fminf(x[r][1], fminf(x[r][2], x[r][3])));
  }
  bad |= lo == -INFINITY;                              // NaN and +inf show in the sum of the weights below
  const float mx = block_max(m, sh_w);
  // lowest index of the maximum: only threads that hold it look
  if (threadIdx.x == 0) sh_i[SB / 64] = 0x7fffffff;
  __syncthreads();
  if (m == mx) {
    int slot = 0;
#pragma unroll
    for (int r = NR - 1; r >= 0; --r)
#pragma unroll
      for (int e = 3; e >= 0; --e)
        if (x[r][e] == mx) slot = r * 4 + e;
    atomicMin(&sh_i[SB / 64], beg + (slot >> 2) * 256 + 4 * lane + (slot & 3));
  }
  __syncthreads();
  const int arg = sh_i[SB / 64];
  float thr = -INFINITY;
  float s = 0.f;
  if (TOPK) {
    // the k-th largest value, bit by bit on the order keys (see block_kth_largest); the keys take the place of
    // the values in the registers and are turned back afterwards (the map is a bijection).  PAD's key lies below
    // the key of every logit, and top_k < V logits exist, so the padding is never counted at the bit that decides
#pragma unroll
    for (int r = 0; r < NR; ++r)
#pragma unroll
      for (int e = 0; e < 4; ++e) x[r][e] = __uint_as_float(order_key(x[r][e]));
    uint32_t t = 0;
    const int w = threadIdx.x >> 6;
    for (int bit = 31; bit >= 0; --bit) {
      const uint32_t c = t | (1u << bit);
      int cnt = 0;
#pragma unroll
      for (int r = 0; r < NR; ++r)
#pragma unroll
        for (int e = 0; e < 4; ++e) cnt += __popcll(__ballot(__float_as_uint(x[r][e]) >= c));
      if (lane == 0) sh_i[w] = cnt;
      __syncthreads();
      int tot = 0;
      for (int i = 0; i < SB / 64; ++i) tot += sh_i[i];
      __syncthreads();
      if (tot >= top_k) t = c;
    }
    thr = key_to_float(t);
#pragma unroll
    for (int r = 0; r < NR; ++r)
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const float v = key_to_float(__float_as_uint(x[r][e]));
        const float wt = v >= thr ? row_weight(v, mx, k) : 0.f;
        x[r][e] = wt;
        s += wt;
      }
  } else {
#pragma unroll
    for (int r = 0; r < NR; ++r)
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const float wt = row_weight(x[r][e], mx, k);   // padding: 0
        x[r][e] = wt;
        s += wt;
      }
  }
  const float total = block_sum(s, sh_w);
  bad |= !(total > 0.f && total < INFINITY);           // a NaN or +inf logit makes the sum NaN
  return RowStat{mx, total, thr, arg};
}

// Any other row (longer, or not 16-byte aligned): strided walks over global memory.
__device__ RowStat row_stat_global(const float* __restrict__ l, int V, float k, int top_k, bool& bad, float* sh_w,
                                   int* sh_i) {
  ArgMax am{-INFINITY, 0x7fffffff};
  for (int v = threadIdx.x; v < V; v += SB) {
    const float x = l[v];
    bad |= !isfinite(x);
    if (x > am.v) am = ArgMax{x, v};                   // strided indices grow, so ties keep the lowest id
  }
  am = block_argmax(am, sh_w, sh_i);
  const float thr = (top_k > 0 && top_k < V) ? block_kth_largest(l, V, top_k, sh_i) : -INFINITY;
  float s = 0.f;
  for (int v = threadIdx.x; v < V; v += SB) s += l[v] >= thr ? row_weight(l[v], am.v, k) : 0.f;
  const float total = block_sum(s, sh_w);
  return RowStat{am.v, total, thr, am.i};
}

__device__ __forceinline__ bool rows_in_regs(const float* l, int V) {
  return V <= REG_V_MAX && (V & 3) == 0 && (reinterpret_cast<uintptr_t>(l) & 15) == 0;
}

// block_sample on weights held in registers (sampling layout): the same additions in the same order.
__device__ __forceinline__ int block_sample_regs(const float (&f)[NR][4], int beg, int end, int lane, float u,
                                                 float* sh_w, int* sh_res) {
  const int t = threadIdx.x, w = t >> 6;
  constexpr int NW = SB / 64;
  // lane sum, inclusive lane scan and total of row r
  auto row_scan = [&](int r, float& ls, float& incl, float& tot) {
    float a = 0.f;
#pragma unroll
    for (int e = 0; e < 4; ++e) a += f[r][e];
    ls = a;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
      const float n = __shfl_up(a, o, WAVE);
      if (lane >= o) a += n;
    }
    incl = a;
    tot = __shfl(a, 63, WAVE);
  };
  float cw = 0.f;
#pragma unroll
  for (int r = 0; r < NR; ++r) {
    float ls, incl, tot;
    row_scan(r, ls, incl, tot);
    if (beg + r * 256 < end) cw += tot;
  }
  if (lane == 0) sh_w[w] = cw;
  if (t == 0) *sh_res = -1;
  __syncthreads();
  float off = 0.f, total = 0.f;
  for (int k = 0; k < NW; ++k) {
    if (k == w) off = total;
    total += sh_w[k];
  }
  if (!(total > 0.f)) {                                // uniform: every thread sees the same total
    __syncthreads();
    return -1;
  }
  const float target = u * total;
  if (off <= target && target < off + cw) {            // wave-uniform: the wavefront whose range holds the target
    float run = 0.f;                                   // repeats its scans (the same additions) to find the element
    bool found = false;
#pragma unroll
    for (int r = 0; r < NR; ++r) {
      if (found || beg + r * 256 >= end) continue;
      float ls, incl, tot;
      row_scan(r, ls, incl, tot);
      if (off + (run + tot) > target) {
        const unsigned long long m = __ballot(off + (run + incl) > target);
        if (lane == __ffsll((long long)m) - 1) {
          float acc = run + (incl - ls);
          int pick = -1, last_pos = -1;
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            acc += f[r][e];
            if (f[r][e] > 0.f) last_pos = e;
            if (pick < 0 && off + acc > target) pick = e;
          }
          *sh_res = beg + r * 256 + 4 * lane + (pick >= 0 ? pick : last_pos);
        }
        found = true;
      } else {
        run += tot;
      }
    }
  }
  __syncthreads();
  int res = *sh_res;
  if (res < 0) {                                       // rounding left no bucket: largest v with mass
    int best = -1;
#pragma unroll
    for (int r = 0; r < NR; ++r)
#pragma unroll
      for (int e = 0; e < 4; ++e)
        if (f[r][e] > 0.f) best = r * 4 + e;                         // indices grow
    if (best >= 0) best = beg + (best >> 2) * 256 + 4 * lane + (best & 3);
    __syncthreads();
    atomicMax(sh_res, best);
    __syncthreads();
    res = *sh_res;
  }
  __syncthreads();                                     // sh_w and sh_res are free again
  return res;
}

// ------------------------------------------------------------------ round bookkeeping
__global__ void begin_round_k(SeqState s, int B, int k_max, int max_seq) {
  const int b = blockIdx.x * blockDim.x + threadIdx.x;
  if (b >= B) return;
  s.K[b] = 0;
  s.stopped[b] = s.active[b] ? 0 : 1;
  s.p_hat[b] = 1.0f;
  s.kcap[b] = min(k_max, max_seq - s.P[b] - 1);
}

// Draft step `step` (1-based): 2 row slots per sequence.  Step 1 ingests the 1 or 2
// finalised tokens the draft cache has not seen; later steps ingest y_{step-1}.
__global__ void plan_draft_k(SeqState s, RowPlan rows, int B, int step, int max_seq) {
  const int b = blockIdx.x * blockDim.x + threadIdx.x;
  if (b >= B) return;
  const int m0 = 2 * b;
  rows.seq[m0] = rows.seq[m0 + 1] = -1;
  rows.pos[m0] = rows.pos[m0 + 1] = 0;
  rows.tok[m0] = rows.tok[m0 + 1] = 0;
  s.last_row[b] = m0;
  rows.gseq[b] = -1;
  rows.gend[b] = 0;
  if (s.stopped[b]) return;
  const int P = s.P[b];
  rows.gseq[b] = b;
  rows.gend[b] = step == 1 ? P : P + step - 1;
  if (step == 1) {
    const int kv = s.kv_d[b];
    const int cnt = min(max(P - kv, 1), 2);
    for (int j = 0; j < cnt; ++j) {
      const int pos = P - cnt + j;
      rows.seq[m0 + j] = b;
      rows.pos[m0 + j] = pos;
      rows.tok[m0 + j] = s.tokens[(size_t)b * max_seq + pos];
    }
    s.last_row[b] = m0 + cnt - 1;
    s.kv_d[b] = P;
  } else {
    const int pos = P + step - 2;
    rows.seq[m0] = b;
    rows.pos[m0] = pos;
    rows.tok[m0] = s.cand[b * CAND_LD + step - 2];
    s.kv_d[b] = pos + 1;
  }
}

// Target pass: rs row slots per sequence (rs > every K of the round) holding x_last, y_1 .. y_K.
__global__ void plan_verify_k(SeqState s, RowPlan rows, int B, int rs, int max_seq) {
  const int b = blockIdx.x;
  const int j = threadIdx.x;
  if (b >= B || j >= rs) return;
  const int m = b * rs + j;
  const int P = s.P[b], K = s.K[b];
  if (j == 0) {
    rows.gseq[b] = s.active[b] ? b : -1;
    rows.gend[b] = P + K;
  }
  if (j <= K && s.active[b]) {
    rows.seq[m] = b;
    rows.pos[m] = P - 1 + j;
    rows.tok[m] = j == 0 ? s.tokens[(size_t)b * max_seq + P - 1] : s.cand[b * CAND_LD + j - 1];
  } else {
    rows.seq[m] = -1;
    rows.pos[m] = 0;
    rows.tok[m] = 0;
  }
}

// Ragged target pass (several sequences, different K): groups of RS row slots, sequence after
// sequence.  One thread per sequence; the group offset is a serial prefix count (B is small).
__global__ void plan_verify_ragged_k(SeqState s, RowPlan rows, int B, int RS, int n_groups, int k_max, int max_seq,
                                     int32_t* __restrict__ dst) {
  const int b = threadIdx.x;
  if (b >= B) return;
  int g0 = 0;
  for (int i = 0; i < b; ++i) g0 += s.active[i] ? (s.K[i] + RS) / RS : 0;       // ceil((K + 1) / RS)
  if (!s.active[b]) return;
  const int P = s.P[b], K = s.K[b];
  const int ng = (K + RS) / RS;
  for (int g = 0; g < ng && g0 + g < n_groups; ++g) {
    rows.gseq[g0 + g] = b;
    rows.gend[g0 + g] = P + min(K, g * RS + RS - 1);                           // largest position of the group + 1
    for (int r = 0; r < RS; ++r) {
      const int j = g * RS + r, m = (g0 + g) * RS + r;
      if (j <= K) {
        rows.seq[m] = b;
        rows.pos[m] = P - 1 + j;
        rows.tok[m] = j == 0 ? s.tokens[(size_t)b * max_seq + P - 1] : s.cand[b * CAND_LD + j - 1];
        dst[m] = b * (k_max + 1) + j;
      } else {
        rows.seq[m] = -1;
        rows.pos[m] = 0;
        rows.tok[m] = 0;
        dst[m] = -1;
      }
    }
  }
}

// ------------------------------------------------------------------ draft sample + stop rule
template <typename T>
__global__ __launch_bounds__(SB) void sample_stop_k(SeqState s, const float* __restrict__ q_logits, int64_t ld_seq,
                                                    const T* __restrict__ z, const int* __restrict__ z_rows, int z_dim,
                                                    const T* __restrict__ w_last, const T* __restrict__ b_last,
                                                    int have_head, DecodeParams p, int V, int step,
                                                    int32_t* __restrict__ host_flags, uint32_t tick) {
  __shared__ float sh_w[SB / 64];
  __shared__ int sh_i[SB / 64];
  __shared__ int sh_res;
  const int b = blockIdx.x;
  if (s.stopped[b]) {
    if (host_flags && threadIdx.x == 0) {
      host_flags[b] = (int32_t)((tick << 1) | 1u);
      __threadfence_system();
    }
    return;
  }
  const float* l = q_logits + (size_t)b * ld_seq + (size_t)(step - 1) * V;

  // row maximum (and argmax), non-finite check
  ArgMax am{-INFINITY, 0x7fffffff};
  bool bad = false;
  if ((V & 3) == 0 && (reinterpret_cast<uintptr_t>(l) & 15) == 0) {
    // a thread's 16-byte loads of a chunk all go out before the first is looked at
    constexpr int NQ = 8;
    const float4* l4 = reinterpret_cast<const float4*>(l);
    const int nq = V / 4;
    for (int q0 = 0; q0 < nq; q0 += NQ * SB) {
      float4 x[NQ];
#pragma unroll
      for (int u = 0; u < NQ; ++u) {
        const int q = q0 + u * SB + threadIdx.x;
        if (q < nq) x[u] = l4[q];
      }
#pragma unroll
      for (int u = 0; u < NQ; ++u) {
        const int q = q0 + u * SB + threadIdx.x;
        if (q < nq) {
          bad |= !(isfinite(x[u].x) && isfinite(x[u].y) && isfinite(x[u].z) && isfinite(x[u].w));
          am = better(am, ArgMax{x[u].x, 4 * q});
          am = better(am, ArgMax{x[u].y, 4 * q + 1});
          am = better(am, ArgMax{x[u].z, 4 * q + 2});
          am = better(am, ArgMax{x[u].w, 4 * q + 3});
        }
      }
    }
  } else {
    for (int v = threadIdx.x; v < V; v += SB) {
      const float x = l[v];
      bad |= !isfinite(x);
      am = better(am, ArgMax{x, v});
    }
  }
  am = block_argmax(am, sh_w, sh_i);
  if (bad) atomicOr(s.err, 1);

  int y;
  if (p.greedy) {
    y = am.i;
  } else {
    const float mx = am.v, inv_t = 1.0f / p.temperature, k2 = inv_t * LOG2E;
    const bool warp = p.top_k > 0 && p.top_k < V;
    const float u = philox_uniform(p.seed, (uint32_t)step, (uint32_t)s.round[b], (uint32_t)b, STREAM_DRAFT);
    if (rows_in_regs(l, V)) {
      // the row (written a moment ago by the LM head's launch: it comes from L2) once more, into registers in the
      // layout of the walk; every weight is evaluated once
      const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
      const int CW = (((V + SB / 64 - 1) / (SB / 64)) + 255) & ~255;
      const int beg = min(w * CW, V), end = min(beg + CW, V);
      const float thr = warp ? block_kth_largest(l, V, p.top_k, sh_i) : -INFINITY;
      float x[NR][4];
      load_row_regs<false>(l, beg, end, lane, x);
#pragma unroll
      for (int r = 0; r < NR; ++r)
#pragma unroll
        for (int e = 0; e < 4; ++e) x[r][e] = x[r][e] >= thr ? row_weight(x[r][e], mx, k2) : 0.f;     // padding: 0
      y = block_sample_regs(x, beg, end, lane, u, sh_w, &sh_res);
    } else {
      const float thr = warp ? block_kth_largest(l, V, p.top_k, sh_i) : -INFINITY;
      y = block_sample([&](int v) { return l[v] >= thr ? row_weight(l[v], mx, k2) : 0.f; }, V, u, sh_w, &sh_res);
    }
    if (y < 0) y = am.i;                // only reachable with non-finite logits
  }

  // acceptance head: last (linear) layer, sigmoid, cumulative product (nothing at step 1)
  float dot = 0.f;
  if (have_head && step > 1) {
    const T* zr = z + (size_t)(z_rows ? z_rows[b] : b) * z_dim;
    for (int i = threadIdx.x; i < z_dim; i += SB) dot = fmaf(Elem<T>::ld(zr + i), Elem<T>::ld(w_last + i), dot);
    dot = block_sum(dot, sh_w);
  }
  if (threadIdx.x == 0) {
    float ph = s.p_hat[b];
    if (have_head && step > 1) {
      const float a = dot + Elem<T>::ld(b_last);
      const float sg = 1.0f / (1.0f + expf(-a));
      s.head_s[b * CAND_LD + step - 2] = sg;
      ph *= sg;
      s.p_hat[b] = ph;
    }
    s.cand[b * CAND_LD + step - 1] = y;
    s.K[b] = step;
    const bool stop = (1.0f - ph > p.h) || (p.eos_id >= 0 && y == p.eos_id) || (step >= s.kcap[b]);
    s.stopped[b] = stop ? 1 : 0;
    if (host_flags) {                    // for the host, which watches this word instead of synchronising
      host_flags[b] = (int32_t)((tick << 1) | (stop ? 1u : 0u));
      __threadfence_system();
    }
  }
}

// ------------------------------------------------------------------ softmax statistics per row
// stats[row] = {max, sum_v w_v, argmax (int bits), top-k threshold or -inf}, w_v = exp((l_v - max)/T) (row_weight).
// One launch covers two logits arrays: blocks x < rows_a serve array A ([B, rows_a, V], row j
// live when j < K[b] + extra_a), the rest array B ([B, rows_b, V], live when j < K[b] + extra_b).
// A row of up to 32768 16-byte-aligned elements is read once, into registers, in the layout of the inverse-CDF
// walk (wavefront w owns the contiguous range [w CW, (w + 1) CW), lane l holds elements 4 l .. 4 l + 3 of each of
// its 256-element rows: a load instruction covers 1 KB): block maximum first, then one weight per element.
struct RowSet { const float* logits; float* stats; int rows, extra; };

// REGS: every row of the call fits the registers (the launcher decides); TOPK: top_k is in (0, V).
template <bool REGS, bool TOPK>
__global__ __launch_bounds__(SB) __attribute__((amdgpu_waves_per_eu(8, 8))) void row_stats_k(
    RowSet A, RowSet Bq, const int32_t* __restrict__ K, int V, float inv_t, int top_k, int32_t* __restrict__ err,
    int32_t* __restrict__ oob) {
  __shared__ float sh_w[SB / 64];
  __shared__ int sh_i[SB / 64 + 1];
  const int b = blockIdx.y;
  const bool first = (int)blockIdx.x < A.rows;
  const RowSet& R = first ? A : Bq;
  const int j = first ? blockIdx.x : blockIdx.x - A.rows;
  // the caller's "inputs out of range" word starts every call at 0; accept_k, next on the stream, sets its bits
  if (oob && blockIdx.x == 0 && b == 0 && threadIdx.x == 0) *oob = 0;
  if (j >= min(max(K[b], 0), Bq.rows) + R.extra) return;       // K_b is clamped into [0, Kmax] (accept_k reports it)
  const size_t row = (size_t)b * R.rows + j;
  const float* l = R.logits + row * V;
  const float k2 = inv_t * LOG2E;
  bool bad = false;
  RowStat st;
  if constexpr (REGS) {
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int CW = (((V + SB / 64 - 1) / (SB / 64)) + 255) & ~255;
    const int beg = min(w * CW, V), end = min(beg + CW, V);
    float x[NR][4];
    load_row_regs<true>(l, beg, end, lane, x);
    st = row_stat_regs<TOPK>(x, beg, lane, k2, top_k, bad, sh_w, sh_i);
  } else {
    st = row_stat_global(l, V, k2, TOPK ? top_k : 0, bad, sh_w, sh_i);
  }
  if (bad && err) atomicOr(err, 1);
  if (threadIdx.x == 0) {
    R.stats[row * 4 + 0] = st.mx;
    R.stats[row * 4 + 1] = st.sum;
    R.stats[row * 4 + 2] = __int_as_float(st.arg);
    R.stats[row * 4 + 3] = st.thr;
  }
}

// ------------------------------------------------------------------ training targets (Sec. 4.4)
// Row i (0-based) of p / q [n, V]: Y ~ q_row with the uniform of (slot0 + i, example,
// sequence 0, stream 3); P = min(1, p_row(Y) / q_row(Y)).  Same warping as the round.
__global__ __launch_bounds__(SB) void label_k(const float* __restrict__ p_logits, const float* __restrict__ q_logits,
                                              int V, float inv_t, int top_k, uint64_t seed, int slot0, int example,
                                              int32_t* __restrict__ Y, float* __restrict__ P) {
  __shared__ float sh_w[SB / 64];
  __shared__ int sh_i[SB / 64];
  __shared__ int sh_res;
  const int i = blockIdx.x;
  const float* lq = q_logits + (size_t)i * V;
  const float* lp = p_logits + (size_t)i * V;
  const bool warp = top_k > 0 && top_k < V;
  // draft row: max, threshold, sample
  ArgMax am{-INFINITY, 0x7fffffff};
  for (int v = threadIdx.x; v < V; v += SB) am = better(am, ArgMax{lq[v], v});
  am = block_argmax(am, sh_w, sh_i);
  const float qmx = am.v;
  const float qthr = warp ? block_kth_largest(lq, V, top_k, sh_i) : -INFINITY;
  const float u = philox_uniform(seed, (uint32_t)(slot0 + i), (uint32_t)example, 0u, 3u);
  const int y = block_sample([&](int v) { return lq[v] >= qthr ? expf((lq[v] - qmx) * inv_t) : 0.f; }, V, u, sh_w, &sh_res);
  __syncthreads();
  float local = 0.f;
  for (int v = threadIdx.x; v < V; v += SB) local += lq[v] >= qthr ? expf((lq[v] - qmx) * inv_t) : 0.f;
  const float qsum = block_sum(local, sh_w);
  // target row: max, threshold, sum
  ArgMax pm{-INFINITY, 0x7fffffff};
  for (int v = threadIdx.x; v < V; v += SB) pm = better(pm, ArgMax{lp[v], v});
  pm = block_argmax(pm, sh_w, sh_i);
  const float pthr = warp ? block_kth_largest(lp, V, top_k, sh_i) : -INFINITY;
  local = 0.f;
  for (int v = threadIdx.x; v < V; v += SB) local += lp[v] >= pthr ? expf((lp[v] - pm.v) * inv_t) : 0.f;
  const float psum = block_sum(local, sh_w);
  if (threadIdx.x == 0) {
    const int yy = y < 0 ? am.i : y;
    const float qy = expf((lq[yy] - qmx) * inv_t) / qsum;
    const float py = lp[yy] >= pthr ? expf((lp[yy] - pm.v) * inv_t) / psum : 0.f;
    Y[i] = yy;
    P[i] = fminf(1.0f, py / qy);
  }
}

// Token mixing: Z_i = X_i when u(slot i + 1, example, 0, stream 4) < r, else Y_i; mask_i = 1 where Z_i = Y_i.
__global__ void mix_k(const int32_t* __restrict__ X, const int32_t* __restrict__ Y, int n, float r, uint64_t seed,
                      int example, int32_t* __restrict__ Z, int32_t* __restrict__ mask) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  const float u = philox_uniform(seed, (uint32_t)(i + 1), (uint32_t)example, 0u, 4u);
  const bool keep = u < r;
  Z[i] = keep ? X[i] : Y[i];
  mask[i] = keep ? 0 : 1;
}

// ------------------------------------------------------------------ accept + resample
__global__ __launch_bounds__(SB) void accept_k(const float* __restrict__ p_logits, const float* __restrict__ q_logits,
                                               const float* __restrict__ p_stats, const float* __restrict__ q_stats,
                                               const int32_t* __restrict__ cand, int cand_ld,
                                               const int32_t* __restrict__ Karr, const int32_t* __restrict__ round_arr,
                                               int round_const, DecodeParams p, int Kmax, int V,
                                               int32_t* __restrict__ n_out, int32_t* __restrict__ tok_out,
                                               uint8_t* __restrict__ flags, int flags_ld, int32_t* __restrict__ oob) {
  __shared__ float sh_w[SB / 64];
  __shared__ int sh_res;
  __shared__ int sh_n;
  const int b = blockIdx.x;
  // K_b and the candidate ids come from the caller (isolated entry point): a count outside [0, Kmax] is clamped
  // and a candidate id outside [0, V) counts as rejected, so that no index below leaves its array; `oob` (may
  // be null) gets bit 0 / bit 1 when that happened
  const int K = min(max(Karr[b], 0), Kmax);
  if (oob && threadIdx.x == 0 && K != Karr[b]) atomicOr(oob, 1);
  const int rnd = round_arr ? round_arr[b] : round_const;
  const float inv_t = 1.0f / p.temperature;
  const float* pl = p_logits + (size_t)b * (Kmax + 1) * V;
  const float* ql = q_logits + (size_t)b * Kmax * V;
  const float* ps = p_stats + (size_t)b * (Kmax + 1) * 4;
  const float* qs = q_stats + (size_t)b * Kmax * 4;

  // the K accept tests, each on its own (thread i-1 takes test i)
  if (threadIdx.x < Kmax) {
    const int i = threadIdx.x + 1;
    uint8_t ok = 0;
    if (i <= K) {
      const int y = cand[b * cand_ld + i - 1];
      if (y < 0 || y >= V) {
        if (oob) atomicOr(oob, 2);
      } else if (p.greedy) {
        ok = (y == __float_as_int(ps[(i - 1) * 4 + 2])) ? 1 : 0;
      } else {
        const float lp = pl[(size_t)(i - 1) * V + y], lq = ql[(size_t)(i - 1) * V + y];
        const float py = lp >= ps[(i - 1) * 4 + 3] ? expf((lp - ps[(i - 1) * 4]) * inv_t) / ps[(i - 1) * 4 + 1] : 0.f;
        const float qy = lq >= qs[(i - 1) * 4 + 3] ? expf((lq - qs[(i - 1) * 4]) * inv_t) / qs[(i - 1) * 4 + 1] : 0.f;
        const float r = philox_uniform(p.seed, (uint32_t)i, (uint32_t)rnd, (uint32_t)b, STREAM_ACCEPT);
        ok = (r * qy < py) ? 1 : 0;                      // accept iff r < p(y)/q(y)
      }
    }
    flags[b * flags_ld + i - 1] = ok;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    int n = K;
    for (int i = 1; i <= K; ++i)
      if (!flags[b * flags_ld + i - 1]) { n = i - 1; break; }
    sh_n = n;
  }
  __syncthreads();
  const int n = sh_n;

  int y;
  if (p.greedy) {
    y = __float_as_int(ps[n * 4 + 2]);
  } else {
    const int nq = min(n, Kmax - 1);                     // the draft row is read when n < K only
    const float* prow = pl + (size_t)n * V;
    const float* qrow = ql + (size_t)nq * V;
    const float pmx = ps[n * 4], pinv = 1.0f / ps[n * 4 + 1], pthr = ps[n * 4 + 3];
    const float qmx = qs[nq * 4], qinv = 1.0f / qs[nq * 4 + 1], qthr = qs[nq * 4 + 3];
    const float k2 = inv_t * LOG2E;
    const float u = philox_uniform(p.seed, (uint32_t)(n + 1), (uint32_t)rnd, (uint32_t)b, STREAM_RESAMPLE);
    y = -1;
    if (rows_in_regs(prow, V) && rows_in_regs(qrow, V)) {
      // both rows were read a moment ago by row_stats_k: they come from L2 or the memory-side cache, into registers
      // in the layout of the walk, and every weight is evaluated once
      const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
      const int CW = (((V + SB / 64 - 1) / (SB / 64)) + 255) & ~255;
      const int beg = min(w * CW, V), end = min(beg + CW, V);
      float x[NR][4], f[NR][4];
      load_row_regs<false>(prow, beg, end, lane, x);
      if (n < K) load_row_regs<false>(qrow, beg, end, lane, f);
#pragma unroll
      for (int r = 0; r < NR; ++r)
#pragma unroll
        for (int e = 0; e < 4; ++e) x[r][e] = x[r][e] >= pthr ? row_weight(x[r][e], pmx, k2) * pinv : 0.f;   // padding: 0
      if (n < K) {                                       // residual Norm[(p_{n+1} - q_{n+1})_+]
#pragma unroll
        for (int r = 0; r < NR; ++r)
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const float qv = f[r][e] >= qthr ? row_weight(f[r][e], qmx, k2) * qinv : 0.f;
            f[r][e] = fmaxf(x[r][e] - qv, 0.f);
          }
        y = block_sample_regs(f, beg, end, lane, u, sh_w, &sh_res);
      }
      if (y < 0) y = block_sample_regs(x, beg, end, lane, u, sh_w, &sh_res);     // bonus token from p_{K+1}, or a residual with no mass
    } else {
      if (n < K) {
        y = block_sample(
            [&](int v) {
              const float pv = prow[v] >= pthr ? row_weight(prow[v], pmx, k2) * pinv : 0.f;
              const float qv = qrow[v] >= qthr ? row_weight(qrow[v], qmx, k2) * qinv : 0.f;
              return fmaxf(pv - qv, 0.f);
            },
            V, u, sh_w, &sh_res);
        __syncthreads();
      }
      if (y < 0)
        y = block_sample([&](int v) { return prow[v] >= pthr ? row_weight(prow[v], pmx, k2) * pinv : 0.f; }, V, u, sh_w, &sh_res);
    }
    if (y < 0) y = __float_as_int(ps[n * 4 + 2]);
  }
  if (y < 0 || y >= V) y = 0;                            // a row without a finite logit has no argmax
  if (threadIdx.x == 0) {
    n_out[b] = n;
    tok_out[b] = y;
  }
}

// ------------------------------------------------------------------ commit + rollback
// x <- x, y_1..y_n, y';  target cache keeps P + n positions, the draft cache
// min(P + n, P + K - 1); P grows by n + 1.  Also packs the round result for the host.
__global__ void commit_k(SeqState s, int32_t* __restrict__ result, int B, int max_seq) {
  const int b = blockIdx.x * blockDim.x + threadIdx.x;
  if (b >= B) return;
  int32_t* r = result + b * RES_LD;
  if (!s.active[b]) {
    for (int i = 0; i < RES_LD; ++i) r[i] = 0;
    r[36] = s.P[b];
    r[37] = s.kv_t[b];
    r[38] = s.kv_d[b];
    r[39] = *s.err;
    return;
  }
  const int P = s.P[b], K = s.K[b], n = s.n_acc[b], y = s.y_new[b];
  int32_t* tk = s.tokens + (size_t)b * max_seq;
  for (int i = 0; i < n; ++i) tk[P + i] = s.cand[b * CAND_LD + i];
  tk[P + n] = y;
  s.kv_t[b] = P + n;
  s.kv_d[b] = min(P + n, P + K - 1);
  s.P[b] = P + n + 1;
  s.round[b] += 1;
  r[0] = K;
  r[1] = n;
  r[2] = y;
  r[3] = __float_as_int(s.p_hat[b]);
  for (int i = 0; i < CAND_LD; ++i) r[4 + i] = i < K ? s.cand[b * CAND_LD + i] : -1;
  r[36] = s.P[b];
  r[37] = s.kv_t[b];
  r[38] = s.kv_d[b];
  r[39] = *s.err;
}

}  // namespace

hipError_t launch_begin_round(hipStream_t st, const SeqState& s, int B, int k_max, int max_seq) {
  if (B < 1 || k_max < 1 || k_max > CAND_LD) return hipErrorInvalidValue;
  hipLaunchKernelGGL(begin_round_k, dim3((B + 63) / 64), dim3(64), 0, st, s, B, k_max, max_seq);
  return hipGetLastError();
}

hipError_t launch_plan_draft(hipStream_t st, const SeqState& s, const RowPlan& rows, int B, int step, int max_seq) {
  if (B < 1 || 2 * B > MAX_ROWS || step < 1 || step > CAND_LD) return hipErrorInvalidValue;
  hipLaunchKernelGGL(plan_draft_k, dim3((B + 63) / 64), dim3(64), 0, st, s, rows, B, step, max_seq);
  return hipGetLastError();
}

hipError_t launch_plan_verify(hipStream_t st, const SeqState& s, const RowPlan& rows, int B, int rs, int max_seq) {
  if (B < 1 || rs < 2 || rs > CAND_LD + 1 || B * rs > MAX_ROWS) return hipErrorInvalidValue;
  hipLaunchKernelGGL(plan_verify_k, dim3(B), dim3(64), 0, st, s, rows, B, rs, max_seq);
  return hipGetLastError();
}

hipError_t launch_plan_verify_ragged(hipStream_t st, const SeqState& s, const RowPlan& rows, int B, int RS, int n_groups,
                                     int k_max, int max_seq, int32_t* dst) {
  if (B < 1 || B > 1024 || RS < 1 || n_groups < 1 || n_groups * RS > MAX_ROWS || !dst) return hipErrorInvalidValue;
  hipLaunchKernelGGL(plan_verify_ragged_k, dim3(1), dim3(((B + 63) / 64) * 64), 0, st, s, rows, B, RS, n_groups, k_max,
                     max_seq, dst);
  return hipGetLastError();
}

hipError_t launch_sample_stop(hipStream_t st, int dtype, const SeqState& s, const float* q_logits, int64_t ld_seq,
                              const void* z, const int* z_rows, int z_dim, const void* w_last, const void* b_last,
                              int have_head, const DecodeParams& p, int B, int V, int step, int32_t* host_flags,
                              uint32_t tick) {
  if (B < 1 || V < 1 || step < 1 || step > CAND_LD || !q_logits || !(p.temperature > 0.f)) return hipErrorInvalidValue;
  if (tick >= (1u << 30)) return hipErrorInvalidValue;
  if (have_head && (!z || !w_last || !b_last || z_dim < 1)) return hipErrorInvalidValue;
  if (dtype == DT_F32)
    hipLaunchKernelGGL(sample_stop_k<float>, dim3(B), dim3(SB), 0, st, s, q_logits, ld_seq, (const float*)z, z_rows,
                       z_dim, (const float*)w_last, (const float*)b_last, have_head, p, V, step, host_flags, tick);
  else if (dtype == DT_BF16)
    hipLaunchKernelGGL(sample_stop_k<bf16_t>, dim3(B), dim3(SB), 0, st, s, q_logits, ld_seq, (const bf16_t*)z, z_rows,
                       z_dim, (const bf16_t*)w_last, (const bf16_t*)b_last, have_head, p, V, step, host_flags, tick);
  else
    return hipErrorInvalidValue;
  return hipGetLastError();
}

hipError_t launch_row_stats(hipStream_t st, const float* p_logits, const float* q_logits, int Kmax, const int32_t* K,
                            int B, int V, float temperature, int top_k, float* p_stats, float* q_stats, int32_t* err,
                            int32_t* bad) {
  if (B < 1 || Kmax < 1 || V < 1 || top_k < 0 || !p_logits || !q_logits || !K || !p_stats || !q_stats ||
      !(temperature > 0.f))
    return hipErrorInvalidValue;
  const RowSet A{p_logits, p_stats, Kmax + 1, 1}, Bq{q_logits, q_stats, Kmax, 0};
  // rows of up to 32768 16-byte-aligned elements are held in registers
  const bool regs = V <= REG_V_MAX && (V & 3) == 0 &&
                    ((reinterpret_cast<uintptr_t>(p_logits) | reinterpret_cast<uintptr_t>(q_logits)) & 15) == 0;
  const bool topk = top_k > 0 && top_k < V;
  const dim3 grid(2 * Kmax + 1, B), block(SB);
  const float inv_t = 1.0f / temperature;
  if (regs && topk)
    hipLaunchKernelGGL((row_stats_k<true, true>), grid, block, 0, st, A, Bq, K, V, inv_t, top_k, err, bad);
  else if (regs)
    hipLaunchKernelGGL((row_stats_k<true, false>), grid, block, 0, st, A, Bq, K, V, inv_t, top_k, err, bad);
  else if (topk)
    hipLaunchKernelGGL((row_stats_k<false, true>), grid, block, 0, st, A, Bq, K, V, inv_t, top_k, err, bad);
  else
    hipLaunchKernelGGL((row_stats_k<false, false>), grid, block, 0, st, A, Bq, K, V, inv_t, top_k, err, bad);
  return hipGetLastError();
}

hipError_t launch_labels(hipStream_t st, const float* p_logits, const float* q_logits, int n, int V, float temperature,
                         int top_k, uint64_t seed, int slot0, int example, int32_t* Y, float* P) {
  if (n < 1 || V < 1 || top_k < 0 || !(temperature > 0.f) || !p_logits || !q_logits || !Y || !P)
    return hipErrorInvalidValue;
  hipLaunchKernelGGL(label_k, dim3(n), dim3(SB), 0, st, p_logits, q_logits, V, 1.0f / temperature, top_k, seed, slot0,
                     example, Y, P);
  return hipGetLastError();
}

hipError_t launch_mix(hipStream_t st, const int32_t* X, const int32_t* Y, int n, float r, uint64_t seed, int example,
                      int32_t* Z, int32_t* mask) {
  if (n < 1 || !X || !Y || !Z || !mask || !(r >= 0.f && r <= 1.f)) return hipErrorInvalidValue;
  hipLaunchKernelGGL(mix_k, dim3((n + 255) / 256), dim3(256), 0, st, X, Y, n, r, seed, example, Z, mask);
  return hipGetLastError();
}

hipError_t launch_accept(hipStream_t st, const float* p_logits, const float* q_logits, const float* p_stats,
                         const float* q_stats, const int32_t* cand, int cand_ld, const int32_t* K,
                         const int32_t* round, int round_const, const DecodeParams& p, int B, int Kmax, int V,
                         int32_t* n_out, int32_t* tok_out, uint8_t* flags, int flags_ld, int32_t* bad) {
  if (B < 1 || Kmax < 1 || Kmax > CAND_LD || V < 1 || cand_ld < Kmax || flags_ld < Kmax || !p_logits || !q_logits ||
      !p_stats || !q_stats || !cand || !K || !n_out || !tok_out || !flags || !(p.temperature > 0.f))
    return hipErrorInvalidValue;
  hipLaunchKernelGGL(accept_k, dim3(B), dim3(SB), 0, st, p_logits, q_logits, p_stats, q_stats, cand, cand_ld, K, round,
                     round_const, p, Kmax, V, n_out, tok_out, flags, flags_ld, bad);
  return hipGetLastError();
}

hipError_t launch_commit(hipStream_t st, const SeqState& s, int32_t* result, int B, int max_seq) {
  if (B < 1 || !result) return hipErrorInvalidValue;
  hipLaunchKernelGGL(commit_k, dim3((B + 63) / 64), dim3(64), 0, st, s, result, B, max_seq);
  return hipGetLastError();
}

}  // namespace sd
