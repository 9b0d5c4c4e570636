// Causal attention of a block of query rows against the KV cache with grouped
// queries (the target pass attends K+1 candidate positions at once; a draft step
// attends 1 or 2).
//
// Cache layout (chosen for this kernel): keys  [seq, kv_head, max_seq, hd]
//                                        values [seq, kv_head, hd, max_seq]  (transposed)
// so that both MFMA operands below are 16-byte loads straight from HBM/L2 and the
// probabilities never change lanes:
//
//   S^T = K Q^T : A operand = 16 keys x 32 d (a lane loads its key's row),
//                 B operand = 32 d x 16 query vectors.  Result lane (qv = lane%16,
//                 g = lane/16) holds scores of one query vector for 4 keys per tile.
//                 The 16 rows of key tile t are the keys key0 + 32 (t/2) + 8 (i/4) + 4 (t%2) + i%4,
//                 so after 4 tiles lane group g owns the keys key0 + 8g .. + 7 (tiles 0, 1) and
//                 key0 + 32 + 8g .. + 7 (tiles 2, 3): the k-blocks of the two value products.
//   O^T = V^T P^T: A operand = 16 d x 32 keys = two 16-byte loads of a transposed
//                 value row; B operand = 32 keys x 16 query vectors = exactly the
//                 registers the scores sit in (after exp and rounding to bf16).
//
// Query vectors of one (sequence, kv head) are the G = Hq/Hkv heads of every row of
// the sequence's row group: up to 17 x 8 = 136 vectors share each streamed K/V tile.
// Every wavefront takes one block of 64 keys (for its share of the query tiles) and
// writes one (max, sum, O) partial; a second kernel merges the partials in block order.
// The prompt pass (hundreds of rows, FULL = true) has enough query tiles to fill the chip
// without splitting the keys: there a wavefront walks every key block its tiles can see,
// carrying the online softmax, and writes the finished rows itself.
#include "common.hpp"
#include "kernels.hpp"

namespace sd {

namespace {

constexpr int KB = 64;          // keys per wavefront: one block, one partial
constexpr float NEG_BIG = -1.0e30f;

__device__ __forceinline__ uint4 ld16(const bf16_t* p) { return *reinterpret_cast<const uint4*>(p); }
__device__ __forceinline__ bf16x8 as_bf16x8(const uint4& v) {
  union { uint4 u; bf16x8 b; } c;
  c.u = v;
  return c.b;
}
__device__ __forceinline__ uint32_t pack2(float lo, float hi) { return (uint32_t)f2bf(lo) | ((uint32_t)f2bf(hi) << 16); }

// ------------------------------------------------------------------ MFMA kernel (bf16)
template <int HD, int QTW, bool FULL>
__global__ __launch_bounds__(256) void attn_mfma_k(const bf16_t* __restrict__ qbuf, const bf16_t* __restrict__ kcache,
                                                   const bf16_t* __restrict__ vcache,
                                                   const int32_t* __restrict__ row_seq,
                                                   const int32_t* __restrict__ row_pos,
                                                   const int32_t* __restrict__ grp_seq,
                                                   const int32_t* __restrict__ grp_end, float* __restrict__ scratch,
                                                   bf16_t* __restrict__ out, int RS, int Hq, int Hkv, int max_seq,
                                                   int QW, int NQG, int NSP) {
  constexpr int DT = HD / 16;          // 16-wide tiles of the head dimension
  constexpr int KS = HD / 32;          // MFMA k-steps of the score product
  constexpr int STRIDE = HD + 4;       // floats per partial: O[HD], max, sum, pad
  const int kh = blockIdx.x / NQG, qg = blockIdx.x % NQG;
  const int grp = blockIdx.y, c = blockIdx.z;
  const int G = Hq / Hkv;
  const int seq = grp_seq[grp], kv_end = grp_end[grp];
  if (seq < 0) return;

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int li = lane & 15, g = lane >> 4;
  const int KW = 4 / QW;
  const int qw = wave % QW, kw = wave / QW;
  const int sp = c * KW + kw;              // this wave's key block, also its partial's index
  if (FULL && kw != 0) return;             // keys are not split: one wave per set of query tiles
  const int kbeg = FULL ? 0 : sp * KB;
  if (kbeg >= kv_end) return;
  int kend = min(kbeg + KB, kv_end);

  const bf16_t* kbase = kcache + ((size_t)seq * Hkv + kh) * (size_t)max_seq * HD;
  const bf16_t* vbase = vcache + ((size_t)seq * Hkv + kh) * (size_t)HD * max_seq;
  const int QV = RS * G;
  const float scale = rsqrtf((float)HD);

  // this lane's query vector in each of the wave's tiles
  uint4 qf[QTW][KS];
  int limit[QTW], orow[QTW], ohead[QTW];
#pragma unroll
  for (int q = 0; q < QTW; ++q) {
    const int qt = qg * (QW * QTW) + qw + QW * q;
    const int qv = qt * 16 + li;
    limit[q] = -1;
    orow[q] = -1;
    ohead[q] = 0;
#pragma unroll
    for (int j = 0; j < KS; ++j) qf[q][j] = uint4{0u, 0u, 0u, 0u};
    if (qv < QV) {
      const int rr = qv / G, gh = qv - rr * G;
      const int m = grp * RS + rr;
      if (row_seq[m] >= 0) {
        limit[q] = row_pos[m];
        orow[q] = m;
        ohead[q] = kh * G + gh;
        // k-step j, lane group g takes the 8 head dimensions 32 j + 8 g .. (the same for keys below), so that
        // one load instruction reads 64 contiguous bytes of each of its rows
        const bf16_t* qp = qbuf + ((size_t)m * Hq + ohead[q]) * HD + g * 8;
#pragma unroll
        for (int j = 0; j < KS; ++j) qf[q][j] = ld16(qp + j * 32);
      }
    }
  }

  if (FULL) {                              // causal: nothing beyond the largest position of the wave's rows
    int lim = -1;
#pragma unroll
    for (int q = 0; q < QTW; ++q) lim = max(lim, limit[q]);
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) lim = max(lim, __shfl_xor(lim, o, WAVE));
    kend = min(lim + 1, kv_end);
  }

  floatx4 o[QTW][DT];
  float mrun[QTW], lrun[QTW];
#pragma unroll
  for (int q = 0; q < QTW; ++q) {
    mrun[q] = NEG_BIG;
    lrun[q] = 0.f;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) o[q][dt] = floatx4{0.f, 0.f, 0.f, 0.f};
  }

  for (int key0 = kbeg; key0 < kend; key0 += KB) {
    // value rows are requested first: they are not needed before the softmax is done
    uint4 vf[DT][2];
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) {
      const bf16_t* vp = vbase + (size_t)(dt * 16 + li) * max_seq + key0 + 8 * g;
      vf[dt][0] = ld16(vp);                    // keys key0 + 8 g .. + 7: the four lane groups read 64 contiguous bytes
      vf[dt][1] = ld16(vp + 32);               // keys key0 + 32 + 8 g ..
    }
    // ---- scores: 4 key tiles x QTW query tiles
    floatx4 sacc[QTW][4];
#pragma unroll
    for (int q = 0; q < QTW; ++q)
#pragma unroll
      for (int kt = 0; kt < 4; ++kt) sacc[q][kt] = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int kt = 0; kt < 4; ++kt) {
      const int key = key0 + 32 * (kt >> 1) + 8 * (li >> 2) + 4 * (kt & 1) + (li & 3);   // < max_seq (multiple of 64)
      const bf16_t* kp = kbase + (size_t)key * HD + g * 8;
      uint4 kf[KS];
#pragma unroll
      for (int j = 0; j < KS; ++j) kf[j] = ld16(kp + j * 32);
#pragma unroll
      for (int j = 0; j < KS; ++j)
#pragma unroll
        for (int q = 0; q < QTW; ++q)
          sacc[q][kt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(kf[j]), as_bf16x8(qf[q][j]),
                                                                sacc[q][kt], 0, 0, 0);
    }
    // ---- online softmax; lane (li, g) holds keys key0 + 32 (kt/2) + 8 g + 4 (kt%2) + r of query vector li
    uint4 pf[QTW][2];
#pragma unroll
    for (int q = 0; q < QTW; ++q) {
      float bmax = NEG_BIG;
#pragma unroll
      for (int kt = 0; kt < 4; ++kt)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const int key = key0 + 32 * (kt >> 1) + 8 * g + 4 * (kt & 1) + r;
          const float s = sacc[q][kt][r] * scale;
          sacc[q][kt][r] = s;
          if (key <= limit[q]) bmax = fmaxf(bmax, s);
        }
      bmax = fmaxf(bmax, __shfl_xor(bmax, 16, WAVE));
      bmax = fmaxf(bmax, __shfl_xor(bmax, 32, WAVE));
      const float mnew = fmaxf(mrun[q], bmax);
      const float alpha = __expf(mrun[q] - mnew);
      float p[4][4];
      float lsum = 0.f;
#pragma unroll
      for (int kt = 0; kt < 4; ++kt)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const int key = key0 + 32 * (kt >> 1) + 8 * g + 4 * (kt & 1) + r;
          const float e = (key <= limit[q]) ? __expf(sacc[q][kt][r] - mnew) : 0.f;
          p[kt][r] = e;
          lsum += e;
        }
      lsum += __shfl_xor(lsum, 16, WAVE);
      lsum += __shfl_xor(lsum, 32, WAVE);
      lrun[q] = lrun[q] * alpha + lsum;
      mrun[q] = mnew;
#pragma unroll
      for (int dt = 0; dt < DT; ++dt) o[q][dt] *= alpha;
#pragma unroll
      for (int u = 0; u < 2; ++u)
        pf[q][u] = uint4{pack2(p[2 * u][0], p[2 * u][1]), pack2(p[2 * u][2], p[2 * u][3]),
                         pack2(p[2 * u + 1][0], p[2 * u + 1][1]), pack2(p[2 * u + 1][2], p[2 * u + 1][3])};
    }
    // ---- O^T += V^T P^T
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) {
      const uint4 v0 = vf[dt][0], v1 = vf[dt][1];
#pragma unroll
      for (int q = 0; q < QTW; ++q) {
        o[q][dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(v0), as_bf16x8(pf[q][0]), o[q][dt], 0, 0, 0);
        o[q][dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(v1), as_bf16x8(pf[q][1]), o[q][dt], 0, 0, 0);
      }
    }
  }

  // lane (qv = li, d = 16 dt + 4 g + r)
  if (FULL) {
#pragma unroll
    for (int q = 0; q < QTW; ++q) {
      if (orow[q] < 0) continue;
      const float inv = lrun[q] > 0.f ? 1.0f / lrun[q] : 0.f;
      bf16_t* dst = out + ((size_t)orow[q] * Hq + ohead[q]) * HD;
#pragma unroll
      for (int dt = 0; dt < DT; ++dt) {
        const floatx4 v = o[q][dt];
        *reinterpret_cast<uint2*>(dst + dt * 16 + 4 * g) = uint2{pack2(v[0] * inv, v[1] * inv), pack2(v[2] * inv, v[3] * inv)};
      }
    }
    return;
  }
#pragma unroll
  for (int q = 0; q < QTW; ++q) {
    if (orow[q] < 0) continue;
    float* dst = scratch + (((size_t)orow[q] * Hq + ohead[q]) * NSP + sp) * STRIDE;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) *reinterpret_cast<floatx4*>(dst + dt * 16 + 4 * g) = o[q][dt];
    if (g == 0) {
      dst[HD] = mrun[q];
      dst[HD + 1] = lrun[q];
    }
  }
}

template <int HD>
__global__ __launch_bounds__(HD) void attn_merge_k(const float* __restrict__ scratch, const int32_t* __restrict__ row_seq,
                                                   const int32_t* __restrict__ grp_end, bf16_t* __restrict__ out, int RS,
                                                   int Hq, int NSP) {
  constexpr int STRIDE = HD + 4;
  constexpr int MAXP = 512;            // key blocks whose weights fit the LDS table (32768 keys)
  __shared__ float s_w[MAXP];
  __shared__ float s_l[MAXP];
  const int m = blockIdx.x, h = blockIdx.y, d = threadIdx.x;
  bf16_t* dst = out + ((size_t)m * Hq + h) * HD + d;
  if (row_seq[m] < 0) {
    *dst = 0;
    return;
  }
  const int kv_end = grp_end[m / RS];
  const float* src = scratch + ((size_t)m * Hq + h) * NSP * STRIDE;
  const int nsp = min(min(NSP, MAXP), (kv_end + KB - 1) / KB);
  // the partials' maxima and sums go through LDS once; every thread then owns one column
  for (int sp = d; sp < nsp; sp += HD) {
    s_w[sp] = src[sp * STRIDE + HD];
    s_l[sp] = src[sp * STRIDE + HD + 1];
  }
  __syncthreads();
  float mx = NEG_BIG;
  for (int sp = 0; sp < nsp; ++sp) mx = fmaxf(mx, s_w[sp]);
  float num = 0.f, den = 0.f;
#pragma unroll 8
  for (int sp = 0; sp < nsp; ++sp) {
    const float w = __expf(s_w[sp] - mx);
    num = fmaf(w, src[sp * STRIDE + d], num);
    den = fmaf(w, s_l[sp], den);
  }
  *dst = f2bf(den > 0.f ? num / den : 0.f);
}

// ------------------------------------------------------------------ plain kernel (fp32 models)
// One workgroup per (query head, row group); rows one after another; scores of the
// whole prefix in LDS.  Sizes are tiny there.
template <typename T>
__global__ __launch_bounds__(256) void attn_plain_k(const T* __restrict__ qbuf, const T* __restrict__ kcache,
                                                    const T* __restrict__ vcache, const int32_t* __restrict__ row_seq,
                                                    const int32_t* __restrict__ row_pos, T* __restrict__ out, int RS,
                                                    int Hq, int Hkv, int hd, int max_seq) {
  extern __shared__ float sm[];
  float* sc = sm;                       // [max_kv_len]
  float* qs = sm + max_seq;             // [hd]
  float* red = qs + hd;                 // [256]
  const int h = blockIdx.x, grp = blockIdx.y;
  const int kh = h / (Hq / Hkv);
  const float scale = 1.0f / sqrtf((float)hd);
  for (int rr = 0; rr < RS; ++rr) {
    const int m = grp * RS + rr;
    const int seq = row_seq[m];
    T* dst = out + ((size_t)m * Hq + h) * hd;
    if (seq < 0) {
      for (int d = threadIdx.x; d < hd; d += 256) Elem<T>::st(dst + d, 0.f);
      continue;
    }
    const int n = row_pos[m] + 1;
    const T* kb = kcache + ((size_t)seq * Hkv + kh) * (size_t)max_seq * hd;
    const T* vb = vcache + ((size_t)seq * Hkv + kh) * (size_t)hd * max_seq;
    __syncthreads();
    for (int d = threadIdx.x; d < hd; d += 256) qs[d] = Elem<T>::ld(qbuf + ((size_t)m * Hq + h) * hd + d);
    __syncthreads();
    float mx = NEG_BIG;
    for (int key = threadIdx.x; key < n; key += 256) {
      float s = 0.f;
      for (int d = 0; d < hd; ++d) s = fmaf(qs[d], Elem<T>::ld(kb + (size_t)key * hd + d), s);
      s *= scale;
      sc[key] = s;
      mx = fmaxf(mx, s);
    }
    mx = block_max(mx, red);
    float l = 0.f;
    for (int key = threadIdx.x; key < n; key += 256) {
      const float e = expf(sc[key] - mx);
      sc[key] = e;
      l += e;
    }
    l = block_sum(l, red);
    // value product: thread (d, part) sums a strided subset of keys, parts combined in order
    const int parts = 256 / hd;                         // hd in {32, 64, 128}
    const int d = threadIdx.x % hd, part = threadIdx.x / hd;
    float acc = 0.f;
    if (part < parts)
      for (int key = part; key < n; key += parts) acc = fmaf(sc[key], Elem<T>::ld(vb + (size_t)d * max_seq + key), acc);
    red[threadIdx.x] = acc;
    __syncthreads();
    if (threadIdx.x < hd) {
      float t = 0.f;
      for (int p = 0; p < parts; ++p) t += red[p * hd + threadIdx.x];
      Elem<T>::st(dst + threadIdx.x, t / l);
    }
  }
}

struct MfmaShape { int QW, QTW, NQG; };

// full (prompt pass: a wavefront walks all its key blocks): two query tiles per wavefront halve the K/V traffic.
// Split keys (a round's passes): one tile per wavefront and more workgroups instead: the launch is a chain of
// latencies (q, keys, products, softmax, values, products, partial), and a wavefront with two tiles walks the softmax
// twice (9..16 rows x 8 grouped heads: 14.0 us with two tiles per wavefront, 8.5 us for the same kernel with one).
MfmaShape mfma_shape(int RS, int G, bool full) {
  const int n_qt = (RS * G + 15) / 16;
  MfmaShape s;
  if (n_qt <= 1) s = {1, 1, 1};
  else if (n_qt <= 2) s = {2, 1, 1};
  else if (n_qt <= 4) s = {4, 1, 1};
  else if (full) s = {4, 2, (n_qt + 7) / 8};
  else s = {4, 1, (n_qt + 3) / 4};
  return s;
}

bool use_plain(int dtype) { return dtype == DT_F32; }

}  // namespace

size_t attn_scratch_floats(int M, int Hq, int hd, int max_seq) {
  const int nsp = (max_seq + KB - 1) / KB;
  return (size_t)M * Hq * nsp * (hd + 4);
}

hipError_t launch_attention(hipStream_t st, int dtype, const void* qbuf, const void* kcache, const void* vcache,
                            const RowPlan& rows, void* out, float* scratch, int M, int RS, int Hq, int Hkv, int hd,
                            int max_seq, int max_kv_len, bool full) {
  if (M < 1 || M > (full ? MAX_PREFILL_ROWS : MAX_ROWS) || RS < 1 || M % RS != 0 || Hq < 1 || Hkv < 1 || Hq % Hkv != 0 || max_kv_len < 1 ||
      max_kv_len > max_seq || !qbuf || !kcache || !vcache || !out || !rows.seq || !rows.pos || !rows.gseq || !rows.gend)
    return hipErrorInvalidValue;
  const int ngroups = M / RS;
  if (use_plain(dtype)) {
    if (full) return hipErrorInvalidValue;
    if (hd != 32 && hd != 64 && hd != 128) return hipErrorInvalidValue;
    const size_t lds = ((size_t)max_seq + hd + 256) * sizeof(float);
    if (lds > 64 * 1024) return hipErrorInvalidValue;
    hipLaunchKernelGGL(attn_plain_k<float>, dim3(Hq, ngroups), dim3(256), lds, st, (const float*)qbuf,
                       (const float*)kcache, (const float*)vcache, rows.seq, rows.pos, (float*)out, RS, Hq, Hkv, hd,
                       max_seq);
    return hipGetLastError();
  }
  if (dtype != DT_BF16 || (hd != 64 && hd != 128) || max_seq % KB != 0 || max_seq > 512 * KB || (!scratch && !full))
    return hipErrorInvalidValue;
  const MfmaShape sh = mfma_shape(RS, Hq / Hkv, full);
  const int KW = 4 / sh.QW;
  const int nsplit = ((max_kv_len + KB - 1) / KB + KW - 1) / KW;
  const int NSP = (max_seq + KB - 1) / KB;
  const dim3 grid(Hkv * sh.NQG, ngroups, full ? 1 : nsplit);
  const bf16_t *q = (const bf16_t*)qbuf, *k = (const bf16_t*)kcache, *v = (const bf16_t*)vcache;
#define SD_ATTN_LAUNCH(HD_, QTW_, FULL_)                                                                       \
  hipLaunchKernelGGL((attn_mfma_k<HD_, QTW_, FULL_>), grid, dim3(256), 0, st, q, k, v, rows.seq, rows.pos,       \
                     rows.gseq, rows.gend, scratch, (bf16_t*)out, RS, Hq, Hkv, max_seq, sh.QW, sh.NQG, NSP)
  if (full) {
    if (hd == 128) {
      if (sh.QTW == 1) SD_ATTN_LAUNCH(128, 1, true); else SD_ATTN_LAUNCH(128, 2, true);
    } else {
      if (sh.QTW == 1) SD_ATTN_LAUNCH(64, 1, true); else SD_ATTN_LAUNCH(64, 2, true);
    }
    return hipGetLastError();
  }
  if (hd == 128) SD_ATTN_LAUNCH(128, 1, false); else SD_ATTN_LAUNCH(64, 1, false);      // split keys: one tile per wavefront
#undef SD_ATTN_LAUNCH
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  if (hd == 128)
    hipLaunchKernelGGL(attn_merge_k<128>, dim3(M, Hq), dim3(128), 0, st, scratch, rows.seq, rows.gend, (bf16_t*)out,
                       RS, Hq, NSP);
  else
    hipLaunchKernelGGL(attn_merge_k<64>, dim3(M, Hq), dim3(64), 0, st, scratch, rows.seq, rows.gend, (bf16_t*)out, RS,
                       Hq, NSP);
  return hipGetLastError();
}

}  // namespace sd
