// Small fused kernels around the weight-streaming GEMMs.  Each consumes the GEMM's
// per-K-slice partial sums (added in slice order, so results are reproducible) and
// fuses the next elementwise step of the Llama-style decoder layer: RMSNorm,
// rotary embedding + KV-cache append, SiLU * up, residual add, head activation.
#include "common.hpp"
#include "kernels.hpp"

namespace sd {

namespace {

constexpr int EW_THREADS = 256;

// RMSNorm is split in two launches so that a handful of rows still fills the chip:
// the first kernel (embedding gather, or residual + partial sums) writes x and one
// sum of squares per 1024-column block; the second adds those in block order and
// scales.  Both run (columns / 1024) x rows workgroups.
constexpr int NORM_COLS = 4 * EW_THREADS;

template <typename T>
__global__ __launch_bounds__(EW_THREADS) void embed_k(const T* __restrict__ emb, const int32_t* __restrict__ tok,
                                                      float* __restrict__ x, float* __restrict__ ssq, int d,
                                                      int vocab) {
  __shared__ float red[EW_THREADS / 64];
  const int m = blockIdx.y;
  int t = tok[m];
  t = t < 0 ? 0 : (t >= vocab ? vocab - 1 : t);
  const T* e = emb + (size_t)t * d;
  float ss = 0.f;
#pragma unroll
  for (int u = 0; u < 4; ++u) {
    const int i = blockIdx.x * NORM_COLS + u * EW_THREADS + threadIdx.x;
    if (i < d) {
      const float v = Elem<T>::ld(e + i);
      x[(size_t)m * d + i] = v;
      ss = fmaf(v, v, ss);
    }
  }
  ss = block_sum(ss, red);
  if (threadIdx.x == 0) ssq[m * gridDim.x + blockIdx.x] = ss;
}

__global__ __launch_bounds__(EW_THREADS) void add_partials_k(const float* __restrict__ part, int S,
                                                             float* __restrict__ x, float* __restrict__ ssq, int M,
                                                             int d) {
  __shared__ float red[EW_THREADS / 64];
  const int m = blockIdx.y;
  float ss = 0.f;
#pragma unroll
  for (int u = 0; u < 4; ++u) {
    const int i = blockIdx.x * NORM_COLS + u * EW_THREADS + threadIdx.x;
    if (i < d) {
      float v = x[(size_t)m * d + i];
      for (int s = 0; s < S; ++s) v += part[((size_t)s * M + m) * d + i];
      x[(size_t)m * d + i] = v;
      ss = fmaf(v, v, ss);
    }
  }
  ss = block_sum(ss, red);
  if (threadIdx.x == 0) ssq[m * gridDim.x + blockIdx.x] = ss;
}

template <typename T>
__global__ __launch_bounds__(EW_THREADS) void norm_k(const float* __restrict__ x, const float* __restrict__ ssq,
                                                     const T* __restrict__ g, float eps, T* __restrict__ xn, int d) {
  const int m = blockIdx.y;
  float ss = 0.f;
  for (int b = 0; b < (int)gridDim.x; ++b) ss += ssq[m * gridDim.x + b];
  const float inv = 1.0f / sqrtf(ss / (float)d + eps);
#pragma unroll
  for (int u = 0; u < 4; ++u) {
    const int i = blockIdx.x * NORM_COLS + u * EW_THREADS + threadIdx.x;
    if (i < d) Elem<T>::st(xn + (size_t)m * d + i, x[(size_t)m * d + i] * inv * Elem<T>::ld(g + i));
  }
}

// Residual add + RMSNorm of one row by one 1024-thread workgroup: every thread owns up
// to 4 float4 column groups, issues all of its partial-sum loads at once, keeps the
// sums in registers across the row-wide reduction, and writes x and xn.  Used when
// d <= 16384 and d % 4 == 0; one launch instead of two.
constexpr int ROW_THREADS = 1024;
constexpr int ROW_MAXU = 4;

template <typename T> struct Pack4;
template <> struct Pack4<float> {
  static __device__ __forceinline__ float4 ld(const float* p) { return *reinterpret_cast<const float4*>(p); }
  static __device__ __forceinline__ void st(float* p, float4 v) { *reinterpret_cast<float4*>(p) = v; }
};
template <> struct Pack4<bf16_t> {
  static __device__ __forceinline__ float4 ld(const bf16_t* p) {
    const uint2 u = *reinterpret_cast<const uint2*>(p);
    return float4{__uint_as_float(u.x << 16), __uint_as_float(u.x & 0xffff0000u), __uint_as_float(u.y << 16),
                  __uint_as_float(u.y & 0xffff0000u)};
  }
  static __device__ __forceinline__ void st(bf16_t* p, float4 v) {
    uint2 u;
    u.x = (uint32_t)f2bf(v.x) | ((uint32_t)f2bf(v.y) << 16);
    u.y = (uint32_t)f2bf(v.z) | ((uint32_t)f2bf(v.w) << 16);
    *reinterpret_cast<uint2*>(p) = u;
  }
};

template <typename T>
__global__ __launch_bounds__(ROW_THREADS) void add_norm_row_k(const float* __restrict__ part, int S,
                                                              const T* __restrict__ g, float eps,
                                                              float* __restrict__ x, T* __restrict__ xn, int M, int d) {
  __shared__ float red[ROW_THREADS / 64];
  const int m = blockIdx.x;
  float4 v[ROW_MAXU];
  float ss = 0.f;
#pragma unroll
  for (int u = 0; u < ROW_MAXU; ++u) {
    const int i = (u * ROW_THREADS + threadIdx.x) * 4;
    if (i < d) {
      float4 a = *reinterpret_cast<const float4*>(x + (size_t)m * d + i);
#pragma unroll 4
      for (int s = 0; s < S; ++s) {
        const float4 p = *reinterpret_cast<const float4*>(part + ((size_t)s * M + m) * d + i);
        a.x += p.x; a.y += p.y; a.z += p.z; a.w += p.w;
      }
      *reinterpret_cast<float4*>(x + (size_t)m * d + i) = a;
      v[u] = a;
      ss += a.x * a.x + a.y * a.y + a.z * a.z + a.w * a.w;
    }
  }
  ss = block_sum(ss, red);
  const float inv = 1.0f / sqrtf(ss / (float)d + eps);
#pragma unroll
  for (int u = 0; u < ROW_MAXU; ++u) {
    const int i = (u * ROW_THREADS + threadIdx.x) * 4;
    if (i < d) {
      const float4 gg = Pack4<T>::ld(g + i);
      Pack4<T>::st(xn + (size_t)m * d + i,
                   float4{v[u].x * inv * gg.x, v[u].y * inv * gg.y, v[u].z * inv * gg.z, v[u].w * inv * gg.w});
    }
  }
}

// Embedding gather + RMSNorm of one row by one workgroup (same conditions as add_norm_row_k): one launch
// instead of two at the head of every forward pass.
template <typename T>
__global__ __launch_bounds__(ROW_THREADS) void embed_norm_row_k(const T* __restrict__ emb, const int32_t* __restrict__ tok,
                                                                const T* __restrict__ g, float eps,
                                                                float* __restrict__ x, T* __restrict__ xn, int d,
                                                                int vocab) {
  __shared__ float red[ROW_THREADS / 64];
  const int m = blockIdx.x;
  int t = tok[m];
  t = t < 0 ? 0 : (t >= vocab ? vocab - 1 : t);
  const T* e = emb + (size_t)t * d;
  float4 v[ROW_MAXU];
  float ss = 0.f;
#pragma unroll
  for (int u = 0; u < ROW_MAXU; ++u) {
    const int i = (u * ROW_THREADS + threadIdx.x) * 4;
    if (i < d) {
      const float4 a = Pack4<T>::ld(e + i);
      *reinterpret_cast<float4*>(x + (size_t)m * d + i) = a;
      v[u] = a;
      ss += a.x * a.x + a.y * a.y + a.z * a.z + a.w * a.w;
    }
  }
  ss = block_sum(ss, red);
  const float inv = 1.0f / sqrtf(ss / (float)d + eps);
#pragma unroll
  for (int u = 0; u < ROW_MAXU; ++u) {
    const int i = (u * ROW_THREADS + threadIdx.x) * 4;
    if (i < d) {
      const float4 gg = Pack4<T>::ld(g + i);
      Pack4<T>::st(xn + (size_t)m * d + i,
                   float4{v[u].x * inv * gg.x, v[u].y * inv * gg.y, v[u].z * inv * gg.z, v[u].w * inv * gg.w});
    }
  }
}

// One block per (row, head slot): slots [0, Hq) are query heads, [Hq, Hq+Hkv) key
// heads, [Hq+Hkv, Hq+2Hkv) value heads.
template <typename T>
__global__ __launch_bounds__(64) void rope_kv_k(const float* __restrict__ part, int S,
                                                const int32_t* __restrict__ row_seq,
                                                const int32_t* __restrict__ row_pos,
                                                const float* __restrict__ cos_sin, T* __restrict__ qbuf,
                                                T* __restrict__ kcache, T* __restrict__ vcache, int M, int Hq,
                                                int Hkv, int hd, int max_seq) {
  const int m = blockIdx.x, slot = blockIdx.y;
  const int seq = row_seq[m];
  if (seq < 0) return;
  const int pos = row_pos[m];
  const int ncols = (Hq + 2 * Hkv) * hd;
  const int half = hd >> 1;
  const float* p0 = part + (size_t)m * ncols + (size_t)slot * hd;
  const size_t sstride = (size_t)M * ncols;
  if (slot < Hq + Hkv) {
    for (int i = threadIdx.x; i < half; i += 64) {
      float a = 0.f, b = 0.f;
#pragma unroll 4
      for (int s = 0; s < S; ++s) {
        a += p0[s * sstride + i];
        b += p0[s * sstride + i + half];
      }
      const float c = cos_sin[((size_t)pos * half + i) * 2], sn = cos_sin[((size_t)pos * half + i) * 2 + 1];
      float ra, rb;
      rope_pair(a, b, c, sn, ra, rb);
      if (slot < Hq) {
        T* q = qbuf + ((size_t)m * Hq + slot) * hd;
        Elem<T>::st(q + i, ra);
        Elem<T>::st(q + i + half, rb);
      } else {
        T* k = kcache + (((size_t)seq * Hkv + (slot - Hq)) * max_seq + pos) * hd;
        Elem<T>::st(k + i, ra);
        Elem<T>::st(k + i + half, rb);
      }
    }
  } else {
    T* v = vcache + ((size_t)seq * Hkv + (slot - Hq - Hkv)) * hd * (size_t)max_seq + pos;
    for (int i = threadIdx.x; i < hd; i += 64) {
      float a = 0.f;
#pragma unroll 4
      for (int s = 0; s < S; ++s) a += p0[s * sstride + i];
      Elem<T>::st(v + (size_t)i * max_seq, a);            // value cache is stored transposed: [hd, max_seq]
    }
  }
}

template <typename T>
__global__ __launch_bounds__(EW_THREADS) void silu_mul_k(const float* __restrict__ part, int S,
                                                         T* __restrict__ act, int M, int ffn) {
  const int m = blockIdx.y;
  const int f = blockIdx.x * EW_THREADS + threadIdx.x;
  if (f >= ffn) return;
  float g = 0.f, u = 0.f;
#pragma unroll 4
  for (int s = 0; s < S; ++s) {
    const float* p = part + ((size_t)s * M + m) * (2 * (size_t)ffn);
    g += p[f];
    u += p[ffn + f];
  }
  Elem<T>::st(act + (size_t)m * ffn + f, g / (1.0f + expf(-g)) * u);
}

// Row m = (group m / RS, slot m % RS) goes to out[group * ld_group + slot * ld_row + n]; with a
// destination map, to out[dst[m] * ld_row + n] instead (rows with dst[m] < 0 are dropped).
__global__ __launch_bounds__(EW_THREADS) void reduce_rows_k(const float* __restrict__ part, int S,
                                                            float* __restrict__ out, int RS, int64_t ld_group,
                                                            int64_t ld_row, const int32_t* __restrict__ dst, int M,
                                                            int N) {
  const int m = blockIdx.y;
  const int n = blockIdx.x * EW_THREADS + threadIdx.x;
  if (n >= N) return;
  if (dst && dst[m] < 0) return;
  float v = 0.f;
#pragma unroll 4
  for (int s = 0; s < S; ++s) v += part[((size_t)s * M + m) * N + n];
  const size_t o = dst ? (size_t)dst[m] * ld_row : (size_t)(m / RS) * ld_group + (size_t)(m % RS) * ld_row;
  out[o + n] = v;
}

template <typename T>
__global__ __launch_bounds__(EW_THREADS) void head_act_k(const float* __restrict__ part, int S,
                                                         const T* __restrict__ bias, const T* __restrict__ z_in,
                                                         const int* __restrict__ z_in_rows, T* __restrict__ z_out,
                                                         int residual, int M, int n) {
  const int m = blockIdx.y;
  const int i = blockIdx.x * EW_THREADS + threadIdx.x;
  if (i >= n) return;
  float a = Elem<T>::ld(bias + i);
  for (int s = 0; s < S; ++s) a += part[((size_t)s * M + m) * n + i];
  a = a / (1.0f + expf(-a));
  if (residual) a += Elem<T>::ld(z_in + (size_t)(z_in_rows ? z_in_rows[m] : m) * n + i);
  Elem<T>::st(z_out + (size_t)m * n + i, a);
}

inline bool bad_rows(int M) { return M < 1 || M > MAX_PREFILL_ROWS; }

}  // namespace

#define SD_DISPATCH_T(dtype, CALL_F32, CALL_BF16) \
  if ((dtype) == DT_F32) { CALL_F32; } else if ((dtype) == DT_BF16) { CALL_BF16; } else return hipErrorInvalidValue;

hipError_t launch_embed_norm(hipStream_t st, int dtype, const void* emb, const void* g, float eps,
                             const int32_t* tok, float* x, void* xn, float* ssq, int M, int d, int vocab) {
  if (bad_rows(M) || d < 1 || !emb || !g || !tok || !x || !xn || !ssq) return hipErrorInvalidValue;
  const dim3 grid((d + NORM_COLS - 1) / NORM_COLS, M);
  if (grid.x > NORM_MAX_BLOCKS) return hipErrorInvalidValue;
  if (d % 4 == 0 && d <= ROW_THREADS * 4 * ROW_MAXU &&
      ((reinterpret_cast<uintptr_t>(emb) | reinterpret_cast<uintptr_t>(g) | reinterpret_cast<uintptr_t>(x) |
        reinterpret_cast<uintptr_t>(xn)) & 15) == 0) {
    SD_DISPATCH_T(dtype,
                  hipLaunchKernelGGL(embed_norm_row_k<float>, dim3(M), dim3(ROW_THREADS), 0, st, (const float*)emb, tok,
                                     (const float*)g, eps, x, (float*)xn, d, vocab),
                  hipLaunchKernelGGL(embed_norm_row_k<bf16_t>, dim3(M), dim3(ROW_THREADS), 0, st, (const bf16_t*)emb,
                                     tok, (const bf16_t*)g, eps, x, (bf16_t*)xn, d, vocab));
    return hipGetLastError();
  }
  SD_DISPATCH_T(dtype,
                hipLaunchKernelGGL(embed_k<float>, grid, dim3(EW_THREADS), 0, st, (const float*)emb, tok, x, ssq, d,
                                   vocab);
                hipLaunchKernelGGL(norm_k<float>, grid, dim3(EW_THREADS), 0, st, x, ssq, (const float*)g, eps,
                                   (float*)xn, d),
                hipLaunchKernelGGL(embed_k<bf16_t>, grid, dim3(EW_THREADS), 0, st, (const bf16_t*)emb, tok, x, ssq, d,
                                   vocab);
                hipLaunchKernelGGL(norm_k<bf16_t>, grid, dim3(EW_THREADS), 0, st, x, ssq, (const bf16_t*)g, eps,
                                   (bf16_t*)xn, d));
  return hipGetLastError();
}

hipError_t launch_add_norm(hipStream_t st, int dtype, const float* part, int S, const void* g, float eps,
                           float* x, void* xn, float* ssq, int M, int d) {
  if (bad_rows(M) || d < 1 || S < 1 || !part || !g || !x || !xn || !ssq) return hipErrorInvalidValue;
  const dim3 grid((d + NORM_COLS - 1) / NORM_COLS, M);
  if (grid.x > NORM_MAX_BLOCKS) return hipErrorInvalidValue;
  if (d % 4 == 0 && d <= ROW_THREADS * 4 * ROW_MAXU) {
    SD_DISPATCH_T(dtype,
                  hipLaunchKernelGGL(add_norm_row_k<float>, dim3(M), dim3(ROW_THREADS), 0, st, part, S,
                                     (const float*)g, eps, x, (float*)xn, M, d),
                  hipLaunchKernelGGL(add_norm_row_k<bf16_t>, dim3(M), dim3(ROW_THREADS), 0, st, part, S,
                                     (const bf16_t*)g, eps, x, (bf16_t*)xn, M, d));
    return hipGetLastError();
  }
  hipLaunchKernelGGL(add_partials_k, grid, dim3(EW_THREADS), 0, st, part, S, x, ssq, M, d);
  SD_DISPATCH_T(dtype,
                hipLaunchKernelGGL(norm_k<float>, grid, dim3(EW_THREADS), 0, st, x, ssq, (const float*)g, eps,
                                   (float*)xn, d),
                hipLaunchKernelGGL(norm_k<bf16_t>, grid, dim3(EW_THREADS), 0, st, x, ssq, (const bf16_t*)g, eps,
                                   (bf16_t*)xn, d));
  return hipGetLastError();
}

hipError_t launch_rope_kv(hipStream_t st, int dtype, const float* part, int S, const RowPlan& rows,
                          const float* cos_sin, void* qbuf, void* kcache, void* vcache, int M, int Hq,
                          int Hkv, int hd, int max_seq) {
  if (bad_rows(M) || S < 1 || Hq < 1 || Hkv < 1 || (hd & 1) || !part || !cos_sin || !qbuf || !kcache || !vcache)
    return hipErrorInvalidValue;
  const dim3 grid(M, Hq + 2 * Hkv);
  SD_DISPATCH_T(dtype,
                hipLaunchKernelGGL(rope_kv_k<float>, grid, dim3(64), 0, st, part, S, rows.seq, rows.pos,
                                   cos_sin, (float*)qbuf, (float*)kcache, (float*)vcache, M, Hq, Hkv, hd,
                                   max_seq),
                hipLaunchKernelGGL(rope_kv_k<bf16_t>, grid, dim3(64), 0, st, part, S, rows.seq, rows.pos,
                                   cos_sin, (bf16_t*)qbuf, (bf16_t*)kcache, (bf16_t*)vcache, M, Hq, Hkv, hd,
                                   max_seq));
  return hipGetLastError();
}

hipError_t launch_silu_mul(hipStream_t st, int dtype, const float* part, int S, void* act, int M, int ffn) {
  if (bad_rows(M) || S < 1 || ffn < 1 || !part || !act) return hipErrorInvalidValue;
  const dim3 grid((ffn + EW_THREADS - 1) / EW_THREADS, M);
  SD_DISPATCH_T(dtype,
                hipLaunchKernelGGL(silu_mul_k<float>, grid, dim3(EW_THREADS), 0, st, part, S, (float*)act, M, ffn),
                hipLaunchKernelGGL(silu_mul_k<bf16_t>, grid, dim3(EW_THREADS), 0, st, part, S, (bf16_t*)act, M,
                                   ffn));
  return hipGetLastError();
}

hipError_t launch_reduce_rows(hipStream_t st, const float* part, int S, float* out, int RS, int64_t ld_group,
                              int64_t ld_row, int M, int N, const int32_t* dst) {
  if (bad_rows(M) || S < 1 || N < 1 || RS < 1 || M % RS != 0 || ld_row < N || !part || !out)
    return hipErrorInvalidValue;
  const dim3 grid((N + EW_THREADS - 1) / EW_THREADS, M);
  hipLaunchKernelGGL(reduce_rows_k, grid, dim3(EW_THREADS), 0, st, part, S, out, RS, ld_group, ld_row, dst, M, N);
  return hipGetLastError();
}

hipError_t launch_head_act(hipStream_t st, int dtype, const float* part, int S, const void* bias,
                           const void* z_in, const int* z_in_rows, void* z_out, int residual, int M, int n) {
  if (bad_rows(M) || S < 1 || n < 1 || !part || !bias || !z_out || (residual && !z_in)) return hipErrorInvalidValue;
  const dim3 grid((n + EW_THREADS - 1) / EW_THREADS, M);
  SD_DISPATCH_T(dtype,
                hipLaunchKernelGGL(head_act_k<float>, grid, dim3(EW_THREADS), 0, st, part, S, (const float*)bias,
                                   (const float*)z_in, z_in_rows, (float*)z_out, residual, M, n),
                hipLaunchKernelGGL(head_act_k<bf16_t>, grid, dim3(EW_THREADS), 0, st, part, S,
                                   (const bf16_t*)bias, (const bf16_t*)z_in, z_in_rows, (bf16_t*)z_out, residual,
                                   M, n));
  return hipGetLastError();
}

}  // namespace sd
