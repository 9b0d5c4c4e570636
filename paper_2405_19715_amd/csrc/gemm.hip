// Weight-streaming skinny GEMM: part[s, m, n] = sum_{k in slice s} X[m, k] * W[n, k].
//
// This is the kernel the verify pass (M = K+1 rows, Algorithm 2's parallel target
// forward) and the draft steps (M = 1 or 2 rows) spend their time in: every weight
// is read from HBM exactly once per call and used for M multiply-adds, so the
// kernel is bound by HBM bandwidth, and its whole design is about keeping many
// 16-byte weight loads in flight per wavefront.
//
// bf16 layout of the work
//   workgroup  = 4 wavefronts = 64 consecutive weight rows x one K-slice
//   wavefront  = 16 weight rows; lane (r = lane % 16, g = lane / 16) loads, per step of
//                128 k, the 64 contiguous bytes W[row0 + r, k0 + 32 g .. k0 + 32 g + 32),
//                so the wave reads 16 rows x 256 B per step and walks each row
//                sequentially.
//   X slice    = staged once per workgroup into LDS, already in the order the
//                multiply needs, then read with conflict-free 16-byte LDS loads.
//   M >= 5     : v_mfma_f32_16x16x32_bf16, weights as the A operand (16 rows x 32 k),
//                X^T as the B operand (32 k x 16 activation rows), one MFMA per 16-row
//                tile of X.  The k index inside an MFMA is a permutation of the real
//                k (lane group g holds k0 + 32 g + 8 j .. + 8 for MFMA j); A and B use
//                the same permutation, and a dot product does not care.
//   M <= 4     : no MFMA; per-lane fp32 dot products over the same loads, then a
//                reduction over the 4 lane groups with two wavefront shuffles.
// fp32 weights (tiny configuration) take a plain wave-per-output-row kernel.
#include "common.hpp"
#include "kernels.hpp"

#include <cstdlib>

namespace sd {

namespace {

constexpr int GEMM_THREADS = 256;
constexpr int ROWS_PER_WG = 64;
constexpr int KSTEP = 128;
constexpr int LDS_BUDGET = 64 * 1024;
constexpr int PREFETCH = 4;              // steps of weight loads in flight per wave

struct Split { int S, steps_per; };

Split plan_bf16(int M, int N, int K) {
  const int total = K / KSTEP;
  int max_steps = LDS_BUDGET / (M * KSTEP * 2);
  if (max_steps < 1) max_steps = 1;
  if (max_steps > total) max_steps = total;
  int S = (total + max_steps - 1) / max_steps;
  const int wgs_n = (N + ROWS_PER_WG - 1) / ROWS_PER_WG;
  // more slices until the grid can fill 256 CUs four deep, but keep slices >= 4 steps
  while (wgs_n * S < 1024 && (total + S) / (S + 1) >= 4) ++S;
  const int steps_per = (total + S - 1) / S;
  S = (total + steps_per - 1) / steps_per;
  return {S, steps_per};
}

__device__ __forceinline__ uint4 ldg128(const bf16_t* p) { return *reinterpret_cast<const uint4*>(p); }

__device__ __forceinline__ bf16x8 as_bf16x8(const uint4& v) {
  union { uint4 u; bf16x8 b; } c;
  c.u = v;
  return c.b;
}

// fp32 dot of 8 bf16 pairs packed in two uint4
__device__ __forceinline__ float dot8(const uint4& a, const uint4& b, float acc) {
  const uint32_t* pa = reinterpret_cast<const uint32_t*>(&a);
  const uint32_t* pb = reinterpret_cast<const uint32_t*>(&b);
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    acc = fmaf(__uint_as_float(pa[i] << 16), __uint_as_float(pb[i] << 16), acc);
    acc = fmaf(__uint_as_float(pa[i] & 0xffff0000u), __uint_as_float(pb[i] & 0xffff0000u), acc);
  }
  return acc;
}

// Stage X[0..M, kbeg .. kbeg + 128*steps) into LDS as 16-byte groups.
//   MFMA order (mfma = true): group (m, step s, lane group g, j) lands at
//     tile_base(m / 16) + (((s*4 + j)*4 + g) * rows_in_tile + m % 16)
//   so that lane (r, g) of MFMA j reads one 16-byte word at a lane-linear address.
//   Row-major order (mfma = false): [m][k].
template <bool MFMA_ORDER>
__device__ __forceinline__ void stage_x(uint4* lds, const bf16_t* X, int ldx, const int* xrow, int M, int kbeg,
                                        int steps) {
  const int groups_per_row = steps * 16;             // 16-byte groups per activation row
  const int last_tile = (M - 1) >> 4;
  const int rows_last = M - (last_tile << 4);
  for (int idx = threadIdx.x; idx < M * groups_per_row; idx += GEMM_THREADS) {
    const int m = idx / groups_per_row, o = idx - m * groups_per_row;
    const int src_row = xrow ? xrow[m] : m;
    const uint4 v = ldg128(X + (size_t)src_row * ldx + kbeg + o * 8);
    if (MFMA_ORDER) {
      const int s = o >> 4, g = (o >> 2) & 3, j = o & 3;
      const int tile = m >> 4, r = m & 15;
      const int rows_in_tile = (tile == last_tile) ? rows_last : 16;
      lds[tile * groups_per_row * 16 + (((s * 4 + j) * 4 + g) * rows_in_tile + r)] = v;
    } else {
      lds[idx] = v;
    }
  }
}

// ----------------------------------------------------------------------------- MFMA path
template <int NT>   // NT = number of 16-row activation tiles, M in (16(NT-1), 16 NT]
__global__ __launch_bounds__(GEMM_THREADS) void gemm_bf16_mfma(const bf16_t* __restrict__ W,
                                                               const bf16_t* __restrict__ X, int ldx,
                                                               const int* __restrict__ xrow,
                                                               float* __restrict__ part, int M, int N, int K,
                                                               int steps_per) {
  extern __shared__ uint4 lds[];
  const int total_steps = K / KSTEP;
  const int sbeg = blockIdx.y * steps_per;
  const int steps = min(steps_per, total_steps - sbeg);
  const int kbeg = sbeg * KSTEP;
  stage_x<true>(lds, X, ldx, xrow, M, kbeg, steps);
  __syncthreads();

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int r = lane & 15, g = lane >> 4;
  const int row0 = blockIdx.x * ROWS_PER_WG + wave * 16;
  if (row0 >= N) return;                              // N is a multiple of 16: whole tile in or out
  const bf16_t* wp = W + (size_t)(row0 + r) * K + kbeg + g * 32;
  const int groups_per_row = steps * 16;
  const int rows_last = M - ((NT - 1) << 4);

  floatx4 acc[NT];
#pragma unroll
  for (int t = 0; t < NT; ++t) acc[t] = floatx4{0.f, 0.f, 0.f, 0.f};

  uint4 a[PREFETCH][4];
#pragma unroll
  for (int p = 0; p < PREFETCH; ++p)
    if (p < steps) {
#pragma unroll
      for (int j = 0; j < 4; ++j) a[p][j] = ldg128(wp + p * KSTEP + j * 8);
    }

  for (int s0 = 0; s0 < steps; s0 += PREFETCH) {
#pragma unroll
    for (int p = 0; p < PREFETCH; ++p) {
      const int s = s0 + p;
      if (s < steps) {
        uint4 cur[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) cur[j] = a[p][j];
        if (s + PREFETCH < steps) {
#pragma unroll
          for (int j = 0; j < 4; ++j) a[p][j] = ldg128(wp + (s + PREFETCH) * KSTEP + j * 8);
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const bf16x8 av = as_bf16x8(cur[j]);
#pragma unroll
          for (int t = 0; t < NT; ++t) {
            uint4 bv;
            if (t < NT - 1) {
              bv = lds[t * groups_per_row * 16 + (((s * 4 + j) * 4 + g) * 16 + r)];
            } else {
              bv = (r < rows_last)
                       ? lds[t * groups_per_row * 16 + (((s * 4 + j) * 4 + g) * rows_last + r)]
                       : uint4{0u, 0u, 0u, 0u};
            }
            acc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av, as_bf16x8(bv), acc[t], 0, 0, 0);
          }
        }
      }
    }
  }

  // D[i, n]: lane (n = lane % 16, i = 4 * (lane / 16) + 0..3): four consecutive weight
  // rows for activation row n -> one 16-byte store.
  float* pout = part + (size_t)blockIdx.y * M * N;
#pragma unroll
  for (int t = 0; t < NT; ++t) {
    const int m = t * 16 + r;
    if (m < M) *reinterpret_cast<floatx4*>(pout + (size_t)m * N + row0 + 4 * g) = acc[t];
  }
}

// ----------------------------------------------------------------------------- dot-product path
template <int MV>   // MV = activation rows, 1..4
__global__ __launch_bounds__(GEMM_THREADS) void gemm_bf16_dot(const bf16_t* __restrict__ W,
                                                              const bf16_t* __restrict__ X, int ldx,
                                                              const int* __restrict__ xrow,
                                                              float* __restrict__ part, int N, int K,
                                                              int steps_per) {
  extern __shared__ uint4 lds[];
  const int total_steps = K / KSTEP;
  const int sbeg = blockIdx.y * steps_per;
  const int steps = min(steps_per, total_steps - sbeg);
  const int kbeg = sbeg * KSTEP;
  stage_x<false>(lds, X, ldx, xrow, MV, kbeg, steps);
  __syncthreads();

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int r = lane & 15, g = lane >> 4;
  const int row0 = blockIdx.x * ROWS_PER_WG + wave * 16;
  if (row0 >= N) return;
  const bf16_t* wp = W + (size_t)(row0 + r) * K + kbeg + g * 32;
  const int groups_per_row = steps * 16;

  float acc[MV];
#pragma unroll
  for (int m = 0; m < MV; ++m) acc[m] = 0.f;

  uint4 a[PREFETCH][4];
#pragma unroll
  for (int p = 0; p < PREFETCH; ++p)
    if (p < steps) {
#pragma unroll
      for (int j = 0; j < 4; ++j) a[p][j] = ldg128(wp + p * KSTEP + j * 8);
    }

  for (int s0 = 0; s0 < steps; s0 += PREFETCH) {
#pragma unroll
    for (int p = 0; p < PREFETCH; ++p) {
      const int s = s0 + p;
      if (s < steps) {
        uint4 cur[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) cur[j] = a[p][j];
        if (s + PREFETCH < steps) {
#pragma unroll
          for (int j = 0; j < 4; ++j) a[p][j] = ldg128(wp + (s + PREFETCH) * KSTEP + j * 8);
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
#pragma unroll
          for (int m = 0; m < MV; ++m) {
            const uint4 xv = lds[m * groups_per_row + s * 16 + g * 4 + j];   // same for the 16 lanes of a group
            acc[m] = dot8(cur[j], xv, acc[m]);
          }
        }
      }
    }
  }
  float* pout = part + (size_t)blockIdx.y * MV * N;
#pragma unroll
  for (int m = 0; m < MV; ++m) {
    float v = acc[m];
    v += __shfl_xor(v, 16, WAVE);
    v += __shfl_xor(v, 32, WAVE);
    if (g == 0) pout[(size_t)m * N + row0 + r] = v;
  }
}

// ----------------------------------------------------------------------------- fp32 path
// One wavefront per output column n; lanes stride over k; up to 8 activation rows at
// a time.  Sizes here are tiny (d = 256), so nothing is tuned.
__global__ __launch_bounds__(256) void gemm_f32(const float* __restrict__ W, const float* __restrict__ X,
                                                int ldx, const int* __restrict__ xrow,
                                                float* __restrict__ part, int M, int N, int K) {
  const int lane = threadIdx.x & 63;
  const int n = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (n >= N) return;
  const float* w = W + (size_t)n * K;
  for (int m0 = 0; m0 < M; m0 += 8) {
    float acc[8];
    const float* xr[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      acc[i] = 0.f;
      const int m = min(m0 + i, M - 1);
      xr[i] = X + (size_t)(xrow ? xrow[m] : m) * ldx;
    }
    for (int k = lane; k < K; k += 64) {
      const float wv = w[k];
#pragma unroll
      for (int i = 0; i < 8; ++i) acc[i] = fmaf(wv, xr[i][k], acc[i]);
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const float v = wave_sum(acc[i]);
      if (lane == 0 && m0 + i < M) part[(size_t)(m0 + i) * N + n] = v;
    }
  }
}

template <int NT>
hipError_t launch_mfma(hipStream_t st, const bf16_t* W, const bf16_t* X, int ldx, const int* xrow, float* part,
                       int M, int N, int K, Split sp) {
  const dim3 grid((N + ROWS_PER_WG - 1) / ROWS_PER_WG, sp.S);
  const size_t lds = (size_t)M * sp.steps_per * KSTEP * 2;
  hipLaunchKernelGGL(gemm_bf16_mfma<NT>, grid, dim3(GEMM_THREADS), lds, st, W, X, ldx, xrow, part, M, N, K,
                     sp.steps_per);
  return hipGetLastError();
}

template <int MV>
hipError_t launch_dot(hipStream_t st, const bf16_t* W, const bf16_t* X, int ldx, const int* xrow, float* part,
                      int N, int K, Split sp) {
  const dim3 grid((N + ROWS_PER_WG - 1) / ROWS_PER_WG, sp.S);
  const size_t lds = (size_t)MV * sp.steps_per * KSTEP * 2;
  hipLaunchKernelGGL(gemm_bf16_dot<MV>, grid, dim3(GEMM_THREADS), lds, st, W, X, ldx, xrow, part, N, K,
                     sp.steps_per);
  return hipGetLastError();
}

}  // namespace

int gemm_splits(int dtype, int M, int N, int K) {
  if (dtype == DT_F32) return 1;
  return plan_bf16(M, N, K).S;
}

hipError_t launch_gemm(hipStream_t st, int dtype, const void* W, const void* X, int ldx, const int* xrow,
                       float* part, int M, int N, int K) {
  if (!W || !X || !part || M < 1 || M > MAX_ROWS || N < 1 || K < 1 || ldx < K) return hipErrorInvalidValue;
  if (dtype == DT_F32) {
    hipLaunchKernelGGL(gemm_f32, dim3((N + 3) / 4), dim3(256), 0, st, (const float*)W, (const float*)X, ldx,
                       xrow, part, M, N, K);
    return hipGetLastError();
  }
  if (dtype != DT_BF16) return hipErrorInvalidValue;
  // 16-byte loads along K, 16-row tiles along N, 16-byte aligned rows
  if (K % KSTEP != 0 || N % 16 != 0 || ldx % 8 != 0) return hipErrorInvalidValue;
  if ((reinterpret_cast<uintptr_t>(W) | reinterpret_cast<uintptr_t>(X) | reinterpret_cast<uintptr_t>(part)) & 15)
    return hipErrorInvalidValue;
  const Split sp = plan_bf16(M, N, K);
  const bf16_t* w = (const bf16_t*)W;
  const bf16_t* x = (const bf16_t*)X;
  if (M <= 4) {
    switch (M) {
      case 1: return launch_dot<1>(st, w, x, ldx, xrow, part, N, K, sp);
      case 2: return launch_dot<2>(st, w, x, ldx, xrow, part, N, K, sp);
      case 3: return launch_dot<3>(st, w, x, ldx, xrow, part, N, K, sp);
      default: return launch_dot<4>(st, w, x, ldx, xrow, part, N, K, sp);
    }
  }
  const int nt = (M + 15) / 16;
  switch (nt) {
    case 1: return launch_mfma<1>(st, w, x, ldx, xrow, part, M, N, K, sp);
    case 2: return launch_mfma<2>(st, w, x, ldx, xrow, part, M, N, K, sp);
    case 3: return launch_mfma<3>(st, w, x, ldx, xrow, part, M, N, K, sp);
    case 4: return launch_mfma<4>(st, w, x, ldx, xrow, part, M, N, K, sp);
    case 5: return launch_mfma<5>(st, w, x, ldx, xrow, part, M, N, K, sp);
    case 6: return launch_mfma<6>(st, w, x, ldx, xrow, part, M, N, K, sp);
    case 7: return launch_mfma<7>(st, w, x, ldx, xrow, part, M, N, K, sp);
    case 8: return launch_mfma<8>(st, w, x, ldx, xrow, part, M, N, K, sp);
    case 9: return launch_mfma<9>(st, w, x, ldx, xrow, part, M, N, K, sp);
    case 10: return launch_mfma<10>(st, w, x, ldx, xrow, part, M, N, K, sp);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace sd
