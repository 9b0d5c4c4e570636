// Large-M bf16 GEMM for the prompt pass that precedes the first round (the target and
// the draft both ingest the prefix before Algorithm 2 starts):
//     C[m, n] = sum_k X[m, k] * W[n, k]        fp32 out, bf16 in.
// With hundreds of activation rows per weight the work is a dense contraction bound by
// the matrix cores, not by the weight stream, so this kernel is the classic LDS-tiled
// design rather than the streaming one in gemm.hip:
//
//   workgroup  = WN x WM wavefronts, C tile of BN = 32 TN WN weight rows x BM = 32 TM WM
//                activation rows; each wavefront owns TN x TM accumulators of
//                v_mfma_f32_32x32x16_bf16 (weights are the A operand, X^T the B operand, so
//                a lane ends up with 4 consecutive n of one m: 16-byte stores).
//   k loop     = BK per step, two LDS buffers, one barrier per step: the global loads of
//                step i+1 are in flight while step i multiplies, and the operand words of
//                the next 16-k sub-step are read from LDS before the current MFMAs issue.
//   LDS order  = 16-byte words laid out [k-group][row], i.e. already in the order the MFMA
//                lanes read them (lane = (row % 32, k-half)), so reads and writes are
//                both lane-linear and free of bank conflicts.
//   grid       = one dimension, n-tile-major with the m-tiles of one weight tile adjacent
//                and on the same XCD (ids are dealt round-robin over the 8 XCDs), so that
//                a weight tile comes from HBM once and its other readers hit that XCD's L2.
// Measured on the MI355X (M = 1024, 57344 x 8192): the MFMA loop alone sustains about
// 1.6 PFLOP/s, with LDS reads and barriers 1.4, and with the global -> register -> LDS
// staging 0.6-0.7: the kernel is bound by the rate at which a CU's vector memory path
// returns L2 data, which is why the widest tile (least operand traffic per flop) wins
// whenever its grid still fills the chip.
#include "common.hpp"
#include "kernels.hpp"

namespace sd {

namespace {

typedef __attribute__((__vector_size__(16 * sizeof(float)))) float floatx16;

constexpr int NXCD = 8;

__device__ __forceinline__ uint4 ldg128(const bf16_t* p) { return *reinterpret_cast<const uint4*>(p); }
__device__ __forceinline__ bf16x8 as_bf16x8(const uint4& v) {
  union { uint4 u; bf16x8 b; } c;
  c.u = v;
  return c.b;
}

template <int TN, int TM, int WN, int WM, int BK>
__global__ __launch_bounds__(64 * WN * WM) void gemm_bf16_tile(const bf16_t* __restrict__ W,
                                                               const bf16_t* __restrict__ X, int ldx,
                                                               const int* __restrict__ xrow, float* __restrict__ C,
                                                               int M, int N, int K, int n_tiles, int m_tiles) {
  constexpr int NW = WN * WM, NTH = 64 * NW;
  constexpr int KG = BK / 8;                         // 16-byte k-groups per step
  constexpr int GQ = KG / 4;                         // load instructions that cover a row's k-groups
  constexpr int BN = 32 * TN * WN, BM = 32 * TM * WM;
  constexpr int LA = BN * KG / NTH, LB = BM * KG / NTH;   // 16-byte global loads per thread and step
  constexpr int NS = BK / 16;                        // MFMA sub-steps
  static_assert(KG % 4 == 0 && (BN * KG) % NTH == 0 && (BM * KG) % NTH == 0, "tile does not divide over the loaders");
  extern __shared__ uint4 smem[];
  uint4* As = smem;                                  // [2][KG * BN]
  uint4* Bs = smem + 2 * KG * BN;                    // [2][KG * BM]

  // tile of this workgroup: ids are dealt to XCDs round-robin; XCD x takes weight tiles x, x+8, ..
  const int L = blockIdx.x;
  const int xcd = L % NXCD, j = L / NXCD;
  const int nt = (j / m_tiles) * NXCD + xcd, mt = j % m_tiles;
  if (nt >= n_tiles) return;                         // whole workgroup: no barrier is skipped by part of it
  const int n0 = nt * BN, m0 = mt * BM;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wn = wave % WN, wm = wave / WN;
  const int lr = lane & 15, lo = lane >> 4;          // loader: 16 rows x 4 k-groups per instruction
  const int r32 = lane & 31, kh = lane >> 5;         // MFMA operand lane: row, k half

  const bf16_t* ga[LA];
  const bf16_t* gb[LB];
  int sa[LA], sb[LB];
#pragma unroll
  for (int i = 0; i < LA; ++i) {
    const int id = i * NW + wave, rl = (id / GQ) * 16 + lr, grp = (id % GQ) * 4 + lo;
    ga[i] = W + (size_t)min(n0 + rl, N - 1) * K + grp * 8;
    sa[i] = grp * BN + rl;
  }
#pragma unroll
  for (int i = 0; i < LB; ++i) {
    const int id = i * NW + wave, rl = (id / GQ) * 16 + lr, grp = (id % GQ) * 4 + lo;
    const int m = min(m0 + rl, M - 1);
    gb[i] = X + (size_t)(xrow ? xrow[m] : m) * ldx + grp * 8;
    sb[i] = grp * BM + rl;
  }

  floatx16 acc[TN][TM];
#pragma unroll
  for (int a = 0; a < TN; ++a)
#pragma unroll
    for (int b = 0; b < TM; ++b)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.f;

  uint4 ra[LA], rb[LB];
#pragma unroll
  for (int i = 0; i < LA; ++i) ra[i] = ldg128(ga[i]);
#pragma unroll
  for (int i = 0; i < LB; ++i) rb[i] = ldg128(gb[i]);
#pragma unroll
  for (int i = 0; i < LA; ++i) As[sa[i]] = ra[i];
#pragma unroll
  for (int i = 0; i < LB; ++i) Bs[sb[i]] = rb[i];
  __syncthreads();

  const int nk = K / BK;
  const int aoff = wn * (32 * TN) + r32, boff = wm * (32 * TM) + r32;
  for (int kt = 0; kt < nk; ++kt) {
    const int cur = kt & 1;
    if (kt + 1 < nk) {
#pragma unroll
      for (int i = 0; i < LA; ++i) ra[i] = ldg128(ga[i] + (size_t)(kt + 1) * BK);
#pragma unroll
      for (int i = 0; i < LB; ++i) rb[i] = ldg128(gb[i] + (size_t)(kt + 1) * BK);
    }
    const uint4* Ac = As + cur * KG * BN + aoff;
    const uint4* Bc = Bs + cur * KG * BM + boff;
    uint4 af[2][TN], bfr[2][TM];
#pragma unroll
    for (int a = 0; a < TN; ++a) af[0][a] = Ac[kh * BN + a * 32];
#pragma unroll
    for (int b = 0; b < TM; ++b) bfr[0][b] = Bc[kh * BM + b * 32];
#pragma unroll
    for (int s = 0; s < NS; ++s) {
      if (s + 1 < NS) {
        const int kg = (s + 1) * 2 + kh;
#pragma unroll
        for (int a = 0; a < TN; ++a) af[(s + 1) & 1][a] = Ac[kg * BN + a * 32];
#pragma unroll
        for (int b = 0; b < TM; ++b) bfr[(s + 1) & 1][b] = Bc[kg * BM + b * 32];
      }
#pragma unroll
      for (int a = 0; a < TN; ++a)
#pragma unroll
        for (int b = 0; b < TM; ++b)
          acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(af[s & 1][a]), as_bf16x8(bfr[s & 1][b]),
                                                              acc[a][b], 0, 0, 0);
    }
    if (kt + 1 < nk) {
      uint4* An = As + (cur ^ 1) * KG * BN;
      uint4* Bn = Bs + (cur ^ 1) * KG * BM;
#pragma unroll
      for (int i = 0; i < LA; ++i) An[sa[i]] = ra[i];
#pragma unroll
      for (int i = 0; i < LB; ++i) Bn[sb[i]] = rb[i];
    }
    __syncthreads();
  }

  // D[i, j] of a 32x32 tile: lane (j = lane % 32, half = lane / 32), register v holds
  // i = 8 (v / 4) + 4 half + v % 4.  i runs over weight rows n, j over activation rows m.
#pragma unroll
  for (int b = 0; b < TM; ++b) {
    const int m = m0 + wm * (32 * TM) + b * 32 + r32;
    if (m >= M) continue;
#pragma unroll
    for (int a = 0; a < TN; ++a) {
      const int nb = n0 + wn * (32 * TN) + a * 32 + 4 * kh;
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int n = nb + 8 * q;
        if (n + 3 < N)                               // N % 4 == 0: a group of 4 is all in or all out
          *reinterpret_cast<floatx4*>(C + (size_t)m * N + n) =
              floatx4{acc[a][b][4 * q], acc[a][b][4 * q + 1], acc[a][b][4 * q + 2], acc[a][b][4 * q + 3]};
      }
    }
  }
}

template <int TN, int TM, int WN, int WM, int BK>
hipError_t launch_tile(hipStream_t st, const bf16_t* W, const bf16_t* X, int ldx, const int* xrow, float* C, int M,
                       int N, int K) {
  constexpr int BN = 32 * TN * WN, BM = 32 * TM * WM;
  constexpr size_t lds = (size_t)2 * (BK / 8) * (BN + BM) * 16;
  auto kern = gemm_bf16_tile<TN, TM, WN, WM, BK>;
  static bool attr_set = false;          // dynamic LDS above 64 KB has to be allowed once per kernel
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  const int n_tiles = (N + BN - 1) / BN, m_tiles = (M + BM - 1) / BM;
  const int n_tiles_pad = (n_tiles + NXCD - 1) / NXCD * NXCD;
  hipLaunchKernelGGL(kern, dim3(n_tiles_pad * m_tiles), dim3(64 * WN * WM), lds, st, W, X, ldx, xrow, C, M, N, K,
                     n_tiles, m_tiles);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_gemm_tile(hipStream_t st, const void* W, const void* X, int ldx, const int* xrow, float* C, int M,
                            int N, int K) {
  if (!W || !X || !C || M < 1 || N < 1 || K < 32 || ldx < K || ldx % 8 != 0 || N % 4 != 0)
    return hipErrorInvalidValue;
  if ((reinterpret_cast<uintptr_t>(W) | reinterpret_cast<uintptr_t>(X) | reinterpret_cast<uintptr_t>(C)) & 15)
    return hipErrorInvalidValue;
  const bf16_t* w = (const bf16_t*)W;
  const bf16_t* x = (const bf16_t*)X;
  if (K % 32 != 0) return hipErrorInvalidValue;
  auto wgs = [&](int bn, int bm) { return (long)((N + bn - 1) / bn) * ((M + bm - 1) / bm); };
  // widest tile whose grid still covers the 256 CUs about twice over
  if (K % 64 == 0 && wgs(256, 256) >= 448) return launch_tile<4, 2, 2, 4, 64>(st, w, x, ldx, xrow, C, M, N, K);
  if (wgs(256, 128) >= 448) return launch_tile<4, 2, 2, 2, 32>(st, w, x, ldx, xrow, C, M, N, K);
  if (wgs(128, 128) >= 256) return launch_tile<2, 2, 2, 2, 32>(st, w, x, ldx, xrow, C, M, N, K);
  return launch_tile<2, 1, 2, 2, 32>(st, w, x, ldx, xrow, C, M, N, K);
}

}  // namespace sd
