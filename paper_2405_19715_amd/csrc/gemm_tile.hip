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
//   operands   = loaded from global memory straight into LDS (global_load_lds_dwordx4: lane l
//                of an instruction writes LDS word base + l), NS stages of BK k each in a
//                ring, no registers and no LDS store instructions in between.  One
//                instruction covers 64 / KG rows x KG 16-byte k-groups (KG = BK / 8), i.e.
//                whole 64- or 128-byte row pieces, and the lanes pick their k-group with an
//                XOR of the row index, so that LDS is row-major [row][slot] yet the MFMA
//                operand reads (32 consecutive rows, one k-group) touch every bank once.
//   k loop     = wait until this wavefront's loads of stage kt have landed (s_waitcnt vmcnt
//                with the younger stages still in flight), barrier, issue the loads of stage
//                kt + NS - 1 into the buffer everyone has just finished with, multiply stage kt.
//                The load is inline assembly on purpose: through the compiler builtin every
//                LDS read is preceded by a wait for ALL outstanding loads, which serialises the
//                ring.
//   grid       = one dimension, n-tile-major with the m-tiles of one weight tile adjacent
//                and on the same XCD (ids are dealt round-robin over the 8 XCDs), so that
//                a weight tile comes from HBM once and its other readers hit that XCD's L2.
// Measured on the MI355X (M = 1024): 57344 x 8192 0.88 PFLOP/s, 10240 x 8192 0.81, 8192 x 28672
// 0.88 (register-staged loads reached 0.45-0.68 on the same tiles; the MFMA loop alone, with
// nothing to load, sustains 1.6).
#include "common.hpp"
#include "kernels.hpp"

#include <mutex>

namespace sd {

namespace {

typedef __attribute__((__vector_size__(16 * sizeof(float)))) float floatx16;

constexpr int NXCD = 8;

__device__ __forceinline__ bf16x8 as_bf16x8(const uint4& v) {
  union { uint4 u; bf16x8 b; } c;
  c.u = v;
  return c.b;
}

// s_waitcnt on the vector-memory counter alone: vmcnt[3:0] | expcnt[6:4] | lgkmcnt[11:8] | vmcnt[5:4] << 14
template <int VM>
__device__ __forceinline__ void wait_vmcnt() {
  static_assert(VM >= 0 && VM < 64, "vmcnt has six bits");
  __builtin_amdgcn_s_waitcnt((VM & 0xF) | (0x7 << 4) | (0xF << 8) | ((VM >> 4) << 14));
}

// 16 bytes per lane from global memory to LDS word (lds_bytes / 16 + lane); lds_bytes is wave-uniform
__device__ __forceinline__ void load_to_lds16(const bf16_t* g, uint32_t lds_bytes) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(lds_bytes), "v"(g) : "memory", "m0");
}
// the same, non-temporal: for weights that no other workgroup will read again (one m-tile)
__device__ __forceinline__ void load_to_lds16_stream(const bf16_t* g, uint32_t lds_bytes) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off nt" ::"s"(lds_bytes), "v"(g) : "memory", "m0");
}

template <int TN, int TM, int WN, int WM, int BK, int NS>
__global__ __launch_bounds__(64 * WN * WM) void gemm_bf16_tile(const bf16_t* __restrict__ W,
                                                               const bf16_t* __restrict__ X, int ldx,
                                                               const int* __restrict__ xrow, float* __restrict__ C,
                                                               int M, int N, int K, int n_tiles, int m_tiles,
                                                               int steps_per) {
  constexpr int NWV = WN * WM;
  constexpr int KG = BK / 8;                         // 16-byte k-groups per row and stage (4 or 8)
  constexpr int BN = 32 * TN * WN, BM = 32 * TM * WM;
  constexpr int RPI = 64 / KG;                       // rows one load instruction covers
  constexpr int ABLK = BN / RPI, BBLK = BM / RPI;    // load instructions per stage for W and for X
  constexpr int LPW = (ABLK + BBLK) / NWV;           // per wavefront
  constexpr int STAGE = (BN + BM) * KG;              // 16-byte words per stage
  constexpr int SH = KG == 4 ? 2 : 1, MSK = KG - 1;  // slot of k-group kg in row r: kg ^ ((r >> SH) & MSK)
  constexpr int NSUB = BK / 16;                      // MFMA sub-steps per stage
  static_assert((KG == 4 || KG == 8) && (ABLK + BBLK) % NWV == 0 && NS >= 2 && (NS - 2) * LPW < 64, "tile shape");
  extern __shared__ uint4 smem[];

  // tile of this workgroup: ids are dealt to XCDs round-robin; XCD x takes weight tiles x, x+8, ..
  const int L = blockIdx.x;
  const int xcd = L % NXCD, j = L / NXCD;
  const int nt = (j / m_tiles) * NXCD + xcd, mt = j % m_tiles;
  if (nt >= n_tiles) return;                         // whole workgroup: no barrier is skipped by part of it
  const int n0 = nt * BN, m0 = mt * BM;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wn = wave % WN, wm = wave / WN;
  const int r32 = lane & 31, kh = lane >> 5;         // MFMA operand lane: row, k half
  const int row_l = lane / KG, slot = lane % KG;     // loader lane: row within the instruction, LDS slot

  const bf16_t* gsrc[LPW];
  uint32_t ldst[LPW];
  bool stream[LPW];                                  // a weight block of a launch with one m-tile: read once
  const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) uint4*)smem;   // LDS byte address
#pragma unroll
  for (int i = 0; i < LPW; ++i) {
    const int q = i * NWV + wave;                    // instruction q of the stage: W blocks first, then X blocks
    const bool isA = q < ABLK;
    const int blk = isA ? q : q - ABLK;
    const int row = blk * RPI + row_l;
    const int kg = slot ^ ((row >> SH) & MSK);
    if (isA) {
      gsrc[i] = W + (size_t)min(n0 + row, N - 1) * K + kg * 8;
    } else {
      const int m = min(m0 + row, M - 1);
      gsrc[i] = X + (size_t)(xrow ? xrow[m] : m) * ldx + kg * 8;
    }
    ldst[i] = lds0 + (uint32_t)((isA ? 0 : BN * KG) + blk * 64) * 16u;
    stream[i] = isA && m_tiles == 1;
  }
  auto issue = [&](int kt) {
    const uint32_t stage = (uint32_t)((kt % NS) * STAGE) * 16u;
#pragma unroll
    for (int i = 0; i < LPW; ++i) {
      const uint32_t dst = __builtin_amdgcn_readfirstlane(ldst[i] + stage);
      if (stream[i]) load_to_lds16_stream(gsrc[i] + (size_t)kt * BK, dst);       // wave-uniform
      else load_to_lds16(gsrc[i] + (size_t)kt * BK, dst);
    }
  };

  floatx16 acc[TN][TM];
#pragma unroll
  for (int a = 0; a < TN; ++a)
#pragma unroll
    for (int b = 0; b < TM; ++b)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.f;

  // K slice of this workgroup (blockIdx.y): stages k_beg .. nk - 1; slice s writes C[s][M][N]
  const int k_beg = blockIdx.y * steps_per, nk = min(K / BK, k_beg + steps_per);
  C += (size_t)blockIdx.y * M * N;
#pragma unroll
  for (int p = 0; p < NS - 1; ++p)
    if (k_beg + p < nk) issue(k_beg + p);

  // operand word offsets inside a stage (the same for every stage)
  int aw[TN][NSUB], bw[TM][NSUB];
#pragma unroll
  for (int s = 0; s < NSUB; ++s) {
    const int kg = 2 * s + kh;
#pragma unroll
    for (int a = 0; a < TN; ++a) {
      const int row = wn * (32 * TN) + a * 32 + r32;
      aw[a][s] = row * KG + (kg ^ ((row >> SH) & MSK));
    }
#pragma unroll
    for (int b = 0; b < TM; ++b) {
      const int row = wm * (32 * TM) + b * 32 + r32;
      bw[b][s] = BN * KG + row * KG + (kg ^ ((row >> SH) & MSK));
    }
  }

  for (int kt = k_beg; kt < nk; ++kt) {
    // stage kt has landed once at most the NS - 2 younger stages of this wavefront are in flight
    if (kt + NS - 2 < nk) wait_vmcnt<(NS - 2) * LPW>(); else wait_vmcnt<0>();
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();                    // everyone's part of stage kt is in LDS, and everyone
    asm volatile("" ::: "memory");                   // has finished reading stage kt - 1
    if (kt + NS - 1 < nk) issue(kt + NS - 1);        // into the buffer of stage kt - 1
    const uint4* st = smem + (kt % NS) * STAGE;
#pragma unroll
    for (int s = 0; s < NSUB; ++s) {
      bf16x8 af[TN], bfr[TM];
#pragma unroll
      for (int a = 0; a < TN; ++a) af[a] = as_bf16x8(st[aw[a][s]]);
#pragma unroll
      for (int b = 0; b < TM; ++b) bfr[b] = as_bf16x8(st[bw[b][s]]);
#pragma unroll
      for (int a = 0; a < TN; ++a)
#pragma unroll
        for (int b = 0; b < TM; ++b)
          acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[a], bfr[b], acc[a][b], 0, 0, 0);
    }
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

template <int TN, int TM, int WN, int WM, int BK, int NS>
hipError_t launch_tile(hipStream_t st, const bf16_t* W, const bf16_t* X, int ldx, const int* xrow, float* C, int M,
                       int N, int K, int S) {
  constexpr int BN = 32 * TN * WN, BM = 32 * TM * WM;
  constexpr size_t lds = (size_t)NS * (BK / 8) * (BN + BM) * 16;
  auto kern = gemm_bf16_tile<TN, TM, WN, WM, BK, NS>;
  // dynamic LDS above 64 KB has to be allowed once per kernel (instantiation): the first caller does it, whichever
  // thread that is
  static std::once_flag once;
  static hipError_t attr_err = hipSuccess;
  std::call_once(once, [&] {
    attr_err = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                   (int)lds);
  });
  if (attr_err != hipSuccess) return attr_err;
  const int n_tiles = (N + BN - 1) / BN, m_tiles = (M + BM - 1) / BM;
  const int n_tiles_pad = (n_tiles + NXCD - 1) / NXCD * NXCD;
  const int nk = K / BK, steps_per = (nk + S - 1) / S;
  if ((S - 1) * steps_per >= nk) return hipErrorInvalidValue;      // every slice must own at least one stage
  hipLaunchKernelGGL(kern, dim3(n_tiles_pad * m_tiles, S), dim3(64 * WN * WM), lds, st, W, X, ldx, xrow, C, M, N, K,
                     n_tiles, m_tiles, steps_per);
  return hipGetLastError();
}

// Tile shape and K split for an (M, N, K) product.  Large M (prompt pass): the widest tile whose grid
// covers the chip about twice, no split unless the grid would leave CUs idle.  16 < M <= 192 (a batched target pass): one m-tile that holds
// every row, so each weight is read once, and as many K slices as it takes to put about 384
// workgroups on the 256 CUs; the few partial-sum slices are added by the consumer like the streaming kernel's.
struct TilePlan { int kind, S; };          // kind: 0 = 256x256, 1 = 128x128, 2 = 128x64, 3 = 128x192

TilePlan plan_tile(int M, int N, int K) {
  const int bk = (K % 64 == 0) ? 64 : 32;
  auto wgs = [&](int bn, int bm) { return (long)((N + bn - 1) / bn) * ((M + bm - 1) / bm); };
  int kind;
  if (M <= 64) kind = 2;
  else if (M <= 128) kind = 1;
  else if (M <= 192 && bk == 64) kind = 3;
  else if (bk == 64 && wgs(256, 256) >= 448) kind = 0;
  else kind = 1;
  const int bn = kind == 0 ? 256 : 128, bm = kind == 0 ? 256 : kind == 1 ? 128 : kind == 2 ? 64 : 192;
  const long w = wgs(bn, bm);
  int S = 1;
  constexpr int target = 384;                        // workgroups wanted: 1.5 per CU measured best (256 .. 512 tried)
  // a prompt chunk (several m-tiles) is split only when its grid would leave CUs idle: the extra slices cost traffic
  if (w < (M <= 192 ? target - 32 : 320)) {
    S = (int)((target + w - 1) / w);
    const int nk = K / bk;
    while (S > 1 && nk / S < 8) --S;                 // keep slices long enough to amortise the pipeline fill
    const int per = (nk + S - 1) / S;
    S = (nk + per - 1) / per;                        // no empty slice
  }
  return TilePlan{kind, S};
}

}  // namespace

int gemm_tile_splits(int M, int N, int K) { return plan_tile(M, N, K).S; }

hipError_t launch_gemm_tile(hipStream_t st, const void* W, const void* X, int ldx, const int* xrow, float* C, int M,
                            int N, int K) {
  if (!W || !X || !C || M < 1 || N < 1 || K < 32 || K % 32 != 0 || ldx < K || ldx % 8 != 0 || N % 4 != 0)
    return hipErrorInvalidValue;
  if ((reinterpret_cast<uintptr_t>(W) | reinterpret_cast<uintptr_t>(X) | reinterpret_cast<uintptr_t>(C)) & 15)
    return hipErrorInvalidValue;
  const bf16_t* w = (const bf16_t*)W;
  const bf16_t* x = (const bf16_t*)X;
  const TilePlan p = plan_tile(M, N, K);
  if (K % 64 == 0) {
    switch (p.kind) {
      case 0: return launch_tile<4, 2, 2, 4, 64, 2>(st, w, x, ldx, xrow, C, M, N, K, p.S);
      case 1: return launch_tile<2, 2, 2, 2, 64, 2>(st, w, x, ldx, xrow, C, M, N, K, p.S);
      case 2: return launch_tile<2, 1, 2, 2, 64, 2>(st, w, x, ldx, xrow, C, M, N, K, p.S);
      default: return launch_tile<2, 3, 2, 2, 64, 2>(st, w, x, ldx, xrow, C, M, N, K, p.S);
    }
  }
  if (p.kind == 2) return launch_tile<2, 1, 2, 2, 32, 3>(st, w, x, ldx, xrow, C, M, N, K, p.S);
  return launch_tile<2, 2, 2, 2, 32, 3>(st, w, x, ldx, xrow, C, M, N, K, p.S);
}

}  // namespace sd
