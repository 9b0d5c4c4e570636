// Row-stripe GEMM for 9 .. 17 activation rows: the verify pass of a round that drafted 8 .. 16 candidates
// (Algorithm 2's parallel target forward over K + 1 positions).
//
// Same organisation as the vector-ALU row-stripe kernel (gemm.hip): a wavefront owns one K piece of a contiguous
// range of weight rows, every load instruction covers 1 KB of ONE row (the access pattern that reads HBM fastest),
// its piece of X lives in registers for the whole pass, the K pieces of a row range all belong to one workgroup,
// which adds them at the end, so there is ONE slice of finished sums and the final sweep does the elementwise work
// of the decoder layer (SiLU * up, residual + norm, rotary embedding + KV append: stripe_epilogue.hpp).  What
// differs is the multiply: 16 * M dot products per 16 bytes of weights do not fit the vector ALU beyond 8 rows
// (it is 54 % busy there), so the products run on the matrix cores, v_mfma_f32_16x16x32_bf16 with the weights
// as the A operand (16 rows x 32 k) and X^T as the B operand.
//
// The matrix core wants lane (i, g) to hold 16 bytes of weight row i, a row-contiguous load gives lane l 16 bytes
// of ONE row: the tile is transposed through a per-wavefront LDS buffer.  A wavefront takes 8 weight rows at a
// time (rows 8 .. 15 of the A operand read a row of zeros: the matrix cores have time to spare, LDS space is what
// is short): row r of the 8 goes to LDS as it arrives, 16-byte block b of the row at slot b ^ r of the row's 1 KB,
// and lane (i, g) reads block t + 16 g of row i for MFMA t: both the 64-lane write and the read hit 16 distinct
// 16-byte bank groups per 16 lanes.  The 16 row registers of a wavefront are a ring over two such half tiles, each
// reloaded as soon as it has been written to LDS, so 16 KB per wavefront are in flight all the time, as in the
// vector-ALU kernel.  LDS operations of one wavefront execute in order, so the next half tile's writes cannot
// overtake this one's reads.
//
// X: the B operand of MFMA t is X[m = lane % 16][k0 + 8 (t + 16 g) ..], 16 registers of 16 bytes for the first 16
// activation rows.  A 17th row (K = 16 candidates) would need 16 more for one live lane in 16; its operands are
// packed four to a register (lanes 0, 4, 8, 12 of each 16 hold the operands of four consecutive MFMAs) and moved
// into lane 0 by a DPP row shift when used.
#include "common.hpp"
#include "kernels.hpp"
#include "stripe_epilogue.hpp"

#include <mutex>

namespace sd {

namespace {

constexpr int MS_WAVES = 8;
constexpr int MS_THREADS = 64 * MS_WAVES;
constexpr int MS_PIECE = 512;                      // k per piece: 1 KB of a weight row
constexpr int MS_HALF = 8;                         // weight rows per transposed half tile
constexpr int MS_BUF_BYTES = (MS_HALF + 1) * 1024; // 8 rows + a row of zeros per wavefront
constexpr int MS_MAX_M = 17;
constexpr size_t MS_LDS_MAX = 158 * 1024;

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 ms_bf16x8;

__device__ __forceinline__ ms_bf16x8 ms_as_bf16x8(const uint4& v) {
  union { uint4 u; ms_bf16x8 b; } c;
  c.u = v;
  return c.b;
}

__device__ __forceinline__ uint4 ms_ld_stream(const bf16_t* p) {      // read once: non-temporal
  const uint32_t* q = reinterpret_cast<const uint32_t*>(p);
  uint4 v;
  v.x = __builtin_nontemporal_load(q);
  v.y = __builtin_nontemporal_load(q + 1);
  v.z = __builtin_nontemporal_load(q + 2);
  v.w = __builtin_nontemporal_load(q + 3);
  return v;
}

// lanes 0 .. 3 of every 16 take `src` from the lane SHL further up (lane 0 <- lane SHL), all other lanes 0
template <int SHL>
__device__ __forceinline__ uint32_t ms_take_lane(uint32_t src) {
  constexpr int CTRL = SHL == 0 ? 0xE4 : 0x100 + SHL;        // quad_perm identity, or row_shl:SHL
  return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)src, CTRL, 0xF, 0x1, false);
}
template <int SHL>
__device__ __forceinline__ uint4 ms_take_lane4(const uint4& v) {
  return uint4{ms_take_lane<SHL>(v.x), ms_take_lane<SHL>(v.y), ms_take_lane<SHL>(v.z), ms_take_lane<SHL>(v.w)};
}
// operand of MFMA t from the packed 17th-row registers (t = 4 q + jj sits in lanes 4 jj of register q)
template <int T>
__device__ __forceinline__ uint4 ms_row16_operand(const uint4 (&xp)[4]) {
  return ms_take_lane4<4 * (T & 3)>(xp[T >> 2]);
}

// MT = 1: up to 16 activation rows; MT = 2: 17.
template <int MT, int EPI>
__global__ __launch_bounds__(MS_THREADS) void gemm_bf16_mstripe(const bf16_t* __restrict__ W,
                                                                const bf16_t* __restrict__ X, int ldx,
                                                                const int* __restrict__ xrow,
                                                                float* __restrict__ part, StripeEpi epi, int M, int N,
                                                                int K, int cs, int rpg, int ranges, int rpw,
                                                                int npass) {
  constexpr bool SILU = EPI == EPI_SILU;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int li = lane & 15, g = lane >> 4;
  const int lr = wave / cs, ls = wave - lr * cs;     // local row range, local K slot
  const int rg = SILU ? blockIdx.x * (rpg >> 1) + (lr >> 1) : blockIdx.x * rpg + lr;
  // SILU: gate and up are a multiple of 2^26 bytes apart for the 70B shape (the same DRAM channel and bank at equal
  // k), and a pair's wavefronts run side by side: the up wavefronts take their pieces one slot further
  const int c0 = SILU && (lr & 1) ? (ls + 1 == cs ? 0 : ls + 1) : ls;
  const int r0 = rg * rpw + (SILU && (lr & 1) ? N : 0);          // SILU: odd local ranges are the rows of `up`
  const int rows = rg < ranges ? min(rpw, N - rg * rpw) : 0;     // a wavefront without rows still meets the barrier
  const int nh = (rows + MS_HALF - 1) / MS_HALF;                 // half tiles of this wavefront's range
  const bf16_t* const idle = W + lane * 8;                       // a line every wavefront shares; its data is unused

  __shared__ float s_scale[MS_MAX_M];
  float sq[3][STRIPE_SSQ_PER_LANE];                              // 3 * 8 wavefronts >= 17 rows
  if constexpr (EPI != EPI_RESID) stripe_load_ssq<3>(epi, M, sq);

  extern __shared__ __attribute__((aligned(16))) unsigned char ms_lds[];
  // [wavefront][9 KB] transposition buffers, then the wavefronts' output tiles [M][rpw]
  unsigned char* const buf = ms_lds + (size_t)wave * MS_BUF_BYTES;
  float* const obuf = reinterpret_cast<float*>(ms_lds + (size_t)MS_WAVES * MS_BUF_BYTES);
  float* const otile = obuf + (size_t)wave * M * rpw;
  // the row of zeros that lanes 8 .. 15 of every 16 read as their A operand
  *reinterpret_cast<uint4*>(buf + MS_HALF * 1024 + lane * 16) = uint4{0u, 0u, 0u, 0u};
  // this lane's write slot for row r of a half tile is (lane ^ r); its read for MFMA t is block (t + 16 g) of row
  // li (or of the zero row), at slot block ^ li
  const unsigned char* const rd_row = buf + (li < MS_HALF ? li : MS_HALF) * 1024;

  for (int ps = 0; ps < npass; ++ps) {
    const int c = ps * cs + c0;                        // this pass's piece of K
    const int roth = nh > 0 ? ((rg * npass * cs + c) * 5) % nh : 0;      // the wavefronts start at different rows
    // row r of half tile h -> address of this lane's 16 bytes (or the idle line past the range)
    auto at = [&](int h, int r) -> const bf16_t* {
      int hh = h + roth;
      if (hh >= nh) hh -= nh;
      const int j = hh * MS_HALF + r;
      if (h >= nh || j >= rows) return idle;
      int row = r0 + j;
      if constexpr (EPI == EPI_ROPE) {                 // local index -> row of W: (head, i, half) order
        const int hs = epi.hshift;
        const int p = row >> 1;
        row = ((p >> hs) << (hs + 1)) + (p & ((1 << hs) - 1)) + ((row & 1) << hs);
      }
      return W + (size_t)row * K + c * MS_PIECE + lane * 8;
    };

    // X first: its loads are then older than every weight load
    uint4 xb[16];
    uint4 xp[4];
    {
      const int m = min(li, M - 1);
      const bf16_t* xr = X + (size_t)(xrow ? xrow[m] : m) * ldx + c * MS_PIECE + g * 128;
#pragma unroll
      for (int t = 0; t < 16; ++t) xb[t] = *reinterpret_cast<const uint4*>(xr + t * 8);
      if constexpr (MT == 2) {
        const bf16_t* x16 = X + (size_t)(xrow ? xrow[16] : 16) * ldx + c * MS_PIECE + g * 128 + (li >> 2) * 8;
#pragma unroll
        for (int q = 0; q < 4; ++q) xp[q] = *reinterpret_cast<const uint4*>(x16 + q * 32);
      }
    }
    uint4 a[2 * MS_HALF];
#pragma unroll
    for (int i = 0; i < 2 * MS_HALF; ++i) a[i] = ms_ld_stream(at(i / MS_HALF, i % MS_HALF));
    __builtin_amdgcn_sched_barrier(0);
    if (li >= M) {                                     // fewer than 16 rows: the missing ones multiply zeros
#pragma unroll
      for (int t = 0; t < 16; ++t) xb[t] = uint4{0u, 0u, 0u, 0u};
    }
    if constexpr (MT == 2) {
      if (li & 3) {                                    // only lanes 0, 4, 8, 12 of every 16 carry 17th-row operands
#pragma unroll
        for (int q = 0; q < 4; ++q) xp[q] = uint4{0u, 0u, 0u, 0u};
      }
    }

    for (int h0 = 0; h0 < nh; h0 += 2) {
#pragma unroll
      for (int p = 0; p < 2; ++p) {
        const int h = h0 + p;
        __builtin_amdgcn_sched_barrier(0);             // half tiles stay in order: the next one's data is still in flight
#pragma unroll
        for (int r = 0; r < MS_HALF; ++r) {
          *reinterpret_cast<uint4*>(buf + r * 1024 + ((lane ^ r) << 4)) = a[p * MS_HALF + r];
          a[p * MS_HALF + r] = ms_ld_stream(at(h + 2, r));
        }
        floatx4 acc0 = floatx4{0.f, 0.f, 0.f, 0.f}, acc1 = floatx4{0.f, 0.f, 0.f, 0.f};
#define SD_MS_STEP(T)                                                                                              \
        {                                                                                                          \
          const uint4 f = *reinterpret_cast<const uint4*>(rd_row + ((((T) + 16 * g) ^ li) << 4));                  \
          acc0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ms_as_bf16x8(f), ms_as_bf16x8(xb[T]), acc0, 0, 0, 0);     \
          if constexpr (MT == 2)                                                                                   \
            acc1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ms_as_bf16x8(f), ms_as_bf16x8(ms_row16_operand<T>(xp)), \
                                                           acc1, 0, 0, 0);                                         \
        }
        SD_MS_STEP(0) SD_MS_STEP(1) SD_MS_STEP(2) SD_MS_STEP(3) SD_MS_STEP(4) SD_MS_STEP(5) SD_MS_STEP(6) SD_MS_STEP(7)
        SD_MS_STEP(8) SD_MS_STEP(9) SD_MS_STEP(10) SD_MS_STEP(11) SD_MS_STEP(12) SD_MS_STEP(13) SD_MS_STEP(14)
        SD_MS_STEP(15)
#undef SD_MS_STEP
        // D[i][m]: lane (m = li, g) holds weight rows 4 g .. 4 g + 3 of the half tile (g < 2) for activation row m
        if (h < nh && g < 2) {
          int hh = h + roth;
          if (hh >= nh) hh -= nh;
          const int r = hh * MS_HALF + 4 * g;          // rpw is a multiple of 8: the four rows stay inside the tile
          if (li < M) {
            floatx4* dst = reinterpret_cast<floatx4*>(otile + li * rpw + r);
            *dst = ps == 0 ? acc0 : *dst + acc0;       // later pieces of the same wavefront, in piece order
          }
          if constexpr (MT == 2) {
            if (li == 0) {
              floatx4* dst = reinterpret_cast<floatx4*>(otile + 16 * rpw + r);
              *dst = ps == 0 ? acc1 : *dst + acc1;
            }
          }
        }
      }
    }
  }
  stripe_finish<EPI, 3>(obuf, s_scale, sq, part, epi, M, N, cs, rpg, ranges, rpw);
}

struct MsPlan { int ok, cs, rpg, G, ranges, rpw, npass; size_t lds; };

// cs K slots x rpg row ranges = 8 wavefronts; a wavefront takes npass pieces one after the other.  One workgroup
// per CU (the LDS says so), so the ranges are sized for 256 workgroups.
MsPlan plan_mstripe(int M, int N, int K, bool paired, bool even_rows) {
  MsPlan bad{0, 0, 0, 0, 0, 0, 0, 0};
  if (M < 9 || M > MS_MAX_M || N < 1 || K < MS_PIECE || K % MS_PIECE != 0) return bad;
  if (even_rows && (N & 1)) return bad;
  const int pieces = K / MS_PIECE;
  MsPlan best = bad;
  for (int cs = MS_WAVES; cs >= 1; cs >>= 1) {
    if (pieces % cs) continue;
    const int rpg = MS_WAVES / cs;
    if (paired && (rpg & 1)) continue;
    const int npass = pieces / cs;
    if (npass > 16) continue;
    const int units = paired ? rpg / 2 : rpg;
    int ranges = 256 * units;
    int rpw = (N + ranges - 1) / ranges;
    rpw = (rpw + MS_HALF - 1) / MS_HALF * MS_HALF;                 // whole half tiles (and an even number of rows)
    ranges = (N + rpw - 1) / rpw;
    const int G = (ranges + units - 1) / units;
    const size_t lds = (size_t)MS_WAVES * MS_BUF_BYTES + (size_t)MS_WAVES * M * rpw * sizeof(float);
    if (lds > MS_LDS_MAX) continue;
    best = MsPlan{1, cs, rpg, G, ranges, rpw, npass, lds};
    break;                                                          // the most K slots that fit: fewest passes
  }
  return best;
}

template <int MT, int EPI>
hipError_t launch_ms(hipStream_t st, const bf16_t* W, const bf16_t* X, int ldx, const int* xrow, float* part,
                     const StripeEpi& epi, int M, int N, int K, const MsPlan& sp) {
  auto kern = gemm_bf16_mstripe<MT, EPI>;
  static std::once_flag once;                        // dynamic LDS above 64 KB has to be allowed once per kernel
  static hipError_t attr_err = hipSuccess;
  std::call_once(once, [&] {
    attr_err = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                   (int)MS_LDS_MAX);
  });
  if (attr_err != hipSuccess) return attr_err;
  hipLaunchKernelGGL(kern, dim3(sp.G), dim3(MS_THREADS), sp.lds, st, W, X, ldx, xrow, part, epi, M, N, K, sp.cs, sp.rpg,
                     sp.ranges, sp.rpw, sp.npass);
  return hipGetLastError();
}

}  // namespace

bool mstripe_ok(int M, int N, int K, int epi) {
  return plan_mstripe(M, N, K, epi == EPI_SILU, epi == EPI_ROPE).ok != 0;
}

int mstripe_groups(int M, int N, int K, int epi) {
  const MsPlan sp = plan_mstripe(M, N, K, epi == EPI_SILU, epi == EPI_ROPE);
  return sp.ok ? sp.G : 0;
}

hipError_t launch_mstripe(hipStream_t st, int epi_kind, const void* W, const void* X, int ldx, const int* xrow,
                          float* part, const StripeEpi& epi, int M, int N, int K) {
  const MsPlan sp = plan_mstripe(M, N, K, epi_kind == EPI_SILU, epi_kind == EPI_ROPE);
  if (!sp.ok || !W || !X || ldx < K || ldx % 8 != 0) return hipErrorInvalidValue;
  if ((reinterpret_cast<uintptr_t>(W) | reinterpret_cast<uintptr_t>(X)) & 15) return hipErrorInvalidValue;
  const bf16_t* w = (const bf16_t*)W;
  const bf16_t* x = (const bf16_t*)X;
#define SD_MS_LAUNCH(EPI_)                                                                                   \
  return M > 16 ? launch_ms<2, EPI_>(st, w, x, ldx, xrow, part, epi, M, N, K, sp)                            \
                : launch_ms<1, EPI_>(st, w, x, ldx, xrow, part, epi, M, N, K, sp)
  switch (epi_kind) {
    case EPI_PART: SD_MS_LAUNCH(EPI_PART);
    case EPI_SILU: SD_MS_LAUNCH(EPI_SILU);
    case EPI_RESID: SD_MS_LAUNCH(EPI_RESID);
    case EPI_ROPE: SD_MS_LAUNCH(EPI_ROPE);
    default: return hipErrorInvalidValue;
  }
#undef SD_MS_LAUNCH
}

}  // namespace sd
