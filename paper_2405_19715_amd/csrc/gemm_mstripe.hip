// Row-stripe GEMM for 9 .. 17 activation rows: the verify pass of a round that drafted 8 .. 16 candidates
// (Algorithm 2's parallel target forward over K + 1 positions).
//
// Same organisation as the vector-ALU row-stripe kernel (gemm.hip): a wavefront owns one K piece of a contiguous
// range of weight rows, every load instruction covers 1 KB of ONE row (the access pattern that reads HBM fastest),
// its piece of X lives in registers for the whole pass, the K pieces of a row range all belong to one workgroup,
// which adds them at the end, so there is ONE slice of finished sums and the final sweep does the elementwise work
// of the decoder layer (SiLU * up, residual + norm, rotary embedding + KV append: stripe_common.hpp).  What
// differs is the multiply: 16 * M dot products per 16 bytes of weights do not fit the vector ALU beyond 8 rows
// (it is 54 % busy there), so the products run on the matrix cores, v_mfma_f32_16x16x32_bf16 with the weights
// as the A operand (16 rows x 32 k) and X^T as the B operand.
//
// The matrix core wants lane (i, g) to hold 16 bytes of weight row i, a row-contiguous load gives lane l 16 bytes
// of ONE row: the tile is transposed through a per-wavefront LDS buffer.  A wavefront takes 8 weight rows at a
// time (rows 8 .. 15 of the A operand read a row of zeros: the matrix cores have time to spare, LDS space is what
// is short): row r of the 8 goes to LDS as it arrives, 16-byte block b of the row at slot b ^ r of the row's 1 KB,
// and lane (i, g) reads block 4 t + g of row i for MFMA t: both the 64-lane write and the read hit 16 distinct
// 16-byte bank groups per 16 lanes.  The 16 row registers of a wavefront are a ring over two such half tiles, each
// reloaded as soon as it has been written to LDS, so 16 KB per wavefront are in flight all the time, as in the
// vector-ALU kernel.  LDS operations of one wavefront execute in order, so the next half tile's writes cannot
// overtake this one's reads.
//
// X: the B operand of MFMA t is X[m = lane % 16][k0 + 8 (4 t + g) ..], 16 registers of 16 bytes for the first 16
// activation rows (a load instruction reads 64 contiguous bytes of each row: with block t + 16 g instead, 64 separate
// 16-byte pieces per instruction, the X loads of a pass cost the CU's address path about 4 us, seven times per
// launch on the 70B down projection).  A 17th row (K = 16 candidates) would need a second MFMA per step for one live
// column in 16; it is multiplied on the vector ALU instead, where the weight rows pass through registers in row
// order anyway: its piece of X is ONE register quad (lane l: the 8 k of block l, as the weights), four v_dot2 per
// weight row before the row goes to LDS, and one transposing butterfly over the 8 sums of a half tile.
#include "common.hpp"
#include "kernels.hpp"
#include "stripe_common.hpp"

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

// MT = 1: up to 16 activation rows; MT = 2: 17.
template <int MT, int EPI>
__global__ __launch_bounds__(MS_THREADS) void gemm_bf16_mstripe(const bf16_t* __restrict__ W,
                                                                const bf16_t* __restrict__ X, int ldx,
                                                                const int* __restrict__ xrow,
                                                                float* __restrict__ part, StripeEpi epi, int M, int N,
                                                                int K, int cs, int rpg, int ranges, int rpw,
                                                                int npass) {
  constexpr bool SILU = EPI == EPI_SILU;
  // the wavefront's index as a scalar: everything derived from it (row range, pieces, loop bounds) then lives in
  // scalar registers and the address selection below costs no vector compares or exec-mask branches
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
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
  // this lane's write slot for row r of a half tile is (lane ^ r); its read for MFMA t is block (4 t + g) of row
  // li (or of the zero row), at slot block ^ li
  const unsigned char* const rd_row = buf + (li < MS_HALF ? li : MS_HALF) * 1024;

  // The weight stream runs across the passes: the ring is refilled from the next pass's piece while this pass's last
  // half tiles are multiplied, so only the X operands change at a pass boundary.  NH = half tiles per pass rounded
  // up to the ring's two halves (a padding half tile reads the idle line, goes through LDS unread, and is neither
  // multiplied nor stored).
  const int NH = (nh + 1) & ~1;
  const int ps_off = rg % npass;
  auto piece_of = [&](int ps) { int q = ps + ps_off; q = q >= npass ? q - npass : q; return q * cs + c0; };
  // start row per pass: the same for the K slots of a row range, so that together they read 8 (4) KB contiguous
  // pieces of a row at about the same time; different from range to range
  auto rot_of = [&](int ps) { return nh > 0 ? ((rg * npass + ps) * 5) % nh : 0; };
  // row r of half tile h of the pass whose piece is c (< 0: past the last pass) and whose walk starts at half tile
  // rot -> address of this lane's 16 bytes (or the idle line past the range / the end)
  auto at = [&](int c, int rot, int h, int r) -> const bf16_t* {
    int hh = h + rot;
    hh = hh >= nh ? hh - nh : hh;
    const int j = hh * MS_HALF + r;
    const bool dead = c < 0 || h >= nh || j >= rows;   // no branch: the address is formed either way, then selected
    int row = dead ? 0 : r0 + j;
    if constexpr (EPI == EPI_ROPE) {                   // local index -> row of W: (head, i, half) order
      const int hs = epi.hshift;
      const int p = row >> 1;
      row = ((p >> hs) << (hs + 1)) + (p & ((1 << hs) - 1)) + ((row & 1) << hs);
    }
    const bf16_t* q = W + (size_t)row * K + (dead ? 0 : c) * MS_PIECE + lane * 8;
    return dead ? idle : q;
  };
  // B operands of a pass: MFMA t, lane (m, g) takes the 8 k of 16-byte block 4 t + g of its row, so that one load
  // instruction reads 64 contiguous bytes of each of its 16 rows
  uint4 xb[16];
  uint4 x16 = uint4{0u, 0u, 0u, 0u};                   // MT == 2: the 17th row's piece, lane l: block l
  // with fewer than 16 rows the lanes beyond take the last row again: their columns of the product are finite and
  // never stored.  The gather indices are read once, here: a dependent load inside a pass would make the pass wait
  // for every weight load in flight.
  const int xm = xrow ? xrow[min(li, M - 1)] : min(li, M - 1);
  const int xm16 = MT == 2 ? (xrow ? xrow[16] : 16) : 0;
  auto load_x = [&](int ps) {
    const int c = piece_of(ps);
    const bf16_t* xr = X + (size_t)xm * ldx + c * MS_PIECE + g * 8;
#pragma unroll
    for (int t = 0; t < 16; ++t) xb[t] = *reinterpret_cast<const uint4*>(xr + t * 32);
    if constexpr (MT == 2)
      x16 = *reinterpret_cast<const uint4*>(X + (size_t)xm16 * ldx + c * MS_PIECE + lane * 8);
  };
  // The weight ring first: HBM starts working at once.  X is not needed before the first MFMA, by when the ring's
  // first half tile must have arrived anyway (and the second is needed right after).
  uint4 a[2 * MS_HALF];
  int roth = rot_of(0);
#pragma unroll
  for (int i = 0; i < 2 * MS_HALF; ++i) a[i] = ms_ld_stream(at(piece_of(0), roth, i / MS_HALF, i % MS_HALF));
  __builtin_amdgcn_sched_barrier(0);
  load_x(0);
  __builtin_amdgcn_sched_barrier(0);

  for (int ps = 0; ps < npass; ++ps) {
    if (ps > 0) load_x(ps);                            // behind the ring's loads, which the pass needs first anyway
    const int c = piece_of(ps);
    const int c_next = ps + 1 < npass ? piece_of(ps + 1) : -1, rot_next = rot_of(ps + 1);
    for (int h0 = 0; h0 < NH; h0 += 2) {
#pragma unroll
      for (int p = 0; p < 2; ++p) {
        const int h = h0 + p;
        __builtin_amdgcn_sched_barrier(0);             // half tiles stay in order: the next one's data is still in flight
        float s16[MS_HALF];                            // MT == 2: this lane's share of the 17th row's 8 sums
#pragma unroll
        for (int r = 0; r < MS_HALF; ++r) {
          *reinterpret_cast<uint4*>(buf + r * 1024 + ((lane ^ r) << 4)) = a[p * MS_HALF + r];
          if constexpr (MT == 2) s16[r] = dot8(a[p * MS_HALF + r], x16, 0.f);
          const bool nx = h + 2 >= NH;                 // the ring runs on into the next pass's piece
          a[p * MS_HALF + r] = ms_ld_stream(at(nx ? c_next : c, nx ? rot_next : roth, nx ? h + 2 - NH : h + 2, r));
        }
        __builtin_amdgcn_sched_barrier(0);
        if (h < nh) {                                  // not the padding half tile of an odd count (no load in here)
          int hh = h + roth;
          hh = hh >= nh ? hh - nh : hh;                // this half tile's place in the range
          if constexpr (MT == 2) {
            // lane l ends with the whole-wavefront sum of weight row l / 8 of the half tile
            const float v16 = reduce_lanes<MS_HALF>(s16, lane);
            if ((lane & 7) == 0) {
              float* dst = otile + 16 * rpw + hh * MS_HALF + (lane >> 3);
              *dst = ps == 0 ? v16 : *dst + v16;
            }
          }
          // A operands: AHEAD LDS reads are requested before the first MFMA and one more with every MFMA, so that
          // an MFMA never waits for the read issued just before it; two accumulators, so that consecutive MFMAs
          // do not wait for each other's results either (even t, odd t; added at the end)
          constexpr int AHEAD = 8;
          floatx4 acc0[2] = {floatx4{0.f, 0.f, 0.f, 0.f}, floatx4{0.f, 0.f, 0.f, 0.f}};
          uint4 f[16];
#define SD_MS_READ(T) f[T] = *reinterpret_cast<const uint4*>(rd_row + (((4 * (T) + g) ^ li) << 4));
#define SD_MS_MUL(T)                                                                                                 \
          acc0[(T) & 1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ms_as_bf16x8(f[T]), ms_as_bf16x8(xb[T]), acc0[(T) & 1], \
                                                                   0, 0, 0);
#define SD_MS_STEP(T)                                             \
          if constexpr ((T) + AHEAD < 16) { SD_MS_READ((T) + AHEAD) } \
          SD_MS_MUL(T)                                            \
          __builtin_amdgcn_sched_barrier(0);
          SD_MS_READ(0) SD_MS_READ(1) SD_MS_READ(2) SD_MS_READ(3) SD_MS_READ(4) SD_MS_READ(5) SD_MS_READ(6)
          SD_MS_READ(7)
          __builtin_amdgcn_sched_barrier(0);
          SD_MS_STEP(0) SD_MS_STEP(1) SD_MS_STEP(2) SD_MS_STEP(3) SD_MS_STEP(4) SD_MS_STEP(5) SD_MS_STEP(6)
          SD_MS_STEP(7) SD_MS_STEP(8) SD_MS_STEP(9) SD_MS_STEP(10) SD_MS_STEP(11) SD_MS_STEP(12) SD_MS_STEP(13)
          SD_MS_STEP(14) SD_MS_STEP(15)
#undef SD_MS_STEP
#undef SD_MS_MUL
#undef SD_MS_READ
          const floatx4 acc0s = acc0[0] + acc0[1];
          // D[i][m]: lane (m = li, g) holds weight rows 4 g .. 4 g + 3 of the half tile (g < 2) for activation row m
          if (g < 2 && li < M) {
            // rpw is a multiple of 8: the four rows stay inside the wavefront's tile
            floatx4* dst = reinterpret_cast<floatx4*>(otile + li * rpw + hh * MS_HALF + 4 * g);
            *dst = ps == 0 ? acc0s : *dst + acc0s;     // later pieces of the same wavefront, in pass order
          }
        }
      }
    }
    roth = rot_next;
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
