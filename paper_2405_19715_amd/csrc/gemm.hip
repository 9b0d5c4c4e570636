// Weight-streaming skinny GEMMs: part[s, m, n] = sum_{k in slice s} X[m, k] * W[n, k].
//
// These are the kernels the verify pass (M = K+1 rows, Algorithm 2's parallel target
// forward) and the draft steps (M = 1 or 2 rows) spend their time in: every weight
// is read from HBM exactly once per call and used for M multiply-adds, so the
// kernels are bound by HBM bandwidth and their design is about how the weight stream
// is laid over workgroups, wavefronts and time.  Three of them: the row-stripe kernel
// (up to 8 rows, vector-ALU dot products, described where it is defined below), its sibling
// for 9 .. 17 rows (matrix-core products on LDS-transposed half tiles, gemm_mstripe.hip) and
// the older MFMA kernel described here (what is left up to 16 rows: K below 2048, or, beyond 8
// rows, K not a multiple of 512).
//
// bf16 layout of the work of the MFMA kernel
//   grid       = G row groups x S K-slices.  A workgroup (8 wavefronts) belongs to one
//                K-slice for its whole life: it stages that slice of X into LDS once
//                (already in the order the multiply needs) and never synchronises again.
//   wavefront  = walks its own list of 16-row weight tiles (tile = slot, slot + NW, ...)
//                (NW = 8 G) with ONE continuous software pipeline of 16-byte loads that runs across
//                tile boundaries; per 128-k step it issues 4 load instructions, each covering
//                8 rows x one whole 128-byte line (lane (r = lane % 16, g = lane / 16) of
//                instruction 2 seg + a: row 8 a + r % 8, bytes seg * 128 + ((r / 8) * 4 + g) * 16).
//                The MFMA wants lane (r, g) to hold row r, so half of every operand sits 8 lanes
//                away: one v_mov_b32_dpp row_ror:8 per dword puts it in place (the vector ALU is
//                idle anyway).  Whole lines per instruction are what lets non-temporal loads pay:
//                a pure-read test of this pattern streams 6.4 TB/s with them against 5.9-6.0
//                without, or with 64-byte row pieces per instruction (the MFMA's native operand
//                layout, 16 rows x 64 B) with or without them.
//   rotation   = each wavefront starts its slice at a different k-step (and wraps), so
//                that the thousands of concurrent row streams, whose row stride is a
//                large power of two, do not all hit the same HBM channels at once.
//   few, long-lived workgroups (about one per CU) measured faster than many short ones:
//                fewer concurrent DRAM streams and no repeated X staging.
//   multiply   = v_mfma_f32_16x16x32_bf16 for every M, weights as the A operand (16 rows
//                x 32 k), X^T as the B operand (32 k x 16 activation rows), one MFMA per
//                16-row tile of X; the last tile keeps only its live rows in LDS.  Per-lane
//                fp32 dot products with a shuffle reduction ON THIS LAYOUT were measured for
//                M <= 4 and were slower (M = 1, 12288 x 4096: 29 us against 23 us): the matrix
//                core costs the wavefront one issue slot per 64 B of weights where the dot
//                product costs sixteen.
// Per-slice partial sums go to part[s] and are added by the consumer in slice order,
// so results do not depend on scheduling.
// fp32 weights (tiny configuration) take a plain wave-per-output-row kernel.
#include "common.hpp"
#include "kernels.hpp"
#include "stripe_common.hpp"

#include <cstdlib>
#include <mutex>
#include <vector>

namespace sd {

namespace {

constexpr int GEMM_WAVES = 8;            // wavefronts per workgroup, all sharing one staged X slice
constexpr int GEMM_THREADS = 64 * GEMM_WAVES;
constexpr int KSTEP = 128;
constexpr int LDS_MAX = 144 * 1024;      // largest X slice per workgroup (one workgroup per CU, 160 KB of LDS)
constexpr int PREFETCH = 4;              // steps of weight loads in flight per wave

struct Split { int S, steps_per, G; };

// Pick the K-slice length (steps_per) and the number of row groups G by a small cost
// model of the stream, fitted to measurements on the MI355X:
//   - every workgroup must be resident at once (it is a persistent design): one per CU;
//   - a wavefront with PREFETCH steps in flight sustains about 3.6 GB/s under load, and all
//     of them together about 6.2 TB/s (whole-line non-temporal loads; 2.6 GB/s and 5.3 TB/s before them);
//   - the slowest wavefront (most tiles x steps) ends the kernel;
//   - partial sums are written once and read once by the consumer, slice after slice.
Split plan_bf16_search(int M, int N, int K) {
  const int total = K / KSTEP;
  const int ntiles = N / 16;
  int max_steps = LDS_MAX / (M * KSTEP * 2);
  if (max_steps < 1) max_steps = 1;
  if (max_steps > total) max_steps = total;
  const int g_max = (ntiles + GEMM_WAVES - 1) / GEMM_WAVES;
  const double bw = 6.2e12, wave_rate = 3.6e9, step_bytes = 16.0 * KSTEP * 2;
  Split best{1, total, 1};
  double best_cost = 1e30;
  for (int sp = max_steps; sp >= 1; --sp) {
    const int S = (total + sp - 1) / sp;
    const size_t lds = (size_t)M * sp * KSTEP * 2;
    const int resident = 1;                // one workgroup per CU measured best
    int g_hi = (256 * resident) / S;
    if (g_hi > g_max) g_hi = g_max;
    if (g_hi < 1) {
      if (S > 256 * resident) continue;       // would not be resident all at once
      g_hi = 1;
    }
    for (int G = 1; G <= g_hi; ++G) {
      const int slots = G * GEMM_WAVES;
      const int per = (ntiles + slots - 1) / slots;               // tiles of the busiest wavefront
      const double waves = (double)(ntiles < slots ? ntiles : slots) * S;
      // more than ~2048 concurrent row streams cost DRAM locality (measured: -8 % per doubling)
      double bw_eff = bw;
      for (double w = 2048.0; w < waves; w *= 2.0) bw_eff *= (waves >= 2.0 * w) ? 0.92 : 1.0 - 0.08 * (waves / w - 1.0);
      const double rate = wave_rate < bw_eff / waves ? wave_rate : bw_eff / waves;
      const double t_stream = (double)per * sp * step_bytes / rate;
      const double t_stage = (double)lds / 60.0e9;                // X slice through one CU's L2 port
      const double t_part = 2.0 * S * M * (double)N * 4.0 / bw;
      const double cost = 3.0e-6 + t_stage + t_stream + t_part + 0.25e-6 * S;   // consumers walk S slices
      if (cost < best_cost) { best_cost = cost; best = {S, sp, G}; }
    }
  }
  return best;
}

// The search walks a few thousand candidates (tens of microseconds on the host), and every launch and every
// consumer of the partial sums asks for the plan: remember it per shape (a forward pass has a handful of
// shapes; the table is per host thread).
Split plan_bf16(int M, int N, int K) {
  struct Entry { int M, N, K; Split sp; };
  static thread_local std::vector<Entry> table;
  for (const Entry& e : table)
    if (e.M == M && e.N == N && e.K == K) return e.sp;
  const Split sp = plan_bf16_search(M, N, K);
  if (table.size() >= 1024) table.clear();
  table.push_back(Entry{M, N, K, sp});
  return sp;
}

__device__ __forceinline__ uint4 ldg128(const bf16_t* p) { return *reinterpret_cast<const uint4*>(p); }

// 16-byte non-temporal load (compiles to one global_load_dwordx4 ... nt): for the weights, which are read
// once per call.  It only pays when one instruction covers whole 128-byte lines (see the file comment).
__device__ __forceinline__ uint4 ldg128_stream(const bf16_t* p) {
  const uint32_t* q = reinterpret_cast<const uint32_t*>(p);
  uint4 v;
  v.x = __builtin_nontemporal_load(q);
  v.y = __builtin_nontemporal_load(q + 1);
  v.z = __builtin_nontemporal_load(q + 2);
  v.w = __builtin_nontemporal_load(q + 3);
  return v;
}

// dst lanes 8..15 (HI) or 0..7 (!HI) of every 16-lane row take `src` from the lane 8 away; the rest keep `old`.
template <bool HI>
__device__ __forceinline__ uint4 take_rot8(const uint4& old, const uint4& src) {
  constexpr int ROW_ROR8 = 0x128, BANKS = HI ? 0xC : 0x3;
  uint4 r;
  r.x = (uint32_t)__builtin_amdgcn_update_dpp((int)old.x, (int)src.x, ROW_ROR8, 0xF, BANKS, false);
  r.y = (uint32_t)__builtin_amdgcn_update_dpp((int)old.y, (int)src.y, ROW_ROR8, 0xF, BANKS, false);
  r.z = (uint32_t)__builtin_amdgcn_update_dpp((int)old.z, (int)src.z, ROW_ROR8, 0xF, BANKS, false);
  r.w = (uint32_t)__builtin_amdgcn_update_dpp((int)old.w, (int)src.w, ROW_ROR8, 0xF, BANKS, false);
  return r;
}

__device__ __forceinline__ bf16x8 as_bf16x8(const uint4& v) {
  union { uint4 u; bf16x8 b; } c;
  c.u = v;
  return c.b;
}

// Stage X[0..M, kbeg .. kbeg + 128*steps) into LDS as 16-byte groups.  Group o of a row
// covers k = kbeg + 8 o ..; within a 128-k step it is (j = (o / 4) % 4, g = o % 4).
//   MFMA order: group (m, step s, j, g) lands at
//     tile_base(m / 16) + (((s*4 + j)*4 + g) * rows_in_tile + m % 16)
//   so that lane (r, g) of MFMA j reads one 16-byte word at a lane-linear address.
__device__ __forceinline__ void stage_x(uint4* lds, const bf16_t* X, int ldx, const int* xrow, int M, int kbeg,
                                        int steps) {
  const int groups_per_row = steps * 16;
  const int last_tile = (M - 1) >> 4;
  const int rows_last = M - (last_tile << 4);
  for (int idx = threadIdx.x; idx < M * groups_per_row; idx += GEMM_THREADS) {
    const int m = idx / groups_per_row, o = idx - m * groups_per_row;
    const int src_row = xrow ? xrow[m] : m;
    const uint4 v = ldg128(X + (size_t)src_row * ldx + kbeg + o * 8);
    const int s = o >> 4, j = (o >> 2) & 3, g = o & 3;
    const int tile = m >> 4, r = m & 15;
    const int rows_in_tile = (tile == last_tile) ? rows_last : 16;
    lds[tile * groups_per_row * 16 + (((s * 4 + j) * 4 + g) * rows_in_tile + r)] = v;
  }
}

// What a wavefront needs to walk its tiles: see the file comment.
struct WaveWalk {
  const bf16_t* base;      // this lane's address at (tile 0 of the wave, step 0, j = 0)
  size_t tile_stride;      // elements between consecutive tiles of the wave
  int steps, rot, nwork;
  __device__ __forceinline__ const bf16_t* at(int idx) const {
    const int t = idx / steps;
    int s = idx - t * steps + rot;
    if (s >= steps) s -= steps;
    return base + (size_t)t * tile_stride + s * KSTEP;
  }
};

// NT = number of 16-row activation tiles, ceil(M / 16).
template <int NT>
__global__ __launch_bounds__(GEMM_THREADS) void gemm_bf16_stream(const bf16_t* __restrict__ W,
                                                                 const bf16_t* __restrict__ X, int ldx,
                                                                 const int* __restrict__ xrow,
                                                                 float* __restrict__ part, int M, int N, int K,
                                                                 int steps_per, int G) {
  extern __shared__ uint4 lds[];
  const int total_steps = K / KSTEP;
  const int ks = blockIdx.y, grp = blockIdx.x;
  const int sbeg = ks * steps_per;
  const int steps = min(steps_per, total_steps - sbeg);
  const int kbeg = sbeg * KSTEP;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int r = lane & 15, g = lane >> 4;
  const int ntiles = N >> 4;
  const int wslot = grp * GEMM_WAVES + wave, nslots = G * GEMM_WAVES;
  const int my_tiles = wslot < ntiles ? (ntiles - wslot + nslots - 1) / nslots : 0;

  WaveWalk ww;
  // lane (r, g) of load instruction j = 2 seg + a of a step: row 8 a + r % 8 of the tile, 16 bytes at byte
  // seg * 128 + ((r / 8) * 4 + g) * 16 of the step's 256: eight lanes cover one 128-byte line of a row
  ww.base = W + ((size_t)wslot * 16 + (r & 7)) * K + kbeg + ((r >> 3) * 4 + g) * 8;
  const size_t half_tile = (size_t)8 * K;            // elements from row i to row i + 8
  ww.tile_stride = (size_t)nslots * 16 * K;
  ww.steps = steps;
  ww.rot = (wslot * 5 + ks * 3) % steps;
  ww.nwork = my_tiles * steps;

  // weight loads go out before X is staged, so HBM is busy while the workgroup sets up
  uint4 a[PREFETCH][4];
#pragma unroll
  for (int p = 0; p < PREFETCH; ++p)
    if (p < ww.nwork) {
      const bf16_t* q = ww.at(p);
#pragma unroll
      for (int j = 0; j < 4; ++j) a[p][j] = ldg128_stream(q + (j & 1) * half_tile + (j >> 1) * 64);
    }

  stage_x(lds, X, ldx, xrow, M, kbeg, steps);
  __syncthreads();

  const int groups_per_row = steps * 16;
  const int rows_last = M - ((NT - 1) << 4);
  floatx4 acc[NT];
#pragma unroll
  for (int t = 0; t < NT; ++t) acc[t] = floatx4{0.f, 0.f, 0.f, 0.f};
  float* pout = part + (size_t)ks * M * N;
  int sl = 0, tile = 0;

  for (int i0 = 0; i0 < ww.nwork; i0 += PREFETCH) {
#pragma unroll
    for (int p = 0; p < PREFETCH; ++p) {
      const int i = i0 + p;
      if (i < ww.nwork) {
        // MFMA 2 seg + m wants lane (r, g) to hold row r, bytes seg * 128 + m * 64 + 16 g: lanes r < 8 have that
        // for m = 0 from instruction a = 0 and lanes r >= 8 for m = 1 from a = 1; the other halves sit 8 lanes away
        uint4 cur[4];
        cur[0] = take_rot8<true>(a[p][0], a[p][1]);
        cur[1] = take_rot8<false>(a[p][1], a[p][0]);
        cur[2] = take_rot8<true>(a[p][2], a[p][3]);
        cur[3] = take_rot8<false>(a[p][3], a[p][2]);
        if (i + PREFETCH < ww.nwork) {
          const bf16_t* q = ww.at(i + PREFETCH);
#pragma unroll
          for (int j = 0; j < 4; ++j) a[p][j] = ldg128_stream(q + (j & 1) * half_tile + (j >> 1) * 64);
        }
        int s = sl + ww.rot;
        if (s >= steps) s -= steps;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const bf16x8 av = as_bf16x8(cur[j]);
#pragma unroll
          for (int t = 0; t < NT; ++t) {
            uint4 bv;
            if (t < NT - 1) {
              bv = lds[t * groups_per_row * 16 + (((s * 4 + j) * 4 + g) * 16 + r)];
            } else {
              bv = (r < rows_last) ? lds[t * groups_per_row * 16 + (((s * 4 + j) * 4 + g) * rows_last + r)]
                                   : uint4{0u, 0u, 0u, 0u};
            }
            acc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av, as_bf16x8(bv), acc[t], 0, 0, 0);
          }
        }
        if (++sl == steps) {                  // tile finished: write its partial sums, start the next
          const int row0 = (wslot + tile * nslots) * 16;
          // D[i, n]: lane (n = lane % 16, i = 4 * (lane / 16) + 0..3): four consecutive weight
          // rows for activation row n -> one 16-byte store.
#pragma unroll
          for (int t = 0; t < NT; ++t) {
            const int m = t * 16 + r;
            if (m < M) *reinterpret_cast<floatx4*>(pout + (size_t)m * N + row0 + 4 * g) = acc[t];
            acc[t] = floatx4{0.f, 0.f, 0.f, 0.f};
          }
          sl = 0;
          ++tile;
        }
      }
    }
  }
}


// ----------------------------------------------------------------------------- stripe kernel
// Few activation rows (M <= 8).  Every load instruction covers 1 KB of ONE weight row (lane l: k = 8 l .. 8 l + 7
// of a 512-k piece); a step is four such pieces, 4 KB contiguous.  A wavefront owns one 2048-k stripe of a
// contiguous range of rows and takes one row per step, so its stripe of X (4 x 16 bytes per lane and
// activation row) lives in registers: no LDS and no barrier inside the stream.  This access pattern reads
// HBM at 6.5-6.8 TB/s in a pure-read test (70B gate|up) where the MFMA kernel's 8 rows x 128 B per instruction
// reach 6.4: rows are 16 KB apart, and addresses 16 KB apart meet in the same DRAM channel (the interleave is
// 4 KB).  The matrix core cannot take operands laid out this way (it wants 16 rows x 32 k across the lanes), so
// the products are v_dot2_f32_bf16 on the vector ALU, 4 per 16 bytes of weights and activation row, and each
// row ends with a butterfly over the 64 lanes that reduces all MM sums at once (the lanes halve the set of
// sums they carry at each of the first log2 MM exchanges).  The stripes of a row range all belong to one
// workgroup, which adds them at the end: one slice of finished sums, on which the final sweep can also do the
// elementwise work that follows the product in a decoder layer (see EPI below).
constexpr int STRIPE_MAX_M = 8;
constexpr size_t STRIPE_LDS_MAX = 64 * 1024;
constexpr int PIECE = 512;               // k per 1 KB piece
constexpr int RSTEP = 4 * PIECE;         // k per stripe = per step of 4 load instructions

// The stripes of a row range all sit in one workgroup and are added there: cs wavefronts, each taking npass stripes
// one after the other (the 70B down projection: 14 stripes = 7 wavefronts x 2), so part[] always gets ONE slice.
struct StripePlan { int S, cs, rpg, G, ranges, rpw, npass; };   // rpg row ranges per workgroup (cs * rpg wavefronts); G workgroups

// paired: N is the row count of each half of a [gate; up] matrix, and a workgroup takes its ranges in pairs
// (needs one slice and an even number of ranges per workgroup)
// even_rows: every range holds an even number of rows (the rotary pairs of EPI_ROPE stay inside one wavefront)
StripePlan plan_stripe(int M, int N, int K, bool paired = false, bool even_rows = false) {
  StripePlan sp{0, 0, 0, 0, 0, 0, 0};
  if (M < 1 || M > STRIPE_MAX_M || N < 1 || K < RSTEP || K % 8 != 0) return sp;
  const int stripes = (K + RSTEP - 1) / RSTEP;       // the last one may be short (K % 2048 != 0)
  int cs = 1;
  for (int d = 2; d <= GEMM_WAVES; ++d)
    if (stripes % d == 0) cs = d;
  const int npass = stripes / cs;                    // stripes a wavefront takes one after the other
  if (npass > 8) return sp;
  const int rpg = GEMM_WAVES / cs;
  if (paired && (rpg & 1)) return sp;
  const int units = paired ? rpg / 2 : rpg;          // ranges of N a workgroup covers
  int ranges = 256 * units;                          // one workgroup per CU
  if (ranges > N) ranges = N;
  int rpw = (N + ranges - 1) / ranges;
  if (even_rows) {
    if (N & 1) return sp;
    rpw += rpw & 1;
  }
  ranges = (N + rpw - 1) / rpw;
  const int G = (ranges + units - 1) / units;
  if ((size_t)cs * rpg * M * rpw * sizeof(float) > STRIPE_LDS_MAX) return sp;         // the wavefronts' output tiles
  return StripePlan{1, cs, rpg, G, ranges, rpw, npass};
}

// RAGGED: K is not a multiple of 2048; a lane of the last stripe whose piece lies beyond K reads the first 16 bytes
// of the stripe instead (lane 0's piece 0, which every stripe has: a fixed per-lane offset, nothing changes in the
// loop) against zeros in X.
template <int MM, int EPI, bool RAGGED>
__global__ __launch_bounds__(GEMM_THREADS) void gemm_bf16_stripe(const bf16_t* __restrict__ W,
                                                                 const bf16_t* __restrict__ X, int ldx,
                                                                 const int* __restrict__ xrow,
                                                                 float* __restrict__ part, StripeEpi epi, int M, int N,
                                                                 int K, int cs, int rpg, int ranges, int rpw,
                                                                 int npass) {
  constexpr bool SILU = EPI == EPI_SILU;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int lr = wave / cs, ls = wave - lr * cs;     // local row range, local stripe
  const int rg = SILU ? blockIdx.x * (rpg >> 1) + (lr >> 1) : blockIdx.x * rpg + lr;
  // first stripe of K.  SILU: gate and up are a multiple of 2^26 bytes apart for the 70B shape (the same DRAM channel
  // and bank at equal k), and a pair's wavefronts run side by side: the up wavefronts take their stripes one further
  const int c0 = SILU && (lr & 1) ? (ls + 1 == cs ? 0 : ls + 1) : ls;
  const int r0 = rg * rpw + (SILU && (lr & 1) ? N : 0);          // SILU: odd local ranges are the rows of `up`
  const int rows = rg < ranges ? min(rpw, N - rg * rpw) : 0;     // a wavefront without rows still meets the barrier
  const bf16_t* const idle = W + lane * 8;

  __shared__ float s_scale[STRIPE_MAX_M];            // the rows' RMSNorm factors (1 unless the producer left them out)
  float sq[2][STRIPE_SSQ_PER_LANE];                  // up to 2 * 7 wavefronts >= 8 rows
  if constexpr (EPI != EPI_RESID) stripe_load_ssq<2>(epi, MM, sq);

  // after the butterfly lane l holds the sum of activation row l / (64 / P2); its lanes with the low bits
  // clear put it into the wave's LDS tile [MM][rpw]; the tiles of the cs stripes are added and go to part[] in
  // one coalesced sweep at the end (no global store inside the loop: stores count like loads, and a store
  // under a branch would make the compiler wait for every load in flight)
  extern __shared__ float obuf[];
  constexpr int P2 = MM <= 1 ? 1 : MM <= 2 ? 2 : MM <= 4 ? 4 : 8;
  constexpr int LPM = 64 / P2;
  const int my_m = lane / LPM;
  const bool writer = (lane % LPM) == 0 && my_m < MM;
  float* otile = obuf + (size_t)wave * MM * rpw;

  for (int ps = 0; ps < npass; ++ps) {
    const int c = ps * cs + c0;                        // this pass's stripe of K
    const int rot = rows > 0 ? ((rg * npass * cs + c) * 5) % rows : 0;
    const bf16_t* base = W + (size_t)(rows > 0 ? r0 : 0) * K + c * RSTEP + lane * 8;
    auto at = [&](int t) -> const bf16_t* {
      int r = t + rot;
      if (r >= rows) r -= rows;
      if constexpr (EPI == EPI_ROPE) {                 // local index -> row of W: (head, i, half) order
        const int hs = epi.hshift;
        const int j = r0 + r, p = j >> 1;
        const int row = ((p >> hs) << (hs + 1)) + (p & ((1 << hs) - 1)) + ((j & 1) << hs);
        return W + (size_t)row * K + c * RSTEP + lane * 8;
      }
      return base + (size_t)r * K;
    };
    int off[4];                                        // element offset of this lane's piece j from its piece 0
    bool live[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      live[j] = !RAGGED || c * RSTEP + j * PIECE + lane * 8 < K;
      off[j] = live[j] ? j * PIECE : -lane * 8;        // dead: the stripe's first 16 bytes (k = c * RSTEP < K)
    }

    // X first: its loads are then older than every weight load, and waiting for a weight step never waits for them
    uint4 x[MM][4];                                    // M == MM (the launcher picks the instantiation)
#pragma unroll
    for (int m = 0; m < MM; ++m) {
      const bf16_t* xp = X + (size_t)(xrow ? xrow[m] : m) * ldx + c * RSTEP + lane * 8;
#pragma unroll
      for (int j = 0; j < 4; ++j) x[m][j] = ldg128(RAGGED ? xp + off[j] : xp + j * PIECE);
    }

    // Every step issues its four loads without a branch around them, so that the compiler can count the loads in
    // flight and wait for the oldest step only; past the wave's last row the address is the start of W (a
    // line every wave shares: served by L2) and the data is not used.
    uint4 a[PREFETCH][4];
#pragma unroll
    for (int p = 0; p < PREFETCH; ++p) {
      const bf16_t* q = p < rows ? at(p) : idle;
#pragma unroll
      for (int j = 0; j < 4; ++j) a[p][j] = ldg128_stream(RAGGED ? q + off[j] : q + j * PIECE);
    }
    if constexpr (RAGGED) {                            // after the prefetch went out: pieces beyond K count as zeros
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int m = 0; m < MM; ++m)
#pragma unroll
        for (int j = 0; j < 4; ++j)
          if (!live[j]) x[m][j] = uint4{0u, 0u, 0u, 0u};
    }

    for (int i0 = 0; i0 < rows; i0 += PREFETCH) {
#pragma unroll
      for (int p = 0; p < PREFETCH; ++p) {
        const int i = i0 + p;
        __builtin_amdgcn_sched_barrier(0);           // steps stay in order: the next step's data is still in flight
        float acc[P2];
#pragma unroll
        for (int m = 0; m < P2; ++m) acc[m] = 0.f;
        // the sums of one activation row form a dependent chain: the chains of the MM rows interleave
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
          for (int m = 0; m < MM; ++m) acc[m] = dot8(a[p][j], x[m][j], acc[m]);
        {
          const bool more = i + PREFETCH < rows;
          const bf16_t* q = more ? at(i + PREFETCH) : idle;
#pragma unroll
          for (int j = 0; j < 4; ++j) a[p][j] = ldg128_stream(RAGGED ? q + off[j] : q + j * PIECE);
        }
        const float v = reduce_lanes<P2>(acc, lane);
        int r = i + rot;
        if (r >= rows) r -= rows;
        if (writer && i < rows) {
          if (ps == 0) otile[my_m * rpw + r] = v;
          else otile[my_m * rpw + r] += v;             // later stripes of the same wavefront, in stripe order
        }
      }
    }
  }
  stripe_finish<EPI, 2>(obuf, s_scale, sq, part, epi, MM, N, cs, rpg, ranges, rpw);
}

template <int MM, int EPI>
hipError_t launch_stripe_mm(hipStream_t st, const bf16_t* W, const bf16_t* X, int ldx, const int* xrow, float* part,
                            const StripeEpi& epi, int M, int N, int K, StripePlan sp) {
  const size_t lds = (size_t)sp.cs * sp.rpg * MM * sp.rpw * sizeof(float);
  if (lds > STRIPE_LDS_MAX) return hipErrorInvalidValue;
  const dim3 grid(sp.G), block(sp.cs * sp.rpg * WAVE);
  if (K % RSTEP)
    hipLaunchKernelGGL((gemm_bf16_stripe<MM, EPI, true>), grid, block, lds, st, W, X, ldx, xrow, part, epi, M, N, K, sp.cs,
                       sp.rpg, sp.ranges, sp.rpw, sp.npass);
  else
    hipLaunchKernelGGL((gemm_bf16_stripe<MM, EPI, false>), grid, block, lds, st, W, X, ldx, xrow, part, epi, M, N, K, sp.cs,
                       sp.rpg, sp.ranges, sp.rpw, sp.npass);
  return hipGetLastError();
}

template <int EPI>
hipError_t launch_stripe(hipStream_t st, const bf16_t* W, const bf16_t* X, int ldx, const int* xrow, float* part,
                         const StripeEpi& epi, int M, int N, int K, StripePlan sp) {
  switch (M) {
    case 1: return launch_stripe_mm<1, EPI>(st, W, X, ldx, xrow, part, epi, M, N, K, sp);
    case 2: return launch_stripe_mm<2, EPI>(st, W, X, ldx, xrow, part, epi, M, N, K, sp);
    case 3: return launch_stripe_mm<3, EPI>(st, W, X, ldx, xrow, part, epi, M, N, K, sp);
    case 4: return launch_stripe_mm<4, EPI>(st, W, X, ldx, xrow, part, epi, M, N, K, sp);
    case 5: return launch_stripe_mm<5, EPI>(st, W, X, ldx, xrow, part, epi, M, N, K, sp);
    case 6: return launch_stripe_mm<6, EPI>(st, W, X, ldx, xrow, part, epi, M, N, K, sp);
    case 7: return launch_stripe_mm<7, EPI>(st, W, X, ldx, xrow, part, epi, M, N, K, sp);
    case 8: return launch_stripe_mm<8, EPI>(st, W, X, ldx, xrow, part, epi, M, N, K, sp);
    default: return hipErrorInvalidValue;
  }
}

// Up to 8 activation rows and K >= 2048 (up to 8 stripes per wavefront): measured equal or faster than the MFMA
// kernel on every such matrix of the 70B / 7B / 1.1B shapes, alone and inside the forward pass (70B target pass,
// 1 .. 8 rows: 2 - 6 % shorter before the fused epilogues, 8 - 12 % with them).
bool use_stripe(int M, int N, int K) { return plan_stripe(M, N, K).S > 0; }

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
hipError_t launch_stream(hipStream_t st, const bf16_t* W, const bf16_t* X, int ldx, const int* xrow, float* part, int M,
                         int N, int K, Split sp) {
  const dim3 grid(sp.G, sp.S);
  const size_t lds = (size_t)M * sp.steps_per * KSTEP * 2;
  // dynamic LDS above 64 KB has to be allowed once per kernel: the first caller does it, whichever thread that is
  static std::once_flag once;
  static hipError_t attr_err = hipSuccess;
  std::call_once(once, [] {
    attr_err = hipFuncSetAttribute(reinterpret_cast<const void*>(gemm_bf16_stream<NT>),
                                   hipFuncAttributeMaxDynamicSharedMemorySize, LDS_MAX + 8 * 1024);
  });
  if (attr_err != hipSuccess) return attr_err;
  hipLaunchKernelGGL(gemm_bf16_stream<NT>, grid, dim3(GEMM_THREADS), lds, st, W, X, ldx, xrow, part, M, N, K,
                     sp.steps_per, sp.G);
  return hipGetLastError();
}

// One 16-row MFMA tile of activations: up to here this kernel wins or ties on every matrix (6 rows, 70B gate|up:
// 164 us against 174 us); from 17 rows on the tiled kernel with its non-temporal whole-line loads is equal or
// faster (17 rows: 173 against 179 us, 32 rows: 176 against 189 us).
constexpr int STREAM_MAX_ROWS = 16;

bool use_tile(int M, int N, int K) { return M > STREAM_MAX_ROWS && K % 32 == 0 && N % 4 == 0; }

}  // namespace

int gemm_splits(int dtype, int M, int N, int K) {
  if (dtype == DT_F32) return 1;
  if (mstripe_ok(M, N, K, EPI_PART)) return 1;
  if (use_tile(M, N, K)) return gemm_tile_splits(M, N, K);
  if (use_stripe(M, N, K)) return plan_stripe(M, N, K).S;
  return plan_bf16(M, N, K).S;
}

hipError_t launch_gemm(hipStream_t st, int dtype, const void* W, const void* X, int ldx, const int* xrow,
                       float* part, int M, int N, int K) {
  if (!W || !X || !part || M < 1 || M > MAX_PREFILL_ROWS || N < 1 || K < 1 || ldx < K) return hipErrorInvalidValue;
  if (M > MAX_ROWS && !(dtype == DT_BF16 && use_tile(M, N, K))) return hipErrorInvalidValue;
  if (dtype == DT_F32) {
    hipLaunchKernelGGL(gemm_f32, dim3((N + 3) / 4), dim3(256), 0, st, (const float*)W, (const float*)X, ldx,
                       xrow, part, M, N, K);
    return hipGetLastError();
  }
  if (dtype != DT_BF16) return hipErrorInvalidValue;
  if (mstripe_ok(M, N, K, EPI_PART)) {
    if (reinterpret_cast<uintptr_t>(part) & 15) return hipErrorInvalidValue;
    return launch_mstripe(st, EPI_PART, W, X, ldx, xrow, part, StripeEpi{}, M, N, K);
  }
  if (use_tile(M, N, K)) return launch_gemm_tile(st, W, X, ldx, xrow, part, M, N, K);
  if (use_stripe(M, N, K)) {
    if (ldx % 8 != 0 ||
        ((reinterpret_cast<uintptr_t>(W) | reinterpret_cast<uintptr_t>(X) | reinterpret_cast<uintptr_t>(part)) & 15))
      return hipErrorInvalidValue;
    return launch_stripe<EPI_PART>(st, (const bf16_t*)W, (const bf16_t*)X, ldx, xrow, part, StripeEpi{}, M, N, K,
                                   plan_stripe(M, N, K));
  }
  // 16-byte loads along K, 16-row tiles along N, 16-byte aligned rows
  if (K % KSTEP != 0 || N % 16 != 0 || ldx % 8 != 0) return hipErrorInvalidValue;
  if ((reinterpret_cast<uintptr_t>(W) | reinterpret_cast<uintptr_t>(X) | reinterpret_cast<uintptr_t>(part)) & 15)
    return hipErrorInvalidValue;
  const Split sp = plan_bf16(M, N, K);
  const bf16_t* w = (const bf16_t*)W;
  const bf16_t* x = (const bf16_t*)X;
  // more than one 16-row activation tile never gets here (use_tile took it); the kernel itself is written
  // for any number of tiles, which is how the two paths were compared
  if (M > 16) return hipErrorInvalidValue;
  return launch_stream<1>(st, w, x, ldx, xrow, part, M, N, K, sp);
}

bool gemm_silu_fused(int dtype, int M, int ffn, int K) {
  return dtype == DT_BF16 && (plan_stripe(M, ffn, K, true).S == 1 || mstripe_ok(M, ffn, K, EPI_SILU));
}

hipError_t launch_gemm_silu(hipStream_t st, int dtype, const void* W, const void* X, int ldx, const int* xrow,
                            void* act, int M, int ffn, int K, const float* ssq, int ssq_n, int d_in, float eps) {
  if (!W || !X || !act || ldx < K || ldx % 8 != 0 || !gemm_silu_fused(dtype, M, ffn, K)) return hipErrorInvalidValue;
  if ((reinterpret_cast<uintptr_t>(W) | reinterpret_cast<uintptr_t>(X)) & 15) return hipErrorInvalidValue;
  if (ssq && (ssq_n < 1 || ssq_n > 256 || d_in < 1)) return hipErrorInvalidValue;
  StripeEpi epi{};
  epi.act = (bf16_t*)act;
  epi.ssq_in = ssq;
  epi.ssq_n = ssq_n;
  epi.inv_d = ssq ? 1.0f / (float)d_in : 0.f;
  epi.eps = eps;
  if (M > STRIPE_MAX_M) return launch_mstripe(st, EPI_SILU, W, X, ldx, xrow, nullptr, epi, M, ffn, K);
  return launch_stripe<EPI_SILU>(st, (const bf16_t*)W, (const bf16_t*)X, ldx, xrow, nullptr, epi, M, ffn, K,
                                 plan_stripe(M, ffn, K, true));
}

bool gemm_scaled_ok(int dtype, int M, int N, int K) {
  return dtype == DT_BF16 && (use_stripe(M, N, K) || mstripe_ok(M, N, K, EPI_PART));
}

hipError_t launch_gemm_scaled(hipStream_t st, int dtype, const void* W, const void* X, int ldx, const int* xrow,
                              float* part, int M, int N, int K, const float* ssq, int ssq_n, int d_in, float eps) {
  if (!W || !X || !part || !ssq || ldx < K || ldx % 8 != 0 || !gemm_scaled_ok(dtype, M, N, K) || ssq_n < 1 ||
      ssq_n > 256 || d_in < 1)
    return hipErrorInvalidValue;
  if ((reinterpret_cast<uintptr_t>(W) | reinterpret_cast<uintptr_t>(X) | reinterpret_cast<uintptr_t>(part)) & 15)
    return hipErrorInvalidValue;
  StripeEpi epi{};
  epi.ssq_in = ssq;
  epi.ssq_n = ssq_n;
  epi.inv_d = 1.0f / (float)d_in;
  epi.eps = eps;
  if (M > STRIPE_MAX_M) return launch_mstripe(st, EPI_PART, W, X, ldx, xrow, part, epi, M, N, K);
  return launch_stripe<EPI_PART>(st, (const bf16_t*)W, (const bf16_t*)X, ldx, xrow, part, epi, M, N, K,
                                 plan_stripe(M, N, K));
}

namespace {
int log2_exact(int v) {                 // -1 unless v is a power of two
  if (v < 1 || (v & (v - 1))) return -1;
  int s = 0;
  while ((1 << s) < v) ++s;
  return s;
}
}  // namespace

bool gemm_rope_fused(int dtype, int M, int Hq, int Hkv, int hd, int K) {
  if (dtype != DT_BF16 || Hq < 1 || Hkv < 1 || hd < 2 || log2_exact(hd) < 1) return false;
  return plan_stripe(M, (Hq + 2 * Hkv) * hd, K, false, true).S == 1 || mstripe_ok(M, (Hq + 2 * Hkv) * hd, K, EPI_ROPE);
}

hipError_t launch_gemm_rope(hipStream_t st, int dtype, const void* W, const void* X, int ldx, int M, int Hq, int Hkv,
                            int hd, int K, const int32_t* row_seq, const int32_t* row_pos, const float* cos_sin,
                            void* qbuf, void* kcache, void* vcache, int max_seq, const float* ssq, int ssq_n, int d_in,
                            float eps) {
  if (!W || !X || !row_seq || !row_pos || !cos_sin || !qbuf || !kcache || !vcache || max_seq < 1 || ldx < K ||
      ldx % 8 != 0 || !gemm_rope_fused(dtype, M, Hq, Hkv, hd, K))
    return hipErrorInvalidValue;
  if (ssq && (ssq_n < 1 || ssq_n > 256 || d_in < 1)) return hipErrorInvalidValue;
  if ((reinterpret_cast<uintptr_t>(W) | reinterpret_cast<uintptr_t>(X)) & 15) return hipErrorInvalidValue;
  StripeEpi epi{};
  epi.ssq_in = ssq;
  epi.ssq_n = ssq ? ssq_n : 0;
  epi.inv_d = ssq ? 1.0f / (float)d_in : 0.f;
  epi.eps = eps;
  epi.row_seq = row_seq;
  epi.row_pos = row_pos;
  epi.cos_sin = cos_sin;
  epi.qbuf = (bf16_t*)qbuf;
  epi.kcache = (bf16_t*)kcache;
  epi.vcache = (bf16_t*)vcache;
  epi.Hq = Hq;
  epi.Hkv = Hkv;
  epi.hshift = log2_exact(hd) - 1;
  epi.max_seq = max_seq;
  const int N = (Hq + 2 * Hkv) * hd;
  if (M > STRIPE_MAX_M) return launch_mstripe(st, EPI_ROPE, W, X, ldx, nullptr, nullptr, epi, M, N, K);
  return launch_stripe<EPI_ROPE>(st, (const bf16_t*)W, (const bf16_t*)X, ldx, nullptr, nullptr, epi, M, N, K,
                                 plan_stripe(M, N, K, false, true));
}

bool gemm_head_fused(int dtype, int M, int N, int K) { return dtype == DT_BF16 && plan_stripe(M, N, K).S == 1; }

hipError_t launch_gemm_head(hipStream_t st, int dtype, const void* W, const void* X, int ldx, const int* xrow,
                            const void* bias, const void* z_in, const int* z_rows, void* z_out, int M, int N, int K) {
  if (!W || !X || !bias || !z_out || ldx < K || ldx % 8 != 0 || !gemm_head_fused(dtype, M, N, K)) return hipErrorInvalidValue;
  if (z_in && N != K) return hipErrorInvalidValue;              // a skip connection needs a square layer
  if ((reinterpret_cast<uintptr_t>(W) | reinterpret_cast<uintptr_t>(X)) & 15) return hipErrorInvalidValue;
  StripeEpi epi{};
  epi.act = (bf16_t*)z_out;
  epi.bias = (const bf16_t*)bias;
  epi.z_in = (const bf16_t*)z_in;
  epi.z_rows = z_rows;
  return launch_stripe<EPI_HEAD>(st, (const bf16_t*)W, (const bf16_t*)X, ldx, xrow, nullptr, epi, M, N, K,
                                 plan_stripe(M, N, K));
}

int gemm_resid_groups(int dtype, int M, int N, int K) {
  if (dtype != DT_BF16) return 0;
  if (M > STRIPE_MAX_M) return mstripe_groups(M, N, K, EPI_RESID);
  const StripePlan sp = plan_stripe(M, N, K);
  return sp.S == 1 ? sp.G : 0;
}

hipError_t launch_gemm_resid(hipStream_t st, int dtype, const void* W, const void* X, int ldx, const int* xrow,
                             float* x, const void* gain, void* xg, float* ssq, int M, int N, int K) {
  if (!W || !X || !x || !gain || !xg || !ssq || ldx < K || ldx % 8 != 0 || gemm_resid_groups(dtype, M, N, K) < 1)
    return hipErrorInvalidValue;
  if ((reinterpret_cast<uintptr_t>(W) | reinterpret_cast<uintptr_t>(X)) & 15) return hipErrorInvalidValue;
  StripeEpi epi{};
  epi.act = (bf16_t*)xg;
  epi.x = x;
  epi.gain = (const bf16_t*)gain;
  epi.ssq_out = ssq;
  if (M > STRIPE_MAX_M) return launch_mstripe(st, EPI_RESID, W, X, ldx, xrow, nullptr, epi, M, N, K);
  return launch_stripe<EPI_RESID>(st, (const bf16_t*)W, (const bf16_t*)X, ldx, xrow, nullptr, epi, M, N, K,
                                  plan_stripe(M, N, K));
}

}  // namespace sd
