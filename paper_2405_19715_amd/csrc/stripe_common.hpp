// What the row-stripe GEMM kernels share: the vector-ALU dot product and the 64-lane butterfly of the few-row
// kernel (the many-row kernel uses them for its 17th activation row), and the final sweep: every wavefront of a workgroup has left its partial sums
// of one K stripe set in an LDS tile [M][rpw] (tile of wavefront w at obuf + w * M * rpw; the wavefronts of local
// row range l are l * cs .. l * cs + cs - 1, in stripe order); the sweep adds the cs tiles of a range in that order
// and does the elementwise work that follows the product in a decoder layer.
#pragma once
#include "common.hpp"

namespace sd {

// What the final sweep of the stripe kernel does with the sums (EPI):
//   EPI_PART  part[m][n] = r_m sum
//   EPI_SILU  W = [gate; up] with N rows each (2 N in all), one slice, rpg even: the workgroup's local ranges come
//             in pairs, range g of gate and range g of up, and act[m, n] = silu(r_m gate) * (r_m up) in bf16: the
//             MLP's activation without a launch of its own.
//             (both: r_m = 1 unless the input rows were left unscaled by an EPI_RESID launch, whose sums of squares
//             then give r_m = rsqrt(mean(x_m^2) + eps))
//   EPI_RESID one slice: x[m, n] += sum (the residual stream, fp32); act[m, n] = bf16(x[m, n] * gain[n]), the next
//             product's input WITHOUT the RMSNorm factor of its row (a per-row scalar commutes with the product, so
//             the consumer applies it to its sums); ssq_out[m][workgroup] = sum of x[m, n]^2 over the workgroup's
//             columns, added by the consumer in workgroup order.  Residual + RMSNorm without a launch of their own.
//   EPI_ROPE  W = [q; k; v] rows of a decoder layer, head dimension 2^(hshift+1).  The row ranges walk the rows in
//             the order (head, i, half): local index j stands for row (j/2 / half) hd + (j/2 % half) + (j%2) half,
//             so the two sums of a rotary pair (i, i + hd/2) sit side by side in one wavefront's tile, and the sweep
//             rotates them at the row's position and writes q (bf16 [M, Hq hd]), the key cache row and the
//             (transposed) value cache column itself: no launch of its own for the rotary embedding and the KV append.
//   EPI_HEAD  one slice: act[m, n] = bf16(silu(sum + bias[n]) (+ z_in[z_rows ? z_rows[m] : m][n] when z_in is set)): a
//             hidden layer of the acceptance head (Sec. 4.2: a small ResNet with SiLU) without a launch of its own
//             for the bias, the activation and the skip connection.
enum { EPI_PART = 0, EPI_SILU = 1, EPI_RESID = 2, EPI_ROPE = 3, EPI_HEAD = 4 };
struct StripeEpi {
  bf16_t* act;             // SILU / RESID / HEAD output [M][N]
  float* x;                // RESID: residual rows [M][N], updated in place
  const bf16_t* gain;      // RESID: [N]
  float* ssq_out;          // RESID: [M][gridDim.x]
  const float* ssq_in;     // PART / SILU: [M][ssq_n] or null
  int ssq_n;
  float inv_d, eps;        // 1 / (length of the input rows whose squares ssq_in sums), RMSNorm epsilon
  // ROPE
  const int32_t* row_seq;  // [M] sequence of the row, < 0 = padding row (nothing written)
  const int32_t* row_pos;  // [M] position of the row's token
  const float* cos_sin;    // [max_seq][hd / 2][2]
  bf16_t* qbuf;            // [M][Hq * hd]
  bf16_t* kcache;          // [seq][Hkv][max_seq][hd]
  bf16_t* vcache;          // [seq][Hkv][hd][max_seq]
  int Hq, Hkv, hshift, max_seq;
  // HEAD
  const bf16_t* bias;      // [N]
  const bf16_t* z_in;      // skip connection rows [.][N] (N = K) or null
  const int32_t* z_rows;   // [M] row of z_in for activation row m, or null (row m)
};

typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2;

__device__ __forceinline__ float dot8(const uint4& w, const uint4& x, float c) {
  union { uint32_t u; bf16x2 v; } a, b;
  a.u = w.x; b.u = x.x; c = __builtin_amdgcn_fdot2_f32_bf16(a.v, b.v, c, false);
  a.u = w.y; b.u = x.y; c = __builtin_amdgcn_fdot2_f32_bf16(a.v, b.v, c, false);
  a.u = w.z; b.u = x.z; c = __builtin_amdgcn_fdot2_f32_bf16(a.v, b.v, c, false);
  a.u = w.w; b.u = x.w; c = __builtin_amdgcn_fdot2_f32_bf16(a.v, b.v, c, false);
  return c;
}

// Cross-lane sums without the LDS crossbar.  v_permlane32_swap (a, b) returns {a with its upper 32 lanes replaced
// by b's lower 32, b with its lower 32 lanes replaced by a's upper 32}; v_permlane16_swap does the same with the
// odd 16-lane rows of a and the even rows of b.  So for a pair of per-lane values (lo, hi), r = swap(lo, hi) and
// r[0] + r[1] leaves, in the lanes whose OFF bit is clear, their own lo plus the partner's (lane ^ OFF) lo, and in
// the lanes whose bit is set, their own hi plus the partner's hi: one exchange of a transposing butterfly.
template <int OFF>
__device__ __forceinline__ float swap_add(float lo, float hi) {
  static_assert(OFF == 32 || OFF == 16, "row-crossing exchanges");
  if constexpr (OFF == 32) {
    const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(lo), __float_as_uint(hi), false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
  } else {
    const auto r = __builtin_amdgcn_permlane16_swap(__float_as_uint(lo), __float_as_uint(hi), false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
  }
}

template <int CTRL>
__device__ __forceinline__ float dpp_move(float v) {
  return __uint_as_float((uint32_t)__builtin_amdgcn_update_dpp(0, (int)__float_as_uint(v), CTRL, 0xF, 0xF, false));
}
constexpr int DPP_QUAD_XOR1 = 0xB1, DPP_QUAD_XOR2 = 0x4E, DPP_HALF_MIRROR = 0x141, DPP_ROR8 = 0x128;

// N sums per lane become N / 2; lanes with bit OFF set keep the upper half.
template <int N, int OFF>
__device__ __forceinline__ void fold_stage(float* acc, int lane) {
  constexpr int H = N / 2;
  if constexpr (OFF >= 16) {
#pragma unroll
    for (int k = 0; k < H; ++k) acc[k] = swap_add<OFF>(acc[k], acc[k + H]);
  } else {
    static_assert(OFF == 8, "inside a 16-lane row only the 8-lane exchange is used");
    const bool hi = (lane & 8) != 0;
#pragma unroll
    for (int k = 0; k < H; ++k) {
      const float keep = hi ? acc[k + H] : acc[k];
      const float send = hi ? acc[k] : acc[k + H];
      acc[k] = keep + dpp_move<DPP_ROR8>(send);
    }
  }
}

// Sums P2 (a power of two <= 8) per-lane values over the 64 lanes; lane l ends with the total of value l / (64 / P2).
template <int P2>
__device__ __forceinline__ float reduce_lanes(float* acc, int lane) {
  static_assert(P2 == 1 || P2 == 2 || P2 == 4 || P2 == 8, "power of two");
  if constexpr (P2 == 8) { fold_stage<8, 32>(acc, lane); fold_stage<4, 16>(acc, lane); fold_stage<2, 8>(acc, lane); }
  if constexpr (P2 == 4) { fold_stage<4, 32>(acc, lane); fold_stage<2, 16>(acc, lane); }
  if constexpr (P2 == 2) { fold_stage<2, 32>(acc, lane); }
  float v = acc[0];
  if constexpr (P2 <= 1) v = swap_add<32>(v, v);
  if constexpr (P2 <= 2) v = swap_add<16>(v, v);
  if constexpr (P2 <= 4) v += dpp_move<DPP_ROR8>(v);
  v += dpp_move<DPP_QUAD_XOR1>(v);
  v += dpp_move<DPP_QUAD_XOR2>(v);
  v += dpp_move<DPP_HALF_MIRROR>(v);
  return v;
}

constexpr int STRIPE_SSQ_PER_LANE = 4;      // a consumer adds at most 4 * 64 = 256 per-workgroup sums of squares per row

// The RMSNorm factors of the input rows come from the producer's per-workgroup sums of squares (at most 256 per
// row).  Wavefront w takes rows w, w + nw, ..: the loads go out first of all (before the weight stream starts)
// and are added after it, in a fixed order (four per lane, then the butterfly).
template <int U>
__device__ __forceinline__ void stripe_load_ssq(const StripeEpi& epi, int M, float (*sq)[STRIPE_SSQ_PER_LANE]) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nw = blockDim.x >> 6;
#pragma unroll
  for (int u = 0; u < U; ++u) {
#pragma unroll
    for (int i = 0; i < STRIPE_SSQ_PER_LANE; ++i) sq[u][i] = 0.f;
    if (epi.ssq_in) {
      const int m = min(wave + u * nw, M - 1);
#pragma unroll
      for (int i = 0; i < STRIPE_SSQ_PER_LANE; ++i) {
        const int idx = lane + WAVE * i;
        sq[u][i] = idx < epi.ssq_n ? epi.ssq_in[m * epi.ssq_n + idx] : 0.f;
      }
    }
  }
}

// s_scale: LDS, at least M floats.  Contains the barrier that separates the wavefronts' tile writes from the sweep.
template <int EPI, int U>
__device__ __forceinline__ void stripe_finish(const float* obuf, float* s_scale, const float (*sq)[STRIPE_SSQ_PER_LANE],
                                              float* __restrict__ part, const StripeEpi& epi, int M, int N, int cs,
                                              int rpg, int ranges, int rpw) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  if constexpr (EPI != EPI_RESID) {
    const int nw = blockDim.x >> 6;
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int m = wave + u * nw;
      const float t = wave_sum((sq[u][0] + sq[u][1]) + (sq[u][2] + sq[u][3]));
      if (m < M && lane == 0) s_scale[m] = epi.ssq_in ? 1.0f / sqrtf(t * epi.inv_d + epi.eps) : 1.0f;
    }
  }
  __syncthreads();
  // stripe tiles of one row range are added in stripe order
  const int tile = M * rpw;
  if constexpr (EPI == EPI_SILU) {
    for (int idx = threadIdx.x; idx < (rpg >> 1) * tile; idx += blockDim.x) {
      const int l = idx / tile, rem = idx - l * tile;
      const int m = rem / rpw, r = rem - m * rpw;
      const int g = blockIdx.x * (rpg >> 1) + l;
      if (g >= ranges || g * rpw + r >= N) continue;
      const float* sg = obuf + (size_t)(2 * l) * cs * tile + rem;
      const float* su = sg + (size_t)cs * tile;
      // both in stripe order (stripe t of `up` sits in the tile of local wavefront t - 1)
      float gate = sg[0], up = su[(size_t)(cs - 1) * tile];
      for (int t = 1; t < cs; ++t) {
        gate += sg[(size_t)t * tile];
        up += su[(size_t)(t - 1) * tile];
      }
      const float rm = s_scale[m];
      gate *= rm;
      up *= rm;
      epi.act[(size_t)m * N + g * rpw + r] = f2bf(gate / (1.0f + expf(-gate)) * up);
    }
  } else if constexpr (EPI == EPI_ROPE) {
    const int hw = rpw >> 1, hs = epi.hshift, half = 1 << hs, hd = 2 << hs;
    for (int idx = threadIdx.x; idx < rpg * M * hw; idx += blockDim.x) {
      const int l = idx / (M * hw), rem = idx - l * (M * hw);
      const int m = rem / hw, q = rem - m * hw;
      const int g = blockIdx.x * rpg + l;
      const int j = g * rpw + 2 * q;                   // local index of the pair's first row
      if (g >= ranges || j >= N) continue;
      const int seq = epi.row_seq[m];
      if (seq < 0) continue;
      const int pos = epi.row_pos[m];
      const float* src = obuf + (size_t)l * cs * tile + m * rpw + 2 * q;
      float a = src[0], b = src[1];
      for (int t = 1; t < cs; ++t) {
        a += src[(size_t)t * tile];
        b += src[(size_t)t * tile + 1];
      }
      a *= s_scale[m];
      b *= s_scale[m];
      const int p = j >> 1, slot = p >> hs, i = p & (half - 1);
      if (slot < epi.Hq + epi.Hkv) {
        const float* cs2 = epi.cos_sin + ((size_t)pos * half + i) * 2;
        float ra, rb;
        rope_pair(a, b, cs2[0], cs2[1], ra, rb);
        bf16_t* dst = slot < epi.Hq
                          ? epi.qbuf + ((size_t)m * epi.Hq + slot) * hd + i
                          : epi.kcache + (((size_t)seq * epi.Hkv + (slot - epi.Hq)) * epi.max_seq + pos) * hd + i;
        dst[0] = f2bf(ra);
        dst[half] = f2bf(rb);
      } else {
        bf16_t* v = epi.vcache + ((size_t)seq * epi.Hkv + (slot - epi.Hq - epi.Hkv)) * hd * (size_t)epi.max_seq + pos;
        v[(size_t)i * epi.max_seq] = f2bf(a);
        v[(size_t)(i + half) * epi.max_seq] = f2bf(b);
      }
    }
  } else if constexpr (EPI == EPI_RESID) {
    // wavefront w takes activation rows w, w + (wavefronts), ...: a row's sum of squares stays inside one wavefront
    const int nw = blockDim.x >> 6;
    for (int m = wave; m < M; m += nw) {
      float ssq = 0.f;
      for (int e = lane; e < rpg * rpw; e += WAVE) {
        const int l = e / rpw, r = e - l * rpw;
        const int g = blockIdx.x * rpg + l;
        const int n = g * rpw + r;
        if (g >= ranges || n >= N) continue;
        const float* src = obuf + (size_t)l * cs * tile + m * rpw + r;
        float sum = src[0];
        for (int t = 1; t < cs; ++t) sum += src[(size_t)t * tile];
        const float xv = epi.x[(size_t)m * N + n] + sum;
        epi.x[(size_t)m * N + n] = xv;
        epi.act[(size_t)m * N + n] = f2bf(xv * bf2f(epi.gain[n]));
        ssq += xv * xv;
      }
      ssq = wave_sum(ssq);
      if (lane == 0) epi.ssq_out[m * gridDim.x + blockIdx.x] = ssq;
    }
  } else if constexpr (EPI == EPI_HEAD) {
    for (int idx = threadIdx.x; idx < rpg * tile; idx += blockDim.x) {
      const int l = idx / tile, rem = idx - l * tile;
      const int m = rem / rpw, r = rem - m * rpw;
      const int g = blockIdx.x * rpg + l;
      const int n = g * rpw + r;
      if (g >= ranges || n >= N) continue;
      const float* src = obuf + (size_t)l * cs * tile + rem;
      float sum = src[0];
      for (int t = 1; t < cs; ++t) sum += src[(size_t)t * tile];
      float a = bf2f(epi.bias[n]) + sum;
      a = a / (1.0f + expf(-a));
      if (epi.z_in) a += bf2f(epi.z_in[(size_t)(epi.z_rows ? epi.z_rows[m] : m) * N + n]);
      epi.act[(size_t)m * N + n] = f2bf(a);
    }
  } else {
    for (int idx = threadIdx.x; idx < rpg * tile; idx += blockDim.x) {
      const int l = idx / tile, rem = idx - l * tile;
      const int m = rem / rpw, r = rem - m * rpw;
      const int g = blockIdx.x * rpg + l;
      if (g >= ranges || g * rpw + r >= N) continue;
      const float* src = obuf + (size_t)l * cs * tile + rem;
      float sum = src[0];
      for (int t = 1; t < cs; ++t) sum += src[(size_t)t * tile];
      part[(size_t)m * N + g * rpw + r] = sum * s_scale[m];      // s_scale = 1 unless the input rows lack their norm factor
    }
  }
}

// The 9 .. 17-row member of the family (gemm_mstripe.hip): matrix-core products on LDS-transposed half tiles.
// epi_kind = the EPI_* of the sweep.  mstripe_groups: workgroups of the launch (EPI_RESID writes one sum of squares
// per row and workgroup), 0 where the kernel does not apply.
bool mstripe_ok(int M, int N, int K, int epi_kind);
int mstripe_groups(int M, int N, int K, int epi_kind);
hipError_t launch_mstripe(hipStream_t st, int epi_kind, const void* W, const void* X, int ldx, const int* xrow,
                          float* part, const StripeEpi& epi, int M, int N, int K);

}  // namespace sd
