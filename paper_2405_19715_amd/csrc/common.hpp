// Device-side helpers shared by the HIP kernels of the draft-verify-correct round
// (gfx950 only: 64-wide wavefronts, 16x16x32 bf16 MFMA, 160 KB LDS per CU).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace sd {

typedef uint16_t bf16_t;                                   // raw bfloat16 bits in memory
typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float floatx4;

constexpr int WAVE = 64;

__device__ __forceinline__ float bf2f(bf16_t h) { return __uint_as_float(((uint32_t)h) << 16); }

// round-to-nearest-even float -> bfloat16 (NaN stays NaN)
__device__ __forceinline__ bf16_t f2bf(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (bf16_t)0x7fc0;
  u += 0x7fffu + ((u >> 16) & 1u);
  return (bf16_t)(u >> 16);
}

// Element access in the model's storage type.
template <typename T> struct Elem;
template <> struct Elem<float> {
  static __device__ __forceinline__ float ld(const float* p) { return *p; }
  static __device__ __forceinline__ void st(float* p, float v) { *p = v; }
};
template <> struct Elem<bf16_t> {
  static __device__ __forceinline__ float ld(const bf16_t* p) { return bf2f(*p); }
  static __device__ __forceinline__ void st(bf16_t* p, float v) { *p = f2bf(v); }
};

// Rotary embedding of the pair (a, b) = (v[i], v[i + hd/2]) by the angle whose cosine and sine are c and s.  One
// definition with its roundings spelled out, so that every kernel that rotates gives the same bits.
__device__ __forceinline__ void rope_pair(float a, float b, float c, float s, float& ra, float& rb) {
  ra = fmaf(a, c, -__fmul_rn(b, s));
  rb = fmaf(b, c, __fmul_rn(a, s));
}

// Butterfly reductions over the 64 lanes of a wavefront (fixed order, so results
// do not depend on scheduling).
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, WAVE);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, WAVE));
  return v;
}

// Block-wide sum / max through LDS; `red` needs blockDim.x / 64 floats.  Every
// thread gets the result.  Ends with a barrier, so `red` may be reused at once.
__device__ __forceinline__ float block_sum(float v, float* red) {
  v = wave_sum(v);
  const int w = threadIdx.x >> 6, nw = (blockDim.x + 63) >> 6;
  if ((threadIdx.x & 63) == 0) red[w] = v;
  __syncthreads();
  float t = 0.f;
  for (int i = 0; i < nw; ++i) t += red[i];
  __syncthreads();
  return t;
}
__device__ __forceinline__ float block_max(float v, float* red) {
  v = wave_max(v);
  const int w = threadIdx.x >> 6, nw = (blockDim.x + 63) >> 6;
  if ((threadIdx.x & 63) == 0) red[w] = v;
  __syncthreads();
  float t = red[0];
  for (int i = 1; i < nw; ++i) t = fmaxf(t, red[i]);
  __syncthreads();
  return t;
}

// Philox4x32-10 (Salmon et al., SC'11): counter (c0..c3), key (k0,k1) -> word 0.
__device__ __forceinline__ uint32_t philox4x32_10_w0(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                                     uint32_t k0, uint32_t k1) {
  const uint32_t M0 = 0xD2511F53u, M1 = 0xCD9E8D57u, W0 = 0x9E3779B9u, W1 = 0xBB67AE85u;
#pragma unroll
  for (int r = 0; r < 10; ++r) {
    if (r > 0) { k0 += W0; k1 += W1; }
    const uint32_t hi0 = __umulhi(M0, c0), lo0 = M0 * c0;
    const uint32_t hi1 = __umulhi(M1, c2), lo1 = M1 * c2;
    const uint32_t n0 = hi1 ^ c1 ^ k0, n2 = hi0 ^ c3 ^ k1;
    c0 = n0; c1 = lo1; c2 = n2; c3 = lo0;
  }
  return c0;
}

// The round's uniform for (seed, slot, round, sequence, stream): 24 bits in [0,1).
__device__ __forceinline__ float philox_uniform(uint64_t seed, uint32_t slot, uint32_t rnd, uint32_t seq,
                                                uint32_t stream) {
  const uint32_t w = philox4x32_10_w0(slot, rnd, seq, stream, (uint32_t)seed, (uint32_t)(seed >> 32));
  return (float)(w >> 8) * (1.0f / 16777216.0f);
}

enum { STREAM_DRAFT = 0, STREAM_ACCEPT = 1, STREAM_RESAMPLE = 2 };

}  // namespace sd
