// Training of the acceptance-prediction head (Sec. 4.4) on the device: forward of the
// (D+1)-layer head over a batch of draft embeddings, the weighted binary cross-entropy
// against the targets P_i = min(1, p/q), its gradient through every layer, and Adam.
// Everything is fp32 (the head is tiny next to the models: three 4096 x 4096 matrices at
// the paper's width, a few GFLOP per step), so one plain LDS-tiled SGEMM with free operand
// strides serves the forward product and both backward products.
#include "common.hpp"
#include "kernels.hpp"
#include "../../include/specdec.h"

#include <algorithm>
#include <cmath>
#include <new>
#include <vector>

namespace sd {

namespace {

constexpr int TS = 64;      // SGEMM tile: 64 x 64 outputs, 16 k per step, 4 x 4 outputs per thread
constexpr int TK = 16;

// C[i, j] = sum_k A(i, k) B(j, k),  A(i, k) = A[i sai + k sak],  B(j, k) = B[j sbj + k sbk]
__global__ __launch_bounds__(256) void sgemm_k(const float* __restrict__ A, long sai, long sak,
                                               const float* __restrict__ B, long sbj, long sbk,
                                               float* __restrict__ C, int ldc, int M, int N, int K) {
  __shared__ float As[TK][TS + 1];
  __shared__ float Bs[TK][TS + 1];
  const int i0 = blockIdx.y * TS, j0 = blockIdx.x * TS;
  const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
  float acc[4][4] = {};
  for (int k0 = 0; k0 < K; k0 += TK) {
    // the unit-stride index runs fastest over the threads
#pragma unroll
    for (int l = 0; l < 4; ++l) {
      const int idx = threadIdx.x + 256 * l;
      int r, k;
      if (sak == 1) { k = idx & 15; r = idx >> 4; } else { r = idx & 63; k = idx >> 6; }
      const int gi = i0 + r, gk = k0 + k;
      As[k][r] = (gi < M && gk < K) ? A[gi * sai + gk * sak] : 0.f;
      if (sbk == 1) { k = idx & 15; r = idx >> 4; } else { r = idx & 63; k = idx >> 6; }
      const int gj = j0 + r, gk2 = k0 + k;
      Bs[k][r] = (gj < N && gk2 < K) ? B[gj * sbj + gk2 * sbk] : 0.f;
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < TK; ++k) {
      float a[4], b[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) { a[u] = As[k][ty * 4 + u]; b[u] = Bs[k][tx * 4 + u]; }
#pragma unroll
      for (int u = 0; u < 4; ++u)
#pragma unroll
        for (int v = 0; v < 4; ++v) acc[u][v] = fmaf(a[u], b[v], acc[u][v]);
    }
    __syncthreads();
  }
#pragma unroll
  for (int u = 0; u < 4; ++u)
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      const int i = i0 + ty * 4 + u, j = j0 + tx * 4 + v;
      if (i < M && j < N) C[(size_t)i * ldc + j] = acc[u][v];
    }
}

__device__ __forceinline__ float silu(float a) { return a / (1.0f + expf(-a)); }
__device__ __forceinline__ float silu_grad(float a) {
  const float s = 1.0f / (1.0f + expf(-a));
  return s * (1.0f + a * (1.0f - s));
}

// pre = C + b (kept for the backward pass); z_out = SiLU(pre) (+ z_in with the skip connection)
__global__ void bias_act_k(float* __restrict__ pre, const float* __restrict__ b, const float* __restrict__ z_in,
                           float* __restrict__ z_out, int skip, int n, int width) {
  const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= (size_t)n * width) return;
  const int o = idx % width;
  const float a = pre[idx] + b[o];
  pre[idx] = a;
  z_out[idx] = silu(a) + (skip ? z_in[idx] : 0.f);
}

// Last layer and loss.  One workgroup per row computes logit_i = z_i . w + b.
__global__ __launch_bounds__(256) void logit_k(const float* __restrict__ z, const float* __restrict__ w,
                                               const float* __restrict__ b, float* __restrict__ logit, int width) {
  __shared__ float red[4];
  const int i = blockIdx.x;
  float acc = 0.f;
  for (int k = threadIdx.x; k < width; k += 256) acc = fmaf(z[(size_t)i * width + k], w[k], acc);
  acc = block_sum(acc, red);
  if (threadIdx.x == 0) logit[i] = acc + b[0];
}

// One workgroup: loss = (1/n_m) sum_i mask_i (-w_acc P_i log s_i - w_rej (1 - P_i) log(1 - s_i)),
// dlogit_i = mask_i (-w_acc P_i (1 - s_i) + w_rej (1 - P_i) s_i) / n_m, gb_last = sum_i dlogit_i.
// out = {loss, n_m, gb_last}.  Fixed summation order.
__global__ __launch_bounds__(1024) void bce_k(const float* __restrict__ logit, const float* __restrict__ P,
                                              const int32_t* __restrict__ mask, int n, float w_acc, float w_rej,
                                              float* __restrict__ dlogit, float* __restrict__ out) {
  __shared__ float red[16];
  float cnt = 0.f;
  for (int i = threadIdx.x; i < n; i += 1024) cnt += mask[i] ? 1.f : 0.f;
  cnt = block_sum(cnt, red);
  const float nm = fmaxf(cnt, 1.f);
  float loss = 0.f, gsum = 0.f;
  for (int i = threadIdx.x; i < n; i += 1024) {
    const float x = logit[i], p = P[i];
    // log sigmoid(x) and log(1 - sigmoid(x)) without overflow
    const float sp = fmaxf(-x, 0.f) + log1pf(expf(-fabsf(x)));       // softplus(-x) = -log s
    const float sn = fmaxf(x, 0.f) + log1pf(expf(-fabsf(x)));        // softplus(x)  = -log(1 - s)
    const float s = 1.0f / (1.0f + expf(-x));
    const float m = mask[i] ? 1.f : 0.f;
    loss += m * (w_acc * p * sp + w_rej * (1.f - p) * sn);
    const float g = m * (-w_acc * p * (1.f - s) + w_rej * (1.f - p) * s) / nm;
    dlogit[i] = g;
    gsum += g;
  }
  loss = block_sum(loss, red);
  gsum = block_sum(gsum, red);
  if (threadIdx.x == 0) {
    out[0] = loss / nm;
    out[1] = cnt;
    out[2] = gsum;
  }
}

// dz[i, k] = dlogit_i w[k]; gw[k] = sum_i dlogit_i z[i, k]  (one thread per k, rows in order)
__global__ void last_back_k(const float* __restrict__ dlogit, const float* __restrict__ w, const float* __restrict__ z,
                            float* __restrict__ dz, float* __restrict__ gw, int n, int width) {
  const int k = blockIdx.x * blockDim.x + threadIdx.x;
  if (k >= width) return;
  const float wk = w[k];
  float g = 0.f;
  for (int i = 0; i < n; ++i) {
    const float dl = dlogit[i];
    dz[(size_t)i * width + k] = dl * wk;
    g = fmaf(dl, z[(size_t)i * width + k], g);
  }
  gw[k] = g;
}

// da = dz * SiLU'(pre); gb[o] = sum_i da[i, o]   (one thread per column o, rows in order)
__global__ void act_back_k(const float* __restrict__ dz, const float* __restrict__ pre, float* __restrict__ da,
                           float* __restrict__ gb, int n, int width) {
  const int o = blockIdx.x * blockDim.x + threadIdx.x;
  if (o >= width) return;
  float g = 0.f;
  for (int i = 0; i < n; ++i) {
    const size_t idx = (size_t)i * width + o;
    const float v = dz[idx] * silu_grad(pre[idx]);
    da[idx] = v;
    g += v;
  }
  gb[o] = g;
}

__global__ void add_k(float* __restrict__ y, const float* __restrict__ x, size_t n) {
  const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx < n) y[idx] += x[idx];
}

__global__ void adam_k(float* __restrict__ p, const float* __restrict__ g, float* __restrict__ m, float* __restrict__ v,
                       size_t n, float lr, float b1, float b2, float eps, float c1, float c2) {
  const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= n) return;
  const float gi = g[idx];
  const float mi = b1 * m[idx] + (1.f - b1) * gi;
  const float vi = b2 * v[idx] + (1.f - b2) * gi * gi;
  m[idx] = mi;
  v[idx] = vi;
  p[idx] -= lr * (mi / c1) / (sqrtf(vi / c2) + eps);
}

__global__ void to_bf16_k(const float* __restrict__ x, bf16_t* __restrict__ y, size_t n) {
  const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx < n) y[idx] = f2bf(x[idx]);
}
__global__ void from_bf16_k(const bf16_t* __restrict__ x, float* __restrict__ y, size_t n) {
  const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx < n) y[idx] = bf2f(x[idx]);
}

inline dim3 grid1(size_t n, int b = 256) { return dim3((unsigned)((n + b - 1) / b)); }

void sgemm(hipStream_t st, const float* A, long sai, long sak, const float* B, long sbj, long sbk, float* C, int ldc,
           int M, int N, int K) {
  hipLaunchKernelGGL(sgemm_k, dim3((N + TS - 1) / TS, (M + TS - 1) / TS), dim3(256), 0, st, A, sai, sak, B, sbj, sbk, C,
                     ldc, M, N, K);
}

}  // namespace

hipError_t launch_to_f32(hipStream_t st, int dtype, const void* x, float* y, size_t n) {
  if (!x || !y || n < 1) return hipErrorInvalidValue;
  if (dtype == DT_F32) return hipMemcpyAsync(y, x, n * 4, hipMemcpyDeviceToDevice, st);
  if (dtype != DT_BF16) return hipErrorInvalidValue;
  hipLaunchKernelGGL(from_bf16_k, grid1(n), dim3(256), 0, st, (const bf16_t*)x, y, n);
  return hipGetLastError();
}

}  // namespace sd

using namespace sd;

struct sd_trainer {
  hipStream_t st = nullptr;
  int n_layers = 0, residual = 0, n_max = 0;
  std::vector<int> dims;
  std::vector<float*> W, b, gW, gb, mW, vW, mb, vb;   // per layer
  std::vector<float*> z, pre;                         // z[j]: input of layer j [n_max, dims[j]]; pre[j]: [n_max, dims[j+1]]
  float *da = nullptr, *dz = nullptr, *dz2 = nullptr, *logit = nullptr, *dlogit = nullptr, *out3 = nullptr;
  int64_t t = 0;
  std::vector<void*> allocs;
};

namespace {

bool talloc(sd_trainer* t, float** p, size_t floats) {
  void* q = nullptr;
  if (hipMalloc(&q, std::max<size_t>(floats, 4) * 4) != hipSuccess) { (void)hipGetLastError(); return false; }
  if (hipMemsetAsync(q, 0, std::max<size_t>(floats, 4) * 4, t->st) != hipSuccess) return false;
  t->allocs.push_back(q);
  *p = (float*)q;
  return true;
}

bool skip_layer(const sd_trainer* t, int j) { return t->residual && t->dims[j] == t->dims[j + 1]; }

// forward over n rows already in t->z[0]; leaves logits in t->logit
void head_forward(sd_trainer* t, int n) {
  const int L = t->n_layers;
  for (int j = 0; j + 1 < L; ++j) {
    const int K = t->dims[j], N = t->dims[j + 1];
    sgemm(t->st, t->z[j], K, 1, t->W[j], K, 1, t->pre[j], N, n, N, K);
    hipLaunchKernelGGL(bias_act_k, grid1((size_t)n * N), dim3(256), 0, t->st, t->pre[j], t->b[j], t->z[j], t->z[j + 1],
                       skip_layer(t, j) ? 1 : 0, n, N);
  }
  hipLaunchKernelGGL(logit_k, dim3(n), dim3(256), 0, t->st, t->z[L - 1], t->W[L - 1], t->b[L - 1], t->logit,
                     t->dims[L - 1]);
}

}  // namespace

#pragma GCC visibility push(default)
extern "C" {

sd_status sd_trainer_destroy(sd_trainer* t) {
  if (!t) return SD_EINVAL;
  (void)hipStreamSynchronize(t->st);
  for (void* p : t->allocs) (void)hipFree(p);
  delete t;
  return SD_OK;
}

sd_status sd_trainer_create(sd_trainer** out, const sd_head* init, int32_t n_max, void* hip_stream) {
  if (!out || !init || init->n_layers < 1 || init->n_layers > 16 || n_max < 1 || n_max > 4096 || !init->dims || !init->W ||
      !init->b || (init->dtype != SD_F32 && init->dtype != SD_BF16))
    return SD_EINVAL;
  const int L = init->n_layers;
  if (init->dims[L] != 1) return SD_EINVAL;
  for (int j = 0; j <= L; ++j)
    if (init->dims[j] < 1) return SD_EINVAL;
  sd_trainer* t = new (std::nothrow) sd_trainer();
  if (!t) return SD_ENOMEM;
  t->st = (hipStream_t)hip_stream;
  t->n_layers = L;
  t->residual = init->residual;
  t->n_max = n_max;
  t->dims.assign(init->dims, init->dims + L + 1);
  auto fail = [&](sd_status e) { sd_trainer_destroy(t); return e; };
  int wmax = 1;
  for (int j = 0; j <= L; ++j) wmax = std::max(wmax, t->dims[j]);
  for (auto* v : {&t->W, &t->b, &t->gW, &t->gb, &t->mW, &t->vW, &t->mb, &t->vb, &t->pre}) v->assign(L, nullptr);
  t->z.assign(L, nullptr);
  for (int j = 0; j < L; ++j) {
    const size_t nw = (size_t)t->dims[j + 1] * t->dims[j], nb = t->dims[j + 1];
    if (!talloc(t, &t->W[j], nw) || !talloc(t, &t->gW[j], nw) || !talloc(t, &t->mW[j], nw) || !talloc(t, &t->vW[j], nw) ||
        !talloc(t, &t->b[j], nb) || !talloc(t, &t->gb[j], nb) || !talloc(t, &t->mb[j], nb) || !talloc(t, &t->vb[j], nb) ||
        !talloc(t, &t->z[j], (size_t)n_max * t->dims[j]) || !talloc(t, &t->pre[j], (size_t)n_max * t->dims[j + 1]))
      return fail(SD_ENOMEM);
    if (launch_to_f32(t->st, init->dtype, init->W[j], t->W[j], nw) != hipSuccess ||
        launch_to_f32(t->st, init->dtype, init->b[j], t->b[j], nb) != hipSuccess)
      return fail(SD_EDEVICE);
  }
  if (!talloc(t, &t->da, (size_t)n_max * wmax) || !talloc(t, &t->dz, (size_t)n_max * wmax) ||
      !talloc(t, &t->dz2, (size_t)n_max * wmax) || !talloc(t, &t->logit, n_max) || !talloc(t, &t->dlogit, n_max) ||
      !talloc(t, &t->out3, 4))
    return fail(SD_ENOMEM);
  if (hipStreamSynchronize(t->st) != hipSuccess) return fail(SD_EDEVICE);
  *out = t;
  return SD_OK;
}

sd_status sd_trainer_step(sd_trainer* t, const float* E, const float* P, const int32_t* mask, int32_t n, float w_acc,
                          float w_rej, float lr, float beta1, float beta2, float eps, int32_t apply, float* loss_host) {
  if (!t || !E || !P || !mask || n < 1 || n > t->n_max || !(w_acc >= 0.f) || !(w_rej >= 0.f) || !(lr >= 0.f) ||
      !(beta1 >= 0.f && beta1 < 1.f) || !(beta2 >= 0.f && beta2 < 1.f) || !(eps > 0.f))
    return SD_EINVAL;
  hipStream_t st = t->st;
  const int L = t->n_layers;
#define TR_HIP(x) do { if ((x) != hipSuccess) { (void)hipGetLastError(); return SD_EDEVICE; } } while (0)
  TR_HIP(hipMemcpyAsync(t->z[0], E, (size_t)n * t->dims[0] * 4, hipMemcpyDeviceToDevice, st));
  head_forward(t, n);
  hipLaunchKernelGGL(bce_k, dim3(1), dim3(1024), 0, st, t->logit, P, mask, n, w_acc, w_rej, t->dlogit, t->out3);
  // last layer: gW, gb, and the gradient flowing into its input
  const int wl = t->dims[L - 1];
  hipLaunchKernelGGL(last_back_k, grid1(wl), dim3(256), 0, st, t->dlogit, t->W[L - 1], t->z[L - 1], t->dz, t->gW[L - 1], n,
                     wl);
  TR_HIP(hipMemcpyAsync(t->gb[L - 1], t->out3 + 2, 4, hipMemcpyDeviceToDevice, st));
  float* dz = t->dz;
  float* dz_other = t->dz2;
  for (int j = L - 2; j >= 0; --j) {
    const int K = t->dims[j], N = t->dims[j + 1];
    hipLaunchKernelGGL(act_back_k, grid1(N), dim3(256), 0, st, dz, t->pre[j], t->da, t->gb[j], n, N);
    // gW[o, k] = sum_i da[i, o] z[i, k]
    sgemm(st, t->da, 1, N, t->z[j], 1, K, t->gW[j], K, N, K, n);
    if (j > 0) {                                   // the gradient of the embeddings is not needed
      // dz_in[i, k] = sum_o da[i, o] W[o, k]  (+ dz with the skip connection)
      sgemm(st, t->da, N, 1, t->W[j], 1, K, dz_other, K, n, K, N);
      if (skip_layer(t, j)) hipLaunchKernelGGL(add_k, grid1((size_t)n * K), dim3(256), 0, st, dz_other, dz, (size_t)n * K);
      std::swap(dz, dz_other);
    }
  }
  TR_HIP(hipGetLastError());
  if (apply) {
    t->t += 1;
    const float c1 = 1.0f - (float)std::pow((double)beta1, (double)t->t);
    const float c2 = 1.0f - (float)std::pow((double)beta2, (double)t->t);
    for (int j = 0; j < L; ++j) {
      const size_t nw = (size_t)t->dims[j + 1] * t->dims[j], nb = t->dims[j + 1];
      hipLaunchKernelGGL(adam_k, grid1(nw), dim3(256), 0, st, t->W[j], t->gW[j], t->mW[j], t->vW[j], nw, lr, beta1, beta2,
                         eps, c1, c2);
      hipLaunchKernelGGL(adam_k, grid1(nb), dim3(256), 0, st, t->b[j], t->gb[j], t->mb[j], t->vb[j], nb, lr, beta1, beta2,
                         eps, c1, c2);
    }
    TR_HIP(hipGetLastError());
  }
  if (loss_host) {
    TR_HIP(hipMemcpyAsync(loss_host, t->out3, 4, hipMemcpyDeviceToHost, st));
    TR_HIP(hipStreamSynchronize(st));
  }
#undef TR_HIP
  return SD_OK;
}

sd_status sd_trainer_predict(sd_trainer* t, const float* E, int32_t n, float* logits_dev) {
  if (!t || !E || !logits_dev || n < 1 || n > t->n_max) return SD_EINVAL;
  if (hipMemcpyAsync(t->z[0], E, (size_t)n * t->dims[0] * 4, hipMemcpyDeviceToDevice, t->st) != hipSuccess)
    return SD_EDEVICE;
  head_forward(t, n);
  if (hipMemcpyAsync(logits_dev, t->logit, (size_t)n * 4, hipMemcpyDeviceToDevice, t->st) != hipSuccess)
    return SD_EDEVICE;
  return hipGetLastError() == hipSuccess ? SD_OK : SD_EDEVICE;
}

sd_status sd_trainer_read(sd_trainer* t, int32_t layer, int32_t what, float* host) {
  if (!t || !host || layer < 0 || layer >= t->n_layers || what < 0 || what > 3) return SD_EINVAL;
  const size_t nw = (size_t)t->dims[layer + 1] * t->dims[layer], nb = t->dims[layer + 1];
  const float* src = what == 0 ? t->W[layer] : what == 1 ? t->b[layer] : what == 2 ? t->gW[layer] : t->gb[layer];
  const size_t n = (what == 0 || what == 2) ? nw : nb;
  if (hipStreamSynchronize(t->st) != hipSuccess) return SD_EDEVICE;
  if (hipMemcpy(host, src, n * 4, hipMemcpyDeviceToHost) != hipSuccess) return SD_EDEVICE;
  return SD_OK;
}

sd_status sd_trainer_export(sd_trainer* t, int32_t dtype, void* const* W_out, void* const* b_out) {
  if (!t || !W_out || !b_out || (dtype != SD_F32 && dtype != SD_BF16)) return SD_EINVAL;
  for (int j = 0; j < t->n_layers; ++j) {
    const size_t nw = (size_t)t->dims[j + 1] * t->dims[j], nb = t->dims[j + 1];
    if (!W_out[j] || !b_out[j]) return SD_EINVAL;
    if (dtype == SD_F32) {
      if (hipMemcpyAsync(W_out[j], t->W[j], nw * 4, hipMemcpyDeviceToDevice, t->st) != hipSuccess ||
          hipMemcpyAsync(b_out[j], t->b[j], nb * 4, hipMemcpyDeviceToDevice, t->st) != hipSuccess)
        return SD_EDEVICE;
    } else {
      hipLaunchKernelGGL(to_bf16_k, grid1(nw), dim3(256), 0, t->st, t->W[j], (bf16_t*)W_out[j], nw);
      hipLaunchKernelGGL(to_bf16_k, grid1(nb), dim3(256), 0, t->st, t->b[j], (bf16_t*)b_out[j], nb);
    }
  }
  if (hipStreamSynchronize(t->st) != hipSuccess) return SD_EDEVICE;
  return hipGetLastError() == hipSuccess ? SD_OK : SD_EDEVICE;
}

}  // extern "C"
#pragma GCC visibility pop
