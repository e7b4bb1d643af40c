// Fused in-place parameter updates: momentum-SGD and Adam.
//
// Momentum-SGD (paper, Algorithm 1: theta <- theta - eta * gradient; heavy-ball
// momentum in the form of the large-minibatch recipe the paper follows, Section 4.1):
//     g = grad + wd * w;  v = mu * v + g;  w -= lr * (nesterov ? g + mu * v : v)
// HBM-bound: 12 bytes read and 8 (+2 for the bf16 copy) written per parameter.
#include "common.h"
#include <math.h>

namespace cd {

template <bool LOWP>
__global__ void __launch_bounds__(256) sgd_kernel(float* __restrict__ w, float* __restrict__ v,
                                                  const float* __restrict__ g, bf16_t* __restrict__ lp, int64_t n,
                                                  float lr, float mu, float wd, int nesterov) {
  const int64_t n4 = n >> 2;
  const int64_t stride = (int64_t)gridDim.x * 256;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n4; i += stride) {
    float4 W = reinterpret_cast<float4*>(w)[i];
    float4 V = reinterpret_cast<float4*>(v)[i];
    const float4 G = reinterpret_cast<const float4*>(g)[i];
    float wv[4] = {W.x, W.y, W.z, W.w}, vv[4] = {V.x, V.y, V.z, V.w};
    const float gv[4] = {G.x, G.y, G.z, G.w};
#pragma unroll
    for (int k = 0; k < 4; k++) {
      const float gg = gv[k] + wd * wv[k];
      vv[k] = mu * vv[k] + gg;
      wv[k] -= lr * (nesterov ? gg + mu * vv[k] : vv[k]);
    }
    reinterpret_cast<float4*>(w)[i] = make_float4(wv[0], wv[1], wv[2], wv[3]);
    reinterpret_cast<float4*>(v)[i] = make_float4(vv[0], vv[1], vv[2], vv[3]);
    if (LOWP) {
      ushort4 o;
      o.x = f32_to_bf16(wv[0]); o.y = f32_to_bf16(wv[1]); o.z = f32_to_bf16(wv[2]); o.w = f32_to_bf16(wv[3]);
      reinterpret_cast<ushort4*>(lp)[i] = o;
    }
  }
  // ragged tail (n not a multiple of 4)
  if (blockIdx.x == 0 && threadIdx.x < (n & 3)) {
    const int64_t i = (n4 << 2) + threadIdx.x;
    const float gg = g[i] + wd * w[i];
    const float vn = mu * v[i] + gg;
    const float wn = w[i] - lr * (nesterov ? gg + mu * vn : vn);
    v[i] = vn;
    w[i] = wn;
    if (LOWP) lp[i] = f32_to_bf16(wn);
  }
}

// Adam (Kingma & Ba), the optimiser of the translation recipe the paper follows (Section 4):
//     g = grad + wd * w;  m = b1 m + (1 - b1) g;  v = b2 v + (1 - b2) g^2;
//     w -= lr * (m / c1) / (sqrt(v / c2) + eps),  c1 = 1 - b1^t, c2 = 1 - b2^t (computed on the host in double)
// The kernel takes step = lr / c1 and rs = 1 / sqrt(c2).  16 bytes read and 12 (+2) written per parameter.
__device__ inline void adam_one(float& w, float& m, float& v, float g, float b1, float b2, float step, float rs,
                                float eps, float wd) {
  const float gg = g + wd * w;
  m = b1 * m + (1.f - b1) * gg;
  v = b2 * v + (1.f - b2) * gg * gg;
  w -= step * m / (sqrtf(v) * rs + eps);
}

template <bool LOWP>
__global__ void __launch_bounds__(256) adam_kernel(float* __restrict__ w, float* __restrict__ m, float* __restrict__ v,
                                                   const float* __restrict__ g, bf16_t* __restrict__ lp, int64_t n,
                                                   float b1, float b2, float step, float rs, float eps, float wd) {
  const int64_t n4 = n >> 2;
  const int64_t stride = (int64_t)gridDim.x * 256;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n4; i += stride) {
    const float4 W = reinterpret_cast<float4*>(w)[i], M = reinterpret_cast<float4*>(m)[i];
    const float4 V = reinterpret_cast<float4*>(v)[i], G = reinterpret_cast<const float4*>(g)[i];
    float wv[4] = {W.x, W.y, W.z, W.w}, mv[4] = {M.x, M.y, M.z, M.w}, vv[4] = {V.x, V.y, V.z, V.w};
    const float gv[4] = {G.x, G.y, G.z, G.w};
#pragma unroll
    for (int k = 0; k < 4; k++) adam_one(wv[k], mv[k], vv[k], gv[k], b1, b2, step, rs, eps, wd);
    reinterpret_cast<float4*>(w)[i] = make_float4(wv[0], wv[1], wv[2], wv[3]);
    reinterpret_cast<float4*>(m)[i] = make_float4(mv[0], mv[1], mv[2], mv[3]);
    reinterpret_cast<float4*>(v)[i] = make_float4(vv[0], vv[1], vv[2], vv[3]);
    if (LOWP) {
      ushort4 o;
      o.x = f32_to_bf16(wv[0]); o.y = f32_to_bf16(wv[1]); o.z = f32_to_bf16(wv[2]); o.w = f32_to_bf16(wv[3]);
      reinterpret_cast<ushort4*>(lp)[i] = o;
    }
  }
  if (blockIdx.x == 0 && threadIdx.x < (n & 3)) {  // ragged tail
    const int64_t i = (n4 << 2) + threadIdx.x;
    float wn = w[i], mn = m[i], vn = v[i];
    adam_one(wn, mn, vn, g[i], b1, b2, step, rs, eps, wd);
    w[i] = wn; m[i] = mn; v[i] = vn;
    if (LOWP) lp[i] = f32_to_bf16(wn);
  }
}

}  // namespace cd

using namespace cd;

extern "C" int codistill_sgd_step(float* master_w, float* momentum_v, const float* grad, void* lowp_w_out, int64_t n,
                                  float lr, float momentum, float weight_decay, int nesterov, void* stream) {
  CD_REQUIRE(master_w && momentum_v && grad, "sgd_step: NULL pointer argument");
  CD_REQUIRE(n >= 1, "sgd_step: n=%lld must be positive", (long long)n);
  CD_REQUIRE(aligned16(master_w) && aligned16(momentum_v) && aligned16(grad) &&
                 (reinterpret_cast<uintptr_t>(lowp_w_out) & 7) == 0,
             "sgd_step: fp32 pointers must be 16-byte aligned, the bf16 pointer 8-byte aligned");
  CD_REQUIRE(lr == lr && momentum == momentum && weight_decay == weight_decay, "sgd_step: NaN hyper-parameter");
  hipStream_t s = static_cast<hipStream_t>(stream);
  const int64_t n4 = n >> 2;
  int64_t blocks = cdiv(n4 > 0 ? n4 : 1, 256);
  if (blocks > 256 * 16) blocks = 256 * 16;
  ProfScope prof(CD_K_SGD, s, 6.0 * n, (lowp_w_out ? 22.0 : 20.0) * n);
  if (lowp_w_out)
    hipLaunchKernelGGL(sgd_kernel<true>, dim3((unsigned)blocks), dim3(256), 0, s, master_w, momentum_v, grad,
                       static_cast<bf16_t*>(lowp_w_out), n, lr, momentum, weight_decay, nesterov);
  else
    hipLaunchKernelGGL(sgd_kernel<false>, dim3((unsigned)blocks), dim3(256), 0, s, master_w, momentum_v, grad,
                       static_cast<bf16_t*>(nullptr), n, lr, momentum, weight_decay, nesterov);
  return check_launch("sgd_step");
}

extern "C" int codistill_adam_step(float* master_w, float* exp_avg, float* exp_avg_sq, const float* grad, void* lowp_w_out,
                                   int64_t n, float lr, float beta1, float beta2, float eps, float weight_decay,
                                   int64_t t, void* stream) {
  CD_REQUIRE(master_w && exp_avg && exp_avg_sq && grad, "adam_step: NULL pointer argument");
  CD_REQUIRE(n >= 1, "adam_step: n=%lld must be positive", (long long)n);
  CD_REQUIRE(t >= 1, "adam_step: the update counter t=%lld starts at 1", (long long)t);
  CD_REQUIRE(aligned16(master_w) && aligned16(exp_avg) && aligned16(exp_avg_sq) && aligned16(grad) &&
                 (reinterpret_cast<uintptr_t>(lowp_w_out) & 7) == 0,
             "adam_step: fp32 pointers must be 16-byte aligned, the bf16 pointer 8-byte aligned");
  CD_REQUIRE(lr == lr && weight_decay == weight_decay && beta1 >= 0.f && beta1 < 1.f && beta2 >= 0.f && beta2 < 1.f &&
                 eps > 0.f,
             "adam_step: need 0 <= beta1, beta2 < 1, eps > 0 and no NaN hyper-parameter");
  hipStream_t s = static_cast<hipStream_t>(stream);
  const double c1 = 1.0 - pow((double)beta1, (double)t), c2 = 1.0 - pow((double)beta2, (double)t);
  const float step = (float)((double)lr / c1), rs = (float)(1.0 / sqrt(c2));
  const int64_t n4 = n >> 2;
  int64_t blocks = cdiv(n4 > 0 ? n4 : 1, 256);
  if (blocks > 256 * 16) blocks = 256 * 16;
  ProfScope prof(CD_K_SGD, s, 12.0 * n, (lowp_w_out ? 30.0 : 28.0) * n);
  if (lowp_w_out)
    hipLaunchKernelGGL(adam_kernel<true>, dim3((unsigned)blocks), dim3(256), 0, s, master_w, exp_avg, exp_avg_sq, grad,
                       static_cast<bf16_t*>(lowp_w_out), n, beta1, beta2, step, rs, eps, weight_decay);
  else
    hipLaunchKernelGGL(adam_kernel<false>, dim3((unsigned)blocks), dim3(256), 0, s, master_w, exp_avg, exp_avg_sq, grad,
                       static_cast<bf16_t*>(nullptr), n, beta1, beta2, step, rs, eps, weight_decay);
  return check_launch("adam_step");
}
