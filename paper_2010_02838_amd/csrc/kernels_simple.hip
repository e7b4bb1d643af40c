// Plain layer kernels: one thread per output element, fp32 arithmetic, fp32 or bf16 storage.
// They define the layers for any shape; the fp32 models run on them entirely, the bf16 models
// use them for the small layers around the MFMA convolutions.
#include "kernels.h"

namespace cd {

#define CD_DISPATCH_T(dtype, ...)                         \
  do {                                                    \
    if ((dtype) == CD_BF16) { typedef bf16_t T; __VA_ARGS__; } \
    else { typedef float T; __VA_ARGS__; }                \
  } while (0)

static inline dim3 grid1d(int64_t n, int block = 256) { return dim3((unsigned)cdiv(n, block)); }

// ------------------------------------------------------------------------------ convolution
template <typename T>
__global__ void __launch_bounds__(256) conv_fprop_simple_k(const T* __restrict__ x, const T* __restrict__ w,
                                                           const T* __restrict__ bias, T* __restrict__ y, ConvGeom g,
                                                           int relu) {
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= g.M() * g.Cout) return;
  const int n = idx % g.Cout;
  int64_t m = idx / g.Cout;
  const int wo = m % g.Wo; m /= g.Wo;
  const int ho = m % g.Ho;
  const int64_t b = m / g.Ho;
  float acc = bias ? Cvt<T>::ld(bias[n]) : 0.f;
  for (int r = 0; r < g.kh; r++) {
    const int hi = ho * g.stride - g.pad + r;
    if (hi < 0 || hi >= g.H) continue;
    for (int s = 0; s < g.kw; s++) {
      const int wi = wo * g.stride - g.pad + s;
      if (wi < 0 || wi >= g.W) continue;
      const T* xp = x + ((b * g.H + hi) * g.W + wi) * g.Cin;
      const T* wp = w + (((int64_t)n * g.kh + r) * g.kw + s) * g.Cin;
      for (int c = 0; c < g.Cin; c++) acc += Cvt<T>::ld(xp[c]) * Cvt<T>::ld(wp[c]);
    }
  }
  if (relu) acc = fmaxf(acc, 0.f);
  y[idx] = Cvt<T>::st(acc);
}

template <typename T>
__global__ void __launch_bounds__(256) conv_dgrad_simple_k(const T* __restrict__ dy, const T* __restrict__ w,
                                                           T* __restrict__ dx, ConvGeom g, int accumulate) {
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= g.B * g.H * g.W * g.Cin) return;
  const int c = idx % g.Cin;
  int64_t p = idx / g.Cin;
  const int wi = p % g.W; p /= g.W;
  const int hi = p % g.H;
  const int64_t b = p / g.H;
  float acc = 0.f;
  for (int r = 0; r < g.kh; r++) {
    const int hn = hi + g.pad - r;
    if (hn < 0 || hn % g.stride) continue;
    const int ho = hn / g.stride;
    if (ho >= g.Ho) continue;
    for (int s = 0; s < g.kw; s++) {
      const int wn = wi + g.pad - s;
      if (wn < 0 || wn % g.stride) continue;
      const int wo = wn / g.stride;
      if (wo >= g.Wo) continue;
      const T* dp = dy + ((b * g.Ho + ho) * g.Wo + wo) * g.Cout;
      const T* wp = w + ((int64_t)r * g.kw + s) * g.Cin + c;
      const int64_t wstride = (int64_t)g.kh * g.kw * g.Cin;
      for (int n = 0; n < g.Cout; n++) acc += Cvt<T>::ld(dp[n]) * Cvt<T>::ld(wp[n * wstride]);
    }
  }
  if (accumulate) acc += Cvt<T>::ld(dx[idx]);
  dx[idx] = Cvt<T>::st(acc);
}

// one block per weight element, threads stride over the B*Ho*Wo output positions
template <typename T>
__global__ void __launch_bounds__(256) conv_wgrad_simple_k(const T* __restrict__ x, const T* __restrict__ dy,
                                                           float* __restrict__ dw, ConvGeom g) {
  __shared__ float red[4];
  int64_t e = blockIdx.x;
  const int c = e % g.Cin; e /= g.Cin;
  const int s = e % g.kw; e /= g.kw;
  const int r = e % g.kh;
  const int n = e / g.kh;
  float acc = 0.f;
  const int64_t M = g.M();
  for (int64_t m = threadIdx.x; m < M; m += 256) {
    int64_t q = m;
    const int wo = q % g.Wo; q /= g.Wo;
    const int ho = q % g.Ho;
    const int64_t b = q / g.Ho;
    const int hi = ho * g.stride - g.pad + r, wi = wo * g.stride - g.pad + s;
    if (hi < 0 || hi >= g.H || wi < 0 || wi >= g.W) continue;
    acc += Cvt<T>::ld(dy[m * g.Cout + n]) * Cvt<T>::ld(x[((b * g.H + hi) * g.W + wi) * g.Cin + c]);
  }
  acc = wave_sum(acc);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = acc;
  __syncthreads();
  if (threadIdx.x == 0) dw[blockIdx.x] = red[0] + red[1] + red[2] + red[3];
}

void conv_fprop_simple(int dtype, const void* x, const void* w, const void* bias, void* y, const ConvGeom& g,
                       bool relu, hipStream_t s) {
  CD_DISPATCH_T(dtype, hipLaunchKernelGGL(conv_fprop_simple_k<T>, grid1d(g.M() * g.Cout), dim3(256), 0, s,
                                          (const T*)x, (const T*)w, (const T*)bias, (T*)y, g, (int)relu));
}
void conv_dgrad_simple(int dtype, const void* dy, const void* w, void* dx, const ConvGeom& g, bool accumulate,
                       hipStream_t s) {
  CD_DISPATCH_T(dtype, hipLaunchKernelGGL(conv_dgrad_simple_k<T>, grid1d(g.B * g.H * g.W * g.Cin), dim3(256), 0, s,
                                          (const T*)dy, (const T*)w, (T*)dx, g, (int)accumulate));
}
void conv_wgrad_simple(int dtype, const void* x, const void* dy, float* dw, const ConvGeom& g, hipStream_t s) {
  const int64_t n = (int64_t)g.Cout * g.K();
  CD_DISPATCH_T(dtype, hipLaunchKernelGGL(conv_wgrad_simple_k<T>, dim3((unsigned)n), dim3(256), 0, s, (const T*)x,
                                          (const T*)dy, dw, g));
}

// ------------------------------------------------------------------------------------- glue
template <typename T>
__global__ void __launch_bounds__(256) relu_bwd_k(T* __restrict__ dy, const T* __restrict__ y, int64_t n) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i < n && !(Cvt<T>::ld(y[i]) > 0.f)) dy[i] = Cvt<T>::st(0.f);
}
template <typename T>
__global__ void __launch_bounds__(256) channel_slice_k(const T* __restrict__ x, T* __restrict__ y, int64_t n, int Cx, int c0,
                                                       int Cy) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= n) return;
  const int64_t m = i / Cy;
  y[i] = x[m * Cx + c0 + (int)(i - m * Cy)];
}
void channel_slice(int dtype, const void* x, void* y, int64_t M, int Cx, int c0, int Cy, hipStream_t s) {
  const int64_t n = M * Cy;
  const dim3 grid((unsigned)cdiv(n, 256));
  if (dtype == CD_BF16)
    hipLaunchKernelGGL(channel_slice_k<bf16_t>, grid, dim3(256), 0, s, static_cast<const bf16_t*>(x), static_cast<bf16_t*>(y), n, Cx, c0, Cy);
  else
    hipLaunchKernelGGL(channel_slice_k<float>, grid, dim3(256), 0, s, static_cast<const float*>(x), static_cast<float*>(y), n, Cx, c0, Cy);
}
__global__ void __launch_bounds__(256) fill_zero_f32_k(float* p, int64_t n) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i < n) p[i] = 0.f;
}
void fill_zero_f32(float* p, int64_t n, hipStream_t s) {
  if (n > 0) hipLaunchKernelGGL(fill_zero_f32_k, dim3((unsigned)cdiv(n, 256)), dim3(256), 0, s, p, n);
}

void relu_bwd_inplace(int dtype, void* dy, const void* y, int64_t n, hipStream_t s) {
  CD_DISPATCH_T(dtype, hipLaunchKernelGGL(relu_bwd_k<T>, grid1d(n), dim3(256), 0, s, (T*)dy, (const T*)y, n));
}

// V channels per thread (V = 8 bf16 / 4 fp32 when the channel count allows 16-byte vectors)
template <typename T, int V> struct PoolVec {
  __device__ static void ld(const T* p, float (&v)[V]) {
#pragma unroll
    for (int i = 0; i < V; i++) v[i] = Cvt<T>::ld(p[i]);
  }
  __device__ static void st(T* p, const float (&v)[V]) {
#pragma unroll
    for (int i = 0; i < V; i++) p[i] = Cvt<T>::st(v[i]);
  }
};
template <> struct PoolVec<bf16_t, 8> {
  __device__ static void ld(const bf16_t* p, float (&v)[8]) {
    const uint4 t = *reinterpret_cast<const uint4*>(p);
    const uint32_t u[4] = {t.x, t.y, t.z, t.w};
#pragma unroll
    for (int i = 0; i < 4; i++) { v[2 * i] = __uint_as_float(u[i] << 16); v[2 * i + 1] = __uint_as_float(u[i] & 0xffff0000u); }
  }
  __device__ static void st(bf16_t* p, const float (&v)[8]) {
    uint32_t u[4];
#pragma unroll
    for (int i = 0; i < 4; i++) u[i] = (uint32_t)f32_to_bf16(v[2 * i]) | ((uint32_t)f32_to_bf16(v[2 * i + 1]) << 16);
    *reinterpret_cast<uint4*>(p) = make_uint4(u[0], u[1], u[2], u[3]);
  }
};

template <typename T, int V>
__global__ void __launch_bounds__(256) maxpool_fwd_k(const T* __restrict__ x, T* __restrict__ y,
                                                     uint8_t* __restrict__ argmax, int64_t B, int H, int W, int C,
                                                     int Ho, int Wo, int k, int stride, int pad) {
  const int CV = C / V;
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= B * Ho * Wo * CV) return;
  const int c = (int)(idx % CV) * V;
  int64_t p = idx / CV;
  const int wo = p % Wo; p /= Wo;
  const int ho = p % Ho;
  const int64_t b = p / Ho;
  float best[V];
  uint8_t arg[V];
#pragma unroll
  for (int i = 0; i < V; i++) { best[i] = -INFINITY; arg[i] = 0; }
  for (int r = 0; r < k; r++) {
    const int hi = ho * stride - pad + r;
    if (hi < 0 || hi >= H) continue;
    for (int s = 0; s < k; s++) {
      const int wi = wo * stride - pad + s;
      if (wi < 0 || wi >= W) continue;
      float v[V];
      PoolVec<T, V>::ld(x + ((b * H + hi) * W + wi) * C + c, v);
#pragma unroll
      for (int i = 0; i < V; i++)
        if (v[i] > best[i]) { best[i] = v[i]; arg[i] = (uint8_t)(r * k + s); }  // strict: the first maximum wins
    }
  }
  const int64_t o = ((b * Ho + ho) * Wo + wo) * C + c;
  PoolVec<T, V>::st(y + o, best);
  if (argmax) {
#pragma unroll
    for (int i = 0; i < V; i++) argmax[o + i] = arg[i];
  }
}

// backward from the stored argmax: 8 channels per thread, at most ceil(k/stride)^2 windows per pixel
__global__ void __launch_bounds__(256) maxpool_bwd_idx_k(const bf16_t* __restrict__ dy, const uint8_t* __restrict__ argmax,
                                                         bf16_t* __restrict__ dx, int accumulate, int64_t B, int H,
                                                         int W, int C, int Ho, int Wo, int k, int stride, int pad) {
  const int CV = C / 8;
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= B * H * W * CV) return;
  const int c = (int)(idx % CV) * 8;
  int64_t p = idx / CV;
  const int wi = p % W; p /= W;
  const int hi = p % H;
  const int64_t b = p / H;
  float acc[8];
#pragma unroll
  for (int i = 0; i < 8; i++) acc[i] = 0.f;
  int ho0 = hi + pad - k + 1; ho0 = ho0 <= 0 ? 0 : (ho0 + stride - 1) / stride;
  int wo0 = wi + pad - k + 1; wo0 = wo0 <= 0 ? 0 : (wo0 + stride - 1) / stride;
  int ho1 = (hi + pad) / stride; if (ho1 > Ho - 1) ho1 = Ho - 1;
  int wo1 = (wi + pad) / stride; if (wo1 > Wo - 1) wo1 = Wo - 1;
  for (int ho = ho0; ho <= ho1; ho++)
    for (int wo = wo0; wo <= wo1; wo++) {
      const uint32_t tap = (uint32_t)((hi - (ho * stride - pad)) * k + (wi - (wo * stride - pad)));
      const int64_t o = ((b * Ho + ho) * Wo + wo) * C + c;
      const uint2 a = *reinterpret_cast<const uint2*>(argmax + o);
      float g[8];
      PoolVec<bf16_t, 8>::ld(dy + o, g);
#pragma unroll
      for (int i = 0; i < 8; i++) {
        const uint32_t ai = ((i < 4 ? a.x : a.y) >> (8 * (i & 3))) & 0xffu;
        acc[i] += ai == tap ? g[i] : 0.f;
      }
    }
  bf16_t* dp = dx + ((b * H + hi) * W + wi) * C + c;
  if (accumulate) {
    float o[8];
    PoolVec<bf16_t, 8>::ld(dp, o);
#pragma unroll
    for (int i = 0; i < 8; i++) acc[i] += o[i];
  }
  PoolVec<bf16_t, 8>::st(dp, acc);
}

// Gradient goes to the first maximum of each window in row-major tap order (recomputed here).
template <typename T, int V>
__global__ void __launch_bounds__(256) maxpool_bwd_k(const T* __restrict__ x, const T* __restrict__ dy,
                                                     T* __restrict__ dx, int accumulate, int64_t B, int H, int W,
                                                     int C, int Ho, int Wo, int k, int stride, int pad) {
  const int CV = C / V;
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= B * H * W * CV) return;
  const int c = (int)(idx % CV) * V;
  int64_t p = idx / CV;
  const int wi = p % W; p /= W;
  const int hi = p % H;
  const int64_t b = p / H;
  float acc[V], mine[V];
#pragma unroll
  for (int i = 0; i < V; i++) acc[i] = 0.f;
  PoolVec<T, V>::ld(x + ((b * H + hi) * W + wi) * C + c, mine);
  // output windows that contain (hi, wi): ho*stride - pad <= hi <= ho*stride - pad + k - 1
  int ho0 = hi + pad - k + 1; ho0 = ho0 <= 0 ? 0 : (ho0 + stride - 1) / stride;
  int wo0 = wi + pad - k + 1; wo0 = wo0 <= 0 ? 0 : (wo0 + stride - 1) / stride;
  int ho1 = (hi + pad) / stride; if (ho1 > Ho - 1) ho1 = Ho - 1;
  int wo1 = (wi + pad) / stride; if (wo1 > Wo - 1) wo1 = Wo - 1;
  for (int ho = ho0; ho <= ho1; ho++) {
    const int h0 = ho * stride - pad;
    for (int wo = wo0; wo <= wo1; wo++) {
      const int w0 = wo * stride - pad;
      // this position wins the window iff no earlier tap is >= it and no later tap is > it
      bool win[V];
#pragma unroll
      for (int i = 0; i < V; i++) win[i] = true;
      for (int r = 0; r < k; r++) {
        const int hh = h0 + r;
        if (hh < 0 || hh >= H) continue;
        for (int s = 0; s < k; s++) {
          const int ww = w0 + s;
          if (ww < 0 || ww >= W || (hh == hi && ww == wi)) continue;
          float v[V];
          PoolVec<T, V>::ld(x + ((b * H + hh) * W + ww) * C + c, v);
          const bool earlier = hh < hi || (hh == hi && ww < wi);
#pragma unroll
          for (int i = 0; i < V; i++) win[i] = win[i] && (earlier ? v[i] < mine[i] : v[i] <= mine[i]);
        }
      }
      float g[V];
      PoolVec<T, V>::ld(dy + ((b * Ho + ho) * Wo + wo) * C + c, g);
#pragma unroll
      for (int i = 0; i < V; i++) acc[i] += win[i] ? g[i] : 0.f;
    }
  }
  T* dp = dx + ((b * H + hi) * W + wi) * C + c;
  if (accumulate) {
    float o[V];
    PoolVec<T, V>::ld(dp, o);
#pragma unroll
    for (int i = 0; i < V; i++) acc[i] += o[i];
  }
  PoolVec<T, V>::st(dp, acc);
}

void maxpool_fwd(int dtype, const void* x, void* y, uint8_t* argmax, int64_t B, int H, int W, int C, int k, int stride,
                 int pad, hipStream_t s) {
  const int Ho = (H + 2 * pad - k) / stride + 1, Wo = (W + 2 * pad - k) / stride + 1;
  if (dtype == CD_BF16 && C % 8 == 0 && aligned16(x) && aligned16(y))
    hipLaunchKernelGGL((maxpool_fwd_k<bf16_t, 8>), grid1d(B * Ho * Wo * (C / 8)), dim3(256), 0, s, (const bf16_t*)x,
                       (bf16_t*)y, argmax, B, H, W, C, Ho, Wo, k, stride, pad);
  else
    CD_DISPATCH_T(dtype, hipLaunchKernelGGL((maxpool_fwd_k<T, 1>), grid1d(B * Ho * Wo * C), dim3(256), 0, s,
                                            (const T*)x, (T*)y, argmax, B, H, W, C, Ho, Wo, k, stride, pad));
}
void maxpool_bwd(int dtype, const void* x, const void* dy, const uint8_t* argmax, void* dx, bool accumulate, int64_t B,
                 int H, int W, int C, int k, int stride, int pad, hipStream_t s) {
  const int Ho = (H + 2 * pad - k) / stride + 1, Wo = (W + 2 * pad - k) / stride + 1;
  if (argmax && dtype == CD_BF16 && C % 8 == 0 && aligned16(dy) && aligned16(dx) && aligned16(argmax))
    hipLaunchKernelGGL(maxpool_bwd_idx_k, grid1d(B * H * W * (C / 8)), dim3(256), 0, s, (const bf16_t*)dy, argmax,
                       (bf16_t*)dx, (int)accumulate, B, H, W, C, Ho, Wo, k, stride, pad);
  else if (dtype == CD_BF16 && C % 8 == 0 && aligned16(x) && aligned16(dy) && aligned16(dx))
    hipLaunchKernelGGL((maxpool_bwd_k<bf16_t, 8>), grid1d(B * H * W * (C / 8)), dim3(256), 0, s, (const bf16_t*)x,
                       (const bf16_t*)dy, (bf16_t*)dx, (int)accumulate, B, H, W, C, Ho, Wo, k, stride, pad);
  else
    CD_DISPATCH_T(dtype, hipLaunchKernelGGL((maxpool_bwd_k<T, 1>), grid1d(B * H * W * C), dim3(256), 0, s,
                                            (const T*)x, (const T*)dy, (T*)dx, (int)accumulate, B, H, W, C, Ho, Wo, k,
                                            stride, pad));
}

template <typename T>
__global__ void __launch_bounds__(256) gap_fwd_k(const T* __restrict__ x, T* __restrict__ y, int64_t B, int HW, int C) {
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= B * C) return;
  const int c = idx % C;
  const int64_t b = idx / C;
  float acc = 0.f;
  for (int i = 0; i < HW; i++) acc += Cvt<T>::ld(x[(b * HW + i) * C + c]);
  y[idx] = Cvt<T>::st(acc / (float)HW);
}
template <typename T>
__global__ void __launch_bounds__(256) gap_bwd_k(const T* __restrict__ dy, T* __restrict__ dx, int accumulate,
                                                 int64_t B, int HW, int C) {
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= B * HW * C) return;
  const int c = idx % C;
  const int64_t b = idx / ((int64_t)HW * C);
  float v = Cvt<T>::ld(dy[b * C + c]) / (float)HW;
  if (accumulate) v += Cvt<T>::ld(dx[idx]);
  dx[idx] = Cvt<T>::st(v);
}
void gap_fwd(int dtype, const void* x, void* y, int64_t B, int HW, int C, hipStream_t s) {
  CD_DISPATCH_T(dtype, hipLaunchKernelGGL(gap_fwd_k<T>, grid1d(B * C), dim3(256), 0, s, (const T*)x, (T*)y, B, HW, C));
}
void gap_bwd(int dtype, const void* dy, void* dx, bool accumulate, int64_t B, int HW, int C, hipStream_t s) {
  CD_DISPATCH_T(dtype, hipLaunchKernelGGL(gap_bwd_k<T>, grid1d(B * HW * C), dim3(256), 0, s, (const T*)dy, (T*)dx,
                                          (int)accumulate, B, HW, C));
}

// ----------------------------------------------------------------------------------- linear
// one wave per output element: lanes stride over the F input features
template <typename T>
__global__ void __launch_bounds__(256) linear_fwd_k(const T* __restrict__ x, const T* __restrict__ w,
                                                    const T* __restrict__ bias, float* __restrict__ y, int64_t B,
                                                    int F, int C) {
  const int64_t o = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (o >= B * C) return;
  const int c = o % C;
  const int64_t b = o / C;
  float acc = 0.f;
  for (int f = threadIdx.x & 63; f < F; f += 64) acc += Cvt<T>::ld(x[b * F + f]) * Cvt<T>::ld(w[(int64_t)c * F + f]);
  acc = wave_sum(acc);
  if ((threadIdx.x & 63) == 0) y[o] = acc + (bias ? Cvt<T>::ld(bias[c]) : 0.f);
}
template <typename T>
__global__ void __launch_bounds__(256) linear_dx_k(const float* __restrict__ dy, const T* __restrict__ w,
                                                   T* __restrict__ dx, int accumulate, int64_t B, int F, int C) {
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= B * F) return;
  const int f = idx % F;
  const int64_t b = idx / F;
  float acc = 0.f;
  for (int c = 0; c < C; c++) acc += dy[b * C + c] * Cvt<T>::ld(w[(int64_t)c * F + f]);
  if (accumulate) acc += Cvt<T>::ld(dx[idx]);
  dx[idx] = Cvt<T>::st(acc);
}
template <typename T>
__global__ void __launch_bounds__(256) linear_dw_k(const float* __restrict__ dy, const T* __restrict__ x,
                                                   float* __restrict__ dw, float* __restrict__ db, int64_t B, int F,
                                                   int C) {
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= (int64_t)C * (F + 1)) return;
  const int f = idx % (F + 1);
  const int c = idx / (F + 1);
  float acc = 0.f;
  if (f < F) {
    for (int64_t b = 0; b < B; b++) acc += dy[b * C + c] * Cvt<T>::ld(x[b * F + f]);
    dw[(int64_t)c * F + f] = acc;
  } else {
    if (!db) return;
    for (int64_t b = 0; b < B; b++) acc += dy[b * C + c];
    db[c] = acc;
  }
}
void linear_fwd(int dtype, const void* x, const void* w, const void* b, float* y, int64_t B, int F, int C,
                hipStream_t s) {
  CD_DISPATCH_T(dtype, hipLaunchKernelGGL(linear_fwd_k<T>, grid1d(B * C, 4), dim3(256), 0, s, (const T*)x, (const T*)w,
                                          (const T*)b, y, B, F, C));
}
void linear_bwd(int dtype, const void* x, const void* w, const float* dy, void* dx, bool accumulate, float* dw,
                float* db, int64_t B, int F, int C, hipStream_t s) {
  CD_DISPATCH_T(dtype, {
    hipLaunchKernelGGL(linear_dx_k<T>, grid1d(B * F), dim3(256), 0, s, dy, (const T*)w, (T*)dx, (int)accumulate, B, F, C);
    hipLaunchKernelGGL(linear_dw_k<T>, grid1d((int64_t)C * (F + 1)), dim3(256), 0, s, dy, (const T*)x, dw, db, B, F, C);
  });
}

// ----------------------------------------------------------------------------- padding gaps
struct GapList { Gap g[128]; int n; };
__global__ void __launch_bounds__(64) zero_gaps_k(float* base, GapList l) {
  const int i = blockIdx.x;
  if (i < l.n && (int)threadIdx.x < l.g[i].len) base[l.g[i].off + threadIdx.x] = 0.f;
}
void zero_gaps(float* base, const Gap* gaps, int n, hipStream_t s) {
  for (int i = 0; i < n; i += 128) {
    GapList l;
    l.n = n - i < 128 ? n - i : 128;
    for (int j = 0; j < l.n; j++) l.g[j] = gaps[i + j];
    hipLaunchKernelGGL(zero_gaps_k, dim3(l.n), dim3(64), 0, s, base, l);
  }
}

}  // namespace cd
