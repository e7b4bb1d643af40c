// BatchNorm forward / backward with batch statistics, fused ReLU and residual add, and the
// per-channel column sums they are built on.  (The paper's networks are the standard ResNets,
// Section 3; BatchNorm normalises each channel with the biased variance over batch and space.)
//
// All of it is HBM-bound.  A tensor is [M rows][C channels] with channels contiguous, so a block
// reads whole rows (consecutive threads -> consecutive 16-byte channel vectors) and every thread
// accumulates its own channels down the rows: reductions run along the strided axis while every
// load stays coalesced.  Partial sums per row chunk go to a scratch array and a second, tiny
// kernel adds them in a fixed order (deterministic, no atomics).
#include "kernels.h"

namespace cd {

typedef float f32x4_ext __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4_ext __attribute__((ext_vector_type(4)));

template <typename T, int VEC> struct Vec;
// ld / st convert to and from fp32; ldraw + unpack split the load from the conversion, so that a kernel
// can hold several loads in flight in their packed form (a quarter of the registers for bf16).
template <> struct Vec<float, 1> {
  typedef float Raw;
  __device__ static Raw ldraw(const float* p) { return *p; }
  __device__ static Raw ldraw_nt(const float* p) { return __builtin_nontemporal_load(p); }
  __device__ static void unpack(const Raw& r, float (&v)[1]) { v[0] = r; }
  __device__ static void ld(const float* p, float (&v)[1]) { v[0] = *p; }
  __device__ static void st(float* p, const float (&v)[1]) { *p = v[0]; }
};
template <> struct Vec<float, 4> {
  typedef float4 Raw;
  __device__ static Raw ldraw(const float* p) { return *reinterpret_cast<const float4*>(p); }
  __device__ static Raw ldraw_nt(const float* p) {
    const f32x4_ext v = __builtin_nontemporal_load(reinterpret_cast<const f32x4_ext*>(p));
    return make_float4(v.x, v.y, v.z, v.w);
  }
  __device__ static void unpack(const Raw& t, float (&v)[4]) { v[0] = t.x; v[1] = t.y; v[2] = t.z; v[3] = t.w; }
  __device__ static void ld(const float* p, float (&v)[4]) {
    float4 t = *reinterpret_cast<const float4*>(p);
    v[0] = t.x; v[1] = t.y; v[2] = t.z; v[3] = t.w;
  }
  __device__ static void st(float* p, const float (&v)[4]) {
    *reinterpret_cast<float4*>(p) = make_float4(v[0], v[1], v[2], v[3]);
  }
};
template <> struct Vec<bf16_t, 1> {
  typedef bf16_t Raw;
  __device__ static Raw ldraw(const bf16_t* p) { return *p; }
  __device__ static Raw ldraw_nt(const bf16_t* p) { return __builtin_nontemporal_load(p); }
  __device__ static void unpack(const Raw& r, float (&v)[1]) { v[0] = bf16_to_f32(r); }
  __device__ static void ld(const bf16_t* p, float (&v)[1]) { v[0] = bf16_to_f32(*p); }
  __device__ static void st(bf16_t* p, const float (&v)[1]) { *p = f32_to_bf16(v[0]); }
};
template <> struct Vec<bf16_t, 8> {
  typedef uint4 Raw;
  __device__ static Raw ldraw(const bf16_t* p) { return *reinterpret_cast<const uint4*>(p); }
  // read-once data: the non-temporal hint keeps it from displacing what later kernels re-read from the caches
  __device__ static Raw ldraw_nt(const bf16_t* p) {
    const u32x4_ext v = __builtin_nontemporal_load(reinterpret_cast<const u32x4_ext*>(p));
    return make_uint4(v.x, v.y, v.z, v.w);
  }
  __device__ static void unpack(const Raw& t, float (&v)[8]) {
    const uint32_t u[4] = {t.x, t.y, t.z, t.w};
#pragma unroll
    for (int i = 0; i < 4; i++) {
      v[2 * i] = __uint_as_float(u[i] << 16);
      v[2 * i + 1] = __uint_as_float(u[i] & 0xffff0000u);
    }
  }
  __device__ static void ld(const bf16_t* p, float (&v)[8]) { unpack(ldraw(p), v); }
  __device__ static void st(bf16_t* p, const float (&v)[8]) {
    uint32_t u[4];
#pragma unroll
    for (int i = 0; i < 4; i++) u[i] = (uint32_t)f32_to_bf16(v[2 * i]) | ((uint32_t)f32_to_bf16(v[2 * i + 1]) << 16);
    *reinterpret_cast<uint4*>(p) = make_uint4(u[0], u[1], u[2], u[3]);
  }
};

// MODE 0: sums of x and x^2.  MODE 1: sums of dz and dz*xhat with dz = dy * (relu ? y > 0 : 1).
// MODE 2: sum of a0.  partials: [chunks][stat_pitch(C)].
// mask (MODE 1, VEC 8 only, nullable): one byte per 8-channel vector, bit k = (y[k] > 0); read instead of y.
template <typename T, int VEC, int MODE>
__global__ void __launch_bounds__(256) col_reduce_k(const T* __restrict__ a0, const T* __restrict__ a1,
                                                    const T* __restrict__ a2, const float* __restrict__ stats,
                                                    int relu, int64_t M, int C, int64_t rows_per_chunk,
                                                    float* __restrict__ partials,
                                                    const uint8_t* __restrict__ mask) {
  __shared__ float sm[2][256 * VEC];
  const int vc = C / VEC;
  const int v0 = blockIdx.y * 256;
  const int vcb = vc - v0 < 256 ? vc - v0 : 256;  // channel vectors handled by this block
  const int rpi = 256 / vcb;                      // rows per iteration
  const int ty = threadIdx.x / vcb, tx = threadIdx.x % vcb;
  const int c0 = (v0 + tx) * VEC;
  float s0[VEC], s1[VEC], mean[VEC], istd[VEC];
#pragma unroll
  for (int k = 0; k < VEC; k++) { s0[k] = 0.f; s1[k] = 0.f; mean[k] = 0.f; istd[k] = 0.f; }
  if (ty < rpi) {
    if (MODE == 1) {
#pragma unroll
      for (int k = 0; k < VEC; k++) { mean[k] = stats[c0 + k]; istd[k] = stats[C + c0 + k]; }
    }
    // Row groups are dealt to the blocks round-robin: at any moment the grid reads one contiguous
    // window of each tensor (as the elementwise passes do), not one distant stream per block.
    const int64_t rstride = (int64_t)gridDim.x * rpi;
    int64_t r = (int64_t)blockIdx.x * rpi + ty;
    if (MODE == 1) {
      // full trips of UR row groups: every load of the trip is issued before the arithmetic
      constexpr int UR = 2;
      const bool use_mask = VEC == 8 && mask != nullptr;
      for (; r + (UR - 1) * rstride < M; r += UR * rstride) {
        typename Vec<T, VEC>::Raw ra[UR], rx[UR], ry[UR];
        uint32_t bits[UR];
#pragma unroll
        for (int u = 0; u < UR; u++) {
          const int64_t off = (r + u * rstride) * C + c0;
          ra[u] = Vec<T, VEC>::ldraw(a0 + off);
          rx[u] = Vec<T, VEC>::ldraw(a2 + off);
          if (relu) {
            if (use_mask) bits[u] = mask[off >> 3];
            else ry[u] = Vec<T, VEC>::ldraw(a1 + off);
          }
        }
#pragma unroll
        for (int u = 0; u < UR; u++) {
          float a[VEC], x[VEC], y[VEC];
          Vec<T, VEC>::unpack(ra[u], a);
          Vec<T, VEC>::unpack(rx[u], x);
          if (relu && !use_mask) Vec<T, VEC>::unpack(ry[u], y);
#pragma unroll
          for (int k = 0; k < VEC; k++) {
            float d = a[k];
            if (relu) d = (use_mask ? ((bits[u] >> k) & 1u) != 0u : y[k] > 0.f) ? d : 0.f;
            s0[k] += d;
            s1[k] += d * (x[k] - mean[k]) * istd[k];
          }
        }
      }
    }
    for (; r < M; r += rstride) {
      const int64_t off = r * C + c0;
      float a[VEC];
      Vec<T, VEC>::ld(a0 + off, a);
      if (MODE == 0) {
#pragma unroll
        for (int k = 0; k < VEC; k++) { s0[k] += a[k]; s1[k] += a[k] * a[k]; }
      } else if (MODE == 1) {
        float x[VEC];
        Vec<T, VEC>::ld(a2 + off, x);
        if (relu) {
          if (VEC == 8 && mask) {
            const uint32_t bits = mask[off >> 3];
#pragma unroll
            for (int k = 0; k < VEC; k++) a[k] = (bits >> k) & 1u ? a[k] : 0.f;
          } else {
            float y[VEC];
            Vec<T, VEC>::ld(a1 + off, y);
#pragma unroll
            for (int k = 0; k < VEC; k++) a[k] = y[k] > 0.f ? a[k] : 0.f;
          }
        }
#pragma unroll
        for (int k = 0; k < VEC; k++) { s0[k] += a[k]; s1[k] += a[k] * (x[k] - mean[k]) * istd[k]; }
      } else {
#pragma unroll
        for (int k = 0; k < VEC; k++) s0[k] += a[k];
      }
    }
#pragma unroll
    for (int k = 0; k < VEC; k++) { sm[0][threadIdx.x * VEC + k] = s0[k]; sm[1][threadIdx.x * VEC + k] = s1[k]; }
  }
  __syncthreads();
  if ((int)threadIdx.x < vcb) {
#pragma unroll
    for (int k = 0; k < VEC; k++) {
      float t0 = 0.f, t1 = 0.f;
      for (int j = 0; j < rpi; j++) {
        t0 += sm[0][(j * vcb + tx) * VEC + k];
        t1 += sm[1][(j * vcb + tx) * VEC + k];
      }
      partials[(int64_t)blockIdx.x * stat_pitch(C) + c0 + k] = t0;
      partials[(int64_t)blockIdx.x * stat_pitch(C) + C + c0 + k] = t1;
    }
  }
}

// FIN 0: BatchNorm statistics.  FIN 1: BatchNorm backward sums.  FIN 2: plain column sum.
// Block = 64 channels x 16 chunk lanes: every lane adds every 16th chunk (loads unrolled so that
// several are in flight), the 16 lanes of a channel are combined in LDS in a fixed order.
template <typename T, int FIN>
__global__ void __launch_bounds__(1024) col_finalize_k(const float* __restrict__ partials, int chunks, int64_t M, int C,
                                                       const T* __restrict__ gamma, const T* __restrict__ beta,
                                                       float* __restrict__ stats, float* __restrict__ out0,
                                                       float* __restrict__ out1, float* __restrict__ coef) {
  __shared__ double sm[2][16][64];
  const int cl = threadIdx.x & 63, lane = threadIdx.x >> 6;
  const int c = blockIdx.x * 64 + cl;
  double a0 = 0.0, a1 = 0.0;
  if (c < C) {
#pragma unroll 4
    for (int j = lane; j < chunks; j += 16) {
      a0 += (double)partials[(int64_t)j * stat_pitch(C) + c];
      if (FIN != 2) a1 += (double)partials[(int64_t)j * stat_pitch(C) + C + c];
    }
  }
  sm[0][lane][cl] = a0;
  sm[1][lane][cl] = a1;
  __syncthreads();
  if (lane != 0 || c >= C) return;
  double s0 = 0.0, s1 = 0.0;
#pragma unroll
  for (int j = 0; j < 16; j++) { s0 += sm[0][j][cl]; s1 += sm[1][j][cl]; }
  if (FIN == 0) {
    const double mean = s0 / (double)M;
    double var = s1 / (double)M - mean * mean;
    if (var < 0.0) var = 0.0;
    const float istd = (float)(1.0 / sqrt(var + (double)kBnEps));
    const float scale = Cvt<T>::ld(gamma[c]) * istd;
    stats[c] = (float)mean;
    stats[C + c] = istd;
    stats[2 * C + c] = scale;
    stats[3 * C + c] = Cvt<T>::ld(beta[c]) - (float)mean * scale;
  } else if (FIN == 1) {
    // dx = c1*dz + c2*x + c3 with xhat = (x - mean)*invstd
    const float mean = stats[c], istd = stats[C + c];
    const float dbeta = (float)s0, dgamma = (float)s1;
    out0[c] = dgamma;
    out1[c] = dbeta;
    const float c1 = Cvt<T>::ld(gamma[c]) * istd;
    const float c2 = -c1 * istd * dgamma / (float)M;
    coef[c] = c1;
    coef[C + c] = c2;
    coef[2 * C + c] = -c1 * dbeta / (float)M - c2 * mean;
  } else {
    out0[c] = (float)s0;
  }
}

// Elementwise passes.  FIXC: the number of channel vectors per row divides the grid stride, so a
// thread keeps the same channels through all of its iterations and holds their coefficients in
// registers; each thread has UNROLL independent vectors in flight.
constexpr int kEltUnroll = 4;

// Fold many chunks of partial sums into 32: block = 64 channels x 16 lanes, grid.y = 32 slices.
__global__ void __launch_bounds__(1024) col_fold_k(const float* __restrict__ partials, int chunks, int C,
                                                   float* __restrict__ out) {
  __shared__ float sm[2][16][64];
  const int cl = threadIdx.x & 63, lane = threadIdx.x >> 6;
  const int c = blockIdx.x * 64 + cl;
  const int per = (chunks + gridDim.y - 1) / gridDim.y;
  const int j0 = blockIdx.y * per, j1 = j0 + per < chunks ? j0 + per : chunks;
  float a0 = 0.f, a1 = 0.f;
  if (c < C) {
#pragma unroll 4
    for (int j = j0 + lane; j < j1; j += 16) {
      a0 += partials[(int64_t)j * stat_pitch(C) + c];
      a1 += partials[(int64_t)j * stat_pitch(C) + C + c];
    }
  }
  sm[0][lane][cl] = a0;
  sm[1][lane][cl] = a1;
  __syncthreads();
  if (lane != 0 || c >= C) return;
  float s0 = 0.f, s1 = 0.f;
#pragma unroll
  for (int j = 0; j < 16; j++) { s0 += sm[0][j][cl]; s1 += sm[1][j][cl]; }
  out[(int64_t)blockIdx.y * stat_pitch(C) + c] = s0;
  out[(int64_t)blockIdx.y * stat_pitch(C) + C + c] = s1;
}

// mask (VEC 8 only, nullable): receives one byte per vector, bit k = (y[k] > 0), for the backward pass
template <typename T, int VEC, bool FIXC>
__global__ void __launch_bounds__(256) bn_apply_k(const T* __restrict__ x, const T* __restrict__ res, T* __restrict__ y,
                                                  const float* __restrict__ stats, int relu, int64_t nvec, int C,
                                                  uint8_t* __restrict__ mask) {
  const int vc = C / VEC;
  const int64_t stride = (int64_t)gridDim.x * 256;
  // last rows first: the producing convolution wrote them most recently, so they are the part of x
  // that the caches still hold
  const int64_t i0 = (int64_t)(gridDim.x - 1 - blockIdx.x) * 256 + threadIdx.x;
  float sc[VEC], sh[VEC];
  if (FIXC) {
    const int c0 = (int)(i0 % vc) * VEC;
#pragma unroll
    for (int k = 0; k < VEC; k++) { sc[k] = stats[2 * C + c0 + k]; sh[k] = stats[3 * C + c0 + k]; }
  }
  for (int64_t ib = i0; ib < nvec; ib += stride * kEltUnroll) {
    typename Vec<T, VEC>::Raw ra[kEltUnroll], rr[kEltUnroll];
#pragma unroll
    for (int u = 0; u < kEltUnroll; u++) {
      const int64_t i = ib + u * stride;
      if (i < nvec) {
        ra[u] = Vec<T, VEC>::ldraw_nt(x + i * VEC);
        if (res) rr[u] = Vec<T, VEC>::ldraw_nt(res + i * VEC);
      }
    }
#pragma unroll
    for (int u = 0; u < kEltUnroll; u++) {
      const int64_t i = ib + u * stride;
      if (i < nvec) {
        if (!FIXC) {
          const int c0 = (int)(i % vc) * VEC;
#pragma unroll
          for (int k = 0; k < VEC; k++) { sc[k] = stats[2 * C + c0 + k]; sh[k] = stats[3 * C + c0 + k]; }
        }
        float a[VEC], r[VEC];
        Vec<T, VEC>::unpack(ra[u], a);
        if (res) Vec<T, VEC>::unpack(rr[u], r);
        uint32_t bits = 0;
#pragma unroll
        for (int k = 0; k < VEC; k++) {
          float v = a[k] * sc[k] + sh[k];
          if (res) v += r[k];
          a[k] = relu ? fmaxf(v, 0.f) : v;
          bits |= (a[k] > 0.f ? 1u : 0u) << k;
        }
        Vec<T, VEC>::st(y + i * VEC, a);
        if (VEC == 8 && mask) mask[i] = (uint8_t)bits;
      }
    }
  }
}

// BatchNorm apply + ReLU + 3x3 stride-2 pad-1 max-pool in one pass (bf16, C % 8 == 0, even H and W): the
// normalised tensor is never written.  One thread per pooled 8-channel vector; the window's values are
// normalised on the fly (each input is read by 2.25 windows on average, from cache).  argmax
// (nullable) receives the window tap r*3+s of the first maximum, as maxpool_fwd_k writes it.  mask
// (nullable) receives the ReLU sign bits of the whole normalised tensor, as bn_apply_k writes them:
// every input pixel belongs to exactly one window as one of its taps (1..2, 1..2), and that window's
// thread writes its byte.
__global__ void __launch_bounds__(256) bn_relu_pool_k(const bf16_t* __restrict__ x, const float* __restrict__ stats,
                                                      bf16_t* __restrict__ y, uint8_t* __restrict__ argmax,
                                                      uint8_t* __restrict__ mask, int64_t B, int H, int W, int C) {
  const int Ho = H / 2, Wo = W / 2, vc = C / 8;
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= B * Ho * Wo * vc) return;
  const int cv = (int)(idx % vc);
  int64_t p = idx / vc;
  const int wo = (int)(p % Wo); p /= Wo;
  const int ho = (int)(p % Ho);
  const int64_t b = p / Ho;
  float sc[8], sh[8], best[8];
  uint32_t arg[8];
#pragma unroll
  for (int k = 0; k < 8; k++) {
    sc[k] = stats[2 * C + cv * 8 + k];
    sh[k] = stats[3 * C + cv * 8 + k];
    best[k] = -1.f;   // below every ReLU output: the first tap inside the image always wins
    arg[k] = 0;
  }
  // all loads of the window first (taps outside the image re-read the centre, and are skipped below)
  Vec<bf16_t, 8>::Raw raw[9];
#pragma unroll
  for (int r = 0; r < 3; r++)
#pragma unroll
    for (int t = 0; t < 3; t++) {
      const int hi = 2 * ho - 1 + r, wi = 2 * wo - 1 + t;
      const bool in = hi >= 0 && wi >= 0;   // hi <= H - 1 and wi <= W - 1 always (even H, W)
      raw[r * 3 + t] = Vec<bf16_t, 8>::ldraw(x + ((b * H + (in ? hi : 2 * ho)) * W + (in ? wi : 2 * wo)) * C + cv * 8);
    }
#pragma unroll
  for (int r = 0; r < 3; r++)
#pragma unroll
    for (int t = 0; t < 3; t++) {
      const int hi = 2 * ho - 1 + r, wi = 2 * wo - 1 + t;
      if (hi < 0 || wi < 0) continue;
      float a[8];
      Vec<bf16_t, 8>::unpack(raw[r * 3 + t], a);
      uint32_t bits = 0;
#pragma unroll
      for (int k = 0; k < 8; k++) {
        a[k] = fmaxf(a[k] * sc[k] + sh[k], 0.f);
        bits |= (a[k] > 0.f ? 1u : 0u) << k;
        if (a[k] > best[k]) { best[k] = a[k]; arg[k] = (uint32_t)(r * 3 + t); }  // strict: the first maximum wins
      }
      if (mask && r >= 1 && t >= 1) mask[((b * H + hi) * W + wi) * vc + cv] = (uint8_t)bits;
    }
  const int64_t o = ((b * Ho + ho) * Wo + wo) * C + cv * 8;
  Vec<bf16_t, 8>::st(y + o, best);
  if (argmax) {
    uint2 pk;
    pk.x = arg[0] | (arg[1] << 8) | (arg[2] << 16) | (arg[3] << 24);
    pk.y = arg[4] | (arg[5] << 8) | (arg[6] << 16) | (arg[7] << 24);
    *reinterpret_cast<uint2*>(argmax + o) = pk;
  }
}

// ---- backward of bn_relu_pool_k: the gradient of the (unwritten) normalised tensor is gathered from the
// pooled gradient and the argmax wherever it is needed, instead of being written by a max-pool backward
// kernel and read twice.  Pixel (h, w) lies in the windows (h/2, w/2) as tap (1 + h%2, 1 + w%2) and, for
// odd h or w, in the next window down or right as tap row / column 0.
__device__ inline void pool_grad8(const bf16_t* __restrict__ dp, const uint8_t* __restrict__ arg, int b, int h, int w,
                                  int H, int W, int C, int c0, float (&dz)[8]) {
  const int Ho = H >> 1, Wo = W >> 1;
#pragma unroll
  for (int k = 0; k < 8; k++) dz[k] = 0.f;
#pragma unroll
  for (int dh = 0; dh < 2; dh++) {
    const int ho = (h >> 1) + dh, r = dh ? 0 : 1 + (h & 1);
    if (dh && (!(h & 1) || ho >= Ho)) continue;
#pragma unroll
    for (int dw = 0; dw < 2; dw++) {
      const int wo = (w >> 1) + dw, t = dw ? 0 : 1 + (w & 1);
      if (dw && (!(w & 1) || wo >= Wo)) continue;
      const uint32_t o = (uint32_t)((b * Ho + ho) * Wo + wo) * (uint32_t)C + (uint32_t)c0;   // < 2^31 (checked on the host)
      const uint2 a8 = *reinterpret_cast<const uint2*>(arg + o);
      float g[8];
      Vec<bf16_t, 8>::ld(dp + o, g);
      const uint32_t tap = (uint32_t)(r * 3 + t);
#pragma unroll
      for (int k = 0; k < 8; k++) {
        const uint32_t ak = ((k < 4 ? a8.x : a8.y) >> (8 * (k & 3))) & 0xffu;
        dz[k] += ak == tap ? g[k] : 0.f;
      }
    }
  }
}

// sums of dz and dz * xhat over the rows; same partials as col_reduce_k MODE 1 (finalised by col_finalize_k<., 1>)
__global__ void __launch_bounds__(256) bn_pool_bwd_reduce_k(const bf16_t* __restrict__ dp, const uint8_t* __restrict__ arg,
                                                            const bf16_t* __restrict__ x, const float* __restrict__ stats,
                                                            const uint8_t* __restrict__ mask, int64_t B, int H, int W,
                                                            int C, float* __restrict__ partials) {
  __shared__ float sm[2][256 * 8];
  const int vc = C / 8;
  const int v0 = blockIdx.y * 256;
  const int vcb = vc - v0 < 256 ? vc - v0 : 256;
  const int rpi = 256 / vcb;
  const int ty = threadIdx.x / vcb, tx = threadIdx.x % vcb;
  const int c0 = (v0 + tx) * 8;
  const int64_t M = B * H * W;
  float s0[8], s1[8], mean[8], istd[8];
#pragma unroll
  for (int k = 0; k < 8; k++) { s0[k] = 0.f; s1[k] = 0.f; mean[k] = 0.f; istd[k] = 0.f; }
  if (ty < rpi) {
#pragma unroll
    for (int k = 0; k < 8; k++) { mean[k] = stats[c0 + k]; istd[k] = stats[C + c0 + k]; }
    const uint32_t rstride = gridDim.x * (uint32_t)rpi;
    for (uint32_t r = blockIdx.x * (uint32_t)rpi + (uint32_t)ty; r < (uint32_t)M; r += rstride) {
      const uint32_t q = r / (uint32_t)W;
      const int w = (int)(r - q * (uint32_t)W);
      const int b = (int)(q / (uint32_t)H);
      const int h = (int)(q - (uint32_t)b * (uint32_t)H);
      const uint32_t off = r * (uint32_t)C + (uint32_t)c0;
      const typename Vec<bf16_t, 8>::Raw rx = Vec<bf16_t, 8>::ldraw(x + off);
      const uint32_t bits = mask[off >> 3];
      float dz[8], xv[8];
      pool_grad8(dp, arg, b, h, w, H, W, C, c0, dz);
      Vec<bf16_t, 8>::unpack(rx, xv);
#pragma unroll
      for (int k = 0; k < 8; k++) {
        const float d = (bits >> k) & 1u ? dz[k] : 0.f;
        s0[k] += d;
        s1[k] += d * (xv[k] - mean[k]) * istd[k];
      }
    }
#pragma unroll
    for (int k = 0; k < 8; k++) { sm[0][threadIdx.x * 8 + k] = s0[k]; sm[1][threadIdx.x * 8 + k] = s1[k]; }
  }
  __syncthreads();
  if ((int)threadIdx.x < vcb) {
#pragma unroll
    for (int k = 0; k < 8; k++) {
      float t0 = 0.f, t1 = 0.f;
      for (int j = 0; j < rpi; j++) {
        t0 += sm[0][(j * vcb + tx) * 8 + k];
        t1 += sm[1][(j * vcb + tx) * 8 + k];
      }
      partials[(int64_t)blockIdx.x * stat_pitch(C) + c0 + k] = t0;
      partials[(int64_t)blockIdx.x * stat_pitch(C) + C + c0 + k] = t1;
    }
  }
}

// dx = c1 * dz + c2 * x + c3 with the coefficients col_finalize_k<., 1> left in coef
__global__ void __launch_bounds__(256) bn_pool_bwd_apply_k(const bf16_t* __restrict__ dp, const uint8_t* __restrict__ arg,
                                                           const bf16_t* __restrict__ x, const float* __restrict__ coef,
                                                           const uint8_t* __restrict__ mask, bf16_t* __restrict__ dx,
                                                           int64_t B, int H, int W, int C) {
  const int vc = C / 8;
  const uint32_t i = blockIdx.x * 256u + threadIdx.x;
  if (i >= (uint32_t)(B * H * W * vc)) return;
  const uint32_t r = i / (uint32_t)vc, q = r / (uint32_t)W;
  const int c0 = (int)(i - r * (uint32_t)vc) * 8;
  const int w = (int)(r - q * (uint32_t)W);
  const int b = (int)(q / (uint32_t)H);
  const int h = (int)(q - (uint32_t)b * (uint32_t)H);
  const typename Vec<bf16_t, 8>::Raw rx = Vec<bf16_t, 8>::ldraw(x + (size_t)i * 8);
  const uint32_t bits = mask[i];
  float dz[8], xv[8], o[8];
  pool_grad8(dp, arg, b, h, w, H, W, C, c0, dz);
  Vec<bf16_t, 8>::unpack(rx, xv);
#pragma unroll
  for (int k = 0; k < 8; k++) {
    const float d = (bits >> k) & 1u ? dz[k] : 0.f;
    o[k] = coef[c0 + k] * d + coef[C + c0 + k] * xv[k] + coef[2 * C + c0 + k];
  }
  Vec<bf16_t, 8>::st(dx + (size_t)i * 8, o);
}

template <typename T, int VEC, bool FIXC>
__global__ void __launch_bounds__(256) bn_bwd_apply_k(const T* __restrict__ dy, const T* __restrict__ y,
                                                      const T* __restrict__ x, const float* __restrict__ coef, int relu,
                                                      T* __restrict__ dx, int acc_dx, T* __restrict__ dres,
                                                      int acc_dres, int64_t nvec, int C,
                                                      const uint8_t* __restrict__ mask) {
  constexpr int U = 2;
  const bool use_mask = VEC == 8 && mask != nullptr;
  const int vc = C / VEC;
  const int64_t stride = (int64_t)gridDim.x * 256;
  // last rows first: the reduction that ran just before read them last, so they are the part of dy
  // and x that the memory-side cache still holds
  const int64_t i0 = (int64_t)(gridDim.x - 1 - blockIdx.x) * 256 + threadIdx.x;
  float c1[VEC], c2[VEC], c3[VEC];
  if (FIXC) {
    const int c0 = (int)(i0 % vc) * VEC;
#pragma unroll
    for (int k = 0; k < VEC; k++) { c1[k] = coef[c0 + k]; c2[k] = coef[C + c0 + k]; c3[k] = coef[2 * C + c0 + k]; }
  }
  for (int64_t ib = i0; ib < nvec; ib += stride * U) {
    typename Vec<T, VEC>::Raw rdz[U], rxv[U], ryv[U], rpdx[U], rpdr[U];
    uint32_t bits[U];
#pragma unroll
    for (int u = 0; u < U; u++) {
      const int64_t i = ib + u * stride;
      if (i < nvec) {
        rdz[u] = Vec<T, VEC>::ldraw(dy + i * VEC);
        rxv[u] = Vec<T, VEC>::ldraw(x + i * VEC);
        if (relu) {
          if (use_mask) bits[u] = mask[i];
          else ryv[u] = Vec<T, VEC>::ldraw(y + i * VEC);
        }
        if (acc_dx) rpdx[u] = Vec<T, VEC>::ldraw(dx + i * VEC);
        if (dres && acc_dres) rpdr[u] = Vec<T, VEC>::ldraw(dres + i * VEC);
      }
    }
#pragma unroll
    for (int u = 0; u < U; u++) {
      const int64_t i = ib + u * stride;
      if (i < nvec) {
        if (!FIXC) {
          const int c0 = (int)(i % vc) * VEC;
#pragma unroll
          for (int k = 0; k < VEC; k++) { c1[k] = coef[c0 + k]; c2[k] = coef[C + c0 + k]; c3[k] = coef[2 * C + c0 + k]; }
        }
        float dz[VEC], xv[VEC], yv[VEC], pdx[VEC], pdr[VEC], o[VEC];
        Vec<T, VEC>::unpack(rdz[u], dz);
        Vec<T, VEC>::unpack(rxv[u], xv);
        if (relu && !use_mask) Vec<T, VEC>::unpack(ryv[u], yv);
        if (acc_dx) Vec<T, VEC>::unpack(rpdx[u], pdx);
        if (dres && acc_dres) Vec<T, VEC>::unpack(rpdr[u], pdr);
#pragma unroll
        for (int k = 0; k < VEC; k++) {
          if (relu) dz[k] = (use_mask ? ((bits[u] >> k) & 1u) != 0u : yv[k] > 0.f) ? dz[k] : 0.f;
          o[k] = c1[k] * dz[k] + c2[k] * xv[k] + c3[k];
          if (acc_dx) o[k] += pdx[k];
        }
        Vec<T, VEC>::st(dx + i * VEC, o);
        if (dres) {
          if (acc_dres) {
#pragma unroll
            for (int k = 0; k < VEC; k++) dz[k] += pdr[k];
          }
          Vec<T, VEC>::st(dres + i * VEC, dz);
        }
      }
    }
  }
}

// grid for the elementwise passes: one trip of `unroll` vectors per thread; *fixc tells whether a
// thread keeps its channels (the grid stride is then a multiple of the vectors per row)
static unsigned elt_grid(int64_t nvec, int vc, int unroll, bool* fixc) {
  int64_t blocks = cdiv(nvec, (int64_t)256 * unroll);
  if (blocks < 1) blocks = 1;
  int g = vc, b = 256;  // blocks*256 % vc == 0  <=>  blocks % (vc / gcd(vc, 256)) == 0
  while (b) { const int t = g % b; g = b; b = t; }
  const int mult = vc / g;
  blocks = cdiv(blocks, mult) * mult;
  *fixc = (blocks * 256) % vc == 0 && blocks < (1 << 30);
  return (unsigned)blocks;
}

// How the rows are cut into chunks; the same rule sizes the launch and bounds the partials.
struct ReducePlan { int chunks; int64_t rows_per_chunk; int cgroups; };
static ReducePlan reduce_plan(int64_t M, int C, int vec) {
  ReducePlan p;
  const int vc = C / vec;
  p.cgroups = (int)cdiv(vc, 256);
  const int vcb = vc < 256 ? vc : 256;
  const int rpi = 256 / vcb;
  int64_t target = 1024 / p.cgroups;                      // blocks to fill the chip several times
  const int64_t cap = (int64_t)(kPartialsBytes / ((size_t)stat_pitch(C) * 4));
  if (target > cap) target = cap;
  if (target < 1) target = 1;
  int64_t rpc = cdiv(M, target);
  const int64_t min_rows = (int64_t)rpi * 8;              // at least a few iterations per block
  if (rpc < min_rows) rpc = min_rows;
  p.rows_per_chunk = rpc;
  p.chunks = (int)cdiv(M, rpc);
  return p;
}

template <typename T> static int pick_vec(int C, const void* p0, const void* p1, const void* p2, const void* p3) {
  const int v = sizeof(T) == 2 ? 8 : 4;
  const bool al = aligned16(p0) && aligned16(p1) && aligned16(p2) && aligned16(p3);
  return (C % v == 0 && al) ? v : 1;
}

template <typename T, int VEC, int MODE>
static ReducePlan launch_reduce(const T* a0, const T* a1, const T* a2, const float* stats, bool relu, int64_t M, int C,
                                float* partials, hipStream_t s, const uint8_t* mask = nullptr) {
  ReducePlan p = reduce_plan(M, C, VEC);
  hipLaunchKernelGGL((col_reduce_k<T, VEC, MODE>), dim3(p.chunks, p.cgroups), dim3(256), 0, s, a0, a1, a2, stats,
                     (int)relu, M, C, p.rows_per_chunk, partials, mask);
  return p;
}

// Batch statistics -> stats.  pre_chunks > 0: the column sums are already in partials (written by the
// producing convolution); otherwise x is reduced first.
template <typename T>
static void bn_stats_t(const T* x, const T* gamma, const T* beta, int64_t M, int C, float* stats, float* partials,
                       int pre_chunks, float* scratch, hipStream_t s) {
  const int vec = pick_vec<T>(C, x, nullptr, nullptr, nullptr);
  constexpr int V = sizeof(T) == 2 ? 8 : 4;
  int chunks = pre_chunks;
  const float* src = partials;
  if (pre_chunks == 0) {
    ReducePlan p = vec > 1 ? launch_reduce<T, V, 0>(x, nullptr, nullptr, nullptr, false, M, C, partials, s)
                           : launch_reduce<T, 1, 0>(x, nullptr, nullptr, nullptr, false, M, C, partials, s);
    chunks = p.chunks;
  } else if (pre_chunks > 256) {
    hipLaunchKernelGGL(col_fold_k, dim3((unsigned)cdiv(C, 64), 32), dim3(1024), 0, s, partials, pre_chunks, C, scratch);
    chunks = 32;
    src = scratch;
  }
  hipLaunchKernelGGL((col_finalize_k<T, 0>), dim3((unsigned)cdiv(C, 64)), dim3(1024), 0, s, src, chunks, M, C,
                     gamma, beta, stats, (float*)nullptr, (float*)nullptr, (float*)nullptr);
}

// y = relu?(scale * x + shift (+ res)) with the scale and shift that bn_stats_t left in stats
template <typename T>
static void bn_apply_t(const T* x, const T* res, bool relu, T* y, int64_t M, int C, const float* stats, uint8_t* mask,
                       hipStream_t s) {
  const int vec = pick_vec<T>(C, x, res, y, nullptr);
  constexpr int V = sizeof(T) == 2 ? 8 : 4;
  const int64_t nvec = M * C / vec;
  bool fixc;
  const unsigned blocks = elt_grid(nvec, C / vec, kEltUnroll, &fixc);
#define CD_BN_APPLY(VV, FC) \
  hipLaunchKernelGGL((bn_apply_k<T, VV, FC>), dim3(blocks), dim3(256), 0, s, x, res, y, stats, (int)relu, nvec, C, \
                     relu ? mask : (uint8_t*)nullptr)
  if (vec > 1) { if (fixc) CD_BN_APPLY(V, true); else CD_BN_APPLY(V, false); }
  else { if (fixc) CD_BN_APPLY(1, true); else CD_BN_APPLY(1, false); }
#undef CD_BN_APPLY
}

template <typename T>
static void bn_backward_t(const T* dy, const T* y, const T* x, const T* gamma, const float* stats, bool relu, T* dx,
                          bool acc_dx, T* dres, bool acc_dres, float* dgamma, float* dbeta, float* coef,
                          float* partials, const uint8_t* mask, int64_t M, int C, hipStream_t s, int pre_chunks) {
  int vec = pick_vec<T>(C, dy, y, x, dx);
  if (!aligned16(dres)) vec = 1;
  constexpr int V = sizeof(T) == 2 ? 8 : 4;
  int chunks = pre_chunks;
  const float* src = partials;
  if (pre_chunks == 0) {
    ReducePlan p = vec > 1 ? launch_reduce<T, V, 1>(dy, y, x, stats, relu, M, C, partials, s, mask)
                           : launch_reduce<T, 1, 1>(dy, y, x, stats, relu, M, C, partials, s);
    chunks = p.chunks;
  } else if (pre_chunks > 256) {   // the sums came per row tile of the data gradient that wrote dy: fold them first
    float* scratch = partials + (size_t)pre_chunks * stat_pitch(C);
    hipLaunchKernelGGL(col_fold_k, dim3((unsigned)cdiv(C, 64), 32), dim3(1024), 0, s, partials, pre_chunks, C, scratch);
    chunks = 32;
    src = scratch;
  }
  hipLaunchKernelGGL((col_finalize_k<T, 1>), dim3((unsigned)cdiv(C, 64)), dim3(1024), 0, s, src, chunks, M, C,
                     gamma, (const T*)nullptr, const_cast<float*>(stats), dgamma, dbeta, coef);
  const int64_t nvec = M * C / vec;
  bool fixc;
  const unsigned blocks = elt_grid(nvec, C / vec, 2, &fixc);
#define CD_BN_BWD(VV, FC)                                                                                          \
  hipLaunchKernelGGL((bn_bwd_apply_k<T, VV, FC>), dim3(blocks), dim3(256), 0, s, dy, y, x, coef, (int)relu, dx, \
                     (int)acc_dx, dres, (int)acc_dres, nvec, C, mask)
  if (vec > 1) { if (fixc) CD_BN_BWD(V, true); else CD_BN_BWD(V, false); }
  else { if (fixc) CD_BN_BWD(1, true); else CD_BN_BWD(1, false); }
#undef CD_BN_BWD
}

template <typename T>
static void colsum_t(const T* a, int64_t M, int C, float* out, float* partials, hipStream_t s) {
  const int vec = pick_vec<T>(C, a, nullptr, nullptr, nullptr);
  constexpr int V = sizeof(T) == 2 ? 8 : 4;
  ReducePlan p = vec > 1 ? launch_reduce<T, V, 2>(a, nullptr, nullptr, nullptr, false, M, C, partials, s)
                         : launch_reduce<T, 1, 2>(a, nullptr, nullptr, nullptr, false, M, C, partials, s);
  hipLaunchKernelGGL((col_finalize_k<T, 2>), dim3((unsigned)cdiv(C, 64)), dim3(1024), 0, s, partials, p.chunks, M, C,
                     (const T*)nullptr, (const T*)nullptr, (float*)nullptr, out, (float*)nullptr, (float*)nullptr);
}

// ---- running averages (evaluation mode) ----------------------------------------------------------
// running = [mean[C] | var[C]].  After a training-mode pass: (1 - mom) * old + mom * batch value, the batch
// variance in its unbiased form (rows / (rows - 1) times the biased one that stats holds as 1 / invstd^2 - eps).
__global__ void __launch_bounds__(256) bn_running_update_k(const float* __restrict__ stats, float* __restrict__ running,
                                                           int C, float mom, float unbias) {
  const int c = blockIdx.x * 256 + threadIdx.x;
  if (c >= C) return;
  const float mean = stats[c], istd = stats[C + c];
  const float var = fmaxf(1.f / (istd * istd) - kBnEps, 0.f) * unbias;
  running[c] = (1.f - mom) * running[c] + mom * mean;
  running[C + c] = (1.f - mom) * running[C + c] + mom * var;
}

// stats (mean, invstd, scale, shift) from the running averages instead of the batch
template <typename T>
__global__ void __launch_bounds__(256) bn_stats_from_running_k(const float* __restrict__ running, const T* __restrict__ gamma,
                                                               const T* __restrict__ beta, float* __restrict__ stats, int C) {
  const int c = blockIdx.x * 256 + threadIdx.x;
  if (c >= C) return;
  const float mean = running[c], istd = 1.f / sqrtf(running[C + c] + kBnEps);
  const float scale = Cvt<T>::ld(gamma[c]) * istd;
  stats[c] = mean;
  stats[C + c] = istd;
  stats[2 * C + c] = scale;
  stats[3 * C + c] = Cvt<T>::ld(beta[c]) - mean * scale;
}

void bn_running_update(const float* stats, float* running, int64_t M, int C, float momentum, hipStream_t s) {
  hipLaunchKernelGGL(bn_running_update_k, dim3((unsigned)cdiv(C, 256)), dim3(256), 0, s, stats, running, C, momentum,
                     M > 1 ? (float)((double)M / (double)(M - 1)) : 1.f);
}

void bn_stats_from_running(int dtype, const float* running, const void* gamma, const void* beta, float* stats, int C,
                           hipStream_t s) {
  if (dtype == CD_BF16)
    hipLaunchKernelGGL(bn_stats_from_running_k<bf16_t>, dim3((unsigned)cdiv(C, 256)), dim3(256), 0, s, running,
                       (const bf16_t*)gamma, (const bf16_t*)beta, stats, C);
  else
    hipLaunchKernelGGL(bn_stats_from_running_k<float>, dim3((unsigned)cdiv(C, 256)), dim3(256), 0, s, running,
                       (const float*)gamma, (const float*)beta, stats, C);
}

void bn_stats(int dtype, const void* x, const void* gamma, const void* beta, int64_t M, int C, float* stats,
              float* partials, int pre_chunks, float* scratch, hipStream_t s) {
  if (dtype == CD_BF16)
    bn_stats_t<bf16_t>((const bf16_t*)x, (const bf16_t*)gamma, (const bf16_t*)beta, M, C, stats, partials, pre_chunks,
                       scratch, s);
  else
    bn_stats_t<float>((const float*)x, (const float*)gamma, (const float*)beta, M, C, stats, partials, pre_chunks, scratch, s);
}
void bn_relu_pool(const bf16_t* x, const float* stats, bf16_t* y, uint8_t* argmax, uint8_t* relu_mask, int64_t B, int H,
                  int W, int C, hipStream_t s) {
  const int64_t n = B * (H / 2) * (W / 2) * (C / 8);
  hipLaunchKernelGGL(bn_relu_pool_k, dim3((unsigned)cdiv(n, 256)), dim3(256), 0, s, x, stats, y, argmax, relu_mask, B, H,
                     W, C);
}
void bn_relu_pool_backward(const bf16_t* dpool, const uint8_t* argmax, const bf16_t* x, const bf16_t* gamma,
                           const float* stats, bf16_t* dx, float* dgamma, float* dbeta, float* coef, float* partials,
                           const uint8_t* relu_mask, int64_t B, int H, int W, int C, hipStream_t s) {
  const int64_t M = B * H * W;
  ReducePlan p = reduce_plan(M, C, 8);
  // the gathers leave a thread one row in flight at a time: four times the usual number of blocks keeps
  // the memory system busy instead
  const int64_t cap = (int64_t)(kPartialsBytes / ((size_t)stat_pitch(C) * 4));
  p.chunks = (int)(p.chunks * 4 < cap ? p.chunks * 4 : cap);
  hipLaunchKernelGGL(bn_pool_bwd_reduce_k, dim3(p.chunks, p.cgroups), dim3(256), 0, s, dpool, argmax, x, stats, relu_mask, B,
                     H, W, C, partials);
  hipLaunchKernelGGL((col_finalize_k<bf16_t, 1>), dim3((unsigned)cdiv(C, 64)), dim3(1024), 0, s, partials, p.chunks, M, C,
                     gamma, (const bf16_t*)nullptr, const_cast<float*>(stats), dgamma, dbeta, coef);
  hipLaunchKernelGGL(bn_pool_bwd_apply_k, dim3((unsigned)cdiv(M * (C / 8), 256)), dim3(256), 0, s, dpool, argmax, x, coef,
                     relu_mask, dx, B, H, W, C);
}
void bn_apply(int dtype, const void* x, const void* res, bool relu, void* y, int64_t M, int C, const float* stats,
              uint8_t* relu_mask, hipStream_t s) {
  if (dtype == CD_BF16)
    bn_apply_t<bf16_t>((const bf16_t*)x, (const bf16_t*)res, relu, (bf16_t*)y, M, C, stats, relu_mask, s);
  else
    bn_apply_t<float>((const float*)x, (const float*)res, relu, (float*)y, M, C, stats, relu_mask, s);
}
void bn_backward(int dtype, const void* dy, const void* y, const void* x, const void* gamma, const float* stats,
                 bool relu, void* dx, bool acc_dx, void* dres, bool acc_dres, float* dgamma, float* dbeta, float* coef,
                 float* partials, const uint8_t* relu_mask, int64_t M, int C, hipStream_t s, int pre_chunks) {
  if (dtype == CD_BF16)
    bn_backward_t<bf16_t>((const bf16_t*)dy, (const bf16_t*)y, (const bf16_t*)x, (const bf16_t*)gamma, stats, relu,
                          (bf16_t*)dx, acc_dx, (bf16_t*)dres, acc_dres, dgamma, dbeta, coef, partials, relu_mask, M, C, s,
                          pre_chunks);
  else
    bn_backward_t<float>((const float*)dy, (const float*)y, (const float*)x, (const float*)gamma, stats, relu,
                         (float*)dx, acc_dx, (float*)dres, acc_dres, dgamma, dbeta, coef, partials, nullptr, M, C, s, 0);
}
void colsum(int dtype, const void* a, int64_t M, int C, float* out, float* partials, hipStream_t s) {
  if (dtype == CD_BF16) colsum_t<bf16_t>((const bf16_t*)a, M, C, out, partials, s);
  else colsum_t<float>((const float*)a, M, C, out, partials, s);
}

}  // namespace cd
