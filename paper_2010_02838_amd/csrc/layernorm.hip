// LayerNorm forward / backward with a fused residual add (post-LayerNorm of a Transformer sublayer:
// y = LN(a + r); the paper's translation experiments, Section 4, train the Transformer of Vaswani
// et al.).  Rows are normalised over their last axis with the biased variance, eps 1e-5.
//
// HBM-bound.  One wavefront owns a row at a time: the row (sum of the two inputs) sits in registers
// between the reductions and the output (each input element is read once, each output written
// once), lanes hold 16-byte vectors at a 64-vector stride so that a wave's loads are contiguous,
// and the two row reductions are wave shuffles.  The backward pass also needs the column sums
// dgamma = sum_rows dy*xhat and dbeta = sum_rows dy: every wave keeps running sums of its own
// columns over the rows it visits (rows are dealt round-robin), writes them once, and a second
// kernel adds the per-wave partials in a fixed order (deterministic, no atomics).
#include "kernels.h"

namespace cd {

constexpr float kLnEps = 1e-5f;

template <typename T> struct LnVec;
template <> struct LnVec<float> {
  static constexpr int N = 4;
  typedef float4 Raw;
  __device__ static void unpack(const Raw& t, float (&v)[4]) { v[0] = t.x; v[1] = t.y; v[2] = t.z; v[3] = t.w; }
  __device__ static Raw pack(const float (&v)[4]) { return make_float4(v[0], v[1], v[2], v[3]); }
};
template <> struct LnVec<bf16_t> {
  static constexpr int N = 8;
  typedef uint4 Raw;
  __device__ static void unpack(const Raw& t, float (&v)[8]) {
    const uint32_t u[4] = {t.x, t.y, t.z, t.w};
#pragma unroll
    for (int i = 0; i < 4; i++) {
      v[2 * i] = __uint_as_float(u[i] << 16);
      v[2 * i + 1] = __uint_as_float(u[i] & 0xffff0000u);
    }
  }
  __device__ static Raw pack(const float (&v)[8]) {
    uint32_t u[4];
#pragma unroll
    for (int i = 0; i < 4; i++) u[i] = (uint32_t)f32_to_bf16(v[2 * i]) | ((uint32_t)f32_to_bf16(v[2 * i + 1]) << 16);
    return make_uint4(u[0], u[1], u[2], u[3]);
  }
};

// Vector path: d is a multiple of the vector width and at most 64 * NV vectors long; a lane holds
// vectors lane, lane + 64, ... of the row.  stats: [rows][2] = mean, rstd.
template <typename T, int NV>
__global__ void __launch_bounds__(256) ln_fwd_k(const T* __restrict__ a, const T* __restrict__ r,
                                                const T* __restrict__ gamma, const T* __restrict__ beta,
                                                T* __restrict__ y, float* __restrict__ stats, int64_t rows, int d) {
  constexpr int V = LnVec<T>::N;
  typedef typename LnVec<T>::Raw Raw;
  const int lane = threadIdx.x & 63;
  const int64_t wave = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6), nwaves = (int64_t)gridDim.x * 4;
  const int nvec = d / V;
  const float inv_d = 1.f / (float)d;
  for (int64_t row = wave; row < rows; row += nwaves) {
    const T* ap = a + row * d;
    const T* rp = r ? r + row * d : nullptr;
    float s[NV][V];
    float sum = 0.f;
#pragma unroll
    for (int j = 0; j < NV; j++) {
      const int v = lane + 64 * j;
      if (v < nvec) {
        LnVec<T>::unpack(*reinterpret_cast<const Raw*>(ap + v * V), s[j]);
        if (rp) {
          float t[V];
          LnVec<T>::unpack(*reinterpret_cast<const Raw*>(rp + v * V), t);
#pragma unroll
          for (int k = 0; k < V; k++) s[j][k] += t[k];
        }
#pragma unroll
        for (int k = 0; k < V; k++) sum += s[j][k];
      }
    }
    const float mean = wave_sum(sum) * inv_d;
    float sq = 0.f;
#pragma unroll
    for (int j = 0; j < NV; j++)
      if (lane + 64 * j < nvec) {
#pragma unroll
        for (int k = 0; k < V; k++) { const float c = s[j][k] - mean; sq += c * c; }
      }
    const float rstd = rsqrtf(wave_sum(sq) * inv_d + kLnEps);
    if (lane == 0 && stats) { stats[row * 2] = mean; stats[row * 2 + 1] = rstd; }
#pragma unroll
    for (int j = 0; j < NV; j++) {
      const int v = lane + 64 * j;
      if (v < nvec) {
        float g[V], b[V], o[V];
        LnVec<T>::unpack(*reinterpret_cast<const Raw*>(gamma + v * V), g);
        LnVec<T>::unpack(*reinterpret_cast<const Raw*>(beta + v * V), b);
#pragma unroll
        for (int k = 0; k < V; k++) o[k] = (s[j][k] - mean) * rstd * g[k] + b[k];
        *reinterpret_cast<Raw*>(y + row * d + v * V) = LnVec<T>::pack(o);
      }
    }
  }
}

// dx = rstd * (g - mean(g) - xhat * mean(g * xhat)), g = dy * gamma, xhat = (a + r - mean) * rstd.
// dx goes to da (added to what is there if acc_a) and to dr (the residual input, likewise).
// partials: [waves][2][d] = this wave's sums of dy (dbeta) and dy * xhat (dgamma).
template <typename T, int NV>
__global__ void __launch_bounds__(256) ln_bwd_k(const T* __restrict__ dy, const T* __restrict__ a,
                                                const T* __restrict__ r, const T* __restrict__ gamma,
                                                const float* __restrict__ stats, T* __restrict__ da, int acc_a,
                                                T* __restrict__ dr, int acc_r, float* __restrict__ partials,
                                                int64_t rows, int d) {
  constexpr int V = LnVec<T>::N;
  typedef typename LnVec<T>::Raw Raw;
  const int lane = threadIdx.x & 63;
  const int64_t wave = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6), nwaves = (int64_t)gridDim.x * 4;
  const int nvec = d / V;
  const float inv_d = 1.f / (float)d;
  float g[NV][V], sb[NV][V], sg[NV][V];
#pragma unroll
  for (int j = 0; j < NV; j++) {
    const int v = lane + 64 * j;
#pragma unroll
    for (int k = 0; k < V; k++) { sb[j][k] = 0.f; sg[j][k] = 0.f; g[j][k] = 0.f; }
    if (v < nvec) LnVec<T>::unpack(*reinterpret_cast<const Raw*>(gamma + v * V), g[j]);
  }
  for (int64_t row = wave; row < rows; row += nwaves) {
    const float mean = stats[row * 2], rstd = stats[row * 2 + 1];
    float xh[NV][V], gy[NV][V];
    float s1 = 0.f, s2 = 0.f;
#pragma unroll
    for (int j = 0; j < NV; j++) {
      const int v = lane + 64 * j;
      if (v < nvec) {
        float t[V], u[V];
        LnVec<T>::unpack(*reinterpret_cast<const Raw*>(a + row * d + v * V), xh[j]);
        if (r) {
          LnVec<T>::unpack(*reinterpret_cast<const Raw*>(r + row * d + v * V), t);
#pragma unroll
          for (int k = 0; k < V; k++) xh[j][k] += t[k];
        }
        LnVec<T>::unpack(*reinterpret_cast<const Raw*>(dy + row * d + v * V), u);
#pragma unroll
        for (int k = 0; k < V; k++) {
          xh[j][k] = (xh[j][k] - mean) * rstd;
          sb[j][k] += u[k];
          sg[j][k] += u[k] * xh[j][k];
          gy[j][k] = u[k] * g[j][k];
          s1 += gy[j][k];
          s2 += gy[j][k] * xh[j][k];
        }
      }
    }
    const float m1 = wave_sum(s1) * inv_d, m2 = wave_sum(s2) * inv_d;
#pragma unroll
    for (int j = 0; j < NV; j++) {
      const int v = lane + 64 * j;
      if (v < nvec) {
        float o[V];
#pragma unroll
        for (int k = 0; k < V; k++) o[k] = rstd * (gy[j][k] - m1 - xh[j][k] * m2);
        if (da) {
          float w[V];
          if (acc_a) {
            LnVec<T>::unpack(*reinterpret_cast<const Raw*>(da + row * d + v * V), w);
#pragma unroll
            for (int k = 0; k < V; k++) w[k] += o[k];
          } else {
#pragma unroll
            for (int k = 0; k < V; k++) w[k] = o[k];
          }
          *reinterpret_cast<Raw*>(da + row * d + v * V) = LnVec<T>::pack(w);
        }
        if (dr) {
          float w[V];
          if (acc_r) {
            LnVec<T>::unpack(*reinterpret_cast<const Raw*>(dr + row * d + v * V), w);
#pragma unroll
            for (int k = 0; k < V; k++) w[k] += o[k];
          } else {
#pragma unroll
            for (int k = 0; k < V; k++) w[k] = o[k];
          }
          *reinterpret_cast<Raw*>(dr + row * d + v * V) = LnVec<T>::pack(w);
        }
      }
    }
  }
#pragma unroll
  for (int j = 0; j < NV; j++) {
    const int v = lane + 64 * j;
    if (v < nvec) {
#pragma unroll
      for (int k = 0; k < V; k++) {
        partials[(wave * 2 + 0) * d + v * V + k] = sb[j][k];
        partials[(wave * 2 + 1) * d + v * V + k] = sg[j][k];
      }
    }
  }
}

// Any d, any alignment: one wave per row, scalar accesses, the row re-read per pass.
template <typename T>
__global__ void __launch_bounds__(256) ln_fwd_generic_k(const T* __restrict__ a, const T* __restrict__ r,
                                                        const T* __restrict__ gamma, const T* __restrict__ beta,
                                                        T* __restrict__ y, float* __restrict__ stats, int64_t rows, int d) {
  const int lane = threadIdx.x & 63;
  const int64_t wave = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6), nwaves = (int64_t)gridDim.x * 4;
  for (int64_t row = wave; row < rows; row += nwaves) {
    float sum = 0.f;
    for (int c = lane; c < d; c += 64) sum += Cvt<T>::ld(a[row * d + c]) + (r ? Cvt<T>::ld(r[row * d + c]) : 0.f);
    const float mean = wave_sum(sum) / (float)d;
    float sq = 0.f;
    for (int c = lane; c < d; c += 64) {
      const float v = Cvt<T>::ld(a[row * d + c]) + (r ? Cvt<T>::ld(r[row * d + c]) : 0.f) - mean;
      sq += v * v;
    }
    const float rstd = rsqrtf(wave_sum(sq) / (float)d + kLnEps);
    if (lane == 0 && stats) { stats[row * 2] = mean; stats[row * 2 + 1] = rstd; }
    for (int c = lane; c < d; c += 64) {
      const float v = Cvt<T>::ld(a[row * d + c]) + (r ? Cvt<T>::ld(r[row * d + c]) : 0.f);
      y[row * d + c] = Cvt<T>::st((v - mean) * rstd * Cvt<T>::ld(gamma[c]) + Cvt<T>::ld(beta[c]));
    }
  }
}

// Generic backward: one wave per row for dx (no column sums here; see ln_colsum_generic_k).
template <typename T>
__global__ void __launch_bounds__(256) ln_bwd_generic_k(const T* __restrict__ dy, const T* __restrict__ a,
                                                        const T* __restrict__ r, const T* __restrict__ gamma,
                                                        const float* __restrict__ stats, T* __restrict__ da, int acc_a,
                                                        T* __restrict__ dr, int acc_r, int64_t rows, int d) {
  const int lane = threadIdx.x & 63;
  const int64_t wave = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6), nwaves = (int64_t)gridDim.x * 4;
  for (int64_t row = wave; row < rows; row += nwaves) {
    const float mean = stats[row * 2], rstd = stats[row * 2 + 1];
    float s1 = 0.f, s2 = 0.f;
    for (int c = lane; c < d; c += 64) {
      const float xh = (Cvt<T>::ld(a[row * d + c]) + (r ? Cvt<T>::ld(r[row * d + c]) : 0.f) - mean) * rstd;
      const float gy = Cvt<T>::ld(dy[row * d + c]) * Cvt<T>::ld(gamma[c]);
      s1 += gy;
      s2 += gy * xh;
    }
    const float m1 = wave_sum(s1) / (float)d, m2 = wave_sum(s2) / (float)d;
    for (int c = lane; c < d; c += 64) {
      const float xh = (Cvt<T>::ld(a[row * d + c]) + (r ? Cvt<T>::ld(r[row * d + c]) : 0.f) - mean) * rstd;
      const float gy = Cvt<T>::ld(dy[row * d + c]) * Cvt<T>::ld(gamma[c]);
      const float o = rstd * (gy - m1 - xh * m2);
      if (da) da[row * d + c] = Cvt<T>::st(o + (acc_a ? Cvt<T>::ld(da[row * d + c]) : 0.f));
      if (dr) dr[row * d + c] = Cvt<T>::st(o + (acc_r ? Cvt<T>::ld(dr[row * d + c]) : 0.f));
    }
  }
}
// Generic column sums: thread = column, block y = row slice; partials [slices][2][d].
template <typename T>
__global__ void __launch_bounds__(256) ln_colsum_generic_k(const T* __restrict__ dy, const T* __restrict__ a,
                                                           const T* __restrict__ r, const float* __restrict__ stats,
                                                           float* __restrict__ partials, int64_t rows, int d) {
  const int c = blockIdx.x * 256 + threadIdx.x;
  if (c >= d) return;
  float sb = 0.f, sg = 0.f;
  for (int64_t row = blockIdx.y; row < rows; row += gridDim.y) {
    const float xh = (Cvt<T>::ld(a[row * d + c]) + (r ? Cvt<T>::ld(r[row * d + c]) : 0.f) - stats[row * 2]) * stats[row * 2 + 1];
    const float u = Cvt<T>::ld(dy[row * d + c]);
    sb += u;
    sg += u * xh;
  }
  partials[((int64_t)blockIdx.y * 2 + 0) * d + c] = sb;
  partials[((int64_t)blockIdx.y * 2 + 1) * d + c] = sg;
}

// Adds the per-wave partials in a fixed order: block = 64 columns x 16 lanes, every lane adds every
// 16th partial, the 16 lanes of a column are combined in LDS.
__global__ void __launch_bounds__(1024) ln_finalize_k(const float* __restrict__ partials, int chunks, int d,
                                                      float* __restrict__ dgamma, float* __restrict__ dbeta) {
  __shared__ float sm[2][16][64];
  const int cl = threadIdx.x & 63, lane = threadIdx.x >> 6;
  const int c = blockIdx.x * 64 + cl;
  float a0 = 0.f, a1 = 0.f;
  if (c < d) {
#pragma unroll 4
    for (int j = lane; j < chunks; j += 16) {
      a0 += partials[((int64_t)j * 2 + 0) * d + c];
      a1 += partials[((int64_t)j * 2 + 1) * d + c];
    }
  }
  sm[0][lane][cl] = a0;
  sm[1][lane][cl] = a1;
  __syncthreads();
  if (lane != 0 || c >= d) return;
  float s0 = 0.f, s1 = 0.f;
#pragma unroll
  for (int j = 0; j < 16; j++) { s0 += sm[0][j][cl]; s1 += sm[1][j][cl]; }
  dbeta[c] = s0;
  dgamma[c] = s1;
}

// waves to launch.  Backward: enough to fill the chip, few enough that the per-wave partials stay
// small.  Forward: a wave per row up to 64 Ki waves (a row's load, reductions and store are serial).
static int ln_blocks(int64_t rows, int64_t max_waves = 1024) {
  int64_t waves = rows < max_waves ? rows : max_waves;
  return (int)cdiv(waves, 4);
}

template <typename T>
static void ln_forward_t(const T* a, const T* r, const T* gamma, const T* beta, T* y, float* stats, int64_t rows, int d,
                         hipStream_t s) {
  constexpr int V = LnVec<T>::N;
  const bool vec = d % V == 0 && aligned16(a) && aligned16(r) && aligned16(gamma) && aligned16(beta) && aligned16(y) &&
                   d <= 64 * 8 * V;
  const dim3 grid(ln_blocks(rows, 65536)), block(256);
  if (!vec) {
    hipLaunchKernelGGL((ln_fwd_generic_k<T>), grid, block, 0, s, a, r, gamma, beta, y, stats, rows, d);
    return;
  }
  const int nv = (int)cdiv(d / V, 64);
#define CD_LN_FWD(NV) hipLaunchKernelGGL((ln_fwd_k<T, NV>), grid, block, 0, s, a, r, gamma, beta, y, stats, rows, d)
  if (nv <= 1) CD_LN_FWD(1); else if (nv <= 2) CD_LN_FWD(2); else if (nv <= 4) CD_LN_FWD(4); else CD_LN_FWD(8);
#undef CD_LN_FWD
}

template <typename T>
static void ln_backward_t(const T* dy, const T* a, const T* r, const T* gamma, const float* stats, T* da, bool acc_a,
                          T* dr, bool acc_r, float* dgamma, float* dbeta, float* partials, int64_t rows, int d,
                          hipStream_t s) {
  constexpr int V = LnVec<T>::N;
  const bool vec = d % V == 0 && aligned16(dy) && aligned16(a) && aligned16(r) && aligned16(gamma) && aligned16(da) &&
                   aligned16(dr) && d <= 64 * 2 * V;   // (the row, its gradient and the running sums stay in registers)
  const int blocks = ln_blocks(rows);
  int chunks;
  if (vec) {
    const int nv = (int)cdiv(d / V, 64);
    chunks = blocks * 4;
#define CD_LN_BWD(NV)                                                                                          \
  hipLaunchKernelGGL((ln_bwd_k<T, NV>), dim3(blocks), dim3(256), 0, s, dy, a, r, gamma, stats, da, (int)acc_a, dr, \
                     (int)acc_r, partials, rows, d)
    if (nv <= 1) CD_LN_BWD(1); else CD_LN_BWD(2);
#undef CD_LN_BWD
  } else {
    hipLaunchKernelGGL((ln_bwd_generic_k<T>), dim3(blocks), dim3(256), 0, s, dy, a, r, gamma, stats, da, (int)acc_a, dr,
                       (int)acc_r, rows, d);
    chunks = rows < 64 ? (int)rows : 64;
    hipLaunchKernelGGL((ln_colsum_generic_k<T>), dim3((unsigned)cdiv(d, 256), chunks), dim3(256), 0, s, dy, a, r, stats,
                       partials, rows, d);
  }
  hipLaunchKernelGGL(ln_finalize_k, dim3((unsigned)cdiv(d, 64)), dim3(1024), 0, s, partials, chunks, d, dgamma, dbeta);
}

void ln_forward(int dtype, const void* a, const void* r, const void* gamma, const void* beta, void* y, float* stats,
                int64_t rows, int d, hipStream_t s) {
  if (dtype == CD_BF16)
    ln_forward_t<bf16_t>((const bf16_t*)a, (const bf16_t*)r, (const bf16_t*)gamma, (const bf16_t*)beta, (bf16_t*)y, stats,
                         rows, d, s);
  else
    ln_forward_t<float>((const float*)a, (const float*)r, (const float*)gamma, (const float*)beta, (float*)y, stats, rows,
                        d, s);
}

void ln_backward(int dtype, const void* dy, const void* a, const void* r, const void* gamma, const float* stats, void* da,
                 bool acc_a, void* dr, bool acc_r, float* dgamma, float* dbeta, float* partials, int64_t rows, int d,
                 hipStream_t s) {
  if (dtype == CD_BF16)
    ln_backward_t<bf16_t>((const bf16_t*)dy, (const bf16_t*)a, (const bf16_t*)r, (const bf16_t*)gamma, stats, (bf16_t*)da,
                          acc_a, (bf16_t*)dr, acc_r, dgamma, dbeta, partials, rows, d, s);
  else
    ln_backward_t<float>((const float*)dy, (const float*)a, (const float*)r, (const float*)gamma, stats, (float*)da, acc_a,
                         (float*)dr, acc_r, dgamma, dbeta, partials, rows, d, s);
}

}  // namespace cd
