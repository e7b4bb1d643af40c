// Fused codistillation loss: row-wise log-softmax, cross-entropy, distillation term and the
// gradient with respect to the local logits, in one pass over HBM.
//
// Paper, Algorithm 1: the objective is L(y, z) + alpha * mean over peers of D(z, z').  D is the
// mean squared error between raw logits (appendix "Implementation Details") or the KL divergence
// of the prior work named in Section 2, or the squared error between logits centred per row (the
// variant the same appendix reports trying).  Peer logits are constants (Section 3).
//
// HBM-bound: each logit of z and z' is read once and each gradient element written once
// (12 bytes per logit pair).  A row lives in registers between the reduction and the gradient:
// one group of TPR threads owns one row, every thread holds V float4 of z and V float4 of z'.
#include "common.h"
#include <math.h>
#include <mutex>

namespace cd {

// Streaming accesses for wide rows: every logit is read once and every gradient element written once, so the
// loads and stores of the register-resident kernel carry the non-temporal hint (measured at 8192 x 32768:
// 5.1 -> 5.5 TB/s; a plain two-reads-one-write copy goes from 6.0 to 6.4 TB/s with it).
typedef float f32x4_nt __attribute__((ext_vector_type(4)));
template <bool NT>
__device__ inline float4 load4(const float* p) {
  if (NT) {
    const f32x4_nt v = __builtin_nontemporal_load(reinterpret_cast<const f32x4_nt*>(p));
    return make_float4(v.x, v.y, v.z, v.w);
  }
  return *reinterpret_cast<const float4*>(p);
}
template <bool NT>
__device__ inline void store4(float* p, float4 v) {
  if (NT) {
    const f32x4_nt q = {v.x, v.y, v.z, v.w};
    __builtin_nontemporal_store(q, reinterpret_cast<f32x4_nt*>(p));
  } else {
    *reinterpret_cast<float4*>(p) = v;
  }
}

struct LossArgs {
  const float* z;
  const float* zp[CD_LOSS_MAX_PEERS];
  const int32_t* targets;
  float* dz;
  int64_t rows, cols;
  float alpha, eps;
  float tau, inv_tau;   // temperature of the KL term (1 = the paper's); only the generic kernel reads it
  int32_t dist, mse_reduction, ignore_index, n_peers;
  int32_t* meta;    // [0] number of valid rows, [1] status bits
  float* row_task;  // [rows]
  float* row_dist;  // [rows] un-normalised per-row distillation sums (summed over peers)
};

// ---- step 1: count valid rows ---------------------------------------------------------------
__global__ void __launch_bounds__(1024) loss_prep_kernel(LossArgs a) {
  __shared__ int s_cnt[16], s_bad[16];
  int cnt = 0, bad = 0;
  for (int64_t r = threadIdx.x; r < a.rows; r += 1024) {
    int t = a.targets[r];
    if (t == a.ignore_index) continue;
    if (t < 0 || t >= a.cols) bad = 1; else cnt++;
  }
  for (int o = 32; o > 0; o >>= 1) {
    cnt += __shfl_xor(cnt, o, 64);
    bad |= __shfl_xor(bad, o, 64);
  }
  if ((threadIdx.x & 63) == 0) { s_cnt[threadIdx.x >> 6] = cnt; s_bad[threadIdx.x >> 6] = bad; }
  __syncthreads();
  if (threadIdx.x == 0) {
    int c = 0, b = 0;
    for (int i = 0; i < 16; i++) { c += s_cnt[i]; b |= s_bad[i]; }
    a.meta[0] = c;
    a.meta[1] = b;
  }
}

// Reduce NV values at once over a group of TPR threads (TPR = 64: one wave, no LDS; otherwise the
// group is the whole block).  MAXMASK bit i set -> value i is reduced with max, else with sum.
template <int TPR, int NV, unsigned MAXMASK>
__device__ inline void group_reduce(float (&v)[NV], float* smem) {
#pragma unroll
  for (int i = 0; i < NV; i++) v[i] = ((MAXMASK >> i) & 1) ? wave_max(v[i]) : wave_sum(v[i]);
  if (TPR > 64) {
    constexpr int NW = TPR / 64;
    const int w = threadIdx.x >> 6;
    __syncthreads();  // smem may still be read from a previous call
    if ((threadIdx.x & 63) == 0) {
#pragma unroll
      for (int i = 0; i < NV; i++) smem[i * NW + w] = v[i];
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < NV; i++) {
      float r = smem[i * NW];
      for (int k = 1; k < NW; k++) r = ((MAXMASK >> i) & 1) ? fmaxf(r, smem[i * NW + k]) : r + smem[i * NW + k];
      v[i] = r;
    }
  }
}

__device__ inline bool row_target(const LossArgs& a, int64_t row, int& t) {
  t = a.targets[row];
  return t != a.ignore_index && t >= 0 && t < a.cols;
}

// MODE: 0 = no peer, 1 = MSE between logits, 2 = KL(p'||p), 3 = MSE between logits centred per row
// (one peer only).
template <int TPR, int V, int MODE>
__global__ void __launch_bounds__((TPR > 256 ? TPR : 256)) loss_row_kernel(LossArgs a) {
  constexpr int BLOCK = TPR > 256 ? TPR : 256;
  constexpr bool NT = TPR * V * 4 > 8192;   // rows of more than 32 KiB stream past the caches
  constexpr int RPB = BLOCK / TPR;
  __shared__ float smem[5 * 16];
  const int g = threadIdx.x / TPR;      // row group inside the block
  const int lane = threadIdx.x % TPR;   // thread inside the group
  const int64_t row = (int64_t)blockIdx.x * RPB + g;
  if (RPB > 1 && row >= a.rows) return;  // only wave-sized groups can leave early (no barriers)
  const int64_t cols = a.cols;
  // dz may be the buffer of z (in place): neither pointer is restrict-qualified, and everything the
  // row needs from z (its elements and z[target]) is loaded before the first store.
  const float* zr = a.z + row * cols;
  const float* __restrict__ pr = MODE ? a.zp[0] + row * cols : nullptr;
  float* outr = a.dz + row * cols;
  // The row's loads are issued before anything that depends on the target (whose own load would
  // otherwise sit in front of them as a full memory latency).
  float4 x[V], y[V];
#pragma unroll
  for (int i = 0; i < V; i++) {
    int64_t c = ((int64_t)i * TPR + lane) * 4;
    if (c < cols) {
      x[i] = load4<NT>(zr + c);
      if (MODE) y[i] = load4<NT>(pr + c);
    } else {
      x[i] = make_float4(-INFINITY, -INFINITY, -INFINITY, -INFINITY);
      if (MODE) y[i] = x[i];
    }
  }
  // Several peers (MSE only): the gradient needs z - mean_j z'_j and the loss sum_j (z - z'_j)^2, so each
  // further peer is folded in as it arrives: its squared distance into a scalar, its logits into the
  // running sum that takes the place of z'.  (One peer: sq_extra stays 0 and y is that peer.)
  float sq_extra = 0.f;
  const bool many = MODE == 1 && a.n_peers > 1;
  if (many) {
#pragma unroll
    for (int i = 0; i < V; i++) {   // the first peer, already in y
      int64_t c = ((int64_t)i * TPR + lane) * 4;
      if (c < cols) {
        const float d0 = x[i].x - y[i].x, d1 = x[i].y - y[i].y, d2 = x[i].z - y[i].z, d3 = x[i].w - y[i].w;
        sq_extra += d0 * d0 + d1 * d1 + d2 * d2 + d3 * d3;
      }
    }
    for (int j = 1; j < a.n_peers; j++) {
      const float* __restrict__ pj = a.zp[j] + row * cols;
#pragma unroll
      for (int i = 0; i < V; i++) {
        int64_t c = ((int64_t)i * TPR + lane) * 4;
        if (c < cols) {
          const float4 t = load4<NT>(pj + c);
          const float d0 = x[i].x - t.x, d1 = x[i].y - t.y, d2 = x[i].z - t.z, d3 = x[i].w - t.w;
          sq_extra += d0 * d0 + d1 * d1 + d2 * d2 + d3 * d3;
          y[i].x += t.x; y[i].y += t.y; y[i].z += t.z; y[i].w += t.w;
        }
      }
    }
    const float inv_n = 1.f / (float)a.n_peers;
#pragma unroll
    for (int i = 0; i < V; i++) {   // y becomes the mean over the peers
      y[i].x *= inv_n; y[i].y *= inv_n; y[i].z *= inv_n; y[i].w *= inv_n;
    }
  }
  int t;
  const bool valid = row_target(a, row, t);
  const int nvalid = a.meta[0];
  if (!valid) {  // uniform over the group
#pragma unroll
    for (int i = 0; i < V; i++) {
      int64_t c = ((int64_t)i * TPR + lane) * 4;
      if (c < cols) store4<NT>(outr + c, make_float4(0.f, 0.f, 0.f, 0.f));
    }
    if (lane == 0) { a.row_task[row] = 0.f; a.row_dist[row] = 0.f; }
    return;
  }
  const float zt = zr[t];
  // row maxima
  float mx[2] = {-INFINITY, -INFINITY};
#pragma unroll
  for (int i = 0; i < V; i++) {
    mx[0] = fmaxf(mx[0], fmaxf(fmaxf(x[i].x, x[i].y), fmaxf(x[i].z, x[i].w)));
    if (MODE == 2) mx[1] = fmaxf(mx[1], fmaxf(fmaxf(y[i].x, y[i].y), fmaxf(y[i].z, y[i].w)));
  }
  group_reduce<TPR, 2, 3u>(mx, smem);
  const float m = mx[0], mp = mx[1];
  // sums: [0] sum exp(z-m)  [1] sum z  [2] MSE: sum (z-z')^2 | KL: sum exp(z'-m')
  //       [3] KL: sum exp(z'-m')(z'-z) | centred MSE: sum (z-z')
  // The registers are reused for what the gradient needs: z becomes e = exp(z-m), z' becomes z-z'
  // (MSE) or e' = exp(z'-m') (KL), so that the gradient costs no second exponential per element.
  float s[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int i = 0; i < V; i++) {
    int64_t c = ((int64_t)i * TPR + lane) * 4;
    if (c < cols) {
      float xv[4] = {x[i].x, x[i].y, x[i].z, x[i].w};
      float yv[4] = {MODE ? y[i].x : 0.f, MODE ? y[i].y : 0.f, MODE ? y[i].z : 0.f, MODE ? y[i].w : 0.f};
#pragma unroll
      for (int k = 0; k < 4; k++) {
        const float e = __expf(xv[k] - m);
        s[0] += e;
        s[1] += xv[k];
        if (MODE == 1) { const float d = xv[k] - yv[k]; s[2] += many ? 0.f : d * d; yv[k] = d; }
        if (MODE == 2) { const float ep = __expf(yv[k] - mp); s[2] += ep; s[3] += ep * (yv[k] - xv[k]); yv[k] = ep; }
        if (MODE == 3) { const float d = xv[k] - yv[k]; s[3] += d; yv[k] = d; }
        xv[k] = e;
      }
      x[i] = make_float4(xv[0], xv[1], xv[2], xv[3]);
      if (MODE) y[i] = make_float4(yv[0], yv[1], yv[2], yv[3]);
    }
  }
  s[2] += sq_extra;
  group_reduce<TPR, 4, 0u>(s, smem);
  if (MODE == 3) {
    // Centring both rows subtracts the mean of z - z' from their difference.  The squared error is
    // summed from the centred differences (not as sum d^2 - C mean^2, which cancels when the two
    // models differ mostly by a constant).
    const float md = s[3] / (float)cols;
    float q[1] = {0.f};
#pragma unroll
    for (int i = 0; i < V; i++) {
      int64_t c = ((int64_t)i * TPR + lane) * 4;
      if (c < cols) {
        y[i].x -= md; y[i].y -= md; y[i].z -= md; y[i].w -= md;
        q[0] += y[i].x * y[i].x + y[i].y * y[i].y + y[i].z * y[i].z + y[i].w * y[i].w;
      }
    }
    group_reduce<TPR, 1, 0u>(q, smem);
    s[2] = q[0];
  }
  const float lse = m + logf(s[0]);
  float lsep = 0.f;
  if (MODE == 2) lsep = mp + logf(s[2]);
  if (lane == 0) {
    a.row_task[row] = lse - (1.f - a.eps) * zt - (a.eps / (float)cols) * s[1];
    float d = 0.f;
    if (MODE == 1 || MODE == 3) d = s[2];
    if (MODE == 2) d = s[3] / s[2] - lsep + lse;
    a.row_dist[row] = d;
  }
  // gradient: p = e / sum e, p' = e' / sum e'
  const float invn = 1.f / (float)nvalid;
  const float epsc = a.eps / (float)cols;
  float cm = 0.f;
  if (MODE == 1 || MODE == 3) cm = a.alpha * 2.f * invn / (a.mse_reduction == CD_MEAN_ALL ? (float)cols : 1.f);
  const float onehot = (1.f - a.eps) * invn;
  const float fp = invn / s[0];                                   // p * invn = e * fp
  const float fq = MODE == 2 ? invn / s[2] : 0.f;                 // p' * invn = e' * fq (same form as fp: an identical peer cancels exactly)
  const float base = -epsc * invn;
#pragma unroll
  for (int i = 0; i < V; i++) {
    int64_t c = ((int64_t)i * TPR + lane) * 4;
    if (c < cols) {
      const float xv[4] = {x[i].x, x[i].y, x[i].z, x[i].w};
      const float yv[4] = {MODE ? y[i].x : 0.f, MODE ? y[i].y : 0.f, MODE ? y[i].z : 0.f, MODE ? y[i].w : 0.f};
      float o[4];
#pragma unroll
      for (int k = 0; k < 4; k++) {
        float gk = xv[k] * fp + base;
        if (MODE == 1 || MODE == 3) gk += cm * yv[k];
        if (MODE == 2) gk += a.alpha * (__fmul_rn(xv[k], fp) - __fmul_rn(yv[k], fq));  // no fma: exact cancellation
        if (c + k == t) gk -= onehot;
        o[k] = gk;
      }
      store4<NT>(outr + c, make_float4(o[0], o[1], o[2], o[3]));
    }
  }
}

// Any column count, any number of peers: one block per row, several passes over the row (later
// passes hit in cache).  Scalar accesses, so rows need no alignment.
__global__ void __launch_bounds__(256) loss_row_generic_kernel(LossArgs a) {
  __shared__ float smem[5 * 4];
  __shared__ float s_lsep[CD_LOSS_MAX_PEERS];  // KL: log-sum-exp of peer j; squared errors: mean of z - z'_j (0 uncentred)
  const bool squared = a.dist == CD_DIST_MSE_LOGITS || a.dist == CD_DIST_MSE_CENTERED;
  const int64_t row = blockIdx.x;
  const int64_t cols = a.cols;
  const float* zr = a.z + row * cols;
  float* outr = a.dz + row * cols;
  int t;
  const bool valid = row_target(a, row, t);
  const int nvalid = a.meta[0];
  if (!valid) {
    for (int64_t c = threadIdx.x; c < cols; c += 256) outr[c] = 0.f;
    if (threadIdx.x == 0) { a.row_task[row] = 0.f; a.row_dist[row] = 0.f; }
    return;
  }
  const float zt = zr[t];
  float v1[1] = {-INFINITY};
  for (int64_t c = threadIdx.x; c < cols; c += 256) v1[0] = fmaxf(v1[0], zr[c]);
  group_reduce<256, 1, 1u>(v1, smem);
  const float m = v1[0];
  float v2[2] = {0.f, 0.f};
  for (int64_t c = threadIdx.x; c < cols; c += 256) { float x = zr[c]; v2[0] += __expf(x - m); v2[1] += x; }
  group_reduce<256, 2, 0u>(v2, smem);
  const float lse = m + logf(v2[0]);
  // KL with a temperature: tau^2 KL(softmax(z'/tau) || softmax(z/tau)); lse_t = log-sum-exp of z / tau
  const float it = a.inv_tau;
  float lse_t = lse;
  if (!squared && a.n_peers > 0 && it != 1.f) {
    float u[1] = {0.f};
    for (int64_t c = threadIdx.x; c < cols; c += 256) u[0] += __expf((zr[c] - m) * it);
    group_reduce<256, 1, 0u>(u, smem);
    lse_t = m * it + logf(u[0]);
  }
  float dsum = 0.f;
  for (int j = 0; j < a.n_peers; j++) {
    const float* pr = a.zp[j] + row * cols;
    if (squared) {
      float md = 0.f;
      if (a.dist == CD_DIST_MSE_CENTERED) {
        float u[1] = {0.f};
        for (int64_t c = threadIdx.x; c < cols; c += 256) u[0] += zr[c] - pr[c];
        group_reduce<256, 1, 0u>(u, smem);
        md = u[0] / (float)cols;
      }
      float q[1] = {0.f};
      for (int64_t c = threadIdx.x; c < cols; c += 256) { float d = zr[c] - pr[c] - md; q[0] += d * d; }
      group_reduce<256, 1, 0u>(q, smem);
      dsum += q[0];
      if (threadIdx.x == 0) s_lsep[j] = md;
    } else {
      float q[1] = {-INFINITY};
      for (int64_t c = threadIdx.x; c < cols; c += 256) q[0] = fmaxf(q[0], pr[c]);
      group_reduce<256, 1, 1u>(q, smem);
      const float mp = q[0];
      float w[2] = {0.f, 0.f};
      for (int64_t c = threadIdx.x; c < cols; c += 256) {
        float y = pr[c], e = __expf((y - mp) * it);
        w[0] += e;
        w[1] += e * ((y - zr[c]) * it);
      }
      group_reduce<256, 2, 0u>(w, smem);
      const float lsep = mp * it + logf(w[0]);
      dsum += (w[1] / w[0] - lsep + lse_t) * (a.tau * a.tau);
      if (threadIdx.x == 0) s_lsep[j] = lsep;
    }
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    a.row_task[row] = lse - (1.f - a.eps) * zt - (a.eps / (float)cols) * v2[1];
    a.row_dist[row] = dsum;
  }
  const float invn = 1.f / (float)nvalid;
  const float epsc = a.eps / (float)cols;
  const float wj = a.n_peers > 0 ? 1.f / (float)a.n_peers : 0.f;
  const float cm = a.alpha * wj * 2.f * invn / (a.mse_reduction == CD_MEAN_ALL ? (float)cols : 1.f);
  const float ck = a.alpha * wj * invn * a.tau;   // d/dz of tau^2 KL = tau (p_tau - p'_tau)
  for (int64_t c = threadIdx.x; c < cols; c += 256) {
    const float x = zr[c];
    const float p = __expf(x - lse);
    const float pt = it != 1.f ? __expf(x * it - lse_t) : p;
    float gk = (p - epsc) * invn;
    for (int j = 0; j < a.n_peers; j++) {
      const float y = a.zp[j][row * cols + c];
      if (squared) gk += cm * (x - y - s_lsep[j]);
      else gk += ck * (pt - __expf(y * it - s_lsep[j]));
    }
    if (c == t) gk -= (1.f - a.eps) * invn;
    outr[c] = gk;
  }
}

// ---- step 3: deterministic sum of the per-row terms ------------------------------------------
__global__ void __launch_bounds__(1024) loss_finalize_kernel(LossArgs a, float* loss_out) {
  __shared__ double s_t[1024], s_d[1024];
  // every thread adds its rows in a fixed order, four independent loads in flight at a time
  double st[4] = {0.0, 0.0, 0.0, 0.0}, sd[4] = {0.0, 0.0, 0.0, 0.0};
  for (int64_t r0 = threadIdx.x; r0 < a.rows; r0 += 4096) {
#pragma unroll
    for (int u = 0; u < 4; u++) {
      const int64_t r = r0 + 1024 * u;
      if (r < a.rows) { st[u] += (double)a.row_task[r]; sd[u] += (double)a.row_dist[r]; }
    }
  }
  s_t[threadIdx.x] = (st[0] + st[1]) + (st[2] + st[3]);
  s_d[threadIdx.x] = (sd[0] + sd[1]) + (sd[2] + sd[3]);
  __syncthreads();
  for (int o = 512; o > 0; o >>= 1) {
    if ((int)threadIdx.x < o) { s_t[threadIdx.x] += s_t[threadIdx.x + o]; s_d[threadIdx.x] += s_d[threadIdx.x + o]; }
    __syncthreads();
  }
  if (threadIdx.x == 0) {
    const int n = a.meta[0];
    double task = 0.0, dist = 0.0;
    if (n > 0) {
      task = s_t[0] / n;
      if (a.n_peers > 0) {
        double denom = (double)n * a.n_peers;
        if ((a.dist == CD_DIST_MSE_LOGITS || a.dist == CD_DIST_MSE_CENTERED) && a.mse_reduction == CD_MEAN_ALL)
          denom *= (double)a.cols;
        dist = s_d[0] / denom;
      }
    }
    loss_out[0] = (float)(task + (double)a.alpha * dist);
    loss_out[1] = (float)task;
    loss_out[2] = (float)dist;
    reinterpret_cast<int32_t*>(loss_out)[3] = a.meta[1];
  }
}

template <int TPR, int V>
static void launch_rows(const LossArgs& a, int mode, hipStream_t s) {
  constexpr int BLOCK = TPR > 256 ? TPR : 256;
  constexpr int RPB = BLOCK / TPR;
  dim3 grid((unsigned)cdiv(a.rows, RPB));
  if (mode == 0) hipLaunchKernelGGL((loss_row_kernel<TPR, V, 0>), grid, dim3(BLOCK), 0, s, a);
  else if (mode == 1) hipLaunchKernelGGL((loss_row_kernel<TPR, V, 1>), grid, dim3(BLOCK), 0, s, a);
  else if (mode == 3) hipLaunchKernelGGL((loss_row_kernel<TPR, V, 3>), grid, dim3(BLOCK), 0, s, a);
  else hipLaunchKernelGGL((loss_row_kernel<TPR, V, 2>), grid, dim3(BLOCK), 0, s, a);
}

}  // namespace cd

using namespace cd;

static size_t loss_scratch_need(int64_t rows) { return 16 + align_up((size_t)rows * 4, 16) * 2; }

extern "C" int codistill_loss_scratch_bytes(int64_t rows, int64_t cols, size_t* bytes) {
  CD_REQUIRE(bytes != nullptr, "loss_scratch_bytes: bytes is NULL");
  CD_REQUIRE(rows >= 1 && rows <= 2147483647LL, "loss_scratch_bytes: rows=%lld out of range", (long long)rows);
  CD_REQUIRE(cols >= 1 && cols <= (1LL << 24), "loss_scratch_bytes: cols=%lld out of range", (long long)cols);
  *bytes = loss_scratch_need(rows);
  return CD_OK;
}

// Validation and launches shared by the two entry points; `scratch` is device memory of at least
// loss_scratch_need(rows) bytes (the caller's, or this library's static array).
static int loss_grad_run(const float* z_local, const float* const* z_peers, const int32_t* targets,
                         int64_t rows, int64_t cols, const cd_loss_cfg* cfg, float* loss_out,
                         float* dz_out, void* scratch, size_t scratch_bytes, void* stream) {
  CD_REQUIRE(z_local && targets && cfg && loss_out && dz_out && scratch, "loss_grad: NULL pointer argument");
  CD_REQUIRE(rows >= 1 && rows <= 2147483647LL, "loss_grad: rows=%lld out of range [1, 2^31-1]", (long long)rows);
  CD_REQUIRE(cols >= 1 && cols <= (1LL << 24), "loss_grad: cols=%lld out of range [1, 2^24]", (long long)cols);
  CD_REQUIRE(cfg->n_peers >= 0 && cfg->n_peers <= CD_LOSS_MAX_PEERS, "loss_grad: n_peers=%d out of range [0, %d]",
             cfg->n_peers, CD_LOSS_MAX_PEERS);
  CD_REQUIRE(cfg->dist_kind == CD_DIST_MSE_LOGITS || cfg->dist_kind == CD_DIST_KL ||
                 cfg->dist_kind == CD_DIST_MSE_CENTERED,
             "loss_grad: unknown dist_kind %d", cfg->dist_kind);
  CD_REQUIRE(cfg->mse_reduction == CD_MEAN_ALL || cfg->mse_reduction == CD_MEAN_ROWS,
             "loss_grad: unknown mse_reduction %d", cfg->mse_reduction);
  CD_REQUIRE(cfg->label_smoothing >= 0.f && cfg->label_smoothing < 1.f, "loss_grad: label_smoothing %g outside [0,1)",
             (double)cfg->label_smoothing);
  CD_REQUIRE(cfg->alpha == cfg->alpha, "loss_grad: alpha is NaN");
  CD_REQUIRE(cfg->temperature >= 0.f && cfg->temperature <= 1e6f, "loss_grad: temperature %g outside [0, 1e6] (0 means 1)",
             (double)cfg->temperature);
  CD_REQUIRE(cfg->n_peers == 0 || z_peers != nullptr, "loss_grad: z_peers is NULL with n_peers=%d", cfg->n_peers);
  CD_REQUIRE(aligned16(z_local) && aligned16(dz_out) && aligned16(scratch) && aligned16(loss_out),
             "loss_grad: pointers must be 16-byte aligned");
  for (int j = 0; j < cfg->n_peers; j++)
    CD_REQUIRE(z_peers[j] != nullptr && aligned16(z_peers[j]), "loss_grad: z_peers[%d] is NULL or misaligned", j);
  if (scratch_bytes < loss_scratch_need(rows))
    return set_error(CD_ERR_WORKSPACE_TOO_SMALL, "loss_grad: scratch %zu < %zu bytes", scratch_bytes,
                     loss_scratch_need(rows));

  LossArgs a;
  a.z = z_local;
  for (int j = 0; j < CD_LOSS_MAX_PEERS; j++) a.zp[j] = j < cfg->n_peers ? z_peers[j] : nullptr;
  a.targets = targets;
  a.dz = dz_out;
  a.rows = rows;
  a.cols = cols;
  a.alpha = cfg->alpha;
  a.eps = cfg->label_smoothing;
  a.tau = cfg->temperature > 0.f ? cfg->temperature : 1.f;
  a.inv_tau = 1.f / a.tau;
  a.dist = cfg->dist_kind;
  a.mse_reduction = cfg->mse_reduction;
  a.ignore_index = cfg->ignore_index;
  a.n_peers = cfg->n_peers;
  char* sc = static_cast<char*>(scratch);
  a.meta = reinterpret_cast<int32_t*>(sc);
  a.row_task = reinterpret_cast<float*>(sc + 16);
  a.row_dist = reinterpret_cast<float*>(sc + 16 + align_up((size_t)rows * 4, 16));
  hipStream_t s = static_cast<hipStream_t>(stream);

  const double bytes = (double)rows * cols * 4.0 * (2 + cfg->n_peers);
  ProfScope prof(CD_K_LOSS, s, (double)rows * cols * 12.0, bytes);
  hipLaunchKernelGGL(loss_prep_kernel, dim3(1), dim3(1024), 0, s, a);
  const int mode = cfg->n_peers == 0 ? 0
                   : cfg->dist_kind == CD_DIST_MSE_LOGITS ? 1
                   : cfg->dist_kind == CD_DIST_KL         ? 2
                                                          : 3;
  // register-resident kernel: one peer, or several with the MSE term (folded into a running mean)
  // (a temperature other than 1 needs a second softmax of the local row: the generic kernel has it)
  const bool fast = cols % 4 == 0 && cols <= 32768 && (cfg->n_peers <= 1 || mode == 1) && (mode != 2 || a.tau == 1.f);
  if (!fast) {
    hipLaunchKernelGGL(loss_row_generic_kernel, dim3((unsigned)rows), dim3(256), 0, s, a);
  } else if (cols <= 256) launch_rows<64, 1>(a, mode, s);
  else if (cols <= 1024) launch_rows<64, 4>(a, mode, s);
  else if (cols <= 4096) launch_rows<256, 4>(a, mode, s);
  else if (cols <= 8192) launch_rows<1024, 2>(a, mode, s);
  else if (cols <= 16384) launch_rows<1024, 4>(a, mode, s);
  else launch_rows<512, 16>(a, mode, s);   // fewer, fatter threads than 1024 x 8: fewer waves to synchronise per reduction
  hipLaunchKernelGGL(loss_finalize_kernel, dim3(1), dim3(1024), 0, s, a, loss_out);
  return check_launch("loss_grad");
}

extern "C" int codistill_loss_grad(const float* z_local, const float* const* z_peers, const int32_t* targets,
                                   int64_t rows, int64_t cols, const cd_loss_cfg* cfg, float* loss_out,
                                   float* dz_out, void* scratch, size_t scratch_bytes, void* stream) {
  return loss_grad_run(z_local, z_peers, targets, rows, cols, cfg, loss_out, dz_out, scratch, scratch_bytes, stream);
}

// ---- the same call for callers that cannot allocate ---------------------------------------------
// The per-row terms and the row counter live in a device array that is part of the loaded code object
// (one copy per GPU, held until the process ends).  The array's name is only a host-side handle: its
// device address is looked up once per device and that address is what the kernels receive.
static constexpr size_t kStaticScratchBytes = 16 + 2 * (size_t)CD_LOSS_STATIC_MAX_ROWS * 4;
static __device__ __align__(256) unsigned char g_loss_static_scratch[kStaticScratchBytes];

static constexpr int kMaxDevices = 64;
static std::mutex g_static_mu;
static void* g_static_ptr[kMaxDevices] = {};

static int loss_static_scratch_ptr(void** out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) {
    (void)hipGetLastError();
    return set_error(CD_ERR_HIP, "loss_grad_static: no current device (or device index above %d)", kMaxDevices - 1);
  }
  std::lock_guard<std::mutex> lk(g_static_mu);
  if (!g_static_ptr[dev]) {
    void* p = nullptr;
    hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(g_loss_static_scratch));
    if (e != hipSuccess || !p) {
      (void)hipGetLastError();
      return set_error(CD_ERR_HIP, "loss_grad_static: hipGetSymbolAddress: %s", hipGetErrorString(e));
    }
    g_static_ptr[dev] = p;
  }
  *out = g_static_ptr[dev];
  return CD_OK;
}

extern "C" int codistill_loss_grad_static(const float* z_local, const float* const* z_peers, const int32_t* targets,
                                          int64_t rows, int64_t cols, const cd_loss_cfg* cfg, float* loss_out,
                                          float* dz_out, void* stream) {
  CD_REQUIRE(rows >= 1 && rows <= CD_LOSS_STATIC_MAX_ROWS,
             "loss_grad_static: rows=%lld outside [1, %d] (use codistill_loss_grad with a caller scratch for more rows)",
             (long long)rows, CD_LOSS_STATIC_MAX_ROWS);
  void* scratch = nullptr;
  int rc = loss_static_scratch_ptr(&scratch);
  if (rc != CD_OK) return rc;
  // Every word of the scratch that a call reads (the row counter, status bits and the first `rows` per-row terms)
  // is written earlier in the same call, so what the previous call left behind needs no clearing.
  return loss_grad_run(z_local, z_peers, targets, rows, cols, cfg, loss_out, dz_out, scratch, kStaticScratchBytes, stream);
}
