// Multi-head scaled dot-product attention (forward, backward) and the token embedding of the
// encoder-decoder Transformer that the paper trains (Section 4; Vaswani et al.).
//
// out[i] = sum_j softmax_j(q_i . k_j / sqrt(dh)) v_j per sentence and head, keys j <= i only under the
// causal mask.  q, k, v are column ranges of bf16 row-major tensors (the fused projections write
// [rows][3d] or [rows][2d]); head h owns columns h*dh .. (h+1)*dh of each range.
//
// Two sets of kernels.  Head dimensions 64 and 32 run on the matrix cores (second half of this file).  The others use
// plain fp32 arithmetic: a pair of threads owns one query (forward, dq) or one key
// (dk, dv), each thread one half of the head dimension; the dot products are completed with one
// exchange inside the pair.  The other operand streams through LDS in chunks of 64 rows, every thread
// reading the same address (a broadcast).  The forward pass keeps only the log-sum-exp of every row
// (softmax is recomputed in the backward pass), so nothing of size Tq x Tk is ever stored.
#include "common.h"
#include "kernels.h"
#include <math.h>
#include <stdlib.h>

namespace cd {

namespace {

constexpr int ATT_ROWS = 128;  // rows (queries or keys) per workgroup: two threads each
constexpr int ATT_KC = 64;     // rows of the streamed operand per LDS chunk

__device__ inline float pair_sum(float v) { return v + __shfl_xor(v, 1, 64); }

// bf16 row (row pitch ld elements) -> n floats at dst, 8 at a time
__device__ inline void load_bf16_8(const bf16_t* p, float* dst) {
  const uint4 u = *reinterpret_cast<const uint4*>(p);
  const uint32_t w[4] = {u.x, u.y, u.z, u.w};
#pragma unroll
  for (int q = 0; q < 4; q++) {
    dst[2 * q] = __uint_as_float(w[q] << 16);
    dst[2 * q + 1] = __uint_as_float(w[q] & 0xffff0000u);
  }
}

// A chunk of up to ATT_KC rows x DH columns of a bf16 tensor into LDS as fp32 (rows past n are zero).
template <int DH>
__device__ inline void stage_chunk(const bf16_t* __restrict__ base, int64_t ld, int n, float* __restrict__ dst) {
  constexpr int VPR = DH / 8;  // 16-byte vectors per row
  for (int v = threadIdx.x; v < ATT_KC * VPR; v += 256) {
    const int r = v / VPR, c = (v % VPR) * 8;
    float t[8];
    if (r < n) load_bf16_8(base + (int64_t)r * ld + c, t);
    else {
#pragma unroll
      for (int e = 0; e < 8; e++) t[e] = 0.f;
    }
#pragma unroll
    for (int e = 0; e < 8; e++) dst[r * DH + c + e] = t[e];
  }
}

struct AttArgs {
  const bf16_t* q; const bf16_t* k; const bf16_t* v;   // already offset to their first column
  int64_t ldq, ldkv;                                  // row pitches in elements
  bf16_t* out; int64_t ldo;                           // forward output [S*Tq][d]
  float* lse;                                         // [S][heads][Tq] log-sum-exp of the scaled scores
  float* dsum;                                        // [S][heads][Tq] backward: dO . O per row
  const bf16_t* dout;                                 // backward: gradient of out, pitch ldo
  bf16_t* dq; bf16_t* dk; bf16_t* dv;                 // backward outputs, pitches ldq / ldkv
  int S, heads, Tq, Tk, causal;
  float scale;                                        // 1 / sqrt(dh)
  // Padding (nullable): token ids [S][tok_pitch]; the keys of sentence s come from columns ktok0 .. ktok0 + Tk,
  // and only those before the first negative id are real.
  const int32_t* ktok; int64_t tok_pitch; int ktok0;
  // Packed sentences (nullable, both or neither): tables of max_sent + 2 entries, [i] = first row of sentence i of the
  // query / key tensor, [n] = one past the last row of the last sentence, [max_sent + 1] = n, the number of sentences.
  // S is then max_sent, Tq and Tk the longest sentence the launch covers, and lse / dsum are [heads][lse_rows],
  // indexed by the query's row in its tensor.
  // The workgroups of "sentence" n (the grid has max_sent + 1 of them) clear the rows behind the last sentence in what
  // the kernel writes, so that no tensor holds rows that were never written (k_rows: rows of the key tensor).
  const int32_t* q_tab; const int32_t* k_tab; int max_sent; int lse_rows; int k_rows;
};

// Number of real keys of sentence s (at least 1), the same value in every thread of the workgroup.
// Contains barriers: every thread of the workgroup calls it.
__device__ inline int key_count(const AttArgs& a, int s) {
  if (!a.ktok) return a.Tk;
  int n = 0;
  for (int j0 = 0; j0 < a.Tk; j0 += 256) {
    const int j = j0 + (int)threadIdx.x;
    n += __syncthreads_count(j < a.Tk && a.ktok[(int64_t)s * a.tok_pitch + a.ktok0 + j] >= 0);
  }
  return max(n, 1);
}

// Where sentence s lives: first row and number of rows of its queries and of its keys, number of real keys, and the
// first element of its rows in lse / dsum (head h).  Padded batches: every sentence has Tq and Tk rows.  Packed
// batches: rows and lengths come from the tables.  Returns SEG_ROWS for a sentence, SEG_TAIL for the index right
// behind the last sentence (qrow / krow are then the first rows that belong to no sentence), SEG_NONE beyond that:
// in the last two cases the whole workgroup leaves.  Contains barriers (key_count): every thread of the workgroup calls it.
struct Seg { int qrow, Tq, krow, Tk, nk; int64_t lrow; };
enum { SEG_NONE = 0, SEG_ROWS = 1, SEG_TAIL = 2 };
__device__ inline int segment(const AttArgs& a, int s, int h, Seg& g) {
  if (!a.q_tab) {
    g.qrow = s * a.Tq; g.Tq = a.Tq; g.krow = s * a.Tk; g.Tk = a.Tk;
    g.nk = key_count(a, s);
    g.lrow = ((int64_t)s * a.heads + h) * a.Tq;
    return SEG_ROWS;
  }
  const int n = min(min(a.q_tab[a.max_sent + 1], a.k_tab[a.max_sent + 1]), a.max_sent);
  if (s > n) return SEG_NONE;
  g.qrow = a.q_tab[s];
  g.krow = a.k_tab[s];
  if (s == n) return SEG_TAIL;
  g.Tq = min(a.q_tab[s + 1] - g.qrow, a.Tq);
  g.Tk = min(a.k_tab[s + 1] - g.krow, a.Tk);
  g.nk = g.Tk;
  g.lrow = (int64_t)h * a.lse_rows + g.qrow;
  return g.Tq > 0 && g.Tk > 0 ? SEG_ROWS : SEG_NONE;
}
// zeros in columns h*DH .. (h+1)*DH of rows first .. rows of a bf16 tensor with row pitch ld (the whole workgroup)
template <int DH>
__device__ inline void clear_rows(bf16_t* __restrict__ p, int64_t ld, int first, int rows, int h) {
  constexpr int VPR = DH / 8;
  for (int v = threadIdx.x; v < (rows - first) * VPR; v += 256)
    *reinterpret_cast<uint4*>(p + (int64_t)(first + v / VPR) * ld + h * DH + (v % VPR) * 8) = make_uint4(0, 0, 0, 0);
}

// blockIdx.x = (sentence * heads + head) * tiles + tile of ATT_ROWS queries
template <int DH>
__global__ void __launch_bounds__(256) attn_fwd_k(AttArgs a) {
  constexpr int HALF = DH / 2;
  __shared__ float Ks[ATT_KC * DH], Vs[ATT_KC * DH];
  const int tiles = (a.Tq + ATT_ROWS - 1) / ATT_ROWS;
  const int tile = blockIdx.x % tiles, sh = blockIdx.x / tiles;
  const int h = sh % a.heads, s = sh / a.heads;
  Seg sg;
  const int seg = segment(a, s, h, sg);
  if (seg != SEG_ROWS) {   // (packed batches) no such sentence; the first index behind the last one clears the unused rows
    if (seg == SEG_TAIL && tile == 0) clear_rows<DH>(a.out, a.ldo, sg.qrow, a.lse_rows, h);
    return;
  }
  if (tile * ATT_ROWS >= sg.Tq) return;   // (packed batches) the sentence ends before this tile
  const int i = tile * ATT_ROWS + (threadIdx.x >> 1), hf = threadIdx.x & 1;
  const bool live = i < sg.Tq;
  float q[HALF], o[HALF];
#pragma unroll
  for (int c = 0; c < HALF; c++) { q[c] = 0.f; o[c] = 0.f; }
  if (live) {
    const bf16_t* qp = a.q + ((int64_t)sg.qrow + i) * a.ldq + h * DH + hf * HALF;
#pragma unroll
    for (int c = 0; c < HALF; c++) q[c] = bf16_to_f32(qp[c]) * a.scale;
  }
  float m = -INFINITY, l = 0.f;
  const int nk = sg.nk;
  const int last = a.causal ? min(nk, tile * ATT_ROWS + ATT_ROWS) : nk;   // keys any query of the tile sees
  for (int j0 = 0; j0 < last; j0 += ATT_KC) {
    const int n = min(ATT_KC, nk - j0);
    __syncthreads();
    stage_chunk<DH>(a.k + ((int64_t)sg.krow + j0) * a.ldkv + h * DH, a.ldkv, n, Ks);
    stage_chunk<DH>(a.v + ((int64_t)sg.krow + j0) * a.ldkv + h * DH, a.ldkv, n, Vs);
    __syncthreads();
    for (int j = 0; j < n; j++) {
      float part = 0.f;
#pragma unroll
      for (int c = 0; c < HALF; c++) part += q[c] * Ks[j * DH + hf * HALF + c];
      const float sc = pair_sum(part);
      if (!live || (a.causal && j0 + j > i)) continue;
      if (sc > m) {   // a new maximum: rescale what has been accumulated (rare after the first keys)
        const float r = __expf(m - sc);
        l *= r;
#pragma unroll
        for (int c = 0; c < HALF; c++) o[c] *= r;
        m = sc;
      }
      const float p = __expf(sc - m);
      l += p;
#pragma unroll
      for (int c = 0; c < HALF; c++) o[c] += p * Vs[j * DH + hf * HALF + c];
    }
  }
  if (!live) return;
  const float inv = 1.f / l;
  bf16_t* op = a.out + ((int64_t)sg.qrow + i) * a.ldo + h * DH + hf * HALF;
#pragma unroll
  for (int c = 0; c < HALF; c++) op[c] = f32_to_bf16(o[c] * inv);
  if (hf == 0 && a.lse) a.lse[sg.lrow + i] = m + __logf(l);
}

// dq: one pair of threads per query.  p_ij = exp(s_ij - lse_i); D_i = dO_i . O_i = sum_j p_ij dP_ij;
// dS_ij = p_ij (dP_ij - D_i); dq_i = scale * sum_j dS_ij k_j.  D_i is accumulated on the way (first
// pass over the keys) so that the stored output is not needed, then dq in a second pass.
template <int DH>
__global__ void __launch_bounds__(256) attn_bwd_dq_k(AttArgs a) {
  constexpr int HALF = DH / 2;
  __shared__ float Ks[ATT_KC * DH], Vs[ATT_KC * DH];
  const int tiles = (a.Tq + ATT_ROWS - 1) / ATT_ROWS;
  const int tile = blockIdx.x % tiles, sh = blockIdx.x / tiles;
  const int h = sh % a.heads, s = sh / a.heads;
  Seg sg;
  const int seg = segment(a, s, h, sg);
  if (seg != SEG_ROWS) {   // (packed batches) no such sentence; the first index behind the last one clears the unused rows
    if (seg == SEG_TAIL && tile == 0) clear_rows<DH>(a.dq, a.ldq, sg.qrow, a.lse_rows, h);
    return;
  }
  if (tile * ATT_ROWS >= sg.Tq) return;   // (packed batches) the sentence ends before this tile
  const int i = tile * ATT_ROWS + (threadIdx.x >> 1), hf = threadIdx.x & 1;
  const bool live = i < sg.Tq;
  float q[HALF], go[HALF], dq[HALF];
#pragma unroll
  for (int c = 0; c < HALF; c++) { q[c] = 0.f; go[c] = 0.f; dq[c] = 0.f; }
  float lse = 0.f;
  if (live) {
    const bf16_t* qp = a.q + ((int64_t)sg.qrow + i) * a.ldq + h * DH + hf * HALF;
    const bf16_t* gp = a.dout + ((int64_t)sg.qrow + i) * a.ldo + h * DH + hf * HALF;
#pragma unroll
    for (int c = 0; c < HALF; c++) { q[c] = bf16_to_f32(qp[c]) * a.scale; go[c] = bf16_to_f32(gp[c]); }
    lse = a.lse[sg.lrow + i];
  }
  const int nk = sg.nk;
  const int last = a.causal ? min(nk, tile * ATT_ROWS + ATT_ROWS) : nk;
  // Where the weights are nearly uniform dq is a small difference of large terms (10^4 times smaller at the base
  // model's initialisation), so relative errors of 1e-7 in the recomputed probabilities matter.  Two measures:
  // the weights are recomputed as w_j = exp(s_j - (lse - log n)), n the number of visible keys, whose exponent is
  // near zero exactly in the uniform case (small exponents round finely), and they are normalised by their own
  // sum Z, which makes sum_j w_j (dp_j - D) vanish whatever Z is: D = sum w dp / Z, dq = sum w (dp - D) k / Z.
  // Third, dp is taken relative to the first key's (dp_j - dp_0; dp - D does not change): when the values are
  // nearly alike D then is as small as the differences, and its rounding error, which every term shares and
  // which multiplies the keys' common part, shrinks with it.
  const int visible = a.causal ? min(i + 1, nk) : nk;
  const float ref = lse - __logf((float)max(visible, 1));
  float D = 0.f, Z = 0.f, dp0 = 0.f;
  for (int pass = 0; pass < 2; pass++) {
    if (pass == 1 && Z > 0.f) D /= Z;
    for (int j0 = 0; j0 < last; j0 += ATT_KC) {
      const int n = min(ATT_KC, nk - j0);
      __syncthreads();
      stage_chunk<DH>(a.k + ((int64_t)sg.krow + j0) * a.ldkv + h * DH, a.ldkv, n, Ks);
      stage_chunk<DH>(a.v + ((int64_t)sg.krow + j0) * a.ldkv + h * DH, a.ldkv, n, Vs);
      __syncthreads();
      for (int j = 0; j < n; j++) {
        float ps = 0.f, pd = 0.f;
#pragma unroll
        for (int c = 0; c < HALF; c++) {
          ps += q[c] * Ks[j * DH + hf * HALF + c];
          pd += go[c] * Vs[j * DH + hf * HALF + c];
        }
        const float sc = pair_sum(ps);
        float dp = pair_sum(pd);
        if (!live || (a.causal && j0 + j > i)) continue;
        if (pass == 0 && j0 + j == 0) dp0 = dp;
        dp -= dp0;
        const float p = __expf(sc - ref);
        if (pass == 0) {
          D += p * dp;
          Z += p;
        } else {
          const float ds = p * (dp - D);
#pragma unroll
          for (int c = 0; c < HALF; c++) dq[c] += ds * Ks[j * DH + hf * HALF + c];
        }
      }
    }
  }
  if (!live) return;
  bf16_t* dp_ = a.dq + ((int64_t)sg.qrow + i) * a.ldq + h * DH + hf * HALF;
  const float fin = Z > 0.f ? a.scale / Z : 0.f;
#pragma unroll
  for (int c = 0; c < HALF; c++) dp_[c] = f32_to_bf16(dq[c] * fin);
  if (hf == 0) a.dsum[sg.lrow + i] = D + dp0;
}

// dk, dv: one pair of threads per key; the queries (scaled), their output gradients, log-sum-exps and
// D_i stream through LDS.  dv_j = sum_i p_ij dO_i; dk_j = scale * sum_i dS_ij q_i.
template <int DH>
__global__ void __launch_bounds__(256) attn_bwd_dkv_k(AttArgs a) {
  constexpr int HALF = DH / 2;
  __shared__ float Qs[ATT_KC * DH], Gs[ATT_KC * DH], Ls[ATT_KC], Ds[ATT_KC];
  const int tiles = (a.Tk + ATT_ROWS - 1) / ATT_ROWS;
  const int tile = blockIdx.x % tiles, sh = blockIdx.x / tiles;
  const int h = sh % a.heads, s = sh / a.heads;
  Seg sg;
  const int seg = segment(a, s, h, sg);
  if (seg != SEG_ROWS) {   // (packed batches) no such sentence; the first index behind the last one clears the unused rows
    if (seg == SEG_TAIL && tile == 0) { clear_rows<DH>(a.dk, a.ldkv, sg.krow, a.k_rows, h); clear_rows<DH>(a.dv, a.ldkv, sg.krow, a.k_rows, h); }
    return;
  }
  if (tile * ATT_ROWS >= sg.Tk) return;   // (packed batches) the sentence ends before this tile
  const int j = tile * ATT_ROWS + (threadIdx.x >> 1), hf = threadIdx.x & 1;
  const bool live = j < sg.Tk;
  float k[HALF], v[HALF], dk[HALF], dv[HALF];
#pragma unroll
  for (int c = 0; c < HALF; c++) { k[c] = 0.f; v[c] = 0.f; dk[c] = 0.f; dv[c] = 0.f; }
  if (live) {
    const bf16_t* kp = a.k + ((int64_t)sg.krow + j) * a.ldkv + h * DH + hf * HALF;
    const bf16_t* vp = a.v + ((int64_t)sg.krow + j) * a.ldkv + h * DH + hf * HALF;
#pragma unroll
    for (int c = 0; c < HALF; c++) { k[c] = bf16_to_f32(kp[c]); v[c] = bf16_to_f32(vp[c]); }
  }
  const bool real = j < sg.nk;   // a padded key gets no weight from any query: its dk, dv stay zero
  const int first = a.causal ? tile * ATT_ROWS / ATT_KC * ATT_KC : 0;   // queries before the tile's first key see none of it
  for (int i0 = first; i0 < sg.Tq; i0 += ATT_KC) {
    const int n = min(ATT_KC, sg.Tq - i0);
    __syncthreads();
    stage_chunk<DH>(a.q + ((int64_t)sg.qrow + i0) * a.ldq + h * DH, a.ldq, n, Qs);
    stage_chunk<DH>(a.dout + ((int64_t)sg.qrow + i0) * a.ldo + h * DH, a.ldo, n, Gs);
    if ((int)threadIdx.x < ATT_KC) {
      const bool in = (int)threadIdx.x < n;
      Ls[threadIdx.x] = in ? a.lse[sg.lrow + i0 + threadIdx.x] : 0.f;
      Ds[threadIdx.x] = in ? a.dsum[sg.lrow + i0 + threadIdx.x] : 0.f;
    }
    __syncthreads();
    for (int i = 0; i < n; i++) {
      float ps = 0.f, pd = 0.f;
#pragma unroll
      for (int c = 0; c < HALF; c++) {
        ps += k[c] * Qs[i * DH + hf * HALF + c];
        pd += v[c] * Gs[i * DH + hf * HALF + c];
      }
      const float sc = pair_sum(ps) * a.scale, dp = pair_sum(pd);
      if (!real || (a.causal && j > i0 + i)) continue;
      const float p = __expf(sc - Ls[i]);
      const float ds = p * (dp - Ds[i]);
#pragma unroll
      for (int c = 0; c < HALF; c++) {
        dv[c] += p * Gs[i * DH + hf * HALF + c];
        dk[c] += ds * Qs[i * DH + hf * HALF + c];
      }
    }
  }
  if (!live) return;
  bf16_t* dkp = a.dk + ((int64_t)sg.krow + j) * a.ldkv + h * DH + hf * HALF;
  bf16_t* dvp = a.dv + ((int64_t)sg.krow + j) * a.ldkv + h * DH + hf * HALF;
#pragma unroll
  for (int c = 0; c < HALF; c++) { dkp[c] = f32_to_bf16(dk[c] * a.scale); dvp[c] = f32_to_bf16(dv[c]); }
}

// ---- matrix-core kernels (head dimensions 64 and 32) -------------------------------------------------------
// v_mfma_f32_32x32x16_bf16 computes D[32x32] += A[32x16] B[16x32]: lane l holds row l % 32 of A and
// column l % 32 of B, eight contraction elements 8 (l / 32) .. + 7 each, and column l % 32 of D, whose
// register v is row 8 (v / 4) + 4 (l / 32) + v % 4.
//
// All three kernels put the 32 rows a wave owns (queries in the forward pass and for dq, keys for dk and dv)
// on the lanes, as the B operand, so that everything per row (running maximum, sums, rescaling) is per lane
// and a score tile leaves the matrix core as [streamed rows on registers][own row on the lane].  Rounded
// to bf16, eight registers of such a tile are a B operand again, with the streamed rows as contraction index
// in the order 8 (e / 4) + 4 (l / 32) + e % 4 (e = 0..7) inside each group of 16: the A operand of that second
// product is read from a transposed copy of the streamed tensor in LDS, as two 8-byte pieces 8 elements
// apart, which is exactly that order.
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));

constexpr int MF_KC = 64;     // streamed rows per LDS chunk
constexpr int MF_PITCH = 72;  // LDS row pitch in elements: 144 bytes, so that 16-byte reads of 8 rows cover all banks

__device__ inline uint32_t pack_bf16_pair(float lo, float hi) {
  const f32x2_t v = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
}

__device__ inline bf16x8_t frag_from(uint4 u) { return __builtin_bit_cast(bf16x8_t, u); }

// eight consecutive registers 8 * t2 .. of a tile, rounded to bf16: one B operand
__device__ inline bf16x8_t tile_to_operand(const f32x16_t& d, int t2) {
  uint4 u;
  u.x = pack_bf16_pair(d[8 * t2 + 0], d[8 * t2 + 1]);
  u.y = pack_bf16_pair(d[8 * t2 + 2], d[8 * t2 + 3]);
  u.z = pack_bf16_pair(d[8 * t2 + 4], d[8 * t2 + 5]);
  u.w = pack_bf16_pair(d[8 * t2 + 6], d[8 * t2 + 7]);
  return frag_from(u);
}

// A operand from a transposed LDS copy: row `row`, contraction group u of 16, for the lane half hh
__device__ inline bf16x8_t transposed_operand(const bf16_t* t, int row, int u, int hh) {
  const bf16_t* p = t + row * MF_PITCH + 16 * u + 4 * hh;
  const uint2 lo = *reinterpret_cast<const uint2*>(p), hi = *reinterpret_cast<const uint2*>(p + 8);
  return frag_from(make_uint4(lo.x, lo.y, hi.x, hi.y));
}

// n rows x DH columns of a bf16 tensor into LDS, row-major with pitch MF_PITCH; rows n .. MF_KC-1 are zero
template <int DH>
__device__ inline void stage_rows(const bf16_t* __restrict__ base, int64_t ld, int n, bf16_t* __restrict__ dst) {
  constexpr int VPR = DH / 8;
  for (int v = threadIdx.x; v < MF_KC * VPR; v += 256) {
    const int r = v / VPR, c = (v % VPR) * 8;
    const uint4 u = r < n ? *reinterpret_cast<const uint4*>(base + (int64_t)r * ld + c) : make_uint4(0, 0, 0, 0);
    *reinterpret_cast<uint4*>(dst + r * MF_PITCH + c) = u;
  }
}

// The same rows transposed: dst[column][row].  Consecutive lanes take consecutive rows, so the 2-byte LDS
// writes of a wave fall into consecutive addresses.  With CENTRE, ref[column] (fp32) is subtracted first.
template <int DH, bool CENTRE>
__device__ inline void stage_transposed(const bf16_t* __restrict__ base, int64_t ld, int n, bf16_t* __restrict__ dst,
                                        const float* __restrict__ ref) {
  constexpr int VPR = DH / 8;
  for (int v = threadIdx.x; v < MF_KC * VPR; v += 256) {
    const int r = v % MF_KC, g = v / MF_KC;
    float t[8];
    if (r < n) {
      load_bf16_8(base + (int64_t)r * ld + 8 * g, t);
      if (CENTRE) {
#pragma unroll
        for (int e = 0; e < 8; e++) t[e] -= ref[8 * g + e];
      }
    } else {
#pragma unroll
      for (int e = 0; e < 8; e++) t[e] = 0.f;
    }
#pragma unroll
    for (int e = 0; e < 8; e++) dst[(8 * g + e) * MF_PITCH + r] = f32_to_bf16(t[e]);
  }
}

// One wave: 32 queries on the lanes.  Per chunk of 64 keys: S^T = K Q^T (two 32-key tiles), online softmax per
// lane (the two half-waves of a query exchange their maxima; their partial sums are added at the end),
// O^T += V^T P^T with P rounded to bf16.
template <int DH>
__global__ void __launch_bounds__(256) attn_fwd_mfma_k(AttArgs a) {
  constexpr int KS = DH / 16, DT = DH / 32;
  __shared__ __attribute__((aligned(16))) bf16_t Ks[MF_KC * MF_PITCH];
  __shared__ __attribute__((aligned(16))) bf16_t Vt[DH * MF_PITCH];
  const int tiles = (a.Tq + ATT_ROWS - 1) / ATT_ROWS;
  const int tile = blockIdx.x % tiles, sh = blockIdx.x / tiles;
  const int h = sh % a.heads, s = sh / a.heads;
  Seg sg;
  const int seg = segment(a, s, h, sg);
  if (seg != SEG_ROWS) {   // (packed batches) no such sentence; the first index behind the last one clears the unused rows
    if (seg == SEG_TAIL && tile == 0) clear_rows<DH>(a.out, a.ldo, sg.qrow, a.lse_rows, h);
    return;
  }
  if (tile * ATT_ROWS >= sg.Tq) return;   // (packed batches) the sentence ends before this tile
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int c = lane & 31, hh = lane >> 5;
  const int qi = tile * ATT_ROWS + wave * 32 + c;
  const bool live = qi < sg.Tq;
  bf16x8_t qf[KS];
#pragma unroll
  for (int t = 0; t < KS; t++) {
    uint4 u = make_uint4(0, 0, 0, 0);
    if (live) u = *reinterpret_cast<const uint4*>(a.q + ((int64_t)sg.qrow + qi) * a.ldq + h * DH + 16 * t + 8 * hh);
    qf[t] = frag_from(u);
  }
  f32x16_t o[DT];
#pragma unroll
  for (int dt = 0; dt < DT; dt++)
#pragma unroll
    for (int v = 0; v < 16; v++) o[dt][v] = 0.f;
  float m = -INFINITY, lsum = 0.f;
  const int nk = sg.nk;
  const int last = a.causal ? min(nk, tile * ATT_ROWS + ATT_ROWS) : nk;
  for (int j0 = 0; j0 < last; j0 += MF_KC) {
    const int n = min(MF_KC, nk - j0);
    __syncthreads();
    stage_rows<DH>(a.k + ((int64_t)sg.krow + j0) * a.ldkv + h * DH, a.ldkv, n, Ks);
    stage_transposed<DH, false>(a.v + ((int64_t)sg.krow + j0) * a.ldkv + h * DH, a.ldkv, n, Vt, nullptr);
    __syncthreads();
    f32x16_t sc[2];
    float mx = -INFINITY;
#pragma unroll
    for (int kt = 0; kt < 2; kt++) {
#pragma unroll
      for (int v = 0; v < 16; v++) sc[kt][v] = 0.f;
#pragma unroll
      for (int t = 0; t < KS; t++) {
        const bf16x8_t kf = frag_from(*reinterpret_cast<const uint4*>(Ks + (32 * kt + c) * MF_PITCH + 16 * t + 8 * hh));
        sc[kt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[t], sc[kt], 0, 0, 0);
      }
#pragma unroll
      for (int v = 0; v < 16; v++) {
        const int kj = j0 + 32 * kt + 8 * (v >> 2) + 4 * hh + (v & 3);
        float x = sc[kt][v] * a.scale;
        if (kj >= nk || (a.causal && kj > qi)) x = -INFINITY;
        sc[kt][v] = x;
        mx = fmaxf(mx, x);
      }
    }
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
    const float mn = fmaxf(m, mx);          // finite from the first chunk on: key 0 is visible to every query
    const float alpha = __expf(m - mn);     // 0 on the first chunk
    m = mn;
    float ps = 0.f;
#pragma unroll
    for (int kt = 0; kt < 2; kt++)
#pragma unroll
      for (int v = 0; v < 16; v++) {
        const float p = __expf(sc[kt][v] - mn);
        sc[kt][v] = p;
        ps += p;
      }
    lsum = lsum * alpha + ps;
#pragma unroll
    for (int dt = 0; dt < DT; dt++) o[dt] *= alpha;
#pragma unroll
    for (int u = 0; u < 4; u++) {
      const bf16x8_t pb = tile_to_operand(sc[u >> 1], u & 1);
#pragma unroll
      for (int dt = 0; dt < DT; dt++)
        o[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(transposed_operand(Vt, 32 * dt + c, u, hh), pb, o[dt], 0, 0, 0);
    }
  }
  const float lt = lsum + __shfl_xor(lsum, 32, 64);
  if (!live) return;
  const float inv = 1.f / lt;
  bf16_t* op = a.out + ((int64_t)sg.qrow + qi) * a.ldo + h * DH + 4 * hh;
#pragma unroll
  for (int dt = 0; dt < DT; dt++)
#pragma unroll
    for (int g = 0; g < 4; g++)
      *reinterpret_cast<uint2*>(op + 32 * dt + 8 * g) =
          make_uint2(pack_bf16_pair(o[dt][4 * g] * inv, o[dt][4 * g + 1] * inv),
                     pack_bf16_pair(o[dt][4 * g + 2] * inv, o[dt][4 * g + 3] * inv));
  if (hh == 0 && a.lse) a.lse[sg.lrow + qi] = m + __logf(lt);
}

// dq on the matrix cores: 32 queries of a wave on the lanes, two passes over the keys as in the plain kernel
// (the first for Z = sum w and D, the second for dq^T += (K - k_0)^T dS^T).  dS is rounded to bf16 for that last
// product, which breaks sum_j dS_ij = 0 at the 1e-3 level; the keys are therefore taken relative to the first
// key of the sentence (exactly what a vanishing sum allows), so that the rounding errors multiply the keys'
// differences and not their common part.
template <int DH>
__global__ void __launch_bounds__(256, 2) attn_bwd_dq_mfma_k(AttArgs a) {
  constexpr int KS = DH / 16, DT = DH / 32;
  __shared__ __attribute__((aligned(16))) bf16_t Ks[MF_KC * MF_PITCH];
  __shared__ __attribute__((aligned(16))) bf16_t Vs[MF_KC * MF_PITCH];
  __shared__ __attribute__((aligned(16))) bf16_t Kc[DH * MF_PITCH];
  __shared__ float K0[DH];
  const int tiles = (a.Tq + ATT_ROWS - 1) / ATT_ROWS;
  const int tile = blockIdx.x % tiles, sh = blockIdx.x / tiles;
  const int h = sh % a.heads, s = sh / a.heads;
  Seg sg;
  const int seg = segment(a, s, h, sg);
  if (seg != SEG_ROWS) {   // (packed batches) no such sentence; the first index behind the last one clears the unused rows
    if (seg == SEG_TAIL && tile == 0) clear_rows<DH>(a.dq, a.ldq, sg.qrow, a.lse_rows, h);
    return;
  }
  if (tile * ATT_ROWS >= sg.Tq) return;   // (packed batches) the sentence ends before this tile
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int c = lane & 31, hh = lane >> 5;
  const int qi = tile * ATT_ROWS + wave * 32 + c;
  const bool live = qi < sg.Tq;
  bf16x8_t qf[KS], gf[KS];
#pragma unroll
  for (int t = 0; t < KS; t++) {
    uint4 u = make_uint4(0, 0, 0, 0), g = make_uint4(0, 0, 0, 0);
    if (live) {
      u = *reinterpret_cast<const uint4*>(a.q + ((int64_t)sg.qrow + qi) * a.ldq + h * DH + 16 * t + 8 * hh);
      g = *reinterpret_cast<const uint4*>(a.dout + ((int64_t)sg.qrow + qi) * a.ldo + h * DH + 16 * t + 8 * hh);
    }
    qf[t] = frag_from(u);
    gf[t] = frag_from(g);
  }
  const float lse = live ? a.lse[sg.lrow + qi] : 0.f;
  const int nk = sg.nk;
  const int visible = a.causal ? min(qi + 1, nk) : nk;
  const float ref = lse - __logf((float)max(visible, 1));
  if ((int)threadIdx.x < DH) K0[threadIdx.x] = bf16_to_f32(a.k[(int64_t)sg.krow * a.ldkv + h * DH + threadIdx.x]);
  f32x16_t dq[DT];
#pragma unroll
  for (int dt = 0; dt < DT; dt++)
#pragma unroll
    for (int v = 0; v < 16; v++) dq[dt][v] = 0.f;
  const int last = a.causal ? min(nk, tile * ATT_ROWS + ATT_ROWS) : nk;
  float D = 0.f, Z = 0.f, dp0 = 0.f;
  for (int pass = 0; pass < 2; pass++) {
    if (pass == 1) {
      Z += __shfl_xor(Z, 32, 64);
      D += __shfl_xor(D, 32, 64);
      D = Z > 0.f ? D / Z : 0.f;
    }
    for (int j0 = 0; j0 < last; j0 += MF_KC) {
      const int n = min(MF_KC, nk - j0);
      const bf16_t* kb = a.k + ((int64_t)sg.krow + j0) * a.ldkv + h * DH;
      __syncthreads();
      stage_rows<DH>(kb, a.ldkv, n, Ks);
      stage_rows<DH>(a.v + ((int64_t)sg.krow + j0) * a.ldkv + h * DH, a.ldkv, n, Vs);
      if (pass == 1) stage_transposed<DH, true>(kb, a.ldkv, n, Kc, K0);
      __syncthreads();
      f32x16_t sc[2], dp[2];
#pragma unroll
      for (int kt = 0; kt < 2; kt++) {
#pragma unroll
        for (int v = 0; v < 16; v++) { sc[kt][v] = 0.f; dp[kt][v] = 0.f; }
#pragma unroll
        for (int t = 0; t < KS; t++) {
          const int off = (32 * kt + c) * MF_PITCH + 16 * t + 8 * hh;
          sc[kt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_from(*reinterpret_cast<const uint4*>(Ks + off)), qf[t], sc[kt], 0, 0, 0);
          dp[kt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_from(*reinterpret_cast<const uint4*>(Vs + off)), gf[t], dp[kt], 0, 0, 0);
        }
      }
      if (pass == 0 && j0 == 0) dp0 = __shfl(dp[0][0], c, 64);   // register 0 of the lower half-wave is key 0
#pragma unroll
      for (int kt = 0; kt < 2; kt++)
#pragma unroll
        for (int v = 0; v < 16; v++) {
          const int kj = j0 + 32 * kt + 8 * (v >> 2) + 4 * hh + (v & 3);
          float w = __expf(sc[kt][v] * a.scale - ref);
          if (kj >= nk || (a.causal && kj > qi)) w = 0.f;
          const float d = dp[kt][v] - dp0;
          if (pass == 0) {
            Z += w;
            D += w * d;
          } else {
            dp[kt][v] = w * (d - D);
          }
        }
      if (pass == 1) {
#pragma unroll
        for (int u = 0; u < 4; u++) {
          const bf16x8_t dsb = tile_to_operand(dp[u >> 1], u & 1);
#pragma unroll
          for (int dt = 0; dt < DT; dt++)
            dq[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(transposed_operand(Kc, 32 * dt + c, u, hh), dsb, dq[dt], 0, 0, 0);
        }
      }
    }
  }
  if (!live) return;
  const float fin = Z > 0.f ? a.scale / Z : 0.f;
  bf16_t* op = a.dq + ((int64_t)sg.qrow + qi) * a.ldq + h * DH + 4 * hh;
#pragma unroll
  for (int dt = 0; dt < DT; dt++)
#pragma unroll
    for (int g = 0; g < 4; g++)
      *reinterpret_cast<uint2*>(op + 32 * dt + 8 * g) =
          make_uint2(pack_bf16_pair(dq[dt][4 * g] * fin, dq[dt][4 * g + 1] * fin),
                     pack_bf16_pair(dq[dt][4 * g + 2] * fin, dq[dt][4 * g + 3] * fin));
  if (hh == 0) a.dsum[sg.lrow + qi] = D + dp0;
}

// dk, dv on the matrix cores: 32 keys of a wave on the lanes; per chunk of 64 queries S = Q K^T and
// dP = dO V^T (queries on the registers), then dV^T += dO^T P and dK^T += Q^T dS with P, dS rounded to bf16
// and Q, dO read from transposed LDS copies.
template <int DH>
__global__ void __launch_bounds__(256, 2) attn_bwd_dkv_mfma_k(AttArgs a) {
  constexpr int KS = DH / 16, DT = DH / 32;
  __shared__ __attribute__((aligned(16))) bf16_t Qs[MF_KC * MF_PITCH];
  __shared__ __attribute__((aligned(16))) bf16_t Gs[MF_KC * MF_PITCH];
  __shared__ __attribute__((aligned(16))) bf16_t Qt[DH * MF_PITCH];
  __shared__ __attribute__((aligned(16))) bf16_t Gt[DH * MF_PITCH];
  __shared__ float Ls[MF_KC], Ds[MF_KC];
  const int tiles = (a.Tk + ATT_ROWS - 1) / ATT_ROWS;
  const int tile = blockIdx.x % tiles, sh = blockIdx.x / tiles;
  const int h = sh % a.heads, s = sh / a.heads;
  Seg sg;
  const int seg = segment(a, s, h, sg);
  if (seg != SEG_ROWS) {   // (packed batches) no such sentence; the first index behind the last one clears the unused rows
    if (seg == SEG_TAIL && tile == 0) { clear_rows<DH>(a.dk, a.ldkv, sg.krow, a.k_rows, h); clear_rows<DH>(a.dv, a.ldkv, sg.krow, a.k_rows, h); }
    return;
  }
  if (tile * ATT_ROWS >= sg.Tk) return;   // (packed batches) the sentence ends before this tile
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int c = lane & 31, hh = lane >> 5;
  const int kj = tile * ATT_ROWS + wave * 32 + c;
  const bool live = kj < sg.Tk;
  bf16x8_t kf[KS], vf[KS];
#pragma unroll
  for (int t = 0; t < KS; t++) {
    uint4 u = make_uint4(0, 0, 0, 0), w = make_uint4(0, 0, 0, 0);
    if (live) {
      u = *reinterpret_cast<const uint4*>(a.k + ((int64_t)sg.krow + kj) * a.ldkv + h * DH + 16 * t + 8 * hh);
      w = *reinterpret_cast<const uint4*>(a.v + ((int64_t)sg.krow + kj) * a.ldkv + h * DH + 16 * t + 8 * hh);
    }
    kf[t] = frag_from(u);
    vf[t] = frag_from(w);
  }
  f32x16_t dk[DT], dv[DT];
#pragma unroll
  for (int dt = 0; dt < DT; dt++)
#pragma unroll
    for (int v = 0; v < 16; v++) { dk[dt][v] = 0.f; dv[dt][v] = 0.f; }
  const bool real = kj < sg.nk;   // a padded key gets no weight from any query: its dk, dv stay zero
  const int first = a.causal ? tile * ATT_ROWS / MF_KC * MF_KC : 0;   // earlier queries see none of the tile's keys
  for (int i0 = first; i0 < sg.Tq; i0 += MF_KC) {
    const int n = min(MF_KC, sg.Tq - i0);
    const bf16_t* qb = a.q + ((int64_t)sg.qrow + i0) * a.ldq + h * DH;
    const bf16_t* gb = a.dout + ((int64_t)sg.qrow + i0) * a.ldo + h * DH;
    __syncthreads();
    stage_rows<DH>(qb, a.ldq, n, Qs);
    stage_rows<DH>(gb, a.ldo, n, Gs);
    stage_transposed<DH, false>(qb, a.ldq, n, Qt, nullptr);
    stage_transposed<DH, false>(gb, a.ldo, n, Gt, nullptr);
    if ((int)threadIdx.x < MF_KC) {
      const bool in = (int)threadIdx.x < n;
      Ls[threadIdx.x] = in ? a.lse[sg.lrow + i0 + threadIdx.x] : 0.f;
      Ds[threadIdx.x] = in ? a.dsum[sg.lrow + i0 + threadIdx.x] : 0.f;
    }
    __syncthreads();
    f32x16_t sc[2], dp[2];
#pragma unroll
    for (int qt = 0; qt < 2; qt++) {
#pragma unroll
      for (int v = 0; v < 16; v++) { sc[qt][v] = 0.f; dp[qt][v] = 0.f; }
#pragma unroll
      for (int t = 0; t < KS; t++) {
        const int off = (32 * qt + c) * MF_PITCH + 16 * t + 8 * hh;
        sc[qt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_from(*reinterpret_cast<const uint4*>(Qs + off)), kf[t], sc[qt], 0, 0, 0);
        dp[qt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_from(*reinterpret_cast<const uint4*>(Gs + off)), vf[t], dp[qt], 0, 0, 0);
      }
#pragma unroll
      for (int v = 0; v < 16; v++) {
        const int r = 32 * qt + 8 * (v >> 2) + 4 * hh + (v & 3);
        const int qi = i0 + r;
        float p = __expf(sc[qt][v] * a.scale - Ls[r]);
        if (qi >= sg.Tq || !real || (a.causal && kj > qi)) p = 0.f;
        dp[qt][v] = p * (dp[qt][v] - Ds[r]);
        sc[qt][v] = p;
      }
    }
#pragma unroll
    for (int u = 0; u < 4; u++) {
      const bf16x8_t pb = tile_to_operand(sc[u >> 1], u & 1), dsb = tile_to_operand(dp[u >> 1], u & 1);
#pragma unroll
      for (int dt = 0; dt < DT; dt++) {
        dv[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(transposed_operand(Gt, 32 * dt + c, u, hh), pb, dv[dt], 0, 0, 0);
        dk[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(transposed_operand(Qt, 32 * dt + c, u, hh), dsb, dk[dt], 0, 0, 0);
      }
    }
  }
  if (!live) return;
  bf16_t* dkp = a.dk + ((int64_t)sg.krow + kj) * a.ldkv + h * DH + 4 * hh;
  bf16_t* dvp = a.dv + ((int64_t)sg.krow + kj) * a.ldkv + h * DH + 4 * hh;
#pragma unroll
  for (int dt = 0; dt < DT; dt++)
#pragma unroll
    for (int g = 0; g < 4; g++) {
      *reinterpret_cast<uint2*>(dkp + 32 * dt + 8 * g) =
          make_uint2(pack_bf16_pair(dk[dt][4 * g] * a.scale, dk[dt][4 * g + 1] * a.scale),
                     pack_bf16_pair(dk[dt][4 * g + 2] * a.scale, dk[dt][4 * g + 3] * a.scale));
      *reinterpret_cast<uint2*>(dvp + 32 * dt + 8 * g) =
          make_uint2(pack_bf16_pair(dv[dt][4 * g], dv[dt][4 * g + 1]), pack_bf16_pair(dv[dt][4 * g + 2], dv[dt][4 * g + 3]));
    }
}

// ---- embedding ------------------------------------------------------------------------------------
// y[s*T + t][:] = table[tok[s][col0 + t]][:] * sqrt(d) + PE[t][:], PE[t][2i] = sin(t / 10000^(2i/d)),
// PE[t][2i+1] = cos(same).  One thread per pair of columns.
template <typename T>
__global__ void __launch_bounds__(256) embed_fwd_k(const int32_t* __restrict__ tok, int64_t tok_pitch, int col0, int T_,
                                                   const T* __restrict__ table, int vocab, int d, T* __restrict__ y,
                                                   int64_t rows, const int32_t* __restrict__ pos) {
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const int half = d / 2;
  if (idx >= rows * half) return;
  const int i = (int)(idx % half);
  const int64_t row = idx / half;
  int t = (int)(row % T_);
  const int64_t s = row / T_;
  int id = tok[s * tok_pitch + col0 + t];
  if (pos) t = pos[s * tok_pitch + col0 + t];   // packed batches: the position inside the token's own sentence
  const float keep = id < 0 ? 0.f : 1.f;      // a negative id is padding: a zero row (plus the position signal)
  id = id < 0 ? 0 : (id >= vocab ? vocab - 1 : id);   // ids are validated by the caller; clamp keeps the access in bounds
  const float ang = (float)t * __expf(-(float)(2 * i) / (float)d * 9.210340371976184f);   // ln 10000
  const float scale = keep * sqrtf((float)d);
  const T* tr = table + (int64_t)id * d + 2 * i;
  y[row * d + 2 * i] = Cvt<T>::st(Cvt<T>::ld(tr[0]) * scale + sinf(ang));
  y[row * d + 2 * i + 1] = Cvt<T>::st(Cvt<T>::ld(tr[1]) * scale + cosf(ang));
}

// dtable[id] += sqrt(d) * sum of the rows of dy at the positions that hold token id.  One workgroup per position r and
// block of 1024 columns.  The first position of each distinct id owns it: the workgroup first looks for an earlier
// position with the same id (and leaves if there is one), then walks the positions from r on, 256 at a time, and adds
// the matching rows in position order onto the table row it alone writes.  One writer per row and a fixed order of
// additions: the result is bit-reproducible (atomics would not be).  The search is quadratic in the number of
// positions (8192 x 8192 / 256 workgroup steps at the base shape, about 20 us).
constexpr int EMB_COLS = 4;   // columns per thread
template <typename T>
__global__ void __launch_bounds__(256) embed_bwd_k(const int32_t* __restrict__ tok, int64_t tok_pitch, int col0, int T_,
                                                   const T* __restrict__ dy, int vocab, int d, float* __restrict__ dtable,
                                                   int64_t rows) {
  __shared__ unsigned long long hits[4];
  const int64_t r = blockIdx.x;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  auto id_at = [&](int64_t q) {
    const int v = tok[(q / T_) * tok_pitch + col0 + (q % T_)];
    return v >= vocab ? vocab - 1 : v;   // the forward pass clamps the same way; negative = padding
  };
  const int id = id_at(r);
  if (id < 0) return;
  for (int64_t q0 = 0; q0 < r; q0 += 256) {
    const int64_t q = q0 + threadIdx.x;
    if (__syncthreads_or(q < r && id_at(q) == id)) return;   // an earlier position owns this id
  }
  const int cbase = blockIdx.y * (256 * EMB_COLS) + threadIdx.x;
  float acc[EMB_COLS];
#pragma unroll
  for (int k = 0; k < EMB_COLS; k++) acc[k] = 0.f;
  for (int64_t q0 = r / 256 * 256; q0 < rows; q0 += 256) {
    const int64_t q = q0 + threadIdx.x;
    const unsigned long long b = __ballot(q >= r && q < rows && id_at(q) == id);
    __syncthreads();   // the previous chunk's masks have been read
    if (lane == 0) hits[wave] = b;
    __syncthreads();
    for (int w = 0; w < 4; w++) {
      unsigned long long m = hits[w];
      while (m) {
        const int bit = __ffsll((long long)m) - 1;
        m &= m - 1;
        const T* row = dy + (q0 + 64 * w + bit) * d;
#pragma unroll
        for (int k = 0; k < EMB_COLS; k++) {
          const int c = cbase + 256 * k;
          if (c < d) acc[k] += Cvt<T>::ld(row[c]);
        }
      }
    }
  }
  const float scale = sqrtf((float)d);
#pragma unroll
  for (int k = 0; k < EMB_COLS; k++) {
    const int c = cbase + 256 * k;
    if (c < d) dtable[(int64_t)id * d + c] += scale * acc[k];
  }
}

// ---- sentence tables of a packed batch -------------------------------------------------------------
// One workgroup walks the rows 1024 at a time.  A row with a non-negative id and position 0 starts a sentence: its
// rank among the starts (a prefix count over the workgroup) is the sentence's number.  table[i] = first row of
// sentence i (i < max_sent), table[n] = the first row that belongs to no sentence kept (the start of sentence
// max_sent, if there are more, else the number of rows with non-negative ids), table[max_sent + 1] = n.
__global__ void __launch_bounds__(1024) sentence_tables_k(const int32_t* __restrict__ tok, const int32_t* __restrict__ pos,
                                                          int rows, int max_sent, int32_t* __restrict__ table) {
  __shared__ int wave_cnt[16], wave_val[16];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  int starts = 0, valid = 0;   // running totals, the same in every thread
  for (int r0 = 0; r0 < rows; r0 += 1024) {
    const int r = r0 + (int)threadIdx.x;
    const bool ok = r < rows && tok[r] >= 0;
    const bool st = ok && pos[r] == 0;
    const unsigned long long bs = __ballot(st), bv = __ballot(ok);
    __syncthreads();   // the previous chunk's counts have been read
    if (lane == 0) { wave_cnt[wave] = __popcll(bs); wave_val[wave] = __popcll(bv); }
    __syncthreads();
    int before = 0, chunk_starts = 0, chunk_valid = 0;
    for (int w = 0; w < 16; w++) {
      before += w < wave ? wave_cnt[w] : 0;
      chunk_starts += wave_cnt[w];
      chunk_valid += wave_val[w];
    }
    if (st) {
      const int rank = starts + before + __popcll(bs & ((1ull << lane) - 1ull));
      if (rank <= max_sent) table[rank] = r;   // rank == max_sent: the end of the last sentence kept
    }
    starts += chunk_starts;
    valid += chunk_valid;
  }
  if (threadIdx.x == 0) {
    const int n = starts < max_sent ? starts : max_sent;
    if (starts <= max_sent) table[n] = valid;
    table[max_sent + 1] = n;
  }
}

}  // namespace

// The matrix-core kernels read 16-byte vectors: head dimension 64 or 32 and row pitches that keep every row aligned.
// CODISTILL_PLAIN_ATTENTION=1 keeps the plain kernels (for comparing the two).
static bool use_mfma(int dh, int64_t ldq, int64_t ldkv, int64_t ldo) {
  const char* e = getenv("CODISTILL_PLAIN_ATTENTION");
  const bool plain = e && e[0] == '1';
  return !plain && (dh == 64 || dh == 32) && ldq % 8 == 0 && ldkv % 8 == 0 && ldo % 8 == 0;
}

bool attention_supported(int dh) { return dh == 8 || dh == 16 || dh == 32 || dh == 64; }

#define CD_ATT_DISPATCH(KERNEL, grid)                                                                      \
  switch (dh) {                                                                                           \
    case 8: hipLaunchKernelGGL((KERNEL<8>), dim3(grid), dim3(256), 0, s, a); break;                       \
    case 16: hipLaunchKernelGGL((KERNEL<16>), dim3(grid), dim3(256), 0, s, a); break;                     \
    case 32: hipLaunchKernelGGL((KERNEL<32>), dim3(grid), dim3(256), 0, s, a); break;                     \
    default: hipLaunchKernelGGL((KERNEL<64>), dim3(grid), dim3(256), 0, s, a); break;                     \
  }

void attention_forward(const bf16_t* q, int64_t ldq, const bf16_t* k, const bf16_t* v, int64_t ldkv, bf16_t* out, int64_t ldo,
                       float* lse, int S, int heads, int Tq, int Tk, int dh, bool causal, const int32_t* key_tokens,
                       int64_t tok_pitch, int key_col0, const SentenceTables* tab, hipStream_t s) {
  AttArgs a = {};
  a.ktok = key_tokens; a.tok_pitch = tok_pitch; a.ktok0 = key_col0;
  if (tab) {
    a.q_tab = tab->q; a.k_tab = tab->k; a.max_sent = tab->max_sent; a.lse_rows = tab->q_rows; a.k_rows = tab->k_rows;
    a.ktok = nullptr;
    S = tab->max_sent + 1;   // one more row of workgroups: it clears the rows behind the last sentence
  }
  a.q = q; a.k = k; a.v = v; a.ldq = ldq; a.ldkv = ldkv; a.out = out; a.ldo = ldo; a.lse = lse;
  a.S = S; a.heads = heads; a.Tq = Tq; a.Tk = Tk; a.causal = causal ? 1 : 0;
  a.scale = 1.f / sqrtf((float)dh);
  const unsigned grid = (unsigned)((int64_t)S * heads * cdiv(Tq, ATT_ROWS));
  if (use_mfma(dh, ldq, ldkv, ldo)) {
    if (dh == 64) hipLaunchKernelGGL((attn_fwd_mfma_k<64>), dim3(grid), dim3(256), 0, s, a);
    else hipLaunchKernelGGL((attn_fwd_mfma_k<32>), dim3(grid), dim3(256), 0, s, a);
    return;
  }
  CD_ATT_DISPATCH(attn_fwd_k, grid);
}

void attention_backward(const bf16_t* q, int64_t ldq, const bf16_t* k, const bf16_t* v, int64_t ldkv, const bf16_t* dout,
                        int64_t ldo, const float* lse, float* dsum, bf16_t* dq, bf16_t* dk, bf16_t* dv, int S, int heads,
                        int Tq, int Tk, int dh, bool causal, const int32_t* key_tokens, int64_t tok_pitch, int key_col0,
                        const SentenceTables* tab, hipStream_t s) {
  AttArgs a = {};
  a.ktok = key_tokens; a.tok_pitch = tok_pitch; a.ktok0 = key_col0;
  if (tab) {
    a.q_tab = tab->q; a.k_tab = tab->k; a.max_sent = tab->max_sent; a.lse_rows = tab->q_rows; a.k_rows = tab->k_rows;
    a.ktok = nullptr;
    S = tab->max_sent + 1;   // one more row of workgroups: it clears the rows behind the last sentence
  }
  a.q = q; a.k = k; a.v = v; a.ldq = ldq; a.ldkv = ldkv; a.dout = dout; a.ldo = ldo;
  a.lse = const_cast<float*>(lse); a.dsum = dsum; a.dq = dq; a.dk = dk; a.dv = dv;
  a.S = S; a.heads = heads; a.Tq = Tq; a.Tk = Tk; a.causal = causal ? 1 : 0;
  a.scale = 1.f / sqrtf((float)dh);
  const unsigned gq = (unsigned)((int64_t)S * heads * cdiv(Tq, ATT_ROWS));
  const unsigned gk = (unsigned)((int64_t)S * heads * cdiv(Tk, ATT_ROWS));
  if (use_mfma(dh, ldq, ldkv, ldo)) {
    if (dh == 64) {
      hipLaunchKernelGGL((attn_bwd_dq_mfma_k<64>), dim3(gq), dim3(256), 0, s, a);
      hipLaunchKernelGGL((attn_bwd_dkv_mfma_k<64>), dim3(gk), dim3(256), 0, s, a);
    } else {
      hipLaunchKernelGGL((attn_bwd_dq_mfma_k<32>), dim3(gq), dim3(256), 0, s, a);
      hipLaunchKernelGGL((attn_bwd_dkv_mfma_k<32>), dim3(gk), dim3(256), 0, s, a);
    }
    return;
  }
  CD_ATT_DISPATCH(attn_bwd_dq_k, gq);
  CD_ATT_DISPATCH(attn_bwd_dkv_k, gk);
}

void embed_forward(int dtype, const int32_t* tok, int64_t tok_pitch, int col0, int len, const void* table, int vocab, int d,
                   void* y, int64_t rows, const int32_t* pos, hipStream_t s) {
  const unsigned grid = (unsigned)cdiv(rows * (d / 2), 256);
  if (dtype == CD_BF16)
    hipLaunchKernelGGL(embed_fwd_k<bf16_t>, dim3(grid), dim3(256), 0, s, tok, tok_pitch, col0, len, (const bf16_t*)table,
                       vocab, d, (bf16_t*)y, rows, pos);
  else
    hipLaunchKernelGGL(embed_fwd_k<float>, dim3(grid), dim3(256), 0, s, tok, tok_pitch, col0, len, (const float*)table,
                       vocab, d, (float*)y, rows, pos);
}

void sentence_tables(const int32_t* tok, const int32_t* pos, int rows, int max_sent, int32_t* table, hipStream_t s) {
  hipLaunchKernelGGL(sentence_tables_k, dim3(1), dim3(1024), 0, s, tok, pos, rows, max_sent, table);
}

void embed_backward(int dtype, const int32_t* tok, int64_t tok_pitch, int col0, int len, const void* dy, int vocab, int d,
                    float* dtable, int64_t rows, hipStream_t s) {
  const dim3 grid((unsigned)rows, (unsigned)cdiv(d, 256 * EMB_COLS));
  if (dtype == CD_BF16)
    hipLaunchKernelGGL(embed_bwd_k<bf16_t>, dim3(grid), dim3(256), 0, s, tok, tok_pitch, col0, len, (const bf16_t*)dy, vocab,
                       d, dtable, rows);
  else
    hipLaunchKernelGGL(embed_bwd_k<float>, dim3(grid), dim3(256), 0, s, tok, tok_pitch, col0, len, (const float*)dy, vocab, d,
                       dtable, rows);
}

}  // namespace cd
