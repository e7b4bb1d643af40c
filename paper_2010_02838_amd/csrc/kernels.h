// Host launchers of the layer kernels.  `dtype` is CD_F32 or CD_BF16 and selects the storage type
// of activations, activation gradients and parameters; statistics, logits and parameter gradients
// are always fp32.  Nothing here allocates or synchronises.
#pragma once
#include "common.h"
#include <vector>

namespace cd {

struct ConvGeom {
  int64_t B;
  int H, W, Cin, Ho, Wo, Cout, kh, kw, stride, pad;
  __host__ __device__ int64_t M() const { return B * Ho * Wo; }
  __host__ __device__ int K() const { return kh * kw * Cin; }
};

constexpr float kBnEps = 1e-5f;
constexpr size_t kPartialsBytes = 128u << 20;  // reduction / split-K partials inside the workspace
// Per-chunk column sums are stored [chunks][stat_pitch(C)] floats: sums at [0, C), second sums at
// [C, 2C).  The 64 floats of padding keep the chunk pitch off the powers of two that C takes, which
// would send every chunk's writes to the same memory channel.
__host__ __device__ inline int64_t stat_pitch(int C) { return 2 * (int64_t)C + 64; }

// ---- plain kernels: any shape, fp32 or bf16 storage, fp32 arithmetic ------------------------------
void conv_fprop_simple(int dtype, const void* x, const void* w, const void* bias, void* y, const ConvGeom& g,
                       bool relu, hipStream_t s);
void conv_dgrad_simple(int dtype, const void* dy, const void* w, void* dx, const ConvGeom& g, bool accumulate,
                       hipStream_t s);
void conv_wgrad_simple(int dtype, const void* x, const void* dy, float* dw, const ConvGeom& g, hipStream_t s);
void relu_bwd_inplace(int dtype, void* dy, const void* y, int64_t n, hipStream_t s);
void colsum(int dtype, const void* a, int64_t M, int C, float* out, float* partials, hipStream_t s);

// BatchNorm with batch statistics over M rows of C channels, y = relu?(gamma*xhat + beta + res?).
// stats: [4][C] fp32 = mean, invstd, scale, shift (kept for the backward pass).
// relu_mask (nullable; bf16 with C % 8 == 0 only): M*C/8 bytes, bit k of byte i = (y[8i + k] > 0).  The
// forward pass writes it, the backward pass reads it instead of y (an eighth of a byte per element
// instead of two bytes, in both of its passes).
// Two steps.  bn_stats: the batch statistics of x into stats; with pre_chunks > 0 the column sums are
// already in partials ([pre_chunks][stat_pitch(C)], from the producing convolution; scratch: room for
// 32 * stat_pitch(C) floats behind them), with pre_chunks == 0 x is reduced first (partials is scratch).
// bn_apply: the elementwise pass with those statistics.
void bn_stats(int dtype, const void* x, const void* gamma, const void* beta, int64_t M, int C, float* stats,
              float* partials, int pre_chunks, float* scratch, hipStream_t s);
// Running averages [mean[C] | var[C]] (fp32) for the evaluation mode: updated from the statistics of a training-mode
// pass over M rows (momentum 0.1, unbiased variance), or turned into stats in place of the batch's.
void bn_running_update(const float* stats, float* running, int64_t M, int C, float momentum, hipStream_t s);
void bn_stats_from_running(int dtype, const float* running, const void* gamma, const void* beta, float* stats, int C,
                           hipStream_t s);
void bn_apply(int dtype, const void* x, const void* res, bool relu, void* y, int64_t M, int C, const float* stats,
              uint8_t* relu_mask, hipStream_t s);
// bn_apply with ReLU followed by a 3x3 stride-2 pad-1 max-pool, in one pass: y [B][H/2][W/2][C] is the pooled
// tensor, the normalised one is not written.  bf16, C % 8 == 0, even H and W, 16-byte aligned pointers.
// argmax (nullable): as maxpool_fwd writes it; relu_mask (nullable): as bn_apply writes it.
void bn_relu_pool(const bf16_t* x, const float* stats, bf16_t* y, uint8_t* argmax, uint8_t* relu_mask, int64_t B, int H,
                  int W, int C, hipStream_t s);
// Its backward pass: dpool [B][H/2][W/2][C] is the gradient of the pooled tensor, argmax and relu_mask what the
// forward pass wrote; the gradient of the normalised tensor is gathered on the fly in both passes (never
// written).  dx [B][H][W][C] is overwritten; dgamma, dbeta, coef, partials as in bn_backward.
void bn_relu_pool_backward(const bf16_t* dpool, const uint8_t* argmax, const bf16_t* x, const bf16_t* gamma,
                           const float* stats, bf16_t* dx, float* dgamma, float* dbeta, float* coef, float* partials,
                           const uint8_t* relu_mask, int64_t B, int H, int W, int C, hipStream_t s);
// dz = dy * (relu ? y > 0 : 1); dgamma = sum dz*xhat; dbeta = sum dz;
// dx = gamma*invstd*(dz - dbeta/M - xhat*dgamma/M); dres = dz.  coef: [3][C] fp32 scratch.
// pre_chunks > 0: the sums over the rows are already in partials, in pre_chunks chunks of stat_pitch(C) floats (left by
// the data gradient that wrote dy: conv_dgrad_mfma with bn); the reduction pass over dy and x is then left out.
void bn_backward(int dtype, const void* dy, const void* y, const void* x, const void* gamma, const float* stats,
                 bool relu, void* dx, bool acc_dx, void* dres, bool acc_dres, float* dgamma, float* dbeta,
                 float* coef, float* partials, const uint8_t* relu_mask, int64_t M, int C, hipStream_t s,
                 int pre_chunks = 0);

// LayerNorm over the last axis of [rows][d] (biased variance, eps 1e-5) of a + r (r nullable):
// y = gamma * xhat + beta.  stats: [rows][2] fp32 = mean, rstd (kept for the backward pass).
void ln_forward(int dtype, const void* a, const void* r, const void* gamma, const void* beta, void* y, float* stats,
                int64_t rows, int d, hipStream_t s);
// dx = rstd * (g - mean(g) - xhat * mean(g * xhat)) with g = dy * gamma goes to da and dr (each nullable,
// each added to its old contents if its acc flag is set); dgamma = sum dy * xhat, dbeta = sum dy.
// partials: room for 1024 * 2 * d floats.
void ln_backward(int dtype, const void* dy, const void* a, const void* r, const void* gamma, const float* stats, void* da,
                 bool acc_a, void* dr, bool acc_r, float* dgamma, float* dbeta, float* partials, int64_t rows, int d,
                 hipStream_t s);

// argmax: optional [B][Ho][Wo][C] bytes, the window tap (r*k+s) of the first maximum; written by the
// forward pass and, when given, used by the backward pass instead of rescanning the windows
void maxpool_fwd(int dtype, const void* x, void* y, uint8_t* argmax, int64_t B, int H, int W, int C, int k, int stride,
                 int pad, hipStream_t s);
void maxpool_bwd(int dtype, const void* x, const void* dy, const uint8_t* argmax, void* dx, bool accumulate, int64_t B,
                 int H, int W, int C, int k, int stride, int pad, hipStream_t s);
void gap_fwd(int dtype, const void* x, void* y, int64_t B, int HW, int C, hipStream_t s);
void gap_bwd(int dtype, const void* dy, void* dx, bool accumulate, int64_t B, int HW, int C, hipStream_t s);
void linear_fwd(int dtype, const void* x, const void* w, const void* b, float* y, int64_t B, int F, int C,
                hipStream_t s);
void linear_bwd(int dtype, const void* x, const void* w, const float* dy, void* dx, bool accumulate, float* dw,
                float* db, int64_t B, int F, int C, hipStream_t s);

// y[m][j] = x[m][c0 + j], j < Cy (a range of channels of every pixel)
void channel_slice(int dtype, const void* x, void* y, int64_t M, int Cx, int c0, int Cy, hipStream_t s);
void fill_zero_f32(float* p, int64_t n, hipStream_t s);

struct Gap { int64_t off; int32_t len; };
void zero_gaps(float* base, const Gap* gaps, int n, hipStream_t s);

}  // namespace cd

namespace cd {
// ---- bf16 MFMA implicit-GEMM convolution (conv_mfma.hip) -----------------------------------------
// All need the channel count of the gathered tensor to be a multiple of 8 (16-byte vectors).
bool conv_mfma_supported(const ConvGeom& g);
// y[M][Cout] = im2col(x)[M][K] * w[Cout][K]^T.  With stat_partials the kernel also writes per-tile
// column sums and sums of squares, [chunks][stat_pitch(Cout)] fp32, and returns the number of chunks
// (needs (M/128 + 1) * stat_pitch(Cout) floats); see bn_stats.
// bias (nullable, [Cout] bf16) is added and, with relu, the result clamped at zero before rounding.
int conv_fprop_mfma(const bf16_t* x, const bf16_t* w, const bf16_t* bias, bool relu, bf16_t* y, const ConvGeom& g,
                    float* stat_partials, hipStream_t s);
// which kernel conv_fprop_mfma runs this shape with: 0 the 128x128 tiles, 1 the 128x256 tiles, 2 any other
int conv_fprop_tile_class(const ConvGeom& g, bool bias);
// dx[B*H*W][Cin] (+)= gather(dy)[.][taps*Cout] * wt[Cin][taps*Cout]^T.  w is the filter as stored; wt is
// scratch of at least Cout*K + 32 elements that receives its re-laid-out copy (or copies, per parity
// class, for stride 2).  addend (nullable; stride 1 and accumulate == false only): dx = product + addend,
// with addend_gate (nullable, one bit per element of addend) dropping the elements whose bit is clear.
// relu_out (nullable; stride 1 only): dx is the gradient behind a ReLU whose result is relu_out [B*H*W][Cin]; its
// elements where relu_out is not positive are written as zero.
// bn (nullable; stride 1 only): dx completes the gradient of the output of a BatchNorm (input bn->x [B*H*W][Cin], batch
// statistics bn->stats = [mean | invstd], ReLU bit mask bn->mask or NULL): the launch also leaves, per row tile, the
// column sums of dz = dx gated by the mask and of dz * xhat in bn->partials, for bn_backward's pre_chunks.  Returns the
// number of row tiles (the chunks of those sums), 0 without bn.
struct BnBackwardSums { const bf16_t* x; const uint8_t* mask; const float* stats; float* partials; };
// wt_ready: wt already holds the re-laid-out filter (conv_dgrad_layout_jobs + relayout_weights_batch): the launch's own
// re-layout kernels are left out.
int conv_dgrad_mfma(const bf16_t* dy, const bf16_t* w, bf16_t* wt, bf16_t* dx, const ConvGeom& g, bool accumulate,
                    hipStream_t s, const bf16_t* addend = nullptr, const uint8_t* addend_gate = nullptr,
                    const bf16_t* relu_out = nullptr, const BnBackwardSums* bn = nullptr, bool wt_ready = false);
// The filter re-layouts of many data gradients in one launch (a backward pass needs one per convolution, each a few
// microseconds of work behind a launch of its own otherwise).  A job writes wt[c][jh][jw][n] = w[n][r0 + rstep jh][s0 + rstep jw][c]
// for c < cin, jh < th, jw < tw, n < cout; first = the number of elements of the jobs in front of it.
struct WeightLayoutJob { const bf16_t* w; bf16_t* wt; int cout, kh, kw, cin, th, tw, r0, s0, rstep; int64_t first; };
// appends the jobs that conv_dgrad_mfma's own re-layout of this convolution consists of (same places inside wt)
void conv_dgrad_layout_jobs(const bf16_t* w, bf16_t* wt, const ConvGeom& g, std::vector<WeightLayoutJob>& jobs);
// elements of wt that conv_dgrad_mfma uses for this convolution
int64_t conv_dgrad_layout_elems(const ConvGeom& g);
void relayout_weights_batch(std::vector<WeightLayoutJob>& jobs, hipStream_t s);   // sets every job's `first`
// dw[Cout][K] = dy[M][Cout]^T * im2col(x)[M][K], split over M with fp32 partials reduced in fixed order
void conv_wgrad_mfma(const bf16_t* x, const bf16_t* dy, float* dw, const ConvGeom& g, float* partials,
                     size_t partials_bytes, hipStream_t s);
// Grouped convolutions (Cin = Cout = C, groups of C / groups channels) on the same kernels, reading and writing the
// row-major tensors in place: slices of grouped_mfma_slice(C, groups) = 32 or 64 channels (0: this shape is not taken;
// the slice must hold whole groups and divide C).  w is the grouped filter [C][kh][kw][C / groups]; wd is scratch for
// its per-slice form, at least C * kh * kw * 64 + 64 elements (fp32 elements for the weight gradient's dwd).
int grouped_mfma_slice(int C, int groups);
int conv_grouped_fprop_mfma(const bf16_t* x, const bf16_t* w, bf16_t* wd, bf16_t* y, const ConvGeom& g, int groups,
                            float* stat_partials, hipStream_t s);   // returns the number of statistics chunks
void conv_grouped_dgrad_mfma(const bf16_t* dy, const bf16_t* w, bf16_t* wd, bf16_t* dx, const ConvGeom& g, int groups,
                             bool accumulate, hipStream_t s);
void conv_grouped_wgrad_mfma(const bf16_t* x, const bf16_t* dy, float* dwd, float* dw, const ConvGeom& g, int groups,
                             float* partials, size_t partials_bytes, hipStream_t s);
// dense layer on the same kernel: y[B][C] (fp32) = x[B][F] * w[C][F]^T + bias; needs F % 8 == 0
void linear_fwd_mfma(const bf16_t* x, const bf16_t* w, const bf16_t* bias, float* y, int64_t B, int F, int C,
                     hipStream_t s);
void cast_f32_bf16(const float* in, bf16_t* out, int64_t n, hipStream_t s);
// [n][3] -> [n][8] zero padded (input images and the taps of a 3-channel filter)
void pad_c3_to_c8(const bf16_t* in, bf16_t* out, int64_t n, hipStream_t s);
// Space-to-depth form of a stride-2 convolution on 3-channel images (even H, W): xs is
// [B][H/2][W/2][16], ws [cout][ks][ks][16] with ks = ceil((k + shift) / 2), shift = 2*ceil(pad/2) - pad;
// the stride-1 convolution of xs with ws (padding ceil(pad/2)) equals the original one.
void s2d_pack_x(const bf16_t* x, bf16_t* xs, int64_t B, int H, int W, hipStream_t s);
void s2d_pack_w(const bf16_t* w, bf16_t* ws, int cout, int k, int ks, int shift, hipStream_t s);
void s2d_unpack_dw(const float* dws, float* dw, int cout, int k, int ks, int shift, hipStream_t s);
// fp32 [n][8] -> [n][3]
void unpad_c8_to_c3(const float* in, float* out, int64_t n, hipStream_t s);
// w[Cout][taps][Cin] -> wt[Cin][taps][Cout]
void transpose_weight(const bf16_t* w, bf16_t* wt, int cout, int taps, int cin, hipStream_t s);

// ---- conv_grouped.hip: a grouped convolution (Cin = Cout = C) as dense convolutions on channel slices ----
// slices of grouped_slice_width(C) channels (C itself up to 128, else 128), each a whole number of groups
int grouped_slice_width(int C);
bool grouped_conv_supported(int C, int groups);
// x [M][C] -> xs [C / SW][M][SW] and back (accumulate: added to what x holds)
void slices_gather(const bf16_t* x, bf16_t* xs, int64_t M, int C, hipStream_t s);
void slices_scatter(const bf16_t* xs, bf16_t* x, int64_t M, int C, bool accumulate, hipStream_t s);
// w [C][taps][C / groups] -> wd [C / SW][SW][taps][SW], zero outside the groups' diagonal blocks
void expand_group_weights(const bf16_t* w, bf16_t* wd, int C, int taps, int groups, hipStream_t s);
// dwd [C / SW][SW][taps][SW] fp32 -> dw [C][taps][C / groups]: the diagonal blocks
void extract_group_dw(const float* dwd, float* dw, int C, int taps, int groups, hipStream_t s);

// ---- attention.hip: multi-head scaled dot-product attention and the token embedding (bf16 tensors) ----
// q [S*Tq][.] and k, v [S*Tk][.] are bf16 row-major with row pitches ldq / ldkv (elements), already
// pointing at their first column; head h owns columns h*dh .. (h+1)*dh.  out [S*Tq][.] with pitch ldo.
// lse (nullable in a forward pass that keeps nothing): [S][heads][Tq] fp32 log-sum-exp of the scaled
// scores.  dh in {8, 16, 32, 64} (attention_supported).  key_tokens (nullable): int32 token ids [S][tok_pitch]; the keys
// of sentence s belong to columns key_col0 .. key_col0 + Tk, and only those before the first negative id (padding)
// take part; padded keys get zero dk, dv.
// Packed batches (tab != nullptr): the sentences lie one after the other in the query and key tensors.  q and k are
// device tables of max_sent + 2 entries (sentence_tables): [i] = first row of sentence i, [n] = the row after the last
// sentence, [max_sent + 1] = n.  S is then max_sent, Tq / Tk the longest sentence the launch covers, lse and dsum are
// [heads][q_rows] indexed by the query's row, and key_tokens is not used.  q_rows / k_rows: rows of the query / key
// tensors; the rows behind the last sentence are written as zeros in out, dq, dk and dv.
struct SentenceTables { const int32_t* q; const int32_t* k; int max_sent; int q_rows; int k_rows; };
// table (max_sent + 2 entries) from the rows' token ids and positions inside their sentences: a row with a
// non-negative id and position 0 starts a sentence; the rows after the last sentence have negative ids.
// Sentences beyond max_sent are left out.
void sentence_tables(const int32_t* tok, const int32_t* pos, int rows, int max_sent, int32_t* table, hipStream_t s);
bool attention_supported(int dh);
void attention_forward(const bf16_t* q, int64_t ldq, const bf16_t* k, const bf16_t* v, int64_t ldkv, bf16_t* out, int64_t ldo,
                       float* lse, int S, int heads, int Tq, int Tk, int dh, bool causal, const int32_t* key_tokens,
                       int64_t tok_pitch, int key_col0, const SentenceTables* tab, hipStream_t s);
// dq, dk, dv are written (not accumulated), with the pitches of q and k / v; dsum: [S][heads][Tq] fp32 scratch.
void attention_backward(const bf16_t* q, int64_t ldq, const bf16_t* k, const bf16_t* v, int64_t ldkv, const bf16_t* dout,
                        int64_t ldo, const float* lse, float* dsum, bf16_t* dq, bf16_t* dk, bf16_t* dv, int S, int heads,
                        int Tq, int Tk, int dh, bool causal, const int32_t* key_tokens, int64_t tok_pitch, int key_col0,
                        const SentenceTables* tab, hipStream_t s);
// y[s*len + t][:] = table[tok[s*tok_pitch + col0 + t]][:] * sqrt(d) + the sinusoidal position signal of t (d even);
// a negative id (padding) gives the position signal alone and takes no gradient.  pos (nullable, packed batches):
// the position of every token inside its sentence, laid out like tok; t is then read from it.
void embed_forward(int dtype, const int32_t* tok, int64_t tok_pitch, int col0, int len, const void* table, int vocab, int d,
                   void* y, int64_t rows, const int32_t* pos, hipStream_t s);
// dtable[tok] += sqrt(d) * dy[row], added onto a gradient that already holds the other uses of the table; one writer per
// table row, additions in position order (bit-reproducible)
void embed_backward(int dtype, const int32_t* tok, int64_t tok_pitch, int col0, int len, const void* dy, int vocab, int d,
                    float* dtable, int64_t rows, hipStream_t s);

}  // namespace cd
