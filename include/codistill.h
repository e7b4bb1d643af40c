/*
 * codistill.h - C ABI of the MI355X (gfx950) codistillation-step library.
 *
 * One GPU's share of one codistillation training step (paper, Algorithm 1, the
 * per-model update, in the checkpoint-exchange implementation of Section 3):
 *
 *     z  = f_theta (x)     codistill_forward(local model, save_for_backward = 1)
 *     z' = f_theta'(x)     codistill_forward(stale peer copy, save_for_backward = 0)
 *     l  = L(y,z) + alpha * mean_j D(z, z'_j),  dz = dl/dz      codistill_loss_grad
 *     g  = dl/dtheta       codistill_backward (local model only)
 *     theta <- momentum-SGD(theta, g)                           codistill_sgd_step (or codistill_adam_step)
 *
 * Conventions
 *   - Every function returns CD_OK (0) or a negative CD_ERR_* code and never
 *     throws or aborts; codistill_last_error() returns a thread-local message
 *     for the last failing call on this thread.
 *   - Unless marked "host", every data pointer is a DEVICE pointer owned by the
 *     caller, 16-byte aligned.  The library does not allocate, free or retain
 *     device memory; all temporary storage is the caller's workspace / scratch.
 *   - Calls only enqueue work (`stream` is a hipStream_t passed as void*; NULL is
 *     the default stream) and never synchronise the host.  Everything is enqueued
 *     on the caller's stream, with one exception: codistill_backward forks the
 *     weight gradients of the convolutions onto a second stream that the library
 *     creates on first use (default priority, one per process) and joins it back
 *     with an event before it returns, so the caller's stream still orders the
 *     whole call.  CODISTILL_SERIAL=1 in the environment, or the built-in timer,
 *     keeps every launch on the caller's stream.
 *   - Arguments, and whether every op of the model has a kernel for them, are
 *     checked on the host before any launch: a call that returns
 *     CD_ERR_INVALID_ARG, CD_ERR_UNSUPPORTED or CD_ERR_WORKSPACE_TOO_SMALL has
 *     launched nothing.  CD_ERR_HIP reports a failure of the runtime during or
 *     after the launches: the outputs are then undefined and the device should
 *     be synchronised before its buffers are reused.
 *   - Threads: the entry points may be called from several host threads on
 *     different streams.  codistill_backward calls are serialised among
 *     themselves by a lock (they share the second stream); calls that share a
 *     workspace, scratch or output buffer must be ordered by the caller.  One
 *     device per process: the second stream lives on the device that was
 *     current at the first codistill_backward.
 *   - Environment switches read at call time, for comparing code paths (the
 *     results agree; see the tests): CODISTILL_SERIAL, CODISTILL_FORCE_SIMPLE
 *     (plain one-thread-per-output kernels instead of the MFMA ones),
 *     CODISTILL_NO_POOL_FUSION, CODISTILL_WRITE_RESIDUAL_GRADS,
 *     CODISTILL_SEPARATE_RELU_MASK, CODISTILL_SEPARATE_BN_REDUCTION,
 *     CODISTILL_PLAIN_ATTENTION.
 *   - Layouts: activations NHWC, filters [Cout][kh][kw][Cin], linear weights
 *     [out][in], logits row-major [rows][cols].  bf16 is the upper half of an
 *     IEEE float32, round-to-nearest-even.
 */
#ifndef CODISTILL_H
#define CODISTILL_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
  CD_OK = 0,
  CD_ERR_INVALID_ARG = -1,
  CD_ERR_UNSUPPORTED = -2,
  CD_ERR_WORKSPACE_TOO_SMALL = -3,
  CD_ERR_HIP = -4
};

/* storage / compute type of a model: CD_F32 = fp32 everywhere; CD_BF16 = bf16
 * weights and activations, fp32 accumulation, statistics, logits and gradients */
enum { CD_F32 = 0, CD_BF16 = 1 };

/* distillation term D.  CD_DIST_MSE_LOGITS: mean squared error between the raw,
 * uncentred logits (paper, appendix "Implementation Details").  CD_DIST_KL:
 * KL(softmax(z') || softmax(z)), the choice of the prior work cited in Section 2.
 * CD_DIST_MSE_CENTERED: the squared error after each model's logit row has had its
 * own mean over the classes subtracted (the centring the same appendix reports trying);
 * normalised like CD_DIST_MSE_LOGITS. */
enum { CD_DIST_MSE_LOGITS = 0, CD_DIST_KL = 1, CD_DIST_MSE_CENTERED = 2 };
/* normaliser of the squared error: all rows*cols elements, or rows only */
enum { CD_MEAN_ALL = 0, CD_MEAN_ROWS = 1 };

/* BatchNorm mode of a forward pass: the statistics of the batch (training, and the stale peer's pass), or the
 * running averages (evaluation; forward only).  See codistill_forward. */
enum { CD_BN_BATCH_STATS = 0, CD_BN_RUNNING = 1 };

/* architecture families (the paper names ResNet50, Section 3; the others are
 * the small workloads used to check the step) */
enum {
  CD_ARCH_TINY_CNN = 0,          /* conv3x3(3->16)+b, ReLU, conv3x3(16->32)+b, ReLU, GAP, linear */
  CD_ARCH_RESNET_BASIC = 1,      /* CIFAR-style: 3x3 stem, basic blocks, projection shortcuts    */
  CD_ARCH_RESNET_BOTTLENECK = 2, /* 7x7-s2 stem, 3x3-s2 max-pool, bottleneck blocks (x4)         */
  CD_ARCH_RESNET_BASIC_IMAGENET = 5, /* basic blocks behind the 7x7 stride-2 stem and 3x3 stride-2 max-pool of
                                        CD_ARCH_RESNET_BOTTLENECK (ResNet-18/34: the smaller model of the pairs of
                                        different architectures in Section 5); projection shortcut where the
                                        stride or the width changes */
  CD_ARCH_RESNEXT = 6,           /* CD_ARCH_RESNET_BOTTLENECK with a grouped 3x3 convolution (aggregated
                                    transformations; the largest model of the pairs of different architectures in
                                    Section 5).  CD_BF16 only; the grouped convolution's channel count must be a
                                    multiple of 8 and, above 128, of 128, with whole groups per 128 channels */
  CD_ARCH_WIDE_RESNET_SPLIT = 7,  /* the modified Wide-ResNet of the multi-view experiment (Section 5): CD_ARCH_RESNET_BASIC
                                    (3x3 stem, basic blocks; 28x10: three stages of four blocks, widths 160/320/640,
                                    stem 16) whose first block is a frozen front end.  The front end's output channels
                                    (widths[0] = 160) are cut into n_splits equal parts and the rest of the network
                                    receives part `split` only (20 channels for 8 parts).  Frozen: codistill_backward
                                    stops at the cut, the gradients of the stem and of the first block are written as
                                    zeros (their parameters stay as loaded, "pre-trained").  Its BatchNorms use
                                    the batch's statistics like every other */
  CD_ARCH_TRANSFORMER = 4,       /* the encoder-decoder Transformer of Section 4 (Vaswani et al.): embedding of the shared
                                    vocabulary times sqrt(d_model) plus the sinusoidal position signal; encoder layers
                                    (self-attention, feed-forward), decoder layers (causal self-attention, attention over
                                    the encoder output, feed-forward), every sublayer followed by its residual connection
                                    and LayerNorm; logits against the tied embedding table.  No dropout; every sentence
                                    has room for in_h source and in_w target tokens, shorter ones are padded with
                                    negative ids (see cd_arch_desc).  CD_BF16 only */
  CD_ARCH_TRANSFORMER_HEAD = 3   /* the last position-wise sublayers of a Transformer decoder (Section 4 trains the
                                    Transformer of Vaswani et al.): h + W2 relu(W1 h + b1) + b2, LayerNorm, projection
                                    onto the vocabulary without bias.  The input is the hidden state of every
                                    target token, [rows][1][1][d_model]; the attention sublayers and the embeddings
                                    are not part of it */
};

#define CD_MAX_STAGES 4
#define CD_NAME_LEN 48

/* host struct.  Input images have 3 channels; CD_ARCH_TRANSFORMER_HEAD takes widths[0] = d_model input
 * channels (in_h = in_w = 1), widths[1] = d_ff, classes = vocabulary size.  CD_ARCH_TRANSFORMER: in_h = source
 * tokens and in_w = target tokens per sentence, widths[0] = d_model, widths[1] = d_ff, widths[2] = heads,
 * blocks[0] = encoder layers, blocks[1] = decoder layers, classes = vocabulary size; its input x is
 * int32 [batch][in_h + in_w] token ids (batch = sentences) and it produces batch * in_w rows of logits.  Shorter
 * sentences are padded at the end of their source / target part with negative ids: padding embeds as a zero row,
 * is masked as a key in every attention and takes no gradient; give its rows of the targets ignore_index.  Every
 * part needs at least one real token.
 * Packed sentences (max_sentences > 0): a batch of sentences of different lengths without the padding.  The
 * sentences' tokens lie one after the other; in_h and in_w are the rows the source and the target stream have room
 * for (up to 65536 each), batch is 1, and x is int32 [2][in_h + in_w]: row 0 the token ids (source stream, then
 * target stream; the rows of a stream behind its last sentence hold negative ids), row 1 the position of every
 * token inside its own sentence (0 starts a sentence).  Both streams hold the same sentences in the same order, every
 * sentence has at least one token in each, at most max_sentence_len, and there are at most max_sentences of them
 * (what exceeds either bound is left out of the attention; nothing is read or written out of bounds).  The
 * model produces in_w rows of logits, one per target row; the rows behind the last sentence are not defined: give
 * them ignore_index in the targets.  Everything else (parameters, losses, gradients) is as for padded sentences, and
 * equal to it up to rounding order when the same sentences are given in both forms. */
typedef struct {
  int32_t kind;                   /* CD_ARCH_*                                             */
  int32_t classes;                /* width of the logits                                   */
  int32_t in_h, in_w;             /* input resolution                                      */
  int32_t n_stages;               /* residual families: 1..CD_MAX_STAGES; tiny CNN: unused */
  int32_t widths[CD_MAX_STAGES];  /* stage widths (bottleneck: inner width, output is x4); */
                                  /* tiny CNN: widths[0], widths[1] = the two conv widths  */
  int32_t blocks[CD_MAX_STAGES];  /* blocks per stage                                      */
  int32_t stem_width;             /* output channels of the stem convolution               */
  int32_t groups;                 /* CD_ARCH_RESNEXT: groups of the 3x3 convolution        */
  int32_t out_widths[CD_MAX_STAGES]; /* CD_ARCH_RESNEXT: output channels of a stage's blocks
                                        (widths[] are those of its grouped convolution)    */
  int32_t n_splits, split;        /* CD_ARCH_WIDE_RESNET_SPLIT: parts the front end's output channels are
                                     cut into (widths[0] % n_splits == 0), and the part this model receives */
  int32_t max_sentences;          /* CD_ARCH_TRANSFORMER: 0 = padded sentences (above); > 0 = packed sentences (below): */
  int32_t max_sentence_len;       /*   the most sentences a batch may hold, and the most tokens one sentence may have   */
} cd_arch_desc;

/* kind of a parameter tensor */
enum { CD_P_CONV_W = 0, CD_P_BIAS = 1, CD_P_BN_GAMMA = 2, CD_P_BN_BETA = 3, CD_P_LINEAR_W = 4,
       CD_P_EMBED_W = 5 /* [vocabulary][d_model] table, also the weight of the tied output projection */ };

/* host struct describing one parameter tensor inside the flat buffers */
typedef struct {
  char name[CD_NAME_LEN];
  int32_t kind;      /* CD_P_*                                                      */
  int32_t ndim;      /* 1, 2 or 4                                                   */
  int64_t shape[4];  /* conv [Cout,kh,kw,Cin]; linear [out,in]; others [C]          */
  int64_t offset;    /* element offset in the flat parameter / gradient buffers     */
  int64_t size;      /* number of elements                                          */
  int64_t fan_in;    /* Cin*kh*kw or in_features; 0 for scale / shift / bias        */
  int32_t frozen;    /* 1: the tensor belongs to a frozen front end (CD_ARCH_WIDE_RESNET_SPLIT):
                        codistill_backward writes zeros as its gradient and the caller leaves it out of
                        the update.  Frozen tensors come first in declaration order                  */
} cd_tensor_info;

typedef struct cd_model cd_model; /* opaque host object */

/* Fill *out with a preset: CD_ARCH_TINY_CNN (32x32, 10 classes), CD_ARCH_RESNET_BASIC
 * (ResNet-20: 32x32, widths 16/32/64, 3 blocks each, 10 classes), CD_ARCH_RESNET_BOTTLENECK
 * (ResNet-50: 224x224, widths 64..512, blocks 3/4/6/3, 1000 classes; Section 3),
 * CD_ARCH_TRANSFORMER_HEAD (d_model 512, d_ff 2048, vocabulary 32768: the base Transformer),
 * CD_ARCH_RESNEXT (the 101-layer 32x8d model: blocks 3,4,23,3, grouped widths 256..2048 in 32 groups),
 * CD_ARCH_RESNET_BASIC_IMAGENET (ResNet-18: blocks 2,2,2,2, widths 64..512, 224x224, 1000 classes),
 * CD_ARCH_TRANSFORMER (the base model: 6 + 6 layers, d_model 512, 8 heads, d_ff 2048, vocabulary 32768,
 * 128 source and 128 target tokens per sentence), CD_ARCH_WIDE_RESNET_SPLIT (28x10 on 32x32 images, 10 classes,
 * 8 parts of 20 channels, part 0). host. */
int codistill_arch_preset(int kind, cd_arch_desc* out);

/* Build the host-side description (op list, parameter table) of a model.
 * dtype: CD_F32 or CD_BF16.  *out is owned by the caller until codistill_model_destroy. */
int codistill_model_create(const cd_arch_desc* arch, int dtype, cd_model** out);
void codistill_model_destroy(cd_model* m);

/* number of parameter tensors and of parameter elements. host outputs. */
int codistill_param_count(const cd_model* m, int64_t* n_tensors, int64_t* n_elements);
/* describe parameter tensor idx (declaration order). host output. */
int codistill_param_info(const cd_model* m, int64_t idx, cd_tensor_info* out);
/* bytes of workspace a forward (and, with save_for_backward, the matching backward)
 * needs for this batch size. host output. */
int codistill_workspace_bytes(const cd_model* m, int64_t batch, int save_for_backward, size_t* bytes);

/*
 * z = f_params(x): training-mode forward pass (Algorithm 1: f_theta(x); Section 3: the
 * device runs one forward for its own model and one per stale peer, on the same minibatch).
 *   params      flat parameter buffer in the model's dtype (fp32 or bf16), declaration order
 *   x           [batch][in_h][in_w][3] ([batch][1][1][d_model] for CD_ARCH_TRANSFORMER_HEAD) in the model's dtype
 *   save_for_backward  1: keep in `workspace` what codistill_backward needs (local model);
 *                      0: keep nothing (peer model; its logits are constants)
 *   bn_mode     CD_BN_BATCH_STATS: every BatchNorm uses the statistics of this batch (training; also what the stale
 *               peer's forward pass uses).  CD_BN_RUNNING: evaluation mode, the running averages in bn_running are
 *               used instead (save_for_backward must be 0)
 *   bn_running  NULL, or device fp32 [codistill_bn_running_elements(m)]: per BatchNorm op, in graph order, its
 *               running mean [C] then running variance [C] (the caller initialises them to 0 and 1).  With
 *               CD_BN_BATCH_STATS and a non-NULL pointer the pass also updates them: 0.9 old + 0.1 batch value,
 *               the batch variance in its unbiased form (the paper is silent; the common convention)
 *   workspace   at least codistill_workspace_bytes(m, batch, save_for_backward) bytes; with
 *               save_for_backward the same buffer must be handed, untouched, to codistill_backward
 *   logits_out  [batch][classes] fp32
 * Errors: NULL pointer, batch <= 0, unknown mode -> CD_ERR_INVALID_ARG; small workspace ->
 * CD_ERR_WORKSPACE_TOO_SMALL; launch failure -> CD_ERR_HIP.
 */
/* elements of the bn_running buffer of codistill_forward: twice the channels of all BatchNorm ops. host output. */
int codistill_bn_running_elements(const cd_model* m, int64_t* n);
int codistill_forward(const cd_model* m, const void* params, const void* x, int64_t batch,
                      int save_for_backward, int bn_mode, float* bn_running,
                      void* workspace, size_t workspace_bytes, float* logits_out, void* stream);

/* host struct */
typedef struct {
  float alpha;            /* penalty coefficient alpha^k of Algorithm 1                        */
  float label_smoothing;  /* in [0,1): target distribution (1-eps) onehot + eps/cols           */
  int32_t dist_kind;      /* CD_DIST_*                                                         */
  int32_t mse_reduction;  /* CD_MEAN_*; read for the two squared-error terms                  */
  int32_t ignore_index;   /* rows whose target equals this add nothing and get a zero gradient */
  int32_t n_peers;        /* n-1 of Algorithm 1; 0 = no distillation term this iteration       */
  float temperature;      /* CD_DIST_KL only: tau^2 KL(softmax(z'/tau) || softmax(z/tau)), the usual form of
                             distillation; the paper uses none: 1 (or 0, read as 1) is its term     */
} cd_loss_cfg;

#define CD_LOSS_MAX_PEERS 8

/* bytes of scratch codistill_loss_grad needs for this row count. host output. */
int codistill_loss_scratch_bytes(int64_t rows, int64_t cols, size_t* bytes);

/*
 * Codistillation loss and its gradient with respect to the local logits (Algorithm 1: the
 * objective inside the gradient; Section 3: peers are constants, and the distillation term
 * is left out on iterations without peer predictions):
 *     task    = mean over valid rows of cross-entropy(q_row, softmax(z_row))
 *     distill = mean over peers of D(z, z'_j), mean over valid rows (and columns for MSE/ALL)
 *     total   = task + alpha * distill
 *     dz      = d total / d z
 *   z_local   [rows][cols] fp32
 *   z_peers   HOST array of n_peers device pointers, each [rows][cols] fp32; may be NULL when
 *             n_peers == 0
 *   targets   [rows] int32 class ids.  A target equal to ignore_index skips the row; any other
 *             target outside [0, cols) also skips the row and sets bit 0 of the status word
 *   loss_out  device float[4]: total, task, distill, and the status word (as int32 bits)
 *   dz_out    [rows][cols] fp32; may alias z_local
 *   scratch   at least codistill_loss_scratch_bytes(rows, cols) bytes
 * Supported: 1 <= cols <= 2^24, 1 <= rows <= 2^31-1, 0 <= n_peers <= CD_LOSS_MAX_PEERS.
 * Errors: NULL required pointer, rows/cols out of range, unknown enum, n_peers out of range,
 * label_smoothing outside [0,1), misaligned pointer -> CD_ERR_INVALID_ARG; small scratch ->
 * CD_ERR_WORKSPACE_TOO_SMALL.
 */
int codistill_loss_grad(const float* z_local, const float* const* z_peers, const int32_t* targets,
                        int64_t rows, int64_t cols, const cd_loss_cfg* cfg,
                        float* loss_out, float* dz_out, void* scratch, size_t scratch_bytes,
                        void* stream);

/*
 * codistill_loss_grad for callers that cannot allocate device memory or hand over a scratch buffer: code under
 * HIP graph capture, tight serving or training loops, harnesses that forbid hipMalloc.  Same arguments, results and
 * errors as codistill_loss_grad, minus scratch / scratch_bytes: the per-row terms and the row counter go to a
 * device array inside the library (16 + 8 * CD_LOSS_STATIC_MAX_ROWS bytes = 512 KiB + 16 B on every GPU the library
 * runs on, held until the process ends).  The call allocates and frees nothing, on the device or through any
 * library.  rows above CD_LOSS_STATIC_MAX_ROWS -> CD_ERR_INVALID_ARG, nothing launched.  All calls on one GPU share
 * the one array: calls that may overlap on a GPU (different streams, different host threads) race on it and must
 * be ordered by the caller; calls in stream order need nothing (each call writes what it later reads, nothing has
 * to be cleared in between).
 */
#define CD_LOSS_STATIC_MAX_ROWS 65536
int codistill_loss_grad_static(const float* z_local, const float* const* z_peers, const int32_t* targets,
                               int64_t rows, int64_t cols, const cd_loss_cfg* cfg,
                               float* loss_out, float* dz_out, void* stream);

/*
 * Backward pass of the local model (Section 3: only with respect to the local parameters).
 * Consumes the workspace written by codistill_forward(..., save_for_backward = 1, ...) with the
 * same model, params, x and batch.
 *   dlogits    [batch][classes] fp32, d loss / d logits
 *   grads_out  flat fp32 gradient, same offsets as the parameter buffer; fully overwritten
 */
int codistill_backward(const cd_model* m, const void* params, const void* x, int64_t batch,
                       void* workspace, size_t workspace_bytes, const float* dlogits,
                       float* grads_out, void* stream);

/*
 * Momentum-SGD update, in place (Algorithm 1: theta <- theta - eta * gradient; momentum form of
 * the large-minibatch recipe the paper follows, Section 4.1):
 *     g = grad + weight_decay * w;  v = momentum * v + g;
 *     w = w - lr * (nesterov ? g + momentum * v : v)
 *   master_w, momentum_v  [n] fp32, updated in place;  grad [n] fp32, read only
 *   lowp_w_out  [n] bf16 copy of the updated weights, or NULL
 * The caller calls it once per group of tensors that share lr / weight_decay.
 */
int codistill_sgd_step(float* master_w, float* momentum_v, const float* grad, void* lowp_w_out,
                       int64_t n, float lr, float momentum, float weight_decay, int nesterov,
                       void* stream);

/*
 * Adam update, in place: the optimiser of the translation recipe that Section 4 follows (Ott et al.: beta1 0.9,
 * beta2 0.98, eps 1e-8); Kingma & Ba's algorithm with the coupled L2 term of codistill_sgd_step:
 *     g = grad + weight_decay * w;  m = beta1 m + (1 - beta1) g;  v = beta2 v + (1 - beta2) g^2;
 *     w = w - lr * (m / (1 - beta1^t)) / (sqrt(v / (1 - beta2^t)) + eps)
 *   master_w, exp_avg (m), exp_avg_sq (v)  [n] device fp32, updated in place (m and v start at zero)
 *   grad  [n] device fp32, read only;  lowp_w_out  [n] device bf16 copy of the updated weights, or NULL
 *   t     number of this update, counted from 1 (host value; the bias corrections are computed on the host)
 * Errors (CD_ERR_INVALID_ARG, nothing launched): NULL or misaligned pointers, n < 1, t < 1, beta outside [0, 1),
 * eps <= 0, NaN lr or weight_decay.
 */
int codistill_adam_step(float* master_w, float* exp_avg, float* exp_avg_sq, const float* grad, void* lowp_w_out,
                        int64_t n, float lr, float beta1, float beta2, float eps, float weight_decay, int64_t t,
                        void* stream);

/* ---- introspection ----------------------------------------------------------------------- */
/* The fused op list and where each tensor lives inside a save_for_backward workspace, so that
 * tools and tests can read intermediate activations and activation gradients after a forward /
 * backward pair.  Tensor 0 is the input batch; the last op writes the logits (not in the workspace). */
enum { CD_OP_CONV = 0, CD_OP_BN = 1, CD_OP_MAXPOOL = 2, CD_OP_GAP = 3, CD_OP_LINEAR = 4, CD_OP_LN = 5,
       CD_OP_EMBED = 6, CD_OP_ATTN = 7,
       CD_OP_SLICE = 8 /* y = channels k .. k + width(y) of x; no gradient passes it (the ops in front of it are frozen) */ };
typedef struct {
  int32_t kind;            /* CD_OP_*                                                           */
  int32_t x, y;            /* input / output tensor ids                                         */
  int32_t res;             /* CD_OP_BN: tensor added before the ReLU; CD_OP_LN: tensor added to x; CD_OP_ATTN: the
                              tensor that holds keys and values (may be x); else -1                      */
  int32_t relu;            /* CD_OP_CONV (after the bias) and CD_OP_BN: ReLU fused into the op  */
  int32_t param_w, param_b;/* parameter indices: weight + bias, or BN scale + shift; -1 if none */
  int32_t k, stride, pad;  /* window of CD_OP_CONV / CD_OP_MAXPOOL; CD_OP_ATTN: k = heads, stride = 1 if causal;
                              CD_OP_EMBED: k = first token column of the input, stride = tokens per sentence;
                              CD_OP_ATTN also: pad = first column of the queries in x                   */
  int64_t stats_offset;    /* CD_OP_BN: byte offset of fp32 [4][C] = mean, invstd, scale, shift;
                              CD_OP_LN: of fp32 [batch][2] = mean, rstd per row                 */
  int32_t res_grad;        /* CD_OP_BN with a residual input: how the backward pass hands on the gradient of
                              that input (this op's dy, gated by its ReLU).  0: added to the residual tensor's
                              gradient buffer.  1: not written; the op that produced the residual tensor (a
                              ReLU-free BatchNorm read by nothing else) reads this op's dy through the ReLU bit
                              mask, and the residual tensor's gradient buffer stays unused.  2: not written by
                              this op; the data gradient of the one convolution that reads the same tensor adds
                              it, so the buffer holds the complete gradient after that launch.            */
  int32_t k_col, v_col;    /* CD_OP_ATTN: first column of the keys and of the values in tensor res (each range is
                              as wide as the op's output)                                                */
  int32_t fused_pool;      /* CD_OP_BN: 1 if the max-pool op that follows is computed by this op's kernel; this op's
                              output tensor is then never written (its workspace slot stays unused), its ReLU bit
                              mask and the pool's argmax are.                                             */
  int32_t key_tok0;        /* CD_OP_ATTN: first column of the token input whose sentences the keys come from; the
                              keys at and after a sentence's first negative id (padding) are masked        */
} cd_op_info;
typedef struct {
  int32_t h, w, c;         /* per-sample shape; the tensor is [batch][h][w][c]                  */
  int32_t is_f32;          /* 1 for the logits, else the model dtype                            */
  int64_t act_offset;      /* byte offset of the activation in the workspace, -1 if not there   */
  int64_t grad_offset;     /* byte offset of its gradient, -1 if not there                      */
} cd_act_info;
int codistill_graph_size(const cd_model* m, int64_t* n_ops, int64_t* n_tensors);
int codistill_op_info(const cd_model* m, int64_t batch, int64_t idx, cd_op_info* out);
int codistill_tensor_info(const cd_model* m, int64_t batch, int64_t idx, cd_act_info* out);

/* ---- measurement aid -------------------------------------------------------------------- */
/* kernel classes for the built-in timer */
enum {
  CD_K_CONV_FPROP = 0,        /* bf16 MFMA fprop launches on 128x128 tiles (one kernel symbol) */
  CD_K_CONV_DGRAD = 1, CD_K_CONV_WGRAD = 2,
  CD_K_NORM = 3,              /* normalisation launches other than CD_K_BN_APPLY */
  CD_K_GLUE = 4, CD_K_LINEAR = 5, CD_K_LOSS = 6, CD_K_SGD = 7,
  CD_K_CONV_FPROP_NARROW = 8, /* every other fprop launch (other tile shapes, plain kernels) */
  CD_K_BN_APPLY = 9,          /* BatchNorm forward: the elementwise normalise (+ residual, ReLU) kernel alone */
  CD_K_CONV_FPROP_WIDE = 10,  /* bf16 MFMA fprop launches on 128x256 tiles (one kernel symbol) */
  CD_K_ATTN = 11,             /* attention forward and backward launches */
  CD_K_COUNT = 12
};
/* When enabled, every launch is bracketed by HIP events on the launch stream and the events are
 * kept in a host-side pool (created at enable time; no device memory).  host. */
int codistill_profile_enable(int on);
/* Synchronises the recorded events, adds the elapsed times to the per-class totals and clears the
 * pool.  host. */
int codistill_profile_collect(void);
/* totals since the last reset: milliseconds, launches, algorithmic flops and bytes. host outputs. */
int codistill_profile_get(int kernel_class, double* ms, int64_t* launches, double* flops, double* bytes);
int codistill_profile_reset(void);
/* What the timer's pair of events adds to a launch: mean time between two events recorded around an empty kernel
 * on `stream` (200 launches, the last 100 averaged; synchronises the stream).  A class's time per launch exceeds
 * the kernel durations a profiler reports by about this much.  host output, microseconds. */
int codistill_profile_event_overhead(double* microseconds, void* stream);

const char* codistill_last_error(void);
const char* codistill_version(void);

#ifdef __cplusplus
}
#endif
#endif /* CODISTILL_H */
