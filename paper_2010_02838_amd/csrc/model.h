// Host-side model description: parameter table, fused op list, workspace plan.
#pragma once
#include "common.h"
#include <string>
#include <vector>

namespace cd {

enum OpKind { OP_CONV, OP_BN, OP_MAXPOOL, OP_GAP, OP_LINEAR, OP_LN, OP_EMBED, OP_ATTN, OP_SLICE };

struct TensorDesc {
  int h = 1, w = 1, c = 1;  // per-sample shape; a [B, F] tensor has h = w = 1
  bool f32 = false;         // logits are fp32 whatever the model dtype
  int64_t per_sample() const { return (int64_t)h * w * c; }
};

struct Op {
  OpKind kind;
  int x = -1, y = -1;  // input / output tensor ids
  int res = -1;        // OP_BN: tensor added before the ReLU; OP_LN: tensor added to x (-1: none);
                       // OP_ATTN: the tensor that holds keys and values (may be x itself)
  bool relu = false;   // OP_CONV (after the bias) and OP_BN
  int pw = -1, pb = -1;  // parameter indices: conv/linear weight + bias, BN gamma + beta
  int k = 1, stride = 1, pad = 0;
  int bn_slot = -1;    // OP_BN: index into the per-BN statistics area
  // OP_SLICE: a0 = first channel of x that y receives (y is narrower than x); the ops in front of it are frozen.
  // OP_EMBED: a0 = first token column of the input, a1 = tokens per sentence.
  // OP_ATTN: a0, a1, a2 = first column of the queries in x, of the keys and of the values in res;
  //          heads, causal; the width of each column range is the width of y.
  int a0 = 0, a1 = 0, a2 = 0, heads = 0;
  int key_tok0 = 0;    // OP_ATTN: first token column of the sentences the keys come from (their padding is masked)
  int q_stream = 0, k_stream = 0;   // OP_ATTN: which token stream (0 source, 1 target) the queries and the keys belong to
  bool causal = false;
  bool tied = false;   // OP_LINEAR: the weight is another op's parameter (the embedding table)
  int groups = 1;      // OP_CONV: groups of a grouped convolution (input and output channels are then equal)
};

struct ParamDesc {
  std::string name;
  int kind;
  int ndim;
  int64_t shape[4];
  int64_t offset, size, fan_in;
};

// Where everything lives inside the caller's workspace for one batch size.
struct Plan {
  int64_t batch = 0;
  bool save = false;
  std::vector<size_t> act;    // byte offset of every tensor's activation (tensor 0 unused)
  std::vector<size_t> grad;   // byte offset of every tensor's gradient (save only)
  std::vector<size_t> aux;    // per op (save only): max-pool argmax bytes, ReLU sign bits of a BatchNorm,
                              // per-row mean and rstd of a LayerNorm, per (sentence, head, query) log-sum-exp
                              // and dO.O of an attention; 0 = none
  size_t bn_stats = 0;        // per BN slot: mean[C], invstd[C], scale[C], shift[C] fp32
  size_t bn_coef = 0;         // backward coefficients c1,c2,c3 [3][Cmax] fp32
  size_t partials = 0;        // reduction partials / split-K partials
  size_t partials_bytes = 0;
  size_t partials_side = 0;   // split-K partials of the weight gradients that run on the side stream (save only)
  size_t xpack = 0;           // bf16 models: input packed to 8 channels
  size_t wpack = 0;           // bf16 models: re-laid-out weights (stem padding, dgrad transposes)
  size_t wpack_bytes = 0;
  size_t lin_dz = 0;          // bf16 models: bf16 copy of d loss / d logits for the dense-layer MFMA backward
  // grouped convolutions (see conv_grouped.hip)
  std::vector<size_t> gx;     // per op (save only): the op's input in slice-major form, kept for the weight gradient
  size_t gtmp = 0;            // two slice-major tensors of scratch (output / gradients), each gtmp_bytes
  size_t gtmp_bytes = 0;
  size_t gw = 0;              // the dense per-slice filters of the op at hand
  size_t gdw = 0;             // save only: the dense per-slice filter gradients of the op at hand (fp32)
  std::vector<size_t> wt_op;  // per op (save only): where the backward pass keeps the convolution's filter as its data gradient
                              // reads it (all of them are re-laid-out by one launch at the start of the pass); 0 = none
  size_t seq_tab = 0;         // packed Transformer batches: the sentence tables of the source and of the target stream,
                              // max_sentences + 2 int32 each (kernels.h, sentence_tables)
  size_t total = 0;
};

}  // namespace cd

struct cd_model {
  cd_arch_desc arch;
  int dtype;
  std::vector<cd::TensorDesc> tensors;
  std::vector<cd::Op> ops;
  std::vector<cd::ParamDesc> params;
  int64_t n_elements = 0;  // padded flat size
  int n_bn = 0;
  int64_t bn_c_total = 0;  // sum of BN channel counts
  std::vector<int64_t> bn_off;  // per BN slot: channel offset into the statistics area
  int max_c = 1;
  int first_trainable_op = 0;   // ops before it are frozen: the backward pass stops there (index behind an OP_SLICE)
  size_t esize() const { return dtype == CD_BF16 ? 2 : 4; }
};

namespace cd {
Plan make_plan(const cd_model* m, int64_t batch, bool save);
}
