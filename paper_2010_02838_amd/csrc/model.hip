// Model description, workspace plan, and the forward / backward executors.
//
// Paper, Section 3 (checkpoint-exchange implementation of Algorithm 1): per step a device runs
// one forward pass per model (its own, keeping what the backward pass needs, and each stale
// peer's, keeping nothing) and one backward pass, with respect to its own parameters only.
// The executors below enqueue exactly that on the caller's stream.
#include "model.h"
#include <mutex>
#include "kernels.h"
#include <cstdio>
#include <cstdlib>
#include <cstring>

using namespace cd;

// ------------------------------------------------------------------------------ construction
namespace {

struct Builder {
  cd_model* m;
  int add_tensor(int h, int w, int c, bool f32 = false) {
    TensorDesc t;
    t.h = h; t.w = w; t.c = c; t.f32 = f32;
    m->tensors.push_back(t);
    return (int)m->tensors.size() - 1;
  }
  int add_param(const std::string& name, int kind, int ndim, const int64_t* shape, int64_t fan_in) {
    ParamDesc p;
    p.name = name; p.kind = kind; p.ndim = ndim; p.fan_in = fan_in;
    p.size = 1;
    for (int i = 0; i < 4; i++) { p.shape[i] = i < ndim ? shape[i] : 1; p.size *= p.shape[i]; }
    p.offset = m->n_elements;
    m->n_elements += (p.size + 7) / 8 * 8;  // every tensor starts on a 16-byte (bf16) boundary
    m->params.push_back(p);
    return (int)m->params.size() - 1;
  }
  int conv_w(const std::string& n, int cin, int cout, int k) {
    int64_t sh[4] = {cout, k, k, cin};
    return add_param(n + ".w", CD_P_CONV_W, 4, sh, (int64_t)cin * k * k);
  }
  int vec(const std::string& n, int kind, int c) {
    int64_t sh[1] = {c};
    return add_param(n, kind, 1, sh, 0);
  }
  // ops
  int conv(int x, int pw, int pb, int cout, int k, int stride, int pad, bool relu, int groups = 1) {
    const TensorDesc& tx = m->tensors[x];
    Op o;
    o.kind = OP_CONV; o.x = x; o.pw = pw; o.pb = pb; o.k = k; o.stride = stride; o.pad = pad; o.relu = relu;
    o.groups = groups;
    o.y = add_tensor((tx.h + 2 * pad - k) / stride + 1, (tx.w + 2 * pad - k) / stride + 1, cout);
    m->ops.push_back(o);
    return o.y;
  }
  int bn(int x, int pg, int pb, int res, bool relu) {
    const TensorDesc tx = m->tensors[x];
    Op o;
    o.kind = OP_BN; o.x = x; o.pw = pg; o.pb = pb; o.res = res; o.relu = relu;
    o.bn_slot = m->n_bn++;
    m->bn_off.push_back(m->bn_c_total);
    m->bn_c_total += tx.c;
    o.y = add_tensor(tx.h, tx.w, tx.c);
    m->ops.push_back(o);
    return o.y;
  }
  int maxpool(int x, int k, int stride, int pad) {
    const TensorDesc tx = m->tensors[x];
    Op o;
    o.kind = OP_MAXPOOL; o.x = x; o.k = k; o.stride = stride; o.pad = pad;
    o.y = add_tensor((tx.h + 2 * pad - k) / stride + 1, (tx.w + 2 * pad - k) / stride + 1, tx.c);
    m->ops.push_back(o);
    return o.y;
  }
  int slice(int x, int c0, int n) {
    const TensorDesc tx = m->tensors[x];
    Op o;
    o.kind = OP_SLICE; o.x = x; o.a0 = c0;
    o.y = add_tensor(tx.h, tx.w, n);
    m->ops.push_back(o);
    m->first_trainable_op = (int)m->ops.size();
    return o.y;
  }
  int gap(int x) {
    const TensorDesc tx = m->tensors[x];
    Op o;
    o.kind = OP_GAP; o.x = x;
    o.y = add_tensor(1, 1, tx.c);
    m->ops.push_back(o);
    return o.y;
  }
  int ln(int x, int res, int pg, int pb) {
    const TensorDesc tx = m->tensors[x];
    Op o;
    o.kind = OP_LN; o.x = x; o.res = res; o.pw = pg; o.pb = pb;
    o.y = add_tensor(tx.h, tx.w, tx.c);
    m->ops.push_back(o);
    return o.y;
  }
  int linear(int x, const std::string& n, int fin, int fout, bool bias = true) {
    int64_t sh[2] = {fout, fin};
    const TensorDesc tx = m->tensors[x];
    Op o;
    o.kind = OP_LINEAR; o.x = x;
    o.pw = add_param(n + ".w", CD_P_LINEAR_W, 2, sh, fin);
    o.pb = bias ? vec(n + ".b", CD_P_BIAS, fout) : -1;
    o.y = add_tensor(tx.h, tx.w, fout, true);   // one row of logits per row of x
    m->ops.push_back(o);
    return o.y;
  }
  // logits against an existing [fout][fin] table (the embedding), no bias
  int tied_linear(int x, int pw, int fout) {
    const TensorDesc tx = m->tensors[x];
    Op o;
    o.kind = OP_LINEAR; o.x = x; o.pw = pw; o.pb = -1; o.tied = true;
    o.y = add_tensor(tx.h, tx.w, fout, true);
    m->ops.push_back(o);
    return o.y;
  }
  int embed(int pw, int col0, int len, int d) {
    Op o;
    o.kind = OP_EMBED; o.x = 0; o.pw = pw; o.a0 = col0; o.a1 = len;
    o.y = add_tensor(len, 1, d);
    m->ops.push_back(o);
    return o.y;
  }
  int attention(int q, int q_col, int kv, int k_col, int v_col, int d, int heads, bool causal, int key_tok0, int q_stream,
                int k_stream) {
    const TensorDesc tq = m->tensors[q];
    Op o;
    o.kind = OP_ATTN; o.x = q; o.res = kv; o.a0 = q_col; o.a1 = k_col; o.a2 = v_col; o.heads = heads; o.causal = causal;
    o.key_tok0 = key_tok0; o.q_stream = q_stream; o.k_stream = k_stream;
    o.y = add_tensor(tq.h, tq.w, d);
    m->ops.push_back(o);
    return o.y;
  }
};

void build_tiny(Builder& b, const cd_arch_desc& a) {
  const int c1 = a.widths[0], c2 = a.widths[1];
  int w1 = b.conv_w("conv1", 3, c1, 3), b1 = b.vec("conv1.b", CD_P_BIAS, c1);
  int t = b.conv(0, w1, b1, c1, 3, 1, 1, true);
  int w2 = b.conv_w("conv2", c1, c2, 3), b2 = b.vec("conv2.b", CD_P_BIAS, c2);
  t = b.conv(t, w2, b2, c2, 3, 1, 1, true);
  t = b.gap(t);
  b.linear(t, "fc", c2, a.classes);
}

// h + W2 relu(W1 h + b1) + b2 -> LayerNorm -> projection; the dense layers are 1x1 convolutions over
// the [rows][1][1][d] tensor
void build_transformer_head(Builder& b, const cd_arch_desc& a) {
  const int d = a.widths[0], ff = a.widths[1];
  int w1 = b.conv_w("ffn.w1", d, ff, 1), b1 = b.vec("ffn.w1.b", CD_P_BIAS, ff);
  int t = b.conv(0, w1, b1, ff, 1, 1, 0, true);
  int w2 = b.conv_w("ffn.w2", ff, d, 1), b2 = b.vec("ffn.w2.b", CD_P_BIAS, d);
  t = b.conv(t, w2, b2, d, 1, 1, 0, false);
  int g = b.vec("ffn.ln.gamma", CD_P_BN_GAMMA, d), be = b.vec("ffn.ln.beta", CD_P_BN_BETA, d);
  t = b.ln(t, 0, g, be);
  b.linear(t, "proj", d, a.classes, false);
}

// Encoder-decoder Transformer (paper, Section 4; Vaswani et al.): token embedding times sqrt(d) plus
// the sinusoidal position signal; encoder layers of self-attention and feed-forward sublayers, decoder
// layers of causal self-attention, attention over the encoder output and feed-forward, every sublayer
// followed by its residual connection and LayerNorm; logits against the (tied) embedding table.  The
// input projections of an attention sublayer are one dense layer (d -> 3d, or d -> d for the queries and
// d -> 2d for keys and values of the encoder output); dense layers are 1x1 convolutions over
// [sentences][tokens][1][d] tensors ([1][rows of the stream][1][d] for packed sentences).  No dropout.
void build_transformer(Builder& b, const cd_arch_desc& a) {
  const int d = a.widths[0], ff = a.widths[1], heads = a.widths[2];
  const int Ts = a.in_h, Tt = a.in_w;
  auto dense = [&](int x, const std::string& n, int fin, int fout, bool relu) {
    int w = b.conv_w(n, fin, fout, 1), bi = b.vec(n + ".b", CD_P_BIAS, fout);
    return b.conv(x, w, bi, fout, 1, 1, 0, relu);
  };
  auto add_norm = [&](int x, int sub, const std::string& n) {
    int g = b.vec(n + ".gamma", CD_P_BN_GAMMA, d), be = b.vec(n + ".beta", CD_P_BN_BETA, d);
    return b.ln(sub, x, g, be);
  };
  auto ffn = [&](int x, const std::string& p) {
    int u = dense(x, p + ".ffn.w1", d, ff, true);
    u = dense(u, p + ".ffn.w2", ff, d, false);
    return add_norm(x, u, p + ".ffn.ln");
  };
  auto self_attention = [&](int x, const std::string& p, bool causal) {
    int qkv = dense(x, p + ".qkv", d, 3 * d, false);
    int o = b.attention(qkv, 0, qkv, d, 2 * d, d, heads, causal, causal ? Ts : 0, causal, causal);   // decoder keys: target sentences
    return add_norm(x, dense(o, p + ".out", d, d, false), p + ".ln");
  };
  int64_t sh[2] = {a.classes, d};
  const int table = b.add_param("embed.w", CD_P_EMBED_W, 2, sh, d);
  char name[32];
  int x = b.embed(table, 0, Ts, d);
  for (int i = 0; i < a.blocks[0]; i++) {
    snprintf(name, sizeof(name), "enc%d", i);
    x = ffn(self_attention(x, std::string(name) + ".self", false), name);
  }
  const int memory = x;
  int y = b.embed(table, Ts, Tt, d);
  for (int i = 0; i < a.blocks[1]; i++) {
    snprintf(name, sizeof(name), "dec%d", i);
    const std::string p(name);
    y = self_attention(y, p + ".self", true);
    int q = dense(y, p + ".cross.q", d, d, false);
    int kv = dense(memory, p + ".cross.kv", d, 2 * d, false);
    int o = b.attention(q, 0, kv, 0, d, d, heads, false, 0, 1, 0);
    y = add_norm(y, dense(o, p + ".cross.out", d, d, false), p + ".cross.ln");
    y = ffn(y, p);
  }
  b.tied_linear(y, table, a.classes);
}

struct BnP { int g, b; };
BnP bn_params(Builder& b, const std::string& n, int c) {
  BnP p;
  p.g = b.vec(n + ".gamma", CD_P_BN_GAMMA, c);
  p.b = b.vec(n + ".beta", CD_P_BN_BETA, c);
  return p;
}

void build_resnet(Builder& b, const cd_arch_desc& a) {
  const bool next = a.kind == CD_ARCH_RESNEXT;   // bottleneck blocks with a grouped 3x3 and their own output widths
  const bool bott = a.kind == CD_ARCH_RESNET_BOTTLENECK || next;
  const bool big_stem = bott || a.kind == CD_ARCH_RESNET_BASIC_IMAGENET;   // 7x7 stride 2 + max-pool
  const int groups = next ? a.groups : 1;
  char name[64];
  int t, cin = a.stem_width;
  {
    int w = b.conv_w("stem.conv", 3, a.stem_width, big_stem ? 7 : 3);
    BnP p = bn_params(b, "stem.bn", a.stem_width);
    t = big_stem ? b.conv(0, w, -1, a.stem_width, 7, 2, 3, false) : b.conv(0, w, -1, a.stem_width, 3, 1, 1, false);
    t = b.bn(t, p.g, p.b, -1, true);
    if (big_stem) t = b.maxpool(t, 3, 2, 1);
  }
  for (int si = 0; si < a.n_stages; si++) {
    const int wd = a.widths[si];
    const int cout = next ? a.out_widths[si] : (bott ? 4 * wd : wd);
    for (int bi = 0; bi < a.blocks[si]; bi++) {
      const int stride = (si > 0 && bi == 0) ? 2 : 1;
      snprintf(name, sizeof(name), "s%d.b%d", si + 1, bi);
      const std::string p(name);
      const bool proj = bott ? (bi == 0) : (stride != 1 || cin != wd);
      // parameters in declaration order: the main path first, then the projection shortcut
      int w1, w2, w3 = -1, wdn = -1;
      BnP p1, p2, p3 = {-1, -1}, pdn = {-1, -1};
      if (bott) {
        w1 = b.conv_w(p + ".conv1", cin, wd, 1); p1 = bn_params(b, p + ".bn1", wd);
        w2 = b.conv_w(p + ".conv2", wd / groups, wd, 3);  p2 = bn_params(b, p + ".bn2", wd);
        w3 = b.conv_w(p + ".conv3", wd, cout, 1); p3 = bn_params(b, p + ".bn3", cout);
      } else {
        w1 = b.conv_w(p + ".conv1", cin, wd, 3); p1 = bn_params(b, p + ".bn1", wd);
        w2 = b.conv_w(p + ".conv2", wd, wd, 3);  p2 = bn_params(b, p + ".bn2", wd);
      }
      if (proj) { wdn = b.conv_w(p + ".down.conv", cin, cout, 1); pdn = bn_params(b, p + ".down.bn", cout); }
      // ops: shortcut branch before the BatchNorm that adds it
      int sc = t;
      if (proj) {
        sc = b.conv(t, wdn, -1, cout, 1, stride, 0, false);
        sc = b.bn(sc, pdn.g, pdn.b, -1, false);
      }
      int u;
      if (bott) {
        u = b.conv(t, w1, -1, wd, 1, 1, 0, false);
        u = b.bn(u, p1.g, p1.b, -1, true);
        u = b.conv(u, w2, -1, wd, 3, stride, 1, false, groups);
        u = b.bn(u, p2.g, p2.b, -1, true);
        u = b.conv(u, w3, -1, cout, 1, 1, 0, false);
        t = b.bn(u, p3.g, p3.b, sc, true);
      } else {
        u = b.conv(t, w1, -1, wd, 3, stride, 1, false);
        u = b.bn(u, p1.g, p1.b, -1, true);
        u = b.conv(u, w2, -1, wd, 3, 1, 1, false);
        t = b.bn(u, p2.g, p2.b, sc, true);
      }
      cin = cout;
      if (a.kind == CD_ARCH_WIDE_RESNET_SPLIT && si == 0 && bi == 0) {
        // the frozen front end ends here: the rest of the network receives one part of its output channels
        cin = cout / a.n_splits;
        t = b.slice(t, a.split * cin, cin);
      }
    }
  }
  t = b.gap(t);
  b.linear(t, "fc", cin, a.classes);
}

// CODISTILL_FORCE_SIMPLE=1 routes every convolution to the plain kernels (debugging aid)
bool force_simple() {
  const char* e = getenv("CODISTILL_FORCE_SIMPLE");
  return e && e[0] == '1';
}

// CODISTILL_NO_POOL_FUSION=1 keeps a BatchNorm and the max-pool behind it in separate kernels (debugging aid)
bool force_separate_pool() {
  const char* e = getenv("CODISTILL_NO_POOL_FUSION");
  return e && e[0] == '1';
}

// CODISTILL_WRITE_RESIDUAL_GRADS=1 makes every BatchNorm write the gradient of its residual input
// (debugging aid; see residual_grad_route)
bool force_residual_grads() {
  const char* e = getenv("CODISTILL_WRITE_RESIDUAL_GRADS");
  return e && e[0] == '1';
}

// CODISTILL_SEPARATE_RELU_MASK=1 keeps the backward pass of a convolution's fused ReLU in a kernel of its own
// instead of the epilogue of the data-gradient kernel that writes the masked tensor (debugging aid)
bool fuse_off() {
  const char* e = getenv("CODISTILL_SEPARATE_RELU_MASK");
  return e && e[0] == '1';
}

// CODISTILL_SEPARATE_BN_REDUCTION=1 keeps the reduction pass of every BatchNorm's backward pass (debugging aid): without
// it, the data-gradient kernel that completes the gradient of a BatchNorm's output also takes that BatchNorm's column
// sums (dz and dz * xhat) from the values it stores
bool separate_bn_reduction() {
  const char* e = getenv("CODISTILL_SEPARATE_BN_REDUCTION");
  return e && e[0] == '1';
}

// CODISTILL_SERIAL=1 keeps every launch of a call on the caller's stream (debugging aid)
bool force_serial() {
  const char* e = getenv("CODISTILL_SERIAL");
  return e && e[0] == '1';
}

ConvGeom conv_geom(const cd_model* m, const Op& o, int64_t B) {
  const TensorDesc& tx = m->tensors[o.x];
  const TensorDesc& ty = m->tensors[o.y];
  ConvGeom g;
  g.B = B; g.H = tx.h; g.W = tx.w; g.Cin = tx.c; g.Ho = ty.h; g.Wo = ty.w; g.Cout = ty.c;
  g.kh = o.k; g.kw = o.k; g.stride = o.stride; g.pad = o.pad;
  return g;
}

// The geometry the MFMA kernels see for a convolution on 3-channel images: stride 2 on even image
// sizes runs in space-to-depth form (16 channels, stride 1, about half the taps per axis), anything
// else with the channels zero-padded to 8.
bool s2d_form(const ConvGeom& g) { return g.Cin == 3 && g.stride == 2 && g.H % 2 == 0 && g.W % 2 == 0 && g.kh == g.kw; }
ConvGeom packed_geom(const ConvGeom& g) {
  ConvGeom p = g;
  if (s2d_form(g)) {
    const int P = (g.pad + 1) / 2, shift = 2 * P - g.pad;
    p.H = g.H / 2; p.W = g.W / 2; p.Cin = 16;
    p.kh = p.kw = (g.kh + shift + 1) / 2;
    p.stride = 1; p.pad = P;
  } else if (g.Cin == 3) {
    p.Cin = 8;
  }
  return p;
}
// bf16 convolutions run on the MFMA kernels
bool use_mfma(const cd_model* m, const ConvGeom& g) {
  if (m->dtype != CD_BF16 || force_simple()) return false;
  return conv_mfma_supported(packed_geom(g));
}

// Whether a grouped convolution runs as sliced launches on the row-major tensors (conv_grouped_*_mfma): bf16, slices of
// whole groups, 32-bit offsets; otherwise as dense convolutions on slice-major copies (conv_grouped.hip).
bool grouped_sliced(const cd_model* m, const Op& o, int64_t batch) {
  if (m->dtype != CD_BF16 || force_simple() || o.kind != OP_CONV || o.groups <= 1) return false;
  const TensorDesc& tx = m->tensors[o.x];
  const TensorDesc& ty = m->tensors[o.y];
  if (tx.c != ty.c || grouped_mfma_slice(tx.c, o.groups) == 0) return false;
  return batch * tx.per_sample() * 2 < (1LL << 31) && batch * ty.per_sample() * 2 < (1LL << 31);
}

// How the backward pass of BatchNorm op i hands the gradient of its residual input on (that gradient
// is the op's own dy, gated by its ReLU).  Where the branch's next reader can take "dy and the ReLU
// bit mask" in place of a tensor, the gradient is never written out:
//  1: the residual is the output of a ReLU-free BatchNorm used nowhere else (a projection shortcut):
//     that layer's backward pass reads dy through the mask;
//  2: the residual is read by exactly one other op, a stride-1 convolution on the MFMA kernels that
//     comes earlier in the graph (the block input of an identity block): that convolution's data
//     gradient adds the gated dy in its epilogue;
//  0: it is added to the residual tensor's gradient buffer.
// Whether BatchNorm op i (with ReLU) and the 3x3 stride-2 max-pool that follows it run as one kernel
// (bn_relu_pool): the pool is the only reader of the normalised tensor, which is then never written.
bool pool_fused(const cd_model* m, int i) {
  if (i < 0 || i + 1 >= (int)m->ops.size() || m->dtype != CD_BF16 || force_simple() || force_separate_pool()) return false;
  const Op& o = m->ops[i];
  const Op& q = m->ops[i + 1];
  if (o.kind != OP_BN || !o.relu || o.res >= 0 || q.kind != OP_MAXPOOL || q.x != o.y) return false;
  if (q.k != 3 || q.stride != 2 || q.pad != 1) return false;
  const TensorDesc& t = m->tensors[o.y];
  if (t.h % 2 || t.w % 2 || t.c % 8) return false;
  for (int j = 0; j < (int)m->ops.size(); j++)
    if (j != i + 1 && (m->ops[j].x == o.y || m->ops[j].res == o.y)) return false;
  return true;
}

int residual_grad_route(const cd_model* m, int i, int64_t batch) {
  const Op& o = m->ops[i];
  const int r = o.res;
  if (o.kind != OP_BN || r <= 0 || m->dtype != CD_BF16 || force_simple() || force_residual_grads() ||
      m->tensors[r].c % 8 != 0)
    return 0;
  int others = 0, conv = -1, producer = -1;
  for (int j = 0; j < (int)m->ops.size(); j++) {
    const Op& q = m->ops[j];
    if (q.y == r) producer = j;
    if (j == i) continue;
    if (q.x == r || q.res == r) { others++; if (q.kind == OP_CONV && q.x == r && j < i) conv = j; }
  }
  if (others == 0 && producer >= 0) {
    const Op& q = m->ops[producer];
    if (q.kind == OP_BN && !q.relu && q.res < 0) return 1;
  }
  if (others == 1 && conv >= 0) {
    const Op& q = m->ops[conv];
    if (q.stride == 1 && use_mfma(m, conv_geom(m, q, batch))) return 2;
  }
  return 0;
}

}  // namespace

namespace cd {

Plan make_plan(const cd_model* m, int64_t B, bool save) {
  Plan p;
  p.batch = B;
  p.save = save;
  size_t off = 0;
  auto alloc = [&](size_t bytes) { size_t o = off; off += align_up(bytes ? bytes : 16, 256); return o; };
  const int nt = (int)m->tensors.size();
  p.act.assign(nt, 0);
  p.grad.assign(nt, 0);
  for (int t = 1; t < nt; t++)
    if (!m->tensors[t].f32) p.act[t] = alloc((size_t)B * m->tensors[t].per_sample() * m->esize());
  p.bn_stats = alloc((size_t)(m->bn_c_total > 0 ? m->bn_c_total : 1) * 4 * sizeof(float));
  p.bn_coef = alloc((size_t)3 * m->max_c * sizeof(float));
  p.partials_bytes = kPartialsBytes;
  p.partials = alloc(p.partials_bytes);
  if (m->dtype == CD_BF16) {
    if (m->arch.kind != CD_ARCH_TRANSFORMER) p.xpack = alloc((size_t)B * m->arch.in_h * m->arch.in_w * 8 * 2);
    if (m->arch.kind == CD_ARCH_TRANSFORMER && m->arch.max_sentences > 0)
      p.seq_tab = alloc((size_t)2 * (m->arch.max_sentences + 2) * sizeof(int32_t));
    size_t wmax = 0;
    for (const ParamDesc& q : m->params) {
      if (q.kind == CD_P_CONV_W) {
        size_t e = (size_t)q.shape[0] * q.shape[1] * q.shape[2] * (q.shape[3] == 3 ? 8 : q.shape[3]);
        if (e > wmax) wmax = e;
      }
      if ((q.kind == CD_P_LINEAR_W || q.kind == CD_P_EMBED_W) && (size_t)q.size > wmax) wmax = (size_t)q.size;
    }
    for (const Op& o : m->ops)   // the dense per-slice filter of a grouped convolution, re-laid-out for its data gradient
      if (o.kind == OP_CONV && o.groups > 1) {
        const size_t sw = (size_t)grouped_slice_width(m->tensors[o.x].c);
        if (sw * o.k * o.k * sw > wmax) wmax = sw * o.k * o.k * sw;
      }
    p.wpack_bytes = align_up(wmax * 4 + 256, 256);  // also holds the fp32 padded stem weight gradient
    p.wpack = alloc(p.wpack_bytes);
    p.lin_dz = alloc((size_t)B * m->tensors[m->ops.back().y].per_sample() * 2);
  }
  p.aux.assign(m->ops.size(), 0);
  p.gx.assign(m->ops.size(), 0);
  {
    size_t tmax = 0, wdmax = 0;
    for (size_t i = 0; i < m->ops.size(); i++) {
      const Op& o = m->ops[i];
      if (o.kind != OP_CONV || o.groups <= 1) continue;
      const size_t in_b = (size_t)B * m->tensors[o.x].per_sample() * 2, out_b = (size_t)B * m->tensors[o.y].per_sample() * 2;
      const size_t wd = (size_t)m->tensors[o.x].c * o.k * o.k * grouped_slice_width(m->tensors[o.x].c) + 64;
      if (wd > wdmax) wdmax = wd;
      if (grouped_sliced(m, o, B)) continue;   // reads and writes the row-major tensors in place: no copies
      if (in_b > tmax) tmax = in_b;
      if (out_b > tmax) tmax = out_b;
      if (save) p.gx[i] = alloc(in_b);
    }
    if (tmax) {
      p.gtmp_bytes = align_up(tmax, 256);
      p.gtmp = alloc(2 * p.gtmp_bytes);
    }
    if (wdmax) {
      p.gw = alloc(wdmax * 2);
      if (save) p.gdw = alloc(wdmax * 4);
    }
  }
  p.wt_op.assign(m->ops.size(), 0);
  if (save && m->dtype == CD_BF16) {
    for (size_t i = (size_t)m->first_trainable_op; i < m->ops.size(); i++) {
      const Op& o = m->ops[i];
      if (o.kind != OP_CONV || o.groups > 1 || o.x == 0) continue;
      const ConvGeom g = conv_geom(m, o, B);
      if (use_mfma(m, g)) p.wt_op[i] = alloc((size_t)(conv_dgrad_layout_elems(g) + 32) * 2);
    }
  }
  if (save) {
    p.partials_side = alloc(p.partials_bytes);
    for (int t = 1; t < nt; t++)
      if (!m->tensors[t].f32) p.grad[t] = alloc((size_t)B * m->tensors[t].per_sample() * m->esize());
    for (size_t i = 0; i < m->ops.size(); i++) {
      const Op& o = m->ops[i];
      if (o.kind == OP_MAXPOOL) p.aux[i] = alloc((size_t)B * m->tensors[o.y].per_sample());
      // sign bits of a fused ReLU's output, one per element (bf16 vector path only)
      if (o.kind == OP_BN && o.relu && m->dtype == CD_BF16 && m->tensors[o.y].c % 8 == 0)
        p.aux[i] = alloc((size_t)B * m->tensors[o.y].per_sample() / 8);
      if (o.kind == OP_LN) p.aux[i] = alloc((size_t)B * m->tensors[o.y].h * m->tensors[o.y].w * 2 * sizeof(float));
      if (o.kind == OP_ATTN) p.aux[i] = alloc((size_t)B * o.heads * m->tensors[o.y].h * 2 * sizeof(float));
    }
  }
  p.total = off;
  return p;
}

}  // namespace cd

// ------------------------------------------------------------------------------------- C ABI
extern "C" int codistill_arch_preset(int kind, cd_arch_desc* out) {
  CD_REQUIRE(out != nullptr, "arch_preset: out is NULL");
  memset(out, 0, sizeof(*out));
  out->kind = kind;
  if (kind == CD_ARCH_TINY_CNN) {
    out->classes = 10; out->in_h = out->in_w = 32; out->n_stages = 0;
    out->widths[0] = 16; out->widths[1] = 32;
  } else if (kind == CD_ARCH_RESNET_BASIC) {
    out->classes = 10; out->in_h = out->in_w = 32; out->n_stages = 3; out->stem_width = 16;
    const int w[3] = {16, 32, 64};
    for (int i = 0; i < 3; i++) { out->widths[i] = w[i]; out->blocks[i] = 3; }
  } else if (kind == CD_ARCH_RESNET_BOTTLENECK) {
    out->classes = 1000; out->in_h = out->in_w = 224; out->n_stages = 4; out->stem_width = 64;
    const int w[4] = {64, 128, 256, 512}, nb[4] = {3, 4, 6, 3};
    for (int i = 0; i < 4; i++) { out->widths[i] = w[i]; out->blocks[i] = nb[i]; }
  } else if (kind == CD_ARCH_RESNEXT) {
    out->classes = 1000; out->in_h = out->in_w = 224; out->n_stages = 4; out->stem_width = 64; out->groups = 32;
    const int w[4] = {256, 512, 1024, 2048}, nb[4] = {3, 4, 23, 3};
    for (int i = 0; i < 4; i++) { out->widths[i] = w[i]; out->out_widths[i] = w[i]; out->blocks[i] = nb[i]; }
  } else if (kind == CD_ARCH_RESNET_BASIC_IMAGENET) {
    out->classes = 1000; out->in_h = out->in_w = 224; out->n_stages = 4; out->stem_width = 64;
    const int w[4] = {64, 128, 256, 512};
    for (int i = 0; i < 4; i++) { out->widths[i] = w[i]; out->blocks[i] = 2; }
  } else if (kind == CD_ARCH_WIDE_RESNET_SPLIT) {
    out->classes = 10; out->in_h = out->in_w = 32; out->n_stages = 3; out->stem_width = 16; out->n_splits = 8; out->split = 0;
    const int w[3] = {160, 320, 640};
    for (int i = 0; i < 3; i++) { out->widths[i] = w[i]; out->blocks[i] = 4; }
  } else if (kind == CD_ARCH_TRANSFORMER_HEAD) {
    out->classes = 32768; out->in_h = out->in_w = 1; out->n_stages = 0;
    out->widths[0] = 512; out->widths[1] = 2048;
  } else if (kind == CD_ARCH_TRANSFORMER) {
    out->classes = 32768; out->in_h = out->in_w = 128; out->n_stages = 0;
    out->widths[0] = 512; out->widths[1] = 2048; out->widths[2] = 8;
    out->blocks[0] = out->blocks[1] = 6;
  } else {
    return set_error(CD_ERR_INVALID_ARG, "arch_preset: unknown kind %d", kind);
  }
  return CD_OK;
}

extern "C" int codistill_model_create(const cd_arch_desc* a, int dtype, cd_model** out) {
  CD_REQUIRE(a != nullptr && out != nullptr, "model_create: NULL pointer argument");
  CD_REQUIRE(dtype == CD_F32 || dtype == CD_BF16, "model_create: unknown dtype %d", dtype);
  CD_REQUIRE(a->kind == CD_ARCH_TINY_CNN || a->kind == CD_ARCH_RESNET_BASIC || a->kind == CD_ARCH_RESNET_BOTTLENECK ||
                 a->kind == CD_ARCH_RESNET_BASIC_IMAGENET || a->kind == CD_ARCH_RESNEXT ||
                 a->kind == CD_ARCH_TRANSFORMER_HEAD || a->kind == CD_ARCH_TRANSFORMER || a->kind == CD_ARCH_WIDE_RESNET_SPLIT,
             "model_create: unknown architecture kind %d", a->kind);
  CD_REQUIRE(a->classes >= 1 && a->classes <= (1 << 24), "model_create: classes=%d out of range", a->classes);
  const bool packed = a->kind == CD_ARCH_TRANSFORMER && a->max_sentences != 0;
  const int res_max = packed ? 65536 : 4096;
  CD_REQUIRE(a->in_h >= 1 && a->in_w >= 1 && a->in_h <= res_max && a->in_w <= res_max,
             "model_create: input resolution %dx%d out of range", a->in_h, a->in_w);
  CD_REQUIRE(a->kind == CD_ARCH_TRANSFORMER || (a->max_sentences == 0 && a->max_sentence_len == 0),
             "model_create: max_sentences / max_sentence_len belong to CD_ARCH_TRANSFORMER");
  if (a->kind == CD_ARCH_TINY_CNN) {
    CD_REQUIRE(a->widths[0] >= 1 && a->widths[1] >= 1 && a->widths[0] <= 4096 && a->widths[1] <= 4096,
               "model_create: tiny CNN widths out of range");
  } else if (a->kind == CD_ARCH_TRANSFORMER) {
    const int d = a->widths[0], heads = a->widths[2];
    CD_REQUIRE(d >= 8 && d <= 16384 && a->widths[1] >= 8 && a->widths[1] <= 65536 && d % 8 == 0 && a->widths[1] % 8 == 0,
               "model_create: d_model / d_ff out of range or not a multiple of 8");
    CD_REQUIRE(heads >= 1 && d % heads == 0 && attention_supported(d / heads),
               "model_create: d_model / heads must be 8, 16, 32 or 64");
    CD_REQUIRE(a->blocks[0] >= 1 && a->blocks[0] <= 64 && a->blocks[1] >= 1 && a->blocks[1] <= 64,
               "model_create: encoder / decoder layer counts out of range");
    if (packed)
      CD_REQUIRE(a->max_sentences >= 1 && a->max_sentences <= 65536 && a->max_sentence_len >= 1 && a->max_sentence_len <= 65536,
                 "model_create: packed sentences need 1 <= max_sentences, max_sentence_len <= 65536 (got %d, %d)",
                 a->max_sentences, a->max_sentence_len);
    else
      CD_REQUIRE(a->max_sentence_len == 0, "model_create: max_sentence_len without max_sentences");
    if (dtype != CD_BF16) return set_error(CD_ERR_UNSUPPORTED, "model_create: the Transformer is implemented for CD_BF16 only");
  } else if (a->kind == CD_ARCH_TRANSFORMER_HEAD) {
    CD_REQUIRE(a->widths[0] >= 1 && a->widths[1] >= 1 && a->widths[0] <= 16384 && a->widths[1] <= 65536,
               "model_create: d_model / d_ff out of range");
    CD_REQUIRE(a->in_h == 1 && a->in_w == 1, "model_create: the Transformer head takes [rows][1][1][d_model] inputs");
  } else {
    CD_REQUIRE(a->n_stages >= 1 && a->n_stages <= CD_MAX_STAGES, "model_create: n_stages=%d out of range", a->n_stages);
    CD_REQUIRE(a->stem_width >= 1 && a->stem_width <= 4096, "model_create: stem_width=%d out of range", a->stem_width);
    for (int i = 0; i < a->n_stages; i++)
      CD_REQUIRE(a->widths[i] >= 1 && a->widths[i] <= 4096 && a->blocks[i] >= 1 && a->blocks[i] <= 64,
                 "model_create: stage %d width/blocks out of range", i);
    if (a->kind == CD_ARCH_WIDE_RESNET_SPLIT) {
      CD_REQUIRE(a->n_splits >= 1 && a->widths[0] % a->n_splits == 0 && a->split >= 0 && a->split < a->n_splits,
                 "model_create: n_splits=%d must divide widths[0]=%d, and 0 <= split=%d < n_splits", a->n_splits, a->widths[0],
                 a->split);
      CD_REQUIRE(a->blocks[0] >= 2, "model_create: the first stage needs a block behind the frozen one");
    }
    if (a->kind == CD_ARCH_RESNEXT) {
      if (dtype != CD_BF16) return set_error(CD_ERR_UNSUPPORTED, "model_create: grouped convolutions are implemented for CD_BF16 only");
      for (int i = 0; i < a->n_stages; i++) {
        CD_REQUIRE(a->out_widths[i] >= 1 && a->out_widths[i] <= 16384, "model_create: stage %d output width out of range", i);
        if (!grouped_conv_supported(a->widths[i], a->groups))
          return set_error(CD_ERR_UNSUPPORTED,
                           "model_create: stage %d: %d channels in %d groups (need a multiple of 8 channels, of 128 above "
                           "128, and whole groups per 128 channels)", i, a->widths[i], a->groups);
      }
    }
  }
  cd_model* m = new cd_model();
  m->arch = *a;
  m->dtype = dtype;
  m->tensors.push_back(TensorDesc());
  m->tensors[0].h = a->in_h; m->tensors[0].w = a->in_w;
  m->tensors[0].c = a->kind == CD_ARCH_TRANSFORMER_HEAD ? a->widths[0] : 3;
  if (a->kind == CD_ARCH_TRANSFORMER) {   // tensor 0: int32 token ids, per sentence in_h source tokens then in_w target tokens
    m->tensors[0].h = 1; m->tensors[0].w = a->in_h + a->in_w; m->tensors[0].c = 1;
  }
  Builder b{m};
  if (a->kind == CD_ARCH_TINY_CNN) build_tiny(b, *a);
  else if (a->kind == CD_ARCH_TRANSFORMER_HEAD) build_transformer_head(b, *a);
  else if (a->kind == CD_ARCH_TRANSFORMER) build_transformer(b, *a);
  else build_resnet(b, *a);
  for (const TensorDesc& t : m->tensors) {
    if (t.h < 1 || t.w < 1) {
      delete m;
      return set_error(CD_ERR_INVALID_ARG, "model_create: input resolution too small for this architecture");
    }
    if (t.c > m->max_c) m->max_c = t.c;
  }
  *out = m;
  return CD_OK;
}

extern "C" void codistill_model_destroy(cd_model* m) { delete m; }

extern "C" int codistill_bn_running_elements(const cd_model* m, int64_t* n) {
  CD_REQUIRE(m != nullptr && n != nullptr, "bn_running_elements: NULL pointer argument");
  *n = 2 * m->bn_c_total;
  return CD_OK;
}

extern "C" int codistill_param_count(const cd_model* m, int64_t* n_tensors, int64_t* n_elements) {
  CD_REQUIRE(m != nullptr, "param_count: model is NULL");
  if (n_tensors) *n_tensors = (int64_t)m->params.size();
  if (n_elements) *n_elements = m->n_elements;
  return CD_OK;
}

extern "C" int codistill_param_info(const cd_model* m, int64_t idx, cd_tensor_info* out) {
  CD_REQUIRE(m != nullptr && out != nullptr, "param_info: NULL pointer argument");
  CD_REQUIRE(idx >= 0 && idx < (int64_t)m->params.size(), "param_info: index %lld out of range", (long long)idx);
  const ParamDesc& p = m->params[idx];
  memset(out, 0, sizeof(*out));
  snprintf(out->name, CD_NAME_LEN, "%s", p.name.c_str());
  out->kind = p.kind; out->ndim = p.ndim;
  for (int i = 0; i < 4; i++) out->shape[i] = p.shape[i];
  out->offset = p.offset; out->size = p.size; out->fan_in = p.fan_in;
  for (int i = 0; i < m->first_trainable_op; i++)
    if (m->ops[i].pw == idx || m->ops[i].pb == idx) out->frozen = 1;
  return CD_OK;
}

extern "C" int codistill_workspace_bytes(const cd_model* m, int64_t batch, int save, size_t* bytes) {
  CD_REQUIRE(m != nullptr && bytes != nullptr, "workspace_bytes: NULL pointer argument");
  CD_REQUIRE(batch >= 1 && batch <= (1 << 20), "workspace_bytes: batch=%lld out of range", (long long)batch);
  *bytes = make_plan(m, batch, save != 0).total;
  return CD_OK;
}

extern "C" int codistill_graph_size(const cd_model* m, int64_t* n_ops, int64_t* n_tensors) {
  CD_REQUIRE(m != nullptr, "graph_size: model is NULL");
  if (n_ops) *n_ops = (int64_t)m->ops.size();
  if (n_tensors) *n_tensors = (int64_t)m->tensors.size();
  return CD_OK;
}

extern "C" int codistill_op_info(const cd_model* m, int64_t batch, int64_t idx, cd_op_info* out) {
  CD_REQUIRE(m != nullptr && out != nullptr, "op_info: NULL pointer argument");
  CD_REQUIRE(idx >= 0 && idx < (int64_t)m->ops.size(), "op_info: index %lld out of range", (long long)idx);
  CD_REQUIRE(batch >= 1 && batch <= (1 << 20), "op_info: batch=%lld out of range", (long long)batch);
  const Op& o = m->ops[idx];
  out->kind = (int32_t)o.kind; out->x = o.x; out->y = o.y; out->res = o.res; out->relu = o.relu ? 1 : 0;
  out->param_w = o.pw; out->param_b = o.pb; out->k = o.k; out->stride = o.stride; out->pad = o.pad;
  out->stats_offset = -1;
  if (o.kind == OP_BN) {
    Plan p = make_plan(m, batch, true);
    out->stats_offset = (int64_t)(p.bn_stats + (size_t)4 * m->bn_off[o.bn_slot] * sizeof(float));
  }
  if (o.kind == OP_LN) out->stats_offset = (int64_t)make_plan(m, batch, true).aux[idx];
  out->k_col = out->v_col = 0;
  if (o.kind == OP_EMBED) { out->k = o.a0; out->stride = o.a1; }
  if (o.kind == OP_SLICE) out->k = o.a0;
  if (o.kind == OP_ATTN) {
    out->k = o.heads; out->stride = o.causal ? 1 : 0; out->pad = o.a0; out->k_col = o.a1; out->v_col = o.a2;
    out->key_tok0 = o.key_tok0;
  }
  out->res_grad = residual_grad_route(m, (int)idx, batch);
  out->fused_pool = pool_fused(m, (int)idx) ? 1 : 0;
  return CD_OK;
}

extern "C" int codistill_tensor_info(const cd_model* m, int64_t batch, int64_t idx, cd_act_info* out) {
  CD_REQUIRE(m != nullptr && out != nullptr, "tensor_info: NULL pointer argument");
  CD_REQUIRE(idx >= 0 && idx < (int64_t)m->tensors.size(), "tensor_info: index %lld out of range", (long long)idx);
  CD_REQUIRE(batch >= 1 && batch <= (1 << 20), "tensor_info: batch=%lld out of range", (long long)batch);
  const TensorDesc& t = m->tensors[idx];
  Plan p = make_plan(m, batch, true);
  out->h = t.h; out->w = t.w; out->c = t.c; out->is_f32 = t.f32 ? 1 : 0;
  const bool in_ws = idx != 0 && !t.f32;
  out->act_offset = in_ws ? (int64_t)p.act[idx] : -1;
  out->grad_offset = in_ws ? (int64_t)p.grad[idx] : -1;
  return CD_OK;
}

// ---------------------------------------------------------------------------------- forward
namespace {

struct Ctx {
  const cd_model* m;
  Plan plan;
  char* ws;
  const char* params;
  const void* x;
  int64_t B;
  hipStream_t s;
  const void* P(int idx) const { return idx < 0 ? nullptr : params + (size_t)m->params[idx].offset * m->esize(); }
  void* act(int t) const { return ws + plan.act[t]; }
  void* grad(int t) const { return ws + plan.grad[t]; }
  float* stats(const Op& o) const { return reinterpret_cast<float*>(ws + plan.bn_stats) + 4 * m->bn_off[o.bn_slot]; }
  float* partials() const { return reinterpret_cast<float*>(ws + plan.partials); }
  float* partials_side() const { return reinterpret_cast<float*>(ws + plan.partials_side); }
  float* coef() const { return reinterpret_cast<float*>(ws + plan.bn_coef); }
  bf16_t* xpack() const { return reinterpret_cast<bf16_t*>(ws + plan.xpack); }
  bf16_t* wpack() const { return reinterpret_cast<bf16_t*>(ws + plan.wpack); }
  // packed Transformer batches: x is [2][rows] (ids, then positions); one sentence table per token stream
  bool packed() const { return m->arch.kind == CD_ARCH_TRANSFORMER && m->arch.max_sentences > 0; }
  const int32_t* positions() const { return packed() ? static_cast<const int32_t*>(x) + m->tensors[0].w : nullptr; }
  int32_t* table(int stream) const { return reinterpret_cast<int32_t*>(ws + plan.seq_tab) + stream * (m->arch.max_sentences + 2); }
  // the tables an attention op reads, and the sentence count / length its launch covers (padded: batch and the tensors' rows)
  SentenceTables tables(const Op& o, int q_rows, int k_rows) const {
    return SentenceTables{table(o.q_stream), table(o.k_stream), m->arch.max_sentences, q_rows, k_rows};
  }
};

int check_common(const char* fn, const cd_model* m, const void* params, const void* x, int64_t batch, void* ws) {
  CD_REQUIRE(m && params && x && ws, "%s: NULL pointer argument", fn);
  CD_REQUIRE(batch >= 1 && batch <= (1 << 20), "%s: batch=%lld out of range", fn, (long long)batch);
  CD_REQUIRE(!(m->arch.kind == CD_ARCH_TRANSFORMER && m->arch.max_sentences > 0) || batch == 1,
             "%s: a packed batch of sentences is one batch element (batch=%lld)", fn, (long long)batch);
  CD_REQUIRE(aligned16(params) && aligned16(x) && (reinterpret_cast<uintptr_t>(ws) & 255) == 0,
             "%s: params and x must be 16-byte aligned, the workspace 256-byte aligned", fn);
  return CD_OK;
}

double conv_bytes(const cd_model* m, const ConvGeom& g) {
  return (double)m->esize() * ((double)g.B * g.H * g.W * g.Cin + (double)g.M() * g.Cout + (double)g.Cout * g.K());
}

}  // namespace

// What the op loops of forward and backward cannot run, found before the first launch (a call that returns an
// error has launched nothing): grouped convolutions outside the kernels' limits, attention inputs with other readers.
static int check_supported(const char* fn, const cd_model* m, const Plan& plan, int64_t batch, bool backward) {
  const int dt = m->dtype;
  for (size_t i = 0; i < m->ops.size(); i++) {
    const Op& o = m->ops[i];
    if (o.kind == OP_CONV && o.groups > 1) {
      const ConvGeom g = conv_geom(m, o, batch);
      if (dt != CD_BF16 || force_simple() || o.pb >= 0 || o.relu || g.Cin != g.Cout || (backward && ((!plan.gx[i] && !grouped_sliced(m, o, batch)) || o.x == 0)))
        return set_error(CD_ERR_UNSUPPORTED, "%s: this grouped convolution has no kernel (bf16, no bias, Cin = Cout, not on the input batch)", fn);
    }
    if (backward && o.kind == OP_ATTN) {
      for (size_t j = i + 1; j < m->ops.size(); j++) {
        const Op& q = m->ops[j];
        if (q.x == o.x || q.res == o.x || (o.res != o.x && (q.x == o.res || q.res == o.res)))
          return set_error(CD_ERR_UNSUPPORTED, "%s: the inputs of an attention op must have no other reader", fn);
      }
    }
  }
  return CD_OK;
}

extern "C" int codistill_forward(const cd_model* m, const void* params, const void* x, int64_t batch, int save,
                                 int bn_mode, float* bn_running, void* workspace, size_t workspace_bytes,
                                 float* logits_out, void* stream) {
  int rc = check_common("forward", m, params, x, batch, workspace);
  if (rc) return rc;
  CD_REQUIRE(logits_out != nullptr && aligned16(logits_out), "forward: logits_out is NULL or misaligned");
  CD_REQUIRE(bn_mode == CD_BN_BATCH_STATS || bn_mode == CD_BN_RUNNING, "forward: unknown bn_mode %d", bn_mode);
  CD_REQUIRE(bn_mode == CD_BN_BATCH_STATS || bn_running != nullptr, "forward: CD_BN_RUNNING needs the running averages");
  if (bn_mode == CD_BN_RUNNING && save)
    return set_error(CD_ERR_UNSUPPORTED, "forward: no backward pass through an evaluation-mode BatchNorm (save_for_backward = 0)");
  CD_REQUIRE((reinterpret_cast<uintptr_t>(bn_running) & 3) == 0, "forward: bn_running is not 4-byte aligned");
  Ctx c;
  c.m = m;
  c.plan = make_plan(m, batch, save != 0);
  if (workspace_bytes < c.plan.total)
    return set_error(CD_ERR_WORKSPACE_TOO_SMALL, "forward: workspace %zu < %zu bytes", workspace_bytes, c.plan.total);
  rc = check_supported("forward", m, c.plan, batch, false);
  if (rc) return rc;
  c.ws = static_cast<char*>(workspace);
  c.params = static_cast<const char*>(params);
  c.x = x;
  c.B = batch;
  c.s = static_cast<hipStream_t>(stream);
  const int dt = m->dtype;
  const int logits_t = m->ops.back().y;

  if (c.packed()) {   // where the sentences of this batch begin, per stream (the backward pass reads the same tables)
    const int32_t* tok = static_cast<const int32_t*>(x);
    ProfScope pr(CD_K_GLUE, c.s, 0, 8.0 * (m->arch.in_h + m->arch.in_w));
    sentence_tables(tok, c.positions(), m->arch.in_h, m->arch.max_sentences, c.table(0), c.s);
    sentence_tables(tok + m->arch.in_h, c.positions() + m->arch.in_h, m->arch.in_w, m->arch.max_sentences, c.table(1), c.s);
  }
  int stat_chunks = 0, stat_tensor = -1;  // statistics a convolution left in the partials area for its BatchNorm
  for (size_t oi = 0; oi < m->ops.size(); oi++) {
    const Op& o = m->ops[oi];
    const void* in = o.x == 0 ? x : c.act(o.x);
    void* out = o.y == logits_t ? static_cast<void*>(logits_out) : c.act(o.y);
    const TensorDesc& tx = m->tensors[o.x];
    switch (o.kind) {
      case OP_CONV: {
        ConvGeom g = conv_geom(m, o, batch);
        if (grouped_sliced(m, o, batch)) {
          // grouped, in place on the row-major tensors: one launch whose column tiles are slices of whole groups; the
          // BatchNorm that follows gets its column sums from the epilogue like behind a dense convolution
          const bool fuse = bn_mode == CD_BN_BATCH_STATS && oi + 1 < m->ops.size() && m->ops[oi + 1].kind == OP_BN &&
                            m->ops[oi + 1].x == o.y &&
                            (size_t)(g.M() / 128 + 1 + 32) * stat_pitch(g.Cout) * sizeof(float) <= c.plan.partials_bytes;
          ProfScope pr(CD_K_CONV_FPROP_NARROW, c.s, 2.0 * g.M() * g.Cout * (double)g.kh * g.kw * grouped_mfma_slice(g.Cin, o.groups),
                       conv_bytes(m, g));
          stat_chunks = conv_grouped_fprop_mfma(static_cast<const bf16_t*>(in), static_cast<const bf16_t*>(c.P(o.pw)),
                                                reinterpret_cast<bf16_t*>(c.ws + c.plan.gw), static_cast<bf16_t*>(out), g, o.groups,
                                                fuse ? c.partials() : nullptr, c.s);
          stat_tensor = fuse ? o.y : -1;
          break;
        }
        if (o.groups > 1) {
          // grouped: slice-major copy of the input, dense per-slice filters, one dense convolution per slice of
          // channels, copy back (conv_grouped.hip); the BatchNorm behind it takes its statistics from the tensor
          const int C = g.Cin, sw = grouped_slice_width(C), ns = C / sw;
          const int64_t Min = batch * g.H * g.W, Mout = g.M();
          bf16_t* tmp0 = reinterpret_cast<bf16_t*>(c.ws + c.plan.gtmp);
          bf16_t* tmp1 = reinterpret_cast<bf16_t*>(c.ws + c.plan.gtmp + c.plan.gtmp_bytes);
          bf16_t* xs = c.plan.gx[oi] ? reinterpret_cast<bf16_t*>(c.ws + c.plan.gx[oi]) : tmp0;
          bf16_t* wd = reinterpret_cast<bf16_t*>(c.ws + c.plan.gw);
          {
            ProfScope pr(CD_K_GLUE, c.s, 0, 2.0 * (double)(Min + Mout) * C * 2);
            slices_gather(static_cast<const bf16_t*>(in), xs, Min, C, c.s);
            expand_group_weights(static_cast<const bf16_t*>(c.P(o.pw)), wd, C, g.kh * g.kw, o.groups, c.s);
          }
          ConvGeom gs = g;
          gs.Cin = gs.Cout = sw;
          {
            ProfScope pr(CD_K_CONV_FPROP, c.s, 2.0 * Mout * C * (double)sw * g.kh * g.kw, 2.0 * (double)(Min + Mout) * C);
            for (int sl = 0; sl < ns; sl++)
              conv_fprop_mfma(xs + (int64_t)sl * Min * sw, wd + (int64_t)sl * sw * g.kh * g.kw * sw, nullptr, false,
                              tmp1 + (int64_t)sl * Mout * sw, gs, nullptr, c.s);
          }
          {
            ProfScope pr(CD_K_GLUE, c.s, 0, 2.0 * (double)Mout * C * 2);
            slices_scatter(tmp1, static_cast<bf16_t*>(out), Mout, C, false, c.s);
          }
          break;
        }
        if (use_mfma(m, g) && !(o.relu && o.pb < 0)) {   // (a fused ReLU comes with a bias in every graph built here)
          const bf16_t* src = static_cast<const bf16_t*>(in);
          const bf16_t* w = static_cast<const bf16_t*>(c.P(o.pw));
          const ConvGeom gp = packed_geom(g);
          if (g.Cin == 3) {  // re-lay-out image and filter for 16-byte channel vectors
            ProfScope pr(CD_K_GLUE, c.s, 0, (double)batch * g.H * g.W * (3 + 8) * 2);
            if (s2d_form(g)) {
              s2d_pack_x(src, c.xpack(), batch, g.H, g.W, c.s);
              s2d_pack_w(w, c.wpack(), g.Cout, g.kh, gp.kh, 2 * gp.pad - g.pad, c.s);
            } else {
              pad_c3_to_c8(src, c.xpack(), batch * g.H * g.W, c.s);
              pad_c3_to_c8(w, c.wpack(), (int64_t)g.Cout * g.kh * g.kw, c.s);
            }
            src = c.xpack();
            w = c.wpack();
          }
          const int tc = conv_fprop_tile_class(g, o.pb >= 0);
          ProfScope pr(tc == 0 ? CD_K_CONV_FPROP : (tc == 1 ? CD_K_CONV_FPROP_WIDE : CD_K_CONV_FPROP_NARROW), c.s,
                       2.0 * g.M() * g.Cout * g.K(),
                       conv_bytes(m, g));
          // a BatchNorm that follows directly gets its column sums from the convolution's epilogue
          const bool fuse = bn_mode == CD_BN_BATCH_STATS && o.pb < 0 && oi + 1 < m->ops.size() &&
                            m->ops[oi + 1].kind == OP_BN && m->ops[oi + 1].x == o.y &&
                            (size_t)(g.M() / 128 + 1 + 32) * stat_pitch(g.Cout) * sizeof(float) <= c.plan.partials_bytes;
          stat_chunks = conv_fprop_mfma(src, w, static_cast<const bf16_t*>(c.P(o.pb)), o.relu, static_cast<bf16_t*>(out), gp,
                                        fuse ? c.partials() : nullptr, c.s);
          stat_tensor = fuse ? o.y : -1;
        } else {
          ProfScope pr(CD_K_CONV_FPROP_NARROW, c.s, 2.0 * g.M() * g.Cout * g.K(), conv_bytes(m, g));
          conv_fprop_simple(dt, in, c.P(o.pw), c.P(o.pb), out, g, o.relu, c.s);
        }
        break;
      }
      case OP_BN: {
        const int64_t M = batch * tx.h * tx.w;
        uint8_t* mask = c.plan.aux[oi] ? reinterpret_cast<uint8_t*>(c.ws + c.plan.aux[oi]) : nullptr;
        const bool fused = stat_tensor == o.x;   // the column sums came with the convolution
        const void* res = o.res >= 0 ? c.act(o.res) : nullptr;
        float* running = bn_running ? bn_running + 2 * m->bn_off[o.bn_slot] : nullptr;   // this op's [mean | var]
        if (bn_mode == CD_BN_RUNNING) {
          ProfScope pr(CD_K_NORM, c.s, 0, 0.0);
          bn_stats_from_running(dt, running, c.P(o.pw), c.P(o.pb), c.stats(o), tx.c, c.s);
        } else {
          ProfScope pr(CD_K_NORM, c.s, 0, fused ? 0.0 : (double)M * tx.c * m->esize());
          bn_stats(dt, in, c.P(o.pw), c.P(o.pb), M, tx.c, c.stats(o), c.partials(), fused ? stat_chunks : 0,
                   fused ? c.partials() + (size_t)stat_chunks * stat_pitch(tx.c) : nullptr, c.s);
          if (running) bn_running_update(c.stats(o), running, M, tx.c, 0.1f, c.s);
        }
        if (pool_fused(m, (int)oi)) {   // the next op, a max-pool, is computed here; `out` stays unwritten
          const Op& q = m->ops[oi + 1];
          ProfScope pr(CD_K_NORM, c.s, 0, (double)M * tx.c * (m->esize() * 1.25 + (mask ? 0.125 : 0.0) + (c.plan.aux[oi + 1] ? 0.25 : 0.0)));
          bn_relu_pool(static_cast<const bf16_t*>(in), c.stats(o), static_cast<bf16_t*>(c.act(q.y)),
                       c.plan.aux[oi + 1] ? reinterpret_cast<uint8_t*>(c.ws + c.plan.aux[oi + 1]) : nullptr, mask, batch, tx.h,
                       tx.w, tx.c, c.s);
        } else {
          ProfScope pr(CD_K_BN_APPLY, c.s, 0,
                       (double)M * tx.c * (m->esize() * (2 + (res ? 1 : 0)) + (o.relu && mask ? 0.125 : 0.0)));
          bn_apply(dt, in, res, o.relu, out, M, tx.c, c.stats(o), mask, c.s);
        }
        stat_tensor = -1;
        break;
      }
      case OP_LN: {
        const int64_t rows = batch * tx.h * tx.w;
        const void* res = o.res < 0 ? nullptr : (o.res == 0 ? x : c.act(o.res));
        ProfScope pr(CD_K_NORM, c.s, 0, (double)rows * tx.c * m->esize() * (2 + (res ? 1 : 0)));
        ln_forward(dt, in, res, c.P(o.pw), c.P(o.pb), out,
                   c.plan.aux[oi] ? reinterpret_cast<float*>(c.ws + c.plan.aux[oi]) : nullptr, rows, tx.c, c.s);
        break;
      }
      case OP_MAXPOOL: {
        if (pool_fused(m, (int)oi - 1)) break;   // computed by the BatchNorm in front of it
        ProfScope pr(CD_K_GLUE, c.s, 0, (double)batch * tx.per_sample() * m->esize() * 1.25);
        maxpool_fwd(dt, in, out, c.plan.aux[oi] ? reinterpret_cast<uint8_t*>(c.ws + c.plan.aux[oi]) : nullptr, batch, tx.h,
                    tx.w, tx.c, o.k, o.stride, o.pad, c.s);
        break;
      }
      case OP_GAP: {
        ProfScope pr(CD_K_GLUE, c.s, 0, (double)batch * tx.per_sample() * m->esize());
        gap_fwd(dt, in, out, batch, tx.h * tx.w, tx.c, c.s);
        break;
      }
      case OP_SLICE: {
        const TensorDesc& ty = m->tensors[o.y];
        ProfScope pr(CD_K_GLUE, c.s, 0, 2.0 * batch * ty.per_sample() * m->esize());
        channel_slice(dt, in, out, batch * tx.h * tx.w, tx.c, o.a0, ty.c, c.s);
        break;
      }
      case OP_LINEAR: {
        const int F = tx.c, C = m->tensors[o.y].c;
        const int64_t rows = batch * tx.h * tx.w;
        ProfScope pr(CD_K_LINEAR, c.s, 2.0 * rows * F * C,
                     (double)m->esize() * ((double)rows * F + (double)F * C) + 4.0 * rows * C);
        if (dt == CD_BF16 && !force_simple() && F % 8 == 0 && (int64_t)F * C * 2 < (1LL << 31))
          linear_fwd_mfma(static_cast<const bf16_t*>(in), static_cast<const bf16_t*>(c.P(o.pw)),
                          static_cast<const bf16_t*>(c.P(o.pb)), static_cast<float*>(out), rows, F, C, c.s);
        else
          linear_fwd(dt, in, c.P(o.pw), c.P(o.pb), static_cast<float*>(out), rows, F, C, c.s);
        break;
      }
      case OP_EMBED: {
        const TensorDesc& ty = m->tensors[o.y];
        ProfScope pr(CD_K_GLUE, c.s, 0, (double)batch * ty.per_sample() * m->esize() * 2);
        embed_forward(dt, static_cast<const int32_t*>(x), m->tensors[0].w, o.a0, o.a1, c.P(o.pw), m->arch.classes, ty.c, out,
                      batch * ty.h, c.positions(), c.s);
        break;
      }
      case OP_ATTN: {
        const TensorDesc& tkv = m->tensors[o.res];
        const TensorDesc& ty = m->tensors[o.y];
        const int d = ty.c, dh = d / o.heads;
        // packed sentences: one workgroup row per possible sentence, the tables say where each one lies
        const bool pk = c.packed();
        const int S = pk ? m->arch.max_sentences : (int)batch;
        const int Tq = pk ? std::min(m->arch.max_sentence_len, tx.h) : tx.h, Tk = pk ? std::min(m->arch.max_sentence_len, tkv.h) : tkv.h;
        const SentenceTables tab = c.tables(o, tx.h, tkv.h);
        const bf16_t* kvp = static_cast<const bf16_t*>(c.act(o.res));
        // (work figures of a packed batch: as if every row attended to a full-length sentence, an upper bound)
        ProfScope pr(CD_K_ATTN, c.s, 4.0 * batch * o.heads * tx.h * (double)Tk * dh * (o.causal ? 0.5 : 1.0),
                     2.0 * batch * ((double)tx.h * 2 + (double)tkv.h * 2) * d);
        attention_forward(static_cast<const bf16_t*>(in) + o.a0, tx.c, kvp + o.a1, kvp + o.a2, tkv.c,
                          static_cast<bf16_t*>(out), d, c.plan.aux[oi] ? reinterpret_cast<float*>(c.ws + c.plan.aux[oi]) : nullptr,
                          S, o.heads, Tq, Tk, dh, o.causal, static_cast<const int32_t*>(x), m->tensors[0].w, o.key_tok0,
                          pk ? &tab : nullptr, c.s);
        break;
      }
    }
  }
  return check_launch("forward");
}

// --------------------------------------------------------------------------------- backward
extern "C" int codistill_backward(const cd_model* m, const void* params, const void* x, int64_t batch, void* workspace,
                                  size_t workspace_bytes, const float* dlogits, float* grads_out, void* stream) {
  int rc = check_common("backward", m, params, x, batch, workspace);
  if (rc) return rc;
  CD_REQUIRE(dlogits && grads_out && aligned16(dlogits) && aligned16(grads_out),
             "backward: dlogits / grads_out is NULL or misaligned");
  Ctx c;
  c.m = m;
  c.plan = make_plan(m, batch, true);
  if (workspace_bytes < c.plan.total)
    return set_error(CD_ERR_WORKSPACE_TOO_SMALL, "backward: workspace %zu < %zu bytes", workspace_bytes, c.plan.total);
  rc = check_supported("backward", m, c.plan, batch, true);
  if (rc) return rc;
  c.ws = static_cast<char*>(workspace);
  c.params = static_cast<const char*>(params);
  c.x = x;
  c.B = batch;
  c.s = static_cast<hipStream_t>(stream);
  const int dt = m->dtype;
  const int logits_t = m->ops.back().y;
  auto G = [&](int pidx) { return grads_out + m->params[pidx].offset; };

  {  // padding between tensors in the flat gradient
    std::vector<Gap> gaps;
    for (const ParamDesc& p : m->params)
      if (p.size % 8) gaps.push_back(Gap{p.offset + p.size, (int32_t)(8 - p.size % 8)});
    if (!gaps.empty()) zero_gaps(grads_out, gaps.data(), (int)gaps.size(), c.s);
  }

  // The weight gradient of a convolution needs dy and the saved input only, and nothing downstream
  // but the optimizer needs its result: these launches fork onto a second stream (with their own
  // split-K partials) and run beside the data gradients and BatchNorm passes that follow; the
  // caller's stream waits for them at the end.  One stream when the per-launch timer is on.
  // The side stream and its events belong to the library and are shared by every caller of this process: the lock
  // is held from here to the join, so that two host threads never interleave forks on it.  Everything the forks
  // need (the stream, one event per convolution and one for the join) exists before the first launch; if the
  // runtime refuses any of it the call runs on the caller's stream alone.
  std::unique_lock<std::mutex> side_lock(side_mutex(), std::defer_lock);
  hipStream_t side = nullptr;
  if (!timer_enabled() && !force_serial()) {
    side_lock.lock();
    int convs = 0;
    for (const Op& o : m->ops) convs += o.kind == OP_CONV ? 1 : 0;
    side = side_stream();
    if (side && !side_event(convs)) side = nullptr;
    if (!side) side_lock.unlock();
  }
  {   // the filters of all matrix-core data gradients, in the layouts those read them, by one launch (per 48 filters)
    std::vector<WeightLayoutJob> jobs;
    double bytes = 0;
    for (size_t i = (size_t)m->first_trainable_op; i < m->ops.size(); i++)
      if (c.plan.wt_op[i]) {
        const ConvGeom g = conv_geom(m, m->ops[i], batch);
        conv_dgrad_layout_jobs(static_cast<const bf16_t*>(c.P(m->ops[i].pw)), reinterpret_cast<bf16_t*>(c.ws + c.plan.wt_op[i]), g, jobs);
        bytes += 4.0 * g.Cout * g.K();
      }
    if (!jobs.empty()) {
      ProfScope pr(CD_K_GLUE, c.s, 0, bytes);
      relayout_weights_batch(jobs, c.s);
    }
  }
  int forks = 0;
  int late_rc = CD_OK;   // a launch-time failure of the fork / join machinery: reported after the join was attempted
  std::vector<char> written(m->tensors.size(), 0);
  // gradients of residual inputs that are handed on as "dy and a bit mask" instead of being written
  // (see residual_grad_route)
  struct Deferred { const void* src = nullptr; const uint8_t* gate = nullptr; };
  std::vector<Deferred> deferred(m->tensors.size());
  // BatchNorm op b whose kernel also computed the max-pool behind it: its backward pass gathers its dy from
  // the pooled gradient and the argmax, and the max-pool's own backward launch is dropped
  auto pool_fused_bwd = [&](int b) {
    const TensorDesc& t = m->tensors[m->ops[b].y];   // 32-bit element offsets in the gather kernels
    return pool_fused(m, b) && m->ops[b].x != 0 && !written[m->ops[b].x] && c.plan.aux[b] != 0 && c.plan.aux[b + 1] != 0 &&
           batch * t.per_sample() < (1LL << 31);
  };
  // Tensors that are the ReLU'd output of a convolution and have one reader, itself a stride-1 convolution on the
  // matrix-core path: that reader's data-gradient kernel applies the ReLU mask as it writes the tensor's gradient,
  // and the producing convolution's own masking pass is dropped.
  // tensor -> chunks of BatchNorm backward sums that the data gradient which completed its gradient left in the partials
  // area (0: none): the BatchNorm that produced the tensor, the op right in front of that convolution, skips its reduction
  std::vector<int> bn_sums(m->tensors.size(), 0);
  std::vector<int> producer(m->tensors.size(), -1), readers(m->tensors.size(), 0);
  for (size_t j = 0; j < m->ops.size(); j++) {
    producer[m->ops[j].y] = (int)j;
    readers[m->ops[j].x]++;
    if (m->ops[j].res >= 0 && m->ops[j].res != m->ops[j].x) readers[m->ops[j].res]++;
  }
  std::vector<char> relu_done(m->tensors.size(), 0);
  // frozen front end (the ops before first_trainable_op): no gradient reaches it; its parameters' gradients are zeros
  for (int i = 0; i < m->first_trainable_op; i++) {
    const Op& o = m->ops[i];
    for (int pi : {o.pw, o.pb})
      if (pi >= 0) fill_zero_f32(G(pi), m->params[pi].size, c.s);
  }
  for (int i = (int)m->ops.size() - 1; i >= m->first_trainable_op; i--) {
    const Op& o = m->ops[i];
    const TensorDesc& tx = m->tensors[o.x];
    const void* in = o.x == 0 ? x : c.act(o.x);
    void* dy = o.y == logits_t ? nullptr : c.grad(o.y);
    void* dx = o.x == 0 ? nullptr : c.grad(o.x);
    const bool acc = o.x != 0 && written[o.x];
    switch (o.kind) {
      case OP_LINEAR: {
        const int F = tx.c, C = m->tensors[o.y].c;
        const int64_t rows = batch * tx.h * tx.w;
        ConvGeom g;  // the dense layer as a 1x1 convolution over one pixel per row
        g.B = rows; g.H = g.W = g.Ho = g.Wo = 1; g.Cin = F; g.Cout = C; g.kh = g.kw = 1; g.stride = 1; g.pad = 0;
        if (dt == CD_BF16 && !force_simple() && conv_mfma_supported(g)) {
          bf16_t* dzb = reinterpret_cast<bf16_t*>(c.ws + c.plan.lin_dz);
          {
            ProfScope pr(CD_K_GLUE, c.s, 0, (double)rows * C * (6.0 + (o.pb >= 0 ? 4.0 : 0.0)));
            cast_f32_bf16(dlogits, dzb, rows * C, c.s);
            if (o.pb >= 0) colsum(CD_F32, dlogits, rows, C, G(o.pb), c.partials(), c.s);
          }
          {
            // (on the caller's stream: a tied table's gradient is added to by the embedding ops at the end)
            ProfScope pr(CD_K_CONV_WGRAD, c.s, 2.0 * rows * F * C, conv_bytes(m, g) + 2.0 * C * F);
            conv_wgrad_mfma(static_cast<const bf16_t*>(in), dzb, G(o.pw), g, c.partials(), c.plan.partials_bytes, c.s);
          }
          {
            ProfScope pr(CD_K_CONV_DGRAD, c.s, 2.0 * rows * F * C, conv_bytes(m, g));
            conv_dgrad_mfma(dzb, static_cast<const bf16_t*>(c.P(o.pw)), c.wpack(), static_cast<bf16_t*>(dx), g, acc, c.s);
          }
        } else {
          ProfScope pr(CD_K_LINEAR, c.s, 4.0 * rows * F * C, (double)m->esize() * ((double)rows * F + (double)F * C) * 2);
          linear_bwd(dt, in, c.P(o.pw), dlogits, dx, acc, G(o.pw), o.pb >= 0 ? G(o.pb) : nullptr, rows, F, C, c.s);
        }
        break;
      }
      case OP_EMBED: {
        // every occurrence of a token adds its row of dy to the table's gradient, which already holds the
        // gradient of the tied output projection (the first op of this pass)
        const TensorDesc& ty = m->tensors[o.y];
        ProfScope pr(CD_K_GLUE, c.s, 0, (double)batch * ty.per_sample() * (m->esize() + 8.0));
        embed_backward(dt, static_cast<const int32_t*>(x), m->tensors[0].w, o.a0, o.a1, dy, m->arch.classes, ty.c, G(o.pw),
                       batch * ty.h, c.s);
        break;
      }
      case OP_ATTN: {
        const TensorDesc& tkv = m->tensors[o.res];
        const TensorDesc& ty = m->tensors[o.y];
        const int d = ty.c, dh = d / o.heads;
        const bool pk = c.packed();
        const int S = pk ? m->arch.max_sentences : (int)batch;
        const int Tq = pk ? std::min(m->arch.max_sentence_len, tx.h) : tx.h, Tk = pk ? std::min(m->arch.max_sentence_len, tkv.h) : tkv.h;
        const SentenceTables tab = c.tables(o, tx.h, tkv.h);
        // (inputs with another reader were rejected by check_supported before the first launch)
        const bf16_t* kvp = static_cast<const bf16_t*>(c.act(o.res));
        bf16_t* dkv = static_cast<bf16_t*>(c.grad(o.res));
        float* lse = reinterpret_cast<float*>(c.ws + c.plan.aux[i]);
        ProfScope pr(CD_K_ATTN, c.s, 14.0 * batch * o.heads * tx.h * (double)Tk * dh * (o.causal ? 0.5 : 1.0),
                     2.0 * batch * ((double)tx.h * 3 + (double)tkv.h * 4) * d);
        attention_backward(static_cast<const bf16_t*>(in) + o.a0, tx.c, kvp + o.a1, kvp + o.a2, tkv.c,
                           static_cast<const bf16_t*>(dy), d, lse, lse + (size_t)batch * o.heads * tx.h,
                           static_cast<bf16_t*>(dx) + o.a0, dkv + o.a1, dkv + o.a2, S, o.heads, Tq, Tk, dh, o.causal,
                           static_cast<const int32_t*>(x), m->tensors[0].w, o.key_tok0, pk ? &tab : nullptr, c.s);
        written[o.res] = 1;
        break;
      }
      case OP_GAP: {
        ProfScope pr(CD_K_GLUE, c.s, 0, (double)batch * tx.per_sample() * m->esize());
        gap_bwd(dt, dy, dx, acc, batch, tx.h * tx.w, tx.c, c.s);
        break;
      }
      case OP_SLICE: break;   // never reached: the loop stops behind it
      case OP_MAXPOOL: {
        if (pool_fused_bwd(i - 1)) continue;   // gathered by the BatchNorm's backward pass instead (nothing written)
        ProfScope pr(CD_K_GLUE, c.s, 0, (double)batch * tx.per_sample() * m->esize() * 2.25);
        maxpool_bwd(dt, in, dy, c.plan.aux[i] ? reinterpret_cast<const uint8_t*>(c.ws + c.plan.aux[i]) : nullptr, dx, acc,
                    batch, tx.h, tx.w, tx.c, o.k, o.stride, o.pad, c.s);
        break;
      }
      case OP_BN: {
        const int64_t M = batch * tx.h * tx.w;
        void* dres = o.res >= 0 ? c.grad(o.res) : nullptr;
        const bool acc_res = o.res >= 0 && written[o.res];
        const uint8_t* mask = c.plan.aux[i] ? reinterpret_cast<const uint8_t*>(c.ws + c.plan.aux[i]) : nullptr;
        if (pool_fused_bwd(i)) {
          // the max-pool behind this op did not write this op's dy: both passes gather it from the pooled gradient
          const Op& q = m->ops[i + 1];
          ProfScope pr(CD_K_NORM, c.s, 0, (double)M * tx.c * (m->esize() * 3.5 + 0.25 + 0.5));
          bn_relu_pool_backward(static_cast<const bf16_t*>(c.grad(q.y)), reinterpret_cast<const uint8_t*>(c.ws + c.plan.aux[i + 1]),
                                static_cast<const bf16_t*>(in), static_cast<const bf16_t*>(c.P(o.pw)), c.stats(o),
                                static_cast<bf16_t*>(dx), G(o.pw), G(o.pb), c.coef(), c.partials(), mask, batch, tx.h, tx.w,
                                tx.c, c.s);
          break;
        }
        // two passes over dy and x (+ y, or its sign bits, under a ReLU), dx written once (+ the residual's copy).
        // This layer's own dy may be a deferred one (kind 1): read it through the gate it came with.
        const void* dy_in = dy;
        bool gated = o.relu;
        if (deferred[o.y].src) {
          dy_in = deferred[o.y].src;
          if (deferred[o.y].gate) { gated = true; mask = deferred[o.y].gate; }
        }
        const bool defer = o.res >= 0 && !acc_res && residual_grad_route(m, i, batch) != 0;
        if (defer) {
          deferred[o.res].src = dy_in;
          deferred[o.res].gate = gated ? mask : nullptr;
          dres = nullptr;
        }
        const double per_elt = m->esize() * (5 + (dres ? 1 : 0)) + (gated ? (mask ? 0.25 : 2.0 * m->esize()) : 0.0);
        ProfScope pr(CD_K_NORM, c.s, 0, (double)M * tx.c * per_elt);
        // (sums left by the data gradient that wrote dy: only ever set for this op's own, ungated-route dy)
        const int pre = dy_in == dy ? bn_sums[o.y] : 0;
        bn_backward(dt, dy_in, c.act(o.y), in, c.P(o.pw), c.stats(o), gated, dx, acc, dres, acc_res, G(o.pw), G(o.pb),
                    c.coef(), c.partials(), mask, M, tx.c, c.s, pre);
        if (o.res >= 0 && !defer) written[o.res] = 1;
        break;
      }
      case OP_LN: {
        const int64_t rows = batch * tx.h * tx.w;
        const void* res = o.res < 0 ? nullptr : (o.res == 0 ? x : c.act(o.res));
        void* dres = o.res > 0 ? c.grad(o.res) : nullptr;   // the input batch takes no gradient
        const bool acc_res = o.res > 0 && written[o.res];
        ProfScope pr(CD_K_NORM, c.s, 0, (double)rows * tx.c * m->esize() * (3 + (res ? 1 : 0) + (dres ? 1 : 0)));
        ln_backward(dt, dy, in, res, c.P(o.pw), reinterpret_cast<const float*>(c.ws + c.plan.aux[i]), dx, acc, dres,
                    acc_res, G(o.pw), G(o.pb), c.partials(), rows, tx.c, c.s);
        if (o.res > 0) written[o.res] = 1;
        break;
      }
      case OP_CONV: {
        ConvGeom g = conv_geom(m, o, batch);
        if (grouped_sliced(m, o, batch)) {
          const double fl = 2.0 * g.M() * g.Cout * (double)g.kh * g.kw * grouped_mfma_slice(g.Cin, o.groups);
          {
            ProfScope pr(CD_K_CONV_WGRAD, c.s, fl, conv_bytes(m, g));
            conv_grouped_wgrad_mfma(static_cast<const bf16_t*>(in), static_cast<const bf16_t*>(dy),
                                    reinterpret_cast<float*>(c.ws + c.plan.gdw), G(o.pw), g, o.groups, c.partials(),
                                    c.plan.partials_bytes, c.s);
          }
          {
            ProfScope pr(CD_K_CONV_DGRAD, c.s, fl, conv_bytes(m, g));
            conv_grouped_dgrad_mfma(static_cast<const bf16_t*>(dy), static_cast<const bf16_t*>(c.P(o.pw)),
                                    reinterpret_cast<bf16_t*>(c.ws + c.plan.gw), static_cast<bf16_t*>(dx), g, o.groups, acc, c.s);
          }
          break;
        }
        if (o.groups > 1) {
          const int C = g.Cin, sw = grouped_slice_width(C), ns = C / sw, taps = g.kh * g.kw;
          const int64_t Min = batch * g.H * g.W, Mout = g.M();
          bf16_t* dys = reinterpret_cast<bf16_t*>(c.ws + c.plan.gtmp);
          bf16_t* dxs = reinterpret_cast<bf16_t*>(c.ws + c.plan.gtmp + c.plan.gtmp_bytes);
          const bf16_t* xs = reinterpret_cast<const bf16_t*>(c.ws + c.plan.gx[i]);
          bf16_t* wd = reinterpret_cast<bf16_t*>(c.ws + c.plan.gw);
          float* dwd = reinterpret_cast<float*>(c.ws + c.plan.gdw);
          {
            ProfScope pr(CD_K_GLUE, c.s, 0, 2.0 * (double)Mout * C * 2);
            slices_gather(static_cast<const bf16_t*>(dy), dys, Mout, C, c.s);
            expand_group_weights(static_cast<const bf16_t*>(c.P(o.pw)), wd, C, taps, o.groups, c.s);
          }
          ConvGeom gs = g;
          gs.Cin = gs.Cout = sw;
          const int64_t wsl = (int64_t)sw * taps * sw;   // elements of one slice's dense filter
          {
            ProfScope pr(CD_K_CONV_WGRAD, c.s, 2.0 * Mout * C * (double)sw * taps, 2.0 * (double)(Min + Mout) * C);
            for (int sl = 0; sl < ns; sl++)
              conv_wgrad_mfma(xs + (int64_t)sl * Min * sw, dys + (int64_t)sl * Mout * sw, dwd + sl * wsl, gs, c.partials(),
                              c.plan.partials_bytes, c.s);
            extract_group_dw(dwd, G(o.pw), C, taps, o.groups, c.s);
          }
          {
            ProfScope pr(CD_K_CONV_DGRAD, c.s, 2.0 * Mout * C * (double)sw * taps, 2.0 * (double)(Min + Mout) * C);
            for (int sl = 0; sl < ns; sl++)
              conv_dgrad_mfma(dys + (int64_t)sl * Mout * sw, wd + sl * wsl, c.wpack(), dxs + (int64_t)sl * Min * sw, gs, false,
                              c.s);
          }
          {
            ProfScope pr(CD_K_GLUE, c.s, 0, 2.0 * (double)Min * C * (acc ? 3 : 2));
            slices_scatter(dxs, static_cast<bf16_t*>(dx), Min, C, acc, c.s);
          }
          break;
        }
        if (o.relu && !relu_done[o.y]) {
          ProfScope pr(CD_K_GLUE, c.s, 0, (double)g.M() * g.Cout * m->esize() * 3);
          relu_bwd_inplace(dt, dy, c.act(o.y), g.M() * g.Cout, c.s);
        }
        const bool mf = use_mfma(m, g);
        {
          hipStream_t ws_ = c.s;
          float* wpart = c.partials();
          if (mf && side) {
            hipEvent_t ev = side_event(forks);
            if (ev && hipEventRecord(ev, c.s) == hipSuccess && hipStreamWaitEvent(side, ev, 0) == hipSuccess) {
              ws_ = side;
              wpart = c.partials_side();
              forks++;
            }
          }
          if (o.pb >= 0) {  // the bias gradient reads dy only, like the weight gradient: same stream, same partials area
            ProfScope pr(CD_K_GLUE, ws_, 0, (double)g.M() * g.Cout * m->esize());
            colsum(dt, dy, g.M(), g.Cout, G(o.pb), wpart, ws_);
          }
          ProfScope pr(CD_K_CONV_WGRAD, ws_, 2.0 * g.M() * g.Cout * g.K(), conv_bytes(m, g) + 2.0 * g.Cout * g.K());
          if (mf) {
            const ConvGeom gp = packed_geom(g);
            const bf16_t* src = static_cast<const bf16_t*>(in);
            float* dw = G(o.pw);
            if (g.Cin == 3) {  // the forward pass left the re-laid-out image in xpack
              src = c.xpack();
              dw = reinterpret_cast<float*>(c.wpack());
            }
            conv_wgrad_mfma(src, static_cast<const bf16_t*>(dy), dw, gp, wpart, c.plan.partials_bytes, ws_);
            if (s2d_form(g)) s2d_unpack_dw(dw, G(o.pw), g.Cout, g.kh, gp.kh, 2 * gp.pad - g.pad, ws_);
            else if (g.Cin == 3) unpad_c8_to_c3(dw, G(o.pw), (int64_t)g.Cout * g.kh * g.kw, ws_);
          } else {
            conv_wgrad_simple(dt, in, dy, G(o.pw), g, c.s);
          }
        }
        if (o.x != 0) {
          ProfScope pr(CD_K_CONV_DGRAD, c.s, 2.0 * g.M() * g.Cout * g.K(), conv_bytes(m, g));
          if (mf) {
            const Deferred df = deferred[o.x];   // kind 2: set only where this launch can take it
            deferred[o.x] = Deferred();
            const int pi = producer[o.x];
            const bool gate = g.stride == 1 && !acc && readers[o.x] == 1 && pi >= 0 && m->ops[pi].kind == OP_CONV &&
                              m->ops[pi].relu && use_mfma(m, conv_geom(m, m->ops[pi], batch)) && !fuse_off();
            // The op right in front of this convolution is the BatchNorm that produced its input: every other reader of
            // that tensor comes later in the graph and has added its share already, so this launch completes the
            // tensor's gradient and can hand the BatchNorm the column sums of its backward pass (stride 1: one launch
            // writes every row; the BatchNorm's next op in this pass is its own backward, which consumes them).
            BnBackwardSums sums = {};
            bool with_sums = false;
            if (pi == (int)i - 1 && m->ops[pi].kind == OP_BN && g.stride == 1 && !separate_bn_reduction() &&
                !pool_fused(m, pi) && m->ops[pi].x != 0 && (!m->ops[pi].relu || c.plan.aux[pi] != 0) &&
                (size_t)(batch * g.H * g.W / 128 + 1 + 32) * stat_pitch(g.Cin) * sizeof(float) <= c.plan.partials_bytes) {
              const Op& b = m->ops[pi];
              sums.x = static_cast<const bf16_t*>(c.act(b.x));
              sums.mask = b.relu ? reinterpret_cast<const uint8_t*>(c.ws + c.plan.aux[pi]) : nullptr;
              sums.stats = c.stats(b);
              sums.partials = c.partials();
              with_sums = true;
            }
            const bool ready = c.plan.wt_op[i] != 0;   // re-laid-out at the start of the pass
            const int chunks = conv_dgrad_mfma(static_cast<const bf16_t*>(dy), static_cast<const bf16_t*>(c.P(o.pw)),
                                               ready ? reinterpret_cast<bf16_t*>(c.ws + c.plan.wt_op[i]) : c.wpack(),
                                               static_cast<bf16_t*>(dx), g, acc, c.s, static_cast<const bf16_t*>(df.src), df.gate,
                                               gate ? static_cast<const bf16_t*>(c.act(o.x)) : nullptr,
                                               with_sums ? &sums : nullptr, ready);
            if (with_sums) bn_sums[o.x] = chunks;
            if (gate) relu_done[o.x] = 1;
          } else {
            conv_dgrad_simple(dt, dy, c.P(o.pw), dx, g, acc, c.s);
          }
        }
        break;
      }
    }
    if (o.x != 0) written[o.x] = 1;
  }
  if (forks > 0) {  // join: the caller's stream continues after the last weight gradient
    hipEvent_t ev = side_event(forks);
    if (!ev || hipEventRecord(ev, side) != hipSuccess || hipStreamWaitEvent(c.s, ev, 0) != hipSuccess) {
      (void)hipGetLastError();
      late_rc = set_error(CD_ERR_HIP, "backward: could not join the weight-gradient stream (event record / wait failed); "
                                      "synchronise the device before reading or freeing the buffers of this call");
    }
  }
  if (late_rc) return late_rc;
  return check_launch("backward");
}
