// C ABI of the library: spec validation, buffer layout, context life cycle, the local-update step
// (paper section 3) and named-tensor access.
#include <math.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "ctx.h"

using namespace lp;

static thread_local std::string g_init_err;
static int join_pending(lp_ctx* c);

static int fail(lp_ctx* c, int code, const std::string& msg) {
  if (c) c->err = msg; else g_init_err = msg;
  return code;
}

// ------------------------------------------------------------------------------------- validation
static int validate(const lp_model_spec* sp, std::string& err) {
  if (!sp) { err = "spec is null"; return LP_EINVAL; }
  if (sp->n_layers < 1 || !sp->layers) { err = "need at least one layer"; return LP_EINVAL; }
  if (sp->n_heads < 1 || !sp->heads) { err = "need at least one head"; return LP_EINVAL; }
  if (sp->dtype != LP_F32 && sp->dtype != LP_BF16) { err = "bad dtype"; return LP_EINVAL; }
  if (sp->combine != LP_COMBINE_SUM && sp->combine != LP_COMBINE_MEAN) { err = "bad combine"; return LP_EINVAL; }
  if (sp->opt.kind < LP_OPT_SGD || sp->opt.kind > LP_OPT_ADAM) { err = "bad optimizer kind"; return LP_EINVAL; }
  if (sp->max_batch < 1) { err = "max_batch must be >= 1"; return LP_ESHAPE; }
  if (sp->vocab < 0) { err = "vocab must be >= 0"; return LP_EINVAL; }
  if (sp->n_streams < 0 || sp->n_streams > 8) { err = "n_streams must be in [0, 8]"; return LP_EINVAL; }
  int kind0 = sp->layers[0].kind;
  int64_t prev_out = -1;
  for (int i = 0; i < sp->n_layers; ++i) {
    const lp_layer_spec& l = sp->layers[i];
    char where[32]; snprintf(where, sizeof where, "layer %d: ", i + 1);
    if (l.kind != kind0) { err = std::string(where) + "all layers must be of one kind"; return LP_EUNSUPPORTED; }
    if (l.kind == LP_LAYER_RESMLP) {
      if (l.in_dim < 1 || l.width < 1 || l.hidden < 1) { err = std::string(where) + "dims must be >= 1"; return LP_ESHAPE; }
      if (prev_out >= 0 && l.in_dim != prev_out) { err = std::string(where) + "in_dim != previous width"; return LP_ESHAPE; }
      prev_out = l.width;
    } else if (l.kind == LP_LAYER_DECODER) {
      if (l.width < 1 || l.hidden < 1 || l.n_heads < 1 || l.seq_len < 1) { err = std::string(where) + "dims must be >= 1"; return LP_ESHAPE; }
      if (l.width % l.n_heads) { err = std::string(where) + "width not divisible by n_heads"; return LP_ESHAPE; }
      int dh = l.width / l.n_heads;
      if (dh != 4 && dh != 8 && dh != 16 && dh != 32 && dh != 64) { err = std::string(where) + "head size must be 4, 8, 16, 32 or 64"; return LP_ESHAPE; }
      if (l.act != LP_ACT_GELU && l.act != LP_ACT_RELU) { err = std::string(where) + "bad activation"; return LP_EINVAL; }
      if (prev_out >= 0 && l.width != prev_out) { err = std::string(where) + "width changes between layers"; return LP_ESHAPE; }
      if (i > 0 && l.seq_len != sp->layers[0].seq_len) { err = std::string(where) + "seq_len changes between layers"; return LP_ESHAPE; }
      if (sp->vocab == 0) { err = "decoder layers need vocab > 0 (token input)"; return LP_EUNSUPPORTED; }
      prev_out = l.width;
    } else if (l.kind == LP_LAYER_RESNET_STAGE) {
      if (l.in_ch < 1 || l.out_ch < 1 || l.in_hw < 1 || l.n_basic_blocks < 1) { err = std::string(where) + "dims must be >= 1"; return LP_ESHAPE; }
      if (l.stride != 1 && l.stride != 2) { err = std::string(where) + "stride must be 1 or 2"; return LP_ESHAPE; }
      if (l.in_hw % l.stride) { err = std::string(where) + "in_hw not divisible by stride"; return LP_ESHAPE; }
      if (l.has_stem && l.stride != 1) { err = std::string(where) + "a stem stage has stride 1"; return LP_ESHAPE; }
      if (prev_out >= 0 && l.in_ch != prev_out) { err = std::string(where) + "in_ch != previous out_ch"; return LP_ESHAPE; }
      if (i > 0 && l.in_hw != sp->layers[i - 1].in_hw / sp->layers[i - 1].stride) { err = std::string(where) + "in_hw does not match previous stage"; return LP_ESHAPE; }
      prev_out = l.out_ch;
    } else {
      err = std::string(where) + "bad layer kind"; return LP_EINVAL;
    }
  }
  if (kind0 != LP_LAYER_DECODER && sp->vocab > 0) { err = "vocab > 0 needs decoder layers"; return LP_EUNSUPPORTED; }
  int prev_e = 0;
  for (int j = 0; j < sp->n_heads; ++j) {
    const lp_head_spec& h = sp->heads[j];
    char where[32]; snprintf(where, sizeof where, "head %d: ", j + 1);
    if (h.after_layer < 1 || h.after_layer > sp->n_layers) { err = std::string(where) + "after_layer out of range"; return LP_EINVAL; }
    if (h.after_layer < prev_e) { err = std::string(where) + "heads must be ordered by after_layer"; return LP_EINVAL; }
    prev_e = h.after_layer;
    if (h.window < 1) { err = std::string(where) + "window must be >= 1"; return LP_EINVAL; }
    if (h.n_classes < 2) { err = std::string(where) + "n_classes must be >= 2"; return LP_ESHAPE; }
    const lp_layer_spec& l = sp->layers[h.after_layer - 1];
    int want_kind = kind0 == LP_LAYER_RESMLP ? LP_HEAD_LINEAR_CE : kind0 == LP_LAYER_DECODER ? LP_HEAD_LN_LINEAR_CE : LP_HEAD_POOL_LINEAR_CE;
    if (h.kind != want_kind && !(kind0 == LP_LAYER_RESNET_STAGE && h.kind == LP_HEAD_BN_POOL_LINEAR_CE)) {
      err = std::string(where) + "head kind does not fit the layer kind"; return LP_EUNSUPPORTED;
    }
    int feat = kind0 == LP_LAYER_RESNET_STAGE ? l.out_ch : l.width;
    if (h.in_dim != feat) { err = std::string(where) + "in_dim != layer output width"; return LP_ESHAPE; }
    if (kind0 == LP_LAYER_DECODER && h.n_classes != sp->vocab) { err = std::string(where) + "n_classes != vocab"; return LP_ESHAPE; }
    if (kind0 == LP_LAYER_DECODER && h.bias) { err = std::string(where) + "vocabulary heads have no bias"; return LP_EUNSUPPORTED; }
  }
  if (sp->schedule < LP_SCHED_SYNC || sp->schedule > LP_SCHED_PIPELINED_GROUPED) { err = "bad schedule"; return LP_EINVAL; }
  if (sp->schedule == LP_SCHED_PIPELINED_GROUPED) {
    const lp_head_spec& h0 = sp->heads[0];
    const int nl0 = (h0.window < h0.after_layer ? h0.window : h0.after_layer);
    for (int j = 0; j < sp->n_heads; ++j) {
      const lp_head_spec& h = sp->heads[j];
      const int w = h.window < h.after_layer ? h.window : h.after_layer;
      if (kind0 != LP_LAYER_DECODER || w != nl0 || h.kind != LP_HEAD_LN_LINEAR_CE || h.bias) {
        err = "the grouped pipelined schedule needs decoder blocks of equal depth with vocabulary heads";
        return LP_EUNSUPPORTED;
      }
    }
  }
  if (sp->schedule != LP_SCHED_SYNC) {          // blocks must tile the layers: window j starts where window j-1 ends
    int end = 0;
    for (int j = 0; j < sp->n_heads; ++j) {
      const lp_head_spec& h = sp->heads[j];
      int w = h.window < h.after_layer ? h.window : h.after_layer;
      if (h.after_layer - w != end) { err = "the pipelined schedule needs windows that tile the layers"; return LP_EUNSUPPORTED; }
      end = h.after_layer;
    }
  }
  return LP_OK;
}

// ------------------------------------------------------------------------------------- layout
static int add_tensor(lp_ctx* c, const std::string& name, std::initializer_list<int64_t> shape, int owner, int init,
                      float std) {
  Tensor t;
  t.name = name; t.ndim = (int)shape.size(); t.numel = 1;
  int i = 0;
  for (int64_t s : shape) { t.shape[i++] = s; t.numel *= (size_t)s; }
  t.off = c->P; t.owner = owner; t.init = init; t.std = std;
  c->P += (t.numel + 63) & ~(size_t)63;
  c->index[name] = (int)c->tensors.size();
  c->tensors.push_back(t);
  return (int)c->tensors.size() - 1;
}

static void build_params(lp_ctx* c) {
  const lp_model_spec& sp = c->spec;
  int L = sp.n_layers;
  c->layers.assign(L + 1, LayerState());
  for (int li = 1; li <= L; ++li) {
    LayerState& S = c->layers[li];
    S.s = c->layer_specs[li - 1];
    const lp_layer_spec& l = S.s;
    S.p_begin = c->P;
    std::string p = "L" + std::to_string(li) + ".";
    auto kaiming = [](int64_t fan_in) { return (float)sqrt(2.0 / (double)fan_in); };
    auto W = [&](const char* n, std::initializer_list<int64_t> sh, float std) { S.t[n] = add_tensor(c, p + n, sh, li, 0, std); };
    auto Z = [&](const char* n, int64_t k) { S.t[n] = add_tensor(c, p + n, {k}, li, 2, 0.f); };
    auto O = [&](const char* n, int64_t k) { S.t[n] = add_tensor(c, p + n, {k}, li, 1, 0.f); };
    if (l.kind == LP_LAYER_RESMLP) {
      if (l.in_dim != l.width) { W("win", {l.width, l.in_dim}, kaiming(l.in_dim)); Z("bin", l.width); }
      W("w1", {l.hidden, l.width}, kaiming(l.width)); Z("b1", l.hidden);
      W("w2", {l.width, l.hidden}, kaiming(l.hidden)); Z("b2", l.width);
    } else if (l.kind == LP_LAYER_DECODER) {
      int64_t d = l.width, F = l.hidden;
      if (li == 1 && sp.vocab > 0) W("emb", {sp.vocab, d}, 0.02f);
      O("ln1.g", d); Z("ln1.b", d);
      W("wqkv", {3 * d, d}, 0.02f); Z("bqkv", 3 * d);
      W("wo", {d, d}, 0.02f); Z("bo", d);
      O("ln2.g", d); Z("ln2.b", d);
      W("w1", {F, d}, 0.02f); Z("b1", F);
      W("w2", {d, F}, 0.02f); Z("b2", d);
    } else {
      int64_t co = l.out_ch;
      if (l.has_stem) { W("stem.w", {co, 3, 3, l.in_ch}, kaiming(9 * l.in_ch)); O("stem.bn.g", co); Z("stem.bn.b", co); }
      for (int b = 0; b < l.n_basic_blocks; ++b) {
        std::string q = "b" + std::to_string(b + 1) + ".";
        int64_t cin = (l.has_stem || b > 0) ? co : l.in_ch;
        W((q + "conv1.w").c_str(), {co, 3, 3, cin}, kaiming(9 * cin)); O((q + "bn1.g").c_str(), co); Z((q + "bn1.b").c_str(), co);
        W((q + "conv2.w").c_str(), {co, 3, 3, co}, kaiming(9 * co)); O((q + "bn2.g").c_str(), co); Z((q + "bn2.b").c_str(), co);
        if (b == 0 && !l.has_stem && (l.stride != 1 || cin != co)) {
          W((q + "proj.w").c_str(), {co, 1, 1, cin}, kaiming(cin)); O((q + "proj.bn.g").c_str(), co); Z((q + "proj.bn.b").c_str(), co);
        }
      }
    }
    S.p_end = c->P;
  }
  c->heads.assign(sp.n_heads, HeadState());
  for (int hi = 0; hi < sp.n_heads; ++hi) {
    HeadState& Hd = c->heads[hi];
    Hd.s = c->head_specs[hi];
    Hd.e = Hd.s.after_layer;
    Hd.s_lo = Hd.e - Hd.s.window < 0 ? 0 : Hd.e - Hd.s.window;
    Hd.p_begin = c->P;
    std::string p = "H" + std::to_string(hi + 1) + ".";
    int owner = L + hi + 1;
    bool vocab_head = Hd.s.kind == LP_HEAD_LN_LINEAR_CE;
    if (vocab_head) {
      Hd.t["ln.g"] = add_tensor(c, p + "ln.g", {Hd.s.in_dim}, owner, 1, 0.f);
      Hd.t["ln.b"] = add_tensor(c, p + "ln.b", {Hd.s.in_dim}, owner, 2, 0.f);
    }
    if (Hd.s.kind == LP_HEAD_BN_POOL_LINEAR_CE) {
      Hd.t["bn.g"] = add_tensor(c, p + "bn.g", {Hd.s.in_dim}, owner, 1, 0.f);
      Hd.t["bn.b"] = add_tensor(c, p + "bn.b", {Hd.s.in_dim}, owner, 2, 0.f);
    }
    float std = vocab_head ? 0.02f : (float)sqrt(2.0 / (double)Hd.s.in_dim);
    Hd.t["w"] = add_tensor(c, p + "w", {Hd.s.n_classes, Hd.s.in_dim}, owner, 0, std);
    if (Hd.s.bias) Hd.t["b"] = add_tensor(c, p + "b", {Hd.s.n_classes}, owner, 2, 0.f);
    Hd.p_end = c->P;
    for (int li = Hd.s_lo + 1; li <= Hd.e; ++li) c->layers[li].coverage++;
  }
}

static ConvUnit make_unit(lp_ctx* c, const std::string& wname, const std::string& bnpre, int N, int H, int C, int O,
                          int R, int stride, int pad, int relu) {
  ConvUnit u;
  u.a.N = N; u.a.H = H; u.a.W = H; u.a.C = C; u.a.O = O; u.a.R = R; u.a.S = R; u.a.stride = stride; u.a.pad = pad;
  u.a.P = (H + 2 * pad - R) / stride + 1; u.a.Q = u.a.P;
  u.w = c->index[wname]; u.g = c->index[bnpre + "g"]; u.b = c->index[bnpre + "b"];
  u.relu = relu;
  return u;
}

static bool no_linearity() {     // LP_NO_LINEARITY=1: every head runs its own full backward pass (for measurements)
  static int v = -1;
  if (v < 0) { const char* s = getenv("LP_NO_LINEARITY"); v = (s && s[0] == '1') ? 1 : 0; }
  return v != 0;
}

// Assigns every work / params / state region.  With null bases it only measures.
static void plan(lp_ctx* c, const lp_buffers* buf, lp_sizes* sizes) {
  const lp_model_spec& sp = c->spec;
  int dt = c->dt, B = sp.max_batch, L = sp.n_layers;
  size_t es = dtype_size(dt);
  Arena pa, sa, wa;
  if (buf) { pa.base = (char*)buf->params_dev; sa.base = (char*)buf->state_dev; wa.base = (char*)buf->work_dev; }
  c->master = (float*)pa.take(c->P * 4);
  c->lowp = dt == BF16 ? pa.take(c->P * 2) : nullptr;
  c->mom = sp.opt.kind >= LP_OPT_SGDM ? (float*)sa.take(c->P * 4) : nullptr;
  c->var = sp.opt.kind == LP_OPT_ADAM ? (float*)sa.take(c->P * 4) : nullptr;
  // running mean and variance of every batch normalisation (found by its gain tensor "...bn*.g")
  c->run_off.assign(c->tensors.size(), -1);
  c->bn_run_elems = 0;
  for (size_t i = 0; i < c->tensors.size(); ++i) {
    const std::string& n = c->tensors[i].name;
    if (n.size() < 2 || n.compare(n.size() - 2, 2, ".g") != 0) continue;
    size_t dot = n.rfind('.', n.size() - 3);
    if (n.compare(dot + 1, 2, "bn") != 0) continue;
    c->run_off[i] = (long)c->bn_run_elems;
    c->bn_run_elems += 2 * ((c->tensors[i].numel + 63) & ~(size_t)63);
  }
  c->bn_run = c->bn_run_elems ? (float*)sa.take(c->bn_run_elems * 4) : nullptr;
  if (sa.used == 0) sa.take(256);
  c->grads = (float*)wa.take(c->P * 4);

  size_t partial = 4096, max_rows = (size_t)B, max_act = 0, max_head_logits = 0, max_feat = 0;
  int kind0 = sp.layers[0].kind;
  for (int li = 1; li <= L; ++li) {
    LayerState& S = c->layers[li];
    const lp_layer_spec& l = S.s;
    if (l.kind != LP_LAYER_RESNET_STAGE) S.out = wa.take(layer_out_elems(l, B) * es);
    S.gsum = nullptr;
    if (l.kind != LP_LAYER_RESNET_STAGE && S.coverage > 1 && sp.schedule == LP_SCHED_SYNC && !no_linearity())
      S.gsum = wa.take(layer_out_elems(l, B) * es);
    if (l.kind == LP_LAYER_RESMLP) {
      S.mlp_p = l.in_dim != l.width ? wa.take((size_t)B * l.width * es) : nullptr;
      S.mlp_r = wa.take((size_t)B * l.hidden * es);
      size_t w = l.hidden > l.width ? l.hidden : l.width;
      if (w < (size_t)l.in_dim) w = l.in_dim;
      if ((size_t)B * w > max_act) max_act = (size_t)B * w;
      size_t pr = (size_t)((B + 127) / 128) * w;
      if (pr > partial) partial = pr;
    } else if (l.kind == LP_LAYER_DECODER) {
      size_t T = (size_t)B * l.seq_len, d = l.width, F = l.hidden;
      S.a = wa.take(T * d * es); S.qkv = wa.take(T * 3 * d * es); S.o = wa.take(T * d * es);
      S.u = wa.take(T * d * es); S.c = wa.take(T * d * es);
      S.fpre = wa.take(T * F * es); S.f = wa.take(T * F * es);
      S.mean1 = (float*)wa.take(T * 4); S.rstd1 = (float*)wa.take(T * 4);
      S.mean2 = (float*)wa.take(T * 4); S.rstd2 = (float*)wa.take(T * 4);
      S.lse = (float*)wa.take(T * l.n_heads * 4);
      if (T > max_rows) max_rows = T;
      size_t widest = F > 3 * d ? F : 3 * d;
      size_t pr = ((T + 7) / 8) * d * 2;      // LayerNorm backward: dg and db partials of every 8-row block
      size_t pc = ((T + 127) / 128) * (widest > (size_t)sp.vocab ? widest : (size_t)sp.vocab);
      size_t pb = ((T + 127) / 128) * (F + 5 * d);   // the four bias gradients' partial tables side by side
      if (pr > partial) partial = pr;
      if (pc > partial) partial = pc;
      if (pb > partial) partial = pb;
    } else {
      int hw_in = l.in_hw, hw_out = l.in_hw / l.stride;
      std::string p = "L" + std::to_string(li) + ".";
      auto alloc_unit = [&](ConvUnit& u) {
        size_t n = (size_t)B * u.a.P * u.a.Q * u.a.O;
        u.z = wa.take(n * es); u.y = wa.take(n * es);
        u.mean = (float*)wa.take((size_t)u.a.O * 4); u.rstd = (float*)wa.take((size_t)u.a.O * 4);
        size_t nin = (size_t)B * u.a.H * u.a.W * u.a.C;
        if (n > max_act) max_act = n;
        if (nin > max_act) max_act = nin;
        if (sp.debug) { u.dy_keep = wa.take(n * es); u.dx_keep = wa.take(nin * es); }
        size_t pr = (size_t)(2 * 1024 + 2) * u.a.O;   // up to 1024 row slabs, two sums each, plus the totals
        if (pr > partial) partial = pr;
        size_t ps = 3 * (n / 32 + u.a.O);              // statistics left by the convolution: three per 32-row sub-tile and column
        if (ps > partial) partial = ps;
      };
      S.has_stem = l.has_stem != 0;
      S.blocks.clear();
      if (S.has_stem) {
        S.stem = make_unit(c, p + "stem.w", p + "stem.bn.", B, hw_in, l.in_ch, l.out_ch, 3, 1, 1, 1);
        alloc_unit(S.stem);
        c->units[p + "stem"] = {li, 0, 0};
      }
      for (int b = 0; b < l.n_basic_blocks; ++b) {
        std::string q = p + "b" + std::to_string(b + 1) + ".";
        bool first = (b == 0 && !S.has_stem);
        int cin = first ? l.in_ch : l.out_ch;
        int stride = first ? l.stride : 1;
        int hin = first ? hw_in : hw_out;
        BasicBlock bb;
        bb.c1 = make_unit(c, q + "conv1.w", q + "bn1.", B, hin, cin, l.out_ch, 3, stride, 1, 1);
        bb.c2 = make_unit(c, q + "conv2.w", q + "bn2.", B, hw_out, l.out_ch, l.out_ch, 3, 1, 1, 1);
        bb.has_proj = c->index.count(q + "proj.w") > 0;
        if (bb.has_proj) bb.proj = make_unit(c, q + "proj.w", q + "proj.bn.", B, hin, cin, l.out_ch, 1, stride, 0, 0);
        alloc_unit(bb.c1); alloc_unit(bb.c2);
        if (bb.has_proj) alloc_unit(bb.proj);
        c->units[q + "conv1"] = {li, b, 1};
        c->units[q + "conv2"] = {li, b, 2};
        if (bb.has_proj) c->units[q + "proj"] = {li, b, 3};
        S.blocks.push_back(bb);
      }
      // the stage output is the last block's y; keep `out` as an alias instead of a copy
      S.out = S.blocks.back().c2.y;
    }
  }
  for (auto& Hd : c->heads) {
    const lp_layer_spec& l = c->layers[Hd.e].s;
    size_t rows = kind0 == LP_LAYER_DECODER ? (size_t)B * l.seq_len : (size_t)B;
    if (rows * Hd.s.n_classes > max_head_logits) max_head_logits = rows * Hd.s.n_classes;
    if (rows * Hd.s.in_dim > max_feat) max_feat = rows * Hd.s.in_dim;
    if (rows > max_rows) max_rows = rows;
    if ((size_t)Hd.s.in_dim > max_rows) max_rows = Hd.s.in_dim;      // per-channel statistics of a BatchNorm head
    size_t pc = ((rows + 127) / 128) * (size_t)(Hd.s.n_classes > Hd.s.in_dim ? Hd.s.n_classes : Hd.s.in_dim);
    if (pc > partial) partial = pc;
  }
  if (kind0 == LP_LAYER_DECODER) {
    const lp_layer_spec& l = sp.layers[0];
    c->pe = (float*)wa.take((size_t)l.seq_len * l.width * 4);
    c->h0 = wa.take((size_t)B * l.seq_len * l.width * es);
  }
  // transposed bf16 copies of the vocabulary heads' weights (see lp_ctx::wt)
  c->wt.assign(c->tensors.size(), nullptr);
  if (dt == BF16)
    for (auto& Hd : c->heads)
      if (Hd.s.kind == LP_HEAD_LN_LINEAR_CE && Hd.t.count("w")) {
        const Tensor& w = c->tensors[Hd.t["w"]];
        if (w.shape[0] % 8 == 0 && w.shape[1] % 8 == 0) c->wt[Hd.t["w"]] = wa.take(w.numel * 2);
      }
  if (sp.schedule != LP_SCHED_SYNC) {
    const int J = sp.n_heads;
    c->label_elems_per_sample = kind0 == LP_LAYER_DECODER ? (size_t)sp.layers[0].seq_len : 1;
    c->stash_act.assign(J + 1, nullptr);
    c->ybuf.assign(J + 1, nullptr);
    for (int j = 1; j <= J; ++j) {
      if (j >= 2) c->stash_act[j] = wa.take(layer_out_elems(c->layers[c->heads[j - 2].e].s, B) * es);
      c->ybuf[j] = (int32_t*)wa.take((size_t)B * c->label_elems_per_sample * 4);
    }
    c->in_batch.assign(J + 1, 0); c->ran_batch.assign(J + 1, 0); c->blk_updates.assign(J + 1, 0);
  }
  // Grouped pipelined schedule: the blocks are walked in lockstep, stage by stage, so that their same-shaped GEMMs
  // share grouped launches; every block then needs a scratch set of its own.
  c->lockstep = sp.schedule == LP_SCHED_PIPELINED_GROUPED;
  // one scratch set for the caller's stream and one per side stream
  c->n_side = sp.n_streams;
  int nsets = 1 + c->n_side;
  if (c->lockstep && nsets < sp.n_heads) nsets = sp.n_heads;
  c->sets.assign(nsets, lp_scratch());
  for (auto& S : c->sets) {
    S.partial_elems = partial;
    S.partial = (float*)wa.take(partial * 4);
    if (dt == BF16 || kind0 == LP_LAYER_RESNET_STAGE) {   // split-K partial sums
      S.splitk_elems = dt == BF16 ? (size_t)8 * 400 * 128 * 128 : (size_t)1 << 22;
      S.splitk_ws = (float*)wa.take(S.splitk_elems * 4);
    }
    S.loss_rows = (float*)wa.take(max_rows * 4);
    S.feat = wa.take(max_feat * es);
    S.dfeat = wa.take(max_feat * es);
    S.logits = wa.take(max_head_logits * es);
    S.hmean = (float*)wa.take(max_rows * 4);
    S.hrstd = (float*)wa.take(max_rows * 4);
    if (kind0 == LP_LAYER_DECODER) {
      const lp_layer_spec& l = sp.layers[0];
      size_t T = (size_t)B * l.seq_len, d = l.width, F = l.hidden;
      S.dA = wa.take(T * d * es); S.dB = wa.take(T * d * es);
      S.dF = wa.take(T * F * es); S.dc = wa.take(T * d * es); S.du = wa.take(T * d * es);
      S.dO = wa.take(T * d * es); S.dqkv = wa.take(T * 3 * d * es); S.da = wa.take(T * d * es);
      S.delta = (float*)wa.take(T * l.n_heads * 4);
    } else if (kind0 == LP_LAYER_RESMLP) {
      S.dA = wa.take(max_act * es); S.dB = wa.take(max_act * es);
      S.dF = wa.take(max_act * es); S.dc = wa.take(max_act * es);
    } else {
      S.dA = wa.take(max_act * es); S.dB = wa.take(max_act * es);
      S.sG = wa.take(max_act * es); S.sZ = wa.take(max_act * es); S.sR = wa.take(max_act * es);
      S.sD1 = wa.take(max_act * es); S.sD2 = wa.take(max_act * es);
    }
  }
  c->use(0);
  if (sizes) {
    sizes->param_bytes = (pa.used + 255) & ~(size_t)255;
    sizes->state_bytes = (sa.used + 255) & ~(size_t)255;
    sizes->work_bytes = (wa.used + 255) & ~(size_t)255;
  }
}

static lp_ctx* make_host_ctx(const lp_model_spec* sp) {
  lp_ctx* c = new lp_ctx();
  c->spec = *sp;
  c->layer_specs.assign(sp->layers, sp->layers + sp->n_layers);
  c->head_specs.assign(sp->heads, sp->heads + sp->n_heads);
  c->spec.layers = c->layer_specs.data();
  c->spec.heads = c->head_specs.data();
  c->dt = sp->dtype;
  build_params(c);
  return c;
}

extern "C" int lp_query_sizes(const lp_model_spec* spec, lp_sizes* out) {
  std::string err;
  int st = validate(spec, err);
  if (st != LP_OK) return fail(nullptr, st, err);
  if (!out) return fail(nullptr, LP_EINVAL, "out is null");
  lp_ctx* c = make_host_ctx(spec);
  plan(c, nullptr, out);
  delete c;
  return LP_OK;
}

#define CK(expr)                                                                                 \
  do {                                                                                           \
    hipError_t e_ = (expr);                                                                      \
    if (e_ != hipSuccess) return fail(c, LP_EDEVICE, std::string(#expr) + ": " + hipGetErrorString(e_)); \
  } while (0)

// Brings the transposed copies of the weights inside parameter range [off, off + n) up to date with the bf16
// working copy, on the current stream.
static int refresh_wt(lp_ctx* c, size_t off, size_t n) {
  for (size_t ti = 0; ti < c->wt.size(); ++ti) {
    const Tensor& t = c->tensors[ti];
    if (!c->wt[ti] || t.off < off || t.off >= off + n) continue;
    CK(op_transpose_bf16(c->op(), c->W((int)ti), c->wt[ti], (int)t.shape[0], (int)t.shape[1]));
  }
  return LP_OK;
}
static int refresh_lowp(lp_ctx* c, size_t off, size_t n) {
  if (c->dt != BF16) return LP_OK;
  CK(op_cast_to_compute(c->op(), c->master + off, (bf16_t*)c->lowp + off, n));
  return refresh_wt(c, off, n);
}

extern "C" int lp_init_blocks(const lp_model_spec* spec, const lp_buffers* buffers, void* hip_stream, lp_ctx** out) {
  if (out) *out = nullptr;
  std::string err;
  int st = validate(spec, err);
  if (st != LP_OK) return fail(nullptr, st, err);
  if (!out) return fail(nullptr, LP_EINVAL, "out is null");
  if (!buffers || !buffers->params_dev || !buffers->state_dev || !buffers->work_dev)
    return fail(nullptr, LP_EINVAL, "buffers (params, state, work) must be non-null");
  if (((uintptr_t)buffers->params_dev | (uintptr_t)buffers->state_dev | (uintptr_t)buffers->work_dev) & 255)
    return fail(nullptr, LP_EALIGN, "device buffers must be 256-byte aligned");
  lp_ctx* c = make_host_ctx(spec);
  c->stream = (hipStream_t)hip_stream;
  lp_sizes sz;
  plan(c, buffers, &sz);
  auto bail = [&](int code) { g_init_err = c->err; delete c; return code; };
  // the caller vouches for the sizes; probe that the last byte of each buffer is device memory
  {
    struct { const void* p; size_t n; const char* what; } bufs[3] = {
        {buffers->params_dev, sz.param_bytes, "params"}, {buffers->state_dev, sz.state_bytes, "state"},
        {buffers->work_dev, sz.work_bytes, "work"}};
    for (auto& b : bufs) {
      void* base = nullptr; size_t len = 0;
      hipError_t e = hipMemGetAddressRange((hipDeviceptr_t*)&base, &len, (hipDeviceptr_t)b.p);
      if (e != hipSuccess) { c->err = std::string(b.what) + " buffer is not device memory: " + hipGetErrorString(e); (void)hipGetLastError(); return bail(LP_EDEVICE); }
      size_t avail = len - ((const char*)b.p - (const char*)base);
      if (avail < b.n) { c->err = std::string(b.what) + " buffer too small: have " + std::to_string(avail) + " bytes, need " + std::to_string(b.n); return bail(LP_ENOMEM); }
    }
  }
  // streams and events
  c->sets[0].cur_stream = c->stream;
  {
    hipError_t es_ = hipSuccess;
    for (int i = 1; i <= c->n_side && es_ == hipSuccess; ++i)
      es_ = hipStreamCreateWithFlags(&c->sets[i].cur_stream, hipStreamNonBlocking);
    int L = spec->n_layers, J = spec->n_heads;
    c->ev_fwd.assign(L + 1, nullptr); c->ev_contrib.assign(L + 1, nullptr); c->ev_chain.assign(J, nullptr);
    if (c->n_side > 0) {
      for (auto* v : {&c->ev_fwd, &c->ev_contrib, &c->ev_chain})
        for (auto& ev : *v)
          if (es_ == hipSuccess) es_ = hipEventCreateWithFlags(&ev, hipEventDisableTiming);
      if (es_ == hipSuccess) es_ = hipEventCreateWithFlags(&c->ev_pipe, hipEventDisableTiming);
    }
    if (es_ != hipSuccess) { c->err = std::string("stream/event creation: ") + hipGetErrorString(es_); return bail(LP_EDEVICE); }
  }
  c->use(0);
  OpCtx o = c->op();
  hipError_t e;
#define CKI(expr) do { e = (expr); if (e != hipSuccess) { c->err = std::string(#expr) + ": " + hipGetErrorString(e); return bail(LP_EDEVICE); } } while (0)
  CKI(op_fill_f32(o, c->master, c->P, 0.f));
  if (c->mom) CKI(op_fill_f32(o, c->mom, c->P, 0.f));
  if (c->var) CKI(op_fill_f32(o, c->var, c->P, 0.f));
  CKI(op_fill_f32(o, c->grads, c->P, 0.f));
  for (size_t i = 0; i < c->run_off.size(); ++i)
    if (c->bn_run && c->run_off[i] >= 0) {   // mean 0, variance 1
      const size_t C = c->tensors[i].numel;
      CKI(op_fill_f32(o, c->bn_run + c->run_off[i], C, 0.f));
      CKI(op_fill_f32(o, c->bn_run + c->run_off[i] + C, C, 1.f));
    }
  for (size_t i = 0; i < c->tensors.size(); ++i) {
    const Tensor& t = c->tensors[i];
    if (t.init == 0) CKI(op_init_normal(o, c->master + t.off, t.numel, t.std, spec->seed, (uint64_t)i));
    else if (t.init == 1) CKI(op_fill_f32(o, c->master + t.off, t.numel, 1.f));
  }
  if (c->dt == BF16) {
    CKI(op_cast_to_compute(o, c->master, c->lowp, c->P));
    for (size_t ti = 0; ti < c->wt.size(); ++ti)
      if (c->wt[ti]) CKI(op_transpose_bf16(o, c->W((int)ti), c->wt[ti], (int)c->tensors[ti].shape[0], (int)c->tensors[ti].shape[1]));
  }
  if (c->pe) CKI(op_posenc_init(o, c->pe, spec->layers[0].seq_len, spec->layers[0].width));
  CKI(hipStreamSynchronize(c->stream));
#undef CKI
  c->ok = true;
  *out = c;
  return LP_OK;
}

static void prof_free(lp_ctx* c) {
  for (int i = 0; i < c->prof.cap; ++i) { (void)hipEventDestroy(c->prof.pairs[i].a); (void)hipEventDestroy(c->prof.pairs[i].b); }
  delete[] c->prof.pairs;
  c->prof.pairs = nullptr; c->prof.cap = 0; c->prof.used = 0;
}
// Folds finished event pairs into the per-class totals.
static int prof_collect(lp_ctx* c) {
  { int sj = join_pending(c); if (sj != LP_OK) return sj; }
  if (c->prof.used == 0) return LP_OK;
  CK(hipStreamSynchronize(c->stream));
  for (int i = 0; i < c->prof.used; ++i) {
    float ms = 0.f;
    CK(hipEventElapsedTime(&ms, c->prof.pairs[i].a, c->prof.pairs[i].b));
    c->prof.total_ms[c->prof.pairs[i].kc] += ms;
    if (c->prof.pairs[i].tag) { auto& t = c->prof.by_shape[c->prof.pairs[i].tag]; t.ms += ms; t.n += 1; }
    if (c->prof.pairs[i].kname) {
      auto& t = c->prof.by_kernel[c->prof.pairs[i].kname];
      t.ms += ms; t.n += 1; t.flops += c->prof.pairs[i].flops;
    }
  }
  c->prof.used = 0;
  return LP_OK;
}

extern "C" int lp_profile_enable(lp_ctx* c, int on) {
  if (!c) return LP_EINVAL;
  if (!c->ok) return fail(c, LP_ESTATE, "context is not usable");
  { int sj = join_pending(c); if (sj != LP_OK) return sj; }
  if (on && !c->prof.pairs) {
    const int cap = 8192;
    c->prof.pairs = new Profiler::Pair[cap];
    for (int i = 0; i < cap; ++i) {
      CK(hipEventCreate(&c->prof.pairs[i].a));
      CK(hipEventCreate(&c->prof.pairs[i].b));
      c->prof.cap = i + 1;
    }
  }
  if (on) {
    int st = prof_collect(c);
    if (st != LP_OK) return st;
    for (int k = 0; k < KC_COUNT; ++k) { c->prof.total_ms[k] = 0; c->prof.launches[k] = 0; c->prof.flops[k] = 0; }
    c->prof.dropped = 0;
    c->prof.by_shape.clear();
    c->prof.by_kernel.clear();
  }
  c->prof.on = on != 0;
  return LP_OK;
}

extern "C" int lp_profile_read(lp_ctx* c, int kernel_class, double* total_ms, long long* launches, double* flops) {
  if (!c) return LP_EINVAL;
  if (kernel_class < 0 || kernel_class >= KC_COUNT) return fail(c, LP_EINVAL, "bad kernel class");
  int st = prof_collect(c);
  if (st != LP_OK) return st;
  if (c->prof.dropped) return fail(c, LP_ESTATE, "event pool overflowed: read the profile after every step");
  if (total_ms) *total_ms = c->prof.total_ms[kernel_class];
  if (launches) *launches = c->prof.launches[kernel_class];
  if (flops) *flops = c->prof.flops[kernel_class];
  return LP_OK;
}

extern "C" int lp_profile_gemm_shapes(lp_ctx* c, char* out, size_t cap) {
  if (!c) return LP_EINVAL;
  if (!out || cap == 0) return fail(c, LP_EINVAL, "out is null or empty");
  int st = prof_collect(c);
  if (st != LP_OK) return st;
  std::string text;
  for (const auto& kv : c->prof.by_shape) {
    const uint64_t t = kv.first;
    char line[160];
    snprintf(line, sizeof line, "%d %d %d %d %d %d %lld %.6f\n", (int)(t & 0xfffff), (int)(t >> 20 & 0xfffff),
             (int)(t >> 40 & 0xfffff), (int)(t >> 60 & 1), (int)(t >> 61 & 1), (int)(t >> 62 & 1), kv.second.n, kv.second.ms);
    text += line;
  }
  if (text.size() + 1 > cap) return fail(c, LP_ESHAPE, "buffer too small for the shape table");
  memcpy(out, text.c_str(), text.size() + 1);
  return LP_OK;
}

extern "C" int lp_profile_gemm_kernels(lp_ctx* c, char* out, size_t cap) {
  if (!c) return LP_EINVAL;
  if (!out || cap == 0) return fail(c, LP_EINVAL, "out is null or empty");
  int st = prof_collect(c);
  if (st != LP_OK) return st;
  std::string text;
  for (const auto& kv : c->prof.by_kernel) {
    char line[96];
    snprintf(line, sizeof line, "\t%lld\t%.6f\t%.6e\n", kv.second.n, kv.second.ms, kv.second.flops);
    text += kv.first + line;
  }
  if (text.size() + 1 > cap) return fail(c, LP_ESHAPE, "buffer too small for the kernel table");
  memcpy(out, text.c_str(), text.size() + 1);
  return LP_OK;
}

extern "C" void lp_destroy(lp_ctx* c) {
  if (!c) return;
  for (size_t i = 1; i < c->sets.size(); ++i)
    if (c->sets[i].cur_stream) { (void)hipStreamSynchronize(c->sets[i].cur_stream); (void)hipStreamDestroy(c->sets[i].cur_stream); }
  for (auto* v : {&c->ev_fwd, &c->ev_contrib, &c->ev_chain})
    for (auto ev : *v)
      if (ev) (void)hipEventDestroy(ev);
  if (c->ev_pipe) (void)hipEventDestroy(c->ev_pipe);
  if (c->gexec) (void)hipGraphExecDestroy(c->gexec);
  if (c->gstream) (void)hipStreamDestroy(c->gstream);
  prof_free(c);
  delete c;
}

extern "C" const char* lp_last_error(const lp_ctx* c) { return c ? c->err.c_str() : g_init_err.c_str(); }

// ------------------------------------------------------------------------------------- step / eval
// Makes the caller's stream wait for every chain a previous overlapped step left running.
static int join_pending(lp_ctx* c) {
  if (!c->pending_join) return LP_OK;
  for (auto ev : c->ev_chain)
    if (ev) CK(hipStreamWaitEvent(c->stream, ev, 0));
  c->pending_join = false;
  return LP_OK;
}

static int check_call(lp_ctx* c, const void* x, const int32_t* y, int batch, float* losses) {
  if (!c) return LP_EINVAL;
  if (!c->ok) return fail(c, LP_ESTATE, "context is not usable");
  if (!x || !y || !losses) return fail(c, LP_EINVAL, "x_dev, y_dev and losses_dev must be non-null");
  if (batch < 0 || batch > c->spec.max_batch)
    return fail(c, LP_ESHAPE, "batch " + std::to_string(batch) + " outside [0, max_batch=" + std::to_string(c->spec.max_batch) + "]");
  return LP_OK;
}

static int optimizer_range(lp_ctx* c, size_t b, size_t e, float grad_scale, int t = -1) {
  OptArgs a;
  const lp_opt_spec& s = c->spec.opt;
  a.kind = s.kind; a.lr = s.lr; a.momentum = s.momentum; a.beta1 = s.beta1; a.beta2 = s.beta2; a.eps = s.eps;
  a.weight_decay = s.weight_decay; a.t = t >= 0 ? t : c->step_t; a.grad_scale = grad_scale;
  CK(op_optimizer(c->op(), a, c->master + b, c->grads + b, c->mom ? c->mom + b : nullptr,
                  c->var ? c->var + b : nullptr, c->lowp ? (void*)((bf16_t*)c->lowp + b) : nullptr, e - b));
  return c->lowp ? refresh_wt(c, b, e - b) : LP_OK;      // behind the update, on the same stream
}

// Launches the products collected from one stage of several blocks, at most 16 to a grouped launch.
static int launch_collected(lp_ctx* c, std::vector<GemmArgs>& v) {
  for (size_t i = 0; i < v.size(); i += 16) {
    const int n = (int)(v.size() - i < 16 ? v.size() - i : 16);
    CK(op_gemm_grouped(c->op(), v.data() + i, n));
  }
  v.clear();
  return LP_OK;
}

// The blocks of a pipelined call in lockstep (decoder blocks of equal depth): within a call the blocks are
// independent (section 6), so stage s of every block of a team runs before stage s + 1 of any, and the GEMMs that
// a stage hands back, one per block and of one shape, go out as one grouped launch.  With side streams the active
// blocks form two teams on two streams: while one team's memory-bound kernels (normalisation, cross-entropy,
// attention, column sums) run, the other team's grouped GEMM has the matrix cores.  Block j works in scratch
// set j - 1.
static int run_lockstep(lp_ctx* c, const int32_t* ids, float* losses) {
  const int J = c->spec.n_heads, nl = c->heads[0].e - c->heads[0].s_lo;
  std::vector<int> act;
  for (int j = 1; j <= J; ++j) {
    c->ran_batch[j] = c->in_batch[j];
    if (c->in_batch[j] > 0) act.push_back(j);
  }
  // the teams (and with them the composition of every grouped launch, i.e. the order of every sum) do not depend
  // on the number of streams: results are bit-identical with and without side streams
  const int n_teams = act.size() >= 2 ? 2 : 1;
  const bool two_streams = n_teams == 2 && c->n_side >= 2 && !c->prof.on;
  std::vector<int> team[2];
  for (size_t i = 0; i < act.size(); ++i) team[n_teams == 2 ? (int)(i & 1) : 0].push_back(act[i]);
  hipStream_t tstream[2] = {c->stream, c->stream};
  if (two_streams) {
    CK(hipEventRecord(c->ev_pipe, c->stream));
    for (int k = 0; k < 2; ++k) {
      tstream[k] = c->sets[1 + k].cur_stream;
      CK(hipStreamWaitEvent(tstream[k], c->ev_pipe, 0));
    }
  }
  int cur_team = 0;
  auto use_block = [&](int j) { c->use(j - 1); c->cur_stream = tstream[cur_team]; };
  std::vector<GemmArgs> coll;
  StageGemms sg;
  int st;
  for (int j : act)
    if (j >= 2) c->layers[c->heads[j - 1].s_lo + 1].in_override = c->stash_act[j];
  for (int off = 0; off < nl; ++off)
    for (int stage = 0; stage < kDecFwdStages; ++stage)
      for (cur_team = 0; cur_team < n_teams; ++cur_team) {
        for (int j : team[cur_team]) {
          use_block(j);
          if ((st = dec_forward_stage(c, c->heads[j - 1].s_lo + 1 + off, c->in_batch[j], ids, stage, &sg)) != LP_OK) return st;
          coll.insert(coll.end(), sg.g, sg.g + sg.n);
        }
        if ((st = launch_collected(c, coll)) != LP_OK) return st;
      }
  for (int stage = 0; stage < kVocabHeadStages; ++stage)
    for (cur_team = 0; cur_team < n_teams; ++cur_team) {
      for (int j : team[cur_team]) {
        use_block(j);
        if ((st = vocab_head_stage(c, j - 1, c->in_batch[j], c->ybuf[j], losses + (j - 1), true, c->dA, stage, &sg)) != LP_OK) return st;
        coll.insert(coll.end(), sg.g, sg.g + sg.n);
      }
      if ((st = launch_collected(c, coll)) != LP_OK) return st;
    }
  for (int off = nl - 1; off >= 0; --off) {
    const bool flip = ((nl - 1 - off) & 1) != 0;       // the blocks' gradient buffers alternate layer by layer
    for (int stage = 0; stage < kDecBwdStages; ++stage)
      for (cur_team = 0; cur_team < n_teams; ++cur_team) {
        for (int j : team[cur_team]) {
          use_block(j);
          const void* dcur = flip ? c->dB : c->dA;
          void* dnext = flip ? c->dA : c->dB;
          if ((st = dec_backward_stage(c, c->heads[j - 1].s_lo + 1 + off, c->in_batch[j], dcur, dnext, off > 0, 0, ids, true,
                                       stage, &sg)) != LP_OK) return st;
          coll.insert(coll.end(), sg.g, sg.g + sg.n);
        }
        if ((st = launch_collected(c, coll)) != LP_OK) return st;
      }
    for (int j : act) c->layers[c->heads[j - 1].s_lo + 1 + off].seen = 1;
  }
  for (cur_team = 0; cur_team < n_teams; ++cur_team) {
    for (int j : team[cur_team]) {
      use_block(j);
      HeadState& Hd = c->heads[j - 1];
      const int t_blk = ++c->blk_updates[j];          // the block's own number of updates
      if ((st = optimizer_range(c, Hd.p_begin, Hd.p_end, 1.f, t_blk)) != LP_OK) return st;
      for (int lj = Hd.e; lj > Hd.s_lo; --lj)
        if ((st = optimizer_range(c, c->layers[lj].p_begin, c->layers[lj].p_end, 1.f, t_blk)) != LP_OK) return st;
    }
    if (two_streams) {
      CK(hipEventRecord(c->ev_chain[cur_team], tstream[cur_team]));
      CK(hipStreamWaitEvent(c->stream, c->ev_chain[cur_team], 0));
    }
  }
  c->use(0);
  return LP_OK;
}

// One call of the pipelined schedule: first the hand-over on the caller's stream (every block's output of
// the previous call and the labels that go with it move one block forward; the call's labels are kept for
// the following calls), then every block that has an input runs as an independent chain.
static int run_pipelined(lp_ctx* c, const void* x, const int32_t* y, int batch, float* losses) {
  const int J = c->spec.n_heads;
  const size_t es = dtype_size(c->dt), ly = c->label_elems_per_sample * 4;
  c->use(0);
  CK(op_fill_f32(c->op(), losses, (size_t)J, 0.f));
  c->x_in = x;
  c->last_batch = batch;
  c->step_t += 1;
  for (int j = J; j >= 2; --j) {
    const int nb = c->ran_batch[j - 1];            // what block j-1 produced in the previous call
    c->in_batch[j] = nb;
    if (nb == 0) continue;
    const LayerState& src = c->layers[c->heads[j - 2].e];
    CK(hipMemcpyAsync(c->stash_act[j], src.out, layer_out_elems(src.s, nb) * es, hipMemcpyDeviceToDevice, c->stream));
    CK(hipMemcpyAsync(c->ybuf[j], c->ybuf[j - 1], (size_t)nb * ly, hipMemcpyDeviceToDevice, c->stream));
  }
  c->in_batch[1] = batch;
  CK(hipMemcpyAsync(c->ybuf[1], y, (size_t)batch * ly, hipMemcpyDeviceToDevice, c->stream));
  const int32_t* ids = c->spec.vocab > 0 ? (const int32_t*)x : nullptr;
  for (int li = 1; li <= c->spec.n_layers; ++li) { c->layers[li].seen = 0; c->layers[li].in_override = nullptr; }
  if (c->lockstep) return run_lockstep(c, ids, losses);
  const bool side = c->n_side > 0 && !c->prof.on;
  if (side) CK(hipEventRecord(c->ev_pipe, c->stream));
  int chain = 0, st;
  for (int j = 1; j <= J; ++j) {
    const int nb = c->in_batch[j];
    c->ran_batch[j] = nb;
    if (nb == 0) continue;
    HeadState& Hd = c->heads[j - 1];
    const int set = side ? 1 + (chain++ % c->n_side) : 0;
    c->use(set);
    if (set) CK(hipStreamWaitEvent(c->cur_stream, c->ev_pipe, 0));
    if (j >= 2) c->layers[Hd.s_lo + 1].in_override = c->stash_act[j];
    for (int li = Hd.s_lo + 1; li <= Hd.e; ++li)
      if ((st = drv_forward(c, li, nb, ids)) != LP_OK) return st;
    if ((st = drv_head(c, j - 1, nb, c->ybuf[j], losses + (j - 1), true, c->dA)) != LP_OK) return st;
    void* dcur = c->dA; void* dnext = c->dB;
    for (int lj = Hd.e; lj > Hd.s_lo; --lj) {
      if ((st = drv_backward(c, lj, nb, dcur, dnext, lj > Hd.s_lo + 1, 0)) != LP_OK) return st;
      c->layers[lj].seen = 1;
      void* t = dcur; dcur = dnext; dnext = t;
    }
    const int t_blk = ++c->blk_updates[j];          // the block's own number of updates
    if ((st = optimizer_range(c, Hd.p_begin, Hd.p_end, 1.f, t_blk)) != LP_OK) return st;
    for (int lj = Hd.e; lj > Hd.s_lo; --lj)
      if ((st = optimizer_range(c, c->layers[lj].p_begin, c->layers[lj].p_end, 1.f, t_blk)) != LP_OK) return st;
    if (set) CK(hipEventRecord(c->ev_chain[j - 1], c->cur_stream));
    else if (side) CK(hipEventRecord(c->ev_chain[j - 1], c->stream));
  }
  c->use(0);
  if (side)
    for (int j = 1; j <= J; ++j)
      if (c->ran_batch[j] > 0) CK(hipStreamWaitEvent(c->stream, c->ev_chain[j - 1], 0));
  return LP_OK;
}

static int run(lp_ctx* c, const void* x, const int32_t* y, int batch, float* losses, bool train) {
  int st = check_call(c, x, y, batch, losses);
  if (st != LP_OK) return st;
  int L = c->spec.n_layers, J = c->spec.n_heads;
  c->bn_mode = train ? (c->bn_momentum > 0.f ? 1 : 0) : (c->bn_eval_running ? 2 : 0);
  // with per-op timing on, everything runs on the caller's stream so that each duration is the op's own
  const bool side = train && c->n_side > 0 && !c->prof.on;
  const bool overlap = side && c->overlap_steps && batch > 0 && c->spec.schedule == LP_SCHED_SYNC;
  if (!overlap && (st = join_pending(c)) != LP_OK) return st;
  if (train && batch > 0 && c->spec.schedule != LP_SCHED_SYNC) return run_pipelined(c, x, y, batch, losses);
  for (int li = 1; li <= L; ++li) c->layers[li].in_override = nullptr;
  if (batch == 0) {
    CK(op_fill_f32(c->op(), losses, (size_t)J, 0.f));
    return LP_OK;
  }
  c->x_in = x;
  c->last_batch = batch;
  if (train) {
    c->step_t += 1;
    for (int li = 1; li <= L; ++li) c->layers[li].seen = 0;
  }
  const int32_t* ids = c->spec.vocab > 0 ? (const int32_t*)x : nullptr;
  int hj = 0, chain = 0;
  c->use(0);
  for (int li = 1; li <= L; ++li) {
    c->use(0);
    if (c->pending_join) {
      // the previous step's chains may still run: this layer's forward pass overwrites what the chains of the
      // heads whose window covers the layer read (saved activations) and update (its weights), and its output
      // is the saved input of the block that starts after it
      for (int j = 0; j < J; ++j)
        if (c->heads[j].s_lo <= li && li <= c->heads[j].e) CK(hipStreamWaitEvent(c->stream, c->ev_chain[j], 0));
    }
    if ((st = drv_forward(c, li, batch, ids)) != LP_OK) return st;
    if (side && hj < J && c->heads[hj].e == li) CK(hipEventRecord(c->ev_fwd[li], c->stream));
    // every head attached after this layer runs as soon as the activation exists
    for (; hj < J && c->heads[hj].e == li; ++hj) {
      HeadState& Hd = c->heads[hj];
      const int set = side ? 1 + (chain++ % c->n_side) : 0;
      c->use(set);
      if (set) CK(hipStreamWaitEvent(c->cur_stream, c->ev_fwd[li], 0));
      if ((st = drv_head(c, hj, batch, y, losses + hj, train, c->dA)) != LP_OK) return st;
      if (!train) continue;
      void* dcur = c->dA; void* dnext = c->dB;
      for (int lj = Hd.e; lj > Hd.s_lo; --lj) {
        LayerState& S = c->layers[lj];
        bool need_dx = lj > Hd.s_lo + 1;          // the window input is data: no gradient leaves the window
        // contributions of several heads to one layer keep their order: wait for the previous one
        if (set && S.seen > 0) CK(hipStreamWaitEvent(c->cur_stream, c->ev_contrib[lj], 0));
        if (S.gsum) {
          // A layer inside several windows (appendix A.2 counts a backward pass per head; the parameter gradient is
          // linear in the gradient arriving at the layer's output, so the passes can share their parameter part):
          // every head adds its gradient at this layer's output to the layer's sum, in head order, and continues
          // downwards with an input-gradient-only pass driven by ITS OWN gradient (the sum would carry the other
          // heads' losses beyond their windows); the last head to arrive runs the one parameter pass on the sum.
          const size_t n = layer_out_elems(S.s, batch);
          if (S.seen == 0) CK(hipMemcpyAsync(S.gsum, dcur, n * dtype_size(c->dt), hipMemcpyDeviceToDevice, c->cur_stream));
          else CK(op_add(c->op(), S.gsum, dcur, S.gsum, n));
          S.seen += 1;
          if (set && S.seen < S.coverage) CK(hipEventRecord(c->ev_contrib[lj], c->cur_stream));
          if (need_dx && (st = drv_backward(c, lj, batch, dcur, dnext, true, 0, false)) != LP_OK) return st;
          if (S.seen == S.coverage && (st = drv_backward(c, lj, batch, S.gsum, nullptr, false, 0, true)) != LP_OK) return st;
        } else {
          if ((st = drv_backward(c, lj, batch, dcur, dnext, need_dx, S.seen > 0 ? 1 : 0)) != LP_OK) return st;
          S.seen += 1;
          if (set && S.seen < S.coverage) CK(hipEventRecord(c->ev_contrib[lj], c->cur_stream));
        }
        void* t = dcur; dcur = dnext; dnext = t;
      }
      if ((st = optimizer_range(c, Hd.p_begin, Hd.p_end, 1.f)) != LP_OK) return st;
      // a layer is updated as soon as the last head covering it has contributed
      for (int lj = Hd.e; lj > Hd.s_lo; --lj) {
        LayerState& S = c->layers[lj];
        if (S.seen == S.coverage) {
          float gs = c->spec.combine == LP_COMBINE_MEAN ? 1.f / (float)S.coverage : 1.f;
          if ((st = optimizer_range(c, S.p_begin, S.p_end, gs)) != LP_OK) return st;
        }
      }
      if (set) CK(hipEventRecord(c->ev_chain[hj], c->cur_stream));
    }
  }
  c->use(0);
  if (overlap) {
    c->pending_join = true;        // joined by the next call that is not an overlapped step
  } else if (side) {
    for (int j = 0; j < J; ++j) CK(hipStreamWaitEvent(c->stream, c->ev_chain[j], 0));
    c->pending_join = false;
  }
  return LP_OK;
}

static void drop_graph(lp_ctx* c) {
  if (c->gexec) (void)hipGraphExecDestroy(c->gexec);
  c->gexec = nullptr; c->g_batch = -1; c->g_eager = 0;
}

// A training step through a HIP graph.  The first call with a given (x, y, batch, losses) runs eagerly (it
// also does the one-time kernel attribute set-up), the second is captured from the caller's stream (the
// side streams join the capture through the events they wait on and are joined back by the final waits)
// and launched, later ones replay the graph.  What a step leaves on the host is redone by hand on a replay.
static int run_graph(lp_ctx* c, const void* x, const int32_t* y, int batch, float* losses) {
  int st = check_call(c, x, y, batch, losses);
  if (st != LP_OK) return st;
  if (batch == 0 || c->prof.on) return run(c, x, y, batch, losses, true);
  if (c->gexec && c->g_x == x && c->g_y == y && c->g_batch == batch && c->g_losses == losses) {
    for (int li = 1; li <= c->spec.n_layers; ++li) { c->layers[li].in_override = nullptr; c->layers[li].seen = c->layers[li].coverage; }
    c->x_in = x; c->last_batch = batch; c->step_t += 1;
    CK(hipGraphLaunch(c->gexec, c->stream));
    return LP_OK;
  }
  if (!(c->g_x == x && c->g_y == y && c->g_batch == batch && c->g_losses == losses)) {
    drop_graph(c);
    c->g_x = x; c->g_y = y; c->g_batch = batch; c->g_losses = losses;
  }
  if (c->g_eager++ == 0) return run(c, x, y, batch, losses, true);
  // captured on a stream of the context's own, launched on the caller's
  if (!c->gstream) CK(hipStreamCreateWithFlags(&c->gstream, hipStreamNonBlocking));
  hipStream_t user = c->stream;
  CK(hipStreamBeginCapture(c->gstream, hipStreamCaptureModeThreadLocal));
  c->stream = c->gstream; c->sets[0].cur_stream = c->gstream;
  st = run(c, x, y, batch, losses, true);
  c->stream = user; c->sets[0].cur_stream = user; c->use(0);
  hipGraph_t graph = nullptr;
  hipError_t e = hipStreamEndCapture(c->gstream, &graph);
  if (st != LP_OK) { if (graph) (void)hipGraphDestroy(graph); return st; }
  if (e != hipSuccess || !graph) return fail(c, LP_EDEVICE, std::string("stream capture failed: ") + hipGetErrorString(e));
  e = hipGraphInstantiate(&c->gexec, graph, nullptr, nullptr, 0);
  (void)hipGraphDestroy(graph);
  if (e != hipSuccess) { c->gexec = nullptr; return fail(c, LP_EDEVICE, std::string("graph instantiation failed: ") + hipGetErrorString(e)); }
  CK(hipGraphLaunch(c->gexec, c->stream));
  return LP_OK;
}

extern "C" int lp_step_graph(lp_ctx* c, int on) {
  if (!c) return LP_EINVAL;
  if (!c->ok) return fail(c, LP_ESTATE, "context is not usable");
  if (on && c->spec.opt.kind == LP_OPT_ADAM)
    return fail(c, LP_EINVAL, "graph replay needs an optimizer without per-step scalars (Adam's bias correction changes every step)");
  if (on && c->spec.schedule != LP_SCHED_SYNC)
    return fail(c, LP_EINVAL, "graph replay is for the synchronous schedule");
  if (on && c->overlap_steps) return fail(c, LP_EINVAL, "overlapped steps are not replayed through a graph");
  { int sj = join_pending(c); if (sj != LP_OK) return sj; }
  if (!on) drop_graph(c);
  c->graph_on = on != 0;
  return LP_OK;
}

extern "C" int lp_overlap_steps(lp_ctx* c, int on) {
  if (!c) return LP_EINVAL;
  if (!c->ok) return fail(c, LP_ESTATE, "context is not usable");
  if (on && c->graph_on) return fail(c, LP_EINVAL, "steps replayed through a graph are not overlapped");
  if (on && c->spec.schedule != LP_SCHED_SYNC) return fail(c, LP_EINVAL, "overlapping steps is for the synchronous schedule");
  int st = join_pending(c);
  if (st != LP_OK) return st;
  c->overlap_steps = on != 0;
  return LP_OK;
}

extern "C" int lp_join(lp_ctx* c) {
  if (!c) return LP_EINVAL;
  if (!c->ok) return fail(c, LP_ESTATE, "context is not usable");
  return join_pending(c);
}

extern "C" int lp_bn_running(lp_ctx* c, float momentum, int eval_with_running) {
  if (!c) return LP_EINVAL;
  if (!c->ok) return fail(c, LP_ESTATE, "context is not usable");
  if (!(momentum >= 0.f && momentum <= 1.f)) return fail(c, LP_EINVAL, "momentum must lie in [0, 1]");
  { int sj = join_pending(c); if (sj != LP_OK) return sj; }
  if (momentum != c->bn_momentum) drop_graph(c);   // a captured step has the old weight baked into its launches
  c->bn_momentum = momentum;
  c->bn_eval_running = eval_with_running != 0;
  return LP_OK;
}

extern "C" int lp_local_step(lp_ctx* c, const void* x, const int32_t* y, int batch, float* losses) {
  if (c && c->ok && c->graph_on) return run_graph(c, x, y, batch, losses);
  return run(c, x, y, batch, losses, true);
}
extern "C" int lp_eval_loss(lp_ctx* c, const void* x, const int32_t* y, int batch, float* losses) {
  return run(c, x, y, batch, losses, false);
}

// ------------------------------------------------------------------------------------- tensors
struct Resolved { void* ptr; int dtype; int ndim; int64_t shape[4]; size_t bytes; bool is_param; size_t off; size_t numel; };

static int resolve(lp_ctx* c, const char* name, Resolved* r) {
  if (!c) return LP_EINVAL;
  if (!c->ok) return fail(c, LP_ESTATE, "context is not usable");
  if (!name) return fail(c, LP_EINVAL, "name is null");
  { int sj = join_pending(c); if (sj != LP_OK) return sj; }
  std::string n(name);
  memset(r, 0, sizeof *r);
  auto suffix = [&](const char* s) { size_t k = strlen(s); return n.size() > k && n.compare(n.size() - k, k, s) == 0; };
  if (suffix(".out") && n[0] == 'L') {
    int li = atoi(n.c_str() + 1);
    if (li < 0 || li > c->spec.n_layers || n != "L" + std::to_string(li) + ".out") return fail(c, LP_ENOTFOUND, "no tensor " + n);
    int B = c->last_batch;
    if (li == 0) {
      if (!c->h0) return fail(c, LP_ENOTFOUND, "L0.out exists only for models with an embedding");
      const lp_layer_spec& l = c->layers[1].s;
      r->ptr = c->h0; r->ndim = 2; r->shape[0] = (int64_t)B * l.seq_len; r->shape[1] = l.width;
    } else {
      const lp_layer_spec& l = c->layers[li].s;
      r->ptr = c->layers[li].out;
      if (l.kind == LP_LAYER_RESMLP) { r->ndim = 2; r->shape[0] = B; r->shape[1] = l.width; }
      else if (l.kind == LP_LAYER_DECODER) { r->ndim = 2; r->shape[0] = (int64_t)B * l.seq_len; r->shape[1] = l.width; }
      else { int hw = l.in_hw / l.stride; r->ndim = 4; r->shape[0] = B; r->shape[1] = hw; r->shape[2] = hw; r->shape[3] = l.out_ch; }
    }
    r->dtype = c->dt;
    r->numel = 1;
    for (int i = 0; i < r->ndim; ++i) r->numel *= (size_t)r->shape[i];
    r->bytes = r->numel * dtype_size(c->dt);
    return LP_OK;
  }
  if (suffix(".z") || suffix(".y") || suffix(".dy") || suffix(".dx")) {
    const size_t dot = n.rfind('.');
    auto ui = c->units.find(n.substr(0, dot));
    if (ui != c->units.end()) {
      ConvUnit* u = c->unit(ui->second);
      const std::string leaf = n.substr(dot + 1);
      const int B = c->last_batch;
      const bool in_shaped = leaf == "dx";
      r->ptr = leaf == "z" ? u->z : leaf == "y" ? u->y : leaf == "dy" ? u->dy_keep : (u->dx_valid ? u->dx_keep : nullptr);
      if (!r->ptr) return fail(c, LP_ENOTFOUND, "no tensor " + n + " (debug contexts only; .dx only where the unit computed one)");
      r->ndim = 4; r->shape[0] = B;
      r->shape[1] = in_shaped ? u->a.H : u->a.P; r->shape[2] = in_shaped ? u->a.W : u->a.Q;
      r->shape[3] = in_shaped ? u->a.C : u->a.O;
      r->dtype = c->dt;
      r->numel = (size_t)B * r->shape[1] * r->shape[2] * r->shape[3];
      r->bytes = r->numel * dtype_size(c->dt);
      return LP_OK;
    }
  }
  if (suffix(".running_mean") || suffix(".running_var")) {
    const bool is_var = suffix(".running_var");
    std::string gname = n.substr(0, n.rfind('.')) + ".g";
    auto gi = c->index.find(gname);
    if (gi == c->index.end() || !c->bn_run || c->run_off[gi->second] < 0) return fail(c, LP_ENOTFOUND, "no tensor " + n);
    const Tensor& t = c->tensors[gi->second];
    r->ptr = c->bn_run + c->run_off[gi->second] + (is_var ? t.numel : 0);
    r->dtype = F32; r->ndim = 1; r->shape[0] = (int64_t)t.numel; r->numel = t.numel; r->bytes = t.numel * 4;
    return LP_OK;
  }
  float* base = c->master;
  std::string pn = n;
  bool is_param = true;
  if (suffix(".grad")) { base = c->grads; pn = n.substr(0, n.size() - 5); is_param = false; }
  else if (suffix(".m") && c->index.count(n.substr(0, n.size() - 2))) { base = c->mom; pn = n.substr(0, n.size() - 2); is_param = false; }
  else if (suffix(".v") && c->index.count(n.substr(0, n.size() - 2))) { base = c->var; pn = n.substr(0, n.size() - 2); is_param = false; }
  auto it = c->index.find(pn);
  if (it == c->index.end()) return fail(c, LP_ENOTFOUND, "no tensor " + n);
  if (!base) return fail(c, LP_ENOTFOUND, "this optimizer keeps no " + n);
  const Tensor& t = c->tensors[it->second];
  r->ptr = base + t.off; r->dtype = F32; r->ndim = t.ndim;
  for (int i = 0; i < 4; ++i) r->shape[i] = t.shape[i];
  r->numel = t.numel; r->bytes = t.numel * 4; r->is_param = is_param; r->off = t.off;
  return LP_OK;
}

extern "C" int lp_tensor_info(lp_ctx* c, const char* name, int64_t shape[4], int* ndim, int* dtype, size_t* bytes) {
  Resolved r;
  int st = resolve(c, name, &r);
  if (st != LP_OK) return st;
  if (shape) for (int i = 0; i < 4; ++i) shape[i] = r.shape[i];
  if (ndim) *ndim = r.ndim;
  if (dtype) *dtype = r.dtype;
  if (bytes) *bytes = r.bytes;
  return LP_OK;
}

extern "C" int lp_get_tensor(lp_ctx* c, const char* name, void* dst, size_t bytes) {
  Resolved r;
  int st = resolve(c, name, &r);
  if (st != LP_OK) return st;
  if (!dst) return fail(c, LP_EINVAL, "dst_host is null");
  if (bytes != r.bytes) return fail(c, LP_ESHAPE, std::string(name) + ": have " + std::to_string(r.bytes) + " bytes, caller gave " + std::to_string(bytes));
  if ((st = join_pending(c)) != LP_OK) return st;
  CK(hipStreamSynchronize(c->stream));
  if (bytes) CK(hipMemcpy(dst, r.ptr, bytes, hipMemcpyDeviceToHost));
  return LP_OK;
}

extern "C" int lp_set_tensor(lp_ctx* c, const char* name, const void* src, size_t bytes) {
  Resolved r;
  int st = resolve(c, name, &r);
  if (st != LP_OK) return st;
  if (!src) return fail(c, LP_EINVAL, "src_host is null");
  if (bytes != r.bytes) return fail(c, LP_ESHAPE, std::string(name) + ": have " + std::to_string(r.bytes) + " bytes, caller gave " + std::to_string(bytes));
  if ((st = join_pending(c)) != LP_OK) return st;
  CK(hipStreamSynchronize(c->stream));
  if (bytes) CK(hipMemcpy(r.ptr, src, bytes, hipMemcpyHostToDevice));
  if (r.is_param) {
    if ((st = refresh_lowp(c, r.off, r.numel)) != LP_OK) return st;
    CK(hipStreamSynchronize(c->stream));
  }
  return LP_OK;
}

extern "C" int lp_num_params(lp_ctx* c) { return c ? (int)c->tensors.size() : 0; }
extern "C" const char* lp_param_name(lp_ctx* c, int i) {
  if (!c || i < 0 || i >= (int)c->tensors.size()) return nullptr;
  return c->tensors[i].name.c_str();
}
extern "C" int lp_grad_cosine(lp_ctx* a, lp_ctx* b, float* out_dev) {
  if (!a || !b) return LP_EINVAL;
  lp_ctx* c = a;     // errors are recorded on ctx_a
  if (!a->ok || !b->ok) return fail(a, LP_ESTATE, "context is not usable");
  if (!out_dev) return fail(a, LP_EINVAL, "out_dev is null");
  { int sj = join_pending(a); if (sj != LP_OK) return sj; }
  if (b->pending_join)      // ctx_b's chains run on streams of its own: drain them
    for (size_t i = 1; i < b->sets.size(); ++i)
      if (b->sets[i].cur_stream) CK(hipStreamSynchronize(b->sets[i].cur_stream));
  if (a->spec.n_layers != b->spec.n_layers) return fail(a, LP_ESHAPE, "the two contexts have different numbers of layers");
  for (int li = 1; li <= a->spec.n_layers; ++li)
    if (a->layers[li].p_end - a->layers[li].p_begin != b->layers[li].p_end - b->layers[li].p_begin)
      return fail(a, LP_ESHAPE, "layer " + std::to_string(li) + " has different parameters in the two contexts");
  if (b->stream != a->stream) CK(hipStreamSynchronize(b->stream));     // b's gradients are complete
  a->use(0);
  for (int li = 1; li <= a->spec.n_layers; ++li) {
    const LayerState& A = a->layers[li];
    const LayerState& B = b->layers[li];
    CK(op_cosine(a->op(), a->grads + A.p_begin, b->grads + B.p_begin, A.p_end - A.p_begin, out_dev + (li - 1)));
  }
  return LP_OK;
}

extern "C" int lp_get_step(lp_ctx* c) {
  if (!c) return -1;
  if (c->ok) (void)join_pending(c);
  return c->step_t;
}
extern "C" int lp_set_step(lp_ctx* c, int t) {
  if (!c) return LP_EINVAL;
  if (t < 0) return fail(c, LP_EINVAL, "step must be >= 0");
  if (c->ok) { int sj = join_pending(c); if (sj != LP_OK) return sj; }
  c->step_t = t;
  // pipelined schedule: block j has taken part in every call from the j-th on
  for (size_t j = 1; j < c->blk_updates.size(); ++j) c->blk_updates[j] = t - (int)(j - 1) > 0 ? t - (int)(j - 1) : 0;
  return LP_OK;
}
