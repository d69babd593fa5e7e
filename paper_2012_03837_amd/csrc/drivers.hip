// Layer and head drivers: the sequence of kernel launches for the forward pass of one atomic layer,
// its backward pass inside a truncation window, and an auxiliary head's loss and gradient.
#include "ctx.h"

namespace lp {

#define DO(expr)                                                                           \
  do {                                                                                     \
    hipError_t e_ = (expr);                                                                \
    if (e_ != hipSuccess) {                                                                \
      c->err = std::string(#expr) + ": " + hipGetErrorString(e_);                          \
      return LP_EDEVICE;                                                                   \
    }                                                                                      \
  } while (0)

static inline char* bptr(void* p, size_t elems, int dt) { return (char*)p + elems * dtype_size(dt); }

size_t layer_out_elems(const lp_layer_spec& s, int batch) {
  switch (s.kind) {
    case LP_LAYER_RESMLP: return (size_t)batch * s.width;
    case LP_LAYER_DECODER: return (size_t)batch * s.seq_len * s.width;
    case LP_LAYER_RESNET_STAGE: { int hw = s.in_hw / s.stride; return (size_t)batch * hw * hw * s.out_ch; }
  }
  return 0;
}

static const void* layer_input(lp_ctx* c, int li) {
  if (c->layers[li].in_override) return c->layers[li].in_override;
  if (li == 1) return (c->spec.vocab > 0 && c->layers[1].s.kind == LP_LAYER_DECODER) ? c->h0 : c->x_in;
  return c->layers[li - 1].out;
}

// y = x W^T + b with optional activation / saved pre-activation / residual
static GemmArgs lin_fwd(const lp_ctx* c, const void* x, int rows, int ti_w, int ti_b, void* y) {
  const Tensor& w = c->tensors[ti_w];
  GemmArgs g;
  g.A = x; g.lda = w.shape[1]; g.a_kc = 1;
  g.B = c->W(ti_w); g.ldb = w.shape[1]; g.b_kc = 1;
  g.C = y; g.ldc = w.shape[0];
  g.M = rows; g.N = (int)w.shape[0]; g.K = (int)w.shape[1];
  g.bias = ti_b >= 0 ? c->P32(ti_b) : nullptr;
  return g;
}
// dx = dy W  (W is [out, in]: reduction over `out`, which is W's slow index)
static GemmArgs lin_dgrad(const lp_ctx* c, const void* dy, int rows, int ti_w, void* dx) {
  const Tensor& w = c->tensors[ti_w];
  GemmArgs g;
  g.A = dy; g.lda = w.shape[0]; g.a_kc = 1;
  if (c->wt[ti_w]) { g.B = c->wt[ti_w]; g.ldb = w.shape[0]; g.b_kc = 1; }     // transposed copy [in][out]
  else { g.B = c->W(ti_w); g.ldb = w.shape[1]; g.b_kc = 0; }
  g.C = dx; g.ldc = w.shape[1];
  g.M = rows; g.N = (int)w.shape[1]; g.K = (int)w.shape[0];
  return g;
}
// dW[out, in] (+)= dy^T x   (reduction over rows: the slow index of both operands), fp32 output
static GemmArgs lin_wgrad(const lp_ctx* c, const void* dy, const void* x, int rows, int ti_w, int accumulate) {
  const Tensor& w = c->tensors[ti_w];
  GemmArgs g;
  g.A = dy; g.lda = w.shape[0]; g.a_kc = 0;
  g.B = x; g.ldb = w.shape[1]; g.b_kc = 0;
  g.C = c->G32(ti_w); g.ldc = w.shape[1]; g.c_f32 = 1;
  g.M = (int)w.shape[0]; g.N = (int)w.shape[1]; g.K = rows;
  g.accumulate = accumulate;
  return g;
}

// ===================================================================================== residual MLP
static int mlp_forward(lp_ctx* c, int li, int batch) {
  LayerState& L = c->layers[li];
  OpCtx o = c->op();
  const void* x = layer_input(c, li);
  const void* p = x;
  if (L.t.count("win")) {
    GemmArgs g = lin_fwd(c, x, batch, L.t["win"], L.t["bin"], L.mlp_p);
    DO(op_gemm(o, g));
    p = L.mlp_p;
  }
  GemmArgs g1 = lin_fwd(c, p, batch, L.t["w1"], L.t["b1"], L.mlp_r);
  g1.act = ACT_RELU;
  DO(op_gemm(o, g1));
  GemmArgs g2 = lin_fwd(c, L.mlp_r, batch, L.t["w2"], L.t["b2"], L.out);
  g2.res = p; g2.ldr = L.s.width;
  DO(op_gemm(o, g2));
  return LP_OK;
}

static int mlp_backward(lp_ctx* c, int li, int batch, const void* dout, void* dx, bool need_dx, int acc, bool params) {
  LayerState& L = c->layers[li];
  OpCtx o = c->op();
  const void* x = layer_input(c, li);
  bool proj = L.t.count("win") > 0;
  const void* p = proj ? L.mlp_p : x;
  int width = L.s.width, hidden = L.s.hidden;
  if (params) {
    DO(op_colsum(o, dout, width, c->G32(L.t["b2"]), batch, width, acc));
    DO(op_gemm(o, lin_wgrad(c, dout, L.mlp_r, batch, L.t["w2"], acc)));
  }
  // da = (dout W2) * relu'(r)
  GemmArgs gd = lin_dgrad(c, dout, batch, L.t["w2"], c->dF);
  gd.dact = ACT_RELU; gd.dact_src = L.mlp_r; gd.ldd = hidden;
  DO(op_gemm(o, gd));
  if (params) {
    DO(op_colsum(o, c->dF, hidden, c->G32(L.t["b1"]), batch, hidden, acc));
    DO(op_gemm(o, lin_wgrad(c, c->dF, p, batch, L.t["w1"], acc)));
  }
  if (!need_dx && !(proj && params)) return LP_OK;
  // dp = da W1 + dout
  void* dp = proj ? c->dc : dx;
  GemmArgs g1 = lin_dgrad(c, c->dF, batch, L.t["w1"], dp);
  g1.res = dout; g1.ldr = width;
  DO(op_gemm(o, g1));
  if (proj) {
    if (params) {
      DO(op_colsum(o, dp, width, c->G32(L.t["bin"]), batch, width, acc));
      DO(op_gemm(o, lin_wgrad(c, dp, x, batch, L.t["win"], acc)));
    }
    if (need_dx) DO(op_gemm(o, lin_dgrad(c, dp, batch, L.t["win"], dx)));
  }
  return LP_OK;
}

// ===================================================================================== decoder layer
// The forward and backward passes of a decoder layer are written as STAGES: a stage runs the ops that precede a set
// of mutually independent GEMMs and hands those GEMMs back instead of launching them.  One layer at a time, the
// caller launches them at once (dec_forward / dec_backward below); the pipelined schedule walks the same stage of
// all its blocks before it launches, so the same-shaped products of independent blocks share one grouped launch.
int dec_forward_stage(lp_ctx* c, int li, int batch, const int32_t* ids, int stage, StageGemms* out) {
  LayerState& L = c->layers[li];
  OpCtx o = c->op();
  int S = L.s.seq_len, d = L.s.width, H = L.s.n_heads, T = batch * S;
  out->n = 0;
  if (stage == 0) {
    if (li == 1 && c->spec.vocab > 0 && !L.in_override)
      DO(op_embed_fwd(o, ids, c->P32(L.t["emb"]), c->pe, c->h0, T, S, d, c->spec.vocab));
    const void* x = layer_input(c, li);
    DO(op_layernorm_fwd(o, x, c->P32(L.t["ln1.g"]), c->P32(L.t["ln1.b"]), L.a, L.mean1, L.rstd1, T, d));
    out->g[out->n++] = lin_fwd(c, L.a, T, L.t["wqkv"], L.t["bqkv"], L.qkv);
  } else if (stage == 1) {
    DO(op_attn_fwd(o, L.qkv, L.o, L.lse, batch, S, H, d / H, L.s.causal));
    GemmArgs go = lin_fwd(c, L.o, T, L.t["wo"], L.t["bo"], L.u);
    go.res = layer_input(c, li); go.ldr = d;
    out->g[out->n++] = go;
  } else if (stage == 2) {
    DO(op_layernorm_fwd(o, L.u, c->P32(L.t["ln2.g"]), c->P32(L.t["ln2.b"]), L.c, L.mean2, L.rstd2, T, d));
    GemmArgs g1 = lin_fwd(c, L.c, T, L.t["w1"], L.t["b1"], L.f);
    g1.act = L.s.act == LP_ACT_RELU ? ACT_RELU : ACT_GELU;
    g1.pre = L.fpre;
    out->g[out->n++] = g1;
  } else {
    GemmArgs g2 = lin_fwd(c, L.f, T, L.t["w2"], L.t["b2"], L.out);
    g2.res = L.u; g2.ldr = d;
    out->g[out->n++] = g2;
  }
  return LP_OK;
}

static int dec_forward(lp_ctx* c, int li, int batch, const int32_t* ids) {
  StageGemms sg;
  for (int stage = 0; stage < kDecFwdStages; ++stage) {
    int st = dec_forward_stage(c, li, batch, ids, stage, &sg);
    if (st != LP_OK) return st;
    DO(op_gemm_grouped(c->op(), sg.g, sg.n));
  }
  return LP_OK;
}

// The four weight gradients read (dY, X) pairs that all stay alive until the end of the layer's backward pass and
// nothing in the pass reads them: they are collected in L.wg and handed back together by the last stage (one
// grouped launch).
int dec_backward_stage(lp_ctx* c, int li, int batch, const void* dout, void* dx, bool need_dx, int acc,
                       const int32_t* ids, bool params, int stage, StageGemms* out) {
  LayerState& L = c->layers[li];
  OpCtx o = c->op();
  int S = L.s.seq_len, d = L.s.width, H = L.s.n_heads, F = L.s.hidden, T = batch * S;
  bool has_emb = (li == 1 && c->spec.vocab > 0 && !L.in_override);
  out->n = 0;
  if (stage == 0) {            // FFN, second map
    L.wg[0] = lin_wgrad(c, dout, L.f, T, L.t["w2"], acc);
    GemmArgs gd = lin_dgrad(c, dout, T, L.t["w2"], c->dF);
    gd.dact = L.s.act == LP_ACT_RELU ? ACT_RELU : ACT_GELU; gd.dact_src = L.fpre; gd.ldd = F;
    out->g[out->n++] = gd;
  } else if (stage == 1) {     // FFN, first map
    L.wg[1] = lin_wgrad(c, c->dF, L.c, T, L.t["w1"], acc);
    out->g[out->n++] = lin_dgrad(c, c->dF, T, L.t["w1"], c->dc);
  } else if (stage == 2) {     // du = dout + LN2-backward(dc); attention output projection
    DO(op_layernorm_bwd(o, c->dc, L.u, L.mean2, L.rstd2, c->P32(L.t["ln2.g"]), dout, c->du,
                        params ? c->G32(L.t["ln2.g"]) : nullptr, params ? c->G32(L.t["ln2.b"]) : nullptr, T, d, acc));
    L.wg[2] = lin_wgrad(c, c->du, L.o, T, L.t["wo"], acc);
    out->g[out->n++] = lin_dgrad(c, c->du, T, L.t["wo"], c->dO);
  } else if (stage == 3) {     // attention, q/k/v projection
    DO(op_attn_bwd(o, L.qkv, L.o, L.lse, c->dO, c->dqkv, c->delta, batch, S, H, d / H, L.s.causal));
    L.wg[3] = lin_wgrad(c, c->dqkv, L.a, T, L.t["wqkv"], acc);
    out->g[out->n++] = lin_dgrad(c, c->dqkv, T, L.t["wqkv"], c->da);
  } else {
    // dh = du + LN1-backward(da); the input gradient itself is only needed inside a window or for the embedding
    const void* x = layer_input(c, li);
    bool want_dx = need_dx || (has_emb && params);
    void* dh = want_dx ? (has_emb ? c->da : dx) : nullptr;   // LN backward may write over its own dy rows
    if (params || want_dx)
      DO(op_layernorm_bwd(o, c->da, x, L.mean1, L.rstd1, c->P32(L.t["ln1.g"]), c->du, dh,
                          params ? c->G32(L.t["ln1.g"]) : nullptr, params ? c->G32(L.t["ln1.b"]) : nullptr, T, d, acc));
    if (has_emb && params) DO(op_embed_bwd(o, ids, dh, c->G32(L.t["emb"]), T, c->spec.vocab, d, acc));
    if (params) {
      // the four bias gradients: column sums of the same dY matrices the weight gradients read, in one pair of launches
      const void* dys[4] = {dout, c->dF, c->du, c->dqkv};
      const int64_t lds[4] = {d, F, d, 3 * d};
      float* outs[4] = {c->G32(L.t["b2"]), c->G32(L.t["b1"]), c->G32(L.t["bo"]), c->G32(L.t["bqkv"])};
      const int ns[4] = {d, F, d, 3 * d};
      DO(op_colsum_batched(o, 4, dys, lds, outs, T, ns, acc));
      for (int i = 0; i < 4; ++i) out->g[out->n++] = L.wg[i];
    }
  }
  return LP_OK;
}

static int dec_backward(lp_ctx* c, int li, int batch, const void* dout, void* dx, bool need_dx, int acc,
                        const int32_t* ids, bool params) {
  StageGemms sg;
  for (int stage = 0; stage < kDecBwdStages; ++stage) {
    int st = dec_backward_stage(c, li, batch, dout, dx, need_dx, acc, ids, params, stage, &sg);
    if (st != LP_OK) return st;
    DO(op_gemm_grouped(c->op(), sg.g, sg.n));
  }
  return LP_OK;
}

// ===================================================================================== ResNet stage
static int unit_forward(lp_ctx* c, ConvUnit& u, const void* x, const void* res) {
  OpCtx o = c->op();
  // the convolution leaves the normalisation's column statistics in the stream's partial buffer where it can
  // (whole tiles, batch statistics wanted); the normalisation then skips its own pass over z
  const BnRunning* run = c->bn_for(u.g, u.a.O);
  ConvStats st;
  if (!(run && run->use)) { st.buf = o.partial; st.cap = o.partial_elems; }
  DO(op_conv_fwd(o, u.a, x, c->W(u.w), u.z, &st));
  int rows = u.a.N * u.a.P * u.a.Q;
  DO(op_batchnorm_fwd(o, u.z, c->P32(u.g), c->P32(u.b), res, u.y, u.mean, u.rstd, rows, u.a.O, u.relu, run, &st));
  return LP_OK;
}
// dy -> (dz in sZ) -> dw, and dx (+ dx_add, if given) if asked.  dres (if non-null) receives the ReLU-masked dy.
static int unit_backward(lp_ctx* c, ConvUnit& u, const void* x, const void* dy, void* dres, void* dx, int acc,
                         const void* dx_add = nullptr) {
  OpCtx o = c->op();
  int rows = u.a.N * u.a.P * u.a.Q;
  const size_t es = dtype_size(c->dt);
  if (u.dy_keep) DO(hipMemcpyAsync(u.dy_keep, dy, (size_t)rows * u.a.O * es, hipMemcpyDeviceToDevice, o.stream));
  DO(op_batchnorm_bwd(o, dy, u.y, u.z, u.mean, u.rstd, c->P32(u.g), c->sZ, dres, c->G32(u.g), c->G32(u.b), rows,
                      u.a.O, u.relu, acc));
  DO(op_conv_bwd_weight(o, u.a, c->sZ, x, c->G32(u.w), acc));
  if (dx) DO(op_conv_bwd_data(o, u.a, c->sZ, c->W(u.w), dx, dx_add));
  u.dx_valid = dx != nullptr;
  if (dx && u.dx_keep)
    DO(hipMemcpyAsync(u.dx_keep, dx, (size_t)u.a.N * u.a.H * u.a.W * u.a.C * es, hipMemcpyDeviceToDevice, o.stream));
  return LP_OK;
}
static void set_batch(ConvUnit& u, int batch) { u.a.N = batch; }

static int res_forward(lp_ctx* c, int li, int batch) {
  LayerState& L = c->layers[li];
  const void* h = layer_input(c, li);
  int st;
  if (L.has_stem) {
    set_batch(L.stem, batch);
    if ((st = unit_forward(c, L.stem, h, nullptr)) != LP_OK) return st;
    h = L.stem.y;
  }
  for (auto& b : L.blocks) {
    set_batch(b.c1, batch); set_batch(b.c2, batch); set_batch(b.proj, batch);
    if ((st = unit_forward(c, b.c1, h, nullptr)) != LP_OK) return st;
    const void* sc = h;
    if (b.has_proj) {
      if ((st = unit_forward(c, b.proj, h, nullptr)) != LP_OK) return st;
      sc = b.proj.y;
    }
    if ((st = unit_forward(c, b.c2, b.c1.y, sc)) != LP_OK) return st;
    h = b.c2.y;
  }
  return LP_OK;
}

static int res_backward(lp_ctx* c, int li, int batch, const void* dout, void* dx, bool need_dx, int acc) {
  LayerState& L = c->layers[li];
  OpCtx o = c->op();
  const void* g = dout;
  int st;
  for (int bi = (int)L.blocks.size() - 1; bi >= 0; --bi) {
    BasicBlock& b = L.blocks[bi];
    const void* bin = bi > 0 ? L.blocks[bi - 1].c2.y : (L.has_stem ? L.stem.y : layer_input(c, li));
    bool first_op = (bi == 0 && !L.has_stem);
    bool want_dx = need_dx || !first_op;
    // c2: dz2 -> dw2, dt (into sD1); masked upstream gradient ds -> sR
    if ((st = unit_backward(c, b.c2, b.c1.y, g, c->sR, c->sD1, acc)) != LP_OK) return st;
    // c1, and the shortcut's share of the block input's gradient, added in the data-gradient epilogue that
    // finishes last: the identity shortcut's is the masked upstream gradient itself (sR), a projection's is its
    // own data gradient, which then takes c1's (sD1) as its addend
    void* dst = (first_op && need_dx) ? dx : c->sG;
    if (b.has_proj) {
      if ((st = unit_backward(c, b.c1, bin, c->sD1, nullptr, want_dx ? c->sD1 : nullptr, acc)) != LP_OK) return st;
      if ((st = unit_backward(c, b.proj, bin, c->sR, nullptr, want_dx ? dst : nullptr, acc, c->sD1)) != LP_OK) return st;
    } else {
      if ((st = unit_backward(c, b.c1, bin, c->sD1, nullptr, want_dx ? dst : nullptr, acc, c->sR)) != LP_OK) return st;
    }
    g = dst;
  }
  if (L.has_stem) {
    if ((st = unit_backward(c, L.stem, layer_input(c, li), g, nullptr, need_dx ? dx : nullptr, acc)) != LP_OK)
      return st;
  }
  return LP_OK;
}

// ===================================================================================== dispatch
int drv_forward(lp_ctx* c, int li, int batch, const int32_t* ids) {
  switch (c->layers[li].s.kind) {
    case LP_LAYER_RESMLP: return mlp_forward(c, li, batch);
    case LP_LAYER_DECODER: return dec_forward(c, li, batch, ids);
    case LP_LAYER_RESNET_STAGE: return res_forward(c, li, batch);
  }
  return LP_EINVAL;
}
int drv_backward(lp_ctx* c, int li, int batch, const void* dout, void* dx, bool need_dx, int accumulate, bool params) {
  switch (c->layers[li].s.kind) {
    case LP_LAYER_RESMLP: return mlp_backward(c, li, batch, dout, dx, need_dx, accumulate, params);
    case LP_LAYER_DECODER:
      return dec_backward(c, li, batch, dout, dx, need_dx, accumulate, (const int32_t*)c->x_in, params);
    case LP_LAYER_RESNET_STAGE:
      if (!params) { c->err = "a ResNet stage has no input-gradient-only pass"; return LP_EUNSUPPORTED; }
      return res_backward(c, li, batch, dout, dx, need_dx, accumulate);
  }
  return LP_EINVAL;
}

// ===================================================================================== heads
// The vocabulary head (LayerNorm, projection, cross-entropy) in stages, like the decoder layer: stage 0 ends in the
// logits product, stage 1 (loss, dZ) in the head's weight gradient, stage 2 in its input gradient, stage 3 is the
// LayerNorm backward.  Without `backward` only stages 0 and 1 do anything, and stage 1 hands back no product.
int vocab_head_stage(lp_ctx* c, int hi, int batch, const int32_t* y, float* loss_out, bool backward, void* dh,
                     int stage, StageGemms* out) {
  HeadState& Hd = c->heads[hi];
  LayerState& L = c->layers[Hd.e];
  OpCtx o = c->op();
  const int rows = batch * L.s.seq_len, in_dim = Hd.s.in_dim, ncls = Hd.s.n_classes;
  out->n = 0;
  if (stage == 0) {
    DO(op_layernorm_fwd(o, L.out, c->P32(Hd.t["ln.g"]), c->P32(Hd.t["ln.b"]), c->feat, c->hmean, c->hrstd, rows, in_dim));
    out->g[out->n++] = lin_fwd(c, c->feat, rows, Hd.t["w"], -1, c->logits);
  } else if (stage == 1) {
    DO(op_softmax_ce(o, c->logits, ncls, y, c->loss_rows, rows, ncls, backward ? 1 : 0, 1.0f / (float)rows));
    DO(op_mean(o, c->loss_rows, rows, loss_out));
    if (backward) out->g[out->n++] = lin_wgrad(c, c->logits, c->feat, rows, Hd.t["w"], 0);    // logits now hold dZ
  } else if (stage == 2) {
    if (backward) out->g[out->n++] = lin_dgrad(c, c->logits, rows, Hd.t["w"], c->dfeat);
  } else if (backward) {
    DO(op_layernorm_bwd(o, c->dfeat, L.out, c->hmean, c->hrstd, c->P32(Hd.t["ln.g"]), nullptr, dh,
                        c->G32(Hd.t["ln.g"]), c->G32(Hd.t["ln.b"]), rows, in_dim, 0));
  }
  return LP_OK;
}

// Loss of head hi on the output of layer e; if `backward`, also the head's parameter gradients and
// d loss / d h_e into dh.
int drv_head(lp_ctx* c, int hi, int batch, const int32_t* y, float* loss_out, bool backward, void* dh) {
  HeadState& Hd = c->heads[hi];
  LayerState& L = c->layers[Hd.e];
  OpCtx o = c->op();
  if (Hd.s.kind == LP_HEAD_LN_LINEAR_CE && !Hd.t.count("b")) {
    StageGemms sg;
    for (int stage = 0; stage < kVocabHeadStages; ++stage) {
      int st = vocab_head_stage(c, hi, batch, y, loss_out, backward, dh, stage, &sg);
      if (st != LP_OK) return st;
      DO(op_gemm_grouped(c->op(), sg.g, sg.n));
    }
    return LP_OK;
  }
  const void* h = L.out;
  int rows, in_dim = Hd.s.in_dim, ncls = Hd.s.n_classes;
  const void* feat = h;
  int hw = 0;
  if (Hd.s.kind == LP_HEAD_POOL_LINEAR_CE) {
    int side = L.s.in_hw / L.s.stride;
    hw = side * side;
    rows = batch;
    DO(op_avgpool_fwd(o, h, c->feat, batch, hw, in_dim));
    feat = c->feat;
  } else if (Hd.s.kind == LP_HEAD_BN_POOL_LINEAR_CE) {
    // appendix B.3: batch norm, ReLU, spatial mean, linear.  The normalised, rectified activation lives in the
    // stage-backward scratch, which this chain does not touch before the head's own backward pass is done.
    int side = L.s.in_hw / L.s.stride;
    hw = side * side;
    rows = batch;
    DO(op_batchnorm_fwd(o, h, c->P32(Hd.t["bn.g"]), c->P32(Hd.t["bn.b"]), nullptr, c->sG, c->hmean, c->hrstd,
                        batch * hw, in_dim, 1, c->bn_for(Hd.t["bn.g"], in_dim)));
    DO(op_avgpool_fwd(o, c->sG, c->feat, batch, hw, in_dim));
    feat = c->feat;
  } else if (Hd.s.kind == LP_HEAD_LN_LINEAR_CE) {
    rows = batch * L.s.seq_len;
    DO(op_layernorm_fwd(o, h, c->P32(Hd.t["ln.g"]), c->P32(Hd.t["ln.b"]), c->feat, c->hmean, c->hrstd, rows, in_dim));
    feat = c->feat;
  } else {
    rows = batch;
  }
  int tb = Hd.t.count("b") ? Hd.t["b"] : -1;
  DO(op_gemm(o, lin_fwd(c, feat, rows, Hd.t["w"], tb, c->logits)));
  DO(op_softmax_ce(o, c->logits, ncls, y, c->loss_rows, rows, ncls, backward ? 1 : 0, 1.0f / (float)rows));
  DO(op_mean(o, c->loss_rows, rows, loss_out));
  if (!backward) return LP_OK;
  // logits now hold dZ
  if (tb >= 0) DO(op_colsum(o, c->logits, ncls, c->G32(tb), rows, ncls, 0));
  DO(op_gemm(o, lin_wgrad(c, c->logits, feat, rows, Hd.t["w"], 0)));
  if (Hd.s.kind == LP_HEAD_LINEAR_CE) {
    DO(op_gemm(o, lin_dgrad(c, c->logits, rows, Hd.t["w"], dh)));
  } else {
    DO(op_gemm(o, lin_dgrad(c, c->logits, rows, Hd.t["w"], c->dfeat)));
    if (Hd.s.kind == LP_HEAD_POOL_LINEAR_CE) {
      DO(op_avgpool_bwd(o, c->dfeat, dh, batch, hw, in_dim));
    } else if (Hd.s.kind == LP_HEAD_BN_POOL_LINEAR_CE) {
      DO(op_avgpool_bwd(o, c->dfeat, c->sZ, batch, hw, in_dim));
      DO(op_batchnorm_bwd(o, c->sZ, c->sG, h, c->hmean, c->hrstd, c->P32(Hd.t["bn.g"]), dh, nullptr,
                          c->G32(Hd.t["bn.g"]), c->G32(Hd.t["bn.b"]), batch * hw, in_dim, 1, 0));
    } else {
      DO(op_layernorm_bwd(o, c->dfeat, h, c->hmean, c->hrstd, c->P32(Hd.t["ln.g"]), nullptr, dh,
                          c->G32(Hd.t["ln.g"]), c->G32(Hd.t["ln.b"]), rows, in_dim, 0));
    }
  }
  return LP_OK;
}

}  // namespace lp
