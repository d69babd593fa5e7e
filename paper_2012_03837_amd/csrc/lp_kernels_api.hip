// Kernel-level C ABI (include/lp_kernels.h): thin wrappers that build an OpCtx and call one op.
#include <stdio.h>
#include <mutex>

#include "../../include/lp_kernels.h"
#include "common.h"

namespace lp {
hipError_t gemm_plain(const OpCtx& c, const GemmArgs& g);
hipError_t gemm_mfma(const OpCtx& c, const GemmArgs& g);
hipError_t gemm_dma_grouped(const OpCtx& c, const GemmArgs* gs, int n);
hipError_t attn_fwd_plain(const OpCtx& c, const void* qkv, void* o, float* lse, int B, int S, int H, int dh, int causal);
hipError_t attn_bwd_plain(const OpCtx& c, const void* qkv, const void* o, const float* lse, const void* dout,
                          void* dqkv, float* delta, int B, int S, int H, int dh, int causal);
hipError_t conv_fwd_plain(const OpCtx& c, const ConvArgs& a, const void* x, const void* w, void* out);
hipError_t conv_bwd_data_plain(const OpCtx& c, const ConvArgs& a, const void* dout, const void* w, void* dx,
                               const void* add = nullptr);
hipError_t conv_bwd_weight_plain(const OpCtx& c, const ConvArgs& a, const void* dout, const void* x, float* dw,
                                 int accumulate);
}
using namespace lp;

static OpCtx mk(int dtype, void* stream, float* scratch = nullptr, size_t n = 0) {
  OpCtx c; c.stream = (hipStream_t)stream; c.dt = dtype; c.partial = scratch; c.partial_elems = n; c.prof = nullptr;
  return c;
}
static ConvArgs mkconv(int N, int H, int W, int C, int O, int R, int stride, int pad) {
  ConvArgs a; a.N = N; a.H = H; a.W = W; a.C = C; a.O = O; a.R = R; a.S = R; a.stride = stride; a.pad = pad;
  a.P = (H + 2 * pad - R) / stride + 1; a.Q = (W + 2 * pad - R) / stride + 1;
  return a;
}

extern "C" int lpk_gemm(int dtype, const void* A, int64_t lda, int a_kc, const void* B, int64_t ldb, int b_kc, void* C,
                        int64_t ldc, int c_f32, int M, int N, int K, const float* bias, int act, void* pre,
                        const void* dact_src, int dact, int64_t ldd, const void* res, int64_t ldr, int accumulate,
                        int variant, float* splitk_ws, size_t splitk_ws_elems, void* stream) {
  if (variant < 0 || (variant > 11 && (variant < 20 || variant > 22))) return (int)hipErrorInvalidValue;
  GemmArgs g;
  g.A = A; g.lda = lda; g.a_kc = a_kc; g.B = B; g.ldb = ldb; g.b_kc = b_kc; g.C = C; g.ldc = ldc; g.c_f32 = c_f32;
  g.M = M; g.N = N; g.K = K; g.bias = bias; g.act = act; g.pre = pre; g.dact_src = dact_src; g.dact = dact; g.ldd = ldd;
  g.res = res; g.ldr = ldr; g.accumulate = accumulate;
  OpCtx c = mk(dtype, stream);
  c.splitk_ws = splitk_ws; c.splitk_elems = splitk_ws_elems;
  if (variant == 1 || dtype != BF16) return (int)gemm_plain(c, g);
  c.gemm_variant = variant;
  return (int)op_gemm(c, g);
}
extern "C" int lpk_gemm_grouped(int n, const void* const* A, const int64_t* lda, const void* const* B, const int64_t* ldb,
                                void* const* C, const int64_t* ldc, int c_f32, const int* M, const int* N, int K, int a_kc,
                                int b_kc, const float* const* bias, int act, const void* const* res, int accumulate,
                                float* splitk_ws, size_t splitk_ws_elems, void* stream) {
  if (n < 1 || n > 16 || !A || !lda || !B || !ldb || !C || !ldc || !M || !N) return (int)hipErrorInvalidValue;
  GemmArgs g[16];
  for (int i = 0; i < n; ++i) {
    g[i].A = A[i]; g[i].lda = lda[i]; g[i].a_kc = a_kc; g[i].B = B[i]; g[i].ldb = ldb[i]; g[i].b_kc = b_kc;
    g[i].C = C[i]; g[i].ldc = ldc[i]; g[i].c_f32 = c_f32; g[i].M = M[i]; g[i].N = N[i]; g[i].K = K;
    g[i].bias = bias ? bias[i] : nullptr; g[i].act = act;
    g[i].res = res ? res[i] : nullptr; g[i].ldr = ldc[i];
    g[i].accumulate = accumulate;
  }
  OpCtx c = mk(BF16, stream);
  c.splitk_ws = splitk_ws; c.splitk_elems = splitk_ws_elems;
  return (int)gemm_dma_grouped(c, g, n);
}
extern "C" int lpk_attention_fwd(int dtype, const void* qkv, void* o, float* lse, int B, int S, int H, int dh,
                                 int causal, int plain, void* stream) {
  OpCtx c = mk(dtype, stream);
  if (plain) return (int)attn_fwd_plain(c, qkv, o, lse, B, S, H, dh, causal);
  return (int)op_attn_fwd(c, qkv, o, lse, B, S, H, dh, causal);
}
extern "C" int lpk_attention_bwd(int dtype, const void* qkv, const void* o, const float* lse, const void* dout,
                                 void* dqkv, float* delta, int B, int S, int H, int dh, int causal, int plain,
                                 void* stream) {
  OpCtx c = mk(dtype, stream);
  if (plain) return (int)attn_bwd_plain(c, qkv, o, lse, dout, dqkv, delta, B, S, H, dh, causal);
  return (int)op_attn_bwd(c, qkv, o, lse, dout, dqkv, delta, B, S, H, dh, causal);
}
extern "C" int lpk_layernorm_fwd(int dtype, const void* x, const float* g, const float* b, void* y, float* mean,
                                 float* rstd, int rows, int d, void* stream) {
  return (int)op_layernorm_fwd(mk(dtype, stream), x, g, b, y, mean, rstd, rows, d);
}
extern "C" int lpk_layernorm_bwd(int dtype, const void* dy, const void* x, const float* mean, const float* rstd,
                                 const float* g, const void* add, void* dx, float* dg, float* db, int rows, int d,
                                 int accumulate, float* scratch, size_t scratch_elems, void* stream) {
  return (int)op_layernorm_bwd(mk(dtype, stream, scratch, scratch_elems), dy, x, mean, rstd, g, add, dx, dg, db, rows,
                               d, accumulate);
}
// Workspace of lpk_layernorm_bwd_static: every GPU the library runs on holds its own copy of this array until
// the process ends.  In host code the array's name is only a handle for hipGetSymbolAddress; the address the
// kernels get is looked up once per device, with that device current, and kept in g_static_ptr.
static __device__ __align__(256) float scratch[LPK_STATIC_SCRATCH_FLOATS];
static float* g_static_ptr[64];
static std::mutex g_static_mu;

extern "C" int lpk_layernorm_bwd_static(int dtype, const void* dy, const void* x, const float* mean, const float* rstd,
                                        const float* g, const void* add, void* dx, float* dg, float* db, int rows,
                                        int d, int accumulate, void* stream) {
  if (rows < 0 || d < 1) return (int)hipErrorInvalidValue;
  // the vectorised bf16 kernel writes one pair of partial rows per 8 input rows (the generic one per 32)
  const size_t need = (size_t)((rows + 7) / 8) * (size_t)d * 2;
  if (need > (size_t)LPK_STATIC_SCRATCH_FLOATS) {
    fprintf(stderr, "lpk_layernorm_bwd_static: rows=%d d=%d needs %zu floats of workspace, the built-in one holds %zu\n",
            rows, d, need, (size_t)LPK_STATIC_SCRATCH_FLOATS);
    return (int)hipErrorInvalidValue;
  }
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return (int)e;
  if (dev < 0 || dev >= 64) return (int)hipErrorInvalidDevice;
  float* ws;
  {
    std::lock_guard<std::mutex> lock(g_static_mu);
    if (!g_static_ptr[dev]) {
      void* p = nullptr;
      e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
      if (e != hipSuccess) return (int)e;
      g_static_ptr[dev] = (float*)p;
    }
    ws = g_static_ptr[dev];
  }
  // every partial row that is read is written first by the same call: nothing has to start at zero
  return (int)op_layernorm_bwd(mk(dtype, stream, ws, (size_t)LPK_STATIC_SCRATCH_FLOATS), dy, x, mean, rstd, g, add, dx,
                               dg, db, rows, d, accumulate);
}
extern "C" int lpk_softmax_ce(int dtype, void* z, int64_t ld, const int32_t* y, float* loss_rows, int rows, int n,
                              int write_grad, float inv_rows, void* stream) {
  return (int)op_softmax_ce(mk(dtype, stream), z, ld, y, loss_rows, rows, n, write_grad, inv_rows);
}
extern "C" int lpk_optimizer(int kind, float lr, float momentum, float beta1, float beta2, float eps,
                             float weight_decay, int t, float grad_scale, float* p, const float* g, float* m, float* v,
                             void* p_bf16, size_t n, void* stream) {
  OptArgs o; o.kind = kind; o.lr = lr; o.momentum = momentum; o.beta1 = beta1; o.beta2 = beta2; o.eps = eps;
  o.weight_decay = weight_decay; o.t = t; o.grad_scale = grad_scale;
  if (kind < 0 || kind > 2) return (int)hipErrorInvalidValue;
  return (int)op_optimizer(mk(F32, stream), o, p, g, m, v, p_bf16, n);
}
extern "C" int lpk_copy(const void* src, void* dst, size_t bytes, void* stream) {
  if (bytes % 16 || ((uintptr_t)src & 15) || ((uintptr_t)dst & 15)) return (int)hipErrorInvalidValue;
  return (int)op_copy(mk(0, stream), src, dst, bytes);
}
extern "C" int lpk_transpose_bf16(const void* src, void* dst, int R, int C, void* stream) {
  return (int)op_transpose_bf16(mk(1, stream), src, dst, R, C);
}
extern "C" int lpk_embed_bwd(int dtype, const int32_t* ids, const void* dh, float* demb, int T, int V, int d,
                             int accumulate, float* scratch, size_t scratch_elems, void* stream) {
  return (int)op_embed_bwd(mk(dtype, stream, scratch, scratch_elems), ids, dh, demb, T, V, d, accumulate);
}
extern "C" int lpk_conv_fwd(int dtype, const void* x, const void* w, void* out, int N, int H, int W, int C, int O,
                            int R, int stride, int pad, void* stream) {
  return (int)op_conv_fwd(mk(dtype, stream), mkconv(N, H, W, C, O, R, stride, pad), x, w, out);
}
extern "C" int lpk_conv_bwd_data(int dtype, const void* dout, const void* w, void* dx, int N, int H, int W, int C,
                                 int O, int R, int stride, int pad, void* stream) {
  return (int)op_conv_bwd_data(mk(dtype, stream), mkconv(N, H, W, C, O, R, stride, pad), dout, w, dx);
}
extern "C" int lpk_conv_bwd_weight(int dtype, const void* dout, const void* x, float* dw, int N, int H, int W, int C,
                                   int O, int R, int stride, int pad, int accumulate, void* stream) {
  return (int)op_conv_bwd_weight(mk(dtype, stream), mkconv(N, H, W, C, O, R, stride, pad), dout, x, dw, accumulate);
}
extern "C" int lpk_conv_bwd_weight_ws(int dtype, const void* dout, const void* x, float* dw, int N, int H, int W, int C,
                                      int O, int R, int stride, int pad, int accumulate, float* splitk_ws,
                                      size_t splitk_ws_elems, void* stream) {
  OpCtx c = mk(dtype, stream);
  c.splitk_ws = splitk_ws; c.splitk_elems = splitk_ws ? splitk_ws_elems : 0;
  return (int)op_conv_bwd_weight(c, mkconv(N, H, W, C, O, R, stride, pad), dout, x, dw, accumulate);
}
extern "C" int lpk_conv_bn_fwd(int dtype, const void* x, const void* w, void* z, const float* g, const float* b,
                               const void* res, void* y, float* mean, float* rstd, int N, int H, int W, int C, int O,
                               int R, int stride, int pad, int relu, float* scratch, size_t scratch_elems, void* stream) {
  OpCtx c = mk(dtype, stream, scratch, scratch_elems);
  ConvArgs a = mkconv(N, H, W, C, O, R, stride, pad);
  ConvStats st;
  st.buf = scratch; st.cap = scratch ? scratch_elems : 0;
  hipError_t e = op_conv_fwd(c, a, x, w, z, &st);
  if (e != hipSuccess) return (int)e;
  return (int)op_batchnorm_fwd(c, z, g, b, res, y, mean, rstd, a.N * a.P * a.Q, O, relu, nullptr, &st);
}
extern "C" int lpk_batchnorm_fwd(int dtype, const void* z, const float* g, const float* b, const void* res, void* y,
                                 float* mean, float* rstd, int rows, int C, int relu, float* scratch,
                                 size_t scratch_elems, void* stream) {
  return (int)op_batchnorm_fwd(mk(dtype, stream, scratch, scratch_elems), z, g, b, res, y, mean, rstd, rows, C, relu);
}
extern "C" int lpk_batchnorm_bwd(int dtype, const void* dy, const void* y, const void* z, const float* mean,
                                 const float* rstd, const float* g, void* dz, void* dres, float* dg, float* db,
                                 int rows, int C, int relu, int accumulate, float* scratch, size_t scratch_elems,
                                 void* stream) {
  return (int)op_batchnorm_bwd(mk(dtype, stream, scratch, scratch_elems), dy, y, z, mean, rstd, g, dz, dres, dg, db,
                               rows, C, relu, accumulate);
}
