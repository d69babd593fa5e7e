// Shared declarations of the HIP library: element types, error plumbing, and the internal
// kernel-launch API ("ops") that the layer drivers call.  gfx950 only.
#pragma once
#include <map>
#include <string>

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>

namespace lp {

typedef __bf16 bf16_t;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;

enum DType { F32 = 0, BF16 = 1, I32 = 2 };
static inline size_t dtype_size(int dt) { return dt == BF16 ? 2 : 4; }

__device__ __forceinline__ float to_f(float v) { return v; }
__device__ __forceinline__ float to_f(bf16_t v) { return static_cast<float>(v); }
template <typename T> __device__ __forceinline__ T from_f(float f);
template <> __device__ __forceinline__ float from_f<float>(float f) { return f; }
template <> __device__ __forceinline__ bf16_t from_f<bf16_t>(float f) { return static_cast<bf16_t>(f); }

enum Act { ACT_NONE = 0, ACT_RELU = 1, ACT_GELU = 2 };

// GELU in its tanh form, 0.5 x (1 + tanh(u)) with u = c (x + a x^3), written through the identity
// 0.5 (1 + tanh(u)) = sigmoid(2u) = 1 / (1 + e^{-2u}) on the hardware exp2 and reciprocal: absolute error of
// a few 1e-7 and exact limits for large |x| (e^{-2u} = inf gives 0, 0 gives 1).  The library tanhf costs
// several times as many instructions, and in a fused GEMM epilogue the MFMA pipe idles meanwhile.
__device__ __forceinline__ float gelu_gate(float x) {     // sigmoid(2u)
  const float k1 = -2.0f * 0.7978845608028654f * 1.4426950408889634f, k3 = k1 * 0.044715f;
  const float x2 = x * x;
  const float e = __builtin_amdgcn_exp2f(x * (k1 + k3 * x2));          // e^{-2u}
  return __builtin_amdgcn_rcpf(1.0f + e);
}
__device__ __forceinline__ float gelu_f(float x) { return x * gelu_gate(x); }
// d/dx [x s(x)] = s + x s', s' = s (1 - s) 2c (1 + 3 a x^2)
__device__ __forceinline__ float dgelu_f(float x) {
  const float c2 = 2.0f * 0.7978845608028654f, a3 = 3.0f * 0.044715f;
  const float s = gelu_gate(x);
  return s * (1.0f + x * (1.0f - s) * (c2 + c2 * a3 * x * x));
}

// C[M,N] (+)= alpha * sum_k A(m,k) B(n,k), then the epilogue:
//   v = acc (+ bias[n]); if (pre) pre[m,n] = v; v = act(v); if (dact) v *= act'(dact_src[m,n]);
//   if (res) v += res[m,n]; C[m,n] = (accumulate ? C[m,n] : 0) + v.
// A(m,k) = a_kc ? A[m*lda + k] : A[k*lda + m];  B(n,k) = b_kc ? B[n*ldb + k] : B[k*ldb + n].
// Operands, pre, dact_src and res are in the compute dtype; C is compute dtype unless c_f32.
struct GemmArgs {
  const void* A = nullptr; int64_t lda = 0; int a_kc = 1;
  const void* B = nullptr; int64_t ldb = 0; int b_kc = 1;
  void* C = nullptr; int64_t ldc = 0; int c_f32 = 0;
  int M = 0, N = 0, K = 0;
  const float* bias = nullptr;
  int act = ACT_NONE;
  void* pre = nullptr;
  const void* dact_src = nullptr; int dact = ACT_NONE; int64_t ldd = 0;
  const void* res = nullptr; int64_t ldr = 0;
  int accumulate = 0;
};

// Convolution as an implicit GEMM over NHWC activations and [O,R,S,C] filters.
struct ConvArgs {
  int N, H, W, C;      // input
  int O, R, S;         // filters
  int stride, pad;
  int P, Q;            // output spatial
};

// Optional per-kernel-class timing with HIP events recorded on the launch stream.
enum KernelClass { KC_GEMM = 0, KC_ATTN_FWD, KC_ATTN_BWD, KC_LAYERNORM, KC_SOFTMAX_CE, KC_OPTIMIZER, KC_EMBED,
                   KC_COLSUM, KC_CONV, KC_BATCHNORM, KC_OTHER, KC_GEMM_KERNEL, KC_COUNT };
struct Profiler {
  bool on = false;
  struct Pair { hipEvent_t a, b; int kc; uint64_t tag; const char* kname; double flops; };
  Pair* pairs = nullptr; int cap = 0; int used = 0; int dropped = 0;
  double total_ms[KC_COUNT] = {}; long long launches[KC_COUNT] = {}; double flops[KC_COUNT] = {};
  // GEMM ops by shape: tag = M | N << 20 | K << 40 | a_kc << 60 | b_kc << 61 | c_f32 << 62
  struct ShapeTotal { double ms = 0; long long n = 0; };
  std::map<uint64_t, ShapeTotal> by_shape;
  // Main GEMM kernels by instance name (class KC_GEMM_KERNEL: a pair brackets that one launch, without the
  // partial-sum fix-up an op may launch behind it): launches, summed time, algorithmic FLOPs.
  struct KernelTotal { double ms = 0; long long n = 0; double flops = 0; };
  std::map<std::string, KernelTotal> by_kernel;
};

struct OpCtx {
  hipStream_t stream;
  int dt;              // compute dtype
  float* partial;      // fp32 scratch for two-stage reductions
  size_t partial_elems;
  Profiler* prof = nullptr;
  int gemm_variant = 0;         // 0: chosen by the cost model; otherwise a forced GEMM kernel (see lpk_gemm)
  float* splitk_ws = nullptr;   // fp32 workspace for split-K partial sums (may be null: no split-K)
  size_t splitk_elems = 0;
};

// RAII bracket: records an event pair around the launches of one op when profiling is on.
struct ProfScope {
  Profiler* p; hipStream_t s; int idx = -1;
  ProfScope(const OpCtx& c, int kc, double flops = 0.0, uint64_t tag = 0, const char* kname = nullptr)
      : p(c.prof), s(c.stream) {
    if (!p || !p->on) { p = nullptr; return; }
    p->launches[kc] += 1; p->flops[kc] += flops;
    if (p->used >= p->cap) { p->dropped += 1; p = nullptr; return; }
    idx = p->used++;
    p->pairs[idx].kc = kc; p->pairs[idx].tag = tag; p->pairs[idx].kname = kname; p->pairs[idx].flops = flops;
    (void)hipEventRecord(p->pairs[idx].a, s);
  }
  void finish() { if (p) { (void)hipEventRecord(p->pairs[idx].b, s); p = nullptr; } }
  ~ProfScope() { finish(); }
};

// ---- ops (each enqueues on ctx.stream and returns a hipError_t) -------------------------------
hipError_t op_gemm(const OpCtx& c, const GemmArgs& g);
// n independent products in one launch where they qualify (bf16, same reduction length and operand layouts,
// plain fp32 outputs: the weight gradients of one layer), otherwise one after the other.
hipError_t op_gemm_grouped(const OpCtx& c, const GemmArgs* gs, int n);
hipError_t op_fill_f32(const OpCtx& c, float* p, size_t n, float v);
// out[0] = <a, b> / (|a| |b|) over n floats (0 if either norm is 0); uses 3 * 128 floats of c.partial
hipError_t op_cosine(const OpCtx& c, const float* a, const float* b, size_t n, float* out);
hipError_t op_copy(const OpCtx& c, const void* src, void* dst, size_t bytes);   // bytes % 16 == 0
hipError_t op_cast_to_compute(const OpCtx& c, const float* src, void* dst, size_t n);
// dst[C][R] = src[R][C]^T, bf16, R and C multiples of 8 and both pointers 16-byte aligned
hipError_t op_transpose_bf16(const OpCtx& c, const void* src, void* dst, int R, int C);

hipError_t op_embed_fwd(const OpCtx& c, const int32_t* ids, const float* emb, const float* pe, void* out,
                        int T, int S, int d, int V);
hipError_t op_embed_bwd(const OpCtx& c, const int32_t* ids, const void* dh, float* demb, int T, int V, int d,
                        int accumulate);
hipError_t op_posenc_init(const OpCtx& c, float* pe, int S, int d);

hipError_t op_layernorm_fwd(const OpCtx& c, const void* x, const float* g, const float* b, void* y,
                            float* mean, float* rstd, int rows, int d);
// dx = (add ? add : 0) + LN-backward(dy); dg/db accumulate if `accumulate`.  dx may be null; dg and db may
// both be null (input gradient only).
hipError_t op_layernorm_bwd(const OpCtx& c, const void* dy, const void* x, const float* mean, const float* rstd,
                            const float* g, const void* add, void* dx, float* dg, float* db, int rows, int d,
                            int accumulate);
hipError_t op_colsum(const OpCtx& c, const void* dy, int64_t ld, float* out, int rows, int n, int accumulate);
// count (<= 4 for the single pair of launches) column sums over the same rows; the same bits as op_colsum one by one
hipError_t op_colsum_batched(const OpCtx& c, int count, const void* const* dy, const int64_t* ld, float* const* out,
                             int rows, const int* n, int accumulate);

hipError_t op_attn_fwd(const OpCtx& c, const void* qkv, void* o, float* lse, int B, int S, int H, int dh,
                       int causal);
hipError_t op_attn_bwd(const OpCtx& c, const void* qkv, const void* o, const float* lse, const void* dout,
                       void* dqkv, float* delta, int B, int S, int H, int dh, int causal);

// Row-wise softmax cross-entropy over logits z [rows, n] (compute dtype, leading dim ld).
// loss_rows[r] = logsumexp(z_r) - z[r, y_r].  If write_grad: z is overwritten by
// (softmax(z_r) - onehot(y_r)) * inv_rows.
hipError_t op_softmax_ce(const OpCtx& c, void* z, int64_t ld, const int32_t* y, float* loss_rows, int rows,
                         int n, int write_grad, float inv_rows);
hipError_t op_mean(const OpCtx& c, const float* v, int n, float* out);

struct OptArgs {
  int kind; float lr, momentum, beta1, beta2, eps, weight_decay; int t; float grad_scale;
};
hipError_t op_optimizer(const OpCtx& c, const OptArgs& o, float* p, const float* g, float* m, float* v,
                        void* p_lowp, size_t n);

hipError_t op_init_normal(const OpCtx& c, float* p, size_t n, float std, uint64_t seed, uint64_t stream_id);

// conv / batchnorm / pooling
// Column statistics of a convolution's output, left by the convolution kernel itself for the batch normalisation
// behind it: for slab t of slab_rows consecutive rows and column j, p = the slab's first row, s0 = sum (z - p),
// s1 = sum (z - p)^2 over the rounded outputs, stored as buf[(0 * nslab + t) * C + j], [(1 * nslab + t) ...] and
// [(2 * nslab + t) ...].  The caller sets buf / cap (floats); nslab stays 0 if the launch did not produce them.
struct ConvStats {
  float* buf = nullptr;
  size_t cap = 0;
  int nslab = 0, slab_rows = 0;
};
hipError_t op_conv_fwd(const OpCtx& c, const ConvArgs& a, const void* x, const void* w, void* out,
                       ConvStats* stats = nullptr);
// dx = data gradient (+ add, an activation-gradient tensor of dx's shape: the other branch of a residual block).
hipError_t op_conv_bwd_data(const OpCtx& c, const ConvArgs& a, const void* dout, const void* w, void* dx,
                            const void* add = nullptr);
hipError_t op_conv_bwd_weight(const OpCtx& c, const ConvArgs& a, const void* dout, const void* x, float* dw,
                              int accumulate);
// Running statistics of one batch normalisation (the evaluation form of the method appendix B.3 cites).
// use == 0: the forward pass normalises with the batch's statistics and folds them in,
//   mean <- (1 - momentum) mean + momentum mean_B,  var <- (1 - momentum) var + momentum var_B rows / (rows - 1);
// use == 1: it normalises with mean / var as they stand and leaves them alone.
struct BnRunning {
  float* mean = nullptr;
  float* var = nullptr;
  float momentum = 0.f;
  int use = 0;
};
// y = [relu]( bn(z) (+ res) ), batch statistics over rows = N*H*W (or the running ones, see BnRunning);
// saves the mean and reciprocal standard deviation it normalised with.
hipError_t op_batchnorm_fwd(const OpCtx& c, const void* z, const float* g, const float* b, const void* res,
                            void* y, float* mean, float* rstd, int rows, int C, int relu,
                            const BnRunning* run = nullptr, const ConvStats* pre = nullptr);
// dy_eff = relu ? dy * (y > 0) : dy;  dz = bn-backward(dy_eff); dg, db; if dres: dres = dy_eff.
hipError_t op_batchnorm_bwd(const OpCtx& c, const void* dy, const void* y, const void* z, const float* mean,
                            const float* rstd, const float* g, void* dz, void* dres, float* dg, float* db,
                            int rows, int C, int relu, int accumulate);
hipError_t op_avgpool_fwd(const OpCtx& c, const void* x, void* out, int N, int HW, int C);
hipError_t op_avgpool_bwd(const OpCtx& c, const void* dfeat, void* dx, int N, int HW, int C);
hipError_t op_add(const OpCtx& c, const void* a, const void* b, void* out, size_t n);

}  // namespace lp
