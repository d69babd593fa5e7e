// BatchNorm over NHWC activations viewed as [rows = N*H*W, C] with statistics of the current batch
// (biased variance, eps 1e-5), fused with the ReLU and the residual add of a BasicBlock, and the
// global average pool of the classifier head.  Reductions are two-stage with a fixed order.
#include "common.h"

namespace lp {

bool bn_fast_ok(const OpCtx& c, int rows, int C, const void* a, const void* b, const void* cc, const void* d);
hipError_t bn_fwd_fast(const OpCtx& c, const void* z, const float* g, const float* b, const void* res, void* y,
                       float* mean, float* rstd, int rows, int C, int relu, const BnRunning* run, const ConvStats* pre);
hipError_t bn_bwd_fast(const OpCtx& c, const void* dy, const void* y, const void* z, const float* mean,
                       const float* rstd, const float* g, void* dz, void* dres, float* dg, float* db, int rows, int C,
                       int relu, int accumulate);

constexpr float kBnEps = 1e-5f;
constexpr int kSlabRows = 1024;

// MODE 0: sum x.  MODE 1: sum (x - mu)^2.  MODE 2: two sums for backward: dy_eff and dy_eff * xhat.
template <typename T, int MODE>
__global__ void k_bn_partial(const T* a, const T* yrelu, const T* z, const float* mean, const float* rstd,
                             float* partial, int rows, int C, int relu) {
  __shared__ float sh[2][4][64];
  int lc = threadIdx.x & 63, w = threadIdx.x >> 6;
  int col = blockIdx.x * 64 + lc;
  int r0 = blockIdx.y * kSlabRows;
  int r1 = r0 + kSlabRows < rows ? r0 + kSlabRows : rows;
  float s0 = 0.f, s1 = 0.f;
  if (col < C) {
    float mu = (MODE >= 1) ? mean[col] : 0.f;
    float rs = (MODE == 2) ? rstd[col] : 0.f;
    for (int r = r0 + w; r < r1; r += 4) {
      size_t i = (size_t)r * C + col;
      if (MODE == 0) s0 += to_f(a[i]);
      else if (MODE == 1) { float t = to_f(a[i]) - mu; s0 += t * t; }
      else {
        float dy = to_f(a[i]);
        if (relu && !(to_f(yrelu[i]) > 0.f)) dy = 0.f;
        s0 += dy;
        s1 += dy * (to_f(z[i]) - mu) * rs;
      }
    }
  }
  sh[0][w][lc] = s0; sh[1][w][lc] = s1;
  __syncthreads();
  if (w == 0 && col < C) {
    size_t nslab = gridDim.y;
    partial[(size_t)blockIdx.y * C + col] = sh[0][0][lc] + sh[0][1][lc] + sh[0][2][lc] + sh[0][3][lc];
    if (MODE == 2)
      partial[(nslab + blockIdx.y) * C + col] = sh[1][0][lc] + sh[1][1][lc] + sh[1][2][lc] + sh[1][3][lc];
  }
}
// mode 0: out = sum/rows.  mode 1: out = rsqrt(sum/rows + eps).  mode 2: out = sum.
// Block = 64 channels x 4 slab groups; group q adds slabs q, q+4, ... in order, then the four group sums
// are added in order (a fixed tree).
// With ``run`` (modes 0 and 1) the result is also folded into a running statistic: the mean as it is, the
// variance in its unbiased form.
__global__ void k_bn_finalize(const float* partial, int nslab, int C, int rows, float* out, int mode,
                              float* run = nullptr, float momentum = 0.f) {
  __shared__ float sh[4][64];
  int lc = threadIdx.x & 63, q = threadIdx.x >> 6;
  int j = blockIdx.x * 64 + lc;
  float a = 0.f;
  if (j < C)
    for (int b = q; b < nslab; b += 4) a += partial[(size_t)b * C + j];
  sh[q][lc] = a;
  __syncthreads();
  if (q != 0 || j >= C) return;
  a = sh[0][lc] + sh[1][lc] + sh[2][lc] + sh[3][lc];
  if (mode == 0) {
    const float mu = a / (float)rows;
    out[j] = mu;
    if (run) run[j] = (1.f - momentum) * run[j] + momentum * mu;
  } else if (mode == 1) {
    out[j] = rsqrtf(a / (float)rows + kBnEps);
    if (run) run[j] = (1.f - momentum) * run[j] + momentum * (a / (float)(rows > 1 ? rows - 1 : 1));
  } else {
    out[j] = a;
  }
}
// The statistics an evaluation pass normalises with: the running mean, and 1 / sqrt(running variance + eps).
__global__ void k_bn_load_running(const float* run_mean, const float* run_var, float* mean, float* rstd, int C) {
  int j = blockIdx.x * blockDim.x + threadIdx.x;
  if (j < C) { mean[j] = run_mean[j]; rstd[j] = rsqrtf(run_var[j] + kBnEps); }
}
template <typename T>
__global__ void k_bn_apply(const T* z, const float* g, const float* b, const T* res, T* y, const float* mean,
                           const float* rstd, size_t n, int C, int relu) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  size_t st = (size_t)gridDim.x * blockDim.x;
  for (; i < n; i += st) {
    int c = (int)(i % C);
    float v = (to_f(z[i]) - mean[c]) * rstd[c] * g[c] + b[c];
    if (res) v += to_f(res[i]);
    if (relu) v = fmaxf(v, 0.f);
    y[i] = from_f<T>(v);
  }
}
template <typename T>
__global__ void k_bn_bwd_apply(const T* dy, const T* yrelu, const T* z, const float* mean, const float* rstd,
                               const float* g, const float* sums, T* dz, T* dres, size_t n, int C, int rows,
                               int relu) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  size_t st = (size_t)gridDim.x * blockDim.x;
  float inv = 1.f / (float)rows;
  for (; i < n; i += st) {
    int c = (int)(i % C);
    float d = to_f(dy[i]);
    if (relu && !(to_f(yrelu[i]) > 0.f)) d = 0.f;
    float xh = (to_f(z[i]) - mean[c]) * rstd[c];
    float v = g[c] * rstd[c] * (d - sums[c] * inv - xh * sums[C + c] * inv);
    dz[i] = from_f<T>(v);
    if (dres) dres[i] = from_f<T>(d);
  }
}
__global__ void k_accum(const float* src, float* dst, int n, int accumulate) {
  int j = blockIdx.x * blockDim.x + threadIdx.x;
  if (j < n) dst[j] = accumulate ? dst[j] + src[j] : src[j];
}

static int ew_blocks(size_t n) { size_t b = (n + 255) / 256; return (int)(b < 8192 ? b : 8192); }

template <typename T>
static hipError_t bn_fwd_t(const OpCtx& c, const void* z, const float* g, const float* b, const void* res, void* y,
                           float* mean, float* rstd, int rows, int C, int relu, const BnRunning* run) {
  if (!(run && run->use)) {
    int nslab = (rows + kSlabRows - 1) / kSlabRows;
    if ((size_t)nslab * C > c.partial_elems) return hipErrorInvalidValue;
    dim3 grid((C + 63) / 64, nslab);
    float* rm = run ? run->mean : nullptr;
    float* rv = run ? run->var : nullptr;
    float mom = run ? run->momentum : 0.f;
    k_bn_partial<T, 0><<<grid, 256, 0, c.stream>>>((const T*)z, nullptr, nullptr, nullptr, nullptr, c.partial, rows, C, 0);
    k_bn_finalize<<<(C + 63) / 64, 256, 0, c.stream>>>(c.partial, nslab, C, rows, mean, 0, rm, mom);
    k_bn_partial<T, 1><<<grid, 256, 0, c.stream>>>((const T*)z, nullptr, nullptr, mean, nullptr, c.partial, rows, C, 0);
    k_bn_finalize<<<(C + 63) / 64, 256, 0, c.stream>>>(c.partial, nslab, C, rows, rstd, 1, rv, mom);
  }
  size_t n = (size_t)rows * C;
  k_bn_apply<T><<<ew_blocks(n), 256, 0, c.stream>>>((const T*)z, g, b, (const T*)res, (T*)y, mean, rstd, n, C, relu);
  return hipGetLastError();
}
hipError_t op_batchnorm_fwd(const OpCtx& c, const void* z, const float* g, const float* b, const void* res, void* y,
                            float* mean, float* rstd, int rows, int C, int relu, const BnRunning* run,
                            const ConvStats* pre) {
  ProfScope prof_(c, KC_BATCHNORM);
  if (rows == 0) return hipSuccess;
  if (run && (!run->mean || !run->var)) return hipErrorInvalidValue;
  if (run && run->use) k_bn_load_running<<<(C + 255) / 256, 256, 0, c.stream>>>(run->mean, run->var, mean, rstd, C);
  if (bn_fast_ok(c, rows, C, z, y, res, nullptr)) return bn_fwd_fast(c, z, g, b, res, y, mean, rstd, rows, C, relu, run, pre);
  return c.dt == BF16 ? bn_fwd_t<bf16_t>(c, z, g, b, res, y, mean, rstd, rows, C, relu, run)
                      : bn_fwd_t<float>(c, z, g, b, res, y, mean, rstd, rows, C, relu, run);
}

template <typename T>
static hipError_t bn_bwd_t(const OpCtx& c, const void* dy, const void* y, const void* z, const float* mean,
                           const float* rstd, const float* g, void* dz, void* dres, float* dg, float* db, int rows,
                           int C, int relu, int accumulate) {
  int nslab = (rows + kSlabRows - 1) / kSlabRows;
  if ((size_t)(2 * nslab + 2) * C > c.partial_elems) return hipErrorInvalidValue;
  float* sums = c.partial + (size_t)2 * nslab * C;   // [0..C) = sum dy, [C..2C) = sum dy*xhat
  dim3 grid((C + 63) / 64, nslab);
  k_bn_partial<T, 2><<<grid, 256, 0, c.stream>>>((const T*)dy, (const T*)y, (const T*)z, mean, rstd, c.partial, rows, C, relu);
  k_bn_finalize<<<(C + 63) / 64, 256, 0, c.stream>>>(c.partial, nslab, C, rows, sums, 2);
  k_bn_finalize<<<(C + 63) / 64, 256, 0, c.stream>>>(c.partial + (size_t)nslab * C, nslab, C, rows, sums + C, 2);
  size_t n = (size_t)rows * C;
  k_bn_bwd_apply<T><<<ew_blocks(n), 256, 0, c.stream>>>((const T*)dy, (const T*)y, (const T*)z, mean, rstd, g, sums,
                                                       (T*)dz, (T*)dres, n, C, rows, relu);
  k_accum<<<(C + 255) / 256, 256, 0, c.stream>>>(sums, db, C, accumulate);
  k_accum<<<(C + 255) / 256, 256, 0, c.stream>>>(sums + C, dg, C, accumulate);
  return hipGetLastError();
}
hipError_t op_batchnorm_bwd(const OpCtx& c, const void* dy, const void* y, const void* z, const float* mean,
                            const float* rstd, const float* g, void* dz, void* dres, float* dg, float* db, int rows,
                            int C, int relu, int accumulate) {
  ProfScope prof_(c, KC_BATCHNORM);
  if (rows == 0) return hipSuccess;
  if (bn_fast_ok(c, rows, C, dy, y, z, dz) && (!dres || ((uintptr_t)dres & 15) == 0))
    return bn_bwd_fast(c, dy, y, z, mean, rstd, g, dz, dres, dg, db, rows, C, relu, accumulate);
  return c.dt == BF16 ? bn_bwd_t<bf16_t>(c, dy, y, z, mean, rstd, g, dz, dres, dg, db, rows, C, relu, accumulate)
                      : bn_bwd_t<float>(c, dy, y, z, mean, rstd, g, dz, dres, dg, db, rows, C, relu, accumulate);
}

// ------------------------------------------------------------------------------------ pooling
template <typename T>
__global__ void k_avgpool_fwd(const T* x, T* out, int HW, int C) {
  int n = blockIdx.x;
  for (int c = threadIdx.x; c < C; c += blockDim.x) {
    float a = 0.f;
    for (int i = 0; i < HW; ++i) a += to_f(x[((size_t)n * HW + i) * C + c]);
    out[(size_t)n * C + c] = from_f<T>(a / (float)HW);
  }
}
template <typename T>
__global__ void k_avgpool_bwd(const T* dfeat, T* dx, size_t n, int HW, int C) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  size_t st = (size_t)gridDim.x * blockDim.x;
  float inv = 1.f / (float)HW;
  for (; i < n; i += st) {
    size_t img = i / ((size_t)HW * C);
    int c = (int)(i % C);
    dx[i] = from_f<T>(to_f(dfeat[img * C + c]) * inv);
  }
}
// One block per image, 16-byte loads: thread (p, cv) sums channel vector cv over pixels p, p + P, ...
// (P = 256 / channel vectors), then the P partial sums of a channel are added in order of p.
template <typename T>
__global__ void __launch_bounds__(256) k_avgpool_fwd_v(const T* __restrict__ x, T* __restrict__ out, int HW, int C) {
  constexpr int VEC = 16 / (int)sizeof(T);
  typedef T vec_t __attribute__((ext_vector_type(VEC)));
  __shared__ float part[256 * VEC];
  const int CV = C / VEC, P = 256 / CV;
  const int cv = threadIdx.x % CV, p = threadIdx.x / CV;
  const T* xi = x + (size_t)blockIdx.x * HW * C + cv * VEC;
  float a[VEC];
#pragma unroll
  for (int e = 0; e < VEC; ++e) a[e] = 0.f;
  for (int i = p; i < HW; i += P) {
    vec_t v = *reinterpret_cast<const vec_t*>(xi + (size_t)i * C);
#pragma unroll
    for (int e = 0; e < VEC; ++e) a[e] += to_f(v[e]);
  }
#pragma unroll
  for (int e = 0; e < VEC; ++e) part[p * C + cv * VEC + e] = a[e];
  __syncthreads();
  for (int ch = threadIdx.x; ch < C; ch += 256) {
    float t = 0.f;
    for (int q = 0; q < P; ++q) t += part[q * C + ch];
    out[(size_t)blockIdx.x * C + ch] = from_f<T>(t / (float)HW);
  }
}
hipError_t op_avgpool_fwd(const OpCtx& c, const void* x, void* out, int N, int HW, int C) {
  ProfScope prof_(c, KC_OTHER);
  if (N == 0) return hipSuccess;
  const int vec = c.dt == BF16 ? 8 : 4;
  if (C % vec == 0 && C / vec <= 256 && 256 % (C / vec) == 0 && ((uintptr_t)x & 15) == 0) {
    if (c.dt == BF16) k_avgpool_fwd_v<bf16_t><<<N, 256, 0, c.stream>>>((const bf16_t*)x, (bf16_t*)out, HW, C);
    else k_avgpool_fwd_v<float><<<N, 256, 0, c.stream>>>((const float*)x, (float*)out, HW, C);
    return hipGetLastError();
  }
  if (c.dt == BF16) k_avgpool_fwd<bf16_t><<<N, 256, 0, c.stream>>>((const bf16_t*)x, (bf16_t*)out, HW, C);
  else k_avgpool_fwd<float><<<N, 256, 0, c.stream>>>((const float*)x, (float*)out, HW, C);
  return hipGetLastError();
}
hipError_t op_avgpool_bwd(const OpCtx& c, const void* dfeat, void* dx, int N, int HW, int C) {
  ProfScope prof_(c, KC_OTHER);
  size_t n = (size_t)N * HW * C;
  if (n == 0) return hipSuccess;
  if (c.dt == BF16) k_avgpool_bwd<bf16_t><<<ew_blocks(n), 256, 0, c.stream>>>((const bf16_t*)dfeat, (bf16_t*)dx, n, HW, C);
  else k_avgpool_bwd<float><<<ew_blocks(n), 256, 0, c.stream>>>((const float*)dfeat, (float*)dx, n, HW, C);
  return hipGetLastError();
}

}  // namespace lp
