// Vectorised bf16 forms of the HBM-bound kernels: one global read and one global write per element,
// 16 bytes per lane, all intermediate values in registers.
//   LayerNorm forward / backward : rows of up to 1024 elements, one wavefront per row
//   softmax cross-entropy        : rows of up to 32768 logits, one 256-thread block per row
// Shapes outside these limits (or unaligned) use the generic kernels.
#include "common.h"

namespace lp {

namespace {

__device__ __forceinline__ float wsum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
__device__ __forceinline__ float wmax(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}
__device__ __forceinline__ void load8(const bf16_t* p, float* v) {
  bf16x8 t = *reinterpret_cast<const bf16x8*>(p);
#pragma unroll
  for (int e = 0; e < 8; ++e) v[e] = (float)t[e];
}
__device__ __forceinline__ void store8(bf16_t* p, const float* v) {
  bf16x8 t;
#pragma unroll
  for (int e = 0; e < 8; ++e) t[e] = (bf16_t)v[e];
  *reinterpret_cast<bf16x8*>(p) = t;
}
__device__ __forceinline__ void loadf8(const float* p, float* v) {
  f32x4 a = *reinterpret_cast<const f32x4*>(p), b = *reinterpret_cast<const f32x4*>(p + 4);
#pragma unroll
  for (int e = 0; e < 4; ++e) { v[e] = a[e]; v[4 + e] = b[e]; }
}

constexpr float kEps = 1e-5f;

template <int NCH>
__global__ void __launch_bounds__(256) k_ln_fwd_v(const bf16_t* __restrict__ x, const float* __restrict__ g,
                                                  const float* __restrict__ b, bf16_t* __restrict__ y,
                                                  float* __restrict__ mean, float* __restrict__ rstd, int rows, int d) {
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
  if (row >= rows) return;
  const int nch = d >> 3;
  const bf16_t* xr = x + (size_t)row * d;
  float v[NCH][8];
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < NCH; ++i) {
    int c = lane + 64 * i;
    if (c < nch) {
      load8(xr + 8 * c, v[i]);
#pragma unroll
      for (int e = 0; e < 8; ++e) s += v[i][e];
    }
  }
  const float mu = wsum(s) / (float)d;
  float q = 0.f;
#pragma unroll
  for (int i = 0; i < NCH; ++i)
    if (lane + 64 * i < nch) {
#pragma unroll
      for (int e = 0; e < 8; ++e) { float t = v[i][e] - mu; q += t * t; }
    }
  const float rs = rsqrtf(wsum(q) / (float)d + kEps);
  bf16_t* yr = y + (size_t)row * d;
#pragma unroll
  for (int i = 0; i < NCH; ++i) {
    int c = lane + 64 * i;
    if (c < nch) {
      float gg[8], bb[8], o[8];
      loadf8(g + 8 * c, gg); loadf8(b + 8 * c, bb);
#pragma unroll
      for (int e = 0; e < 8; ++e) o[e] = (v[i][e] - mu) * rs * gg[e] + bb[e];
      store8(yr + 8 * c, o);
    }
  }
  if (lane == 0) { mean[row] = mu; rstd[row] = rs; }
}

constexpr int kRowsPerBlock = 32;
// Backward; block partials of dg and db go to partial[blk][d] and partial[nblk + blk][d].
template <int NCH>
__global__ void __launch_bounds__(256) k_ln_bwd_v(const bf16_t* __restrict__ dy, const bf16_t* __restrict__ x,
                                                  const float* __restrict__ mean, const float* __restrict__ rstd,
                                                  const float* __restrict__ g, const bf16_t* __restrict__ add,
                                                  bf16_t* __restrict__ dx, float* __restrict__ partial, int rows,
                                                  int d) {
  extern __shared__ float sh[];   // [4 waves][2][d]
  const int w = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int nch = d >> 3;
  float gg[NCH][8], pg[NCH][8], pb[NCH][8];
#pragma unroll
  for (int i = 0; i < NCH; ++i) {
    int c = lane + 64 * i;
#pragma unroll
    for (int e = 0; e < 8; ++e) { pg[i][e] = 0.f; pb[i][e] = 0.f; gg[i][e] = 0.f; }
    if (c < nch) loadf8(g + 8 * c, gg[i]);
  }
  const int row0 = blockIdx.x * kRowsPerBlock;
  const float invd = 1.f / (float)d;
  for (int r = w; r < kRowsPerBlock; r += 4) {
    const int row = row0 + r;
    if (row >= rows) break;
    const float mu = mean[row], rs = rstd[row];
    float xh[NCH][8], dxh[NCH][8];
    float s1 = 0.f, s2 = 0.f;
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
      int c = lane + 64 * i;
      if (c < nch) {
        float xv[8], dv[8];
        load8(x + (size_t)row * d + 8 * c, xv);
        load8(dy + (size_t)row * d + 8 * c, dv);
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          xh[i][e] = (xv[e] - mu) * rs;
          dxh[i][e] = dv[e] * gg[i][e];
          s1 += dxh[i][e];
          s2 += dxh[i][e] * xh[i][e];
          pg[i][e] += dv[e] * xh[i][e];
          pb[i][e] += dv[e];
        }
      }
    }
    s1 = wsum(s1) * invd;
    s2 = wsum(s2) * invd;
    if (dx) {
#pragma unroll
      for (int i = 0; i < NCH; ++i) {
        int c = lane + 64 * i;
        if (c < nch) {
          float o[8];
#pragma unroll
          for (int e = 0; e < 8; ++e) o[e] = (dxh[i][e] - s1 - xh[i][e] * s2) * rs;
          if (add) {
            float a[8];
            load8(add + (size_t)row * d + 8 * c, a);
#pragma unroll
            for (int e = 0; e < 8; ++e) o[e] += a[e];
          }
          store8(dx + (size_t)row * d + 8 * c, o);
        }
      }
    }
  }
#pragma unroll
  for (int i = 0; i < NCH; ++i) {
    int c = lane + 64 * i;
    if (c < nch) {
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        sh[(size_t)(w * 2) * d + 8 * c + e] = pg[i][e];
        sh[(size_t)(w * 2 + 1) * d + 8 * c + e] = pb[i][e];
      }
    }
  }
  __syncthreads();
  const int nblk = gridDim.x;
  for (int j = threadIdx.x; j < d; j += 256) {
    float a = 0.f, bsum = 0.f;
#pragma unroll
    for (int ww = 0; ww < 4; ++ww) { a += sh[(size_t)(ww * 2) * d + j]; bsum += sh[(size_t)(ww * 2 + 1) * d + j]; }
    partial[(size_t)blockIdx.x * d + j] = a;
    partial[(size_t)(nblk + blockIdx.x) * d + j] = bsum;
  }
}

// Softmax cross-entropy with the whole row in registers (<= 16 chunks of 8 logits per thread).
constexpr int kCeChunks = 16;
__global__ void __launch_bounds__(256) k_softmax_ce_reg(bf16_t* __restrict__ z, int64_t ld, const int32_t* __restrict__ y,
                                                        float* __restrict__ loss_rows, int n, int write_grad,
                                                        float inv_rows) {
  __shared__ float sh[8];
  const int row = blockIdx.x, nch = n >> 3;
  bf16_t* zr = z + (size_t)row * ld;
  bf16x8 v[kCeChunks];
  float m = -INFINITY;
#pragma unroll
  for (int i = 0; i < kCeChunks; ++i) {
    int c = threadIdx.x + 256 * i;
    if (c < nch) {
      v[i] = *reinterpret_cast<const bf16x8*>(zr + 8 * c);
#pragma unroll
      for (int e = 0; e < 8; ++e) m = fmaxf(m, (float)v[i][e]);
    }
  }
  m = wmax(m);
  if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = m;
  __syncthreads();
  m = fmaxf(fmaxf(sh[0], sh[1]), fmaxf(sh[2], sh[3]));
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < kCeChunks; ++i)
    if (threadIdx.x + 256 * i < nch) {
#pragma unroll
      for (int e = 0; e < 8; ++e) s += __expf((float)v[i][e] - m);
    }
  s = wsum(s);
  if ((threadIdx.x & 63) == 0) sh[4 + (threadIdx.x >> 6)] = s;
  __syncthreads();
  s = sh[4] + sh[5] + sh[6] + sh[7];
  const float lse = m + __logf(s);
  const int yy = y[row];
  const bool y_ok = yy >= 0 && yy < n;
  if (threadIdx.x == 0) loss_rows[row] = lse - (y_ok ? (float)zr[yy] : 0.f);
  if (!write_grad) return;
  __syncthreads();   // the label's logit has been read before anything is overwritten
#pragma unroll
  for (int i = 0; i < kCeChunks; ++i) {
    int c = threadIdx.x + 256 * i;
    if (c < nch) {
      bf16x8 o;
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        float p = __expf((float)v[i][e] - lse);
        if (8 * c + e == yy) p -= 1.f;
        o[e] = (bf16_t)(p * inv_rows);
      }
      *reinterpret_cast<bf16x8*>(zr + 8 * c) = o;
    }
  }
}

bool al16(const void* p) { return ((uintptr_t)p & 15) == 0; }

}  // namespace

bool ln_fast_ok(const OpCtx& c, const void* a, const void* b, const void* cc, const void* dd, int d) {
  return c.dt == BF16 && d % 8 == 0 && d <= 1024 && al16(a) && al16(b) && (!cc || al16(cc)) && (!dd || al16(dd));
}
hipError_t ln_fwd_fast(const OpCtx& c, const void* x, const float* g, const float* b, void* y, float* mean, float* rstd,
                       int rows, int d) {
  int blocks = (rows + 3) / 4;
  if (d <= 512) k_ln_fwd_v<1><<<blocks, 256, 0, c.stream>>>((const bf16_t*)x, g, b, (bf16_t*)y, mean, rstd, rows, d);
  else k_ln_fwd_v<2><<<blocks, 256, 0, c.stream>>>((const bf16_t*)x, g, b, (bf16_t*)y, mean, rstd, rows, d);
  return hipGetLastError();
}
// Launches the backward kernel only; the caller reduces the partials (nblk blocks of d floats, twice).
hipError_t ln_bwd_fast(const OpCtx& c, const void* dy, const void* x, const float* mean, const float* rstd,
                       const float* g, const void* add, void* dx, int rows, int d, int* nblk_out) {
  int nblk = (rows + kRowsPerBlock - 1) / kRowsPerBlock;
  *nblk_out = nblk;
  if ((size_t)nblk * d * 2 > c.partial_elems) return hipErrorInvalidValue;
  size_t shm = (size_t)8 * d * sizeof(float);
  if (d <= 512)
    k_ln_bwd_v<1><<<nblk, 256, shm, c.stream>>>((const bf16_t*)dy, (const bf16_t*)x, mean, rstd, g, (const bf16_t*)add,
                                                (bf16_t*)dx, c.partial, rows, d);
  else
    k_ln_bwd_v<2><<<nblk, 256, shm, c.stream>>>((const bf16_t*)dy, (const bf16_t*)x, mean, rstd, g, (const bf16_t*)add,
                                                (bf16_t*)dx, c.partial, rows, d);
  return hipGetLastError();
}
bool ce_fast_ok(const OpCtx& c, const void* z, int64_t ld, int n) {
  return c.dt == BF16 && n % 8 == 0 && ld % 8 == 0 && n <= kCeChunks * 256 * 8 && al16(z);
}
hipError_t ce_fast(const OpCtx& c, void* z, int64_t ld, const int32_t* y, float* loss_rows, int rows, int n,
                   int write_grad, float inv_rows) {
  k_softmax_ce_reg<<<rows, 256, 0, c.stream>>>((bf16_t*)z, ld, y, loss_rows, n, write_grad, inv_rows);
  return hipGetLastError();
}

}  // namespace lp
