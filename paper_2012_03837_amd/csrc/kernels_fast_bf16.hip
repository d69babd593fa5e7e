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

constexpr int kRowsPerBlock = 16;
// Backward; block partials of dg and db go to partial[blk][d] and partial[nblk + blk][d].  A wave owns four
// rows of its block's sixteen and keeps the next row's loads (x, dy and the addend, 16 bytes per lane each) in
// flight while it reduces and writes the current one: with one row at a time the kernel is a chain of memory
// latencies, not a stream.
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
  constexpr int RPW = kRowsPerBlock / 4;
  bf16x8 xr[2][NCH], dr[2][NCH], ar[2][NCH];
  float mu[2], rs[2];
  auto fetch = [&](int slot, int row) {
    if (row >= rows) return;
    mu[slot] = mean[row]; rs[slot] = rstd[row];
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
      const int c = lane + 64 * i;
      if (c < nch) {
        xr[slot][i] = *reinterpret_cast<const bf16x8*>(x + (size_t)row * d + 8 * c);
        dr[slot][i] = *reinterpret_cast<const bf16x8*>(dy + (size_t)row * d + 8 * c);
        if (add && dx) ar[slot][i] = *reinterpret_cast<const bf16x8*>(add + (size_t)row * d + 8 * c);
      }
    }
  };
  fetch(0, row0 + w);
#pragma unroll
  for (int it = 0; it < RPW; ++it) {
    const int row = row0 + w + 4 * it, cur = it & 1;
    if (row >= rows) break;
    if (it + 1 < RPW) fetch(cur ^ 1, row + 4);
    float xh[NCH][8], dxh[NCH][8];
    float s1 = 0.f, s2 = 0.f;
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
      if (lane + 64 * i < nch) {
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const float dv = (float)dr[cur][i][e];
          xh[i][e] = ((float)xr[cur][i][e] - mu[cur]) * rs[cur];
          dxh[i][e] = dv * gg[i][e];
          s1 += dxh[i][e];
          s2 += dxh[i][e] * xh[i][e];
          pg[i][e] += dv * xh[i][e];
          pb[i][e] += dv;
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
          for (int e = 0; e < 8; ++e) o[e] = (dxh[i][e] - s1 - xh[i][e] * s2) * rs[cur];
          if (add) {
#pragma unroll
            for (int e = 0; e < 8; ++e) o[e] += (float)ar[cur][i][e];
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
      v[i] = __builtin_nontemporal_load(reinterpret_cast<const bf16x8*>(zr + 8 * c));
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
      __builtin_nontemporal_store(o, reinterpret_cast<bf16x8*>(zr + 8 * c));
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

// ===================================================================================================
// BatchNorm over [rows, C] bf16 with C % 8 == 0: 16 bytes (8 channels) per lane.
//   statistics : one pass; per-channel sums of (x - p) and (x - p)^2 with the pivot p = the channel's
//                value in row 0 (a sample of the distribution, so the shifted variance formula
//                S2/n - (S1/n)^2 does not cancel), per-slab partials, ordered reduction
//   apply      : y = [relu]((z - mean) * rstd * g + b (+ res))
//   backward   : per-slab partial sums of dy_eff and dy_eff * xhat, then
//                dz = g * rstd * (dy_eff - mean(dy_eff) - xhat * mean(dy_eff * xhat)), dres = dy_eff
// Block = (C/8) channel chunks x (256 / (C/8)) row lanes; C <= 2048.
namespace lp {
namespace {

constexpr float kBnEpsV = 1e-5f;

// MODE 0: s0 = sum (z - p), s1 = sum (z - p)^2.   MODE 1: s0 = sum dy_eff, s1 = sum dy_eff * xhat.
template <int MODE>
__global__ void __launch_bounds__(256) k_bn_partial_v(const bf16_t* __restrict__ a, const bf16_t* __restrict__ yrelu,
                                                      const bf16_t* __restrict__ z, const float* __restrict__ mean,
                                                      const float* __restrict__ rstd, float* __restrict__ partial,
                                                      int rows, int C, int slab, int relu) {
  extern __shared__ float sh[];        // [2][RL][C]
  const int cpr = C >> 3, RL = 256 / cpr;
  const int cc = threadIdx.x % cpr, rl = threadIdx.x / cpr;
  const int r0 = blockIdx.x * slab;
  const int r1 = r0 + slab < rows ? r0 + slab : rows;
  float s0[8], s1[8], p[8], q[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) { s0[e] = 0.f; s1[e] = 0.f; }
  if (rl < RL) {
    if (MODE == 0) load8(z + 8 * cc, p);                      // pivot: row 0
    else { loadf8(mean + 8 * cc, p); loadf8(rstd + 8 * cc, q); }
    for (int r = r0 + rl; r < r1; r += RL) {
      const size_t off = (size_t)r * C + 8 * cc;
      float v[8];
      load8(a + off, v);
      if (MODE == 0) {
#pragma unroll
        for (int e = 0; e < 8; ++e) { float t = v[e] - p[e]; s0[e] += t; s1[e] += t * t; }
      } else {
        float zz[8];
        load8(z + off, zz);
        if (relu) {
          float yy[8];
          load8(yrelu + off, yy);
#pragma unroll
          for (int e = 0; e < 8; ++e) v[e] = yy[e] > 0.f ? v[e] : 0.f;
        }
#pragma unroll
        for (int e = 0; e < 8; ++e) { s0[e] += v[e]; s1[e] += v[e] * (zz[e] - p[e]) * q[e]; }
      }
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      sh[(size_t)rl * C + 8 * cc + e] = s0[e];
      sh[(size_t)(RL + rl) * C + 8 * cc + e] = s1[e];
    }
  }
  __syncthreads();
  const int nslab = gridDim.x;
  for (int j = threadIdx.x; j < C; j += 256) {
    float t0 = 0.f, t1 = 0.f;
    for (int r = 0; r < RL; ++r) { t0 += sh[(size_t)r * C + j]; t1 += sh[(size_t)(RL + r) * C + j]; }
    partial[(size_t)blockIdx.x * C + j] = t0;
    partial[(size_t)(nslab + blockIdx.x) * C + j] = t1;
  }
}
// Adds the slab partials in order (64 channels x 16 slab groups per block: group q adds slabs q, q+16, ...
// with two independent pairs of loads in flight, then the group sums are added in order) and finishes.
// mode 0: forward statistics (needs the pivots from row 0 of z); with aux0 / aux1 the batch mean and unbiased
// variance are also folded into those running statistics with weight auxf.  mode 1: plain sums into out0, out1;
// with aux0 / aux1 they are also written (auxf == 0) or added (auxf != 0) there: the shift and gain gradients.
constexpr int kBnFinishGroups = 16;
__global__ void __launch_bounds__(64 * kBnFinishGroups)
k_bn_finish_v(const float* __restrict__ partial, int nslab, int C, int rows, const bf16_t* __restrict__ z,
              float* __restrict__ out0, float* __restrict__ out1, int mode, float* __restrict__ aux0 = nullptr,
              float* __restrict__ aux1 = nullptr, float auxf = 0.f) {
  __shared__ float sh[2][kBnFinishGroups][64];
  const int lc = threadIdx.x & 63, q = threadIdx.x >> 6;
  const int j = blockIdx.x * 64 + lc;
  float a = 0.f, b = 0.f;
  if (j < C) {
    int s = q;
    for (; s + 3 * kBnFinishGroups < nslab; s += 4 * kBnFinishGroups) {      // eight loads in flight
      float av[4], bv[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        av[u] = partial[(size_t)(s + u * kBnFinishGroups) * C + j];
        bv[u] = partial[(size_t)(nslab + s + u * kBnFinishGroups) * C + j];
      }
#pragma unroll
      for (int u = 0; u < 4; ++u) { a += av[u]; b += bv[u]; }
    }
    for (; s + kBnFinishGroups < nslab; s += 2 * kBnFinishGroups) {
      const float a0 = partial[(size_t)s * C + j], b0 = partial[(size_t)(nslab + s) * C + j];
      const float a1 = partial[(size_t)(s + kBnFinishGroups) * C + j], b1 = partial[(size_t)(nslab + s + kBnFinishGroups) * C + j];
      a += a0; a += a1; b += b0; b += b1;
    }
    for (; s < nslab; s += kBnFinishGroups) { a += partial[(size_t)s * C + j]; b += partial[(size_t)(nslab + s) * C + j]; }
  }
  sh[0][q][lc] = a; sh[1][q][lc] = b;
  __syncthreads();
  if (q != 0 || j >= C) return;
  a = 0.f; b = 0.f;
#pragma unroll
  for (int g = 0; g < kBnFinishGroups; ++g) { a += sh[0][g][lc]; b += sh[1][g][lc]; }
  if (mode == 0) {
    const float inv = 1.f / (float)rows, m1 = a * inv;
    float var = b * inv - m1 * m1;
    var = var > 0.f ? var : 0.f;
    const float mu = (float)z[j] + m1;
    out0[j] = mu;
    out1[j] = rsqrtf(var + kBnEpsV);
    if (aux0) {   // running statistics take the unbiased batch variance
      const float unb = rows > 1 ? var * ((float)rows / (float)(rows - 1)) : var;
      aux0[j] = (1.f - auxf) * aux0[j] + auxf * mu;
      aux1[j] = (1.f - auxf) * aux1[j] + auxf * unb;
    }
  } else {
    out0[j] = a; out1[j] = b;
    if (aux0) {
      aux0[j] = auxf != 0.f ? aux0[j] + a : a;
      aux1[j] = auxf != 0.f ? aux1[j] + b : b;
    }
  }
}
// Forward statistics from the per-slab sums the convolution kernel left (ConvStats: slab t has its own pivot p_t, the
// first of its slab_rows rows): every slab is shifted to slab 0's pivot P, with d = p_t - P
//   sum (z - P) = s0_t + n d,   sum (z - P)^2 = s1_t + 2 d s0_t + n d^2,
// the slabs are added in the order of k_bn_finish_v (16 groups of every 16th slab, then the groups in order), and the
// batch mean, 1 / sqrt(var + eps) and the running pair follow as there.
__global__ void __launch_bounds__(64 * kBnFinishGroups)
k_bn_finish_slabs(const float* __restrict__ st, int nslab, int slab_rows, int C, int rows, float* __restrict__ mean,
                  float* __restrict__ rstd, float* __restrict__ run_mean, float* __restrict__ run_var, float mom) {
  __shared__ float sh[2][kBnFinishGroups][64];
  const int lc = threadIdx.x & 63, q = threadIdx.x >> 6;
  const int j = blockIdx.x * 64 + lc;
  float a = 0.f, b = 0.f, P = 0.f;
  if (j < C) {
    const float* s0p = st + j;
    const float* s1p = st + (size_t)nslab * C + j;
    const float* pp = st + (size_t)2 * nslab * C + j;
    P = pp[0];
    const float n = (float)slab_rows;
    int s = q;
    for (; s + 3 * kBnFinishGroups < nslab; s += 4 * kBnFinishGroups) {      // twelve loads in flight
      float s0[4], s1[4], p[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const size_t o = (size_t)(s + u * kBnFinishGroups) * C;
        s0[u] = s0p[o]; s1[u] = s1p[o]; p[u] = pp[o];
      }
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const float d = p[u] - P;
        a += s0[u] + n * d;
        b += s1[u] + 2.f * d * s0[u] + n * d * d;
      }
    }
    for (; s < nslab; s += kBnFinishGroups) {
      const size_t o = (size_t)s * C;
      const float s0 = s0p[o], s1 = s1p[o], d = pp[o] - P;
      a += s0 + n * d;
      b += s1 + 2.f * d * s0 + n * d * d;
    }
  }
  sh[0][q][lc] = a; sh[1][q][lc] = b;
  __syncthreads();
  if (q != 0 || j >= C) return;
  a = 0.f; b = 0.f;
#pragma unroll
  for (int g = 0; g < kBnFinishGroups; ++g) { a += sh[0][g][lc]; b += sh[1][g][lc]; }
  const float inv = 1.f / (float)rows, m1 = a * inv;
  float var = b * inv - m1 * m1;
  var = var > 0.f ? var : 0.f;
  const float mu = P + m1;
  mean[j] = mu;
  rstd[j] = rsqrtf(var + kBnEpsV);
  if (run_mean) {   // running statistics take the unbiased batch variance
    const float unb = rows > 1 ? var * ((float)rows / (float)(rows - 1)) : var;
    run_mean[j] = (1.f - mom) * run_mean[j] + mom * mu;
    run_var[j] = (1.f - mom) * run_var[j] + mom * unb;
  }
}
__global__ void __launch_bounds__(256) k_bn_apply_v(const bf16_t* __restrict__ z, const float* __restrict__ g,
                                                    const float* __restrict__ b, const bf16_t* __restrict__ res,
                                                    bf16_t* __restrict__ y, const float* __restrict__ mean,
                                                    const float* __restrict__ rstd, size_t nchunks, int C, int relu) {
  size_t i = (size_t)blockIdx.x * 256 + threadIdx.x, st = (size_t)gridDim.x * 256;
  for (; i < nchunks; i += st) {
    const int c = (int)((i * 8) % C);
    float v[8], gg[8], bb[8], mu[8], rs[8];
    load8(z + i * 8, v); loadf8(g + c, gg); loadf8(b + c, bb); loadf8(mean + c, mu); loadf8(rstd + c, rs);
#pragma unroll
    for (int e = 0; e < 8; ++e) v[e] = (v[e] - mu[e]) * rs[e] * gg[e] + bb[e];
    if (res) {
      float r[8];
      load8(res + i * 8, r);
#pragma unroll
      for (int e = 0; e < 8; ++e) v[e] += r[e];
    }
    if (relu) {
#pragma unroll
      for (int e = 0; e < 8; ++e) v[e] = fmaxf(v[e], 0.f);
    }
    store8(y + i * 8, v);
  }
}
__global__ void __launch_bounds__(256) k_bn_bwd_apply_v(const bf16_t* __restrict__ dy, const bf16_t* __restrict__ yrelu,
                                                        const bf16_t* __restrict__ z, const float* __restrict__ mean,
                                                        const float* __restrict__ rstd, const float* __restrict__ g,
                                                        const float* __restrict__ sums, bf16_t* __restrict__ dz,
                                                        bf16_t* __restrict__ dres, size_t nchunks, int C, int rows,
                                                        int relu) {
  size_t i = (size_t)blockIdx.x * 256 + threadIdx.x, st = (size_t)gridDim.x * 256;
  const float inv = 1.f / (float)rows;
  for (; i < nchunks; i += st) {
    const int c = (int)((i * 8) % C);
    float d[8], zz[8], mu[8], rs[8], gg[8], s0[8], s1[8], o[8];
    load8(dy + i * 8, d); load8(z + i * 8, zz);
    loadf8(mean + c, mu); loadf8(rstd + c, rs); loadf8(g + c, gg); loadf8(sums + c, s0); loadf8(sums + C + c, s1);
    if (relu) {
      float yy[8];
      load8(yrelu + i * 8, yy);
#pragma unroll
      for (int e = 0; e < 8; ++e) d[e] = yy[e] > 0.f ? d[e] : 0.f;
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      float xh = (zz[e] - mu[e]) * rs[e];
      o[e] = gg[e] * rs[e] * (d[e] - s0[e] * inv - xh * s1[e] * inv);
    }
    store8(dz + i * 8, o);
    if (dres) store8(dres + i * 8, d);
  }
}

int bn_slab(int rows, int C) {
  int RL = 256 / (C / 8);
  int slab = (rows + 1023) / 1024;         // aim at about a thousand blocks
  int min_slab = RL * 8;
  if (slab < min_slab) slab = min_slab;
  return slab;
}
int blocks_for(size_t n) { size_t b = (n + 255) / 256; return (int)(b < 16384 ? b : 16384); }

}  // namespace

bool bn_fast_ok(const OpCtx& c, int rows, int C, const void* a, const void* b, const void* cc, const void* d) {
  if (c.dt != BF16 || C % 8 || C < 8 || C > 2048 || (256 % (C / 8)) || rows < 1) return false;
  return al16(a) && al16(b) && (!cc || al16(cc)) && (!d || al16(d));
}
size_t bn_fast_scratch(int rows, int C) {
  int slab = bn_slab(rows, C);
  size_t nslab = (rows + slab - 1) / slab;
  return (2 * nslab + 2) * (size_t)C;
}
hipError_t bn_fwd_fast(const OpCtx& c, const void* z, const float* g, const float* b, const void* res, void* y,
                       float* mean, float* rstd, int rows, int C, int relu, const BnRunning* run, const ConvStats* pre) {
  const bool given = run && run->use;   // mean / rstd already hold the statistics to normalise with
  if (!given && pre && pre->nslab > 0 && (size_t)pre->nslab * pre->slab_rows == (size_t)rows) {
    // the convolution in front left the per-slab sums: no pass over z for the statistics
    k_bn_finish_slabs<<<(C + 63) / 64, 64 * kBnFinishGroups, 0, c.stream>>>(
        pre->buf, pre->nslab, pre->slab_rows, C, rows, mean, rstd, run ? run->mean : nullptr, run ? run->var : nullptr,
        run ? run->momentum : 0.f);
  } else if (!given) {
    const int slab = bn_slab(rows, C), nslab = (rows + slab - 1) / slab;
    if ((size_t)2 * nslab * C > c.partial_elems) return hipErrorInvalidValue;
    const int RL = 256 / (C / 8);
    const size_t shm = (size_t)2 * RL * C * sizeof(float);
    k_bn_partial_v<0><<<nslab, 256, shm, c.stream>>>((const bf16_t*)z, nullptr, (const bf16_t*)z, nullptr, nullptr,
                                                     c.partial, rows, C, slab, 0);
    k_bn_finish_v<<<(C + 63) / 64, 64 * kBnFinishGroups, 0, c.stream>>>(
        c.partial, nslab, C, rows, (const bf16_t*)z, mean, rstd, 0, run ? run->mean : nullptr,
        run ? run->var : nullptr, run ? run->momentum : 0.f);
  }
  const size_t nch = (size_t)rows * C / 8;
  k_bn_apply_v<<<blocks_for(nch), 256, 0, c.stream>>>((const bf16_t*)z, g, b, (const bf16_t*)res, (bf16_t*)y, mean, rstd,
                                                     nch, C, relu);
  return hipGetLastError();
}
hipError_t bn_bwd_fast(const OpCtx& c, const void* dy, const void* y, const void* z, const float* mean,
                       const float* rstd, const float* g, void* dz, void* dres, float* dg, float* db, int rows, int C,
                       int relu, int accumulate) {
  const int slab = bn_slab(rows, C), nslab = (rows + slab - 1) / slab;
  if ((size_t)(2 * nslab + 2) * C > c.partial_elems) return hipErrorInvalidValue;
  float* sums = c.partial + (size_t)2 * nslab * C;
  const int RL = 256 / (C / 8);
  const size_t shm = (size_t)2 * RL * C * sizeof(float);
  k_bn_partial_v<1><<<nslab, 256, shm, c.stream>>>((const bf16_t*)dy, (const bf16_t*)y, (const bf16_t*)z, mean, rstd,
                                                   c.partial, rows, C, slab, relu);
  k_bn_finish_v<<<(C + 63) / 64, 64 * kBnFinishGroups, 0, c.stream>>>(c.partial, nslab, C, rows, nullptr, sums, sums + C, 1,
                                                                      db, dg, accumulate ? 1.f : 0.f);
  const size_t nch = (size_t)rows * C / 8;
  k_bn_bwd_apply_v<<<blocks_for(nch), 256, 0, c.stream>>>((const bf16_t*)dy, (const bf16_t*)y, (const bf16_t*)z, mean,
                                                         rstd, g, sums, (bf16_t*)dz, (bf16_t*)dres, nch, C, rows, relu);
  return hipGetLastError();
}

}  // namespace lp
