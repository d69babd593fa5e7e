// Memory-bound kernels: fills and casts, embedding, LayerNorm, column sums, softmax cross-entropy,
// the fused optimizer update, and the weight initialiser.  64-wide wavefront reductions; every
// reduction has a fixed order, so repeated runs are bit-identical.
#include "common.h"

namespace lp {

bool ln_fast_ok(const OpCtx& c, const void* a, const void* b, const void* cc, const void* dd, int d);
hipError_t ln_fwd_fast(const OpCtx& c, const void* x, const float* g, const float* b, void* y, float* mean, float* rstd,
                       int rows, int d);
hipError_t ln_bwd_fast(const OpCtx& c, const void* dy, const void* x, const float* mean, const float* rstd,
                       const float* g, const void* add, void* dx, int rows, int d, int* nblk_out);
bool ce_fast_ok(const OpCtx& c, const void* z, int64_t ld, int n);
hipError_t ce_fast(const OpCtx& c, void* z, int64_t ld, const int32_t* y, float* loss_rows, int rows, int n,
                   int write_grad, float inv_rows);

#define LP_LAUNCH_CHECK() hipGetLastError()

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}
// Sum over a block of 256 threads (4 waves); result valid in every thread.  `sh` holds >= 4 floats.
__device__ __forceinline__ float block_sum_256(float v, float* sh) {
  v = wave_sum(v);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = v;
  __syncthreads();
  return sh[0] + sh[1] + sh[2] + sh[3];
}
__device__ __forceinline__ float block_max_256(float v, float* sh) {
  v = wave_max(v);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = v;
  __syncthreads();
  return fmaxf(fmaxf(sh[0], sh[1]), fmaxf(sh[2], sh[3]));
}

// ------------------------------------------------------------------------------------ fill / cast
__global__ void k_fill_f32(float* p, size_t n, float v) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  size_t st = (size_t)gridDim.x * blockDim.x;
  for (; i < n; i += st) p[i] = v;
}
hipError_t op_fill_f32(const OpCtx& c, float* p, size_t n, float v) {
  if (n == 0) return hipSuccess;
  int blocks = (int)((n + 255) / 256 < 4096 ? (n + 255) / 256 : 4096);
  k_fill_f32<<<blocks, 256, 0, c.stream>>>(p, n, v);
  return LP_LAUNCH_CHECK();
}

// Plain device copy, 16 bytes per lane: the known-size kernel against which hardware traffic counters
// are scaled.
__global__ void k_copy16(const uint4* __restrict__ src, uint4* __restrict__ dst, size_t n16) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  size_t st = (size_t)gridDim.x * blockDim.x;
  for (; i < n16; i += st) dst[i] = src[i];
}
hipError_t op_copy(const OpCtx& c, const void* src, void* dst, size_t bytes) {
  if (bytes == 0) return hipSuccess;
  size_t n16 = bytes / 16;
  int blocks = (int)((n16 + 255) / 256 < 16384 ? (n16 + 255) / 256 : 16384);
  k_copy16<<<blocks, 256, 0, c.stream>>>((const uint4*)src, (uint4*)dst, n16);
  return LP_LAUNCH_CHECK();
}

template <typename T>
__global__ void k_cast(const float* src, T* dst, size_t n) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  size_t st = (size_t)gridDim.x * blockDim.x;
  for (; i < n; i += st) dst[i] = from_f<T>(src[i]);
}
hipError_t op_cast_to_compute(const OpCtx& c, const float* src, void* dst, size_t n) {
  if (n == 0) return hipSuccess;
  int blocks = (int)((n + 255) / 256 < 8192 ? (n + 255) / 256 : 8192);
  if (c.dt == BF16) k_cast<bf16_t><<<blocks, 256, 0, c.stream>>>(src, (bf16_t*)dst, n);
  else k_cast<float><<<blocks, 256, 0, c.stream>>>(src, (float*)dst, n);
  return LP_LAUNCH_CHECK();
}

template <typename T>
__global__ void k_add(const T* a, const T* b, T* out, size_t n) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  size_t st = (size_t)gridDim.x * blockDim.x;
  for (; i < n; i += st) out[i] = from_f<T>(to_f(a[i]) + to_f(b[i]));
}
hipError_t op_add(const OpCtx& c, const void* a, const void* b, void* out, size_t n) {
  ProfScope prof_(c, KC_OTHER);
  if (n == 0) return hipSuccess;
  int blocks = (int)((n + 255) / 256 < 8192 ? (n + 255) / 256 : 8192);
  if (c.dt == BF16) k_add<bf16_t><<<blocks, 256, 0, c.stream>>>((const bf16_t*)a, (const bf16_t*)b, (bf16_t*)out, n);
  else k_add<float><<<blocks, 256, 0, c.stream>>>((const float*)a, (const float*)b, (float*)out, n);
  return LP_LAUNCH_CHECK();
}

// ------------------------------------------------------------------------------------ embedding
// Fixed sinusoidal positions, evaluated once in double precision at init:
// pe[s, 2i] = sin(s / 10000^(2i/d)), pe[s, 2i+1] = cos(same angle).
__global__ void k_posenc(float* pe, int S, int d) {
  int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= S * d) return;
  int s = i / d, j = i % d;
  double ang = (double)s / pow(10000.0, (double)(j / 2 * 2) / (double)d);
  pe[i] = (float)((j & 1) ? cos(ang) : sin(ang));
}
hipError_t op_posenc_init(const OpCtx& c, float* pe, int S, int d) {
  int n = S * d;
  k_posenc<<<(n + 255) / 256, 256, 0, c.stream>>>(pe, S, d);
  return LP_LAUNCH_CHECK();
}

template <typename T>
__global__ void k_embed_fwd(const int32_t* ids, const float* emb, const float* pe, T* out, int T_, int S, int d,
                            int V) {
  int t = blockIdx.x;
  int id = ids[t];
  id = id < 0 ? 0 : (id >= V ? V - 1 : id);   // out-of-range ids are clamped, never read out of bounds
  int s = t % S;
  const float* e = emb + (size_t)id * d;
  const float* p = pe + (size_t)s * d;
  T* o = out + (size_t)t * d;
  for (int j = threadIdx.x; j < d; j += blockDim.x) o[j] = from_f<T>(e[j] + p[j]);
}
hipError_t op_embed_fwd(const OpCtx& c, const int32_t* ids, const float* emb, const float* pe, void* out,
                        int T_, int S, int d, int V) {
  ProfScope prof_(c, KC_EMBED);
  if (T_ == 0) return hipSuccess;
  if (c.dt == BF16) k_embed_fwd<bf16_t><<<T_, 128, 0, c.stream>>>(ids, emb, pe, (bf16_t*)out, T_, S, d, V);
  else k_embed_fwd<float><<<T_, 128, 0, c.stream>>>(ids, emb, pe, (float*)out, T_, S, d, V);
  return LP_LAUNCH_CHECK();
}

// Gradient of the embedding table: row v = sum over the positions t with ids[t] == v of dh[t, :],
// taken in increasing t (fixed order; the only atomics are integer counts, which are exact).  A first
// kernel counts the positions of every id (ids outside [0, V) are clamped as in the forward pass); then
// one block per (row, 256-column slab): a row that does not occur is zero-filled at once (most of a
// Zipf vocabulary), otherwise the block scans all ids, compacts the matching positions in order and
// sums those rows.
__device__ __forceinline__ int clamp_id(int id, int V) { return id < 0 ? 0 : (id >= V ? V - 1 : id); }

__global__ void k_id_count(const int32_t* __restrict__ ids, int* __restrict__ counts, int T_, int V) {
  int t = blockIdx.x * blockDim.x + threadIdx.x;
  if (t < T_) atomicAdd(&counts[clamp_id(ids[t], V)], 1);
}

template <typename T>
__global__ void k_embed_bwd(const int32_t* ids, const int* __restrict__ counts, const T* dh, float* demb, int T_,
                            int V, int d, int accumulate) {
  __shared__ int pos[256];
  __shared__ int wcount[4];
  int v = blockIdx.x;
  int col = blockIdx.y * 256 + threadIdx.x;
  float acc = 0.f;
  const int n_hits = counts ? counts[v] : -1;        // block-uniform
  if (n_hits != 0) {
    int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    int found = 0;
    for (int base = 0; base < T_ && (n_hits < 0 || found < n_hits); base += 256) {
      int t = base + threadIdx.x;
      bool hit = (t < T_) && (clamp_id(ids[t], V) == v);
      unsigned long long mask = __ballot(hit);
      if (lane == 0) wcount[w] = __popcll(mask);
      __syncthreads();
      int off = 0;
      for (int i = 0; i < w; ++i) off += wcount[i];
      int total = wcount[0] + wcount[1] + wcount[2] + wcount[3];
      if (hit) pos[off + __popcll(mask & ((1ull << lane) - 1ull))] = t;
      __syncthreads();
      if (col < d)
        for (int i = 0; i < total; ++i) acc += to_f(dh[(size_t)pos[i] * d + col]);
      found += total;
      __syncthreads();
    }
  }
  if (col < d) {
    size_t o = (size_t)v * d + col;
    if (n_hits != 0 || !accumulate) demb[o] = accumulate ? demb[o] + acc : acc;
  }
}
hipError_t op_embed_bwd(const OpCtx& c, const int32_t* ids, const void* dh, float* demb, int T_, int V, int d,
                        int accumulate) {
  ProfScope prof_(c, KC_EMBED);
  if (V <= 0 || d <= 0) return hipSuccess;
  // per-id counts in the reduction scratch (integers; 0.0f is the zero word)
  int* counts = nullptr;
  if (c.partial && (size_t)V <= c.partial_elems && T_ > 0) {
    counts = reinterpret_cast<int*>(c.partial);
    hipError_t e = op_fill_f32(c, c.partial, (size_t)V, 0.f);
    if (e != hipSuccess) return e;
    k_id_count<<<(T_ + 255) / 256, 256, 0, c.stream>>>(ids, counts, T_, V);
  }
  dim3 grid(V, (d + 255) / 256);
  if (c.dt == BF16)
    k_embed_bwd<bf16_t><<<grid, 256, 0, c.stream>>>(ids, counts, (const bf16_t*)dh, demb, T_, V, d, accumulate);
  else
    k_embed_bwd<float><<<grid, 256, 0, c.stream>>>(ids, counts, (const float*)dh, demb, T_, V, d, accumulate);
  return LP_LAUNCH_CHECK();
}

// ------------------------------------------------------------------------------------ LayerNorm
// One wavefront per row; biased variance, eps 1e-5; statistics in fp32.
constexpr float kLnEps = 1e-5f;

template <typename T>
__global__ void k_ln_fwd(const T* x, const float* g, const float* b, T* y, float* mean, float* rstd, int rows,
                         int d) {
  int row = blockIdx.x * 4 + (threadIdx.x >> 6);
  int lane = threadIdx.x & 63;
  if (row >= rows) return;
  const T* xr = x + (size_t)row * d;
  float s = 0.f;
  for (int j = lane; j < d; j += 64) s += to_f(xr[j]);
  float mu = wave_sum(s) / (float)d;
  float q = 0.f;
  for (int j = lane; j < d; j += 64) { float t = to_f(xr[j]) - mu; q += t * t; }
  float rs = rsqrtf(wave_sum(q) / (float)d + kLnEps);
  T* yr = y + (size_t)row * d;
  for (int j = lane; j < d; j += 64) yr[j] = from_f<T>((to_f(xr[j]) - mu) * rs * g[j] + b[j]);
  if (lane == 0) { mean[row] = mu; rstd[row] = rs; }
}
hipError_t op_layernorm_fwd(const OpCtx& c, const void* x, const float* g, const float* b, void* y, float* mean,
                            float* rstd, int rows, int d) {
  ProfScope prof_(c, KC_LAYERNORM);
  if (rows == 0) return hipSuccess;
  if (ln_fast_ok(c, x, y, nullptr, nullptr, d)) return ln_fwd_fast(c, x, g, b, y, mean, rstd, rows, d);
  int blocks = (rows + 3) / 4;
  if (c.dt == BF16) k_ln_fwd<bf16_t><<<blocks, 256, 0, c.stream>>>((const bf16_t*)x, g, b, (bf16_t*)y, mean, rstd, rows, d);
  else k_ln_fwd<float><<<blocks, 256, 0, c.stream>>>((const float*)x, g, b, (float*)y, mean, rstd, rows, d);
  return LP_LAUNCH_CHECK();
}

// Backward.  Per row: dxhat = dy*g; dx = (dxhat - mean(dxhat) - xhat*mean(dxhat*xhat)) * rstd (+ add).
// Parameter gradients: each block owns a contiguous slab of rows and writes its partial sums of
// dy*xhat and dy to partial[block, 0..d) and partial[nblk + block, 0..d); a second kernel adds the
// partials in block order.
constexpr int kLnBwdRowsPerBlock = 32;
template <typename T>
__global__ void k_ln_bwd(const T* dy, const T* x, const float* mean, const float* rstd, const float* g,
                         const T* add, T* dx, float* partial, int rows, int d) {
  extern __shared__ float sh[];   // [4 waves][2][d]
  int w = threadIdx.x >> 6, lane = threadIdx.x & 63;
  float* pg = sh + (size_t)(w * 2) * d;
  float* pb = pg + d;
  for (int j = lane; j < d; j += 64) { pg[j] = 0.f; pb[j] = 0.f; }
  int row0 = blockIdx.x * kLnBwdRowsPerBlock;
  for (int r = w; r < kLnBwdRowsPerBlock; r += 4) {
    int row = row0 + r;
    if (row >= rows) break;
    const T* xr = x + (size_t)row * d;
    const T* dr = dy + (size_t)row * d;
    float mu = mean[row], rs = rstd[row];
    float s1 = 0.f, s2 = 0.f;
    for (int j = lane; j < d; j += 64) {
      float xh = (to_f(xr[j]) - mu) * rs;
      float dyv = to_f(dr[j]);
      float dxh = dyv * g[j];
      s1 += dxh;
      s2 += dxh * xh;
      pg[j] += dyv * xh;
      pb[j] += dyv;
    }
    s1 = wave_sum(s1) / (float)d;
    s2 = wave_sum(s2) / (float)d;
    if (dx) {
      T* ox = dx + (size_t)row * d;
      const T* ar = add ? add + (size_t)row * d : nullptr;
      for (int j = lane; j < d; j += 64) {
        float xh = (to_f(xr[j]) - mu) * rs;
        float v = (to_f(dr[j]) * g[j] - s1 - xh * s2) * rs;
        if (ar) v += to_f(ar[j]);
        ox[j] = from_f<T>(v);
      }
    }
  }
  __syncthreads();
  int nblk = gridDim.x;
  for (int j = threadIdx.x; j < d; j += blockDim.x) {
    float a = 0.f, bsum = 0.f;
    for (int ww = 0; ww < 4; ++ww) { a += sh[(size_t)(ww * 2) * d + j]; bsum += sh[(size_t)(ww * 2 + 1) * d + j]; }
    partial[(size_t)blockIdx.x * d + j] = a;
    partial[(size_t)(nblk + blockIdx.x) * d + j] = bsum;
  }
}
// out[j] (+)= sum_b partial[b, j].  Block = 64 columns x 16 row groups; group q adds rows q, q+16, ... in
// order (four independent loads in flight at a time) and the sixteen group sums are then added in order:
// a fixed tree, so the result does not depend on the launch.
constexpr int kReduceGroups = 16;
__global__ void __launch_bounds__(64 * kReduceGroups)
k_reduce_partials(const float* __restrict__ partial, int nblk, int n, float* out, int accumulate,
                  float* out_y1 = nullptr) {
  // blockIdx.y == 1: a second table of partials stored right behind the first, summed into out_y1
  if (blockIdx.y == 1) { partial += (size_t)nblk * n; out = out_y1; }
  __shared__ float sh[kReduceGroups][64];
  int lc = threadIdx.x & 63, q = threadIdx.x >> 6;
  int j = blockIdx.x * 64 + lc;
  float a = 0.f;
  if (j < n) {
    int b = q;
    for (; b + 3 * kReduceGroups < nblk; b += 4 * kReduceGroups) {
      float v0 = partial[(size_t)b * n + j], v1 = partial[(size_t)(b + kReduceGroups) * n + j];
      float v2 = partial[(size_t)(b + 2 * kReduceGroups) * n + j], v3 = partial[(size_t)(b + 3 * kReduceGroups) * n + j];
      a += v0; a += v1; a += v2; a += v3;
    }
    for (; b < nblk; b += kReduceGroups) a += partial[(size_t)b * n + j];
  }
  sh[q][lc] = a;
  __syncthreads();
  if (q == 0 && j < n) {
    float t = 0.f;
#pragma unroll
    for (int g = 0; g < kReduceGroups; ++g) t += sh[g][lc];
    out[j] = accumulate ? out[j] + t : t;
  }
}
hipError_t op_layernorm_bwd(const OpCtx& c, const void* dy, const void* x, const float* mean, const float* rstd,
                            const float* g, const void* add, void* dx, float* dg, float* db, int rows, int d,
                            int accumulate) {
  ProfScope prof_(c, KC_LAYERNORM);
  if (rows == 0) return hipSuccess;
  if (ln_fast_ok(c, dy, x, add, dx, d)) {
    int nb = 0;
    hipError_t e = ln_bwd_fast(c, dy, x, mean, rstd, g, add, dx, rows, d, &nb);
    if (e != hipSuccess || !dg) return e;          // no dg: the caller wants the input gradient only
    k_reduce_partials<<<dim3((d + 63) / 64, 2), 64 * kReduceGroups, 0, c.stream>>>(c.partial, nb, d, dg, accumulate, db);
    return LP_LAUNCH_CHECK();
  }
  int nblk = (rows + kLnBwdRowsPerBlock - 1) / kLnBwdRowsPerBlock;
  if ((size_t)nblk * d * 2 > c.partial_elems) return hipErrorInvalidValue;
  size_t shm = (size_t)8 * d * sizeof(float);
  if (c.dt == BF16)
    k_ln_bwd<bf16_t><<<nblk, 256, shm, c.stream>>>((const bf16_t*)dy, (const bf16_t*)x, mean, rstd, g,
                                                   (const bf16_t*)add, (bf16_t*)dx, c.partial, rows, d);
  else
    k_ln_bwd<float><<<nblk, 256, shm, c.stream>>>((const float*)dy, (const float*)x, mean, rstd, g,
                                                  (const float*)add, (float*)dx, c.partial, rows, d);
  hipError_t e = LP_LAUNCH_CHECK();
  if (e != hipSuccess || !dg) return e;
  k_reduce_partials<<<dim3((d + 63) / 64, 2), 64 * kReduceGroups, 0, c.stream>>>(c.partial, nblk, d, dg, accumulate, db);
  return LP_LAUNCH_CHECK();
}

// ------------------------------------------------------------------------------------ column sums
// out[j] (+)= sum_r dy[r, j]  (bias gradients).  Block = 64 columns x 4 row-lanes over a slab of rows.
constexpr int kColsumRows = 128;
constexpr int kMaxColsumBatch = 4;
template <typename T>
__global__ void k_colsum_partial(const T* dy, int64_t ld, float* partial, int rows, int n) {
  __shared__ float sh[4][64];
  int col = blockIdx.x * 64 + (threadIdx.x & 63);
  int w = threadIdx.x >> 6;
  int r0 = blockIdx.y * kColsumRows;
  int r1 = r0 + kColsumRows < rows ? r0 + kColsumRows : rows;
  float a = 0.f;
  if (col < n)
    for (int r = r0 + w; r < r1; r += 4) a += to_f(dy[(size_t)r * ld + col]);
  sh[w][threadIdx.x & 63] = a;
  __syncthreads();
  if (w == 0 && col < n)
    partial[(size_t)blockIdx.y * n + col] = sh[0][threadIdx.x] + sh[1][threadIdx.x] + sh[2][threadIdx.x] + sh[3][threadIdx.x];
}
// bf16, 16-byte loads: block = 16 column chunks of 8 (128 columns) x 16 row lanes over a slab of kColsumRows
// rows; row lane w adds rows w, w+16, ... in order, the 16 lane sums are then added in order.
__global__ void __launch_bounds__(256)
k_colsum_partial_v(const bf16_t* __restrict__ dy, int64_t ld, float* __restrict__ partial, int rows, int n) {
  __shared__ float sh[16][128];
  const int ch = threadIdx.x & 15, w = threadIdx.x >> 4;
  const int col = blockIdx.x * 128 + ch * 8;
  const int r0 = blockIdx.y * kColsumRows;
  const int r1 = r0 + kColsumRows < rows ? r0 + kColsumRows : rows;
  float a[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  if (col < n)
    for (int r = r0 + w; r < r1; r += 16) {
      bf16x8 v = *reinterpret_cast<const bf16x8*>(dy + (size_t)r * ld + col);
#pragma unroll
      for (int x = 0; x < 8; ++x) a[x] += (float)v[x];
    }
#pragma unroll
  for (int x = 0; x < 8; ++x) sh[w][ch * 8 + x] = a[x];
  __syncthreads();
  if (threadIdx.x < 128) {
    const int cc = blockIdx.x * 128 + threadIdx.x;
    if (cc < n) {
      float t = 0.f;
#pragma unroll
      for (int g = 0; g < 16; ++g) t += sh[g][threadIdx.x];
      partial[(size_t)blockIdx.y * n + cc] = t;
    }
  }
}
hipError_t op_colsum(const OpCtx& c, const void* dy, int64_t ld, float* out, int rows, int n, int accumulate) {
  ProfScope prof_(c, KC_COLSUM);
  if (n == 0) return hipSuccess;
  int nslab = (rows + kColsumRows - 1) / kColsumRows;
  if (nslab < 1) nslab = 1;
  if ((size_t)nslab * n > c.partial_elems) return hipErrorInvalidValue;
  // one slab of rows and nothing to add to: the slab's sums are the result, no second kernel
  const bool direct = nslab == 1 && !accumulate;
  float* part = direct ? out : c.partial;
  if (c.dt == BF16 && n % 8 == 0 && ld % 8 == 0 && ((uintptr_t)dy & 15) == 0) {
    k_colsum_partial_v<<<dim3((n + 127) / 128, nslab), 256, 0, c.stream>>>((const bf16_t*)dy, ld, part, rows, n);
  } else {
    dim3 grid((n + 63) / 64, nslab);
    if (c.dt == BF16) k_colsum_partial<bf16_t><<<grid, 256, 0, c.stream>>>((const bf16_t*)dy, ld, part, rows, n);
    else k_colsum_partial<float><<<grid, 256, 0, c.stream>>>((const float*)dy, ld, part, rows, n);
  }
  if (!direct) k_reduce_partials<<<(n + 63) / 64, 64 * kReduceGroups, 0, c.stream>>>(c.partial, nslab, n, out, accumulate);
  return LP_LAUNCH_CHECK();
}

// Several column sums over the same rows in one pair of launches (the four bias gradients of a decoder layer, whose
// dY matrices all stay alive until the end of the layer's backward pass): the column blocks of all problems form one
// grid, each problem keeps a partial table of its own behind the previous one's, and the sums are taken in exactly the
// order of the single-problem kernels above, so the results are the same bits.
struct ColsumBatch {
  const bf16_t* dy[kMaxColsumBatch];
  int64_t ld[kMaxColsumBatch];
  float* out[kMaxColsumBatch];
  int n[kMaxColsumBatch];
  int first128[kMaxColsumBatch + 1];      // first 128-column block of problem p in the partial kernel's grid
  int first64[kMaxColsumBatch + 1];       // first 64-column block in the reduce kernel's grid
  size_t part_off[kMaxColsumBatch];       // start of problem p's [nslab][n] partial table
  int count;
};
__global__ void __launch_bounds__(256)
k_colsum_partial_batched(ColsumBatch b, float* __restrict__ partial, int rows) {
  __shared__ float sh[16][128];
  int p = 0;
#pragma unroll
  for (int i = 1; i < kMaxColsumBatch; ++i)
    if (i < b.count && (int)blockIdx.x >= b.first128[i]) p = i;
  const bf16_t* dy = b.dy[p];
  const int64_t ld = b.ld[p];
  const int n = b.n[p];
  float* part = partial + b.part_off[p];
  const int ch = threadIdx.x & 15, w = threadIdx.x >> 4;
  const int cb = blockIdx.x - b.first128[p];
  const int col = cb * 128 + ch * 8;
  const int r0 = blockIdx.y * kColsumRows;
  const int r1 = r0 + kColsumRows < rows ? r0 + kColsumRows : rows;
  float a[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  if (col < n)
    for (int r = r0 + w; r < r1; r += 16) {
      bf16x8 v = *reinterpret_cast<const bf16x8*>(dy + (size_t)r * ld + col);
#pragma unroll
      for (int x = 0; x < 8; ++x) a[x] += (float)v[x];
    }
#pragma unroll
  for (int x = 0; x < 8; ++x) sh[w][ch * 8 + x] = a[x];
  __syncthreads();
  if (threadIdx.x < 128) {
    const int cc = cb * 128 + threadIdx.x;
    if (cc < n) {
      float t = 0.f;
#pragma unroll
      for (int g = 0; g < 16; ++g) t += sh[g][threadIdx.x];
      part[(size_t)blockIdx.y * n + cc] = t;
    }
  }
}
__global__ void __launch_bounds__(64 * kReduceGroups)
k_reduce_partials_batched(ColsumBatch b, const float* __restrict__ partial, int nblk, int accumulate) {
  __shared__ float sh[kReduceGroups][64];
  int p = 0;
#pragma unroll
  for (int i = 1; i < kMaxColsumBatch; ++i)
    if (i < b.count && (int)blockIdx.x >= b.first64[i]) p = i;
  const float* part = partial + b.part_off[p];
  const int n = b.n[p];
  float* out = b.out[p];
  int lc = threadIdx.x & 63, q = threadIdx.x >> 6;
  int j = (blockIdx.x - b.first64[p]) * 64 + lc;
  float a = 0.f;
  if (j < n) {
    int r = q;
    for (; r + 3 * kReduceGroups < nblk; r += 4 * kReduceGroups) {
      float v0 = part[(size_t)r * n + j], v1 = part[(size_t)(r + kReduceGroups) * n + j];
      float v2 = part[(size_t)(r + 2 * kReduceGroups) * n + j], v3 = part[(size_t)(r + 3 * kReduceGroups) * n + j];
      a += v0; a += v1; a += v2; a += v3;
    }
    for (; r < nblk; r += kReduceGroups) a += part[(size_t)r * n + j];
  }
  sh[q][lc] = a;
  __syncthreads();
  if (q == 0 && j < n) {
    float t = 0.f;
#pragma unroll
    for (int g = 0; g < kReduceGroups; ++g) t += sh[g][lc];
    out[j] = accumulate ? out[j] + t : t;
  }
}
hipError_t op_colsum_batched(const OpCtx& c, int count, const void* const* dy, const int64_t* ld, float* const* out,
                             int rows, const int* n, int accumulate) {
  if (count <= 0) return hipSuccess;
  const int nslab = (rows + kColsumRows - 1) / kColsumRows;
  bool fast = c.dt == BF16 && count <= kMaxColsumBatch && nslab > 1;
  size_t total = 0;
  for (int p = 0; p < count; ++p) {
    fast = fast && n[p] > 0 && n[p] % 8 == 0 && ld[p] % 8 == 0 && ((uintptr_t)dy[p] & 15) == 0;
    total += (size_t)nslab * n[p];
  }
  if (!fast || total > c.partial_elems) {         // one by one: any type, any alignment
    for (int p = 0; p < count; ++p) {
      hipError_t e = op_colsum(c, dy[p], ld[p], out[p], rows, n[p], accumulate);
      if (e != hipSuccess) return e;
    }
    return hipSuccess;
  }
  ProfScope prof_(c, KC_COLSUM);
  ColsumBatch b = {};
  b.count = count;
  size_t off = 0;
  int f128 = 0, f64 = 0;
  for (int p = 0; p < count; ++p) {
    b.dy[p] = (const bf16_t*)dy[p]; b.ld[p] = ld[p]; b.out[p] = out[p]; b.n[p] = n[p];
    b.first128[p] = f128; b.first64[p] = f64; b.part_off[p] = off;
    f128 += (n[p] + 127) / 128; f64 += (n[p] + 63) / 64; off += (size_t)nslab * n[p];
  }
  for (int p = count; p <= kMaxColsumBatch; ++p) { b.first128[p] = f128; b.first64[p] = f64; }
  k_colsum_partial_batched<<<dim3(f128, nslab), 256, 0, c.stream>>>(b, c.partial, rows);
  k_reduce_partials_batched<<<f64, 64 * kReduceGroups, 0, c.stream>>>(b, c.partial, nslab, accumulate);
  return LP_LAUNCH_CHECK();
}

// ------------------------------------------------------------------------------------ softmax CE
// One block of 256 threads per row.  Pass 1: running max and sum of exp (online).  Pass 2 (if
// write_grad): z <- (exp(z - lse) - [j == y]) * inv_rows.
template <typename T>
__global__ void k_softmax_ce(T* z, int64_t ld, const int32_t* y, float* loss_rows, int n, int write_grad,
                             float inv_rows) {
  __shared__ float sh[4];
  int row = blockIdx.x;
  T* zr = z + (size_t)row * ld;
  float m = -INFINITY, s = 0.f;
  for (int j = threadIdx.x; j < n; j += 256) {
    float v = to_f(zr[j]);
    if (v > m) { s = s * __expf(m - v) + 1.f; m = v; }
    else s += __expf(v - m);
  }
  float gm = block_max_256(m, sh);
  float contrib = (m == -INFINITY) ? 0.f : s * __expf(m - gm);
  float gs = block_sum_256(contrib, sh);
  float lse = gm + __logf(gs);
  int yy = y[row];
  bool y_ok = yy >= 0 && yy < n;               // a label outside [0, n) contributes lse and no one-hot term
  if (threadIdx.x == 0) loss_rows[row] = lse - (y_ok ? to_f(zr[yy]) : 0.f);
  if (write_grad) {
    __syncthreads();
    for (int j = threadIdx.x; j < n; j += 256) {
      float p = __expf(to_f(zr[j]) - lse);
      if (j == yy) p -= 1.f;
      zr[j] = from_f<T>(p * inv_rows);
    }
  }
}
hipError_t op_softmax_ce(const OpCtx& c, void* z, int64_t ld, const int32_t* y, float* loss_rows, int rows, int n,
                         int write_grad, float inv_rows) {
  ProfScope prof_(c, KC_SOFTMAX_CE);
  if (rows == 0) return hipSuccess;
  if (ce_fast_ok(c, z, ld, n)) return ce_fast(c, z, ld, y, loss_rows, rows, n, write_grad, inv_rows);
  if (c.dt == BF16) k_softmax_ce<bf16_t><<<rows, 256, 0, c.stream>>>((bf16_t*)z, ld, y, loss_rows, n, write_grad, inv_rows);
  else k_softmax_ce<float><<<rows, 256, 0, c.stream>>>((float*)z, ld, y, loss_rows, n, write_grad, inv_rows);
  return LP_LAUNCH_CHECK();
}

// out[0] = mean(v[0..n)) with a fixed summation tree (one block).
__global__ void k_mean(const float* v, int n, float* out) {
  __shared__ float sh[4];
  float a = 0.f;
  for (int i = threadIdx.x; i < n; i += 256) a += v[i];
  float s = block_sum_256(a, sh);
  if (threadIdx.x == 0) out[0] = s / (float)n;
}
hipError_t op_mean(const OpCtx& c, const float* v, int n, float* out) {
  ProfScope prof_(c, KC_OTHER);
  k_mean<<<1, 256, 0, c.stream>>>(v, n, out);
  return LP_LAUNCH_CHECK();
}

// ------------------------------------------------------------------------------------ cosine
// <a, b>, <a, a>, <b, b> of two fp32 ranges: per-block partial sums in a fixed tree, then one block adds
// the partials in order in double and writes <a, b> / sqrt(<a, a> <b, b>) (0 if either vector is zero).
constexpr int kCosBlocks = 128;
__global__ void __launch_bounds__(256) k_dot3_partial(const float* __restrict__ a, const float* __restrict__ b, size_t n,
                                                      float* __restrict__ partial) {
  __shared__ float sh[4];
  float d = 0.f, aa = 0.f, bb = 0.f;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) {
    const float x = a[i], y = b[i];
    d += x * y; aa += x * x; bb += y * y;
  }
  d = block_sum_256(d, sh);
  aa = block_sum_256(aa, sh);
  bb = block_sum_256(bb, sh);
  if (threadIdx.x == 0) { partial[3 * blockIdx.x] = d; partial[3 * blockIdx.x + 1] = aa; partial[3 * blockIdx.x + 2] = bb; }
}
__global__ void k_cos_finish(const float* __restrict__ partial, int nblk, float* __restrict__ out) {
  if (threadIdx.x != 0) return;
  double d = 0.0, aa = 0.0, bb = 0.0;
  for (int i = 0; i < nblk; ++i) { d += partial[3 * i]; aa += partial[3 * i + 1]; bb += partial[3 * i + 2]; }
  out[0] = (aa > 0.0 && bb > 0.0) ? (float)(d / sqrt(aa * bb)) : 0.f;
}
hipError_t op_cosine(const OpCtx& c, const float* a, const float* b, size_t n, float* out) {
  ProfScope prof_(c, KC_OTHER);
  if ((size_t)3 * kCosBlocks > c.partial_elems) return hipErrorInvalidValue;
  k_dot3_partial<<<kCosBlocks, 256, 0, c.stream>>>(a, b, n, c.partial);
  k_cos_finish<<<1, 64, 0, c.stream>>>(c.partial, kCosBlocks, out);
  return LP_LAUNCH_CHECK();
}

// ------------------------------------------------------------------------------------ optimizer
// One fused pass over a flat parameter range: reads p, g (and m, v), writes p (and m, v) and the
// low-precision working copy.  SGD: p -= lr g.  SGD-momentum: m = mu m + g; p -= lr m.
// Adam: m = b1 m + (1-b1) g; v = b2 v + (1-b2) g^2; p -= lr (m/(1-b1^t)) / (sqrt(v/(1-b2^t)) + eps).
template <int KIND, bool LOWP>
__global__ void k_optimizer(float* __restrict__ p, const float* __restrict__ g, float* __restrict__ m,
                            float* __restrict__ v, bf16_t* __restrict__ pl, size_t n4, size_t n, float lr,
                            float mu, float b1, float b2, float eps, float wd, float c1, float c2, float gs) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  size_t st = (size_t)gridDim.x * blockDim.x;
  for (; i < n4; i += st) {
    f32x4 pp = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(p) + i);
    f32x4 gg = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(g) + i);
    float pv[4] = {pp.x, pp.y, pp.z, pp.w};
    float gv[4] = {gg.x * gs, gg.y * gs, gg.z * gs, gg.w * gs};
    float mv[4], vv[4];
    if (KIND >= 1) { f32x4 t = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(m) + i); mv[0] = t.x; mv[1] = t.y; mv[2] = t.z; mv[3] = t.w; }
    if (KIND == 2) { f32x4 t = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(v) + i); vv[0] = t.x; vv[1] = t.y; vv[2] = t.z; vv[3] = t.w; }
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      float gk = gv[k] + wd * pv[k];
      if (KIND == 0) pv[k] -= lr * gk;
      else if (KIND == 1) { mv[k] = mu * mv[k] + gk; pv[k] -= lr * mv[k]; }
      else {
        mv[k] = b1 * mv[k] + (1.f - b1) * gk;
        vv[k] = b2 * vv[k] + (1.f - b2) * gk * gk;
        pv[k] -= lr * (mv[k] * c1) / (sqrtf(vv[k] * c2) + eps);
      }
    }
    { f32x4 o = {pv[0], pv[1], pv[2], pv[3]}; __builtin_nontemporal_store(o, reinterpret_cast<f32x4*>(p) + i); }
    if (KIND >= 1) { f32x4 o = {mv[0], mv[1], mv[2], mv[3]}; __builtin_nontemporal_store(o, reinterpret_cast<f32x4*>(m) + i); }
    if (KIND == 2) { f32x4 o = {vv[0], vv[1], vv[2], vv[3]}; __builtin_nontemporal_store(o, reinterpret_cast<f32x4*>(v) + i); }
    if (LOWP) {
      bf16x4 o = {static_cast<bf16_t>(pv[0]), static_cast<bf16_t>(pv[1]), static_cast<bf16_t>(pv[2]), static_cast<bf16_t>(pv[3])};
      reinterpret_cast<bf16x4*>(pl)[i] = o;
    }
  }
}
hipError_t op_optimizer(const OpCtx& c, const OptArgs& o, float* p, const float* g, float* m, float* v,
                        void* p_lowp, size_t n) {
  ProfScope prof_(c, KC_OPTIMIZER);
  if (n == 0) return hipSuccess;
  if (n % 4) return hipErrorInvalidValue;   // ranges are padded to 64 elements by the layout
  size_t n4 = n / 4;
  size_t want = (n4 + 255) / 256;
  int blocks = (int)(want < 256 * 16 ? want : 256 * 16);
  float c1 = 1.f, c2 = 1.f;
  if (o.kind == 2) {
    c1 = (float)(1.0 / (1.0 - pow((double)o.beta1, (double)o.t)));
    c2 = (float)(1.0 / (1.0 - pow((double)o.beta2, (double)o.t)));
  }
  bf16_t* pl = (bf16_t*)p_lowp;
#define LP_OPT(K, L) k_optimizer<K, L><<<blocks, 256, 0, c.stream>>>(p, g, m, v, pl, n4, n, o.lr, o.momentum, o.beta1, o.beta2, o.eps, o.weight_decay, c1, c2, o.grad_scale)
  if (o.kind == 0) { if (pl) LP_OPT(0, true); else LP_OPT(0, false); }
  else if (o.kind == 1) { if (pl) LP_OPT(1, true); else LP_OPT(1, false); }
  else { if (pl) LP_OPT(2, true); else LP_OPT(2, false); }
#undef LP_OPT
  return LP_LAUNCH_CHECK();
}

// ------------------------------------------------------------------------------------ transpose
// 64 x 64 tiles through LDS: 16-byte loads of 8 columns, 16-byte stores of 8 rows gathered from a padded tile.
__global__ void __launch_bounds__(256) k_transpose_bf16(const bf16_t* __restrict__ src, bf16_t* __restrict__ dst, int R, int C) {
  __shared__ bf16_t tile[64][64 + 2];
  const int r0 = blockIdx.y * 64, c0 = blockIdx.x * 64;
  const int tr = threadIdx.x >> 3, tc = (threadIdx.x & 7) * 8;
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int r = r0 + tr + 32 * i, c = c0 + tc;
    bf16x8 v;
    if (r < R && c < C) v = *reinterpret_cast<const bf16x8*>(src + (size_t)r * C + c);
    else {
#pragma unroll
      for (int x = 0; x < 8; ++x) v[x] = (bf16_t)0.f;
    }
#pragma unroll
    for (int x = 0; x < 8; ++x) tile[tr + 32 * i][tc + x] = v[x];
  }
  __syncthreads();
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int c = c0 + tr + 32 * i, r = r0 + tc;      // output row c, output columns r .. r+7
    if (c < C && r < R) {
      bf16x8 v;
#pragma unroll
      for (int x = 0; x < 8; ++x) v[x] = tile[tc + x][tr + 32 * i];
      *reinterpret_cast<bf16x8*>(dst + (size_t)c * R + r) = v;
    }
  }
}
hipError_t op_transpose_bf16(const OpCtx& c, const void* src, void* dst, int R, int C) {
  ProfScope prof_(c, KC_OTHER);
  if (R <= 0 || C <= 0) return hipSuccess;
  if (R % 8 || C % 8 || (((uintptr_t)src | (uintptr_t)dst) & 15)) return hipErrorInvalidValue;
  dim3 grid((C + 63) / 64, (R + 63) / 64);
  k_transpose_bf16<<<grid, 256, 0, c.stream>>>((const bf16_t*)src, (bf16_t*)dst, R, C);
  return LP_LAUNCH_CHECK();
}

// ------------------------------------------------------------------------------------ init
// Counter-based normal generator: two 64-bit mixes of (seed, stream, index) -> Box-Muller.
__device__ __forceinline__ uint64_t mix64(uint64_t z) {
  z += 0x9E3779B97F4A7C15ull;
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  return z ^ (z >> 31);
}
__global__ void k_init_normal(float* p, size_t n, float std, uint64_t seed, uint64_t sid) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  size_t st = (size_t)gridDim.x * blockDim.x;
  for (; i < n; i += st) {
    uint64_t a = mix64(mix64(seed ^ (sid * 0xD1342543DE82EF95ull)) + 2 * i);
    uint64_t b = mix64(a + 1);
    float u1 = ((float)(a >> 40) + 1.0f) * (1.0f / 16777217.0f);
    float u2 = (float)(b >> 40) * (1.0f / 16777216.0f);
    p[i] = std * sqrtf(-2.0f * logf(u1)) * cosf(6.283185307179586f * u2);
  }
}
hipError_t op_init_normal(const OpCtx& c, float* p, size_t n, float std, uint64_t seed, uint64_t sid) {
  if (n == 0) return hipSuccess;
  int blocks = (int)((n + 255) / 256 < 4096 ? (n + 255) / 256 : 4096);
  k_init_normal<<<blocks, 256, 0, c.stream>>>(p, n, std, seed, sid);
  return LP_LAUNCH_CHECK();
}

}  // namespace lp
