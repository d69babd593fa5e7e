// Plain tiled FMA GEMM with fp32 accumulation, generic over operand accessors.  It serves the fp32
// compute path (the latency-bound residual-MLP configuration) and any shape or layout the MFMA
// kernels do not take.  Convolutions run through it as implicit GEMMs over NHWC gathers.
#include "common.h"
#include "gemm_common.h"

namespace lp {

template <typename T>
struct PlainOperand {          // logical (i, k) -> p[i*ld + k] if kc else p[k*ld + i]
  const T* p; int64_t ld; int kc;
  __device__ __forceinline__ float operator()(int i, int k) const {
    return to_f(kc ? p[(size_t)i * ld + k] : p[(size_t)k * ld + i]);
  }
};

// Convolution gathers (NHWC activations, [O,R,S,C] filters).
template <typename T>
struct ConvInputPatch {        // (m=(n,p,q), k=(r,s,c)) -> x[n, p*stride+r-pad, q*stride+s-pad, c] or 0
  const T* x; ConvArgs a;
  __device__ __forceinline__ float operator()(int m, int k) const {
    int q = m % a.Q, t = m / a.Q, p = t % a.P, n = t / a.P;
    int c = k % a.C, u = k / a.C, s = u % a.S, r = u / a.S;
    int h = p * a.stride + r - a.pad, w = q * a.stride + s - a.pad;
    if (h < 0 || h >= a.H || w < 0 || w >= a.W) return 0.f;
    return to_f(x[(((size_t)n * a.H + h) * a.W + w) * a.C + c]);
  }
};
template <typename T>
struct ConvOutputGather {      // (m=(n,h,w), k=(r,s,o)) -> dout[n, (h+pad-r)/stride, (w+pad-s)/stride, o] if integral
  const T* d; ConvArgs a;
  __device__ __forceinline__ float operator()(int m, int k) const {
    int w = m % a.W, t = m / a.W, h = t % a.H, n = t / a.H;
    int o = k % a.O, u = k / a.O, s = u % a.S, r = u / a.S;
    int hp = h + a.pad - r, wq = w + a.pad - s;
    if (hp < 0 || wq < 0 || hp % a.stride || wq % a.stride) return 0.f;
    int p = hp / a.stride, q = wq / a.stride;
    if (p >= a.P || q >= a.Q) return 0.f;
    return to_f(d[(((size_t)n * a.P + p) * a.Q + q) * a.O + o]);
  }
};
template <typename T>
struct ConvFilterT {           // (c, k=(r,s,o)) -> w[o, r, s, c]
  const T* w; ConvArgs a;
  __device__ __forceinline__ float operator()(int c, int k) const {
    int o = k % a.O, u = k / a.O;   // u = r*S + s
    return to_f(w[((size_t)o * a.R * a.S + u) * a.C + c]);
  }
};
template <typename T>
struct ConvPatchByCol {        // (j=(r,s,c), k=m) -> input patch element: same gather with arguments swapped
  ConvInputPatch<T> g;
  __device__ __forceinline__ float operator()(int j, int m) const { return g(m, j); }
};

constexpr int PBM = 64, PBN = 64, PBK = 32;

// Which index of an operand is contiguous in memory: a tile is fetched with that index varying fastest
// over the threads, so that a wavefront's loads fall into as few cache lines as possible.
template <typename T>
__device__ __forceinline__ bool k_is_contiguous(const PlainOperand<T>& o) { return o.kc != 0; }
template <typename O>
__device__ __forceinline__ bool k_is_contiguous(const O&) { return true; }

// gridDim.z > 1: split-K.  Block z reduces k in [z*kper, (z+1)*kper) and writes its raw fp32 tile to
// ws[z][M][N]; k_plain_splitk_reduce then adds the slices in order.
// The next k-tile is fetched into registers before the current one is multiplied, so the memory latency of a
// tile (which is what a small product costs: a few blocks, nothing else to switch to) overlaps the FMAs.
// TM rows x 4 columns per thread: block tile 16*TM x 64.  Small products take TM = 2: twice the blocks, and a
// k-tile's multiply phase (which, with a handful of blocks on the chip, is what the product waits for) is
// 14 instead of 24 instructions per k.
template <typename T, typename OA, typename OB, int TM = 4>
__global__ void __launch_bounds__(256) k_gemm_plain(OA A, OB B, Epilogue e, int M, int N, int K, int kper = 0,
                                                    float* ws = nullptr) {
  constexpr int BM_ = 16 * TM;
  __shared__ float As[PBK][BM_ + 1];
  __shared__ float Bs[PBK][PBN + 1];
  constexpr int PER_A = BM_ * PBK / 256, PER_B = PBN * PBK / 256;
  static_assert(BM_ * PBK % 256 == 0 && PBN * PBK % 256 == 0, "tile fetch assumes whole passes");
  int tx = threadIdx.x % 16, ty = threadIdx.x / 16;
  int m0 = blockIdx.y * BM_, n0 = blockIdx.x * PBN;
  float acc[TM][4] = {};
  int kbeg = 0;
  if (ws) {
    kbeg = blockIdx.z * kper;
    K = kbeg + kper < K ? kbeg + kper : K;
  }
  const bool a_kfast = k_is_contiguous(A), b_kfast = k_is_contiguous(B);
  float ra[PER_A], rb[PER_B];
  auto fetch = [&](int k0) {
#pragma unroll
    for (int j = 0; j < PER_A; ++j) {
      const int i = threadIdx.x + 256 * j;
      const int ka = a_kfast ? i % PBK : i / BM_, ma = a_kfast ? i / PBK : i % BM_;
      ra[j] = (m0 + ma < M && k0 + ka < K) ? A(m0 + ma, k0 + ka) : 0.f;
    }
#pragma unroll
    for (int j = 0; j < PER_B; ++j) {
      const int i = threadIdx.x + 256 * j;
      const int kb = b_kfast ? i % PBK : i / PBN, nb = b_kfast ? i / PBK : i % PBN;
      rb[j] = (n0 + nb < N && k0 + kb < K) ? B(n0 + nb, k0 + kb) : 0.f;
    }
  };
  auto stage = [&]() {
#pragma unroll
    for (int j = 0; j < PER_A; ++j) {
      const int i = threadIdx.x + 256 * j;
      const int ka = a_kfast ? i % PBK : i / BM_, ma = a_kfast ? i / PBK : i % BM_;
      As[ka][ma] = ra[j];
    }
#pragma unroll
    for (int j = 0; j < PER_B; ++j) {
      const int i = threadIdx.x + 256 * j;
      const int kb = b_kfast ? i % PBK : i / PBN, nb = b_kfast ? i / PBK : i % PBN;
      Bs[kb][nb] = rb[j];
    }
  };
  if (kbeg < K) fetch(kbeg);
  for (int k0 = kbeg; k0 < K; k0 += PBK) {
    stage();
    __syncthreads();
    if (k0 + PBK < K) fetch(k0 + PBK);
#pragma unroll
    for (int kk = 0; kk < PBK; ++kk) {
      float a[TM], b[4];
#pragma unroll
      for (int i = 0; i < TM; ++i) a[i] = As[kk][ty * TM + i];
#pragma unroll
      for (int i = 0; i < 4; ++i) b[i] = Bs[kk][tx * 4 + i];
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
    }
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      int m = m0 + ty * TM + i, n = n0 + tx * 4 + j;
      if (m < M && n < N) {
        if (ws) ws[((size_t)blockIdx.z * M + m) * N + n] = acc[i][j];
        else epilogue_store<T>(e, m, n, acc[i][j]);
      }
    }
}
// Eight running sums (slices s, s+8, ... each) keep eight loads in flight; they are combined in a fixed order.
__global__ void k_plain_splitk_reduce(const float* ws, float* out, size_t total, int splits, int accumulate) {
  size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= total) return;
  float a[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  int s = 0;
  for (; s + 8 <= splits; s += 8) {
#pragma unroll
    for (int u = 0; u < 8; ++u) a[u] += ws[(size_t)(s + u) * total + idx];
  }
  for (; s < splits; ++s) a[0] += ws[(size_t)s * total + idx];
  const float t = ((a[0] + a[1]) + (a[2] + a[3])) + ((a[4] + a[5]) + (a[6] + a[7]));
  out[idx] = accumulate ? out[idx] + t : t;
}

template <typename T, typename OA, typename OB>
static hipError_t launch_plain(hipStream_t s, OA A, OB B, const Epilogue& e, int M, int N, int K) {
  if (M <= 0 || N <= 0) return hipSuccess;
  const int tn = (N + PBN - 1) / PBN, tm = (M + PBM - 1) / PBM;
  if (tn * ((M + 31) / 32) < 64) {               // a very small product: 16-row tiles
    k_gemm_plain<T, OA, OB, 1><<<dim3(tn, (M + 15) / 16), 256, 0, s>>>(A, B, e, M, N, K);
  } else if (tn * tm < 128 && M > 16) {          // a small product: 32-row tiles
    k_gemm_plain<T, OA, OB, 2><<<dim3(tn, (M + 31) / 32), 256, 0, s>>>(A, B, e, M, N, K);
  } else {
    k_gemm_plain<T, OA, OB, 4><<<dim3(tn, tm), 256, 0, s>>>(A, B, e, M, N, K);
  }
  return hipGetLastError();
}

// A product with a handful of rows or columns (a classifier head over 10 classes: its forward map and its weight
// gradient): as tiles it is one to eight blocks that walk K in 32-deep steps, each step a memory latency, 35 us
// for 10 x 512 x 256.  Here a block owns 64 output elements (neighbouring threads own neighbouring columns, so an
// operand that is contiguous in n is read in whole lines and the other one is broadcast) and its four waves each
// take a quarter of K, 32 k at a time with every load of the step in flight at once (16-byte loads where k is the
// contiguous index); a thread adds its products in k order and the four quarters are added in order through LDS.
template <typename T>
__device__ __forceinline__ void skinny_load8(const PlainOperand<T>& o, int i, int k, int K, bool vec, float (&v)[8]) {
  if (o.kc && vec) {          // k .. k + 7 inside K, 16-byte aligned
    const T* p = o.p + (size_t)i * o.ld + k;
    if constexpr (sizeof(T) == 2) {
      bf16x8 r = *reinterpret_cast<const bf16x8*>(p);
#pragma unroll
      for (int u = 0; u < 8; ++u) v[u] = (float)r[u];
    } else {
      f32x4 r0 = *reinterpret_cast<const f32x4*>(p), r1 = *reinterpret_cast<const f32x4*>(p + 4);
#pragma unroll
      for (int u = 0; u < 4; ++u) { v[u] = r0[u]; v[4 + u] = r1[u]; }
    }
  } else {
    // unconditional loads from a clamped index, then a select: a load under a branch of its own would be waited
    // for before the next one is issued
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const int kk = k + u < K ? k + u : K - 1;
      const float x = o(i, kk);
      v[u] = k + u < K ? x : 0.f;
    }
  }
}
template <typename T>
__global__ void __launch_bounds__(256) k_gemm_skinny(PlainOperand<T> A, PlainOperand<T> B, Epilogue e, int M, int N, int K,
                                                     int a_vec, int b_vec) {
  __shared__ float part[4][64];
  const int lane = threadIdx.x & 63, w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const size_t idx = (size_t)blockIdx.x * 64 + lane;
  const bool live = idx < (size_t)M * N;
  const int m = live ? (int)(idx / N) : 0, n = live ? (int)(idx % N) : 0;
  const int kq = ((K + 3) / 4 + 7) & ~7;            // a wave's share of K, a multiple of 8
  const int k_lo = w * kq, k_hi = k_lo + kq < K ? k_lo + kq : K;
  float acc = 0.f;
  for (int k0 = k_lo; k0 < k_hi; k0 += 32) {
    float a[4][8], b[4][8];
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      const int k = k0 + 8 * c;
      const bool whole = k + 8 <= k_hi;
      if (k < k_hi) {
        skinny_load8(A, m, k, k_hi, a_vec && whole, a[c]);
        skinny_load8(B, n, k, k_hi, b_vec && whole, b[c]);
      } else {
#pragma unroll
        for (int u = 0; u < 8; ++u) { a[c][u] = 0.f; b[c][u] = 0.f; }
      }
    }
#pragma unroll
    for (int c = 0; c < 4; ++c)
#pragma unroll
      for (int u = 0; u < 8; ++u) acc = fmaf(a[c][u], b[c][u], acc);
  }
  part[w][lane] = acc;
  __syncthreads();
  if (w == 0 && live) epilogue_store<T>(e, m, n, ((part[0][lane] + part[1][lane]) + part[2][lane]) + part[3][lane]);
}

template <typename T>
static hipError_t gemm_plain_t(const OpCtx& c, const GemmArgs& g) {
  PlainOperand<T> A{(const T*)g.A, g.lda, g.a_kc}, B{(const T*)g.B, g.ldb, g.b_kc};
  if (g.M > 0 && g.N > 0 && (g.M <= 16 || g.N <= 16) && g.K <= 4096 && (size_t)g.M * g.N <= (size_t)1 << 16) {
    const size_t total = (size_t)g.M * g.N;
    const int per16 = 16 / (int)sizeof(T);          // elements per 16 bytes: vector loads need rows that start on them
    const int a_vec = g.a_kc && g.lda % per16 == 0 && ((uintptr_t)g.A & 15) == 0;
    const int b_vec = g.b_kc && g.ldb % per16 == 0 && ((uintptr_t)g.B & 15) == 0;
    k_gemm_skinny<T><<<(unsigned)((total + 63) / 64), 256, 0, c.stream>>>(A, B, make_epilogue(g), g.M, g.N, g.K, a_vec, b_vec);
    return hipGetLastError();
  }
  return launch_plain<T>(c.stream, A, B, make_epilogue(g), g.M, g.N, g.K);
}
hipError_t gemm_plain(const OpCtx& c, const GemmArgs& g) {
  return c.dt == BF16 ? gemm_plain_t<bf16_t>(c, g) : gemm_plain_t<float>(c, g);
}

static Epilogue plain_out(void* C, int64_t ldc, int c_f32, int accumulate) {
  GemmArgs g; g.C = C; g.ldc = ldc; g.c_f32 = c_f32; g.accumulate = accumulate;
  return make_epilogue(g);
}

// Forward convolution of an input with very few channels (the 3-channel stem): as a GEMM its reduction is
// 27 long and the gather's index arithmetic costs more than the multiplications.  Here a thread owns one output
// pixel and 16 output channels: it walks the filter window once (one bounds test per tap), takes the filter
// from LDS ([k][O] fp32, so the 16 channels are consecutive) and writes 16 consecutive outputs.  Products are
// added in the same order (r, s, c ascending) as the GEMM form adds them.
constexpr int kSmallCMaxK = 64;
// 16 consecutive outputs as 16-byte stores (the caller guarantees 16-byte alignment)
__device__ __forceinline__ void store16(float* p, const float (&v)[16]) {
#pragma unroll
  for (int g = 0; g < 4; ++g) {
    f32x4 o = {v[4 * g], v[4 * g + 1], v[4 * g + 2], v[4 * g + 3]};
    *reinterpret_cast<f32x4*>(p + 4 * g) = o;
  }
}
__device__ __forceinline__ void store16(bf16_t* p, const float (&v)[16]) {
#pragma unroll
  for (int g = 0; g < 2; ++g) {
    bf16x8 o;
#pragma unroll
    for (int j = 0; j < 8; ++j) o[j] = (bf16_t)v[8 * g + j];
    *reinterpret_cast<bf16x8*>(p + 8 * g) = o;
  }
}
template <typename T>
__global__ void __launch_bounds__(256) k_conv_fwd_smallc(const T* __restrict__ x, const T* __restrict__ w,
                                                         T* __restrict__ out, ConvArgs a, int M) {
  extern __shared__ __attribute__((aligned(16))) float wsm[];
  const int K = a.R * a.S * a.C;
  for (int i = threadIdx.x; i < K * a.O; i += 256) {
    const int o = i % a.O, k = i / a.O;
    wsm[i] = to_f(w[(size_t)o * K + k]);
  }
  __syncthreads();
  const int groups = a.O / 16;
  const size_t gid = (size_t)blockIdx.x * 256 + threadIdx.x;
  const size_t m = gid / groups;
  const int og = (int)(gid % groups);
  if (m >= (size_t)M) return;
  const int q = (int)(m % a.Q);
  const size_t t = m / a.Q;
  const int p = (int)(t % a.P), n = (int)(t / a.P);
  float acc[16];
#pragma unroll
  for (int j = 0; j < 16; ++j) acc[j] = 0.f;
  int k = 0;
  for (int r = 0; r < a.R; ++r)
    for (int s2 = 0; s2 < a.S; ++s2) {
      const int h = p * a.stride + r - a.pad, wq = q * a.stride + s2 - a.pad;
      const bool ok = h >= 0 && h < a.H && wq >= 0 && wq < a.W;
      const T* xp = x + (((size_t)n * a.H + (ok ? h : 0)) * a.W + (ok ? wq : 0)) * a.C;
      for (int cc = 0; cc < a.C; ++cc, ++k) {
        const float xv = ok ? to_f(xp[cc]) : 0.f;
        const f32x4* wr = reinterpret_cast<const f32x4*>(wsm + (size_t)k * a.O + og * 16);   // 64-byte aligned
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const f32x4 wv = wr[g];
#pragma unroll
          for (int j = 0; j < 4; ++j) acc[4 * g + j] = fmaf(xv, wv[j], acc[4 * g + j]);
        }
      }
    }
  store16(out + m * a.O + og * 16, acc);
}

template <typename T>
static hipError_t conv_fwd_t(const OpCtx& c, const ConvArgs& a, const void* x, const void* w, void* out) {
  int M = a.N * a.P * a.Q, K = a.R * a.S * a.C;
  if (a.C <= 4 && a.O % 16 == 0 && K <= kSmallCMaxK && M > 0 && ((uintptr_t)out & 15) == 0) {
    const size_t threads = (size_t)M * (a.O / 16);
    const size_t shm = (size_t)K * a.O * sizeof(float);
    if (shm <= 48 * 1024) {
      k_conv_fwd_smallc<T><<<(unsigned)((threads + 255) / 256), 256, shm, c.stream>>>((const T*)x, (const T*)w, (T*)out, a, M);
      return hipGetLastError();
    }
  }
  ConvInputPatch<T> A{(const T*)x, a};
  PlainOperand<T> B{(const T*)w, K, 1};
  return launch_plain<T>(c.stream, A, B, plain_out(out, a.O, 0, 0), M, a.O, K);
}
template <typename T>
static hipError_t conv_bwd_data_t(const OpCtx& c, const ConvArgs& a, const void* dout, const void* w, void* dx,
                                  const void* add) {
  int M = a.N * a.H * a.W, K = a.R * a.S * a.O;
  ConvOutputGather<T> A{(const T*)dout, a};
  ConvFilterT<T> B{(const T*)w, a};
  Epilogue e = plain_out(dx, a.C, 0, 0);
  e.res = add; e.ldr = a.C;
  return launch_plain<T>(c.stream, A, B, e, M, a.C, K);
}
// Filter gradient of a convolution with very few input channels and 64 output channels (the 3-channel stem:
// 64 x 27 sums over 262144 pixels).  As a split-K GEMM it is 512 blocks of one 64 x 64 tile, 27 of whose columns are
// real, each k-step a gather with its index arithmetic: 123 us + 26 us for the reduction.  Here a block takes one image:
// the image sits in LDS as fp32 with its zero border, a thread owns one output channel o and a quarter of the
// (r, s, c) taps, walks the image's pixels in order, reads dy[pixel, o] (a wave reads 64 consecutive channels) and
// its taps from LDS (one address per wave: a broadcast), and leaves its sums in the image's slice of the workspace;
// the slices are added in order by the split-K reduction.
constexpr int kStemMaxTaps = 32;
template <typename T>
__global__ void __launch_bounds__(256) k_conv_wgrad_smallc(const T* __restrict__ dout, const T* __restrict__ x,
                                                           float* __restrict__ ws, ConvArgs a) {
  extern __shared__ __attribute__((aligned(16))) float xs[];
  const int Hp = a.H + 2 * a.pad, Wp = a.W + 2 * a.pad, J = a.R * a.S * a.C;
  const int n = blockIdx.x;
  for (int i = threadIdx.x; i < Hp * Wp * a.C; i += 256) {
    const int c = i % a.C, t = i / a.C, w = t % Wp - a.pad, h = t / Wp - a.pad;
    const bool ok = h >= 0 && h < a.H && w >= 0 && w < a.W;
    xs[i] = ok ? to_f(x[(((size_t)n * a.H + h) * a.W + w) * a.C + c]) : 0.f;
  }
  __syncthreads();
  const int o = threadIdx.x & 63, g = threadIdx.x >> 6;
  const int per = (J + 3) / 4, j0 = g * per;
  int off[kStemMaxTaps / 4];
  float acc[kStemMaxTaps / 4];
#pragma unroll
  for (int t = 0; t < kStemMaxTaps / 4; ++t) {
    const int j = j0 + t < J ? j0 + t : J - 1;
    const int c = j % a.C, rs = j / a.C, s2 = rs % a.S, r = rs / a.S;
    off[t] = (r * Wp + s2) * a.C + c;
    acc[t] = 0.f;
  }
  const T* dy = dout + (size_t)n * a.P * a.Q * a.O + o;
  for (int p = 0; p < a.P; ++p)
    for (int q = 0; q < a.Q; q += 4) {
      float d[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int qq = q + u < a.Q ? q + u : a.Q - 1;
        const float v = to_f(dy[(size_t)(p * a.Q + qq) * a.O]);
        d[u] = q + u < a.Q ? v : 0.f;
      }
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int qq = q + u < a.Q ? q + u : a.Q - 1;
        const float* base = xs + ((p * a.stride) * Wp + qq * a.stride) * a.C;
#pragma unroll
        for (int t = 0; t < kStemMaxTaps / 4; ++t) acc[t] = fmaf(d[u], base[off[t]], acc[t]);
      }
    }
#pragma unroll
  for (int t = 0; t < kStemMaxTaps / 4; ++t)
    if (t < per && j0 + t < J) ws[((size_t)n * a.O + o) * J + j0 + t] = acc[t];
}

template <typename T>
static hipError_t conv_bwd_weight_t(const OpCtx& c, const ConvArgs& a, const void* dout, const void* x, float* dw,
                                    int accumulate) {
  int Mrows = a.N * a.P * a.Q, J = a.R * a.S * a.C;
  PlainOperand<T> A{(const T*)dout, a.O, 0};            // (o, m) -> dout[m*O + o]
  ConvPatchByCol<T> B{ConvInputPatch<T>{(const T*)x, a}};
  {
    const size_t shm = (size_t)(a.H + 2 * a.pad) * (a.W + 2 * a.pad) * a.C * sizeof(float);
    if (a.C <= 4 && a.O == 64 && J <= kStemMaxTaps && a.N >= 2 && shm <= 48 * 1024 && c.splitk_ws &&
        (size_t)a.N * a.O * J <= c.splitk_elems) {
      k_conv_wgrad_smallc<T><<<a.N, 256, shm, c.stream>>>((const T*)dout, (const T*)x, c.splitk_ws, a);
      size_t total = (size_t)a.O * J;
      k_plain_splitk_reduce<<<(unsigned)((total + 255) / 256), 256, 0, c.stream>>>(c.splitk_ws, dw, total, a.N, accumulate);
      return hipGetLastError();
    }
  }
  // few output tiles and a very long reduction (the stem: 64 x 27 outputs over 262144 pixels): split-K
  int tiles = ((J + PBN - 1) / PBN) * ((a.O + PBM - 1) / PBM);
  int splits = tiles >= 256 ? 1 : 512 / tiles;
  if (splits > Mrows / 256) splits = Mrows / 256;
  while (splits > 1 && (size_t)splits * a.O * J > c.splitk_elems) --splits;
  if (!c.splitk_ws || splits < 2) return launch_plain<T>(c.stream, A, B, plain_out(dw, J, 1, accumulate), a.O, J, Mrows);
  int kper = ((Mrows + splits - 1) / splits + PBK - 1) / PBK * PBK;
  splits = (Mrows + kper - 1) / kper;
  dim3 grid((J + PBN - 1) / PBN, (a.O + PBM - 1) / PBM, splits);
  k_gemm_plain<T, PlainOperand<T>, ConvPatchByCol<T>, 4><<<grid, 256, 0, c.stream>>>(A, B, plain_out(dw, J, 1, 0), a.O, J,
                                                                                 Mrows, kper, c.splitk_ws);
  size_t total = (size_t)a.O * J;
  k_plain_splitk_reduce<<<(unsigned)((total + 255) / 256), 256, 0, c.stream>>>(c.splitk_ws, dw, total, splits, accumulate);
  return hipGetLastError();
}

hipError_t conv_fwd_plain(const OpCtx& c, const ConvArgs& a, const void* x, const void* w, void* out) {
  return c.dt == BF16 ? conv_fwd_t<bf16_t>(c, a, x, w, out) : conv_fwd_t<float>(c, a, x, w, out);
}
hipError_t conv_bwd_data_plain(const OpCtx& c, const ConvArgs& a, const void* dout, const void* w, void* dx,
                               const void* add) {
  return c.dt == BF16 ? conv_bwd_data_t<bf16_t>(c, a, dout, w, dx, add) : conv_bwd_data_t<float>(c, a, dout, w, dx, add);
}
hipError_t conv_bwd_weight_plain(const OpCtx& c, const ConvArgs& a, const void* dout, const void* x, float* dw,
                                 int accumulate) {
  return c.dt == BF16 ? conv_bwd_weight_t<bf16_t>(c, a, dout, x, dw, accumulate)
                      : conv_bwd_weight_t<float>(c, a, dout, x, dw, accumulate);
}

}  // namespace lp
