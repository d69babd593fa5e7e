// 3x3 / 1x1 convolutions over NHWC bf16 activations as implicit GEMMs on the matrix cores.  No im2col
// buffer exists: the operand loaders of the MFMA tile kernel gather pixels directly (16 bytes = 8
// consecutive channels per lane) and report zero padding / stride holes as invalid chunks, which the
// LDS staging step zero-fills.
//   forward : out[(n,p,q), o]  = sum_{(r,s,c)} x[n, p*st+r-pad, q*st+s-pad, c] * w[o, r, s, c]
//   dgrad   : dx[(n,h,w), c]   = sum_{(r,s,o)} dout[n, (h+pad-r)/st, (w+pad-s)/st, o] * w[o, r, s, c]
//   wgrad   : dw[o, (r,s,c)]   = sum_{(n,p,q)} dout[(n,p,q), o] * x[n, p*st+r-pad, q*st+s-pad, c]   (fp32, split-K)
// Needs C % 8 == 0 and O % 8 == 0; the 3-channel stem convolution stays on the plain kernel.
#include <stdio.h>
#include <type_traits>
#include "common.h"
#include "gemm_common.h"
#include "mfma_tile.h"

namespace lp {

namespace {

using namespace mfma;

// forward A operand: rows (n,p,q), k = (r,s,c), reduction index contiguous.
struct ConvFwdA {
  static constexpr bool KC = true;
  const bf16_t* x; ConvArgs a; int M;
  int h0[4], w0[4], nb[4];
  template <int ROWS> __device__ __forceinline__ void init(int r0) {
#pragma unroll
    for (int i = 0; i < ROWS / 64; ++i) {
      int row = r0 + (threadIdx.x >> 2) + 64 * i;
      if (row < M) {
        int q = row % a.Q, t = row / a.Q, p = t % a.P, n = t / a.P;
        h0[i] = p * a.stride - a.pad; w0[i] = q * a.stride - a.pad; nb[i] = n * a.H * a.W;
      } else {
        h0[i] = -(1 << 20); w0[i] = 0; nb[i] = 0;
      }
    }
  }
  template <int ROWS> __device__ __forceinline__ unsigned fetch(int, int k0, int K, bf16x8* v) const {
    int kk = k0 + (threadIdx.x & 3) * 8;
    bool kok = kk < K;
    int rs = kok ? kk / a.C : 0, c = kok ? kk - rs * a.C : 0;
    int r = rs / a.S, s = rs - r * a.S;
    unsigned inv = 0;
#pragma unroll
    for (int i = 0; i < ROWS / 64; ++i) {
      int h = h0[i] + r, w = w0[i] + s;
      bool ok = kok && (unsigned)h < (unsigned)a.H && (unsigned)w < (unsigned)a.W;
      size_t off = ok ? ((size_t)(nb[i] + h * a.W + w) * a.C + c) : 0;
      v[i] = *reinterpret_cast<const bf16x8*>(x + off);
      inv |= (ok ? 0u : 1u) << i;
    }
    return inv;
  }
};

// dgrad A operand: rows (n,h,w) of the input, k = (r,s,o), gathered from dout.
struct ConvBwdA {
  static constexpr bool KC = true;
  const bf16_t* d; ConvArgs a; int M;
  int hp0[4], wp0[4], nb[4];
  template <int ROWS> __device__ __forceinline__ void init(int r0) {
#pragma unroll
    for (int i = 0; i < ROWS / 64; ++i) {
      int row = r0 + (threadIdx.x >> 2) + 64 * i;
      if (row < M) {
        int w = row % a.W, t = row / a.W, h = t % a.H, n = t / a.H;
        hp0[i] = h + a.pad; wp0[i] = w + a.pad; nb[i] = n * a.P * a.Q;
      } else {
        hp0[i] = -(1 << 20); wp0[i] = 0; nb[i] = 0;
      }
    }
  }
  template <int ROWS> __device__ __forceinline__ unsigned fetch(int, int k0, int K, bf16x8* v) const {
    int kk = k0 + (threadIdx.x & 3) * 8;
    bool kok = kk < K;
    int rs = kok ? kk / a.O : 0, o = kok ? kk - rs * a.O : 0;
    int r = rs / a.S, s = rs - r * a.S;
    unsigned inv = 0;
#pragma unroll
    for (int i = 0; i < ROWS / 64; ++i) {
      int hp = hp0[i] - r, wq = wp0[i] - s;
      bool ok = kok && hp >= 0 && wq >= 0;
      int p = 0, q = 0;
      if (ok) {
        p = hp / a.stride; q = wq / a.stride;
        ok = (p * a.stride == hp) && (q * a.stride == wq) && p < a.P && q < a.Q;
      }
      size_t off = ok ? ((size_t)(nb[i] + p * a.Q + q) * a.O + o) : 0;
      v[i] = *reinterpret_cast<const bf16x8*>(d + off);
      inv |= (ok ? 0u : 1u) << i;
    }
    return inv;
  }
};

// dgrad B operand: rows = input channel c (contiguous in memory), k = (r,s,o): w[o, r, s, c].
struct ConvFilterT {
  static constexpr bool KC = false;
  const bf16_t* w; ConvArgs a;
  template <int ROWS> __device__ __forceinline__ void init(int) {}
  template <int ROWS> __device__ __forceinline__ unsigned fetch(int r0, int k0, int K, bf16x8* v) const {
    constexpr int CPR = ROWS / 8;
    int row = r0 + (threadIdx.x % CPR) * 8;
    row = row + 8 <= a.C ? row : a.C - 8;
#pragma unroll
    for (int i = 0; i < ROWS / 64; ++i) {
      int k = k0 + threadIdx.x / CPR + (256 / CPR) * i;
      k = k < K ? k : 0;
      int rs = k / a.O, o = k - rs * a.O;
      v[i] = *reinterpret_cast<const bf16x8*>(w + ((size_t)o * a.R * a.S + rs) * a.C + row);
    }
    return 0u;
  }
};

// wgrad B operand: rows j = (r,s,c) (c contiguous), k = output pixel (n,p,q): gathered input patches.
struct ConvPatchT {
  static constexpr bool KC = false;
  const bf16_t* x; ConvArgs a; int J;
  int r, s, c0; bool jok;
  template <int ROWS> __device__ __forceinline__ void init(int r0) {
    constexpr int CPR = ROWS / 8;
    int j = r0 + (threadIdx.x % CPR) * 8;
    jok = j < J;
    int rs = jok ? j / a.C : 0;
    c0 = jok ? j - rs * a.C : 0;
    r = rs / a.S; s = rs - r * a.S;
  }
  template <int ROWS> __device__ __forceinline__ unsigned fetch(int, int k0, int K, bf16x8* v) const {
    constexpr int CPR = ROWS / 8;
    unsigned inv = 0;
#pragma unroll
    for (int i = 0; i < ROWS / 64; ++i) {
      int k = k0 + threadIdx.x / CPR + (256 / CPR) * i;
      bool ok = jok && k < K;
      size_t off = 0;
      if (ok) {
        int q = k % a.Q, t = k / a.Q, p = t % a.P, n = t / a.P;
        int h = p * a.stride + r - a.pad, w = q * a.stride + s - a.pad;
        ok = (unsigned)h < (unsigned)a.H && (unsigned)w < (unsigned)a.W;
        if (ok) off = ((size_t)(n * a.H + h) * a.W + w) * a.C + c0;
      }
      v[i] = *reinterpret_cast<const bf16x8*>(x + off);
      inv |= (ok ? 0u : 1u) << i;
    }
    return inv;
  }
};

__global__ void k_conv_splitk_reduce(const float* __restrict__ ws, float* __restrict__ out, int M, int N, int splits,
                                     int accumulate) {
  size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  size_t total = (size_t)M * N;
  if (idx >= total) return;
  // four running sums (pieces s, s+4, ... each) keep four loads in flight; combined in a fixed order
  float a[4] = {0.f, 0.f, 0.f, 0.f};
  int s = 0;
  for (; s + 4 <= splits; s += 4) {
#pragma unroll
    for (int u = 0; u < 4; ++u) a[u] += ws[(size_t)(s + u) * total + idx];
  }
  for (; s < splits; ++s) a[0] += ws[(size_t)s * total + idx];
  const float t = (a[0] + a[1]) + (a[2] + a[3]);
  out[idx] = accumulate ? out[idx] + t : t;
}

// The same sum for a compute-dtype output: 8 consecutive columns per thread, through the epilogue.
__global__ void k_conv_splitk_reduce8(const float* __restrict__ ws, Epilogue e, int M, int N, int splits) {
  size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int n8 = N >> 3;
  if (idx >= (size_t)M * n8) return;
  const int m = (int)(idx / n8), n = (int)(idx % n8) * 8;
  float v[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  for (int s = 0; s < splits; ++s) {
    const float* p = ws + ((size_t)s * M + m) * N + n;
    f32x4 a = *reinterpret_cast<const f32x4*>(p), b = *reinterpret_cast<const f32x4*>(p + 4);
#pragma unroll
    for (int x = 0; x < 4; ++x) { v[x] += a[x]; v[4 + x] += b[x]; }
  }
  epilogue8(e, m, n, v);
}

Epilogue plain_epilogue(void* C, int64_t ldc, int c_f32, int accumulate) {
  GemmArgs g; g.C = C; g.ldc = ldc; g.c_f32 = c_f32; g.accumulate = accumulate;
  return make_epilogue(g);
}

// `loaders` names the two loader types as a profiler prints them: the launch is timed under the kernel's name.
// st (forward convolutions only): if the launch qualifies (whole tiles, one piece, room in st->buf) the kernel also
// leaves the normalisation's per-sub-tile column statistics there and st->nslab / st->slab_rows say how many.
template <class LA, class LB>
hipError_t launch(const OpCtx& c, LA A, LB B, const Epilogue& e, int M, int N, int K, int splits, const char* loaders,
                  ConvStats* st = nullptr) {
  const bool narrow = N <= 64;                 // 64-column tiles: no padded half (the 64-channel convolutions)
  const int bn = narrow ? 64 : BN;
  const int tn = (N + bn - 1) / bn;
  const bool big = ((M + 255) / 256) * tn * splits >= 400;
  const bool low = M <= 64 && !narrow;         // 64-row tiles (the filter gradient of a 64-channel convolution)
  const int bm = low ? 64 : (big ? 256 : 128);
  const int tm = (M + bm - 1) / bm;
  dim3 grid(tm * tn * splits);
  bool stats = false;
  if constexpr (std::is_same<LA, ConvFwdA>::value) {
    if (st && st->buf && !low && splits == 1 && !e.c_f32 && M % bm == 0 && N % bn == 0) {
      if ((size_t)3 * (M / bm) * N <= st->cap) { stats = true; st->nslab = M / bm; st->slab_rows = bm; }
    }
  }
  static char names[10][104];
  char* kname = names[(low ? 4 : (big ? 1 : 0) + (narrow ? 2 : 0)) + (stats ? 5 : 0)];
  if (!kname[0]) snprintf(kname, sizeof names[0], "mfma::k_mfma_tiles<%s, %d, %d, %s>", loaders, bm, bn, stats ? "true" : "false");
  ProfScope one_(c, KC_GEMM_KERNEL, 2.0 * M * N * K, 0, kname);
  if constexpr (std::is_same<LA, ConvFwdA>::value) {
    if (stats) {
      if (narrow) {
        if (big) k_mfma_tiles<LA, LB, 256, 64, true><<<grid, 256, 0, c.stream>>>(A, B, e, M, N, K, tm, tn, 1, st->buf);
        else k_mfma_tiles<LA, LB, 128, 64, true><<<grid, 256, 0, c.stream>>>(A, B, e, M, N, K, tm, tn, 1, st->buf);
      } else {
        if (big) k_mfma_tiles<LA, LB, 256, 128, true><<<grid, 256, 0, c.stream>>>(A, B, e, M, N, K, tm, tn, 1, st->buf);
        else k_mfma_tiles<LA, LB, 128, 128, true><<<grid, 256, 0, c.stream>>>(A, B, e, M, N, K, tm, tn, 1, st->buf);
      }
      return hipGetLastError();
    }
  }
  if (low) {
    k_mfma_tiles<LA, LB, 64><<<grid, 256, 0, c.stream>>>(A, B, e, M, N, K, tm, tn, splits, c.splitk_ws);
  } else if (narrow) {
    if (big) k_mfma_tiles<LA, LB, 256, 64><<<grid, 256, 0, c.stream>>>(A, B, e, M, N, K, tm, tn, splits, c.splitk_ws);
    else k_mfma_tiles<LA, LB, 128, 64><<<grid, 256, 0, c.stream>>>(A, B, e, M, N, K, tm, tn, splits, c.splitk_ws);
  } else {
    if (big) k_mfma_tiles<LA, LB, 256><<<grid, 256, 0, c.stream>>>(A, B, e, M, N, K, tm, tn, splits, c.splitk_ws);
    else k_mfma_tiles<LA, LB, 128><<<grid, 256, 0, c.stream>>>(A, B, e, M, N, K, tm, tn, splits, c.splitk_ws);
  }
  return hipGetLastError();
}

bool al16(const void* p) { return ((uintptr_t)p & 15) == 0; }

// Forward and data-gradient products of the late stages have few output tiles and a long reduction (4 x 4
// images with 512 channels: 128 tiles, K = 4608): a block alone on its CU cannot hide the gather latency, and
// half the CUs get nothing.  Such products are cut along k into enough pieces for two to three blocks per CU;
// the fp32 partial sums (M x N per piece) are added in piece order.
template <class LA, class LB>
hipError_t launch_cut(const OpCtx& c, LA A, LB B, void* out, int M, int N, int K, const char* loaders,
                      const void* add = nullptr, ConvStats* st = nullptr) {
  const int tiles = ((M + 127) / 128) * (N <= 64 ? 1 : (N + BN - 1) / BN);
  int splits = 1;
  if (c.splitk_ws && tiles < 200 && K >= 1024) {
    splits = (512 + tiles - 1) / tiles;
    if (splits > K / 512) splits = K / 512;
    while (splits > 1 && (size_t)splits * M * N > c.splitk_elems) --splits;
    if (splits < 1) splits = 1;
  }
  Epilogue e = plain_epilogue(out, N, 0, 0);
  e.res = add; e.ldr = N;      // a tensor of the output's shape added to the result
  hipError_t err = launch(c, A, B, e, M, N, K, splits, loaders, st);
  if (err != hipSuccess || splits == 1) return err;
  const size_t work = (size_t)M * (N / 8);
  k_conv_splitk_reduce8<<<(unsigned)((work + 255) / 256), 256, 0, c.stream>>>(c.splitk_ws, e, M, N, splits);
  return hipGetLastError();
}

}  // namespace

bool conv_mfma_ok(const OpCtx& c, const ConvArgs& a, const void* p0, const void* p1, const void* p2) {
  return c.dt == BF16 && a.C % 8 == 0 && a.O % 8 == 0 && a.C >= 8 && a.O >= 8 && al16(p0) && al16(p1) && al16(p2);
}

hipError_t conv_fwd_mfma(const OpCtx& c, const ConvArgs& a, const void* x, const void* w, void* out, ConvStats* st) {
  const int M = a.N * a.P * a.Q, K = a.R * a.S * a.C;
  ConvFwdA A{(const bf16_t*)x, a, M};
  PlainLoader<true> B{Operand{(const bf16_t*)w, K, a.O}};
  return launch_cut(c, A, B, out, M, a.O, K, "ConvFwdA, mfma::PlainLoader<true>", nullptr, st);
}
hipError_t conv_bwd_data_mfma(const OpCtx& c, const ConvArgs& a, const void* dout, const void* w, void* dx,
                              const void* add) {
  const int M = a.N * a.H * a.W, K = a.R * a.S * a.O;
  ConvBwdA A{(const bf16_t*)dout, a, M};
  ConvFilterT B{(const bf16_t*)w, a};
  return launch_cut(c, A, B, dx, M, a.C, K, "ConvBwdA, ConvFilterT", add);
}
hipError_t conv_bwd_weight_mfma(const OpCtx& c, const ConvArgs& a, const void* dout, const void* x, float* dw,
                                int accumulate) {
  const int Mrows = a.N * a.P * a.Q, J = a.R * a.S * a.C;
  PlainLoader<false> A{Operand{(const bf16_t*)dout, a.O, a.O}};
  ConvPatchT B{(const bf16_t*)x, a, J};
  const int tiles = ((a.O + 127) / 128) * ((J + BN - 1) / BN);
  int splits = 1;
  if (c.splitk_ws) {
    splits = (512 + tiles - 1) / tiles;
    if (splits > 64) splits = 64;
    if (splits > Mrows / 512) splits = Mrows / 512;
    while (splits > 1 && (size_t)splits * a.O * J > c.splitk_elems) --splits;
    if (splits < 1) splits = 1;
  }
  hipError_t e = launch(c, A, B, plain_epilogue(dw, J, 1, accumulate), a.O, J, Mrows, splits,
                        "mfma::PlainLoader<false>, ConvPatchT");
  if (e != hipSuccess || splits == 1) return e;
  size_t total = (size_t)a.O * J;
  k_conv_splitk_reduce<<<(unsigned)((total + 255) / 256), 256, 0, c.stream>>>(c.splitk_ws, dw, a.O, J, splits, accumulate);
  return hipGetLastError();
}

}  // namespace lp
