// bf16 GEMM on the CDNA4 matrix cores: v_mfma_f32_32x32x16_bf16, fp32 accumulation, operands staged
// through LDS with the reduction index contiguous.  Block tile 128x128x32, four 64-wide wavefronts
// in a 2x2 arrangement, each owning a 64x64 sub-tile (2x2 MFMA tiles).  Either operand may be stored
// with the reduction index as its slow dimension (dgrad / wgrad forms); such tiles are transposed on
// their way into LDS.
#include <stdlib.h>
#include "common.h"
#include "gemm_common.h"

namespace lp {

hipError_t gemm_plain(const OpCtx& c, const GemmArgs& g);

constexpr int BM = 128, BN = 128, BK = 32;
constexpr int LDK = BK + 8;   // padded LDS row (elements); 80 bytes keeps 16-byte alignment

struct TileSrc { const bf16_t* p; int64_t ld; int kc; int rows; int vec; };

// Fetch the two 8-element chunks this thread stages for one operand tile.
// kc:  tile is [128 rows][32 k]; chunk c -> row c/4, k-chunk c%4 (8 consecutive k).
// !kc: tile is [32 k][128 rows] in memory; chunk c -> k c/16, row-chunk c%16 (8 consecutive rows).
__device__ __forceinline__ void fetch_chunks(const TileSrc& s, int r0, int k0, int K, bf16x8 v[2]) {
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    int c = threadIdx.x + 256 * i;
    bf16x8 val;
    if (s.kc) {
      int row = r0 + c / 4, k = k0 + (c % 4) * 8;
      if (s.vec && row < s.rows && k + 8 <= K) {
        val = *reinterpret_cast<const bf16x8*>(s.p + (size_t)row * s.ld + k);
      } else {
#pragma unroll
        for (int j = 0; j < 8; ++j)
          val[j] = (row < s.rows && k + j < K) ? s.p[(size_t)row * s.ld + k + j] : (bf16_t)0.f;
      }
    } else {
      int k = k0 + c / 16, row = r0 + (c % 16) * 8;
      if (s.vec && k < K && row + 8 <= s.rows) {
        val = *reinterpret_cast<const bf16x8*>(s.p + (size_t)k * s.ld + row);
      } else {
#pragma unroll
        for (int j = 0; j < 8; ++j)
          val[j] = (k < K && row + j < s.rows) ? s.p[(size_t)k * s.ld + row + j] : (bf16_t)0.f;
      }
    }
    v[i] = val;
  }
}
__device__ __forceinline__ void stage_chunks(int kc, bf16_t (*sm)[LDK], const bf16x8 v[2]) {
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    int c = threadIdx.x + 256 * i;
    if (kc) {
      *reinterpret_cast<bf16x8*>(&sm[c / 4][(c % 4) * 8]) = v[i];
    } else {
      int k = c / 16, row = (c % 16) * 8;
#pragma unroll
      for (int j = 0; j < 8; ++j) sm[row + j][k] = v[i][j];
    }
  }
}

__global__ void __launch_bounds__(256) k_gemm_mfma(TileSrc A, TileSrc B, Epilogue e, int M, int N, int K) {
  __shared__ __attribute__((aligned(16))) bf16_t As[BM][LDK];
  __shared__ __attribute__((aligned(16))) bf16_t Bs[BN][LDK];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wm = (wave >> 1) * 64, wn = (wave & 1) * 64;
  const int m0 = blockIdx.y * BM, n0 = blockIdx.x * BN;
  f32x16 acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  bf16x8 ra[2], rb[2];
  fetch_chunks(A, m0, 0, K, ra);
  fetch_chunks(B, n0, 0, K, rb);
  const int lr = lane & 31, lk = (lane >> 5) * 8;
  for (int k0 = 0; k0 < K; k0 += BK) {
    stage_chunks(A.kc, As, ra);
    stage_chunks(B.kc, Bs, rb);
    __syncthreads();
    if (k0 + BK < K) {
      fetch_chunks(A, m0, k0 + BK, K, ra);
      fetch_chunks(B, n0, k0 + BK, K, rb);
    }
#pragma unroll
    for (int ks = 0; ks < BK; ks += 16) {
      bf16x8 fa[2], fb[2];
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        fa[i] = *reinterpret_cast<const bf16x8*>(&As[wm + i * 32 + lr][ks + lk]);
        fb[i] = *reinterpret_cast<const bf16x8*>(&Bs[wn + i * 32 + lr][ks + lk]);
      }
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], fb[j], acc[i][j], 0, 0, 0);
    }
    __syncthreads();
  }
  // accumulator layout of the 32x32 MFMA: value v of lane l is row 8*(v/4) + 4*(l/32) + v%4, column l%32
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        int m = m0 + wm + i * 32 + 8 * (v / 4) + 4 * (lane >> 5) + (v % 4);
        int n = n0 + wn + j * 32 + lr;
        if (m < M && n < N) epilogue_store<bf16_t>(e, m, n, acc[i][j][v]);
      }
}

static bool aligned16(const void* p) { return ((uintptr_t)p & 15) == 0; }

hipError_t gemm_mfma(const OpCtx& c, const GemmArgs& g) {
  if (g.M <= 0 || g.N <= 0) return hipSuccess;
  TileSrc A{(const bf16_t*)g.A, g.lda, g.a_kc, g.M, (aligned16(g.A) && g.lda % 8 == 0) ? 1 : 0};
  TileSrc B{(const bf16_t*)g.B, g.ldb, g.b_kc, g.N, (aligned16(g.B) && g.ldb % 8 == 0) ? 1 : 0};
  dim3 grid((g.N + BN - 1) / BN, (g.M + BM - 1) / BM);
  k_gemm_mfma<<<grid, 256, 0, c.stream>>>(A, B, make_epilogue(g), g.M, g.N, g.K);
  return hipGetLastError();
}

static int use_plain() {
  static int v = -1;
  if (v < 0) { const char* s = getenv("LP_PLAIN_GEMM"); v = (s && s[0] == '1') ? 1 : 0; }
  return v;
}

hipError_t op_gemm(const OpCtx& c, const GemmArgs& g) {
  ProfScope prof_(c, KC_GEMM, 2.0 * g.M * g.N * g.K);
  if (c.dt == BF16 && !use_plain()) return gemm_mfma(c, g);
  return gemm_plain(c, g);
}

}  // namespace lp
