// bf16 GEMM on the CDNA4 matrix cores (v_mfma_f32_32x32x16_bf16, fp32 accumulation).
//
// Block tile 256(m) x 128(n) x 32(k), 256 threads = four 64-wide wavefronts in a 2x2 arrangement, each
// owning 128 x 64 (4 x 2 MFMA tiles, 128 accumulator registers), two blocks per CU.  Operand tiles go
// global -> registers -> LDS (double buffered, one barrier per k-tile).  An operand stored with the
// reduction index contiguous ("kc": forward activations and [out,in] weights) sits in LDS as
// [row][k] and is read with 16-byte ds_read; one stored with the reduction index as the slow
// dimension (dgrad weights, both wgrad operands) sits as [k][row], exactly as in memory, and is read
// with the gfx950 transposing LDS read (ds_read_b64_tr_b16), so nothing is ever transposed by the
// vector ALU.  The MFMA takes the n-side fragment as its first operand, which leaves each lane with
// runs of 8 consecutive n for one m: the fused epilogue (bias, activation, saved pre-activation,
// activation derivative, residual, accumulate) reads and writes 16 bytes per lane.
// Blocks are renumbered so that each XCD (blocks are dealt round-robin to the 8 XCDs) walks a
// compact group of tiles and re-uses its own L2.
#include <stdlib.h>
#include "common.h"
#include "gemm_common.h"
#include "mfma_tile.h"

namespace lp {

hipError_t gemm_plain(const OpCtx& c, const GemmArgs& g);
bool gemm_dma_ok(const GemmArgs& g);
hipError_t gemm_dma(const OpCtx& c, const GemmArgs& g, int nwn, int splits);

namespace {

using namespace mfma;

// Sums split-K partials in split order and applies the epilogue; one thread per 8 columns.
__global__ void k_splitk_reduce(const float* __restrict__ ws, Epilogue e, int M, int N, int splits) {
  size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  int n8 = N >> 3;
  if (idx >= (size_t)M * n8) return;
  int m = (int)(idx / n8), n = (int)(idx % n8) * 8;
  float v[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  for (int s = 0; s < splits; ++s) {
    const float* p = ws + ((size_t)s * M + m) * N + n;
    f32x4 a = *reinterpret_cast<const f32x4*>(p), b = *reinterpret_cast<const f32x4*>(p + 4);
#pragma unroll
    for (int x = 0; x < 4; ++x) { v[x] += a[x]; v[4 + x] += b[x]; }
  }
  epilogue8(e, m, n, v);
}

bool aligned16(const void* p) { return ((uintptr_t)p & 15) == 0; }

// Shapes the MFMA kernel takes: every vector access must be 16-byte aligned and never straddle an edge.
bool fast_ok(const GemmArgs& g) {
  if (g.M < 1 || g.N < 8 || g.K < 1) return false;
  if (g.N % 8 || g.K % 8 || g.lda % 8 || g.ldb % 8 || g.ldc % 8) return false;
  if (!g.a_kc && (g.M % 8 || g.M < 8)) return false;
  if (!aligned16(g.A) || !aligned16(g.B) || !aligned16(g.C)) return false;
  if (g.bias && !aligned16(g.bias)) return false;
  if (g.pre && !aligned16(g.pre)) return false;
  if (g.dact_src && (!aligned16(g.dact_src) || g.ldd % 8)) return false;
  if (g.res && (!aligned16(g.res) || g.ldr % 8)) return false;
  return true;
}

}  // namespace

// Tile and split choice.  Big tiles when they fill the chip; otherwise 128-row tiles, and for long
// reductions over few tiles (weight gradients over all tokens, the head's input gradient over the
// vocabulary) split-K with fp32 partials summed in split order by a second kernel.
static int kernel_choice() {   // LP_GEMM_KERNEL = auto | v2 | dma4 | dma2 (for measurements)
  static int v = -1;
  if (v < 0) {
    const char* s = getenv("LP_GEMM_KERNEL");
    v = !s ? 0 : (s[0] == 'v' ? 1 : (s[0] == 'd' && s[3] == '4' ? 2 : (s[0] == 'd' && s[3] == '2' ? 3 : 0)));
  }
  return v;
}

// Kernel variants and a small cost model to choose among them.  A variant is a tile shape with a
// number of resident blocks per CU and a measured sustained rate for a full CU; the estimate is
// rounds x (tile time + fixed fill/drain time) plus the traffic of split-K partial sums.
struct Variant { int kind; int bm, bn; int per_cu; double flops_per_cycle_cu; double fixed_cycles; };
static const Variant kVariants[] = {
    {2, 256, 256, 1, 1700.0, 9000.0},   // direct-to-LDS, 8 waves, 4 stages
    {3, 256, 128, 2, 1500.0, 7000.0},   // direct-to-LDS, 4 waves, 3 stages
    {1, 256, 128, 2, 1300.0, 6000.0},   // register-staged, big tile
    {0, 128, 128, 2, 1000.0, 5000.0},   // register-staged, small tile
};

hipError_t gemm_mfma(const OpCtx& c, const GemmArgs& g) {
  if (g.M <= 0 || g.N <= 0) return hipSuccess;
  const int choice = kernel_choice();
  const bool dma_ok = gemm_dma_ok(g);
  const double flops = 2.0 * g.M * g.N * g.K;
  double best = 1e300;
  int best_v = 3, best_s = 1;
  for (int vi = 0; vi < 4; ++vi) {
    const Variant& v = kVariants[vi];
    if ((v.kind >= 2) && !dma_ok) continue;
    if (choice == 1 && v.kind >= 2) continue;
    if (choice == 2 && v.kind != 2) continue;
    if (choice == 3 && v.kind != 3) continue;
    const long tiles = (long)((g.M + v.bm - 1) / v.bm) * ((g.N + v.bn - 1) / v.bn);
    const long slots = 256L * v.per_cu;
    for (int sp = 1; sp <= 8; ++sp) {
      if (sp > 1 && (!c.splitk_ws || g.K / sp < 512 || (size_t)sp * g.M * g.N > c.splitk_elems)) break;
      const long blocks = tiles * sp;
      const long rounds = (blocks + slots - 1) / slots;
      const double tile_cycles = 2.0 * v.bm * v.bn * ((double)g.K / sp) / (v.flops_per_cycle_cu / v.per_cu);
      double cycles = rounds * (tile_cycles + v.fixed_cycles);
      if (sp > 1) cycles += 2.0 * sp * (double)g.M * g.N * 4.0 / (5.0e12 / 2.4e9) + 12000.0;
      if (cycles < best) { best = cycles; best_v = vi; best_s = sp; }
    }
  }
  (void)flops;
  const Variant& v = kVariants[best_v];
  const int splits = best_s;
  Epilogue e = make_epilogue(g);
  hipError_t err;
  if (v.kind >= 2) {
    err = gemm_dma(c, g, v.kind == 2 ? 4 : 2, splits);
  } else {
    Operand A{(const bf16_t*)g.A, g.lda, g.M}, B{(const bf16_t*)g.B, g.ldb, g.N};
    const int bm = v.bm, tn = (g.N + BN - 1) / BN, tm = (g.M + bm - 1) / bm;
    dim3 grid(tm * tn * splits);
#define LP_GEMM(AK, BK_, BM_)                                                                             \
  k_mfma_tiles<PlainLoader<AK>, PlainLoader<BK_>, BM_><<<grid, 256, 0, c.stream>>>(                       \
      PlainLoader<AK>{A}, PlainLoader<BK_>{B}, e, g.M, g.N, g.K, tm, tn, splits, c.splitk_ws)
#define LP_GEMM_BM(AK, BK_) do { if (bm == 256) LP_GEMM(AK, BK_, 256); else LP_GEMM(AK, BK_, 128); } while (0)
    if (g.a_kc && g.b_kc) LP_GEMM_BM(true, true);
    else if (g.a_kc && !g.b_kc) LP_GEMM_BM(true, false);
    else if (!g.a_kc && g.b_kc) LP_GEMM_BM(false, true);
    else LP_GEMM_BM(false, false);
#undef LP_GEMM_BM
#undef LP_GEMM
    err = hipGetLastError();
  }
  if (err != hipSuccess || splits == 1) return err;
  size_t work = (size_t)g.M * (g.N / 8);
  k_splitk_reduce<<<(unsigned)((work + 255) / 256), 256, 0, c.stream>>>(c.splitk_ws, e, g.M, g.N, splits);
  return hipGetLastError();
}

static int use_plain() {
  static int v = -1;
  if (v < 0) { const char* s = getenv("LP_PLAIN_GEMM"); v = (s && s[0] == '1') ? 1 : 0; }
  return v;
}

hipError_t op_gemm(const OpCtx& c, const GemmArgs& g) {
  ProfScope prof_(c, KC_GEMM, 2.0 * g.M * g.N * g.K);
  if (c.dt == BF16 && !use_plain() && fast_ok(g)) return gemm_mfma(c, g);
  return gemm_plain(c, g);
}

}  // namespace lp
