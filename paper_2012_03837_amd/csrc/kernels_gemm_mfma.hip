// bf16 GEMM on the CDNA4 matrix cores (v_mfma_f32_32x32x16_bf16, fp32 accumulation): the choice between the
// two MFMA kernels and the launch of the register-staged one.
//
// Register-staged kernel (mfma_tile.h): block tile 256 or 128 (m) x 128 (n) x 32 (k), four wavefronts, two
// blocks per CU; operand tiles go global -> registers -> LDS (double buffered, one barrier per k-tile).  It
// takes every 8-aligned shape (K tails are zero-filled while staging) and splits long reductions over few
// tiles uniformly along k (fp32 partial sums, added in split order by k_splitk_reduce).
// Direct-to-LDS kernel (kernels_gemm_dma.hip): persistent, for K % 32 == 0; see there.
// In both, an operand stored with the reduction index contiguous ("kc": forward activations and [out,in]
// weights) sits in LDS as [row][k] and is read with 16-byte ds_read; one stored with the reduction index as the
// slow dimension (dgrad weights, both wgrad operands) sits as [k][row], exactly as in memory, and is read with
// the gfx950 transposing LDS read (ds_read_b64_tr_b16), so nothing is ever transposed by the vector ALU.  The
// MFMA takes the n-side fragment as its first operand, which leaves each lane with runs of 8 consecutive n for
// one m: the fused epilogue (bias, activation, saved pre-activation, activation derivative, residual,
// accumulate) reads and writes 16 bytes per lane.
#include <stdio.h>
#include <stdlib.h>
#include <map>
#include <string>
#include "common.h"
#include "gemm_common.h"
#include "mfma_tile.h"

namespace lp {

hipError_t gemm_plain(const OpCtx& c, const GemmArgs& g);
bool gemm_dma_ok(const GemmArgs& g);
bool gemm_dma_plan(const OpCtx& c, const GemmArgs& g, int kind, int mode, DmaGemmPlan* out);
hipError_t gemm_dma(const OpCtx& c, const GemmArgs& g, const DmaGemmPlan& d);
hipError_t gemm_dma_grouped(const OpCtx& c, const GemmArgs* gs, int n);

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

// Forced kernel: 0 none; 2 register-staged; 3 + 2*kind + cut for the direct-to-LDS kernel of tile shape
// `kind` (0: 256 x 128; 1: 256 x 256 with 8 waves; 2: 256 x 256 with 4 waves) with the tail whole (cut 0)
// or cut along k (cut 1); 9 + kind for that shape in panel mode; 13 + 2*kind for that shape with any of them.
// LP_GEMM_KERNEL = v2 | dma2 | dma4 | dmaw, optionally followed by w, c or p (dma4c, ...), forces one for a
// whole process (for measurements); a shape the forced kernel does not take falls back to the others.
static int env_choice() {
  static int v = -1;
  if (v < 0) {
    const char* s = getenv("LP_GEMM_KERNEL");
    v = 0;
    if (s && s[0] == 'v') v = 2;
    else if (s && s[0] == 'd' && s[1] == 'm' && s[2] == 'a') {
      const int kind = s[3] == '2' ? 0 : (s[3] == '4' ? 1 : (s[3] == 'w' ? 2 : -1));
      if (kind >= 0) v = s[4] == 'w' ? 3 + 2 * kind : (s[4] == 'c' ? 4 + 2 * kind : (s[4] == 'p' ? 9 + kind : 13 + 2 * kind));
    }
  }
  return v;
}

// A small cost model picks the kernel.  Each variant has a measured cost per 32-deep k-step of one block
// and a fixed cost per tile (pipeline fill, epilogue); split-K and the k-cut tail add the traffic of
// their fp32 partial sums and a second launch.
static const double kPartialBytesPerCycle = 4.0e12 / 2.4e9;   // partial sums: written, then read once more
static const double kSecondLaunchCycles = 12000.0;
struct TileVariant { int bm; int per_cu; double step_cycles; double fixed_cycles; };
static const TileVariant kRegStaged[2] = {
    {128, 2, 2097.0, 5000.0},     // 128 x 128, two blocks per CU share the CU: cycles per step per block
    {256, 2, 3226.0, 6000.0},     // 256 x 128
};
static bool trace_on() {     // LP_GEMM_TRACE=1 prints the chosen kernel and plan of every GEMM (for measurements)
  static int v = -1;
  if (v < 0) { const char* s = getenv("LP_GEMM_TRACE"); v = (s && s[0] == '1') ? 1 : 0; }
  return v != 0;
}
static const double kDmaStep[4] = {2796.0, 2300.0, 2300.0, 4200.0};      // 256 x 128 (two per CU), 256 x 256; 64-deep
static const double kDmaFixed[4] = {7000.0, 9000.0, 9000.0, 9000.0};

static bool deep_auto() {     // LP_GEMM_K64=0 keeps the 64-deep k-tiles out of the automatic choice (for measurements)
  static int v = -1;
  if (v < 0) { const char* s = getenv("LP_GEMM_K64"); v = (s && s[0] == '0') ? 0 : 1; }
  return v != 0;
}

hipError_t gemm_mfma(const OpCtx& c, const GemmArgs& g) {
  if (g.M <= 0 || g.N <= 0) return hipSuccess;
  const int choice = c.gemm_variant ? c.gemm_variant : env_choice();
  double best = 1e300;
  // direct-to-LDS persistent kernel: tile shape x (tail whole, cut along k, panel mode)
  DmaGemmPlan best_dma;
  bool use_dma = false;
  int force_kind = -1, force_cut = -1;
  if (choice >= 20 && choice <= 22) { force_kind = 3; force_cut = choice - 20; }     // 64-deep k-tiles: tail whole / cut / panel mode
  else if (choice >= 13) force_kind = (choice - 13) / 2;
  else if (choice >= 9) { force_kind = choice - 9; force_cut = 2; }
  else if (choice >= 3) { force_kind = (choice - 3) / 2; force_cut = (choice - 3) % 2; }
  // Short reductions over at most two waves of tiles (a layer's K = 768 products): a block that owns its CU
  // has nothing to overlap its fused epilogue with and its pipeline never reaches steady state; the
  // register-staged kernel with two blocks per CU measured 10-30 % faster there, so it takes them.
  const bool short_and_few = g.K <= 1024 && (long)((g.M + 255) / 256) * ((g.N + 255) / 256) <= 512;
  if (gemm_dma_ok(g) && choice != 2 && !(choice == 0 && short_and_few)) {
    for (int kind = 0; kind < 4; ++kind) {
      if (force_kind >= 0 ? kind != force_kind : (kind == 2 || (kind == 3 && !deep_auto()))) continue;   // the 4-wave shape only when asked for
      for (int cut = 0; cut < 3; ++cut) {                 // tail whole / cut along k / panel mode
        if (force_cut >= 0 && cut != force_cut) continue;
        DmaGemmPlan d;
        if (!gemm_dma_plan(c, g, kind, cut, &d)) continue;
        if (cut == 1 && d.partial_bytes == 0 && force_cut < 0) continue;      // same as the uncut plan
        double cycles = d.steps * kDmaStep[kind] + d.items * kDmaFixed[kind];
        if (d.partial_bytes > 0) cycles += 2.0 * d.partial_bytes / kPartialBytesPerCycle + kSecondLaunchCycles;
        // cut along k tile by tile, the tile columns of a row are at different k-steps and each fetches the
        // row's operand for itself: measured ~8 % slower than panel mode on a vocabulary head's gradients
        if (cut == 1 && d.partial_bytes > 0 && d.tiles_n >= 2 && d.tiles_n <= 8) cycles *= 1.12;
        if (cycles < best) { best = cycles; best_dma = d; use_dma = true; }
      }
    }
  }
  // register-staged kernel: any aligned shape, uniform split-K
  int best_v = 0, best_s = 1;
  if (c.gemm_variant > 2 && !use_dma) return hipErrorInvalidValue;   // the forced kernel does not take this shape
  if (choice <= 2 || !use_dma) {
    for (int vi = 0; vi < 2; ++vi) {
      const TileVariant& v = kRegStaged[vi];
      const long tiles = (long)((g.M + v.bm - 1) / v.bm) * ((g.N + BN - 1) / BN);
      const long slots = 256L * v.per_cu;
      for (int sp = 1; sp <= 8; ++sp) {
        if (sp > 1 && (!c.splitk_ws || g.K / sp < 512 || (size_t)sp * g.M * g.N > c.splitk_elems)) break;
        const long rounds = (tiles * sp + slots - 1) / slots;
        double cycles = rounds * (((double)g.K / sp / BK) * v.step_cycles + v.fixed_cycles);
        if (sp > 1) cycles += 2.0 * sp * (double)g.M * g.N * 4.0 / kPartialBytesPerCycle + kSecondLaunchCycles;
        if (cycles < best) { best = cycles; best_v = vi; best_s = sp; use_dma = false; }
      }
    }
  }
  if (trace_on())
    fprintf(stderr, "lp gemm %d x %d x %d (%d%d): %s kind %d full %d tail %d upb %d/%d sib %d split %d est %.0f cycles\n", g.M, g.N, g.K,
            g.a_kc, g.b_kc, use_dma ? "direct-to-LDS" : "register-staged", use_dma ? best_dma.kind : best_v,
            use_dma ? best_dma.full : 0, use_dma ? best_dma.tail_tiles : 0, use_dma ? best_dma.upb : 0,
            use_dma ? best_dma.kt : 0, use_dma ? best_dma.sib : 0, use_dma ? 1 : best_s, best);
  if (use_dma) return gemm_dma(c, g, best_dma);

  const int splits = best_s;
  Epilogue e = make_epilogue(g);
  Operand A{(const bf16_t*)g.A, g.lda, g.M}, B{(const bf16_t*)g.B, g.ldb, g.N};
  const int bm = kRegStaged[best_v].bm, tn = (g.N + BN - 1) / BN, tm = (g.M + bm - 1) / bm;
  dim3 grid(tm * tn * splits);
  char kname_buf[112];
  snprintf(kname_buf, sizeof kname_buf, "mfma::k_mfma_tiles<mfma::PlainLoader<%s>, mfma::PlainLoader<%s>, %d, 128, false>",
           g.a_kc ? "true" : "false", g.b_kc ? "true" : "false", bm);
  static std::map<std::string, std::string> names;       // stable storage for the profiler's name pointers
  const char* kname = names.emplace(kname_buf, kname_buf).first->second.c_str();
  ProfScope one_(c, KC_GEMM_KERNEL, 2.0 * g.M * g.N * g.K, 0, kname);
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
  hipError_t err = hipGetLastError();
  one_.finish();
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
  const uint64_t tag = (uint64_t)(g.M & 0xfffff) | (uint64_t)(g.N & 0xfffff) << 20 | (uint64_t)(g.K & 0xfffff) << 40 |
                       (uint64_t)(g.a_kc != 0) << 60 | (uint64_t)(g.b_kc != 0) << 61 | (uint64_t)(g.c_f32 != 0) << 62;
  ProfScope prof_(c, KC_GEMM, 2.0 * g.M * g.N * g.K, tag);
  if (c.gemm_variant >= 2 && !(c.dt == BF16 && fast_ok(g))) return hipErrorInvalidValue;
  if (c.dt == BF16 && !use_plain() && fast_ok(g)) return gemm_mfma(c, g);
  return gemm_plain(c, g);
}

static bool grouping_off() {     // LP_NO_GROUP=1: every product in a launch of its own (for measurements)
  static int v = -1;
  if (v < 0) { const char* s = getenv("LP_NO_GROUP"); v = (s && s[0] == '1') ? 1 : 0; }
  return v != 0;
}

hipError_t op_gemm_grouped(const OpCtx& c, const GemmArgs* gs, int n) {
  if (n >= 2 && c.dt == BF16 && !use_plain() && !grouping_off() && c.gemm_variant == 0 && env_choice() == 0) {
    bool ok = true;
    for (int i = 0; i < n; ++i) ok = ok && fast_ok(gs[i]);
    if (ok) {
      hipError_t e = gemm_dma_grouped(c, gs, n);
      if (e != hipErrorInvalidValue) return e;          // launched (or failed for a reason of the device's)
    }
  }
  for (int i = 0; i < n; ++i) {
    hipError_t e = op_gemm(c, gs[i]);
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

}  // namespace lp
