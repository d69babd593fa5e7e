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

namespace lp {

hipError_t gemm_plain(const OpCtx& c, const GemmArgs& g);
bool gemm_dma_ok(const GemmArgs& g);
hipError_t gemm_dma(const OpCtx& c, const GemmArgs& g, int nwn, int splits);

namespace {

constexpr int BN = 128, BK = 32;
constexpr int KC_LD = BK + 8;        // [row][k] tiles: 80-byte rows
constexpr int TB_LD = BN + 16;       // [k][row] tiles: padded rows
constexpr int B_ELEMS = BN * KC_LD > BK * TB_LD ? BN * KC_LD : BK * TB_LD;

typedef __attribute__((address_space(3))) bf16x4 lds_bf16x4;

struct Operand { const bf16_t* p; int64_t ld; int rows; };

// MFMA row i of the n-side fragment holds tile column 16*(g/2) + 8*h + 4*(g%2) + j, i = 8g + 4h + j, so
// that accumulator values 0..7 / 8..15 of lane-half h are columns 8h..8h+7 / 16+8h..16+8h+7.
__device__ __forceinline__ int nmap(int i) {
  int g = i >> 3, h = (i >> 2) & 1, j = i & 3;
  return 16 * (g >> 1) + 8 * h + 4 * (g & 1) + j;
}

// ---- global -> registers ------------------------------------------------------------------------
// kc tile [ROWS][32]: ROWS*4 chunks of 8 k; thread takes chunks tid + 256*i.
template <int ROWS>
__device__ __forceinline__ void fetch_kc(const Operand& o, int r0, int k0, int K, bf16x8* v) {
#pragma unroll
  for (int i = 0; i < ROWS / 64; ++i) {
    int c = threadIdx.x + 256 * i;
    int row = r0 + (c >> 2), k = k0 + (c & 3) * 8;
    row = row < o.rows ? row : o.rows - 1;
    v[i] = *reinterpret_cast<const bf16x8*>(o.p + (size_t)row * o.ld + (k < K ? k : 0));
  }
}
// transposed tile, memory [32 k][ROWS]: 32*ROWS/8 chunks of 8 rows; thread takes chunks tid + 256*i.
template <int ROWS>
__device__ __forceinline__ void fetch_t(const Operand& o, int r0, int k0, int K, bf16x8* v) {
  constexpr int CPR = ROWS / 8;   // chunks per k-row
#pragma unroll
  for (int i = 0; i < ROWS / 64; ++i) {
    int c = threadIdx.x + 256 * i;
    int k = k0 + c / CPR, row = r0 + (c % CPR) * 8;
    row = row + 8 <= o.rows ? row : o.rows - 8;
    v[i] = *reinterpret_cast<const bf16x8*>(o.p + (size_t)(k < K ? k : 0) * o.ld + row);
  }
}
// ---- registers -> LDS ---------------------------------------------------------------------------
// Chunks whose k lies beyond K (only in the last k-tile) are zeroed here, at the point where the loaded
// registers are first needed, so that the loads themselves stay in flight across the MFMA phase.
__device__ __forceinline__ bf16x8 zero_if(bf16x8 t, bool z) {
  if (z) {
#pragma unroll
    for (int e = 0; e < 8; ++e) t[e] = (bf16_t)0.f;
  }
  return t;
}
template <int ROWS>
__device__ __forceinline__ void stage_kc(bf16_t* sm, const bf16x8* v, int k0, int K) {
#pragma unroll
  for (int i = 0; i < ROWS / 64; ++i) {
    int c = threadIdx.x + 256 * i;
    *reinterpret_cast<bf16x8*>(sm + (c >> 2) * KC_LD + (c & 3) * 8) = zero_if(v[i], k0 + (c & 3) * 8 >= K);
  }
}
template <int ROWS, int LD>
__device__ __forceinline__ void stage_t(bf16_t* sm, const bf16x8* v, int k0, int K) {
  constexpr int CPR = ROWS / 8;
#pragma unroll
  for (int i = 0; i < ROWS / 64; ++i) {
    int c = threadIdx.x + 256 * i;
    *reinterpret_cast<bf16x8*>(sm + (c / CPR) * LD + (c % CPR) * 8) = zero_if(v[i], k0 + c / CPR >= K);
  }
}
// ---- LDS -> MFMA fragments ----------------------------------------------------------------------
// kc: lane reads 8 consecutive k of its row.
__device__ __forceinline__ bf16x8 frag_kc(const bf16_t* sm, int row, int ks, int lane) {
  return *reinterpret_cast<const bf16x8*>(sm + row * KC_LD + ks + 8 * (lane >> 5));
}
// transposed: two ds_read_b64_tr_b16.  In a 16-lane group, lane s supplies the address of 4 consecutive
// rows at k = kbase + s/4, row chunk s%4; lane j = 4c + e receives rows chunk c element e for k = kbase..+3.
// `rowbase` is the tile row of chunk (lane%4) for this lane's 16-lane group.
template <int LD>
__device__ __forceinline__ bf16x8 frag_t(const bf16_t* sm, int rowbase, int ks, int lane) {
  int kb = ks + 8 * (lane >> 5) + ((lane & 15) >> 2);
  const bf16_t* p = sm + kb * LD + rowbase;
  bf16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4*)(p));
  bf16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4*)(p + 4 * LD));
  bf16x8 r;
#pragma unroll
  for (int e = 0; e < 4; ++e) { r[e] = lo[e]; r[4 + e] = hi[e]; }
  return r;
}

// Fused epilogue on 8 consecutive columns n..n+7 of row m.
__device__ __forceinline__ void epilogue8(const Epilogue& e, int m, int n, float* v) {
  if (e.bias) {
    f32x4 b0 = *reinterpret_cast<const f32x4*>(e.bias + n), b1 = *reinterpret_cast<const f32x4*>(e.bias + n + 4);
#pragma unroll
    for (int x = 0; x < 4; ++x) { v[x] += b0[x]; v[4 + x] += b1[x]; }
  }
  if (e.pre) {
    bf16x8 w;
#pragma unroll
    for (int x = 0; x < 8; ++x) w[x] = (bf16_t)v[x];
    *reinterpret_cast<bf16x8*>(reinterpret_cast<bf16_t*>(e.pre) + (size_t)m * e.ldc + n) = w;
  }
  if (e.act == ACT_RELU) {
#pragma unroll
    for (int x = 0; x < 8; ++x) v[x] = fmaxf(v[x], 0.f);
  } else if (e.act == ACT_GELU) {
#pragma unroll
    for (int x = 0; x < 8; ++x) v[x] = gelu_f(v[x]);
  }
  if (e.dact != ACT_NONE) {
    bf16x8 s = *reinterpret_cast<const bf16x8*>(reinterpret_cast<const bf16_t*>(e.dact_src) + (size_t)m * e.ldd + n);
    if (e.dact == ACT_RELU) {
#pragma unroll
      for (int x = 0; x < 8; ++x) v[x] = (float)s[x] > 0.f ? v[x] : 0.f;
    } else {
#pragma unroll
      for (int x = 0; x < 8; ++x) v[x] *= dgelu_f((float)s[x]);
    }
  }
  if (e.res) {
    bf16x8 r = *reinterpret_cast<const bf16x8*>(reinterpret_cast<const bf16_t*>(e.res) + (size_t)m * e.ldr + n);
#pragma unroll
    for (int x = 0; x < 8; ++x) v[x] += (float)r[x];
  }
  if (e.c_f32) {
    float* cp = reinterpret_cast<float*>(e.C) + (size_t)m * e.ldc + n;
    if (e.accumulate) {
      f32x4 c0 = *reinterpret_cast<const f32x4*>(cp), c1 = *reinterpret_cast<const f32x4*>(cp + 4);
#pragma unroll
      for (int x = 0; x < 4; ++x) { v[x] += c0[x]; v[4 + x] += c1[x]; }
    }
    f32x4 o0 = {v[0], v[1], v[2], v[3]}, o1 = {v[4], v[5], v[6], v[7]};
    *reinterpret_cast<f32x4*>(cp) = o0;
    *reinterpret_cast<f32x4*>(cp + 4) = o1;
  } else {
    bf16_t* cp = reinterpret_cast<bf16_t*>(e.C) + (size_t)m * e.ldc + n;
    if (e.accumulate) {
      bf16x8 c0 = *reinterpret_cast<const bf16x8*>(cp);
#pragma unroll
      for (int x = 0; x < 8; ++x) v[x] += (float)c0[x];
    }
    bf16x8 w;
#pragma unroll
    for (int x = 0; x < 8; ++x) w[x] = (bf16_t)v[x];
    *reinterpret_cast<bf16x8*>(cp) = w;
  }
}

template <bool A_KC, bool B_KC, int BM>
__global__ void __launch_bounds__(256, 2) k_gemm_mfma(Operand A, Operand B, Epilogue e, int M, int N, int K,
                                                      int tiles_m, int tiles_n, int splits, float* ws) {
  constexpr int TM = BM / 64;          // 32-row MFMA tiles per wave along m
  constexpr int TA_LD = BM + 16;
  constexpr int A_ELEMS = BM * KC_LD > BK * TA_LD ? BM * KC_LD : BK * TA_LD;
  __shared__ __attribute__((aligned(16))) bf16_t As[2][A_ELEMS];
  __shared__ __attribute__((aligned(16))) bf16_t Bs[2][B_ELEMS];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  // XCD-aware renumbering, then column-major groups of 8 tile rows
  const int split = blockIdx.x % splits;
  int pid = blockIdx.x / splits;
  {
    const int nb = tiles_m * tiles_n, per = nb / 8;
    if (pid < per * 8) pid = (pid & 7) * per + (pid >> 3);
    const int GROUP = 8;
    int width = GROUP * tiles_n, gid = pid / width;
    int first = gid * GROUP, gs = tiles_m - first < GROUP ? tiles_m - first : GROUP;
    int tm = first + (pid % width) % gs, tn = (pid % width) / gs;
    pid = tm * tiles_n + tn;
  }
  const int m0 = (pid / tiles_n) * BM, n0 = (pid % tiles_n) * BN;
  const int wm = (wave >> 1) * (BM / 2), wn = (wave & 1) * 64;

  f32x16 acc[2][TM];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < TM; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  bf16x8 ra[BM / 64], rb[BN / 64];
  auto fetch = [&](int k0) {
    if (A_KC) fetch_kc<BM>(A, m0, k0, K, ra); else fetch_t<BM>(A, m0, k0, K, ra);
    if (B_KC) fetch_kc<BN>(B, n0, k0, K, rb); else fetch_t<BN>(B, n0, k0, K, rb);
  };
  auto stage = [&](int buf, int k0) {
    if (k0 + BK <= K) k0 = -BK;      // no chunk of this tile can reach K: the masks fold away
    if (A_KC) stage_kc<BM>(As[buf], ra, k0, K); else stage_t<BM, TA_LD>(As[buf], ra, k0, K);
    if (B_KC) stage_kc<BN>(Bs[buf], rb, k0, K); else stage_t<BN, TB_LD>(Bs[buf], rb, k0, K);
  };
  // fragment addressing that does not depend on k
  const int li = lane & 31;
  const int n_row = nmap(li);                                // kc: tile column read by this lane
  const int c4 = lane & 3, half16 = (lane >> 4) & 1;         // transposed: chunk and 16-row half of the group
  // n-side chunk c of half16: MFMA rows 16*half16 + 4c .. +3  ->  columns nmap(16*half16 + 4c) .. +3
  const int n_rowbase_t = nmap(16 * half16 + 4 * c4);
  const int m_rowbase_t = 16 * half16 + 4 * c4;

  const int nt_all = (K + BK - 1) / BK, per = (nt_all + splits - 1) / splits;
  const int t_first = split * per;
  const int nt = nt_all - t_first < per ? (nt_all - t_first > 0 ? nt_all - t_first : 0) : per;
  const int kbase = t_first * BK;
  if (nt > 0) {
    fetch(kbase);
    stage(0, kbase);
  }
  __syncthreads();
  if (nt > 1) fetch(kbase + BK);
  for (int t = 0; t < nt; ++t) {
    const int cur = t & 1;
    if (t + 1 < nt) stage(cur ^ 1, kbase + (t + 1) * BK);
    if (t + 2 < nt) fetch(kbase + (t + 2) * BK);
    const bf16_t* as = As[cur];
    const bf16_t* bs = Bs[cur];
#pragma unroll
    for (int ks = 0; ks < BK; ks += 16) {
      bf16x8 fn[2], fm[TM];
#pragma unroll
      for (int i = 0; i < 2; ++i)
        fn[i] = B_KC ? frag_kc(bs, wn + 32 * i + n_row, ks, lane) : frag_t<TB_LD>(bs, wn + 32 * i + n_rowbase_t, ks, lane);
#pragma unroll
      for (int j = 0; j < TM; ++j)
        fm[j] = A_KC ? frag_kc(as, wm + 32 * j + li, ks, lane) : frag_t<TA_LD>(as, wm + 32 * j + m_rowbase_t, ks, lane);
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < TM; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fn[i], fm[j], acc[i][j], 0, 0, 0);
    }
    __syncthreads();
  }

  // epilogue: lane = row m, accumulator values 8q..8q+7 = columns 16q + 8*(lane/32) .. +7
  const int hf = lane >> 5;
#pragma unroll
  for (int j = 0; j < TM; ++j) {
    const int m = m0 + wm + 32 * j + li;
    if (m >= M) continue;
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int q = 0; q < 2; ++q) {
        const int n = n0 + wn + 32 * i + 16 * q + 8 * hf;
        if (n >= N) continue;
        float v[8];
#pragma unroll
        for (int x = 0; x < 8; ++x) v[x] = acc[i][j][8 * q + x];
        if (splits > 1) {     // raw partial sums; the reduction kernel applies the epilogue
          float* wp = ws + ((size_t)split * M + m) * N + n;
          f32x4 o0 = {v[0], v[1], v[2], v[3]}, o1 = {v[4], v[5], v[6], v[7]};
          *reinterpret_cast<f32x4*>(wp) = o0;
          *reinterpret_cast<f32x4*>(wp + 4) = o1;
        } else {
          epilogue8(e, m, n, v);
        }
      }
  }
}

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
#define LP_GEMM(AK, BK_, BM_) \
  k_gemm_mfma<AK, BK_, BM_><<<grid, 256, 0, c.stream>>>(A, B, e, g.M, g.N, g.K, tm, tn, splits, c.splitk_ws)
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
