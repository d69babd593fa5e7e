// Shared pieces of the register-staged MFMA tile kernel: LDS staging, fragment reads (straight and
// transposing), the fused epilogue, and the kernel template itself, generic over operand loaders.
// A loader turns (tile row, k) into 16-byte global loads; the plain loaders read dense matrices, the
// convolution loaders gather NHWC pixels (implicit GEMM) and report zero padding as invalid chunks.
#pragma once
#include <type_traits>
#include "common.h"
#include "gemm_common.h"

namespace lp {
namespace mfma {

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
__device__ __forceinline__ void stage_kc(bf16_t* sm, const bf16x8* v, int k0, int K, unsigned invalid) {
#pragma unroll
  for (int i = 0; i < ROWS / 64; ++i) {
    int c = threadIdx.x + 256 * i;
    *reinterpret_cast<bf16x8*>(sm + (c >> 2) * KC_LD + (c & 3) * 8) =
        zero_if(v[i], k0 + (c & 3) * 8 >= K || ((invalid >> i) & 1u));
  }
}
template <int ROWS, int LD>
__device__ __forceinline__ void stage_t(bf16_t* sm, const bf16x8* v, int k0, int K, unsigned invalid) {
  constexpr int CPR = ROWS / 8;
#pragma unroll
  for (int i = 0; i < ROWS / 64; ++i) {
    int c = threadIdx.x + 256 * i;
    *reinterpret_cast<bf16x8*>(sm + (c / CPR) * LD + (c % CPR) * 8) =
        zero_if(v[i], k0 + c / CPR >= K || ((invalid >> i) & 1u));
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

// Fused epilogue on 8 consecutive columns n..n+7 of row m.  STORE_BF16 = false leaves the final values in v
// (and the pre-activation, if asked for, in *pre_out) instead of storing a compute-dtype result: for the
// caller that turns a sub-tile around in LDS so as to store whole lines.
template <bool STORE_BF16 = true>
__device__ __forceinline__ void epilogue8(const Epilogue& e, int m, int n, float* v, bf16x8* pre_out = nullptr) {
  if (e.bias) {
    f32x4 b0 = *reinterpret_cast<const f32x4*>(e.bias + n), b1 = *reinterpret_cast<const f32x4*>(e.bias + n + 4);
#pragma unroll
    for (int x = 0; x < 4; ++x) { v[x] += b0[x]; v[4 + x] += b1[x]; }
  }
  if (e.pre) {
    bf16x8 w;
#pragma unroll
    for (int x = 0; x < 8; ++x) w[x] = (bf16_t)v[x];
    if (STORE_BF16) *reinterpret_cast<bf16x8*>(reinterpret_cast<bf16_t*>(e.pre) + (size_t)m * e.ldc + n) = w;
    else *pre_out = w;
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
    if (STORE_BF16) {
      bf16x8 w;
#pragma unroll
      for (int x = 0; x < 8; ++x) w[x] = (bf16_t)v[x];
      *reinterpret_cast<bf16x8*>(cp) = w;
    }
  }
}


// ---- dense-matrix loaders ------------------------------------------------------------------------
// kc tile [ROWS][32]: ROWS*4 chunks of 8 k; thread takes chunks tid + 256*i.
// transposed tile, memory [32 k][ROWS]: 32*ROWS/8 chunks of 8 rows; thread takes chunks tid + 256*i.
template <bool KC_>
struct PlainLoader {
  static constexpr bool KC = KC_;
  Operand o;
  template <int ROWS> __device__ __forceinline__ void init(int) {}
  template <int ROWS>
  __device__ __forceinline__ unsigned fetch(int r0, int k0, int K, bf16x8* v) const {
    if (KC) {
#pragma unroll
      for (int i = 0; i < ROWS / 64; ++i) {
        int c = threadIdx.x + 256 * i;
        int row = r0 + (c >> 2), k = k0 + (c & 3) * 8;
        row = row < o.rows ? row : o.rows - 1;
        v[i] = *reinterpret_cast<const bf16x8*>(o.p + (size_t)row * o.ld + (k < K ? k : 0));
      }
    } else {
      constexpr int CPR = ROWS / 8;   // chunks per k-row
#pragma unroll
      for (int i = 0; i < ROWS / 64; ++i) {
        int c = threadIdx.x + 256 * i;
        int k = k0 + c / CPR, row = r0 + (c % CPR) * 8;
        row = row + 8 <= o.rows ? row : o.rows - 8;
        v[i] = *reinterpret_cast<const bf16x8*>(o.p + (size_t)(k < K ? k : 0) * o.ld + row);
      }
    }
    return 0u;
  }
};

// BN_ = 128: the four waves form a 2 x 2 grid, each BM/2 rows x 64 columns.  BN_ = 64 (outputs at most 64 columns
// wide: the 64-channel convolutions, whose tiles would otherwise be half padding): the waves are stacked, each BM/4
// rows x 64 columns.
//
// STATS (the convolution in front of a batch normalisation; splits == 1, M a multiple of BM and N of BN_, so every
// sub-tile takes the whole-line path): each block also leaves, per output column, the sums the normalisation needs over
// the rows of the tile, taken from the rounded values it stores: p = the tile's first row, s0 = sum (z - p),
// s1 = sum (z - p)^2, in ws as [3][M / BM][N] (s0, s1, p).  The statistics pass over z is then not needed.
template <class LA, class LB, int BM, int BN_ = 128, bool STATS = false>
__global__ void __launch_bounds__(256, BM == 64 ? 4 : (BM == 128 ? 3 : 2)) k_mfma_tiles(LA A, LB B, Epilogue e, int M, int N, int K, int tiles_m,
                                                       int tiles_n, int splits, float* ws) {
  constexpr bool A_KC = LA::KC, B_KC = LB::KC;
  constexpr int WROWS = BN_ == 128 ? BM / 2 : BM / 4;     // rows of a wave's sub-tile
  constexpr int TM = WROWS / 32;        // 32-row MFMA tiles per wave along m
  constexpr int TA_LD = BM + 16;
  constexpr int TBL = BN_ + 16;         // [k][row] tile of the n-side operand: padded rows
  constexpr int A_ELEMS = BM * KC_LD > BK * TA_LD ? BM * KC_LD : BK * TA_LD;
  constexpr int BE = BN_ * KC_LD > BK * TBL ? BN_ * KC_LD : BK * TBL;
  // one block of LDS: operand buffers A0 A1 B0 B1; the epilogue reuses it (>= 32 KB) as its patches
  constexpr int SM_ELEMS = 2 * A_ELEMS + 2 * BE > 4 * 4096 ? 2 * A_ELEMS + 2 * BE : 4 * 4096;
  __shared__ __attribute__((aligned(16))) bf16_t Sm[SM_ELEMS];
  bf16_t* const As[2] = {Sm, Sm + A_ELEMS};
  bf16_t* const Bs[2] = {Sm + 2 * A_ELEMS, Sm + 2 * A_ELEMS + BE};
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
  const int m0 = (pid / tiles_n) * BM, n0 = (pid % tiles_n) * BN_;
  const int wm = (BN_ == 128 ? (wave >> 1) : wave) * WROWS, wn = BN_ == 128 ? (wave & 1) * 64 : 0;

  f32x16 acc[2][TM];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < TM; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  // Global -> register prefetch NSET k-tiles deep: a k-tile's loads are issued NSET k-tiles before its
  // registers are written to LDS, so their latency is covered by the MFMAs of those k-tiles (and of the
  // other block on the CU).  The barrier waits for LDS traffic only: a __syncthreads would also wait for
  // every outstanding global load and put that latency back on the critical path of each k-tile.
  constexpr int NSET = 2;
  bf16x8 ra[NSET][BM / 64], rb[NSET][BN_ / 64];
  unsigned inva[NSET], invb[NSET];       // chunks the loader declared invalid (implicit zero padding)
  A.template init<BM>(m0);
  B.template init<BN_>(n0);
  auto fetch = [&](int s, int k0) {
    inva[s] = A.template fetch<BM>(m0, k0, K, ra[s]);
    invb[s] = B.template fetch<BN_>(n0, k0, K, rb[s]);
  };
  auto stage = [&](int buf, int s, int k0) {
    if (k0 + BK <= K) k0 = -BK;      // no chunk of this tile can reach K: the masks fold away
    if (A_KC) stage_kc<BM>(As[buf], ra[s], k0, K, inva[s]); else stage_t<BM, TA_LD>(As[buf], ra[s], k0, K, inva[s]);
    if (B_KC) stage_kc<BN_>(Bs[buf], rb[s], k0, K, invb[s]); else stage_t<BN_, TBL>(Bs[buf], rb[s], k0, K, invb[s]);
  };
  auto lds_barrier = [] { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); };
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
#pragma unroll
  for (int s = 0; s < NSET; ++s)
    if (s < nt) fetch(s, kbase + s * BK);
  if (nt > 0) stage(0, 0, kbase);
  lds_barrier();
  // k-tile t is in LDS buffer t & 1; register set (t + j) % NSET holds k-tile t + j, j = 1 .. NSET-1, and
  // set t % NSET is free.  The loop is unrolled by NSET so that the sets are named at compile time.
  // STEADY: k-tiles t + 1 and t + NSET exist, so nothing in the body is conditional and the compiler counts
  // the outstanding loads exactly (a conditional fetch makes it wait for all of them at the next stage).
  auto ktile = [&](int t, auto set, auto steady) {
    constexpr int U = decltype(set)::value;
    constexpr bool STEADY = decltype(steady)::value;
    const int cur = t & 1;
    if (STEADY || t + NSET < nt) fetch(U, kbase + (t + NSET) * BK);
    const bf16_t* as = As[cur];
    const bf16_t* bs = Bs[cur];
#pragma unroll
    for (int ks = 0; ks < BK; ks += 16) {
      bf16x8 fn[2], fm[TM];
#pragma unroll
      for (int i = 0; i < 2; ++i)
        fn[i] = B_KC ? frag_kc(bs, wn + 32 * i + n_row, ks, lane) : frag_t<TBL>(bs, wn + 32 * i + n_rowbase_t, ks, lane);
#pragma unroll
      for (int j = 0; j < TM; ++j)
        fm[j] = A_KC ? frag_kc(as, wm + 32 * j + li, ks, lane) : frag_t<TA_LD>(as, wm + 32 * j + m_rowbase_t, ks, lane);
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < TM; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fn[i], fm[j], acc[i][j], 0, 0, 0);
    }
    if (STEADY || t + 1 < nt) stage(cur ^ 1, (U + 1) % NSET, kbase + (t + 1) * BK);
    lds_barrier();
  };
  int t0 = 0;
  for (; t0 + 2 * NSET <= nt; t0 += NSET) {
    ktile(t0, std::integral_constant<int, 0>{}, std::true_type{});
    ktile(t0 + 1, std::integral_constant<int, 1>{}, std::true_type{});
    if (NSET == 3) ktile(t0 + 2, std::integral_constant<int, NSET == 3 ? 2 : 0>{}, std::true_type{});
  }
  for (; t0 < nt; t0 += NSET) {
    ktile(t0, std::integral_constant<int, 0>{}, std::false_type{});
    if (t0 + 1 < nt) ktile(t0 + 1, std::integral_constant<int, 1>{}, std::false_type{});
    if (NSET == 3 && t0 + 2 < nt) ktile(t0 + 2, std::integral_constant<int, NSET == 3 ? 2 : 0>{}, std::false_type{});
  }

  // epilogue: lane = row m, accumulator values 8q..8q+7 = columns 16q + 8*(lane/32) .. +7
  const int hf = lane >> 5;
  // A compute-dtype result of a sub-tile inside the matrix leaves through LDS: in the accumulators a row's
  // 128 bytes sit in two lanes, so a store instruction would touch 32 lines and write a quarter of each.
  // Each wave turns 32 rows x 128 bytes around in a 4 KB patch of the (now idle) operand buffers (16-byte
  // chunk c of row r in slot c ^ ((r >> 1) & 7): conflict-free both ways); lane L then holds chunk L % 8 of
  // row L / 8 (+ 8 per instruction) and an instruction stores 8 whole lines.  The pre-activation, if asked
  // for, goes the same way through a second patch.
  if (splits == 1 && !e.c_f32 && m0 + wm + WROWS <= M && n0 + wn + 64 <= N) {
    char* xs = reinterpret_cast<char*>(Sm) + wave * 8192;
    const int rr = lane >> 3, rc = lane & 7;
    float st_s0 = 0.f, st_s1 = 0.f, st_p = 0.f;
    bf16_t* cbase = reinterpret_cast<bf16_t*>(e.C) + (size_t)(m0 + wm + rr) * e.ldc + n0 + wn + 8 * rc;
    bf16_t* pbase = reinterpret_cast<bf16_t*>(e.pre) + (size_t)(m0 + wm + rr) * e.ldc + n0 + wn + 8 * rc;
#pragma unroll
    for (int j = 0; j < TM; ++j) {
      const int m = m0 + wm + 32 * j + li;
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int q = 0; q < 2; ++q) {
          const int n = n0 + wn + 32 * i + 16 * q + 8 * hf;
          float v[8];
#pragma unroll
          for (int x = 0; x < 8; ++x) v[x] = acc[i][j][8 * q + x];
          bf16x8 pw;
          epilogue8<false>(e, m, n, v, &pw);
          bf16x8 w;
#pragma unroll
          for (int x = 0; x < 8; ++x) w[x] = (bf16_t)v[x];
          const int slot = ((4 * i + 2 * q + hf) ^ ((li >> 1) & 7)) << 4;
          *reinterpret_cast<bf16x8*>(xs + li * 128 + slot) = w;
          if (e.pre) *reinterpret_cast<bf16x8*>(xs + 4096 + li * 128 + slot) = pw;
        }
#pragma unroll
      for (int I = 0; I < 4; ++I) {
        const int r = 8 * I + rr, slot = (rc ^ ((r >> 1) & 7)) << 4;
        const size_t off = (size_t)(32 * j + 8 * I) * e.ldc;
        *reinterpret_cast<bf16x8*>(cbase + off) = *reinterpret_cast<const bf16x8*>(xs + r * 128 + slot);
        if (e.pre) *reinterpret_cast<bf16x8*>(pbase + off) = *reinterpret_cast<const bf16x8*>(xs + 4096 + r * 128 + slot);
      }
      if constexpr (STATS) {       // lane = column: element lane % 8 of chunk lane / 8 of every row of the patch
        const int sc = lane >> 3, se = (lane & 7) * 2;
#pragma unroll
        for (int r = 0; r < 32; ++r) {
          const float v = (float)*reinterpret_cast<const bf16_t*>(xs + r * 128 + ((sc ^ ((r >> 1) & 7)) << 4) + se);
          if (j == 0 && r == 0) st_p = v;
          const float t = v - st_p;
          st_s0 += t;
          st_s1 += t * t;
        }
      }
    }
    if constexpr (STATS) {
      // one set of sums per tile: the waves that share columns (all four, or waves w and w + 2) leave theirs in their
      // own patch, and the first of them shifts the others to its pivot (d = p_w - p: s0 += s0_w + n d,
      // s1 += s1_w + 2 d s0_w + n d^2) in wave order.  Every wave of the block is here (whole tiles only).
      float* mine = reinterpret_cast<float*>(xs);
      mine[lane] = st_s0; mine[64 + lane] = st_s1; mine[128 + lane] = st_p;
      __syncthreads();
      constexpr int SHARE = BN_ == 128 ? 2 : 4, STEP = BN_ == 128 ? 2 : 1;
      if (wave < STEP) {
        const float n = (float)WROWS;
#pragma unroll
        for (int u = 1; u < SHARE; ++u) {
          const float* o = reinterpret_cast<const float*>(reinterpret_cast<const char*>(Sm) + (wave + u * STEP) * 8192);
          const float o0 = o[lane], o1 = o[64 + lane], d = o[128 + lane] - st_p;
          st_s0 += o0 + n * d;
          st_s1 += o1 + 2.f * d * o0 + n * d * d;
        }
        const size_t nslab = (size_t)M / BM, slab = (size_t)m0 / BM;
        float* sp = ws + slab * N + n0 + wn + lane;
        sp[0] = st_s0;
        sp[nslab * N] = st_s1;
        sp[2 * nslab * N] = st_p;
      }
    }
    return;
  }
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


}  // namespace mfma
}  // namespace lp
