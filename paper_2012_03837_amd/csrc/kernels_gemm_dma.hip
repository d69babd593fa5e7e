// bf16 GEMM for large, aligned shapes: operand tiles stream global -> LDS with the gfx950 16-byte
// direct-to-LDS load (global_load_lds_dwordx4: no registers, no VALU), through a ring of NSTAGE LDS
// stages, so several k-tiles of HBM / L2 latency are in flight behind the MFMA phase.
//
// Block tile 256(m) x BN(n) x 32(k); 2 x WNW wavefronts, each owning 128 x 32*TN (4 x TN tiles of
// v_mfma_f32_32x32x16_bf16).  Three shapes:
//   256 x 256, 8 waves of 128 x 64  (WNW 4, TN 2): 4 stages (128 KB LDS), one block per CU, 2 waves per SIMD,
//                hand-pipelined main loop (PIPE)
//   256 x 256, 4 waves of 128 x 128 (WNW 2, TN 4): 5 stages (all 160 KB), one block per CU, 1 wave per SIMD
//                with all 512 registers, hand-pipelined; a third less LDS read traffic per flop (8 fragment
//                reads per 16 MFMAs); fastest on resident operands, slower on cold ones: taken only when forced
//   256 x 128, 4 waves of 128 x 64  (WNW 2, TN 2): 3 stages (72 KB), two blocks per CU, plain main loop.
//
// A direct-to-LDS load writes lane l's 16 bytes at (wave-uniform base) + 16*l, so a wave fills 1 KB of
// contiguous LDS; tiles are therefore unpadded and bank conflicts are avoided by an XOR swizzle that the
// *global* address of each lane undoes:
//   kc tile   [row][4 chunks of 8 k]   : chunk c of row r sits in slot c ^ ((r>>2)&3)
//   k-major   [k][32.. chunks of 8 rows]: chunk j of k-row k sits in slot j ^ ((k&3)<<2)   (read with
//                                         ds_read_b64_tr_b16, as in the register-staged kernel)
// The grid is persistent (one block per resident slot): a block computes several whole tiles, and the last
// partial wave of tiles is cut along k so that every CU gets the same number of k-steps (see SkPlan).
// Plain main loop, one barrier per k-tile: wait until this thread's loads of tile t have landed (s_waitcnt
// vmcnt leaves the younger tiles in flight), barrier, issue the loads of tile t+NSTAGE-1 into the stage that
// was read during tile t-1, then the MFMAs of tile t; the next item's first loads are issued before the
// finished item is written.  Hand-pipelined main loop (PIPE): the k-tiles of all of a block's items form
// one stream through the ring of stages, so the loader stays NSTAGE-1 k-tiles ahead across item boundaries
// and the next item's first k-tiles are in flight while a finished item is written; see the comment in the kernel.
// Requires K % 32 == 0 (no zero fill on this path).
#include <stdio.h>
#include <stdlib.h>
#include <type_traits>
#include "common.h"
#include "gemm_common.h"

namespace lp {

namespace {

constexpr int BM = 256, BK = 32;
// The 8-wave 256 x 256 shape keeps 4 KB of LDS per wave beside its stages to turn a finished plain bf16
// sub-tile around, so that each store instruction writes whole 128-byte lines (see store_subtile).
constexpr int XPOSE_BYTES_PER_WAVE = 32 * 128;
constexpr bool xpose_shape(int WNW, int TN, bool PIPE) { return PIPE && WNW == 4 && TN == 2; }
typedef __attribute__((address_space(3))) bf16x4 lds_bf16x4;
typedef __attribute__((address_space(3))) void lds_void;
typedef __attribute__((address_space(1))) const void glb_void;

struct Operand { const bf16_t* p; int64_t ld; int rows; };

__device__ __forceinline__ int nmap(int i) {
  int g = i >> 3, h = (i >> 2) & 1, j = i & 3;
  return 16 * (g >> 1) + 8 * h + 4 * (g & 1) + j;
}
// Wait until at most VM of this wave's vector-memory loads are outstanding, then the workgroup barrier.
// One asm statement with a memory clobber: the compiler neither moves LDS accesses across it nor turns
// it into a full fence (a fence would wait for *all* loads, i.e. drain the pipeline every k-tile).
template <int VM>
__device__ __forceinline__ void wait_loads_and_barrier() {
  asm volatile("s_waitcnt vmcnt(%0)\n\ts_barrier" ::"n"(VM) : "memory");
}

// Same fused epilogue as the register-staged kernel (8 consecutive columns of one row).
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

// Per-lane global pointers of the direct-to-LDS loads of one operand: NI loads per thread per k-tile.
// ROWS = tile rows of this operand.  The pointers are for k-tile 0; a k-tile step adds `kstep` elements.
template <bool KC, int ROWS, int NI, int KT = 32>
struct DmaPlan {
  const bf16_t* g[NI];
  int lds_off[NI];      // byte offset of the wave's 1 KB destination inside the operand's stage region
  int64_t kstep;
  __device__ __forceinline__ void init(const Operand& o, int r0, int wave, int lane, int kbase) {
#pragma unroll
    for (int i = 0; i < NI; ++i) {
      int q = wave * NI + i;              // which 1 KB of the tile
      lds_off[i] = q * 1024;
      if (KC && KT == 64) {
        // 64-deep k-tiles: a tile row is one whole 128-byte line; an instruction covers 8 rows, lane l carries
        // 16-byte chunk c of row l / 8 into slot c ^ ((row >> 1) & 7)
        int row = q * 8 + (lane >> 3), slot = lane & 7;
        int c = slot ^ ((row >> 1) & 7);
        int rg = r0 + row;
        rg = rg < o.rows ? rg : o.rows - 1;
        g[i] = o.p + (size_t)rg * o.ld + kbase + 8 * c;
      } else if (KC) {
        int row = q * 16 + (lane >> 2), slot = lane & 3;
        int c = slot ^ ((row >> 2) & 3);
        int rg = r0 + row;
        rg = rg < o.rows ? rg : o.rows - 1;
        g[i] = o.p + (size_t)rg * o.ld + kbase + 8 * c;
      } else {
        constexpr int CPR = ROWS / 8;     // 16-byte chunks per k-row
        constexpr int KPI = 64 / CPR;     // k-rows per 1 KB
        int k = q * KPI + lane / CPR, slot = lane % CPR;
        int j = slot ^ ((k & 3) << 2);
        int rg = r0 + 8 * j;
        rg = rg + 8 <= o.rows ? rg : o.rows - 8;
        g[i] = o.p + (size_t)(kbase + k) * o.ld + rg;
      }
    }
    kstep = KC ? (int64_t)KT : (int64_t)KT * o.ld;
  }
  __device__ __forceinline__ void issue(char* stage_base, int tile) const {
#pragma unroll
    for (int i = 0; i < NI; ++i) {
      const bf16_t* src = g[i] + (int64_t)tile * kstep;
      __builtin_amdgcn_global_load_lds((glb_void*)src, (lds_void*)(stage_base + lds_off[i]), 16, 0, 0);
    }
  }
};

// fragment reads
__device__ __forceinline__ bf16x8 frag_kc(const char* sm, int row, int chunk) {
  return *reinterpret_cast<const bf16x8*>(sm + row * 64 + 16 * (chunk ^ ((row >> 2) & 3)));
}
// 64-deep kc tile: 128-byte rows, chunk c (0..7) of row r in slot c ^ ((r >> 1) & 7)
__device__ __forceinline__ bf16x8 frag_kc64(const char* sm, int row, int chunk) {
  return *reinterpret_cast<const bf16x8*>(sm + row * 128 + 16 * (chunk ^ ((row >> 1) & 7)));
}
template <int ROWS>
__device__ __forceinline__ bf16x8 frag_t(const char* sm, int rowbase, int k) {
  const char* p = sm + k * (ROWS * 2) + 16 * ((rowbase >> 3) ^ ((k & 3) << 2)) + (rowbase & 7) * 2;
  bf16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4*)(p));
  bf16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4*)(p + 4 * ROWS * 2));
  bf16x8 r;
#pragma unroll
  for (int e = 0; e < 4; ++e) { r[e] = lo[e]; r[4 + e] = hi[e]; }
  return r;
}

// Work distribution of one launch.  The grid is persistent: G blocks, as many as are resident at once.
//  - Tiles [0, full*G) are computed whole, `full` per block ("waves").  Block b sits on XCD b % 8 (the
//    dispatcher deals blocks round-robin), so XCD x is given the contiguous tile range
//    [x*full*G/8, (x+1)*full*G/8) and walks it G/8 tiles at a time: concurrent blocks of an XCD share
//    operand rows/columns in its L2, and so do successive waves.
//  - The remaining tail_tiles (< G unless upb == kt) are cut along k: the tail is tail_tiles*kt k-steps
//    in tile-major order, block v takes k-steps [v*upb, (v+1)*upb).  A block's piece of a tile that is
//    not the whole tile is written as raw fp32 partial sums to a slab of the workspace (slab 2v when the
//    piece starts inside the tile, 2v+1 when it starts at the tile's first k-step), and k_sk_fixup adds
//    the slabs of each tile in block order and applies the epilogue.  upb == kt degenerates to one whole
//    tile per block and no partial sums.  No block ever waits for another.
//  - Panel mode (sib = tiles_n > 1, full = 0; for outputs only a few tiles wide over a long reduction: the
//    input gradient and the weight gradient of a vocabulary head): the unit of the cut is a panel, the
//    tiles_n tiles of one tile row.  The reduction of all panels, tiles_m*kt k-steps in panel-major order,
//    is cut into equal ranges; a range goes to a group of tiles_n neighbouring blocks of one XCD, block s
//    of the group computing tile column s.  The blocks of a group walk the same k-steps of the same
//    A rows in lockstep, so the big operand is fetched into that XCD's L2 once instead of tiles_n times.
//    Slab numbering and the fix-up are as above with v = group*tiles_n + s; tiles are numbered
//    tile-column-fastest in this mode.
struct SkPlan {
  int tiles_m, tiles_n, kt;
  int full, tail_tiles, upb, G;
  int sib;      // 0: ordinary; otherwise tiles_n (panel mode)
  int ngrp;     // 0: one problem; otherwise the number of problems of a grouped launch (see GroupTable)
};

// Grouped launch: up to kMaxGroup independent products with the same reduction length, operand layouts and a
// plain fp32 epilogue (the weight gradients of one layer: dW_i = dY_i^T X_i over the same rows) run as ONE
// persistent launch.  Their output tiles are numbered one problem after the other (row-major inside a
// problem, first[i] = number of the i-th problem's first tile), and that one sequence of tiles is spread over
// the grid exactly like a single problem's: whole tiles first, the last partial wave cut along k.  Each
// launch by itself has too few tiles for 256 CUs (9 to 36 tiles of 256 x 256 for a width of 768); together
// they fill the chip with pieces a third to a half as many.
constexpr int kMaxGroup = 16;
struct GroupTable {
  Operand A[kMaxGroup], B[kMaxGroup];
  Epilogue e[kMaxGroup];          // every problem has its own fused epilogue and output
  int tiles_n[kMaxGroup];
  int first[kMaxGroup + 1];
};

__device__ __forceinline__ void tile_coords(int q, int tiles_m, int tiles_n, int& tm, int& tn) {
  const int GROUP = 8;   // column-major groups of 8 tile rows
  int width = GROUP * tiles_n, gid = q / width;
  int first = gid * GROUP, gs = tiles_m - first < GROUP ? tiles_m - first : GROUP;
  tm = first + (q % width) % gs;
  tn = (q % width) / gs;
}

__device__ __forceinline__ void plan_tile_coords(const SkPlan& p, int q, int& tm, int& tn) {
  if (p.sib) { tm = q / p.tiles_n; tn = q - tm * p.tiles_n; }
  else tile_coords(q, p.tiles_m, p.tiles_n, tm, tn);
}
// Grouped launch: problem of tile q and the tile's coordinates inside it.
__device__ __forceinline__ int group_tile_coords(const GroupTable& gt, int ngrp, int q, int& tm, int& tn) {
  int g = 0;
#pragma unroll
  for (int i = 1; i < kMaxGroup; ++i)
    if (i < ngrp && q >= gt.first[i]) g = i;
  const int local = q - gt.first[g];
  tm = local / gt.tiles_n[g];
  tn = local - tm * gt.tiles_n[g];
  return g;
}

// Epilogue of one wave's 128 x 64 sub-tile: lane (li, hf) holds, for row m = ..+li of m-tile j, the
// columns 32*i + 16*q + 8*hf .. +7 of n-tile i in acc[i][j][8q .. 8q+7].
template <int TN>
__device__ __forceinline__ void store_subtile(const Epilogue& e, const f32x16 (&acc)[TN][4], int m_base, int n_base,
                                              int li, int hf, int M, int N, char* xs) {
  // Nothing fused and the sub-tile inside the matrix (both wave-uniform): four row pointers, then
  // convert-and-store with immediate offsets.  The general path below costs several microseconds of
  // branches and address arithmetic per tile, during which the block's MFMA pipes idle.
  const bool plain = !e.bias && !e.pre && e.act == ACT_NONE && e.dact == ACT_NONE && !e.res && !e.accumulate;
  if (plain && m_base + 128 <= M && n_base + 32 * TN <= N) {
    if (e.c_f32) {
      float* base = reinterpret_cast<float*>(e.C) + (size_t)(m_base + li) * e.ldc + n_base + 8 * hf;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        float* row = base + (size_t)(32 * j) * e.ldc;
#pragma unroll
        for (int i = 0; i < TN; ++i)
#pragma unroll
          for (int q = 0; q < 2; ++q) {
            f32x4 o0 = {acc[i][j][8 * q], acc[i][j][8 * q + 1], acc[i][j][8 * q + 2], acc[i][j][8 * q + 3]};
            f32x4 o1 = {acc[i][j][8 * q + 4], acc[i][j][8 * q + 5], acc[i][j][8 * q + 6], acc[i][j][8 * q + 7]};
            *reinterpret_cast<f32x4*>(row + 32 * i + 16 * q) = o0;
            *reinterpret_cast<f32x4*>(row + 32 * i + 16 * q + 4) = o1;
          }
      }
    } else if (TN == 2 && xs) {
      // In the accumulators a row's 128 bytes sit in two lanes (32-byte pieces per store instruction: 32 lines
      // touched, a quarter of each).  Through the wave's LDS patch, 32 rows x 128 bytes at a time (16-byte
      // chunk c of row r in slot c ^ ((r >> 1) & 7): conflict-free both ways), lane L then holds chunk L % 8
      // of row L / 8 (+ 8 per instruction), so an instruction writes 8 whole lines.  The stores are
      // non-temporal: whole lines need no combining in L2, and the operands are not evicted by the output.
      const int lane = 32 * hf + li;
      const int rr = lane >> 3, rc = lane & 7;
      bf16_t* base = reinterpret_cast<bf16_t*>(e.C) + (size_t)(m_base + rr) * e.ldc + n_base + 8 * rc;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
#pragma unroll
        for (int i = 0; i < TN; ++i)
#pragma unroll
          for (int q = 0; q < 2; ++q) {
            bf16x8 w;
#pragma unroll
            for (int x = 0; x < 8; ++x) w[x] = (bf16_t)acc[i][j][8 * q + x];
            const int c = 4 * i + 2 * q + hf;
            *reinterpret_cast<bf16x8*>(xs + li * 128 + ((c ^ ((li >> 1) & 7)) << 4)) = w;
          }
#pragma unroll
        for (int I = 0; I < 4; ++I) {
          const int r = 8 * I + rr;
          bf16x8 w = *reinterpret_cast<const bf16x8*>(xs + r * 128 + ((rc ^ ((r >> 1) & 7)) << 4));
          __builtin_nontemporal_store(w, reinterpret_cast<bf16x8*>(base + (size_t)(32 * j + 8 * I) * e.ldc));
        }
      }
    } else {
      bf16_t* base = reinterpret_cast<bf16_t*>(e.C) + (size_t)(m_base + li) * e.ldc + n_base + 8 * hf;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        bf16_t* row = base + (size_t)(32 * j) * e.ldc;
#pragma unroll
        for (int i = 0; i < TN; ++i)
#pragma unroll
          for (int q = 0; q < 2; ++q) {
            bf16x8 w;
#pragma unroll
            for (int x = 0; x < 8; ++x) w[x] = (bf16_t)acc[i][j][8 * q + x];
            *reinterpret_cast<bf16x8*>(row + 32 * i + 16 * q) = w;
          }
      }
    }
    return;
  }
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int m = m_base + 32 * j + li;
    if (m >= M) continue;
#pragma unroll
    for (int i = 0; i < TN; ++i)
#pragma unroll
      for (int q = 0; q < 2; ++q) {
        const int n = n_base + 32 * i + 16 * q + 8 * hf;
        if (n >= N) continue;
        float v[8];
#pragma unroll
        for (int x = 0; x < 8; ++x) v[x] = acc[i][j][8 * q + x];
        epilogue8(e, m, n, v);
      }
  }
}

// Partial-sum slab of one block tile, in accumulator order: 16 bytes per lane, 1 KB per wave store.
template <int TN>
__device__ __forceinline__ size_t slab_index(int wave, int ij, int c, int lane) {
  return ((((size_t)wave * (4 * TN) + ij) * 4 + c) * 64 + lane) * 4;
}

// Scheduling hint for one k-substep: NMF MFMAs, with the NDS LDS reads of the next substep spread over the
// first three quarters of them (the last reads then have time to land before they are waited for) and
// NVM direct-to-LDS loads spread over all of them.  A wave issues in order: a burst of loads that fills
// the memory pipeline's queue would hold back the MFMAs behind it.
template <int NMF, int NDS, int NVM>
__device__ __forceinline__ void interleave_hint() {
  constexpr int RD = NMF * 3 / 4;      // MFMAs over which the LDS reads are spread
#pragma unroll
  for (int g = 0; g < NMF; ++g) {
    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                          // one MFMA
    const int n = g < RD ? (NDS * (g + 1)) / RD - (NDS * g) / RD : 0;           // then this many LDS reads
    if (n == 1) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
    else if (n == 2) __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
    else if (n == 3) __builtin_amdgcn_sched_group_barrier(0x100, 3, 0);
    const int m = (NVM * (g + 1)) / NMF - (NVM * g) / NMF;                      // and this many global loads
    if (m == 1) __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
  }
}

// The same for a substep that also issues direct-to-LDS loads.  Those write LDS and the fragment reads
// read it, so the scheduler keeps the two kinds in program order (reads first): the reads are spread over
// the first half of the MFMAs and the loads over the second half.  Asking for an order that contradicts
// the dependencies makes the scheduler drop the whole hint and emit both as one burst behind the first
// MFMA, which stalls the MFMA pipe of both waves of a SIMD at once.
template <int NMF, int NDS, int NVM>
__device__ __forceinline__ void interleave_hint_loads() {
  constexpr int RD = NMF / 2;
#pragma unroll
  for (int g = 0; g < NMF; ++g) {
    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                          // one MFMA
    const int n = g < RD ? (NDS * (g + 1)) / RD - (NDS * g) / RD : 0;
    if (n == 1) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
    else if (n == 2) __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
    else if (n == 3) __builtin_amdgcn_sched_group_barrier(0x100, 3, 0);
    else if (n == 4) __builtin_amdgcn_sched_group_barrier(0x100, 4, 0);
    const int m = g >= RD ? (NVM * (g - RD + 1)) / (NMF - RD) - (NVM * (g - RD)) / (NMF - RD) : 0;
    if (m == 1) __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
    else if (m == 2) __builtin_amdgcn_sched_group_barrier(0x020, 2, 0);
  }
}

template <bool A_KC, bool B_KC, int WNW, int TN, int NSTAGE, bool PIPE, int KT = 32>
__global__ void __launch_bounds__(128 * WNW, (WNW * TN == 4) ? 2 : (WNW == 4 ? 2 : 1))
k_gemm_dma(Operand A, Operand B, Epilogue e, int M, int N, SkPlan p, float* ws, GroupTable gt) {
  constexpr int BN = 32 * TN * WNW, NWAVES = 2 * WNW;
  constexpr int A_BYTES = BM * KT * 2, B_BYTES = BN * KT * 2, STAGE_BYTES = A_BYTES + B_BYTES;
  constexpr int AI = (A_BYTES / 1024) / NWAVES, BI = (B_BYTES / 1024) / NWAVES, LPT = AI + BI;
  extern __shared__ __attribute__((aligned(1024))) char smem[];
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int wm = (wave / WNW) * 128, wn = (wave % WNW) * (32 * TN);
  const int li = lane & 31, hf = lane >> 5;
  const int n_row = nmap(li);
  const int c4 = lane & 3, half16 = (lane >> 4) & 1;
  const int n_rowbase_t = nmap(16 * half16 + 4 * c4);
  const int m_rowbase_t = 16 * half16 + 4 * c4;
  const int kq = (lane & 15) >> 2;

  // this block's work: `full` whole tiles, then k-steps [u, ue) of the tail
  const int Gx = p.G >> 3, xcd = blockIdx.x & 7, slot_in_xcd = blockIdx.x >> 3;
  int v = xcd * Gx + slot_in_xcd;     // index of this block's range of the cut reduction (and of its slabs)
  long tail_steps = (long)p.tail_tiles * p.kt;
  long u, ue;
  int sibling = 0;
  if (p.sib) {                        // panel mode: groups of p.sib neighbouring blocks of this XCD
    const int per_xcd = Gx / p.sib, grp = slot_in_xcd / p.sib;
    sibling = slot_in_xcd - grp * p.sib;
    const int vg = xcd * per_xcd + grp;
    tail_steps = (long)p.tiles_m * p.kt;
    u = grp < per_xcd ? (long)vg * p.upb : tail_steps;       // blocks left over in an XCD have no work
    v = vg * p.sib + sibling;
  } else {
    u = (long)v * p.upb;
  }
  ue = u + p.upb;
  if (ue > tail_steps) ue = tail_steps;
  // The block's items in order: `full` whole tiles, then the pieces of its range of the cut reduction.
  // The sequence depends only on the block and the plan, so the loader and the MFMA side of the pipelined
  // kernel each walk it with an iterator of their own.
  struct ItemIter { int w, tr, k0, left; int q, ks, ke; };     // item: tile q, k-steps [ks, ke)
  auto first_item = [&]() -> ItemIter {     // before the block's first item
    ItemIter it;
    it.w = 0;
    it.tr = (int)(u / p.kt);                // tail tile (or panel) and k-step at which the block's range starts
    it.k0 = (int)(u - (long)it.tr * p.kt);
    it.left = ue > u ? (int)(ue - u) : 0;
    it.q = it.ks = it.ke = 0;
    return it;
  };
  auto advance = [&](ItemIter& it) -> bool {
    if (it.w < p.full) { it.q = (xcd * p.full + it.w) * Gx + slot_in_xcd; it.ks = 0; it.ke = p.kt; ++it.w; return true; }
    if (it.left > 0) {
      const int len = (p.kt - it.k0) < it.left ? (p.kt - it.k0) : it.left;
      it.ks = it.k0;
      it.ke = it.k0 + len;
      it.q = p.sib ? it.tr * p.tiles_n + sibling : p.full * p.G + it.tr;
      it.left -= len;
      if (it.ke == p.kt) { ++it.tr; it.k0 = 0; } else it.k0 = it.ke;
      return true;
    }
    return false;
  };

  DmaPlan<A_KC, BM, AI, KT> pa;
  DmaPlan<B_KC, BN, BI, KT> pb;

  // Writes one finished item: a whole tile through the fused epilogue, a piece of a cut tile as raw partial sums.
  auto write_item = [&](const f32x16 (&acc)[TN][4], const ItemIter& it) {
    int tm, tn;
    if (it.ks == 0 && it.ke == p.kt) {
      char* xs = xpose_shape(WNW, TN, PIPE) ? smem + NSTAGE * STAGE_BYTES + wave * XPOSE_BYTES_PER_WAVE : nullptr;
      if (p.ngrp) {
        const int g = __builtin_amdgcn_readfirstlane(group_tile_coords(gt, p.ngrp, it.q, tm, tn));
        store_subtile<TN>(gt.e[g], acc, tm * BM + wm, tn * BN + wn, li, hf, gt.A[g].rows, gt.B[g].rows, xs);
        return;
      }
      plan_tile_coords(p, it.q, tm, tn);
      store_subtile<TN>(e, acc, tm * BM + wm, tn * BN + wn, li, hf, M, N, xs);
      return;
    }
    float* sp = ws + (size_t)(2 * v + (it.ks == 0 ? 1 : 0)) * (BM * BN);
#pragma unroll
    for (int i = 0; i < TN; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int c = 0; c < 4; ++c) {
          f32x4 o = {acc[i][j][4 * c], acc[i][j][4 * c + 1], acc[i][j][4 * c + 2], acc[i][j][4 * c + 3]};
          *reinterpret_cast<f32x4*>(sp + slab_index<TN>(wave, i * 4 + j, c, lane)) = o;
        }
  };

  if constexpr (KT == 64) {
    // 64-deep k-tiles (both operands k-contiguous, 8 waves): a tile row is a whole 128-byte line, so a direct-to-LDS
    // instruction asks for 8 whole lines instead of 16 half lines, and there is one barrier per 64 of k.  Two
    // stages of 64 KB: the loads of k-tile t + 2 are issued, into the stage k-tile t has just been read from, in
    // the last of t's four 16-deep substeps (behind the barrier that also says k-tile t + 1 has landed), so they
    // have a whole k-tile of MFMA time to land.  As in the 32-deep loop the k-tiles of all of a block's items form
    // one stream through the two stages.
    static_assert(NSTAGE == 2, "the 64-deep loop has two stages");
    auto read = [&](const char* as, const char* bs, int kk, bf16x8* fn, bf16x8* fm) {
#pragma unroll
      for (int i = 0; i < TN; ++i)
        fn[i] = B_KC ? frag_kc64(bs, wn + 32 * i + n_row, 2 * kk + hf)
                     : frag_t<BN>(bs, wn + 32 * i + n_rowbase_t, 16 * kk + 8 * hf + kq);
#pragma unroll
      for (int j = 0; j < 4; ++j)
        fm[j] = A_KC ? frag_kc64(as, wm + 32 * j + li, 2 * kk + hf)
                     : frag_t<BM>(as, wm + 32 * j + m_rowbase_t, 16 * kk + 8 * hf + kq);
    };
    constexpr int NDS = (A_KC ? 4 : 8) + (B_KC ? TN : 2 * TN);
    ItemIter L = first_item(), C = L;
    int lt = 0, l_left = 0, lstage = 0, cstage = 0, inflight = 0;
    auto loader_ready = [&]() -> bool {
      if (l_left > 0) return true;
      if (!advance(L)) return false;
      int tm, tn;
      if (p.ngrp) {
        const int g = __builtin_amdgcn_readfirstlane(group_tile_coords(gt, p.ngrp, L.q, tm, tn));
        pa.init(gt.A[g], tm * BM, wave, lane, L.ks * KT);
        pb.init(gt.B[g], tn * BN, wave, lane, L.ks * KT);
      } else {
        plan_tile_coords(p, L.q, tm, tn);
        pa.init(A, tm * BM, wave, lane, L.ks * KT);
        pb.init(B, tn * BN, wave, lane, L.ks * KT);
      }
      lt = 0; l_left = L.ke - L.ks;
      return true;
    };
    auto issue_tile = [&]() {
      char* dst = smem + lstage * STAGE_BYTES;
      pa.issue(dst, lt);
      pb.issue(dst + A_BYTES, lt);
      ++lt; --l_left; ++inflight;
      lstage ^= 1;
    };
#pragma unroll 1
    for (int s = 0; s < 2; ++s)
      if (loader_ready()) issue_tile();
    if (!advance(C)) return;
    bf16x8 fn0[TN], fm0[4], fn1[TN], fm1[4];
    if (inflight >= 2) wait_loads_and_barrier<LPT>(); else wait_loads_and_barrier<0>();
    --inflight;
    read(smem, smem + A_BYTES, 0, fn0, fm0);
    for (;;) {
      f32x16 acc[TN][4];
#pragma unroll
      for (int i = 0; i < TN; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
          for (int x = 0; x < 16; ++x) acc[i][j][x] = 0.f;
      auto mma = [&](const bf16x8* fn, const bf16x8* fm) {
#pragma unroll
        for (int i = 0; i < TN; ++i)
#pragma unroll
          for (int j = 0; j < 4; ++j)
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fn[i], fm[j], acc[i][j], 0, 0, 0);
      };
      // One 64-deep k-tile.  STEADY (1: first of a run, 2: later ones): the loader is two k-tiles ahead inside this
      // item, so everything is unconditional: the A half of k-tile t + 2 goes out in t's last substep (behind the
      // barrier), its B half in the first substep of t + 1, so that a wave's eight loads do not reach the memory
      // pipeline in one burst.  Otherwise (0) the whole k-tile goes out in the last substep, if there is one.
      auto step = [&](auto steady, bool last) {
        constexpr int ST = decltype(steady)::value;
        const char* as = smem + cstage * STAGE_BYTES;
        const char* bs = as + A_BYTES;
        read(as, bs, 1, fn1, fm1);
        if (ST == 2) {
          pb.issue(smem + (lstage ^ 1) * STAGE_BYTES + A_BYTES, lt - 1);
          mma(fn0, fm0);
          interleave_hint_loads<4 * TN, NDS, BI>();
        } else {
          mma(fn0, fm0);
          interleave_hint<4 * TN, NDS, 0>();
        }
        __builtin_amdgcn_sched_barrier(0);
        read(as, bs, 2, fn0, fm0);
        mma(fn1, fm1);
        interleave_hint<4 * TN, NDS, 0>();
        __builtin_amdgcn_sched_barrier(0);
        read(as, bs, 3, fn1, fm1);
        mma(fn0, fm0);
        interleave_hint<4 * TN, NDS, 0>();
        __builtin_amdgcn_sched_barrier(0);
        // last substep: behind the barrier every wave has read all of this stage and the next k-tile has landed
        if (ST != 0) {
          wait_loads_and_barrier<0>();
          cstage ^= 1;
          read(smem + cstage * STAGE_BYTES, smem + cstage * STAGE_BYTES + A_BYTES, 0, fn0, fm0);
          pa.issue(smem + lstage * STAGE_BYTES, lt);
          ++lt; --l_left;
          lstage ^= 1;
          mma(fn1, fm1);
          interleave_hint_loads<4 * TN, NDS, AI>();
        } else {
          const bool more = inflight > 0;
          bool load = false;
          if (more) load = loader_ready();
          __builtin_amdgcn_sched_barrier(0);
          if (more) {
            wait_loads_and_barrier<0>();
            --inflight;
            cstage ^= 1;
            if (load) issue_tile();
            if (!last) read(smem + cstage * STAGE_BYTES, smem + cstage * STAGE_BYTES + A_BYTES, 0, fn0, fm0);
          }
          mma(fn1, fm1);
          interleave_hint<4 * TN, NDS, 0>();
        }
        __builtin_amdgcn_sched_barrier(0);
      };
      const int nt = C.ke - C.ks;
      int t = 0;
      typedef std::integral_constant<int, 0> General;
      if (nt >= 3) {           // k-tiles 0 .. nt - 3 have their k-tile t + 2 inside this item
        step(std::integral_constant<int, 1>{}, false);
        for (t = 1; t + 3 <= nt; ++t) step(std::integral_constant<int, 2>{}, false);
        pb.issue(smem + (lstage ^ 1) * STAGE_BYTES + A_BYTES, lt - 1);
      }
      for (; t < nt; ++t) step(General{}, t + 1 == nt);
      const ItemIter done = C;
      const bool have = advance(C);
      write_item(acc, done);
      if (!have) break;
      read(smem + cstage * STAGE_BYTES, smem + cstage * STAGE_BYTES + A_BYTES, 0, fn0, fm0);
    }
  } else if constexpr (PIPE) {
    // The block's k-tiles, item after item, are one stream through the ring of LDS stages: the loader runs
    // NSTAGE-1 k-tiles ahead of the MFMAs *across item boundaries*, so the first k-tiles of the next item are
    // already in flight while the current item finishes and is written.
    //
    // One wave per SIMD (or two): nothing else hides a fragment read's latency, so the reads are software
    // pipelined by hand.  Each 16-deep k-substep's MFMAs run while the next substep's fragments are read
    // into a second register set; the reads of the next k-tile's first substep need that tile in LDS, so
    // the wait + barrier sits in the middle of a k-tile, between its two substeps.
    //
    // A mid-step wait for k-tile X allows as many operations outstanding as the younger k-tiles have loads.
    // vmcnt also counts the finished item's stores; whatever their completion order relative to the loads,
    // "at most n outstanding" then still implies that all but the youngest n loads have landed.  (Letting
    // the stores stay outstanding as well, by exact counting, measured no gain.)
    auto read = [&](const char* as, const char* bs, int kk, bf16x8* fn, bf16x8* fm) {
#pragma unroll
      for (int i = 0; i < TN; ++i)
        fn[i] = B_KC ? frag_kc(bs, wn + 32 * i + n_row, 2 * kk + hf)
                     : frag_t<BN>(bs, wn + 32 * i + n_rowbase_t, 16 * kk + 8 * hf + kq);
#pragma unroll
      for (int j = 0; j < 4; ++j)
        fm[j] = A_KC ? frag_kc(as, wm + 32 * j + li, 2 * kk + hf)
                     : frag_t<BM>(as, wm + 32 * j + m_rowbase_t, 16 * kk + 8 * hf + kq);
    };
    constexpr int NDS = (A_KC ? 4 : 8) + (B_KC ? TN : 2 * TN);   // LDS read instructions per substep
    ItemIter L = first_item(), C = L;
    int lt = 0, l_left = 0;          // loader: next k-tile of its item, k-tiles of that item not yet issued
    int lstage = 0, cstage = 0;      // stage the next issued k-tile goes to; stage of the k-tile being multiplied
    int inflight = 0;                // k-tiles issued and not yet waited for
    // Makes sure the loader has a k-tile to issue, opening the next item if its current one is used up.
    // The address arithmetic of an item belongs here, outside the MFMA phases.
    auto loader_ready = [&]() -> bool {
      if (l_left > 0) return true;
      if (!advance(L)) return false;
      int tm, tn;
      if (p.ngrp) {
        const int g = __builtin_amdgcn_readfirstlane(group_tile_coords(gt, p.ngrp, L.q, tm, tn));
        pa.init(gt.A[g], tm * BM, wave, lane, L.ks * KT);
        pb.init(gt.B[g], tn * BN, wave, lane, L.ks * KT);
      } else {
        plan_tile_coords(p, L.q, tm, tn);
        pa.init(A, tm * BM, wave, lane, L.ks * KT);
        pb.init(B, tn * BN, wave, lane, L.ks * KT);
      }
      lt = 0; l_left = L.ke - L.ks;
      return true;
    };
    auto issue_tile = [&]() {        // the stream's next k-tile, into the stage after the last one issued
      char* dst = smem + lstage * STAGE_BYTES;
      pa.issue(dst, lt);
      pb.issue(dst + A_BYTES, lt);
      ++lt; --l_left; ++inflight;
      lstage = lstage + 1 == NSTAGE ? 0 : lstage + 1;
    };
    // Wait until the oldest k-tile in flight has landed, then the barrier: `younger` k-tiles were issued
    // after it (capped at 2; allowing fewer than are really outstanding only waits longer).
    auto wait_oldest = [&](int younger) {
      if (NSTAGE >= 5 && younger >= 2) wait_loads_and_barrier<2 * LPT>();
      else if (younger >= 1) wait_loads_and_barrier<LPT>();
      else wait_loads_and_barrier<0>();
    };
#pragma unroll 1
    for (int s = 0; s < NSTAGE - 1; ++s)
      if (loader_ready()) issue_tile();
    if (!advance(C)) return;         // this block has no work (and the loader issued nothing)
    bf16x8 fn0[TN], fm0[4], fn1[TN], fm1[4];
    wait_oldest(inflight - 1);
    --inflight;
    read(smem, smem + A_BYTES, 0, fn0, fm0);
    for (;;) {
      f32x16 acc[TN][4];
#pragma unroll
      for (int i = 0; i < TN; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
          for (int x = 0; x < 16; ++x) acc[i][j][x] = 0.f;
      auto mma = [&](const bf16x8* fn, const bf16x8* fm) {
#pragma unroll
        for (int i = 0; i < TN; ++i)
#pragma unroll
          for (int j = 0; j < 4; ++j)
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fn[i], fm[j], acc[i][j], 0, 0, 0);
      };
      // One k-tile.  STEADY: the pipeline is full and the loader is inside this item,
      // so the wait is a constant and the loads are issued unconditionally: the second substep is then one
      // basic block in which the scheduler can spread them between the MFMAs.  Otherwise everything that
      // needs arithmetic is decided before the first MFMA.  `last`: the item's last k-tile; the next item's
      // first fragments are read after this item is written, so that they are not live across the epilogue.
      auto step = [&](auto steady, bool last) {
        constexpr bool STEADY = decltype(steady)::value != 0;
        bool more = false, load = false;
        if (!STEADY) {
          more = inflight > 0;                          // the stream has a k-tile after this one
          load = more && loader_ready();
          __builtin_amdgcn_sched_barrier(0);
        }
        const char* as = smem + cstage * STAGE_BYTES;
        read(as, as + A_BYTES, 1, fn1, fm1);
        if (STEADY && decltype(steady)::value == 2) {   // the B half of the k-tile whose A half went out one substep ago
          const int ps = lstage == 0 ? NSTAGE - 1 : lstage - 1;
          pb.issue(smem + ps * STAGE_BYTES + A_BYTES, lt - 1);
          mma(fn0, fm0);
          interleave_hint_loads<4 * TN, NDS, BI>();
        } else {
          mma(fn0, fm0);
          interleave_hint<4 * TN, NDS, 0>();
        }
        __builtin_amdgcn_sched_barrier(0);
        cstage = cstage + 1 == NSTAGE ? 0 : cstage + 1;
        const char* an = smem + cstage * STAGE_BYTES;
        if (STEADY) {
          wait_loads_and_barrier<(NSTAGE - 3) * LPT>();
          read(an, an + A_BYTES, 0, fn0, fm0);
          char* dst = smem + lstage * STAGE_BYTES;      // the stage that was read one k-tile ago
          pa.issue(dst, lt);
          ++lt; --l_left;
          lstage = lstage + 1 == NSTAGE ? 0 : lstage + 1;
          mma(fn1, fm1);
          interleave_hint_loads<4 * TN, NDS, AI>();
        } else {
          if (more) {
            wait_oldest(inflight - 1);
            --inflight;
            if (load) issue_tile();
            if (!last) read(an, an + A_BYTES, 0, fn0, fm0);
          }
          mma(fn1, fm1);
          interleave_hint<4 * TN, NDS, 0>();
        }
        __builtin_amdgcn_sched_barrier(0);
      };
      const int nt = C.ke - C.ks;
      int t = 0;
      typedef std::integral_constant<int, 0> General;
      // Steady k-tiles issue the A half of a k-tile's loads in their second substep and its B half in the
      // first substep of the next k-tile, so that the loads of all waves are spread over the whole k-tile
      // instead of arriving at the memory pipeline in one burst behind the barrier.
      if (t + NSTAGE <= nt) {
        step(std::integral_constant<int, 1>{}, false);
        for (++t; t + NSTAGE <= nt; ++t) step(std::integral_constant<int, 2>{}, false);
        const int ps = lstage == 0 ? NSTAGE - 1 : lstage - 1;
        pb.issue(smem + ps * STAGE_BYTES + A_BYTES, lt - 1);
      }
      for (; t < nt; ++t) step(General{}, t + 1 == nt);                             // the loader is in the next item
      const ItemIter done = C;
      const bool have = advance(C);
      write_item(acc, done);
      if (!have) break;
      read(smem + cstage * STAGE_BYTES, smem + cstage * STAGE_BYTES + A_BYTES, 0, fn0, fm0);
    }
  } else {
    // Plain main loop, one item after the other.
    ItemIter I = first_item();
    int nt = 0;
    auto start_item = [&]() {          // addresses of the item's operands and the first NSTAGE-1 k-tiles' loads
      int tm, tn;
      nt = I.ke - I.ks;
      if (p.ngrp) {
        const int g = __builtin_amdgcn_readfirstlane(group_tile_coords(gt, p.ngrp, I.q, tm, tn));
        pa.init(gt.A[g], tm * BM, wave, lane, I.ks * KT);
        pb.init(gt.B[g], tn * BN, wave, lane, I.ks * KT);
      } else {
        plan_tile_coords(p, I.q, tm, tn);
        pa.init(A, tm * BM, wave, lane, I.ks * KT);
        pb.init(B, tn * BN, wave, lane, I.ks * KT);
      }
#pragma unroll
      for (int s = 0; s < NSTAGE - 1; ++s)
        if (s < nt) {
          pa.issue(smem + s * STAGE_BYTES, s);
          pb.issue(smem + s * STAGE_BYTES + A_BYTES, s);
        }
    };
    bool have = advance(I);
    if (have) start_item();
    while (have) {
      f32x16 acc[TN][4];
#pragma unroll
      for (int i = 0; i < TN; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
          for (int x = 0; x < 16; ++x) acc[i][j][x] = 0.f;
      for (int t = 0; t < nt; ++t) {
        // The loads of k-tile t are this thread's oldest outstanding loads; the younger k-tiles (at most
        // NSTAGE-2) stay in flight.  The first k-tile of an item waits for everything: behind the loads
        // issued by start_item sit the previous item's output stores.
        if (t == 0) wait_loads_and_barrier<0>();
        else if (t + NSTAGE - 2 < nt) wait_loads_and_barrier<(NSTAGE - 2) * LPT>();
        else if (NSTAGE > 3 && t + NSTAGE - 3 < nt) wait_loads_and_barrier<(NSTAGE > 3 ? NSTAGE - 3 : 0) * LPT>();
        else wait_loads_and_barrier<0>();
        if (t + NSTAGE - 1 < nt) {
          char* dst = smem + ((t + NSTAGE - 1) % NSTAGE) * STAGE_BYTES;
          pa.issue(dst, t + NSTAGE - 1);
          pb.issue(dst + A_BYTES, t + NSTAGE - 1);
        }
        const char* as = smem + (t % NSTAGE) * STAGE_BYTES;
        const char* bs = as + A_BYTES;
#pragma unroll
        for (int kk = 0; kk < 2; ++kk) {
          bf16x8 fn[TN], fm[4];
#pragma unroll
          for (int i = 0; i < TN; ++i)
            fn[i] = B_KC ? frag_kc(bs, wn + 32 * i + n_row, 2 * kk + hf)
                         : frag_t<BN>(bs, wn + 32 * i + n_rowbase_t, 16 * kk + 8 * hf + kq);
#pragma unroll
          for (int j = 0; j < 4; ++j)
            fm[j] = A_KC ? frag_kc(as, wm + 32 * j + li, 2 * kk + hf)
                         : frag_t<BM>(as, wm + 32 * j + m_rowbase_t, 16 * kk + 8 * hf + kq);
#pragma unroll
          for (int i = 0; i < TN; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j)
              acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fn[i], fm[j], acc[i][j], 0, 0, 0);
        }
      }
      const ItemIter done = I;
      have = advance(I);
      // every wave is done reading the LDS stages: the next item's first loads may overwrite them, and
      // they fly while this item's results are written
      asm volatile("s_barrier" ::: "memory");
      if (have) start_item();
      write_item(acc, done);
    }
  }
}

// Adds the partial-sum slabs of every tail tile that was cut, in block order, and applies the epilogue.
// One thread per run of 8 columns (the unit of the fused epilogue), with the main kernel's
// lane-to-element mapping: thread (wave, ij, q, lane) owns acc[i][j][8q .. 8q+7] of that lane.
template <int WNW, int TN>
__global__ void __launch_bounds__(256) k_sk_fixup(const float* __restrict__ ws, Epilogue e, int M, int N, SkPlan p,
                                                  GroupTable gt) {
  constexpr int BN = 32 * TN * WNW, NWAVES = 2 * WNW, UNITS_PER_WAVE = 8 * TN, BLOCKS_PER_TILE = NWAVES * UNITS_PER_WAVE / 4;
  const int tr = blockIdx.x / BLOCKS_PER_TILE;
  const int unit = (blockIdx.x % BLOCKS_PER_TILE) * 4 + (threadIdx.x >> 6);      // (wave, ij, q)
  const int lane = threadIdx.x & 63;
  const int wave = unit / UNITS_PER_WAVE, ij = (unit % UNITS_PER_WAVE) >> 1, q = unit & 1;
  int tm, tn;
  if (p.ngrp) {
    const int g = group_tile_coords(gt, p.ngrp, p.full * p.G + tr, tm, tn);
    e = gt.e[g]; M = gt.A[g].rows; N = gt.B[g].rows;
  } else {
    plan_tile_coords(p, p.sib ? tr : p.full * p.G + tr, tm, tn);
  }
  const int i = ij >> 2, j = ij & 3, li = lane & 31, hf = lane >> 5;
  const int m = tm * BM + (wave / WNW) * 128 + 32 * j + li;
  const int n = tn * BN + (wave % WNW) * (32 * TN) + 32 * i + 16 * q + 8 * hf;
  // the ranges that cut this tile's reduction: of tail tile tr, or in panel mode of the panel of tile tr
  const int cut_unit = p.sib ? tr / p.tiles_n : tr, sibling = p.sib ? tr - cut_unit * p.tiles_n : 0;
  const long u0 = (long)cut_unit * p.kt, u1 = u0 + p.kt;
  const int v_lo = (int)(u0 / p.upb), v_hi = (int)((u1 - 1) / p.upb);
  if (v_lo == v_hi) return;            // computed whole by one block
  float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  for (int vr = v_lo; vr <= v_hi; ++vr) {
    const int v = p.sib ? vr * p.sib + sibling : vr;
    const int slab = 2 * v + ((long)vr * p.upb <= u0 ? 1 : 0);
    const float* sp = ws + (size_t)slab * (BM * BN);
    f32x4 a = *reinterpret_cast<const f32x4*>(sp + slab_index<TN>(wave, ij, 2 * q, lane));
    f32x4 b = *reinterpret_cast<const f32x4*>(sp + slab_index<TN>(wave, ij, 2 * q + 1, lane));
#pragma unroll
    for (int x = 0; x < 4; ++x) { acc[x] += a[x]; acc[4 + x] += b[x]; }
  }
  if (m < M && n < N) epilogue8(e, m, n, acc);
}

int device_cus() {
  static int n = 0;
  if (!n) {
    int dev = 0, v = 0;
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || v < 8)
      v = 256;
    n = v;
  }
  return n;
}

template <bool A_KC, bool B_KC, int WNW, int TN, int NSTAGE, bool PIPE, int KT = 32>
hipError_t launch(const OpCtx& c, const GemmArgs& g, const SkPlan& p, bool partials, const GroupTable* grp = nullptr,
                  double flops = 0.0) {
  constexpr int BN = 32 * TN * WNW;
  constexpr int smem = NSTAGE * (BM + BN) * KT * 2 + (xpose_shape(WNW, TN, PIPE) ? 2 * WNW * XPOSE_BYTES_PER_WAVE : 0);
  static bool configured = false;
  auto kern = k_gemm_dma<A_KC, B_KC, WNW, TN, NSTAGE, PIPE, KT>;
  if (!configured) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, smem);
    if (e != hipSuccess) return e;
    configured = true;
  }
  Operand A{(const bf16_t*)g.A, g.lda, g.M}, B{(const bf16_t*)g.B, g.ldb, g.N};
  Epilogue e = make_epilogue(g);
  static char kname[64];
  if (!kname[0])
    snprintf(kname, sizeof kname, KT == 32 ? "k_gemm_dma<%s, %s, %d, %d, %d, %s>" : "k_gemm_dma<%s, %s, %d, %d, %d, %s, 64>",
             A_KC ? "true" : "false", B_KC ? "true" : "false", WNW, TN, NSTAGE, PIPE ? "true" : "false");
  hipError_t err;
  static const GroupTable no_group = {};
  const GroupTable& gt = grp ? *grp : no_group;
  {
    ProfScope one_(c, KC_GEMM_KERNEL, grp ? flops : 2.0 * g.M * g.N * g.K, 0, kname);
    kern<<<dim3(p.G), 128 * WNW, smem, c.stream>>>(A, B, e, g.M, g.N, p, c.splitk_ws, gt);
    err = hipGetLastError();
  }
  if (err != hipSuccess || !partials) return err;
  k_sk_fixup<WNW, TN><<<dim3((p.sib ? p.tiles_m * p.tiles_n : p.tail_tiles) * (2 * WNW * 8 * TN / 4)), 256, 0, c.stream>>>(c.splitk_ws, e, g.M, g.N, p, gt);
  return hipGetLastError();
}

}  // namespace

// The DMA kernel takes: K a multiple of 32, and an operand stored k-major needs at least one full
// 8-row chunk column set (rows >= 8, rows % 8 == 0 is already required by the caller's checks).
bool gemm_dma_ok(const GemmArgs& g) { return g.K % 32 == 0 && g.K >= 32 && g.M >= 8 && g.N >= 8; }

// Distribution of an M x N x K problem over the persistent grid of one tile shape
// (kind 0: 256 x 128, two blocks per CU; 1: 256 x 256 with 8 waves; 2: 256 x 256 with 4 waves).
// mode 0: every tile whole, one per block per wave; 1: the last, partial wave of tiles cut along k;
// 2: panel mode (see SkPlan).  Modes 1 and 2 need workspace.  Returns false if the mode does not apply.
bool gemm_dma_plan(const OpCtx& c, const GemmArgs& g, int kind, int mode, DmaGemmPlan* out) {
  // kind 3: 256 x 256 with 8 waves and 64-deep k-tiles (K a multiple of 64)
  if (kind == 3 && g.K % 64 != 0) return false;
  const int bk = kind == 3 ? 64 : BK;
  const int bn = kind == 0 ? 128 : 256, per_cu = kind == 0 ? 2 : 1;
  SkPlan p;
  p.G = (device_cus() * per_cu) & ~7;
  p.tiles_m = (g.M + BM - 1) / BM;
  p.tiles_n = (g.N + bn - 1) / bn;
  p.kt = g.K / bk;
  p.sib = 0;
  p.ngrp = 0;
  const long T = (long)p.tiles_m * p.tiles_n;
  const long min_len = kind == 3 ? 2 : 4, max_cut = 16;                 // shortest piece; most pieces per tile
  auto clamp_upb = [&](long upb, bool within_tile) {
    if (upb < min_len) upb = min_len;
    if (upb * max_cut < p.kt) upb = (p.kt + max_cut - 1) / max_cut;
    if (within_tile && upb > p.kt) upb = p.kt;
    return upb;
  };
  // number of pieces that are not whole tiles when `units` k-steps (tile-major, kt per tile) are cut every upb
  auto count_partial = [&](long units, long upb) {
    long n = 0;
    for (long u0 = 0; u0 < units; u0 += upb) {
      long u = u0, ue = u0 + upb < units ? u0 + upb : units;
      while (u < ue) {
        long tr = u / p.kt, ks = u - tr * p.kt, len = (p.kt - ks) < (ue - u) ? (p.kt - ks) : (ue - u);
        if (!(ks == 0 && len == p.kt)) ++n;
        u += len;
      }
    }
    return n;
  };
  long partial_slabs = 0;
  if (mode == 2) {
    const int Gx = p.G >> 3;
    if (p.tiles_n < 2 || p.tiles_n > 8 || p.tiles_n > Gx) return false;
    const long groups = 8L * (Gx / p.tiles_n), units = (long)p.tiles_m * p.kt;
    const long upb = clamp_upb((units + groups - 1) / groups, false);
    // ranges longer than a panel (more panels than groups) work but measured slower than cutting the last
    // wave of tiles; ranges of whole panels would cut nothing
    if (upb >= p.kt) return false;
    p.sib = p.tiles_n; p.full = 0; p.tail_tiles = (int)T; p.upb = (int)upb;
    partial_slabs = count_partial(units, upb) * p.tiles_n;
    if (!c.splitk_ws || (size_t)2 * p.G * BM * bn > c.splitk_elems) return false;
  } else {
    p.full = (int)(T / p.G);
    p.tail_tiles = (int)(T - (long)p.full * p.G);
    p.upb = p.kt;
    if (mode == 1 && p.tail_tiles > 0) {
      const long U = (long)p.tail_tiles * p.kt;
      p.upb = (int)clamp_upb((U + p.G - 1) / p.G, true);
      if (p.upb < p.kt) {
        partial_slabs = count_partial(U, p.upb);
        if (!c.splitk_ws || (size_t)2 * p.G * BM * bn > c.splitk_elems) return false;
      }
    }
  }
  out->kind = kind;
  out->full = p.full; out->tail_tiles = p.tail_tiles; out->upb = p.upb; out->G = p.G; out->kt = p.kt;
  out->tiles_m = p.tiles_m; out->tiles_n = p.tiles_n; out->sib = p.sib;
  out->partial_bytes = (double)partial_slabs * BM * bn * 4.0;
  out->steps = (long)p.full * p.kt + (p.tail_tiles > 0 ? p.upb : 0);
  out->items = p.full + (p.tail_tiles > 0 ? (p.sib ? p.upb / p.kt + 2 : (p.upb < p.kt ? 2 : 1)) : 0);
  return true;
}

hipError_t gemm_dma(const OpCtx& c, const GemmArgs& g, const DmaGemmPlan& d) {
  SkPlan p;
  p.tiles_m = d.tiles_m; p.tiles_n = d.tiles_n; p.kt = d.kt; p.full = d.full; p.tail_tiles = d.tail_tiles;
  p.upb = d.upb; p.G = d.G; p.sib = d.sib; p.ngrp = 0;
  const bool partials = d.partial_bytes > 0;
#define LP_DMA(AK, BK_)                                                    \
  (d.kind == 3 ? launch<AK, BK_, 4, 2, 2, true, 64>(c, g, p, partials)            \
   : d.kind == 1 ? launch<AK, BK_, 4, 2, 4, true>(c, g, p, partials)              \
   : d.kind == 2 ? launch<AK, BK_, 2, 4, 5, true>(c, g, p, partials)              \
                 : launch<AK, BK_, 2, 2, 3, false>(c, g, p, partials))
  if (g.a_kc && g.b_kc) return LP_DMA(true, true);
  if (g.a_kc && !g.b_kc) return LP_DMA(true, false);
  if (!g.a_kc && g.b_kc) return LP_DMA(false, true);
  return LP_DMA(false, false);
#undef LP_DMA
}

// Grouped launch of n products (see GroupTable).  Returns hipErrorInvalidValue, with nothing launched, if the set
// does not qualify (the caller then launches them one by one): bf16 operands, the same K (a multiple of 32) and the
// same operand layouts for all, every pointer and leading dimension fit for 16-byte accesses, at most kMaxGroup
// problems, workspace for the cut tail.  Epilogues and output types may differ from problem to problem.
hipError_t gemm_dma_grouped(const OpCtx& c, const GemmArgs* gs, int n) {
  if (n < 2 || n > kMaxGroup || c.dt != BF16) return hipErrorInvalidValue;
  const GemmArgs& g0 = gs[0];
  GroupTable gt = {};
  long T = 0;
  double flops = 0.0;
  auto al16 = [](const void* p) { return ((uintptr_t)p & 15) == 0; };
  for (int i = 0; i < n; ++i) {
    const GemmArgs& g = gs[i];
    if (!gemm_dma_ok(g) || g.K != g0.K || g.a_kc != g0.a_kc || g.b_kc != g0.b_kc) return hipErrorInvalidValue;
    if (g.M % 8 || g.N % 8 || g.lda % 8 || g.ldb % 8 || g.ldc % 8 || !al16(g.A) || !al16(g.B) || !al16(g.C) ||
        (g.bias && !al16(g.bias)) || (g.pre && !al16(g.pre)) || (g.dact_src && (!al16(g.dact_src) || g.ldd % 8)) ||
        (g.res && (!al16(g.res) || g.ldr % 8)))
      return hipErrorInvalidValue;
    gt.A[i] = Operand{(const bf16_t*)g.A, g.lda, g.M};
    gt.B[i] = Operand{(const bf16_t*)g.B, g.ldb, g.N};
    gt.e[i] = make_epilogue(g);
    gt.tiles_n[i] = (g.N + 255) / 256;
    gt.first[i] = (int)T;
    T += (long)((g.M + BM - 1) / BM) * gt.tiles_n[i];
    flops += 2.0 * g.M * g.N * g.K;
  }
  for (int i = n; i <= kMaxGroup; ++i) gt.first[i] = (int)T;
  for (int i = n; i < kMaxGroup; ++i) gt.tiles_n[i] = 1;
  SkPlan p;
  p.G = device_cus() & ~7;
  p.tiles_m = (int)T; p.tiles_n = 1;                 // only the product is used outside the tile numbering
  static int deep_ok = -1;           // LP_GROUP_K64=0 keeps the 32-deep k-tiles (for measurements)
  if (deep_ok < 0) { const char* e = getenv("LP_GROUP_K64"); deep_ok = (e && e[0] == '0') ? 0 : 1; }
  const bool deep = deep_ok && g0.K % 64 == 0 && g0.K >= 128;
  const int bk = deep ? 64 : BK;
  const long min_len = deep ? 2 : 4;
  p.kt = g0.K / bk;
  p.sib = 0; p.ngrp = n;
  p.full = (int)(T / p.G);
  p.tail_tiles = (int)(T - (long)p.full * p.G);
  p.upb = p.kt;
  bool partials = false;
  if (p.tail_tiles > 0) {
    // Two ways to spread the last partial wave of tiles over the grid.  Balanced: the tail's k-steps in tile-major
    // order are cut into G equal ranges (every CU busy to the end, but ranges start anywhere inside a tile: blocks
    // that run side by side sit at different k-steps of different tiles, so no operand panel is shared in L2, and
    // nearly every block writes partial sums).  Uniform: every tail tile is cut into the same s = floor(G / tiles)
    // equal pieces (s = 1: whole tiles, no partial sums and no fix-up launch at all); blocks of one tile row or
    // column then walk the same k-steps together and share their operand panels.  Measured on a layer's four
    // weight gradients: width 768 (108 tiles: two pieces each, 128 k-steps against 108) 182 -> 172 us alone and the
    // same step time; width 1024 (192 tiles: whole, 256 k-steps against 192) 279 -> 309 us: the k-step of this
    // kernel with both operands k-major costs 1.05 .. 1.2 us however the operands are shared, so idle CUs are not
    // paid back.  The uniform cut is taken when it leaves the longest block at most 1.25 times the balanced work.
    const long U = (long)p.tail_tiles * p.kt;
    long upb = (U + p.G - 1) / p.G;
    if (upb < min_len) upb = min_len;
    if (upb * 16 < p.kt) upb = (p.kt + 15) / 16;
    if (upb > p.kt) upb = p.kt;
    long s = p.G / p.tail_tiles;
    if (s < 1) s = 1;
    while (s > 1 && (p.kt % s != 0 || p.kt / s < min_len)) --s;
    const long upb_uniform = p.kt / s;
    static int forced = -1;           // LP_GROUP_SPLIT=balanced|uniform forces one (for measurements)
    if (forced < 0) { const char* e = getenv("LP_GROUP_SPLIT"); forced = !e ? 0 : (e[0] == 'b' ? 1 : (e[0] == 'u' ? 2 : 0)); }
    const bool uniform = forced == 2 || (forced == 0 && (double)upb_uniform <= 1.25 * (double)upb);
    p.upb = (int)(uniform ? upb_uniform : upb);
    if (p.upb < p.kt) {
      partials = true;
      if (!c.splitk_ws || (size_t)2 * p.G * BM * 256 > c.splitk_elems) return hipErrorInvalidValue;
    }
  }
  ProfScope prof_(c, KC_GEMM, flops);
  GemmArgs g = g0;                                    // epilogue flags (fp32 output, accumulate) are common
#define LP_DMA_G(AK, BK_) \
  (deep ? launch<AK, BK_, 4, 2, 2, true, 64>(c, g, p, partials, &gt, flops) : launch<AK, BK_, 4, 2, 4, true>(c, g, p, partials, &gt, flops))
  if (g.a_kc && g.b_kc) return LP_DMA_G(true, true);
  if (g.a_kc && !g.b_kc) return LP_DMA_G(true, false);
  if (!g.a_kc && g.b_kc) return LP_DMA_G(false, true);
  return LP_DMA_G(false, false);
#undef LP_DMA_G
}

}  // namespace lp
