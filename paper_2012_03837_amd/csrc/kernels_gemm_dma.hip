// bf16 GEMM for large, aligned shapes: operand tiles stream global -> LDS with the gfx950 16-byte
// direct-to-LDS load (global_load_lds_dwordx4: no registers, no VALU), through a ring of NSTAGE LDS
// stages, so several k-tiles of HBM / L2 latency are in flight behind the MFMA phase.
//
// Block tile 256(m) x BN(n) x 32(k), BN = 64*NWN; 2*NWN wavefronts, each owning 128 x 64 (4 x 2 tiles of
// v_mfma_f32_32x32x16_bf16).  BN = 256: 512 threads, 4 stages (128 KB LDS), one block per CU.
// BN = 128: 256 threads, 3 stages (72 KB), two blocks per CU.
//
// A direct-to-LDS load writes lane l's 16 bytes at (wave-uniform base) + 16*l, so a wave fills 1 KB of
// contiguous LDS; tiles are therefore unpadded and bank conflicts are avoided by an XOR swizzle that the
// *global* address of each lane undoes:
//   kc tile   [row][4 chunks of 8 k]   : chunk c of row r sits in slot c ^ ((r>>2)&3)
//   k-major   [k][32.. chunks of 8 rows]: chunk j of k-row k sits in slot j ^ ((k&3)<<2)   (read with
//                                         ds_read_b64_tr_b16, as in the register-staged kernel)
// One barrier per k-tile: wait until this thread's loads of tile t have landed (s_waitcnt vmcnt leaves
// the younger tiles in flight), barrier, issue the loads of tile t+NSTAGE-1 into the stage that was read
// during tile t-1, then 16 MFMAs per wave on tile t.  Requires K % 32 == 0 (no zero fill on this path).
#include "common.h"
#include "gemm_common.h"

namespace lp {

namespace {

constexpr int BM = 256, BK = 32;
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
template <bool KC, int ROWS, int NI>
struct DmaPlan {
  const bf16_t* g[NI];
  int lds_off[NI];      // byte offset of the wave's 1 KB destination inside the operand's stage region
  int64_t kstep;
  __device__ __forceinline__ void init(const Operand& o, int r0, int wave, int lane, int kbase) {
#pragma unroll
    for (int i = 0; i < NI; ++i) {
      int q = wave * NI + i;              // which 1 KB of the tile
      lds_off[i] = q * 1024;
      if (KC) {
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
    kstep = KC ? (int64_t)BK : (int64_t)BK * o.ld;
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

template <bool A_KC, bool B_KC, int NWN, int NSTAGE>
__global__ void __launch_bounds__(128 * NWN, NWN == 4 ? 1 : 2)
k_gemm_dma(Operand A, Operand B, Epilogue e, int M, int N, int K, int tiles_m, int tiles_n, int splits, float* ws) {
  constexpr int BN = 64 * NWN, NWAVES = 2 * NWN;
  constexpr int A_BYTES = BM * BK * 2, B_BYTES = BN * BK * 2, STAGE_BYTES = A_BYTES + B_BYTES;
  constexpr int AI = (A_BYTES / 1024) / NWAVES, BI = (B_BYTES / 1024) / NWAVES, LPT = AI + BI;
  extern __shared__ __attribute__((aligned(1024))) char smem[];
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
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
  const int wm = (wave / NWN) * 128, wn = (wave % NWN) * 64;

  const int nt_all = K / BK, per_split = (nt_all + splits - 1) / splits;
  const int t_first = split * per_split;
  const int nt = nt_all - t_first < per_split ? (nt_all - t_first > 0 ? nt_all - t_first : 0) : per_split;

  DmaPlan<A_KC, BM, AI> pa;
  DmaPlan<B_KC, BN, BI> pb;
  pa.init(A, m0, wave, lane, t_first * BK);
  pb.init(B, n0, wave, lane, t_first * BK);

  f32x16 acc[2][4];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

#pragma unroll
  for (int s = 0; s < NSTAGE - 1; ++s)
    if (s < nt) {
      pa.issue(smem + s * STAGE_BYTES, s);
      pb.issue(smem + s * STAGE_BYTES + A_BYTES, s);
    }

  const int li = lane & 31, hf = lane >> 5;
  const int n_row = nmap(li);
  const int c4 = lane & 3, half16 = (lane >> 4) & 1;
  const int n_rowbase_t = nmap(16 * half16 + 4 * c4);
  const int m_rowbase_t = 16 * half16 + 4 * c4;
  const int kq = (lane & 15) >> 2;

  // Fragments of one 16-wide k-step: 2 on the n side, 4 on the m side.
  auto read_frags = [&](const char* as, const char* bs, int ks, bf16x8* fn, bf16x8* fm) {
#pragma unroll
    for (int i = 0; i < 2; ++i)
      fn[i] = B_KC ? frag_kc(bs, wn + 32 * i + n_row, 2 * ks + hf)
                   : frag_t<BN>(bs, wn + 32 * i + n_rowbase_t, 16 * ks + 8 * hf + kq);
#pragma unroll
    for (int j = 0; j < 4; ++j)
      fm[j] = A_KC ? frag_kc(as, wm + 32 * j + li, 2 * ks + hf)
                   : frag_t<BM>(as, wm + 32 * j + m_rowbase_t, 16 * ks + 8 * hf + kq);
  };
  auto mma = [&](const bf16x8* fn, const bf16x8* fm) {
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j)
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fn[i], fm[j], acc[i][j], 0, 0, 0);
  };

  for (int t = 0; t < nt; ++t) {
    // loads of tile t are the oldest outstanding; the younger tiles (at most NSTAGE-2) stay in flight
    if (t + NSTAGE - 2 < nt) wait_loads_and_barrier<(NSTAGE - 2) * LPT>();
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
    for (int ks = 0; ks < 2; ++ks) {
      bf16x8 fn[2], fm[4];
      read_frags(as, bs, ks, fn, fm);
      mma(fn, fm);
    }
  }

#pragma unroll
  for (int j = 0; j < 4; ++j) {
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
        if (splits > 1) {
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

template <bool A_KC, bool B_KC, int NWN, int NSTAGE>
hipError_t launch(const OpCtx& c, const GemmArgs& g, int splits) {
  constexpr int BN = 64 * NWN;
  constexpr int smem = NSTAGE * (BM + BN) * BK * 2;
  static bool configured = false;
  auto kern = k_gemm_dma<A_KC, B_KC, NWN, NSTAGE>;
  if (!configured) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, smem);
    if (e != hipSuccess) return e;
    configured = true;
  }
  Operand A{(const bf16_t*)g.A, g.lda, g.M}, B{(const bf16_t*)g.B, g.ldb, g.N};
  int tm = (g.M + BM - 1) / BM, tn = (g.N + BN - 1) / BN;
  kern<<<dim3(tm * tn * splits), 128 * NWN, smem, c.stream>>>(A, B, make_epilogue(g), g.M, g.N, g.K, tm, tn, splits,
                                                             c.splitk_ws);
  return hipGetLastError();
}

}  // namespace

// The DMA kernel takes: K a multiple of 32, and an operand stored k-major needs at least one full
// 8-row chunk column set (rows >= 8, rows % 8 == 0 is already required by the caller's checks).
bool gemm_dma_ok(const GemmArgs& g) { return g.K % 32 == 0 && g.K >= 32 && g.M >= 8 && g.N >= 8; }

// nwn = 4: 256 x 256 tiles; nwn = 2: 256 x 128 tiles.
hipError_t gemm_dma(const OpCtx& c, const GemmArgs& g, int nwn, int splits) {
#define LP_DMA(AK, BK_) (nwn == 4 ? launch<AK, BK_, 4, 4>(c, g, splits) : launch<AK, BK_, 2, 3>(c, g, splits))
  if (g.a_kc && g.b_kc) return LP_DMA(true, true);
  if (g.a_kc && !g.b_kc) return LP_DMA(true, false);
  if (!g.a_kc && g.b_kc) return LP_DMA(false, true);
  return LP_DMA(false, false);
#undef LP_DMA
}

}  // namespace lp
