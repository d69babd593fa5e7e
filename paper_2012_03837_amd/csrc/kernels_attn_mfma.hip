// Causal multi-head attention on the CDNA4 matrix cores (bf16 operands, fp32 accumulation and
// softmax), head size 64, flash-style: the S x S score matrix lives only in registers.
//
// All three kernels keep the score tile transposed where that puts one query per lane column, so
// that the running max / sum / log-sum-exp of a query are lane-uniform scalars:
//   forward : S^T[key, q] = K Q^T  -> online softmax ->  O^T[dh, q] += V^T P^T
//   dQ      : S^T, dP^T[key, q] = V dO^T -> dS^T -> dQ^T[dh, q] += K^T dS^T
//   dK, dV  : S[q, key] = Q K^T, dP[q, key] = dO V^T -> P, dS -> dV^T[dh, key] += dO^T P,
//             dK^T[dh, key] += Q^T dS
// The accumulator layout of v_mfma_f32_32x32x16_bf16 (value v of lane l: row 8*(v/4) + 4*(l/32) + v%4,
// column l%32) is exactly the B-operand layout of the next MFMA over the row index, so P and dS
// never pass through LDS.  Operands whose reduction index is the slow one in memory (V for the
// forward, K for dQ, Q and dO for dK/dV) sit in LDS as in memory and are read with the transposing LDS
// read (ds_read_b64_tr_b16).  The next tile's global loads are issued before the current tile's MFMAs.
// Layout: qkv [B*S, 3*H*64] (q | k | v, head h at columns h*64..), o [B*S, H*64], lse [B, H, S].
#include "common.h"

namespace lp {

constexpr int ALD = 72;                  // padded LDS row: 64 + 8 elements (144 bytes)
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

#define MFMA32(a, b, c) __builtin_amdgcn_mfma_f32_32x32x16_bf16((a), (b), (c), 0, 0, 0)

__device__ __forceinline__ bf16x8 zero8() {
  bf16x8 z;
#pragma unroll
  for (int i = 0; i < 8; ++i) z[i] = (bf16_t)0.f;
  return z;
}
__device__ __forceinline__ void zero16(f32x16& a) {
#pragma unroll
  for (int i = 0; i < 16; ++i) a[i] = 0.f;
}
// 8 accumulator values -> bf16 B-operand fragment (values 8*kk .. 8*kk+7 of a 32x32 tile)
__device__ __forceinline__ bf16x8 pack8(const f32x16& a, int kk) {
  bf16x8 r;
#pragma unroll
  for (int e = 0; e < 8; ++e) r[e] = (bf16_t)a[8 * kk + e];
  return r;
}
typedef __attribute__((address_space(3))) bf16x4 lds_bf16x4;

// A-operand fragment over a reduction index that is the ROW index of a straight LDS tile s[row][col] (a
// key or query index), for output rows that are its columns c0 .. c0+31 (head-size index): lane (n, hf)
// gets s[r0 + {4hf..4hf+3}][c0 + n] and s[r0 + 8 + {4hf..4hf+3}][c0 + n], the order in which the previous
// MFMA's accumulator holds P / dS.  Done with the transposing LDS read (ds_read_b64_tr_b16): within a
// 16-lane group, lane 4r+c supplies the 8-byte chunk s[row + r][4c..4c+3] and lane 4c+e receives element e
// of the four chunks r = 0..3, so nothing is ever stored transposed.
__device__ __forceinline__ bf16x8 frag_tr(const bf16_t (*s)[ALD], int r0, int c0, int lane) {
  const int g = lane >> 4, l16 = lane & 15, hf = g >> 1;
  const bf16_t* p = &s[r0 + 4 * hf + (l16 >> 2)][c0 + 16 * (g & 1) + 4 * (l16 & 3)];
  bf16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4*)(p));
  bf16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4*)(p + 8 * ALD));
  bf16x8 r;
#pragma unroll
  for (int e = 0; e < 4; ++e) { r[e] = lo[e]; r[4 + e] = hi[e]; }
  return r;
}
// A [64 rows][64 cols] bf16 tile (rows r0.., row stride ld, rows >= nrows read as zero) on its way into
// LDS: 256 threads, 16 elements each, held in registers between the global load and the LDS store so that
// the next tile's loads fly while the current tile is computed.
struct TileRegs { bf16x8 v0, v1; };
__device__ __forceinline__ TileRegs load_tile(const bf16_t* src, size_t ld, int r0, int nrows) {
  const int r = threadIdx.x >> 2, ch = (threadIdx.x & 3) * 16;
  TileRegs t;
  t.v0 = zero8(); t.v1 = zero8();
  if (r0 + r < nrows) {
    const bf16_t* p = src + (size_t)(r0 + r) * ld + ch;
    t.v0 = *reinterpret_cast<const bf16x8*>(p);
    t.v1 = *reinterpret_cast<const bf16x8*>(p + 8);
  }
  return t;
}
__device__ __forceinline__ void store_tile(const TileRegs& t, bf16_t (*dst)[ALD]) {
  const int r = threadIdx.x >> 2, ch = (threadIdx.x & 3) * 16;
  *reinterpret_cast<bf16x8*>(&dst[r][ch]) = t.v0;
  *reinterpret_cast<bf16x8*>(&dst[r][ch + 8]) = t.v1;
}

// Work order.  The grid is one-dimensional: block L takes sequence block L / (B*H) (counted from the heavy end)
// of head-and-batch index L % (B*H).  With causal masking the work of a 128-row block grows with its position
// (shrinks, for the key blocks of dK/dV), and workgroups go to the eight XCDs round-robin by their linear
// index and to compute units as slots free up: so the heaviest blocks start first and the light ones fill the
// gaps, every XCD gets the same mix when B*H is a multiple of 8, and all blocks of one head and batch entry
// run on one XCD, whose L2 then serves their shared K and V (or Q and dO) tiles.
struct AttnBlock { int x, h, b; };
__device__ __forceinline__ AttnBlock attn_block(int H, int BH, int nblk, bool heavy_last) {
  const int cls = blockIdx.x / BH, bh = blockIdx.x % BH;
  AttnBlock a;
  a.x = heavy_last ? nblk - 1 - cls : cls;
  a.h = bh % H;
  a.b = bh / H;
  return a;
}

// ================================================================================= forward
__global__ void __launch_bounds__(256, 3) k_attn_fwd_mfma(const bf16_t* __restrict__ qkv, bf16_t* __restrict__ o,
                                                       float* __restrict__ lse, int S, int H, int BH, int causal) {
  __shared__ __attribute__((aligned(16))) bf16_t Ks[64][ALD];
  __shared__ __attribute__((aligned(16))) bf16_t Vs[64][ALD];
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), n = lane & 31, hf = lane >> 5;
  const AttnBlock ab = attn_block(H, BH, (S + 127) / 128, causal != 0);
  const int bx = ab.x;
  const int h = ab.h, b = ab.b, d = H * 64;
  const size_t ld = (size_t)3 * d;
  const bf16_t* base = qkv + (size_t)b * S * ld;
  const int q0 = bx * 128 + wave * 32, qi = q0 + n;
  bf16x8 qf[4];
#pragma unroll
  for (int kk = 0; kk < 4; ++kk)
    qf[kk] = qi < S ? *reinterpret_cast<const bf16x8*>(base + (size_t)qi * ld + h * 64 + 16 * kk + 8 * hf) : zero8();
  float m = -INFINITY, l = 0.f;
  f32x16 oacc[2];
  zero16(oacc[0]); zero16(oacc[1]);
  const float c = 0.125f * kLog2e;
  int q_hi = bx * 128 + 127;
  if (q_hi > S - 1) q_hi = S - 1;
  const int n_tiles = causal ? q_hi / 64 + 1 : (S + 63) / 64;
  TileRegs kr = load_tile(base + d + h * 64, ld, 0, S), vr = load_tile(base + 2 * d + h * 64, ld, 0, S);
  for (int jt = 0; jt < n_tiles; ++jt) {
    const int k0 = jt * 64;
    __syncthreads();
    store_tile(kr, Ks);
    store_tile(vr, Vs);
    __syncthreads();
    if (jt + 1 < n_tiles) {      // the next key tile's loads fly during this tile's MFMAs
      kr = load_tile(base + d + h * 64, ld, k0 + 64, S);
      vr = load_tile(base + 2 * d + h * 64, ld, k0 + 64, S);
    }
    const bool active = q0 < S && (!causal || k0 <= q0 + 31);
    if (!active) continue;
    f32x16 st[2];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      zero16(st[i]);
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) {
        bf16x8 kf = *reinterpret_cast<const bf16x8*>(&Ks[32 * i + n][16 * kk + 8 * hf]);
        st[i] = MFMA32(kf, qf[kk], st[i]);
      }
    }
    // The scale 1/sqrt(64) * log2(e) is positive: the running maximum is taken over the raw scores and scaled once,
    // and the scaling of every score rides in the fused multiply-add that feeds the exponential.
    float mt = -INFINITY;
    // only tiles that touch the diagonal or the end of the sequence need the mask (wave-uniform test)
    const bool need_mask = k0 + 63 >= S || (causal && k0 + 63 > q0);
    if (need_mask) {
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          int kj = k0 + 32 * i + 8 * (v / 4) + 4 * hf + (v % 4);
          float s = st[i][v];
          if (kj >= S || (causal && kj > qi)) s = -INFINITY;
          st[i][v] = s;
          mt = fmaxf(mt, s);
        }
    } else {
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) mt = fmaxf(mt, st[i][v]);
    }
    mt = fmaxf(mt, __shfl_xor(mt, 32, 64)) * c;
    float mn = fmaxf(m, mt);
    float mref = mn == -INFINITY ? 0.f : mn;
    float alpha = exp2f(m - mref);
    float rs = 0.f;
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        float p = __builtin_amdgcn_exp2f(__builtin_fmaf(st[i][v], c, -mref));
        st[i][v] = p;
        rs += p;
      }
    l = l * alpha + rs;
    m = mn;
    // once the running maxima have settled every lane's alpha is exactly 1: skip the rescale then (wave-uniform)
    if (__builtin_amdgcn_ballot_w64(alpha != 1.f) != 0) {
#pragma unroll
      for (int dh = 0; dh < 2; ++dh)
#pragma unroll
        for (int v = 0; v < 16; ++v) oacc[dh][v] *= alpha;
    }
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int kk = 0; kk < 2; ++kk) {
        bf16x8 pf = pack8(st[i], kk);
#pragma unroll
        for (int dh = 0; dh < 2; ++dh) oacc[dh] = MFMA32(frag_tr(Vs, 32 * i + 16 * kk, 32 * dh, lane), pf, oacc[dh]);
      }
  }
  float lt = l + __shfl_xor(l, 32, 64);
  if (qi < S) {
    float inv = 1.f / lt;
    bf16_t* op = o + ((size_t)b * S + qi) * d + h * 64;
#pragma unroll
    for (int dh = 0; dh < 2; ++dh)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        bf16x4 w;
#pragma unroll
        for (int j = 0; j < 4; ++j) w[j] = (bf16_t)(oacc[dh][4 * g + j] * inv);
        *reinterpret_cast<bf16x4*>(op + 32 * dh + 8 * g + 4 * hf) = w;
      }
    if (hf == 0) lse[((size_t)b * H + h) * S + qi] = (m + log2f(lt)) * kLn2;
  }
}

// ================================================================================= backward: dQ
__global__ void __launch_bounds__(256, 2) k_attn_bwd_dq_mfma(const bf16_t* __restrict__ qkv, const bf16_t* __restrict__ o,
                                                          const float* __restrict__ lse,
                                                          const bf16_t* __restrict__ dout, bf16_t* __restrict__ dqkv,
                                                          float* __restrict__ delta, int S, int H, int BH, int causal) {
  __shared__ __attribute__((aligned(16))) bf16_t Ks[64][ALD];
  __shared__ __attribute__((aligned(16))) bf16_t Vs[64][ALD];
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), n = lane & 31, hf = lane >> 5;
  const AttnBlock ab = attn_block(H, BH, (S + 127) / 128, causal != 0);
  const int bx = ab.x;
  const int h = ab.h, b = ab.b, d = H * 64;
  const size_t ld = (size_t)3 * d;
  const bf16_t* base = qkv + (size_t)b * S * ld;
  const int q0 = bx * 128 + wave * 32, qi = q0 + n;
  bf16x8 qf[4], dof[4];
  float D = 0.f, lse2 = 0.f;
#pragma unroll
  for (int kk = 0; kk < 4; ++kk) {
    if (qi < S) {
      qf[kk] = *reinterpret_cast<const bf16x8*>(base + (size_t)qi * ld + h * 64 + 16 * kk + 8 * hf);
      size_t off = ((size_t)b * S + qi) * d + h * 64 + 16 * kk + 8 * hf;
      dof[kk] = *reinterpret_cast<const bf16x8*>(dout + off);
      bf16x8 ov = *reinterpret_cast<const bf16x8*>(o + off);
#pragma unroll
      for (int e = 0; e < 8; ++e) D += (float)dof[kk][e] * (float)ov[e];
    } else {
      qf[kk] = zero8(); dof[kk] = zero8();
    }
  }
  D += __shfl_xor(D, 32, 64);
  if (qi < S) {
    size_t si = ((size_t)b * H + h) * S + qi;
    lse2 = lse[si] * kLog2e;
    if (hf == 0) delta[si] = D;
  }
  f32x16 dqa[2];
  zero16(dqa[0]); zero16(dqa[1]);
  const float scale = 0.125f, c = 0.125f * kLog2e;
  int q_hi = bx * 128 + 127;
  if (q_hi > S - 1) q_hi = S - 1;
  const int n_tiles = causal ? q_hi / 64 + 1 : (S + 63) / 64;
  TileRegs kr = load_tile(base + d + h * 64, ld, 0, S), vr = load_tile(base + 2 * d + h * 64, ld, 0, S);
  for (int jt = 0; jt < n_tiles; ++jt) {
    const int k0 = jt * 64;
    __syncthreads();
    store_tile(kr, Ks);
    store_tile(vr, Vs);
    __syncthreads();
    if (jt + 1 < n_tiles) {
      kr = load_tile(base + d + h * 64, ld, k0 + 64, S);
      vr = load_tile(base + 2 * d + h * 64, ld, k0 + 64, S);
    }
    const bool active = q0 < S && (!causal || k0 <= q0 + 31);
    if (!active) continue;
    f32x16 st[2], dp[2];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      zero16(st[i]); zero16(dp[i]);
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) {
        bf16x8 kf = *reinterpret_cast<const bf16x8*>(&Ks[32 * i + n][16 * kk + 8 * hf]);
        bf16x8 vf = *reinterpret_cast<const bf16x8*>(&Vs[32 * i + n][16 * kk + 8 * hf]);
        st[i] = MFMA32(kf, qf[kk], st[i]);
        dp[i] = MFMA32(vf, dof[kk], dp[i]);
      }
    }
    const bool need_mask = k0 + 63 >= S || q0 + 31 >= S || (causal && k0 + 63 > q0);   // wave-uniform
    if (need_mask) {
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          int kj = k0 + 32 * i + 8 * (v / 4) + 4 * hf + (v % 4);
          bool masked = kj >= S || qi >= S || (causal && kj > qi);
          float p = __builtin_amdgcn_exp2f(st[i][v] * c - lse2);
          st[i][v] = masked ? 0.f : p * (dp[i][v] - D);
        }
    } else {
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          float p = __builtin_amdgcn_exp2f(st[i][v] * c - lse2);
          st[i][v] = p * (dp[i][v] - D);        // the factor 1/sqrt(64) of dS is applied once, to the finished dQ
        }
    }
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int kk = 0; kk < 2; ++kk) {
        bf16x8 dsf = pack8(st[i], kk);
#pragma unroll
        for (int dh = 0; dh < 2; ++dh) dqa[dh] = MFMA32(frag_tr(Ks, 32 * i + 16 * kk, 32 * dh, lane), dsf, dqa[dh]);
      }
  }
  if (qi < S) {
    bf16_t* dqp = dqkv + ((size_t)b * S + qi) * ld + h * 64;
#pragma unroll
    for (int dh = 0; dh < 2; ++dh)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        bf16x4 w;
#pragma unroll
        for (int j = 0; j < 4; ++j) w[j] = (bf16_t)(dqa[dh][4 * g + j] * scale);
        *reinterpret_cast<bf16x4*>(dqp + 32 * dh + 8 * g + 4 * hf) = w;
      }
  }
}

// ================================================================================= backward: dK, dV
__global__ void __launch_bounds__(256, 2) k_attn_bwd_dkv_mfma(const bf16_t* __restrict__ qkv,
                                                           const float* __restrict__ lse,
                                                           const float* __restrict__ delta,
                                                           const bf16_t* __restrict__ dout,
                                                           bf16_t* __restrict__ dqkv, int S, int H, int BH, int causal) {
  __shared__ __attribute__((aligned(16))) bf16_t Qs[64][ALD];
  __shared__ __attribute__((aligned(16))) bf16_t dOs[64][ALD];
  __shared__ __attribute__((aligned(16))) float lse2s[64];
  __shared__ __attribute__((aligned(16))) float deltas[64];
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), n = lane & 31, hf = lane >> 5;
  const AttnBlock ab = attn_block(H, BH, (S + 127) / 128, false);
  const int bx = ab.x;
  const int h = ab.h, b = ab.b, d = H * 64;
  const size_t ld = (size_t)3 * d;
  const bf16_t* base = qkv + (size_t)b * S * ld;
  const bf16_t* dob = dout + (size_t)b * S * d;
  const int k0w = bx * 128 + wave * 32, kj = k0w + n;
  bf16x8 kf[4], vf[4];
#pragma unroll
  for (int kk = 0; kk < 4; ++kk) {
    if (kj < S) {
      const bf16_t* kp = base + (size_t)kj * ld + d + h * 64 + 16 * kk + 8 * hf;
      kf[kk] = *reinterpret_cast<const bf16x8*>(kp);
      vf[kk] = *reinterpret_cast<const bf16x8*>(kp + d);
    } else {
      kf[kk] = zero8(); vf[kk] = zero8();
    }
  }
  f32x16 dka[2], dva[2];
  zero16(dka[0]); zero16(dka[1]); zero16(dva[0]); zero16(dva[1]);
  const float scale = 0.125f, c = 0.125f * kLog2e;
  const int t_begin = causal ? (bx * 128) / 64 : 0;
  const int t_end = (S + 63) / 64;
  TileRegs qr = load_tile(base + h * 64, ld, t_begin * 64, S), dor = load_tile(dob + h * 64, (size_t)d, t_begin * 64, S);
  for (int it = t_begin; it < t_end; ++it) {
    const int q0 = it * 64;
    __syncthreads();
    store_tile(qr, Qs);
    store_tile(dor, dOs);
    if (it + 1 < t_end) {
      qr = load_tile(base + h * 64, ld, q0 + 64, S);
      dor = load_tile(dob + h * 64, (size_t)d, q0 + 64, S);
    }
    if (threadIdx.x < 64) {
      int q = q0 + threadIdx.x;
      size_t si = ((size_t)b * H + h) * S + q;
      lse2s[threadIdx.x] = q < S ? lse[si] * kLog2e : 0.f;
      deltas[threadIdx.x] = q < S ? delta[si] : 0.f;
    }
    __syncthreads();
    const bool active = k0w < S && (!causal || q0 + 63 >= k0w);
    if (!active) continue;
    // the mask matters only where this wave's keys reach the tile's queries or either runs off the end
    const bool need_mask = q0 + 63 >= S || k0w + 31 >= S || (causal && k0w + 31 > q0);
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      f32x16 s, dp;
      zero16(s); zero16(dp);
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) {
        bf16x8 qa = *reinterpret_cast<const bf16x8*>(&Qs[32 * i + n][16 * kk + 8 * hf]);
        bf16x8 da = *reinterpret_cast<const bf16x8*>(&dOs[32 * i + n][16 * kk + 8 * hf]);
        s = MFMA32(qa, kf[kk], s);
        dp = MFMA32(da, vf[kk], dp);
      }
      // wave-uniform: the masked form only on tiles that touch the diagonal or the end of the sequence
      if (need_mask) {
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          f32x4 l4 = *reinterpret_cast<const f32x4*>(&lse2s[32 * i + 8 * g + 4 * hf]);
          f32x4 d4 = *reinterpret_cast<const f32x4*>(&deltas[32 * i + 8 * g + 4 * hf]);
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            int v = 4 * g + j;
            float p = __builtin_amdgcn_exp2f(s[v] * c - l4[j]);
            int qrow = q0 + 32 * i + 8 * g + 4 * hf + j;
            bool masked = qrow >= S || kj >= S || (causal && kj > qrow);
            p = masked ? 0.f : p;
            s[v] = p;
            dp[v] = p * (dp[v] - d4[j]);
          }
        }
      } else {
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          f32x4 l4 = *reinterpret_cast<const f32x4*>(&lse2s[32 * i + 8 * g + 4 * hf]);
          f32x4 d4 = *reinterpret_cast<const f32x4*>(&deltas[32 * i + 8 * g + 4 * hf]);
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            int v = 4 * g + j;
            float p = __builtin_amdgcn_exp2f(s[v] * c - l4[j]);
            s[v] = p;
            dp[v] = p * (dp[v] - d4[j]);          // the factor 1/sqrt(64) of dS is applied once, to the finished dK
          }
        }
      }
#pragma unroll
      for (int kk = 0; kk < 2; ++kk) {
        bf16x8 pf = pack8(s, kk), dsf = pack8(dp, kk);
#pragma unroll
        for (int dh = 0; dh < 2; ++dh) {
          dva[dh] = MFMA32(frag_tr(dOs, 32 * i + 16 * kk, 32 * dh, lane), pf, dva[dh]);
          dka[dh] = MFMA32(frag_tr(Qs, 32 * i + 16 * kk, 32 * dh, lane), dsf, dka[dh]);
        }
      }
    }
  }
  if (kj < S) {
    bf16_t* dkp = dqkv + ((size_t)b * S + kj) * ld + d + h * 64;
    bf16_t* dvp = dkp + d;
#pragma unroll
    for (int dh = 0; dh < 2; ++dh)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        bf16x4 wk, wv;
#pragma unroll
        for (int j = 0; j < 4; ++j) { wk[j] = (bf16_t)(dka[dh][4 * g + j] * scale); wv[j] = (bf16_t)dva[dh][4 * g + j]; }
        *reinterpret_cast<bf16x4*>(dkp + 32 * dh + 8 * g + 4 * hf) = wk;
        *reinterpret_cast<bf16x4*>(dvp + 32 * dh + 8 * g + 4 * hf) = wv;
      }
  }
}

hipError_t attn_fwd_mfma(const OpCtx& c, const void* qkv, void* o, float* lse, int B, int S, int H, int causal) {
  if (B * S == 0) return hipSuccess;
  const int grid = ((S + 127) / 128) * H * B;
  k_attn_fwd_mfma<<<grid, 256, 0, c.stream>>>((const bf16_t*)qkv, (bf16_t*)o, lse, S, H, H * B, causal);
  return hipGetLastError();
}
hipError_t attn_bwd_mfma(const OpCtx& c, const void* qkv, const void* o, const float* lse, const void* dout,
                         void* dqkv, float* delta, int B, int S, int H, int causal) {
  if (B * S == 0) return hipSuccess;
  const int grid = ((S + 127) / 128) * H * B;
  k_attn_bwd_dq_mfma<<<grid, 256, 0, c.stream>>>((const bf16_t*)qkv, (const bf16_t*)o, lse, (const bf16_t*)dout,
                                                 (bf16_t*)dqkv, delta, S, H, H * B, causal);
  k_attn_bwd_dkv_mfma<<<grid, 256, 0, c.stream>>>((const bf16_t*)qkv, lse, delta, (const bf16_t*)dout, (bf16_t*)dqkv,
                                                  S, H, H * B, causal);
  return hipGetLastError();
}

}  // namespace lp
