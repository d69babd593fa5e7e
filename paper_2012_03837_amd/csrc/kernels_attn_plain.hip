// Plain causal attention (one thread per query / key row, online softmax, fp32 arithmetic).  It is
// the fp32 compute path's attention and the fallback for head sizes the MFMA kernel does not take.
// Layout: qkv is [B*S, 3*H*dh] with q | k | v side by side and head h at columns h*dh..; o is
// [B*S, H*dh]; lse (log-sum-exp of the scaled scores) is [B, H, S].
#include "common.h"

namespace lp {

template <typename T, int DH>
__global__ void __launch_bounds__(64) k_attn_fwd_plain(const T* qkv, T* o, float* lse, int S, int H, int causal) {
  int i = blockIdx.x * 64 + threadIdx.x;
  int h = blockIdx.y, b = blockIdx.z;
  if (i >= S) return;
  int d = H * DH;
  size_t ld = (size_t)3 * d;
  const T* qp = qkv + ((size_t)b * S + i) * ld + h * DH;
  float q[DH], acc[DH];
  float scale = rsqrtf((float)DH);
#pragma unroll
  for (int c = 0; c < DH; ++c) { q[c] = to_f(qp[c]) * scale; acc[c] = 0.f; }
  float m = -INFINITY, l = 0.f;
  int jend = causal ? i + 1 : S;
  for (int j = 0; j < jend; ++j) {
    const T* kp = qkv + ((size_t)b * S + j) * ld + d + h * DH;
    const T* vp = kp + d;
    float s = 0.f;
#pragma unroll
    for (int c = 0; c < DH; ++c) s += q[c] * to_f(kp[c]);
    float mn = fmaxf(m, s);
    float corr = __expf(m - mn), p = __expf(s - mn);
    l = l * corr + p;
#pragma unroll
    for (int c = 0; c < DH; ++c) acc[c] = acc[c] * corr + p * to_f(vp[c]);
    m = mn;
  }
  T* op = o + ((size_t)b * S + i) * d + h * DH;
  float inv = 1.f / l;
#pragma unroll
  for (int c = 0; c < DH; ++c) op[c] = from_f<T>(acc[c] * inv);
  lse[((size_t)b * H + h) * S + i] = m + __logf(l);
}

// dq and delta_i = sum_c do_i[c] o_i[c]; one thread per query row.
template <typename T, int DH>
__global__ void __launch_bounds__(64) k_attn_bwd_q_plain(const T* qkv, const T* o, const float* lse, const T* dout,
                                                         T* dqkv, float* delta, int S, int H, int causal) {
  int i = blockIdx.x * 64 + threadIdx.x;
  int h = blockIdx.y, b = blockIdx.z;
  if (i >= S) return;
  int d = H * DH;
  size_t ld = (size_t)3 * d;
  size_t row = (size_t)b * S + i;
  const T* qp = qkv + row * ld + h * DH;
  const T* dop = dout + row * d + h * DH;
  const T* op = o + row * d + h * DH;
  float q[DH], go[DH], dq[DH];
  float scale = rsqrtf((float)DH);
  float D = 0.f;
#pragma unroll
  for (int c = 0; c < DH; ++c) {
    q[c] = to_f(qp[c]); go[c] = to_f(dop[c]); dq[c] = 0.f;
    D += go[c] * to_f(op[c]);
  }
  float L = lse[((size_t)b * H + h) * S + i];
  int jend = causal ? i + 1 : S;
  for (int j = 0; j < jend; ++j) {
    const T* kp = qkv + ((size_t)b * S + j) * ld + d + h * DH;
    const T* vp = kp + d;
    float s = 0.f, dp = 0.f;
#pragma unroll
    for (int c = 0; c < DH; ++c) { s += q[c] * to_f(kp[c]); dp += go[c] * to_f(vp[c]); }
    float p = __expf(s * scale - L);
    float ds = p * (dp - D) * scale;
#pragma unroll
    for (int c = 0; c < DH; ++c) dq[c] += ds * to_f(kp[c]);
  }
  T* dqp = dqkv + row * ld + h * DH;
#pragma unroll
  for (int c = 0; c < DH; ++c) dqp[c] = from_f<T>(dq[c]);
  delta[((size_t)b * H + h) * S + i] = D;
}

// dk, dv; one thread per key row, queries visited in increasing order.
template <typename T, int DH>
__global__ void __launch_bounds__(64) k_attn_bwd_kv_plain(const T* qkv, const float* lse, const float* delta,
                                                          const T* dout, T* dqkv, int S, int H, int causal) {
  int j = blockIdx.x * 64 + threadIdx.x;
  int h = blockIdx.y, b = blockIdx.z;
  if (j >= S) return;
  int d = H * DH;
  size_t ld = (size_t)3 * d;
  size_t row = (size_t)b * S + j;
  const T* kp = qkv + row * ld + d + h * DH;
  const T* vp = kp + d;
  float k[DH], v[DH], dk[DH], dv[DH];
  float scale = rsqrtf((float)DH);
#pragma unroll
  for (int c = 0; c < DH; ++c) { k[c] = to_f(kp[c]); v[c] = to_f(vp[c]); dk[c] = 0.f; dv[c] = 0.f; }
  int ibeg = causal ? j : 0;
  for (int i = ibeg; i < S; ++i) {
    size_t ri = (size_t)b * S + i;
    const T* qp = qkv + ri * ld + h * DH;
    const T* dop = dout + ri * d + h * DH;
    float s = 0.f, dp = 0.f;
#pragma unroll
    for (int c = 0; c < DH; ++c) { s += to_f(qp[c]) * k[c]; dp += to_f(dop[c]) * v[c]; }
    size_t si = ((size_t)b * H + h) * S + i;
    float p = __expf(s * scale - lse[si]);
    float ds = p * (dp - delta[si]) * scale;
#pragma unroll
    for (int c = 0; c < DH; ++c) { dv[c] += p * to_f(dop[c]); dk[c] += ds * to_f(qp[c]); }
  }
  T* dkp = dqkv + row * ld + d + h * DH;
  T* dvp = dkp + d;
#pragma unroll
  for (int c = 0; c < DH; ++c) { dkp[c] = from_f<T>(dk[c]); dvp[c] = from_f<T>(dv[c]); }
}

template <typename T, int DH>
static hipError_t fwd_t(const OpCtx& c, const void* qkv, void* o, float* lse, int B, int S, int H, int causal) {
  dim3 grid((S + 63) / 64, H, B);
  k_attn_fwd_plain<T, DH><<<grid, 64, 0, c.stream>>>((const T*)qkv, (T*)o, lse, S, H, causal);
  return hipGetLastError();
}
template <typename T, int DH>
static hipError_t bwd_t(const OpCtx& c, const void* qkv, const void* o, const float* lse, const void* dout,
                        void* dqkv, float* delta, int B, int S, int H, int causal) {
  dim3 grid((S + 63) / 64, H, B);
  k_attn_bwd_q_plain<T, DH><<<grid, 64, 0, c.stream>>>((const T*)qkv, (const T*)o, lse, (const T*)dout, (T*)dqkv,
                                                      delta, S, H, causal);
  k_attn_bwd_kv_plain<T, DH><<<grid, 64, 0, c.stream>>>((const T*)qkv, lse, delta, (const T*)dout, (T*)dqkv, S, H,
                                                       causal);
  return hipGetLastError();
}

#define LP_DH_SWITCH(T, CALL)                                  \
  switch (dh) {                                                \
    case 4: return CALL(T, 4);                                 \
    case 8: return CALL(T, 8);                                 \
    case 16: return CALL(T, 16);                               \
    case 32: return CALL(T, 32);                               \
    case 64: return CALL(T, 64);                               \
    default: return hipErrorInvalidValue;                      \
  }

hipError_t attn_fwd_plain(const OpCtx& c, const void* qkv, void* o, float* lse, int B, int S, int H, int dh,
                          int causal) {
  if (B * S == 0) return hipSuccess;
#define F(T, D) fwd_t<T, D>(c, qkv, o, lse, B, S, H, causal)
  if (c.dt == BF16) { LP_DH_SWITCH(bf16_t, F) } else { LP_DH_SWITCH(float, F) }
#undef F
}
hipError_t attn_bwd_plain(const OpCtx& c, const void* qkv, const void* o, const float* lse, const void* dout,
                          void* dqkv, float* delta, int B, int S, int H, int dh, int causal) {
  if (B * S == 0) return hipSuccess;
#define G(T, D) bwd_t<T, D>(c, qkv, o, lse, dout, dqkv, delta, B, S, H, causal)
  if (c.dt == BF16) { LP_DH_SWITCH(bf16_t, G) } else { LP_DH_SWITCH(float, G) }
#undef G
}

}  // namespace lp
