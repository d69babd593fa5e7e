// Epilogue shared by the GEMM kernels, and operand accessors for the plain (FMA) GEMM.
#pragma once
#include "common.h"

namespace lp {

struct Epilogue {
  const float* bias;
  int act;
  void* pre;
  const void* dact_src; int dact; int64_t ldd;
  const void* res; int64_t ldr;
  void* C; int64_t ldc; int c_f32; int accumulate;
};

static inline Epilogue make_epilogue(const GemmArgs& g) {
  Epilogue e;
  e.bias = g.bias; e.act = g.act; e.pre = g.pre;
  e.dact_src = g.dact_src; e.dact = g.dact; e.ldd = g.ldd;
  e.res = g.res; e.ldr = g.ldr;
  e.C = g.C; e.ldc = g.ldc; e.c_f32 = g.c_f32; e.accumulate = g.accumulate;
  return e;
}

// Applies the epilogue to one accumulator value and stores it.  T is the compute dtype.
template <typename T>
__device__ __forceinline__ void epilogue_store(const Epilogue& e, int m, int n, float v) {
  if (e.bias) v += e.bias[n];
  if (e.pre) reinterpret_cast<T*>(e.pre)[(size_t)m * e.ldc + n] = from_f<T>(v);
  if (e.act == ACT_RELU) v = fmaxf(v, 0.f);
  else if (e.act == ACT_GELU) v = gelu_f(v);
  if (e.dact != ACT_NONE) {
    float s = to_f(reinterpret_cast<const T*>(e.dact_src)[(size_t)m * e.ldd + n]);
    if (e.dact == ACT_RELU) v = s > 0.f ? v : 0.f;
    else v *= dgelu_f(s);
  }
  if (e.res) v += to_f(reinterpret_cast<const T*>(e.res)[(size_t)m * e.ldr + n]);
  size_t o = (size_t)m * e.ldc + n;
  if (e.c_f32) {
    float* c = reinterpret_cast<float*>(e.C);
    c[o] = e.accumulate ? c[o] + v : v;
  } else {
    T* c = reinterpret_cast<T*>(e.C);
    c[o] = from_f<T>(e.accumulate ? to_f(c[o]) + v : v);
  }
}

// Host-side description of how the direct-to-LDS GEMM spreads one problem over its persistent grid
// (filled by gemm_dma_plan, priced by the variant choice, consumed by gemm_dma).
struct DmaGemmPlan {
  int kind = 1;                      // 0: 256 x 128 tiles; 1: 256 x 256, 8 waves; 2: 256 x 256, 4 waves
  int tiles_m = 0, tiles_n = 0, kt = 0;
  int full = 0, tail_tiles = 0, upb = 0, G = 0;
  int sib = 0;                       // panel mode: tile columns that walk one panel's reduction together
  double partial_bytes = 0;          // fp32 partial sums written (and read again by the fix-up kernel)
  long steps = 0;                    // k-steps on the longest block
  int items = 0;                     // tiles or tile pieces on the longest block
};

}  // namespace lp
