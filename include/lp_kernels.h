/*
 * lp_kernels.h -- kernel-level C ABI: the individual HIP ops the local-update step is made of,
 * callable on caller-owned DEVICE buffers.  Used by the per-kernel parity tests and by the bench's
 * per-kernel roofline measurements.  Every call enqueues on `stream` (a hipStream_t, NULL = default)
 * and returns 0 or a nonzero hipError_t code; nothing is allocated.  `dtype` is the compute dtype
 * (0 = fp32, 1 = bf16) of activations and matrix operands; gradients of parameters, statistics and
 * optimizer state are fp32.  `scratch_dev` is fp32 workspace for two-stage reductions
 * (scratch_elems floats; a call that needs more fails with hipErrorInvalidValue).
 */
#ifndef LP_KERNELS_H_
#define LP_KERNELS_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* C[M,N] (+)= sum_k A(m,k) B(n,k) followed by the fused epilogue
 *   v (+= bias[n]); pre[m,n] = v; v = act(v); v *= act'(dact_src[m,n]); v += res[m,n].
 * A(m,k) = a_kc ? A[m*lda+k] : A[k*lda+m]; B(n,k) = b_kc ? B[n*ldb+k] : B[k*ldb+n]  (the forward, dgrad
 * and wgrad forms of a linear layer: paper appendix A, "MLP").  act / dact: 0 none, 1 ReLU, 2 GELU(tanh).
 * variant: 0 lets the library choose the kernel; 1 forces the FMA kernel; for bf16, 2 forces the
 * register-staged MFMA kernel, 3 / 4 the direct-to-LDS kernel with 256 x 128 tiles and the last partial wave
 * of tiles computed whole / cut along k, 5 / 6 the same with 256 x 256 tiles and 8 wavefronts, 7 / 8 with
 * 256 x 256 tiles and 4 wavefronts; 9 / 10 / 11 those three tile shapes in panel mode (outputs 2..8 tiles
 * wide: the tile columns of one tile row walk the same cut of the reduction together, so that the other
 * operand is fetched once per row); 20 / 21 / 22 the 8-wavefront 256 x 256 shape with 64-deep k-tiles (K a
 * multiple of 64), tail whole / cut along k / panel mode; an error if the shape does not qualify (K % 32 != 0, no workspace for
 * a cut, an output too narrow or too wide or a reduction too short for panel mode).  splitk_ws_dev (may be NULL) is fp32 workspace of
 * splitk_ws_elems floats: with it, reductions over few output tiles are split along k and the partial sums
 * added in a fixed order (at most max(8 * M * N, 2^25) floats are used). */
int lpk_gemm(int dtype, const void* A, int64_t lda, int a_kc, const void* B, int64_t ldb, int b_kc, void* C,
             int64_t ldc, int c_f32, int M, int N, int K, const float* bias, int act, void* pre,
             const void* dact_src, int dact, int64_t ldd, const void* res, int64_t ldr, int accumulate, int variant,
             float* splitk_ws_dev, size_t splitk_ws_elems, void* stream);

/* n (2..16) independent bf16 products C_i[M_i, N_i] (+)= epilogue(sum_k A_i(m,k) B_i(n,k)) with one reduction length K
 * (a multiple of 32) and one pair of operand layouts, in ONE persistent launch: the weight gradients of the linear
 * maps of one layer, or the same-shaped products of independent blocks (section 3: blocks are trained in
 * parallel; section 6), each of which alone has too few output tiles for the chip.  Every array is a HOST array of
 * n entries holding DEVICE pointers, leading dimensions and sizes (M_i, N_i multiples of 8).  Outputs are fp32
 * (c_f32) or bf16; per problem an optional bias (fp32 [N_i]) and an optional residual (bf16 [M_i, N_i], leading
 * dimension ldc_i), `bias` and `res` may be NULL; act as in lpk_gemm, common to all.  The tiles of all products form
 * one sequence that is spread over the grid like a single product's; its last partial wave is cut along k through
 * splitk_ws_dev (at least 2^25 floats).  hipErrorInvalidValue, with nothing launched, if the set does not qualify. */
int lpk_gemm_grouped(int n, const void* const* A, const int64_t* lda, const void* const* B, const int64_t* ldb,
                     void* const* C, const int64_t* ldc, int c_f32, const int* M, const int* N, int K, int a_kc,
                     int b_kc, const float* const* bias, int act, const void* const* res, int accumulate,
                     float* splitk_ws_dev, size_t splitk_ws_elems, void* stream);

/* Causal (or full) multi-head attention of a decoder layer (appendix B.2).  qkv [B*S, 3*H*dh]
 * (q | k | v), o [B*S, H*dh], lse [B,H,S] = log-sum-exp of the scaled scores, delta [B,H,S] scratch. */
int lpk_attention_fwd(int dtype, const void* qkv, void* o, float* lse, int B, int S, int H, int dh, int causal,
                      int plain, void* stream);
int lpk_attention_bwd(int dtype, const void* qkv, const void* o, const float* lse, const void* dout, void* dqkv,
                      float* delta, int B, int S, int H, int dh, int causal, int plain, void* stream);

/* LayerNorm over the last dimension (eps 1e-5, biased variance); backward adds `add` to dx if given. */
int lpk_layernorm_fwd(int dtype, const void* x, const float* g, const float* b, void* y, float* mean, float* rstd,
                      int rows, int d, void* stream);
int lpk_layernorm_bwd(int dtype, const void* dy, const void* x, const float* mean, const float* rstd,
                      const float* g, const void* add, void* dx, float* dg, float* db, int rows, int d,
                      int accumulate, float* scratch_dev, size_t scratch_elems, void* stream);

/* lpk_layernorm_bwd for callers that cannot allocate device memory or bring a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments and results as
 * lpk_layernorm_bwd without the scratch pair: the partial sums of dg and db go through an array built into
 * the library (LPK_STATIC_SCRATCH_FLOATS floats = 8 MiB, held on every GPU the library runs on until the
 * process ends).  Nothing is allocated or freed.  hipErrorInvalidValue (and a line on stderr) if
 * ((rows + 7) / 8) * d * 2 exceeds LPK_STATIC_SCRATCH_FLOATS; 8192 rows of width 1024 just fit.  All calls on
 * one GPU share the array, whatever their stream: calls that overlap in time on one GPU race, so order them on
 * one stream or with events.  The array keeps the last call's partial sums; a call reads only what it wrote. */
#define LPK_STATIC_SCRATCH_FLOATS (1u << 21)
int lpk_layernorm_bwd_static(int dtype, const void* dy, const void* x, const float* mean, const float* rstd,
                             const float* g, const void* add, void* dx, float* dg, float* db, int rows, int d,
                             int accumulate, void* stream);

/* Row-wise softmax cross-entropy (the auxiliary objective, section 3): loss_rows[r] = lse(z_r) - z[r,y_r];
 * with write_grad, z is overwritten by (softmax(z_r) - onehot(y_r)) * inv_rows. */
int lpk_softmax_ce(int dtype, void* z, int64_t ld, const int32_t* y, float* loss_rows, int rows, int n,
                   int write_grad, float inv_rows, void* stream);

/* Fused optimizer update over a flat range (kind 0 SGD, 1 SGD-momentum, 2 Adam; appendix B lists the
 * optimizers); n must be a multiple of 4; p_bf16 (may be NULL) receives the bf16 working copy. */
int lpk_optimizer(int kind, float lr, float momentum, float beta1, float beta2, float eps, float weight_decay,
                  int t, float grad_scale, float* p, const float* g, float* m, float* v, void* p_bf16, size_t n,
                  void* stream);

/* Plain device-to-device copy of `bytes` bytes (a multiple of 16; both pointers 16-byte aligned), one
 * 16-byte load and store per lane.  Not part of the method: it is the kernel of known traffic against
 * which the HBM counters (FETCH_SIZE, WRITE_SIZE) are scaled when a kernel's traffic is measured. */
int lpk_copy(const void* src_dev, void* dst_dev, size_t bytes, void* stream);

/* dst[C][R] = transpose of src[R][C], bf16 (R and C multiples of 8, both pointers 16-byte aligned).  Keeps the
 * [in][out] copy of a vocabulary head's weight [out][in] with which the head's input-gradient GEMM
 * (section 3: the backward pass inside a block) has the reduction index fastest in both operands. */
int lpk_transpose_bf16(const void* src_dev, void* dst_dev, int R, int C, void* stream);

/* Embedding-table gradient: demb[v,:] (+)= sum of dh[t,:] over positions with ids[t] == v, in order of t
 * (ids outside [0, V) count as the nearest valid id, as in the forward lookup).  scratch_dev (may be NULL)
 * is device scratch of scratch_elems 4-byte words; with at least V words the kernel first counts every
 * id's positions there and skips the rows that do not occur. */
int lpk_embed_bwd(int dtype, const int32_t* ids, const void* dh, float* demb, int T, int V, int d, int accumulate,
                  float* scratch_dev, size_t scratch_elems, void* stream);

/* NHWC convolution with [O,R,S,C] filters as implicit GEMM (appendix B.3), forward / data gradient /
 * filter gradient (fp32). */
int lpk_conv_fwd(int dtype, const void* x, const void* w, void* out, int N, int H, int W, int C, int O, int R,
                 int stride, int pad, void* stream);
int lpk_conv_bwd_data(int dtype, const void* dout, const void* w, void* dx, int N, int H, int W, int C, int O, int R,
                      int stride, int pad, void* stream);
int lpk_conv_bwd_weight(int dtype, const void* dout, const void* x, float* dw, int N, int H, int W, int C, int O,
                        int R, int stride, int pad, int accumulate, void* stream);
/* The same filter gradient with fp32 workspace (device memory, splitk_ws_elems floats, contents undefined on
 * return): with it the reduction over the N*P*Q output pixels is cut into pieces whose partial sums are added in a
 * fixed order, which is how the step computes it; a 3-channel stem with 64 output channels then takes one image per
 * block (needs N*O*R*R*C floats).  Without enough workspace the call computes the gradient uncut. */
int lpk_conv_bwd_weight_ws(int dtype, const void* dout, const void* x, float* dw, int N, int H, int W, int C, int O,
                           int R, int stride, int pad, int accumulate, float* splitk_ws_dev, size_t splitk_ws_elems,
                           void* stream);

/* One convolution + normalisation unit of a ResNet stage, forward (appendix B.3): z = conv(x, w) as lpk_conv_fwd,
 * then y = [relu](bn(z) (+ res)) as lpk_batchnorm_fwd, with z, y, mean, rstd all written.  Where the convolution's
 * output is whole tiles of the matrix-core kernel, the convolution itself leaves the per-channel sums of its rounded
 * outputs in scratch_dev and the normalisation does not read z for its statistics; otherwise the two run as the
 * separate calls would.  scratch_dev: at least max(3 * (N*P*Q/32 + O), (2*1024 + 2) * O) floats. */
int lpk_conv_bn_fwd(int dtype, const void* x, const void* w, void* z, const float* g, const float* b, const void* res,
                    void* y, float* mean, float* rstd, int N, int H, int W, int C, int O, int R, int stride, int pad,
                    int relu, float* scratch_dev, size_t scratch_elems, void* stream);

/* BatchNorm with batch statistics over rows = N*H*W, fused residual add and ReLU. */
int lpk_batchnorm_fwd(int dtype, const void* z, const float* g, const float* b, const void* res, void* y,
                      float* mean, float* rstd, int rows, int C, int relu, float* scratch_dev, size_t scratch_elems,
                      void* stream);
int lpk_batchnorm_bwd(int dtype, const void* dy, const void* y, const void* z, const float* mean, const float* rstd,
                      const float* g, void* dz, void* dres, float* dg, float* db, int rows, int C, int relu,
                      int accumulate, float* scratch_dev, size_t scratch_elems, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* LP_KERNELS_H_ */
