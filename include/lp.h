/*
 * lp.h -- C ABI of the local-parallelism training step for AMD MI355X (gfx950).
 *
 * The library trains a deep network by *local updates* (paper section 3): the network is an
 * ordered list of atomic layers; a local-training scheme is a list of auxiliary heads, head j
 * attached after layer e_j, whose loss is backpropagated through the last w_j layers ending at
 * e_j and no further (the activation entering layer e_j - w_j + 1 is treated as data).  Greedy
 * local parallelism is one head per layer with w = 1; overlapping is w = 2; chunked is one head
 * every K layers with w = K; ordinary backpropagation is a single head with w = L; the
 * "last K layers" baseline is a single head with w = K.  Every parameter covered by at least one
 * window takes one optimizer update per step, as soon as its gradient is final; nothing waits for
 * a global backward pass.
 *
 * All pointers named *_dev are DEVICE pointers, all others are HOST pointers.  The caller owns
 * every device buffer and the HIP stream; the library owns only host metadata.  No entry point
 * throws or aborts: each returns an lp_status, and lp_last_error() gives the text.  Argument
 * errors are found on the host before anything is launched and leave the context unchanged.
 * One context may be used by one host thread at a time.
 */
#ifndef LP_H_
#define LP_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct lp_ctx lp_ctx; /* opaque */

typedef enum {
  LP_OK = 0,
  LP_EINVAL = 1,       /* null pointer, bad enum, window < 1, heads not ordered by layer, ...     */
  LP_ESHAPE = 2,       /* batch > max_batch, width not divisible by heads, unsupported size      */
  LP_EALIGN = 3,       /* a device buffer is not 256-byte aligned                                 */
  LP_ENOMEM = 4,       /* a device buffer is smaller than lp_query_sizes() asked for              */
  LP_EDEVICE = 5,      /* a HIP call failed (text in lp_last_error)                               */
  LP_ESTATE = 6,       /* context unusable (failed init, destroyed)                               */
  LP_EUNSUPPORTED = 7, /* valid request that this build does not implement                        */
  LP_ENOTFOUND = 8     /* unknown tensor name                                                     */
} lp_status;

typedef enum { LP_F32 = 0, LP_BF16 = 1 } lp_dtype; /* compute dtype; master weights, gradients and
                                                      optimizer state are always fp32 */
typedef enum { LP_I32 = 2 } lp_dtype_extra;        /* reported by lp_tensor_info for index data */

/* Atomic layer forms (appendix A "MLP", appendix B.2 "Transformers", appendix B.3 "ResNets"). */
typedef enum {
  LP_LAYER_RESMLP = 0,       /* p = x (or x Win^T + bin if in_dim != width);
                                out = p + W2 relu(W1 p + b1) + b2                                   */
  LP_LAYER_DECODER = 1,      /* pre-LN causal decoder layer: u = h + Wo attn(LN1 h); out = u + FFN(LN2 u) */
  LP_LAYER_RESNET_STAGE = 2  /* optional stem conv3x3+BN+ReLU, then n BasicBlocks (conv-BN-ReLU-conv-BN,
                                add shortcut, ReLU); first block strided with a 1x1 conv+BN shortcut */
} lp_layer_kind;

/* Auxiliary heads: same form as the global objective (section 3). */
typedef enum {
  LP_HEAD_LINEAR_CE = 0,      /* Linear(in_dim -> n_classes) + softmax cross-entropy              */
  LP_HEAD_POOL_LINEAR_CE = 1, /* mean over H x W, then Linear + CE                                 */
  LP_HEAD_LN_LINEAR_CE = 2,   /* LayerNorm, Linear to the vocabulary (no bias), next-token CE      */
  LP_HEAD_BN_POOL_LINEAR_CE = 3 /* BatchNorm (batch statistics), ReLU, mean over H x W, Linear + CE:
                                 the ResNet auxiliary head of appendix B.3                           */
} lp_head_kind;

typedef enum { LP_OPT_SGD = 0, LP_OPT_SGDM = 1, LP_OPT_ADAM = 2 } lp_opt_kind;
typedef enum { LP_COMBINE_SUM = 0, LP_COMBINE_MEAN = 1 } lp_combine;
typedef enum { LP_ACT_GELU = 0, LP_ACT_RELU = 1 } lp_act;
/* LP_SCHED_SYNC: every block works on the call's minibatch (one forward pass with the current weights).
 * LP_SCHED_PIPELINED: the steady-state pipeline of section 6 / section 3: block 1 works on the call's
 * minibatch, block j >= 2 on the activation that block j-1 produced in the previous call, with the labels
 * that travelled with it; blocks are then independent within a call.  Needs windows that tile the layers.
 * LP_SCHED_PIPELINED_GROUPED: the same schedule and the same results up to the order of floating-point sums; the
 * blocks of a call are walked in lockstep (stage s of every block before stage s + 1 of any) and the GEMMs of one
 * stage, one per block and of one shape, go out as grouped launches (two teams of blocks on two of the side streams
 * if there are any).  For decoder layers in blocks of equal depth with vocabulary heads: LP_EUNSUPPORTED otherwise.
 * Measured on one MI355X it costs the same per call as LP_SCHED_PIPELINED (independent chains over the side
 * streams): what the grouped products gain, the coarser interleaving of memory-bound and matrix kernels loses. */
typedef enum { LP_SCHED_SYNC = 0, LP_SCHED_PIPELINED = 1, LP_SCHED_PIPELINED_GROUPED = 2 } lp_schedule;

typedef struct {
  int kind;                 /* lp_layer_kind */
  int in_dim, width, hidden;                 /* resmlp: in, width, hidden.  decoder: width d, hidden F */
  int n_heads, seq_len, causal, act;         /* decoder */
  int in_ch, out_ch, stride, n_basic_blocks, has_stem, in_hw; /* resnet stage (square NHWC input) */
} lp_layer_spec;

typedef struct {
  int kind;                 /* lp_head_kind */
  int after_layer;          /* e_j, 1-based; heads must be listed with non-decreasing e_j          */
  int window;               /* w_j >= 1; clamped to e_j                                            */
  int in_dim, n_classes, bias;
} lp_head_spec;

typedef struct {
  int kind;                 /* lp_opt_kind */
  float lr, momentum, beta1, beta2, eps, weight_decay;
} lp_opt_spec;

typedef struct {
  int n_layers;
  const lp_layer_spec* layers;
  int n_heads;
  const lp_head_spec* heads;
  lp_opt_spec opt;
  int combine;              /* lp_combine: how the contributions of several heads to one layer merge
                               (the paper averages duplicated layers; a config may ask for the sum)  */
  int dtype;                /* lp_dtype */
  int max_batch;
  int vocab;                /* > 0: layer 1 owns a token embedding [vocab, width] + fixed sinusoidal
                               positions, and x is int32 token ids                                  */
  uint64_t seed;            /* seed of the built-in weight initialiser                              */
  int n_streams;            /* 0: everything on the caller's stream.  n > 0: each head's loss, in-window
                               backward pass and updates run on one of n side streams (the library creates
                               them, default priority) as soon as the head's activation exists, while the
                               forward pass continues on the caller's stream; all of them are joined back
                               into the caller's stream before lp_local_step returns.  Results do not depend
                               on n (every per-parameter accumulation keeps its order).  At most 8.        */
  int schedule;             /* lp_schedule: how lp_local_step feeds the blocks (see there)                 */
  int debug;                /* != 0: keep, for every convolution + normalisation unit of a ResNet stage, a copy of
                               the upstream gradient its backward pass was given and of the input gradient it
                               produced (named tensors "<unit>.dy", "<unit>.dx", see lp_get_tensor), so that a unit
                               can be checked in isolation; costs two activation-sized buffers per unit and two
                               copies per unit per step.  0 for training.                                   */
} lp_model_spec;

typedef struct { size_t param_bytes, state_bytes, work_bytes; } lp_sizes;
typedef struct { void* params_dev; void* state_dev; void* work_dev; } lp_buffers;

/* Sizes of the three caller-allocated device buffers for this model (host only, no HIP call).
 * params: fp32 master weights (+ a bf16 working copy when dtype is bf16); state: optimizer
 * moments; work: gradients, activations and scratch. */
int lp_query_sizes(const lp_model_spec* spec, lp_sizes* out);

/* Build a context over caller-allocated buffers (each 256-byte aligned and at least as large as
 * lp_query_sizes says), zero the optimizer state, and initialise the weights from spec->seed
 * (Kaiming-normal for MLP / conv / small heads, N(0, 0.02) for decoder layers and vocabulary
 * heads, gains 1, biases 0).  `hip_stream` is a hipStream_t (NULL = default stream); all later
 * work of this context is enqueued on it.  The spec is copied; the buffers are borrowed until
 * lp_destroy.  On failure *out is NULL. */
int lp_init_blocks(const lp_model_spec* spec, const lp_buffers* buffers, void* hip_stream, lp_ctx** out);

/* One local-update step on one minibatch (section 3): forward through all layers with the
 * current weights; for every head, its loss, the gradient inside its window only, and the
 * optimizer update of every covered parameter.  x_dev: fp32 [batch, in_dim] (resmlp), fp32 or bf16
 * NHWC [batch, H, W, C] in the compute dtype (resnet), int32 [batch, seq_len] token ids (decoder
 * with vocab).  y_dev: int32 [batch] class labels, or int32 [batch, seq_len] next-token targets.
 * losses_dev: fp32 [n_heads], head j's mean loss at the PRE-update weights.  Asynchronous: results
 * are valid once the context's stream has been synchronised.
 * With schedule LP_SCHED_PIPELINED, call t gives block 1 the minibatch (x, y) and block j >= 2 the output
 * of block j-1 from call t-1 (computed with the weights block j-1 had then) and minibatch t-j+1's labels;
 * each block runs forward, loss, in-block backward and its update (its optimizer step count is its own
 * number of updates).  A block whose input has not arrived yet (t < j) does nothing and reports loss 0.
 * x_dev and y_dev are copied where a later call needs them and may be reused after the call.  A call with
 * batch 0 does not advance the pipeline.  lp_eval_loss is the same in both schedules. */
int lp_local_step(lp_ctx* ctx, const void* x_dev, const int32_t* y_dev, int batch, float* losses_dev);

/* Forward pass and head losses only; no state changes.  (By default BatchNorm uses the statistics of the
 * batch given, so this equals the losses a step on the same batch would report; see lp_bn_running.) */
int lp_eval_loss(lp_ctx* ctx, const void* x_dev, const int32_t* y_dev, int batch, float* losses_dev);

/* Running statistics of batch normalisation (appendix B.3 normalises the ResNet blocks and their auxiliary
 * heads with the method of Ioffe & Szegedy; the paper does not say how it evaluates, so this is that method's
 * usual evaluation form).  Every lp_local_step folds the statistics of each batch normalisation it evaluates,
 * once, into that normalisation's running pair (fp32, in the state buffer, started at mean 0, variance 1):
 *   running_mean <- (1 - momentum) running_mean + momentum * mean_B
 *   running_var  <- (1 - momentum) running_var  + momentum * var_B * n / (n - 1),   n = batch * H * W.
 * momentum in [0, 1]; 0 keeps them as they are; the default is 0.1.  With eval_with_running != 0,
 * lp_eval_loss normalises with the running pair instead of the batch's own statistics (each sample is then
 * evaluated independently of the rest of its batch); the default is 0.  Steps always normalise with the batch.
 * The pairs are the named tensors "<prefix>.running_mean" / "<prefix>.running_var" for every gain tensor
 * "<prefix>.g" of a batch normalisation ("L1.stem.bn", "L2.b1.bn1", "H3.bn", ...).
 * LP_EINVAL for a momentum outside [0, 1]. */
int lp_bn_running(lp_ctx* ctx, float momentum, int eval_with_running);

/* Named tensors.  Parameters "L3.wqkv", "H2.w" (fp32 master; setting one also refreshes the bf16
 * working copy); their gradients of the last step "L3.wqkv.grad" and optimizer moments ".m", ".v"
 * (fp32); batch-normalisation running statistics "L2.b1.bn1.running_mean", ".running_var" (fp32); layer outputs of the last forward "L3.out" and the embedded input "L0.out" (compute
 * dtype, shaped for the batch of that call).  For every convolution + normalisation unit of a ResNet stage,
 * named like its filter without the ".w" ("L1.stem", "L2.b1.conv1", "L2.b1.conv2", "L2.b1.proj"): the stored
 * convolution output "<unit>.z" and the unit's output "<unit>.y" of the last forward pass (compute dtype, NHWC)
 * and, in a context created with spec.debug != 0, the upstream gradient "<unit>.dy" given to the unit's last
 * backward pass and the input gradient "<unit>.dx" it produced (including the shortcut's share where the
 * library adds it in the same kernel); LP_ENOTFOUND without the debug flag or when the unit computed none.  lp_tensor_info reports shape, lp_dtype and bytes.
 * get/set copy synchronously between host memory and the device after draining the stream;
 * `bytes` must equal the tensor's size. */
int lp_tensor_info(lp_ctx* ctx, const char* name, int64_t shape[4], int* ndim, int* dtype, size_t* bytes);
int lp_get_tensor(lp_ctx* ctx, const char* name, void* dst_host, size_t bytes);
int lp_set_tensor(lp_ctx* ctx, const char* name, const void* src_host, size_t bytes);
/* Number of parameter tensors, and the i-th name (storage order: layers, then heads). */
int lp_num_params(lp_ctx* ctx);
const char* lp_param_name(lp_ctx* ctx, int i);
/* Optimizer step counter t = number of lp_local_step calls so far (Adam bias correction uses t counted from 1;
 * with the pipelined schedule block j's own count is max(0, t - j + 1), which lp_set_step restores). */
int lp_get_step(lp_ctx* ctx);
int lp_set_step(lp_ctx* ctx, int t);

/* Replay of lp_local_step through a HIP graph, for configurations whose step is bound by kernel launches
 * rather than by the kernels (small blocks: the residual-MLP setting of section 4 on one GPU).  While on, the
 * first lp_local_step with given (x_dev, y_dev, batch, losses_dev) runs as usual, the second is captured
 * (side streams included) and launched as a graph, later ones with the same four arguments replay it; other
 * arguments start over.  The caller refills the same device buffers between steps.  Results are those of the
 * ordinary step, bit for bit.  Only for optimizers whose kernels take no per-step scalar (SGD, SGD with
 * momentum) and the synchronous schedule: LP_EINVAL otherwise.  Steps taken while per-kernel timing is
 * enabled, and lp_eval_loss, run as usual. */
int lp_step_graph(lp_ctx* ctx, int on);

/* Overlap of consecutive synchronous steps (section 6: updates are applied asynchronously and the blocks keep
 * working without a global barrier).  By default a call ends by making the caller's stream wait for every
 * block's chain, so whatever the caller enqueues next sees the finished step.  With overlap on, lp_local_step
 * leaves its chains running on the library's side streams and the next lp_local_step starts at once: its forward
 * pass of a layer waits only for the chains of the heads that read or update that layer, so the first layers of
 * step t+1 run beside the last blocks of step t.  Each step computes exactly what it computes without overlap
 * (bit for bit).  The price is a weaker contract: x_dev, y_dev and losses_dev of a call must stay untouched
 * (and losses_dev unread) until lp_join, or any entry point that takes the context other than lp_local_step,
 * lp_last_error, lp_num_params, lp_param_name and lp_destroy (which drains the side streams itself), has been
 * called on the context and the caller's stream has reached that point.  Needs side streams (n_streams > 0; otherwise it
 * has no effect); LP_EINVAL with the pipelined schedule or while graph replay is on. */
int lp_overlap_steps(lp_ctx* ctx, int on);
/* Makes the caller's stream wait for everything earlier calls left running (stream-ordered, does not block
 * the host).  A no-op unless steps are overlapped. */
int lp_join(lp_ctx* ctx);

/* Gradient similarity (section 5, "Gradient Angles"; Fig. 6a): out_dev[l-1] (device, n_layers floats) =
 * cosine of the angle between the gradients that the last lp_local_step of ctx_a and of ctx_b left for
 * layer l's parameters, all of the layer's tensors taken as one vector; 0 where either gradient is zero
 * (a layer outside every window).  The contexts must describe the same layers (their heads may differ:
 * e.g. greedy heads in one, a single head with a full window in the other).  Enqueued on ctx_a's stream
 * after ctx_b's stream has been drained. */
int lp_grad_cosine(lp_ctx* ctx_a, lp_ctx* ctx_b, float* out_dev);

/* Per-kernel-class timing.  While enabled, every op brackets its launches with a pair of HIP events
 * on the context's stream, and the side streams are not used (each duration is then the op's own, not
 * shared with a concurrent chain; results are bit-identical either way).  lp_profile_read drains the stream and returns, for one class, the summed
 * event time in ms, the number of ops launched and (for GEMM / convolution classes) the FLOPs
 * launched, all since profiling was last enabled.  Read after every step: the event pool holds 8192
 * pairs.  Enabling resets the totals. */
typedef enum {
  LP_KC_GEMM = 0, LP_KC_ATTN_FWD, LP_KC_ATTN_BWD, LP_KC_LAYERNORM, LP_KC_SOFTMAX_CE, LP_KC_OPTIMIZER, LP_KC_EMBED,
  LP_KC_COLSUM, LP_KC_CONV, LP_KC_BATCHNORM, LP_KC_OTHER,
  LP_KC_GEMM_KERNEL,   /* the main kernel launch of every bf16 GEMM op alone (see lp_profile_gemm_kernels) */
  LP_KC_COUNT
} lp_kernel_class;
int lp_profile_enable(lp_ctx* ctx, int on);
/* GEMM ops by shape since profiling was enabled, as text into the host buffer `out` of `cap` bytes, one
 * line per shape: "M N K a_kc b_kc c_f32 count total_ms" (operand layouts as in lpk_gemm).  LP_ESHAPE if
 * the buffer is too small. */
int lp_profile_gemm_shapes(lp_ctx* ctx, char* out, size_t cap);
/* The main kernel of every bf16 GEMM op (and of every convolution run as implicit GEMM) since profiling was enabled, grouped by kernel instance, as text into
 * the host buffer `out`: one line per instance, "name<TAB>launches<TAB>total_ms<TAB>algorithmic_flops", where the
 * name is the kernel's name as a profiler prints it ("k_gemm_dma<true, true, 4, 2, 4, true>") and the time is
 * that of the one launch (an event pair around it; the op's partial-sum fix-up kernel, if any, is outside).
 * LP_ESHAPE if the buffer is too small. */
int lp_profile_gemm_kernels(lp_ctx* ctx, char* out, size_t cap);
int lp_profile_read(lp_ctx* ctx, int kernel_class, double* total_ms, long long* launches, double* flops);

/* Text of the last error on this context (or of the last failed init when ctx is NULL); valid
 * until the next call. */
const char* lp_last_error(const lp_ctx* ctx);

/* Free host metadata.  Never frees caller memory. */
void lp_destroy(lp_ctx* ctx);

/* ---- FLOP cost model (appendix A, "Calculation of Total FLOPs and Sequential FLOPs") ----------------
 * Host arithmetic only; no device is touched.  A model is four numbers: average forward FLOPs per layer per
 * example, auxiliary-loss FLOPs per example, the backward multiplier, and its parameter count (the optimizer
 * costs 10 FLOPs per parameter per step; overlapping adds 2 per parameter for averaging duplicated layers).
 *   cost_per_example: backprop (1+bm)(L f + a); greedy (1+bm) L (f + a);
 *                     overlapping L (f + a) + (L-1) bm (2 f + a) + bm (f + a);
 *                     K chunks (1+bm)(L f + K a); last K layers (L f + a) + bm (K f + a)
 *   cost = cost_per_example * steps * batch + steps * per-step optimizer cost
 *   time = cost / (batch * parallelism), parallelism = 1, L, L, K, (L + K bm) / (K (1 + bm)) respectively.
 * (The chunk and last-K lines are printed damaged in the paper; these forms reduce to greedy at K = L and to
 * backprop at K = 1 resp. K = L, as the prose requires.)  K is ignored by the first three methods. */
typedef enum { LP_METHOD_BACKPROP = 0, LP_METHOD_GREEDY = 1, LP_METHOD_OVERLAP = 2, LP_METHOD_CHUNK = 3,
               LP_METHOD_LAST_K = 4 } lp_method;
typedef struct {
  double forward_cost;         /* average forward FLOPs per layer per example */
  double aux_cost;             /* FLOPs of one auxiliary loss per example */
  double backward_multiplier;
  double parameters;
  int layers;
} lp_cost_inputs;
typedef struct { double cost_per_example, cost, time, parallelism; } lp_cost;
/* LP_EINVAL on a null pointer, an unknown method, layers < 1, K outside [1, layers] for the chunk / last-K
 * methods, or non-positive steps / batch_size. */
int lp_cost_model(const lp_cost_inputs* in, int method, int K, double steps, double batch_size, lp_cost* out);
/* The MLP's constants (appendix A, "MLP"): layer = (2 I N - I) + N + 2 N with I = input_size for the first
 * layer and N after it, averaged over `layers`; auxiliary classifier = (2 N 10 - N) + 10 + 5*10. */
int lp_mlp_flops(int input_size, int hidden, int layers, double* forward_cost, double* aux_cost);

#ifdef __cplusplus
}
#endif
#endif /* LP_H_ */
