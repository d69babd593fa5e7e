// Host-side context of the library: copied spec, parameter table, buffer layout, per-layer
// activation slots.  Nothing here is visible through the C ABI.
#pragma once

#include <map>
#include <string>
#include <vector>

#include "../../include/lp.h"
#include "common.h"

namespace lp {

struct Tensor {
  std::string name;
  int ndim = 0;
  int64_t shape[4] = {0, 0, 0, 0};
  size_t numel = 0;
  size_t off = 0;        // element offset in the flat parameter space (multiple of 64)
  int owner = 0;         // layer index 1..L, or L + head index (1-based)
  int init = 0;          // 0: normal(std), 1: ones, 2: zeros
  float std = 0.f;
};

// One convolution + BatchNorm unit of a ResNet stage.
struct ConvUnit {
  ConvArgs a;
  int w = -1, g = -1, b = -1;   // tensor indices: filter, BN gain, BN shift
  void* z = nullptr;            // conv output
  void* y = nullptr;            // BN (+res) (+ReLU) output
  float* mean = nullptr;
  float* rstd = nullptr;
  int relu = 0;
  // debug contexts only: copies of the upstream gradient of the last backward pass and of the input gradient
  void* dy_keep = nullptr;
  void* dx_keep = nullptr;
  bool dx_valid = false;
};
struct BasicBlock { ConvUnit c1, c2, proj; bool has_proj = false; };

struct LayerState {
  lp_layer_spec s;
  size_t p_begin = 0, p_end = 0;     // flat parameter range [begin, end)
  int coverage = 0;                  // number of heads whose window covers this layer
  int seen = 0;                      // contributions received so far in the current step
  void* out = nullptr;               // layer output (compute dtype)
  // Layers inside several windows (overlapping schemes): the sum of the heads' gradients with respect to this
  // layer's output, in the compute dtype.  The layer's parameter gradient is linear in that upstream gradient,
  // so one pass on the sum replaces one pass per head (null: every head runs its own full backward pass).
  void* gsum = nullptr;
  const void* in_override = nullptr; // pipelined schedule: this layer reads its input here (a block's first layer)
  size_t out_elems_per_sample = 0;
  // tensor indices (−1 if absent)
  std::map<std::string, int> t;
  // residual MLP
  void *mlp_p = nullptr, *mlp_r = nullptr;
  // decoder
  void *a = nullptr, *qkv = nullptr, *o = nullptr, *u = nullptr, *c = nullptr, *fpre = nullptr, *f = nullptr;
  float *mean1 = nullptr, *rstd1 = nullptr, *mean2 = nullptr, *rstd2 = nullptr, *lse = nullptr;
  lp::GemmArgs wg[4];                  // decoder: the weight-gradient products of the backward pass in flight
  // resnet stage
  bool has_stem = false;
  ConvUnit stem;
  std::vector<BasicBlock> blocks;
};

struct HeadState {
  lp_head_spec s;
  size_t p_begin = 0, p_end = 0;
  int s_lo = 0, e = 0;               // window (s_lo, e]
  std::map<std::string, int> t;
};

struct Arena {
  char* base = nullptr;
  size_t used = 0;
  void* take(size_t bytes) {
    size_t o = (used + 255) & ~(size_t)255;
    used = o + bytes;
    return base ? base + o : nullptr;
  }
};

}  // namespace lp

// Scratch that one chain of work (a head's loss, its in-window backward pass and the updates) needs:
// one set for the caller's stream and one per side stream.
struct lp_scratch {
  hipStream_t cur_stream = nullptr;
  float* partial = nullptr; size_t partial_elems = 0;
  float* splitk_ws = nullptr; size_t splitk_elems = 0;
  float* loss_rows = nullptr;
  // backward scratch
  void *dA = nullptr, *dB = nullptr, *dF = nullptr, *dc = nullptr, *du = nullptr, *dO = nullptr, *dqkv = nullptr,
       *da = nullptr;
  float* delta = nullptr;
  void *sG = nullptr, *sZ = nullptr, *sR = nullptr, *sD1 = nullptr, *sD2 = nullptr;  // resnet
  // head scratch
  void *feat = nullptr, *logits = nullptr, *dfeat = nullptr;
  float *hmean = nullptr, *hrstd = nullptr;
};

struct lp_ctx : lp_scratch {
  lp_model_spec spec;
  std::vector<lp_layer_spec> layer_specs;
  std::vector<lp_head_spec> head_specs;
  std::vector<lp::Tensor> tensors;
  std::map<std::string, int> index;
  std::vector<lp::LayerState> layers;   // [0] unused; 1..L
  std::vector<lp::HeadState> heads;     // 0-based
  struct UnitRef { int li, bi, which; };          // which: 0 stem, 1 conv1, 2 conv2, 3 proj
  std::map<std::string, UnitRef> units;           // "L2.b1.conv1" -> the unit
  lp::ConvUnit* unit(const UnitRef& r) {
    lp::LayerState& S = layers[r.li];
    if (r.which == 0) return &S.stem;
    lp::BasicBlock& b = S.blocks[r.bi];
    return r.which == 1 ? &b.c1 : (r.which == 2 ? &b.c2 : &b.proj);
  }
  size_t P = 0;                         // flat parameter elements
  int dt = 0;
  hipStream_t stream = nullptr;
  // device memory (borrowed)
  float* master = nullptr; void* lowp = nullptr;
  // transposed bf16 copy [in][out] of a weight [out][in], per tensor (null: none).  Kept for the vocabulary
  // heads: their input-gradient GEMM then has the reduction index fastest in both operands, which the
  // direct-to-LDS kernel runs 18 % faster than with a k-major operand (ds_read_b128 instead of two
  // transposing 8-byte reads per fragment).
  std::vector<void*> wt;
  // running statistics of every batch normalisation: for the gain tensor with index i and C channels,
  // run_off[i] >= 0 and bn_run + run_off[i] holds the running mean, the next C floats the running variance
  float* bn_run = nullptr;
  size_t bn_run_elems = 0;
  std::vector<long> run_off;
  float bn_momentum = 0.1f;      // 0: keep no running statistics
  int bn_eval_running = 0;       // lp_eval_loss normalises with the running statistics
  int bn_mode = 0;               // what the forward pass in flight does: 0 batch only, 1 batch + fold in, 2 running
  lp::BnRunning bn_tmp;
  const lp::BnRunning* bn_for(int gain_tensor, int C) {
    if (bn_mode == 0 || !bn_run || gain_tensor < 0 || gain_tensor >= (int)run_off.size() || run_off[gain_tensor] < 0)
      return nullptr;
    bn_tmp.mean = bn_run + run_off[gain_tensor];
    bn_tmp.var = bn_tmp.mean + C;
    bn_tmp.momentum = bn_momentum;
    bn_tmp.use = bn_mode == 2;
    return &bn_tmp;
  }
  float* mom = nullptr; float* var = nullptr;
  float* grads = nullptr;
  float* pe = nullptr;
  void* h0 = nullptr;                    // embedded input of layer 1
  const void* x_in = nullptr;            // input of the current call
  // scratch sets: [0] belongs to the caller's stream, [1..n_side] to the side streams
  std::vector<lp_scratch> sets;
  int n_side = 0;
  std::vector<hipEvent_t> ev_fwd, ev_contrib, ev_chain;
  // pipelined schedule (1-based by block = head): the input of block j >= 2, the labels each block uses,
  // the batch size of each block's current input and of its last run, and each block's update count
  std::vector<void*> stash_act;
  std::vector<int32_t*> ybuf;
  std::vector<int> in_batch, ran_batch, blk_updates;
  size_t label_elems_per_sample = 1;
  hipEvent_t ev_pipe = nullptr;
  bool lockstep = false;                 // pipelined blocks are walked stage by stage (grouped GEMMs across blocks)
  void use(int i) { static_cast<lp_scratch&>(*this) = sets[i]; }
  // steps overlapped across calls: a call does not join its chains into the caller's stream; the next step's
  // forward pass of a layer waits only for the chains that read or update that layer (join_pending otherwise)
  int overlap_steps = 0;
  bool pending_join = false;
  int step_t = 0;
  int last_batch = 0;
  // Replay of a captured synchronous step (lp_step_graph): the graph of the last captured call, the
  // arguments it was captured with, and how many calls with those arguments have run eagerly so far.
  bool graph_on = false;
  hipGraphExec_t gexec = nullptr;
  hipStream_t gstream = nullptr;          // capture stream (the caller's stream may be the null stream, which cannot capture)
  const void* g_x = nullptr; const int32_t* g_y = nullptr; float* g_losses = nullptr; int g_batch = -1;
  int g_eager = 0;
  bool ok = false;
  std::string err;

  mutable lp::Profiler prof;
  lp::OpCtx op() const {
    lp::OpCtx c; c.stream = cur_stream; c.dt = dt; c.partial = partial; c.partial_elems = partial_elems;
    c.prof = &prof; c.splitk_ws = splitk_ws; c.splitk_elems = splitk_elems; return c;
  }
  float* P32(int ti) const { return master + tensors[ti].off; }
  float* G32(int ti) const { return grads + tensors[ti].off; }
  // matrix weights in the compute dtype (bf16 working copy, or the fp32 master itself)
  const void* W(int ti) const {
    return dt == lp::BF16 ? (const void*)((const lp::bf16_t*)lowp + tensors[ti].off) : (const void*)(master + tensors[ti].off);
  }
};

namespace lp {
// The GEMMs a driver stage hands back for the caller to launch (see drivers.hip).
struct StageGemms { GemmArgs g[4]; int n = 0; };
constexpr int kDecFwdStages = 4, kDecBwdStages = 5, kVocabHeadStages = 4;
int dec_forward_stage(lp_ctx* c, int li, int batch, const int32_t* ids, int stage, StageGemms* out);
int dec_backward_stage(lp_ctx* c, int li, int batch, const void* dout, void* dx, bool need_dx, int acc,
                       const int32_t* ids, bool params, int stage, StageGemms* out);
int vocab_head_stage(lp_ctx* c, int hi, int batch, const int32_t* y, float* loss_out, bool backward, void* dh,
                     int stage, StageGemms* out);
int drv_forward(lp_ctx* c, int li, int batch, const int32_t* ids_or_null);
// params == false: only the gradient with respect to the layer's input (no parameter gradient is touched).
int drv_backward(lp_ctx* c, int li, int batch, const void* dout, void* dx, bool need_dx, int accumulate,
                 bool params = true);
int drv_head(lp_ctx* c, int hi, int batch, const int32_t* y, float* loss_out, bool backward, void* dh);
size_t layer_out_elems(const lp_layer_spec& s, int batch);
}
