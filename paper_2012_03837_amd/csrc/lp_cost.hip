// FLOP cost model of the paper's appendix A: total FLOPs of a training run and its sequential FLOPs
// ("time") for backpropagation, greedy / overlapping / chunked local parallelism and the last-K-layers
// baseline.  Host arithmetic; nothing here touches a device.
#include "../../include/lp.h"

namespace {

// FLOPs of one MLP layer with I inputs and N outputs: matrix-vector product, bias add, ReLU
// (appendix A, "MLP", as printed).
double mlp_layer_flops(double I, double N) { return (2.0 * I * N - I) + N + 2.0 * N; }

}  // namespace

extern "C" int lp_mlp_flops(int input_size, int hidden, int layers, double* forward_cost, double* aux_cost) {
  if (!forward_cost || !aux_cost || input_size < 1 || hidden < 1 || layers < 1) return LP_EINVAL;
  const double first = mlp_layer_flops(input_size, hidden), rest = mlp_layer_flops(hidden, hidden);
  *forward_cost = (first + (layers - 1) * rest) / layers;
  *aux_cost = (2.0 * hidden * 10.0 - hidden) + 10.0 + 5.0 * 10.0;
  return LP_OK;
}

extern "C" int lp_cost_model(const lp_cost_inputs* in, int method, int K, double steps, double batch_size,
                             lp_cost* out) {
  if (!in || !out || in->layers < 1 || !(steps > 0.0) || !(batch_size > 0.0)) return LP_EINVAL;
  const double f = in->forward_cost, a = in->aux_cost, bm = in->backward_multiplier, L = in->layers;
  if ((method == LP_METHOD_CHUNK || method == LP_METHOD_LAST_K) && (K < 1 || K > in->layers)) return LP_EINVAL;
  double per_example, par, per_step = 10.0 * in->parameters;   // optimizer: ten FLOPs per parameter
  switch (method) {
    case LP_METHOD_BACKPROP:   // one forward + backward of the network and of the single head
      per_example = (1.0 + bm) * (f * L + a); par = 1.0; break;
    case LP_METHOD_GREEDY:     // every layer with its own head, all layers concurrently
      per_example = (1.0 + bm) * ((f + a) * L); par = L; break;
    case LP_METHOD_OVERLAP:    // one forward, two backward passes per non-terminal layer, gradient averaging
      per_example = (f + a) * L + (L - 1.0) * bm * (2.0 * f + a) + bm * (f + a);
      par = L; per_step += 2.0 * in->parameters; break;
    case LP_METHOD_CHUNK:      // forward + backward of every layer, K heads, K chunks concurrently
      per_example = (1.0 + bm) * (f * L + K * a); par = K; break;
    case LP_METHOD_LAST_K:     // full forward, one head, backward through the last K layers (the atomic chunk)
      per_example = (L * f + a) + bm * (K * f + a); par = (L + K * bm) / (K * (1.0 + bm)); break;
    default: return LP_EINVAL;
  }
  out->cost_per_example = per_example;
  out->cost = per_example * steps * batch_size + steps * per_step;
  out->parallelism = par;
  out->time = out->cost / (batch_size * par);
  return LP_OK;
}
