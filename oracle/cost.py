"""FLOP cost model of the paper's appendix A ("Calculation of Total FLOPs and Sequential FLOPs").

TEST INFRASTRUCTURE ONLY: plain Python written from the appendix' formulas, one function per paragraph.
Only tests, the smoke check and the benchmark's CPU leg may import this package.

Four numbers describe a model (average forward FLOPs per layer per example, auxiliary-loss FLOPs per
example, the backward multiplier, the optimizer cost per step = 10 FLOPs per parameter); a method turns
them into total cost and into "time" = sequential FLOPs, the cost divided by the parallelism the method
admits (appendix A, "Calculations per Method").

Readings where the printed formulas are damaged (each is forced by the prose beside it and checked by
the reductions in the tests: K chunks = L gives greedy, K = 1 gives backprop, last-K with K = L gives
backprop with parallelism 1):
  * "Two/Three chunk": the forward cost is that of all layers, (1 + bm) * (layers * forward + K * aux).
  * "Last One/Two Layers": (layers * forward + aux) + bm * (K * forward + aux)   (a '+' is missing in print).
  * cost_per_example and cost_per_step_example name the same quantity.
"""


def mlp_flops(input_size, hidden, layers):
    """Appendix A, "MLP": a layer is a matrix-vector product (2*I*N - I), a bias add (N) and a ReLU (2*N as
    printed); the first layer has I = input_size, the others I = hidden; returns the average over layers
    and the auxiliary classifier's cost (matrix-vector to 10 classes, bias, softmax-CE at 5 FLOPs/class)."""
    def layer(i, n):
        return (2 * i * n - i) + n + 2 * n
    total = layer(input_size, hidden) + (layers - 1) * layer(hidden, hidden)
    aux = (2 * hidden * 10 - hidden) + 10 + 5 * 10
    return total / layers, float(aux)


def optimizer_cost(parameters):
    """Appendix A, first paragraph: ten FLOPs per parameter per step."""
    return 10.0 * parameters


def cost_per_example(method, forward_cost, aux_cost, backward_multiplier, layers, K=1):
    bm, f, a, L = backward_multiplier, forward_cost, aux_cost, layers
    if method == "backprop":
        return (1 + bm) * (f * L + a)
    if method == "greedy":
        return (1 + bm) * ((f + a) * L)
    if method == "overlap":
        return (f + a) * L + (L - 1) * bm * (2 * f + a) + bm * (f + a)
    if method == "chunk":
        return (1 + bm) * (f * L + K * a)
    if method == "last_k":
        return (L * f + a) + bm * (K * f + a)
    raise ValueError(method)


def parallelism(method, backward_multiplier, layers, K=1):
    """What "time" divides the per-batch-element cost by."""
    if method == "backprop":
        return 1.0
    if method in ("greedy", "overlap"):
        return float(layers)
    if method == "chunk":
        return float(K)
    if method == "last_k":
        return (layers + K * backward_multiplier) / (K * (1 + backward_multiplier))
    raise ValueError(method)


def cost_and_time(method, forward_cost, aux_cost, backward_multiplier, layers, parameters, steps, batch_size, K=1):
    """Total FLOPs to run `steps` steps at `batch_size`, and the sequential FLOPs ("time")."""
    cpe = cost_per_example(method, forward_cost, aux_cost, backward_multiplier, layers, K)
    per_step_extra = optimizer_cost(parameters)
    if method == "overlap":
        per_step_extra += 2.0 * parameters          # averaging the duplicated layers' gradients
    cost = cpe * steps * batch_size + steps * per_step_extra
    time = cost / (batch_size * parallelism(method, backward_multiplier, layers, K))
    return cpe, cost, time
