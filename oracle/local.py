"""The local-update step, written out step by step (CPU oracle; test infrastructure only).

One synchronous step on a minibatch (paper section 3; cost accounting of appendix A.2 counts one
forward per layer per step for every variant, which fixes the synchronous reading):

  1. h_0 = x;  h_l = f_l(h_{l-1}; theta_l) for l = 1..L  (one forward pass, weights theta_t).
  2. For each auxiliary head j attached after layer e_j with window w_j: s_j = max(e_j - w_j, 0);
     loss_j = CE(head_j(f_{e_j} o ... o f_{s_j+1}(const(h_{s_j}))), y), where const() blocks the
     gradient ("each block ... receives the activations output by the previous block as input").
  3. grad(head_j params) = d loss_j / d(head params); grad(theta_l) = combine over the heads whose
     window covers l of d loss_j / d theta_l  (greedy / overlapping / chunked / backprop differ
     only in the list of (e_j, w_j)); combine is a sum, or a mean ("averaging updates").
  4. Every covered parameter tensor takes one optimizer update; layers covered by no window and
     their state are left untouched (the "last K layers" baseline).
  5. Return loss_j evaluated at theta_t for every head.

Each loss_j is differentiated separately, exactly as defined; no fusion of overlapping windows.
"""
from __future__ import annotations

import copy

import numpy as np

from . import layers as L
from . import ops


def _policy(stored):
    """Storage precision of forward activations and matrix weight operands: None = exact (float64),
    "bf16" = rounded to bfloat16 wherever a "bf16 compute" configuration keeps them in memory."""
    if stored is None:
        return ops.identity
    if stored == "bf16":
        return ops.bf16_round
    raise ValueError(stored)


def _cast(P, dtype, q=ops.identity):
    """Weights as the forward/backward passes see them: vectors exact, matrices in storage precision."""
    return {k: (q(np.asarray(v, dtype=dtype)) if np.ndim(v) >= 2 else np.asarray(v, dtype=dtype))
            for k, v in P.items()}


def _as_mode(bn, mode):
    """The same running statistics (shared dictionaries), seen by a forward pass in the given mode."""
    v = copy.copy(bn)
    v.mode = mode
    return v


def _windows(cfg):
    return [(max(h.after_layer - h.window, 0), h.after_layer) for h in cfg.heads]


def forward_all(cfg, P, x, q=ops.identity, bn=None):
    """Step 1.  Returns activations hs[0..L] (hs[0] = x) and per-layer caches[1..L]."""
    hs = [x]
    caches = [None]
    for li in range(1, cfg.n_layers + 1):
        out, c = L.layer_fwd(cfg, P, li, hs[-1], q, bn)
        hs.append(out)
        caches.append(c)
    return hs, caches


def eval_loss(cfg, params, x, y, dtype=np.float64, stored=None, bn=None):
    """Steps 1-2, values only: the loss of every head at the current weights.  With ``bn`` (a
    BatchNormRunning) every batch normalisation uses the running statistics instead of the batch's."""
    if bn is not None:
        bn = _as_mode(bn, "use")
    q = _policy(stored)
    P = _cast(params, dtype, q)
    xx = x if np.issubdtype(np.asarray(x).dtype, np.integer) else np.asarray(x, dtype=dtype)
    hs, _ = forward_all(cfg, P, xx, q, bn)
    return np.array([L.head_loss(cfg, P, hi, hs[h.after_layer], y, q, bn)[0]
                     for hi, h in enumerate(cfg.heads, start=1)], dtype=np.float64)


def head_gradients(cfg, P, hi, hs, caches, y, q=ops.identity, bn=None):
    """Steps 2-3 for one head: loss_j and the gradient of loss_j w.r.t. everything in its window.

    hs[s_j] is treated as data: the backward pass stops there (need_dx False at layer s_j + 1).
    """
    s, e = _windows(cfg)[hi - 1]
    loss, hc = L.head_loss(cfg, P, hi, hs[e], y, q, bn)
    dh, grads = L.head_bwd(cfg, P, hi, hc)
    for li in range(e, s, -1):
        dh, g = L.layer_bwd(cfg, P, li, caches[li], dh, need_dx=(li > s + 1))
        grads.update(g)
    return loss, grads


def local_gradients(cfg, params, x, y, dtype=np.float64, per_head=False, stored=None, bn=None):
    """Steps 1-3.  Returns (losses[n_heads], grads by parameter name, coverage count by name).

    Parameters covered by no window are absent from ``grads``.  With ``bn`` (a BatchNormRunning) every
    batch normalisation the step evaluates folds its batch statistics into the running ones, once.
    """
    if bn is not None:
        bn = _as_mode(bn, "update")
    q = _policy(stored)
    P = _cast(params, dtype, q)
    xx = x if np.issubdtype(np.asarray(x).dtype, np.integer) else np.asarray(x, dtype=dtype)
    hs, caches = forward_all(cfg, P, xx, q, bn)
    losses = []
    total, count, each = {}, {}, []
    for hi in range(1, len(cfg.heads) + 1):
        loss, g = head_gradients(cfg, P, hi, hs, caches, y, q, bn)
        losses.append(loss)
        each.append(g)
        for k, v in g.items():
            if k in total:
                total[k] = total[k] + v
                count[k] += 1
            else:
                total[k] = v.copy()
                count[k] = 1
    if cfg.combine == "mean":
        total = {k: v / count[k] for k, v in total.items()}
    elif cfg.combine != "sum":
        raise ValueError(cfg.combine)
    if per_head:
        return np.array(losses), total, count, each
    return np.array(losses), total, count


def block_gradients(cfg, params, hi, h_s, y, dtype=np.float64, stored=None, bn=None):
    """Head hi alone, fed its window input h_s as data (that input is detached by definition, so
    the block's loss and gradients depend on the rest of the network only through h_s)."""
    if bn is not None:
        bn = _as_mode(bn, "update")
    q = _policy(stored)
    P = _cast(params, dtype, q)
    s, e = _windows(cfg)[hi - 1]
    x = h_s if np.issubdtype(np.asarray(h_s).dtype, np.integer) else np.asarray(h_s, dtype=dtype)
    hs = {s: x}
    caches = {}
    for li in range(s + 1, e + 1):
        hs[li], caches[li] = L.layer_fwd(cfg, P, li, hs[li - 1], q, bn)
    loss, hc = L.head_loss(cfg, P, hi, hs[e], y, q, bn)
    dh, grads = L.head_bwd(cfg, P, hi, hc)
    for li in range(e, s, -1):
        dh, g = L.layer_bwd(cfg, P, li, caches[li], dh, need_dx=(li > s + 1))
        grads.update(g)
    return loss, grads, hs[e]


# ----------------------------------------------------------------------------- optimizers
def new_state(cfg, params, dtype=np.float64):
    st = {"t": 0}
    if cfg.opt.kind in ("sgdm", "adam"):
        st["m"] = {k: np.zeros(v.shape, dtype) for k, v in params.items()}
    if cfg.opt.kind == "adam":
        st["v"] = {k: np.zeros(v.shape, dtype) for k, v in params.items()}
    return st


def optimizer_update(opt, p, g, state, name, t):
    """One update of one tensor.  SGD: p -= lr g.  SGD-momentum: v = mu v + g; p -= lr v.
    Adam: m = b1 m + (1-b1) g; v = b2 v + (1-b2) g^2; p -= lr (m/(1-b1^t)) / (sqrt(v/(1-b2^t)) + eps).
    Optional L2 weight decay adds wd*p to g first."""
    if opt.weight_decay:
        g = g + opt.weight_decay * p
    if opt.kind == "sgd":
        return p - opt.lr * g
    if opt.kind == "sgdm":
        m = opt.momentum * state["m"][name] + g
        state["m"][name] = m
        return p - opt.lr * m
    if opt.kind == "adam":
        m = opt.beta1 * state["m"][name] + (1.0 - opt.beta1) * g
        v = opt.beta2 * state["v"][name] + (1.0 - opt.beta2) * g * g
        state["m"][name] = m
        state["v"][name] = v
        mhat = m / (1.0 - opt.beta1 ** t)
        vhat = v / (1.0 - opt.beta2 ** t)
        return p - opt.lr * mhat / (np.sqrt(vhat) + opt.eps)
    raise ValueError(opt.kind)


def local_step(cfg, params, state, x, y, dtype=np.float64, stored=None, bn=None):
    """Steps 1-5.  Returns (losses, new params, grads).  ``state`` is updated in place.  The update
    always acts on the exact (master) weights, whatever the storage precision of the passes."""
    losses, grads, _ = local_gradients(cfg, params, x, y, dtype, stored=stored, bn=bn)
    state["t"] += 1
    t = state["t"]
    new = {}
    for k, p in params.items():
        p = np.asarray(p, dtype=dtype)
        new[k] = optimizer_update(cfg.opt, p, grads[k], state, k, t) if k in grads else p
    return losses, new, grads


def layer_gradient_cosines(cfg, grads_a, grads_b):
    """Section 5, "Gradient Angles" (Fig. 6a): for every layer l, the cosine of the angle between two
    gradients of all of layer l's parameters taken as one vector,
        cos_l = <a_l, b_l> / (|a_l| |b_l|),
    here between the gradients two schemes (e.g. greedy local updates and backprop) leave for the same
    parameters and minibatch.  A layer for which either gradient is absent or zero gets 0."""
    out = np.zeros(cfg.n_layers)
    for l in range(1, cfg.n_layers + 1):
        names = sorted(k for k in set(grads_a) | set(grads_b) if k.startswith(f"L{l}."))
        dot = na = nb = 0.0
        for k in names:
            a = np.asarray(grads_a.get(k, 0.0), dtype=np.float64)
            b = np.asarray(grads_b.get(k, 0.0), dtype=np.float64)
            if k in grads_a:
                na += float(np.sum(a * a))
            if k in grads_b:
                nb += float(np.sum(b * b))
            if k in grads_a and k in grads_b:
                dot += float(np.sum(a * b))
        out[l - 1] = dot / np.sqrt(na * nb) if na > 0.0 and nb > 0.0 else 0.0
    return out


# ----------------------------------------------------------------------------- pipelined schedule
def new_pipeline(cfg):
    """State of the pipelined schedule: for every block j >= 2 the (activation, labels) pair that block j-1
    produced in the previous call (None while the pipeline is still filling), and every block's own
    number of updates."""
    J = len(cfg.heads)
    return {"stash": [None] * (J + 2), "updates": [0] * (J + 1)}


def pipelined_step(cfg, params, state, pipe, x, y, dtype=np.float64, stored=None, bn=None):
    """One call of the pipelined form of local parallelism (section 6: the pipeline runs in steady state
    after a ramp-up, updates applied asynchronously; section 3: activations and labels move forward one
    stage per iteration, so every stage has the input and target it needs for local learning).

    The heads' windows must tile the layers (block j = layers e_{j-1}+1 .. e_j).  In call t block 1 takes the
    call's minibatch (x, y); block j >= 2 takes the activation block j-1 produced in call t-1 (with the
    weights block j-1 had then) together with the labels that travelled with it, i.e. minibatch t-j+1.
    Every block runs forward, its head's loss, the backward pass inside the block and its own update; a
    block whose input has not arrived yet (t < j) does nothing and reports loss 0.  The optimizer's step
    count of a block is the number of updates that block has taken.
    Returns (losses, new params); ``state`` and ``pipe`` are updated in place."""
    wins = _windows(cfg)
    assert wins[0][0] == 0 and all(wins[j][0] == wins[j - 1][1] for j in range(1, len(wins))), "windows must tile"
    J = len(cfg.heads)
    losses = np.zeros(J)
    new = {k: np.asarray(v, dtype=dtype) for k, v in params.items()}
    nxt = [None] * (J + 2)
    for j in range(1, J + 1):
        inp = (x, y) if j == 1 else pipe["stash"][j]
        if inp is None:
            continue
        loss, grads, out = block_gradients(cfg, params, j, inp[0], inp[1], dtype, stored, bn)
        losses[j - 1] = loss
        pipe["updates"][j] += 1
        for k, g in grads.items():
            new[k] = optimizer_update(cfg.opt, np.asarray(params[k], dtype=dtype), g, state, k, pipe["updates"][j])
        nxt[j + 1] = (out, inp[1])
    pipe["stash"] = nxt
    return losses, new
