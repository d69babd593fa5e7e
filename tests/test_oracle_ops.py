"""Pins for the oracle's primitives: brute-force loops on tiny shapes, closed forms, and
independent library routines (torch CPU, autograd) that the primitives must reduce to."""
import math

import numpy as np
import pytest
import torch

from oracle import ops
from oracle import local as OLoc
import lp_inputs as LI

RNG = np.random.default_rng(11)


def T(a, grad=False):
    t = torch.tensor(np.asarray(a, dtype=np.float64), dtype=torch.float64)
    t.requires_grad_(grad)
    return t


def close(a, b, tol=1e-11):
    a = np.asarray(a)
    b = b.detach().numpy() if isinstance(b, torch.Tensor) else np.asarray(b)
    assert a.shape == b.shape, (a.shape, b.shape)
    assert np.abs(a - b).max() <= tol * max(1.0, np.abs(b).max()), np.abs(a - b).max()


# ----------------------------------------------------------------------------- brute force
def test_conv_brute_force_seven_loops():
    for stride, pad, R in [(1, 1, 3), (2, 1, 3), (2, 0, 1)]:
        N, H, W, C, O = 2, 5, 6, 3, 4
        x = RNG.standard_normal((N, H, W, C))
        w = RNG.standard_normal((O, R, R, C))
        got = ops.conv2d_fwd(x, w, stride, pad)
        P = (H + 2 * pad - R) // stride + 1
        Q = (W + 2 * pad - R) // stride + 1
        ref = np.zeros((N, P, Q, O))
        for n in range(N):
            for p in range(P):
                for q in range(Q):
                    for o in range(O):
                        acc = 0.0
                        for r in range(R):
                            for s in range(R):
                                for c in range(C):
                                    hh, ww = p * stride + r - pad, q * stride + s - pad
                                    if 0 <= hh < H and 0 <= ww < W:
                                        acc += x[n, hh, ww, c] * w[o, r, s, c]
                        ref[n, p, q, o] = acc
        close(got, ref, 1e-13)


def test_attention_brute_force_rows():
    B, H, S, dh = 2, 2, 5, 3
    q, k, v = (RNG.standard_normal((B, H, S, dh)) for _ in range(3))
    o, p = ops.attention_fwd(q, k, v, causal=True)
    for b in range(B):
        for h in range(H):
            for i in range(S):
                sc = [sum(q[b, h, i, t] * k[b, h, j, t] for t in range(dh)) / math.sqrt(dh)
                      for j in range(i + 1)]
                m = max(sc)
                e = [math.exp(s_ - m) for s_ in sc]
                z = sum(e)
                for t in range(dh):
                    ref = sum(e[j] / z * v[b, h, j, t] for j in range(i + 1))
                    assert abs(o[b, h, i, t] - ref) < 1e-13
                assert np.all(p[b, h, i, i + 1:] == 0)


@pytest.mark.parametrize("kind", ["sgd", "sgdm", "adam"])
def test_optimizers_scalar_loop_and_torch(kind):
    opt = LI.OptCfg(kind, lr=0.01, momentum=0.9, beta1=0.9, beta2=0.999, eps=1e-8)
    p0 = RNG.standard_normal(7)
    gs = [RNG.standard_normal(7) for _ in range(4)]
    # oracle
    st = {"t": 0, "m": {"p": np.zeros(7)}, "v": {"p": np.zeros(7)}}
    p = p0.copy()
    for t, g in enumerate(gs, start=1):
        p = OLoc.optimizer_update(opt, p, g, st, "p", t)
    # scalar loop, from the update rules
    ref = p0.copy()
    for i in range(7):
        m = v = 0.0
        x = p0[i]
        for t, g in enumerate(gs, start=1):
            gi = g[i]
            if kind == "sgd":
                x -= 0.01 * gi
            elif kind == "sgdm":
                m = 0.9 * m + gi
                x -= 0.01 * m
            else:
                m = 0.9 * m + 0.1 * gi
                v = 0.999 * v + 0.001 * gi * gi
                x -= 0.01 * (m / (1 - 0.9 ** t)) / (math.sqrt(v / (1 - 0.999 ** t)) + 1e-8)
        ref[i] = x
    close(p, ref, 1e-14)
    # library routine
    tp = T(p0, True)
    topt = {"sgd": lambda: torch.optim.SGD([tp], lr=0.01),
            "sgdm": lambda: torch.optim.SGD([tp], lr=0.01, momentum=0.9),
            "adam": lambda: torch.optim.Adam([tp], lr=0.01, betas=(0.9, 0.999), eps=1e-8)}[kind]()
    for g in gs:
        tp.grad = T(g)
        topt.step()
    close(p, tp, 1e-12)


# ----------------------------------------------------------------------------- closed forms
def test_norm_closed_forms():
    x = RNG.standard_normal((6, 9)) * 3 + 2
    y, _ = ops.layernorm_fwd(x, np.ones(9), np.zeros(9))
    assert np.abs(y.mean(-1)).max() < 1e-14
    assert np.abs(y.var(-1) - x.var(-1) / (x.var(-1) + 1e-5)).max() < 1e-12
    xb = RNG.standard_normal((3, 4, 5, 2)) * 2 - 1
    yb, _ = ops.batchnorm_fwd(xb, np.ones(2), np.zeros(2))
    assert np.abs(yb.mean((0, 1, 2))).max() < 1e-14
    assert np.abs(yb.var((0, 1, 2)) - 1).max() < 1e-4


def test_ce_closed_forms():
    z = np.zeros((5, 10))
    y = np.array([0, 3, 3, 9, 1])
    loss, p = ops.softmax_ce_fwd(z, y)
    assert abs(loss - math.log(10)) < 1e-15
    dz = ops.softmax_ce_bwd(p, y)
    assert np.abs(dz.sum(-1)).max() < 1e-16
    assert abs(dz[0, 0] - (0.1 - 1) / 5) < 1e-16 and abs(dz[0, 1] - 0.1 / 5) < 1e-16
    # shift invariance and large logits (max-subtracted)
    z = RNG.standard_normal((5, 10)) * 5
    l1, _ = ops.softmax_ce_fwd(z, y)
    l2, _ = ops.softmax_ce_fwd(z + 1000.0, y)
    assert abs(l1 - l2) < 1e-10


def test_gelu_values():
    assert ops.gelu_fwd(np.array([0.0]))[0] == 0.0
    assert abs(ops.gelu_fwd(np.array([10.0]))[0] - 10.0) < 1e-9
    assert abs(ops.gelu_fwd(np.array([-10.0]))[0]) < 1e-9
    # tanh-form value at 1: 0.5*(1+tanh(0.79788456*(1.044715)))
    assert abs(ops.gelu_fwd(np.array([1.0]))[0] - 0.8411919906082768) < 1e-12


def test_sinusoid_positions():
    pe = ops.sinusoid_positions(7, 6)
    assert np.all(pe[0, 0::2] == 0) and np.all(pe[0, 1::2] == 1)
    assert abs(pe[3, 0] - math.sin(3.0)) < 1e-15 and abs(pe[3, 1] - math.cos(3.0)) < 1e-15
    assert abs(pe[5, 4] - math.sin(5.0 / 10000 ** (4 / 6))) < 1e-15
    assert abs(pe[5, 5] - math.cos(5.0 / 10000 ** (4 / 6))) < 1e-15


# ----------------------------------------------------------------------------- library routines
def test_linear_layernorm_gelu_vs_torch():
    x, w, b = RNG.standard_normal((5, 7)), RNG.standard_normal((4, 7)), RNG.standard_normal(4)
    dy = RNG.standard_normal((5, 4))
    tx, tw, tb = T(x, True), T(w, True), T(b, True)
    ty = torch.nn.functional.linear(tx, tw, tb)
    ty.backward(T(dy))
    close(ops.linear_fwd(x, w, b), ty)
    dx, dw, db = ops.linear_bwd(x, w, dy)
    close(dx, tx.grad), close(dw, tw.grad), close(db, tb.grad)

    g, bb = RNG.standard_normal(7), RNG.standard_normal(7)
    dy = RNG.standard_normal((5, 7))
    tx, tg, tbb = T(x, True), T(g, True), T(bb, True)
    ty = torch.nn.functional.layer_norm(tx, (7,), tg, tbb, eps=1e-5)
    ty.backward(T(dy))
    y, c = ops.layernorm_fwd(x, g, bb)
    close(y, ty)
    dx, dg, db = ops.layernorm_bwd(c, g, dy)
    close(dx, tx.grad), close(dg, tg.grad), close(db, tbb.grad)

    tx = T(x, True)
    ty = torch.nn.functional.gelu(tx, approximate="tanh")
    ty.backward(T(dy))
    close(ops.gelu_fwd(x), ty)
    close(ops.gelu_bwd(x, dy), tx.grad)


def test_batchnorm_conv_vs_torch():
    x = RNG.standard_normal((3, 5, 6, 4))
    g, b = RNG.standard_normal(4), RNG.standard_normal(4)
    dy = RNG.standard_normal(x.shape)
    tx, tg, tb = T(x.transpose(0, 3, 1, 2), True), T(g, True), T(b, True)
    ty = torch.nn.functional.batch_norm(tx, None, None, tg, tb, training=True, eps=1e-5)
    ty.backward(T(dy.transpose(0, 3, 1, 2)))
    y, c = ops.batchnorm_fwd(x, g, b)
    close(y, ty.permute(0, 2, 3, 1))
    dx, dg, db = ops.batchnorm_bwd(c, g, dy)
    close(dx, tx.grad.permute(0, 2, 3, 1)), close(dg, tg.grad), close(db, tb.grad)

    for stride, pad, R in [(1, 1, 3), (2, 1, 3), (2, 0, 1)]:
        w = RNG.standard_normal((5, R, R, 4))
        tx, tw = T(x.transpose(0, 3, 1, 2), True), T(w.transpose(0, 3, 1, 2), True)
        ty = torch.nn.functional.conv2d(tx, tw, stride=stride, padding=pad)
        out = ops.conv2d_fwd(x, w, stride, pad)
        close(out, ty.permute(0, 2, 3, 1))
        dout = RNG.standard_normal(out.shape)
        ty.backward(T(dout.transpose(0, 3, 1, 2)))
        dx, dw = ops.conv2d_bwd(x, w, stride, pad, dout)
        close(dx, tx.grad.permute(0, 2, 3, 1)), close(dw, tw.grad.permute(0, 2, 3, 1))


def test_attention_ce_embed_vs_torch():
    B, H, S, dh = 2, 3, 6, 4
    q, k, v, do = (RNG.standard_normal((B, H, S, dh)) for _ in range(4))
    tq, tk, tv = T(q, True), T(k, True), T(v, True)
    to = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, is_causal=True)
    to.backward(T(do))
    o, p = ops.attention_fwd(q, k, v, True)
    close(o, to)
    dq, dk, dv = ops.attention_bwd(q, k, v, p, do)
    close(dq, tq.grad), close(dk, tk.grad), close(dv, tv.grad)

    z = RNG.standard_normal((7, 9)) * 3
    y = RNG.integers(0, 9, 7)
    tz = T(z, True)
    tl = torch.nn.functional.cross_entropy(tz, torch.tensor(y))
    tl.backward()
    loss, pr = ops.softmax_ce_fwd(z, y)
    assert abs(loss - tl.item()) < 1e-13
    close(ops.softmax_ce_bwd(pr, y), tz.grad)

    ids = RNG.integers(0, 5, (2, 6))
    ids[0, :3] = 2                                   # repeated token: gradients must accumulate
    emb = RNG.standard_normal((5, 4))
    temb = T(emb, True)
    th = torch.nn.functional.embedding(torch.tensor(ids), temb)
    dh_ = RNG.standard_normal((2, 6, 4))
    th.backward(T(dh_))
    close(ops.embed_fwd(ids, emb, np.zeros((6, 4))), th)
    close(ops.embed_bwd(ids, 5, dh_), temb.grad)


def test_decoder_layer_vs_torch_autograd():
    """A whole pre-LN causal decoder layer + LN/linear/CE head, rebuilt from torch library calls."""
    from oracle import layers as OL
    cfg = LI.configs.decoder_config("t", n_layers=2, width=8, n_heads=2, hidden=12, seq_len=5, batch=2,
                                    vocab=11, scheme="backprop")
    P = LI.perturb_params(LI.init_params(cfg, seed=2, head_scale=3.0), 4, 0.2)
    P = {k: v.astype(np.float64) * (6.0 if v.ndim == 2 else 1.0) for k, v in P.items()}
    x, y = LI.make_batch(cfg, 0)
    import oracle
    losses, grads, _ = oracle.local_gradients(cfg, P, x, y)
    tP = {k: T(v, True) for k, v in P.items()}
    F = torch.nn.functional
    pe = T(ops.sinusoid_positions(5, 8))
    h = F.embedding(torch.tensor(x), tP["L1.emb"]) + pe
    for li in (1, 2):
        p = f"L{li}."
        a = F.layer_norm(h, (8,), tP[p + "ln1.g"], tP[p + "ln1.b"])
        qkv = F.linear(a, tP[p + "wqkv"], tP[p + "bqkv"])
        q, k, v = (t.reshape(2, 5, 2, 4).transpose(1, 2) for t in qkv.split(8, dim=-1))
        o = F.scaled_dot_product_attention(q, k, v, is_causal=True).transpose(1, 2).reshape(2, 5, 8)
        u = h + F.linear(o, tP[p + "wo"], tP[p + "bo"])
        c = F.layer_norm(u, (8,), tP[p + "ln2.g"], tP[p + "ln2.b"])
        h = u + F.linear(F.gelu(F.linear(c, tP[p + "w1"], tP[p + "b1"]), approximate="tanh"),
                         tP[p + "w2"], tP[p + "b2"])
    z = F.linear(F.layer_norm(h, (8,), tP["H1.ln.g"], tP["H1.ln.b"]), tP["H1.w"])
    loss = F.cross_entropy(z.reshape(-1, 11), torch.tensor(y.reshape(-1)).long())
    loss.backward()
    assert abs(loss.item() - losses[0]) < 1e-12
    for k in P:
        close(grads[k], tP[k].grad, 1e-10)


def test_resnet_stage_vs_torch_autograd():
    cfg = LI.configs.resnet_config("t", channels=(4, 6), in_hw=6, in_ch=3, n_classes=3, batch=3,
                                   n_basic_blocks=2, scheme="backprop")
    P = LI.perturb_params(LI.init_params(cfg, seed=2, head_scale=3.0), 4, 0.2)
    P = {k: v.astype(np.float64) for k, v in P.items()}
    x, y = LI.make_batch(cfg, 0)
    import oracle
    losses, grads, _ = oracle.local_gradients(cfg, P, x, y)
    tP = {k: T(v.transpose(0, 3, 1, 2) if v.ndim == 4 else v, True) for k, v in P.items()}
    F = torch.nn.functional

    def cb(h, w, bn, stride, pad, relu):
        z = F.conv2d(h, tP[w], stride=stride, padding=pad)
        z = F.batch_norm(z, None, None, tP[bn + "g"], tP[bn + "b"], training=True, eps=1e-5)
        return F.relu(z) if relu else z

    h = T(x.transpose(0, 3, 1, 2))
    h = cb(h, "L1.stem.w", "L1.stem.bn.", 1, 1, True)
    for li, stride0 in ((1, 1), (2, 2)):
        for b in (1, 2):
            q = f"L{li}.b{b}."
            st = stride0 if b == 1 else 1
            t = cb(h, q + "conv1.w", q + "bn1.", st, 1, True)
            t = cb(t, q + "conv2.w", q + "bn2.", 1, 1, False)
            sc = cb(h, q + "proj.w", q + "proj.bn.", st, 0, False) if (q + "proj.w") in tP else h
            h = F.relu(t + sc)
    z = F.linear(h.mean(dim=(2, 3)), tP["H1.w"], tP["H1.b"])
    loss = F.cross_entropy(z, torch.tensor(y).long())
    loss.backward()
    assert abs(loss.item() - losses[0]) < 1e-12
    for k in P:
        tg = tP[k].grad
        close(grads[k], tg.permute(0, 2, 3, 1) if tg.ndim == 4 else tg, 1e-10)


def test_bf16_round_vs_library():
    """The oracle's own round-to-nearest-even bf16 rounding equals the library conversion, bit for bit."""
    x = np.concatenate([RNG.standard_normal(5000) * 10.0 ** RNG.integers(-6, 6, 5000),
                        np.array([0.0, -0.0, 1.0, 1.00390625, 1.001953125, 1.005859375, 3.3895314e38])])
    got = ops.bf16_round(x)
    ref = torch.tensor(x, dtype=torch.float32).to(torch.bfloat16).to(torch.float64).numpy()
    assert got.dtype == np.float64
    np.testing.assert_array_equal(got, ref)


def test_stored_precision_mode_keeps_structure():
    """With bf16 storage the oracle still obeys the window rule and stays close to the exact one."""
    import oracle
    cfg = LI.make_config("cfg2_small")
    P = LI.init_params(cfg)
    x, y = LI.make_batch(cfg)
    l0, g0, _ = oracle.local_gradients(cfg, P, x, y)
    l1, g1, _ = oracle.local_gradients(cfg, P, x, y, stored="bf16")
    assert set(g0) == set(g1)
    assert np.abs(l0 - l1).max() < 2e-2
    assert np.abs(l0 - l1).max() > 0


# ----------------------------------------------------------------------------- storage rounding rule
# The rule of the oracle's stored="bf16" mode, stated on its own: in a "bf16 compute, fp32 master weights"
# configuration every tensor that one operation hands to the next through memory is a bf16 tensor: the input,
# the matrix weights as the passes see them, each convolution output, each normalisation (+ shortcut) (+ ReLU)
# output, the pooled features and the logits.  What lives inside an operation (sums, batch statistics, the
# normalised value before it is stored) and every quantity of the backward pass is exact.  A ReLU's derivative
# is read off the stored output (out > 0), and rounding passes gradients through unchanged.
# The pin below builds the same network from torch's own convolution / batch-norm / cross-entropy routines with
# autograd, applies that rule with two tiny autograd functions, and must reproduce the oracle to rounding error;
# a rounding dropped from, added to or moved inside the oracle changes values by ~2^-9 and fails it.
class _StoreBf16(torch.autograd.Function):
    @staticmethod
    def forward(ctx, t):
        return t.to(torch.float32).to(torch.bfloat16).to(torch.float64)

    @staticmethod
    def backward(ctx, g):
        return g


class _ReluStoreBf16(torch.autograd.Function):
    @staticmethod
    def forward(ctx, t):
        out = torch.relu(t).to(torch.float32).to(torch.bfloat16).to(torch.float64)
        ctx.save_for_backward(out)
        return out

    @staticmethod
    def backward(ctx, g):
        (out,) = ctx.saved_tensors
        return g * (out > 0).to(g.dtype)


@pytest.mark.parametrize("head", ["pool_linear_ce", "bn_pool_linear_ce"])
def test_stored_precision_rule_vs_torch_straight_through(head):
    import oracle
    cfg = LI.configs.resnet_config("t", channels=(4, 6), in_hw=6, in_ch=3, n_classes=3, batch=5,
                                   n_basic_blocks=2, scheme="greedy", head=head)
    P = LI.perturb_params(LI.init_params(cfg, seed=2, head_scale=3.0), 4, 0.2)
    P = {k: v.astype(np.float64) for k, v in P.items()}
    x, y = LI.make_batch(cfg, 0)
    x = ops.bf16_round(x.astype(np.float64))
    losses, grads, _ = oracle.local_gradients(cfg, P, x, y, stored="bf16")
    exact_losses, exact_grads, _ = oracle.local_gradients(cfg, P, x, y)
    tP = {k: T(v.transpose(0, 3, 1, 2) if v.ndim == 4 else v, True) for k, v in P.items()}
    W = {k: (_StoreBf16.apply(v) if v.ndim >= 2 else v) for k, v in tP.items()}      # matrices as the passes see them
    F = torch.nn.functional
    st, rl = _StoreBf16.apply, _ReluStoreBf16.apply

    def cb(h, w, bn, stride, pad, relu, res=None):
        z = st(F.conv2d(h, W[w], stride=stride, padding=pad))
        v = F.batch_norm(z, None, None, W[bn + "g"], W[bn + "b"], training=True, eps=1e-5)
        if res is not None:
            v = v + res
        return rl(v) if relu else st(v)

    def stage(h, li, stride0):
        if li == 1:
            h = cb(h, "L1.stem.w", "L1.stem.bn.", 1, 1, True)
        for b in (1, 2):
            q = f"L{li}.b{b}."
            s_ = stride0 if b == 1 else 1
            t = cb(h, q + "conv1.w", q + "bn1.", s_, 1, True)
            sc = cb(h, q + "proj.w", q + "proj.bn.", s_, 0, False) if (q + "proj.w") in W else h
            h = cb(t, q + "conv2.w", q + "bn2.", 1, 1, True, res=sc)
        return h

    def head_loss(h, hi):
        p = f"H{hi}."
        if head == "bn_pool_linear_ce":
            h = rl(F.batch_norm(h, None, None, W[p + "bn.g"], W[p + "bn.b"], training=True, eps=1e-5))
        feat = st(h.mean(dim=(2, 3)))
        z = st(F.linear(feat, W[p + "w"], W[p + "b"]))
        return F.cross_entropy(z, torch.tensor(y).long())

    h1 = stage(T(x.transpose(0, 3, 1, 2)), 1, 1)
    l1 = head_loss(h1, 1)
    h2 = stage(h1.detach(), 2, 2)           # the block's input is data
    l2 = head_loss(h2, 2)
    (l1 + l2).backward()
    assert abs(l1.item() - losses[0]) < 1e-12 and abs(l2.item() - losses[1]) < 1e-12
    assert abs(losses[0] - exact_losses[0]) > 1e-7       # the rounding is really there
    for k in P:
        tg = tP[k].grad
        close(grads[k], tg.permute(0, 2, 3, 1) if tg.ndim == 4 else tg, 1e-10)
    # and the mode stays within the bf16 tolerance of the exact step on this network
    assert max(abs(losses - exact_losses) / exact_losses) < 2e-2
