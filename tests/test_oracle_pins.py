"""Pins for the CPU oracle: properties fixed by the paper's definition of local updates
(section 3; appendix A.2 for the overlap bookkeeping) and by calculus, none of which is the
oracle's own formula retyped."""
import dataclasses
import math

import numpy as np
import pytest

import lp_inputs as LI
import oracle
from oracle import layers as OL
from oracle import local as OLoc


def tiny(name, **over):
    if name == "mlp":
        return LI.configs.mlp_config("t_mlp", n_layers=3, in_dim=5, width=6, hidden=7, n_classes=4,
                                     batch=5, **over)
    if name == "dec":
        kw = dict(n_layers=3, width=8, n_heads=2, hidden=12, seq_len=5, batch=2, vocab=11)
        kw.update(over)
        return LI.configs.decoder_config("t_dec", **kw)
    if name == "res":
        kw = dict(channels=(4, 6, 8), in_hw=6, in_ch=3, n_classes=3, batch=3, n_basic_blocks=1)
        kw.update(over)
        return LI.configs.resnet_config("t_res", **kw)
    raise KeyError(name)


def setup(cfg, seed=3):
    P = LI.perturb_params(LI.init_params(cfg, seed=seed, head_scale=3.0), seed + 1, 0.1)
    if cfg.layers[0].kind == "decoder":   # larger weights so attention / GELU are far from linear
        P = {k: (v * (8.0 if v.ndim == 2 else 1.0)).astype(np.float32) for k, v in P.items()}
    P = {k: v.astype(np.float64) for k, v in P.items()}
    x, y = LI.make_batch(cfg, 0)
    return P, x, y


def fd_check(f, P, names, analytic, n_probe=6, h=1e-6, rtol=2e-6, seed=0):
    """Central differences of scalar f(P) at a few random entries of each named tensor."""
    rng = np.random.default_rng(seed)
    for name in names:
        t = P[name]
        flat = t.reshape(-1)
        idx = rng.choice(flat.size, size=min(n_probe, flat.size), replace=False)
        for i in idx:
            old = flat[i]
            flat[i] = old + h
            fp = f(P)
            flat[i] = old - h
            fm = f(P)
            flat[i] = old
            num = (fp - fm) / (2 * h)
            ana = analytic[name].reshape(-1)[i]
            assert abs(num - ana) <= rtol * max(1.0, abs(num)) + 1e-9, (name, i, num, ana)


@pytest.mark.parametrize("kind", ["mlp", "dec", "res"])
@pytest.mark.parametrize("scheme", ["greedy", "overlap", "chunk"])
def test_p1_finite_differences_per_head(kind, scheme):
    """Every d loss_j / d theta with the window input h_{s_j} held constant is a true gradient."""
    cfg = tiny(kind, scheme=scheme, chunk=2)
    P, x, y = setup(cfg)
    hs, _ = oracle.forward_all(cfg, P, x if kind == "dec" else x.astype(np.float64))
    losses, total, count, each = oracle.local_gradients(cfg, P, x, y, per_head=True)
    for hi, (s, e) in enumerate(LI.head_windows(cfg), start=1):
        h_s = hs[s]

        def f(Pp, hi=hi, h_s=h_s):
            return OLoc.block_gradients(cfg, Pp, hi, h_s, y)[0]

        assert abs(f(P) - losses[hi - 1]) < 1e-12
        fd_check(f, P, sorted(each[hi - 1].keys()), each[hi - 1], n_probe=4, seed=hi)


@pytest.mark.parametrize("kind", ["mlp", "dec", "res"])
def test_p2_truncation_boundary(kind):
    """No head's gradient reaches a layer at or below its window start; with one head and SGD the
    parameters outside the window are bit-unchanged by the step."""
    cfg = tiny(kind, scheme="last1")
    P, x, y = setup(cfg)
    _, grads, _, each = oracle.local_gradients(cfg, P, x, y, per_head=True)
    Lmax = cfg.n_layers
    assert all(k.startswith(f"L{Lmax}.") or k.startswith("H1.") for k in grads)
    # the loss really does depend on the earlier layers (so the zero is the method's, not the data's)
    P2 = {k: v.copy() for k, v in P.items()}
    key = [k for k in P if k.startswith("L1.") and P[k].ndim >= 2][0]
    P2[key] = P2[key] + 0.3 * np.random.default_rng(5).standard_normal(P2[key].shape)
    assert abs(oracle.eval_loss(cfg, P2, x, y)[0] - oracle.eval_loss(cfg, P, x, y)[0]) > 1e-6
    cfg_sgd = dataclasses.replace(cfg, opt=LI.OptCfg("sgd", lr=0.1))
    st = oracle.new_state(cfg_sgd, P)
    _, newP, _ = oracle.local_step(cfg_sgd, P, st, x, y)
    for k in P:
        if k.startswith(f"L{Lmax}.") or k.startswith("H1."):
            assert not np.array_equal(newP[k], P[k]), k
        else:
            assert np.array_equal(newP[k], P[k]), k
    # overlapping scheme: head j contributes nothing to layers <= j-2
    cfg = tiny(kind, scheme="overlap")
    P, x, y = setup(cfg)
    _, _, _, each = oracle.local_gradients(cfg, P, x, y, per_head=True)
    for hi, (s, e) in enumerate(LI.head_windows(cfg), start=1):
        layers_hit = {int(k.split(".")[0][1:]) for k in each[hi - 1] if k.startswith("L")}
        assert layers_hit == set(range(s + 1, e + 1))


@pytest.mark.parametrize("kind", ["mlp", "dec", "res"])
def test_p3_single_block_is_backprop(kind):
    """J = 1 (one head, window = all layers) is ordinary backprop of the final loss: check against
    finite differences of the whole network's loss, input included in nothing."""
    cfg = tiny(kind, scheme="backprop")
    P, x, y = setup(cfg)
    losses, grads, _ = oracle.local_gradients(cfg, P, x, y)
    assert set(grads) == set(P)

    def f(Pp):
        return oracle.eval_loss(cfg, Pp, x, y)[0]

    fd_check(f, P, sorted(P), grads, n_probe=3)


@pytest.mark.parametrize("kind", ["mlp", "dec", "res"])
def test_p4_full_windows_sum_is_deep_supervision(kind):
    """If every head's window reaches layer 1 and contributions are summed, the total is the
    gradient of the single scalar sum_j loss_j."""
    cfg = tiny(kind, scheme="deep_supervision")
    P, x, y = setup(cfg)
    _, grads, _ = oracle.local_gradients(cfg, P, x, y)

    def f(Pp):
        return oracle.eval_loss(cfg, Pp, x, y).sum()

    fd_check(f, P, sorted(P), grads, n_probe=3)


@pytest.mark.parametrize("kind", ["mlp", "dec", "res"])
def test_p5_last_block_matches_backprop(kind):
    """Greedy: the last layer and the last head get exactly the gradients of global backprop
    (section 5: gradients in the last layers are identical to backprop's)."""
    g_cfg = tiny(kind, scheme="greedy")
    b_cfg = tiny(kind, scheme="backprop")
    P, x, y = setup(g_cfg)
    _, gg, _ = oracle.local_gradients(g_cfg, P, x, y)
    Pb = {k: v for k, v in P.items() if not k.startswith("H")}
    nh = len(g_cfg.heads)
    for k, v in P.items():
        if k.startswith(f"H{nh}."):
            Pb["H1." + k.split(".", 1)[1]] = v
    _, gb, _ = oracle.local_gradients(b_cfg, Pb, x, y)
    L = g_cfg.n_layers
    for k in gg:
        if k.startswith(f"L{L}."):
            np.testing.assert_allclose(gg[k], gb[k], rtol=1e-12, atol=1e-15)
        if k.startswith(f"H{nh}."):
            np.testing.assert_allclose(gg[k], gb["H1." + k.split(".", 1)[1]], rtol=1e-12, atol=1e-15)
    # and a middle layer differs (local updates are not proportional to the global gradient)
    k_mid = [k for k in gg if k.startswith("L1.") and gg[k].ndim >= 2][0]
    assert np.linalg.norm(gg[k_mid] - gb[k_mid]) > 1e-3 * np.linalg.norm(gb[k_mid])


def backprop_params(g_cfg, P):
    """The backprop scheme's parameters: the same layers, and the greedy scheme's last head as its only head."""
    Pb = {k: v for k, v in P.items() if not k.startswith("H")}
    nh = len(g_cfg.heads)
    for k, v in P.items():
        if k.startswith(f"H{nh}."):
            Pb["H1." + k.split(".", 1)[1]] = v
    return Pb


@pytest.mark.parametrize("kind", ["mlp", "dec", "res"])
def test_p11_gradient_cosines(kind):
    """Section 5, "Gradient Angles": cosine per layer between greedy local and backprop gradients.  The last
    layer's is exactly 1 (its local gradient is backprop's); the definition is checked on vectors with a known
    angle, and for invariance under positive rescaling of either side."""
    g_cfg = tiny(kind, scheme="greedy")
    b_cfg = tiny(kind, scheme="backprop")
    P, x, y = setup(g_cfg)
    _, gg, _ = oracle.local_gradients(g_cfg, P, x, y)
    _, gb, _ = oracle.local_gradients(b_cfg, backprop_params(g_cfg, P), x, y)
    cos = oracle.layer_gradient_cosines(g_cfg, gg, gb)
    L = g_cfg.n_layers
    assert cos.shape == (L,)
    assert abs(cos[L - 1] - 1.0) <= 1e-12
    assert np.all(np.abs(cos) <= 1.0 + 1e-12)
    assert abs(cos[0]) < 1.0 - 1e-6                      # an early layer is not parallel to backprop's gradient
    # brute force for layer 1: one concatenated vector per side
    a = np.concatenate([gg[k].ravel() for k in sorted(gg) if k.startswith("L1.")])
    b = np.concatenate([gb[k].ravel() for k in sorted(gb) if k.startswith("L1.")])
    assert cos[0] == pytest.approx(float(a @ b) / float(np.sqrt((a @ a) * (b @ b))), rel=1e-12)
    # invariances: rescaling one side, and identical / opposite gradients
    cos2 = oracle.layer_gradient_cosines(g_cfg, {k: 3.5 * v for k, v in gg.items()}, gb)
    np.testing.assert_allclose(cos2, cos, rtol=1e-12)
    np.testing.assert_allclose(oracle.layer_gradient_cosines(g_cfg, gg, gg), 1.0, rtol=1e-12)
    np.testing.assert_allclose(oracle.layer_gradient_cosines(g_cfg, gg, {k: -v for k, v in gg.items()}), -1.0, rtol=1e-12)
    # a known angle: 60 degrees between (1, 0) and (1/2, sqrt(3)/2) spread over two tensors of layer 1
    k1, k2 = sorted(k for k in gg if k.startswith("L1."))[:2]
    ea = {k1: np.zeros_like(gg[k1]), k2: np.zeros_like(gg[k2])}
    eb = {k1: np.zeros_like(gg[k1]), k2: np.zeros_like(gg[k2])}
    ea[k1].flat[0] = 1.0
    eb[k1].flat[0] = 0.5
    eb[k2].flat[0] = np.sqrt(3.0) / 2.0
    assert oracle.layer_gradient_cosines(g_cfg, ea, eb)[0] == pytest.approx(0.5, rel=1e-12)
    # a layer without a gradient on one side gets 0
    assert oracle.layer_gradient_cosines(g_cfg, {k: v for k, v in gg.items() if not k.startswith("L1.")}, gb)[0] == 0.0


@pytest.mark.parametrize("kind", ["mlp", "dec", "res"])
def test_p12_pipelined_schedule(kind):
    """Pipelined form (section 6; section 3, labels travel with the activations).  (a) one block: identical to
    the synchronous step; (b) frozen weights (lr 0): head j in call t reports exactly the synchronous loss of
    minibatch t-j+1, and 0 while the pipeline fills; (c) with updates on, block 2's input in call t is block 1's
    output of call t-1 under the weights block 1 had then (a delay line written out by hand), and a block
    that has not started keeps its weights bit for bit."""
    # (a)
    b_cfg = tiny(kind, scheme="backprop")
    P, x, y = setup(b_cfg)
    st_a, st_b = oracle.new_state(b_cfg, P), oracle.new_state(b_cfg, P)
    pipe = oracle.new_pipeline(b_cfg)
    la, Pa, _ = oracle.local_step(b_cfg, P, st_a, x, y)
    lb, Pb = oracle.pipelined_step(b_cfg, P, st_b, pipe, x, y)
    np.testing.assert_array_equal(la, lb)
    for k in Pa:
        np.testing.assert_array_equal(Pa[k], Pb[k])
    # (b)
    g_cfg = tiny(kind, scheme="greedy")
    frozen = dataclasses.replace(g_cfg, opt=dataclasses.replace(g_cfg.opt, kind="sgd", lr=0.0))
    P, _, _ = setup(frozen)
    J = len(frozen.heads)
    batches = [LI.make_batch(frozen, i) for i in range(J + 2)]
    sync = [oracle.eval_loss(frozen, P, bx, by) for bx, by in batches]
    st, pipe, cur = oracle.new_state(frozen, P), oracle.new_pipeline(frozen), P
    for t, (bx, by) in enumerate(batches, start=1):
        losses, cur = oracle.pipelined_step(frozen, cur, st, pipe, bx, by)
        for j in range(1, J + 1):
            want = sync[t - j][j - 1] if t - j >= 0 else 0.0
            assert losses[j - 1] == pytest.approx(want, rel=1e-13, abs=0.0), (t, j)
    # (c)
    P, _, _ = setup(g_cfg)
    st, pipe = oracle.new_state(g_cfg, P), oracle.new_pipeline(g_cfg)
    (x1, y1), (x2, y2) = LI.make_batch(g_cfg, 0), LI.make_batch(g_cfg, 1)
    l1, P1 = oracle.pipelined_step(g_cfg, P, st, pipe, x1, y1)
    assert np.all(l1[1:] == 0.0)
    for k in P:
        if not (k.startswith("L1.") or k.startswith("H1.")):
            np.testing.assert_array_equal(P1[k], np.asarray(P[k], np.float64))     # blocks 2.. have not started
    l2, P2 = oracle.pipelined_step(g_cfg, P1, st, pipe, x2, y2)
    # by hand: block 1's output on minibatch 1 under the ORIGINAL weights feeds block 2 now, with labels y1
    _, _, a1 = oracle.block_gradients(g_cfg, P, 1, x1, y1)
    loss2, grads2, _ = oracle.block_gradients(g_cfg, P1, 2, a1, y1)
    assert l2[1] == pytest.approx(loss2, rel=1e-14)
    st_hand = oracle.new_state(g_cfg, P)
    for k, g in grads2.items():
        np.testing.assert_allclose(P2[k], oracle.optimizer_update(g_cfg.opt, np.asarray(P1[k], np.float64), g, st_hand, k, 1),
                                   rtol=1e-14, atol=0)
    # ... and not the output under the updated weights (the input really is one call stale)
    _, _, a1_new = oracle.block_gradients(g_cfg, P1, 1, x1, y1)
    assert np.linalg.norm(a1_new - a1) > 1e-9 * np.linalg.norm(a1)
    # block 1 meanwhile works on minibatch 2
    assert l2[0] == pytest.approx(oracle.block_gradients(g_cfg, P1, 1, x2, y2)[0], rel=1e-14)


def test_p13_paper_form_resnet_head():
    """Appendix B.3's auxiliary head (batch norm, ReLU, spatial mean, linear): finite differences of the head's
    own parameters and of the block below it; a whole network with this head against torch autograd."""
    import torch
    cfg = tiny("res", head="bn_pool_linear_ce")
    P, x, y = setup(cfg)
    assert "H1.bn.g" in P and "H1.bn.b" in P
    losses, grads, _ = oracle.local_gradients(cfg, P, x, y)
    for hi in (1, 3):
        s, e = LI.head_windows(cfg)[hi - 1]
        names = [k for k in P if k.startswith(f"H{hi}.") or k.startswith(f"L{e}.")]

        def f(Pq, hi=hi):
            return oracle.eval_loss(cfg, Pq, x, y)[hi - 1]
        fd_check(f, P, names, grads, n_probe=4, h=1e-6, rtol=5e-6)
    # library pin: the head alone in torch (batch_norm in training mode, relu, mean, linear, cross_entropy)
    hs, _ = oracle.forward_all(cfg, P, x)
    h1 = torch.tensor(hs[1], dtype=torch.float64, requires_grad=True)
    w = torch.tensor(P["H1.w"], dtype=torch.float64, requires_grad=True)
    b = torch.tensor(P["H1.b"], dtype=torch.float64, requires_grad=True)
    gg = torch.tensor(P["H1.bn.g"], dtype=torch.float64, requires_grad=True)
    bb = torch.tensor(P["H1.bn.b"], dtype=torch.float64, requires_grad=True)
    a = torch.nn.functional.batch_norm(h1.permute(0, 3, 1, 2), None, None, gg, bb, training=True, eps=1e-5)
    feat = torch.relu(a).mean(dim=(2, 3))
    loss = torch.nn.functional.cross_entropy(feat @ w.T + b, torch.tensor(y, dtype=torch.long))
    loss.backward()
    # (torch's CPU batch_norm keeps some statistics in single precision even for double inputs)
    assert float(loss) == pytest.approx(losses[0], rel=1e-7)
    np.testing.assert_allclose(grads["H1.w"], w.grad.numpy(), rtol=1e-5, atol=1e-8)
    np.testing.assert_allclose(grads["H1.bn.g"], gg.grad.numpy(), rtol=1e-5, atol=1e-8)
    np.testing.assert_allclose(grads["H1.bn.b"], bb.grad.numpy(), rtol=1e-5, atol=1e-8)


def test_p6_overlap_bookkeeping():
    """Overlapping scheme (appendix A.2): two backward passes for each non-terminal layer, one
    for the terminal layer: 2L-1 (head, layer) pairs; mean = sum / coverage."""
    cfg = tiny("dec", scheme="overlap", n_layers=4)
    P, x, y = setup(cfg)
    _, gsum, count, each = oracle.local_gradients(cfg, P, x, y, per_head=True)
    L = cfg.n_layers
    pairs = sum(len({int(k.split(".")[0][1:]) for k in g if k.startswith("L")}) for g in each)
    assert pairs == 2 * L - 1
    for k, c in count.items():
        if k.startswith("H") or k.startswith(f"L{L}."):
            assert c == 1
        else:
            assert c == 2
    cfg_m = dataclasses.replace(cfg, combine="mean")
    _, gmean, _ = oracle.local_gradients(cfg_m, P, x, y)
    for k in gsum:
        np.testing.assert_allclose(gmean[k] * count[k], gsum[k], rtol=1e-13)
    # the sum over two heads differs from either contribution alone
    k = "L2.w1"
    assert np.linalg.norm(gsum[k] - each[1][k]) > 1e-6


@pytest.mark.parametrize("kind,C", [("mlp", 4), ("dec", 11), ("res", 3)])
def test_p7_zero_head_closed_form(kind, C):
    """Head weights = 0 => every loss is exactly ln(C) and dZ = (1/C - onehot)/N."""
    cfg = tiny(kind)
    P, x, y = setup(cfg)
    for k in P:
        if k.startswith("H") and k.split(".")[-1] in ("w", "b"):
            P[k] = np.zeros_like(P[k])
    losses, grads, _ = oracle.local_gradients(cfg, P, x, y)
    np.testing.assert_allclose(losses, math.log(C), rtol=1e-14)
    # with W = 0 nothing flows into the blocks
    for k, g in grads.items():
        if k.startswith("L"):
            assert np.all(g == 0), k
    # head bias gradient = mean(1/C - onehot)
    if cfg.heads[0].bias:
        yy = y.reshape(-1)
        expect = np.full(C, 1.0 / C) - np.bincount(yy, minlength=C) / yy.size
        np.testing.assert_allclose(grads["H1.b"], expect, rtol=1e-12, atol=1e-15)


def test_p9_chunk_is_backprop_on_subnetwork():
    """A chunk of K layers with one head = backprop on that K-layer network fed h_s as data."""
    cfg = tiny("dec", scheme="chunk", chunk=2, n_layers=4)
    P, x, y = setup(cfg)
    hs, _ = oracle.forward_all(cfg, P, x)
    _, grads, _ = oracle.local_gradients(cfg, P, x, y)
    # second chunk = layers 3..4 as a stand-alone 2-layer network without an embedding
    sub = LI.configs.decoder_config("sub", n_layers=2, width=8, n_heads=2, hidden=12, seq_len=5,
                                    batch=2, vocab=11, scheme="backprop")
    sub = dataclasses.replace(sub, vocab=0)
    Ps = {}
    for k, v in P.items():
        if k.startswith("L3."):
            Ps["L1." + k[3:]] = v
        if k.startswith("L4."):
            Ps["L2." + k[3:]] = v
        if k.startswith("H2."):
            Ps["H1." + k[3:]] = v
    _, gs, _ = oracle.local_gradients(sub, Ps, hs[2], y)

    def f(Pp):
        return oracle.eval_loss(sub, Pp, hs[2], y)[0]

    fd_check(f, Ps, sorted(Ps), gs, n_probe=2)
    for k, v in gs.items():
        kk = k.replace("L1.", "L3.").replace("L2.", "L4.").replace("H1.", "H2.")
        np.testing.assert_allclose(grads[kk], v, rtol=1e-12, atol=1e-15)


def test_p10_eval_equals_step_losses_and_uncovered_layers_keep_state():
    cfg = tiny("res", scheme="last1")
    P, x, y = setup(cfg)
    st = oracle.new_state(cfg, P)
    losses, newP, grads = oracle.local_step(cfg, P, st, x, y)
    np.testing.assert_allclose(losses, oracle.eval_loss(cfg, P, x, y), rtol=1e-14)
    assert st["t"] == 1
    for k in P:
        if k not in grads:
            assert np.all(st["m"][k] == 0)


def test_zipf_generator_matches_law():
    """The token generator follows the truncated Zipf(1.1) law it claims (shape of LM1B stand-in)."""
    pmf = LI.zipf_pmf(32000, 1.1)
    assert abs(pmf.sum() - 1) < 1e-12
    assert abs(pmf[0] - 0.1420) < 5e-4 and abs(pmf[1] - 0.0663) < 5e-4
    assert abs(pmf[:10].sum() - 0.381) < 2e-3
    ids = LI.zipf_tokens(np.random.default_rng(0), (64, 1024), 32000)
    assert ids.min() >= 0 and ids.max() < 32000
    assert abs((ids == 0).mean() - pmf[0]) < 5e-3
