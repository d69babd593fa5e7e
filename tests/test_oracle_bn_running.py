"""Pins for the oracle's running batch-normalisation statistics (the evaluation form of the batch
normalisation that appendix B.3 cites).  The paper fixes no convention; the oracle takes the usual one
(exponential moving average, unbiased batch variance, start at mean 0 / variance 1), so the pins are
an independent library module that implements that convention, a closed form, and invariants."""
import numpy as np
import pytest
import torch

import lp_inputs as LI
import oracle
from oracle import ops as O


def _res(head="bn_pool_linear_ce", **over):
    kw = dict(channels=(4, 6, 8), in_hw=6, in_ch=3, n_classes=3, batch=4, n_basic_blocks=1, head=head)
    kw.update(over)
    return LI.configs.resnet_config("t_res", **kw)


def _params(cfg, seed=3):
    P = LI.perturb_params(LI.init_params(cfg, seed=seed, head_scale=3.0), seed + 1, 0.1)
    return {k: v.astype(np.float64) for k, v in P.items()}


def _bn_prefixes(P):
    out = set()
    for k in P:
        parts = k.split(".")
        if parts[-1] == "g" and parts[-2].startswith("bn"):
            out.add(k[:-1])
    return out


@pytest.mark.parametrize("momentum", [0.1, 0.37, 1.0])
def test_running_statistics_match_library_module(momentum):
    """Three training batches through torch's BatchNorm2d (NCHW) and through the oracle (NHWC), then one
    evaluation batch: running mean, running variance and the evaluation output agree."""
    rng = np.random.default_rng(0)
    C = 5
    g = rng.normal(1.0, 0.3, C)
    b = rng.normal(0.0, 0.3, C)
    mod = torch.nn.BatchNorm2d(C, eps=O.BN_EPS, momentum=momentum).double()
    with torch.no_grad():
        mod.weight.copy_(torch.from_numpy(g))
        mod.bias.copy_(torch.from_numpy(b))
    run = O.BatchNormRunning(momentum, "update")
    mod.train()
    for i in range(3):
        x = rng.normal(0.5 * i, 1.0 + i, (3, 4, 2, C))
        y_lib = mod(torch.from_numpy(x).permute(0, 3, 1, 2)).permute(0, 2, 3, 1).detach().numpy()
        y, _ = O.batchnorm(x, g, b, run, "u.")
        np.testing.assert_allclose(y, y_lib, rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(run.mean["u."], mod.running_mean.numpy(), rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(run.var["u."], mod.running_var.numpy(), rtol=1e-12, atol=1e-14)
    mod.eval()
    run.mode = "use"
    x = rng.normal(0.0, 2.0, (2, 3, 3, C))
    y_lib = mod(torch.from_numpy(x).permute(0, 3, 1, 2)).permute(0, 2, 3, 1).detach().numpy()
    y, cache = O.batchnorm(x, g, b, run, "u.")
    assert cache is None
    np.testing.assert_allclose(y, y_lib, rtol=1e-10, atol=1e-12)


def test_running_statistics_closed_form_on_a_repeated_batch():
    """The same batch t times: run_mean = (1 - (1-m)^t) mean, run_var = (1-m)^t + (1 - (1-m)^t) var_unbiased."""
    rng = np.random.default_rng(1)
    x = rng.normal(2.0, 3.0, (6, 2, 2, 4))
    m, t = 0.2, 7
    run = O.BatchNormRunning(m, "update")
    for _ in range(t):
        run.observe("a.", x)
    keep = (1.0 - m) ** t
    x2 = x.reshape(-1, 4)
    np.testing.assert_allclose(run.mean["a."], (1 - keep) * x2.mean(axis=0), rtol=1e-12)
    np.testing.assert_allclose(run.var["a."], keep + (1 - keep) * x2.var(axis=0, ddof=1), rtol=1e-12)


@pytest.mark.parametrize("head", ["pool_linear_ce", "bn_pool_linear_ce"])
def test_one_update_per_normalisation_per_step(head):
    """After one step with momentum 1 every batch normalisation of the model (and of the heads) holds the
    statistics of exactly one batch: the mean of its own input, which for the stem is computable directly."""
    cfg = _res(head)
    P = _params(cfg)
    x, y = LI.make_batch(cfg, 0)
    run = O.BatchNormRunning(1.0)
    oracle.local_gradients(cfg, P, x.astype(np.float64), y, bn=run)
    assert set(run.mean) == _bn_prefixes(P)
    z = O.conv2d_fwd(x.astype(np.float64), P["L1.stem.w"], 1, 1).reshape(-1, cfg.layers[0].out_ch)
    np.testing.assert_allclose(run.mean["L1.stem.bn."], z.mean(axis=0), rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(run.var["L1.stem.bn."], z.var(axis=0, ddof=1), rtol=1e-10)
    # overlapping windows evaluate a layer's forward once, so its statistics are still folded in once
    cfg2 = _res(head, scheme="overlap")
    run2 = O.BatchNormRunning(0.25)
    oracle.local_gradients(cfg2, _params(cfg2), x.astype(np.float64), y, bn=run2)
    np.testing.assert_allclose(run2.mean["L1.stem.bn."], 0.25 * z.mean(axis=0), rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(run2.var["L1.stem.bn."], 0.75 + 0.25 * z.var(axis=0, ddof=1), rtol=1e-10)


class _ExactBatch(O.BatchNormRunning):
    """Keeps the biased statistics of the last batch, so that normalising with them repeats batch mode."""

    def observe(self, name, x):
        x2 = np.asarray(x, dtype=np.float64).reshape(-1, x.shape[-1])
        self.mean[name] = x2.mean(axis=0)
        self.var[name] = x2.var(axis=0)


@pytest.mark.parametrize("head", ["pool_linear_ce", "bn_pool_linear_ce"])
def test_evaluation_with_the_batch_s_own_statistics_repeats_batch_mode(head):
    cfg = _res(head)
    P = _params(cfg)
    x, y = LI.make_batch(cfg, 0)
    x = x.astype(np.float64)
    run = _ExactBatch(1.0)
    oracle.local_gradients(cfg, P, x, y, bn=run)
    want = oracle.eval_loss(cfg, P, x, y)
    got = oracle.eval_loss(cfg, P, x, y, bn=run)
    np.testing.assert_allclose(got, want, rtol=1e-9)
    # and it is a different function of the input once the batch changes: the running form normalises each
    # sample independently of the others
    x2, y2 = LI.make_batch(cfg, 1)
    x2 = x2.astype(np.float64)
    whole = oracle.eval_loss(cfg, P, x2, y2, bn=run)
    n = x2.shape[0]
    per = np.mean([oracle.eval_loss(cfg, P, x2[i:i + 1], y2[i:i + 1], bn=run) for i in range(n)], axis=0)
    np.testing.assert_allclose(whole, per, rtol=1e-9)


def test_evaluation_leaves_the_running_statistics_alone_and_steps_move_them():
    cfg = _res()
    P = _params(cfg)
    st = oracle.new_state(cfg, P)
    run = O.BatchNormRunning(0.1)
    x, y = LI.make_batch(cfg, 0)
    _, P1, _ = oracle.local_step(cfg, P, st, x.astype(np.float64), y, bn=run)
    snap = {k: v.copy() for k, v in run.mean.items()}
    oracle.eval_loss(cfg, P1, x.astype(np.float64), y, bn=run)
    for k in snap:
        np.testing.assert_array_equal(run.mean[k], snap[k])
    x, y = LI.make_batch(cfg, 1)
    oracle.local_step(cfg, P1, st, x.astype(np.float64), y, bn=run)
    assert any(np.abs(run.mean[k] - snap[k]).max() > 0 for k in snap)
