"""Parity at the full benchmark sizes, in the launch configuration bench.py times.

The whole-step oracle at these sizes would take minutes of float64 BLAS, so each transformer
configuration is checked block by block: the input of a block is detached by definition (section
3: a block receives the previous block's output as data), so the oracle is fed the device's own
activation entering the sampled block and must then reproduce that block's loss, every gradient
inside its window and the updated weights.  Blocks are sampled at both ends of the network.  The
ResNet configuration is small enough for the whole step."""
import dataclasses
import time

import numpy as np
import pytest

import lp_inputs as LI
import oracle
from oracle import local as OL

pytestmark = [pytest.mark.gpu, pytest.mark.timeout(900)]

from gpu_util import bf16_round, data_for, relerr, updated_param_err  # noqa: E402


@pytest.fixture(scope="module")
def lpmod():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2012_03837_amd as lp
    return lp


def block_names(cfg, hi):
    s, e = LI.head_windows(cfg)[hi - 1]
    names = [k for k in LI.param_shapes(cfg) if k.startswith(f"H{hi}.")
             or (k[0] == "L" and s < int(k.split(".")[0][1:]) <= e)]
    return s, e, names


def check_block(lpmod, tr, cfg, hi, x, y, P_before, tol=2e-2):
    """Oracle on one block, fed the device's activation entering the block."""
    s, e, names = block_names(cfg, hi)
    h_s = x if s == 0 else tr.get(f"L{s}.out").astype(np.float64)
    t0 = time.time()
    ref_loss, grads, h_e = oracle.block_gradients(cfg, P_before, hi, h_s, y)
    print(f"  oracle block {hi} (layers {s + 1}..{e}) took {time.time() - t0:.1f} s", flush=True)
    got_loss = float(tr.losses.cpu().numpy()[hi - 1])
    assert abs(got_loss - ref_loss) <= tol * abs(ref_loss), (hi, got_loss, ref_loss)
    assert relerr(tr.get(f"L{e}.out"), h_e) <= tol
    worst = 0.0
    st = oracle.new_state(cfg, {k: P_before[k] for k in names})
    for k in names:
        g = tr.get(k + ".grad")
        err = relerr(g, grads[k])
        worst = max(worst, err)
        assert err <= tol, (hi, k, "grad", err)
        newp = OL.optimizer_update(cfg.opt, P_before[k].astype(np.float64), grads[k], st, k, 1)
        assert updated_param_err(tr.get(k), newp, grads[k], cfg.opt.kind) <= tol, (hi, k, "param")
        if "m" in st:
            assert relerr(tr.get(k + ".m"), st["m"][k]) <= 2 * tol, (hi, k, "m")
        if "v" in st:
            assert relerr(tr.get(k + ".v"), st["v"][k]) <= 2 * tol, (hi, k, "v")
    print(f"  block {hi}: loss {got_loss:.5f} vs {ref_loss:.5f}, worst grad rel err {worst:.4f}", flush=True)


def run_transformer(lpmod, name, sample_heads, single_contribution_only=True):
    cfg = LI.make_config(name)
    print(f"[case] {name} full size", flush=True)
    tr = lpmod.LocalTrainer(cfg, n_streams=lpmod.default_side_streams(cfg))   # the launch configuration bench.py times
    x, y = data_for(cfg)
    xd, yd = tr.stage(x, y)
    wanted = set()
    for hi in sample_heads:
        wanted |= set(block_names(cfg, hi)[2])
    P_before = {k: tr.get(k) for k in sorted(wanted)}
    ev = tr.eval(xd, yd).cpu().numpy().copy()
    got = tr.step(xd, yd).cpu().numpy().copy()
    np.testing.assert_array_equal(ev, got)
    assert np.all(np.isfinite(got))
    # at initialisation every head predicts close to uniformly: loss near ln(vocab) for all heads
    assert np.all(np.abs(got - np.log(cfg.vocab)) < 0.5), got
    for hi in sample_heads:
        check_block(lpmod, tr, cfg, hi, x, y, P_before)
    tr.close()


def test_cfg3_full_blocks(lpmod):
    run_transformer(lpmod, "cfg3", [1, 12])


def test_cfg4_full_last_block(lpmod):
    """Overlapping windows at full size: the last layer and the last head receive one contribution
    only (head 12 through layers 11..12), so they can be compared block-wise; layer 11 also gets
    head 11's contribution and is covered by the scaled-down overlap tests."""
    cfg = LI.make_config("cfg4")
    print("[case] cfg4 full size", flush=True)
    tr = lpmod.LocalTrainer(cfg, n_streams=lpmod.default_side_streams(cfg))   # the launch configuration bench.py times
    x, y = data_for(cfg)
    xd, yd = tr.stage(x, y)
    hi = 12
    s, e, names = block_names(cfg, hi)
    P_before = {k: tr.get(k) for k in names}
    tr.step(xd, yd)
    h_s = tr.get(f"L{s}.out").astype(np.float64)
    ref_loss, grads, _ = oracle.block_gradients(cfg, P_before, hi, h_s, y)
    got_loss = float(tr.losses.cpu().numpy()[hi - 1])
    assert abs(got_loss - ref_loss) <= 2e-2 * abs(ref_loss)
    for k in names:
        if k.startswith("H12.") or k.startswith("L12."):
            assert relerr(tr.get(k + ".grad"), grads[k]) <= 2e-2, k
    # layer 11: the device holds the sum of two contributions, which must differ from head 12's alone
    k = "L11.w1"
    assert relerr(tr.get(k + ".grad"), grads[k]) > 5e-2
    tr.close()


def test_cfg5_full_first_chunk(lpmod):
    run_transformer(lpmod, "cfg5", [1])


def test_cfg2_full_step(lpmod):
    """The ResNet configuration at full size.  End to end (oracle fed only x, y and the initial
    weights): every loss and every head gradient.  Stage by stage (oracle fed the device's own
    activation entering the stage, which the method treats as data): every gradient, updated
    weight and momentum inside the stage.  ReLU decisions are taken on the stored bf16 activations
    on both sides.  In-stage gradients are held to 3.5e-2 instead of 2e-2: with bf16 activations a
    fraction f of 1e-4 .. 3e-4 of the ReLU units of a stage decide differently on the two sides however
    the kernels are written (one-ulp rounding differences spread through a convolution stack), each
    flipped unit moves its gradient entry by O(1), and that alone is a relative error of sqrt(2 f),
    1.4 .. 2.5 %, on top of the bf16 rounding of the backward activations (measured worst: 3.05 % on one
    BatchNorm shift of stage 4, whose 4x4 maps leave the fewest units to average over).
    A whole-network element-wise comparison of the convolution gradients is not
    meaningful in bf16: one-ulp rounding differences flip ReLU units a few layers on, and a flipped
    unit changes a gradient entry by O(1), so the two sides drift apart with depth although each
    stage is reproduced to well under a percent."""
    cfg = LI.make_config("cfg2")
    print("[case] cfg2 full size", flush=True)
    tr = lpmod.LocalTrainer(cfg, n_streams=lpmod.default_side_streams(cfg))   # the launch configuration bench.py times
    P0 = LI.init_params(cfg)
    tr.set_params(P0)
    x, y = data_for(cfg)
    xd, yd = tr.stage(x, y)
    got = tr.step(xd, yd).cpu().numpy().copy()
    P64 = {k: v.astype(np.float64) for k, v in P0.items()}
    t0 = time.time()
    ref, newP, grads = oracle.local_step(cfg, P64, oracle.new_state(cfg, P0), x, y, stored="bf16")
    print(f"  oracle whole step took {time.time() - t0:.1f} s", flush=True)
    assert np.all(np.abs(got - ref) <= 2e-2 * np.abs(ref)), (got, ref)
    for k in P0:
        if k.startswith("H"):
            assert relerr(tr.get(k + ".grad"), grads[k]) <= 2e-2, k
            assert relerr(tr.get(k), newP[k]) <= 2e-2, k
    worst = 0.0
    for hi in range(1, len(cfg.heads) + 1):
        s, e, names = block_names(cfg, hi)
        h_s = x if s == 0 else tr.get(f"L{s}.out").astype(np.float64)
        loss, g, h_e = oracle.block_gradients(cfg, P64, hi, h_s, y, stored="bf16")
        assert abs(got[hi - 1] - loss) <= 2e-2 * abs(loss)
        assert relerr(tr.get(f"L{e}.out"), h_e) <= 2e-2
        st = oracle.new_state(cfg, {k: P64[k] for k in names})
        stage_worst = 0.0
        for k in names:
            err = relerr(tr.get(k + ".grad"), g[k])
            worst = max(worst, err)
            stage_worst = max(stage_worst, err)
            assert err <= 3.5e-2, (hi, k, err)
            newp = OL.optimizer_update(cfg.opt, P64[k], g[k], st, k, 1)
            # zero-initialised shifts: the updated value is -lr * g, so it carries the gradient's error
            assert relerr(tr.get(k), newp) <= 3.5e-2, (hi, k)
            assert relerr(tr.get(k + ".m"), st["m"][k]) <= 3.5e-2, (hi, k)
        print(f"  stage {hi}: worst grad rel err {stage_worst:.4f}", flush=True)
    print("  worst per-stage grad rel err", worst, flush=True)
    tr.close()
