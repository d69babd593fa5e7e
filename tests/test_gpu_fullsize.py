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
            assert relerr(tr.get(k + ".m"), st["m"][k]) <= tol, (hi, k, "m")
        if "v" in st:
            assert relerr(tr.get(k + ".v"), st["v"][k]) <= tol, (hi, k, "v")
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
    head_params = {k: tr.get(k) for k in tr.names() if k.startswith("H")}
    ev = tr.eval(xd, yd).cpu().numpy().copy()
    got = tr.step(xd, yd).cpu().numpy().copy()
    np.testing.assert_array_equal(ev, got)
    assert np.all(np.isfinite(got))
    # at initialisation every head predicts close to uniformly: loss near ln(vocab) for all heads
    assert np.all(np.abs(got - np.log(cfg.vocab)) < 0.5), got
    for hi in sample_heads:
        check_block(lpmod, tr, cfg, hi, x, y, P_before)
    # every head's loss against the oracle's head (LayerNorm, projection to the vocabulary, cross-entropy over all
    # 8192 positions in float64) on the device's activation entering the head
    from oracle import layers as OLay
    t0 = time.time()
    for hi in range(1, len(cfg.heads) + 1):
        if hi in sample_heads:
            continue                                   # compared above, together with its gradients
        e = cfg.heads[hi - 1].after_layer
        Ph = {k: head_params[k].astype(np.float64) for k in head_params if k.startswith(f"H{hi}.")}
        ref, _ = OLay.head_loss(cfg, Ph, hi, tr.get(f"L{e}.out").astype(np.float64), y)
        assert abs(got[hi - 1] - ref) <= 2e-2 * abs(ref), (hi, got[hi - 1], ref)
        print(f"  head {hi}: loss {got[hi - 1]:.5f} vs {ref:.5f}", flush=True)
    print(f"  oracle head losses took {time.time() - t0:.1f} s", flush=True)
    tr.close()


def test_cfg3_full_blocks(lpmod):
    run_transformer(lpmod, "cfg3", [1, 12])


def test_cfg4_full_overlapped_layer(lpmod):
    """Overlapping windows at full size (appendix A.2: every non-terminal layer takes two backward passes).  Heads
    11 and 12 are differentiated separately by the oracle, each fed the device's activation entering its window
    (layer 9's output for head 11, layer 10's for head 12).  Layer 11 lies in both windows: the device's gradient
    (second contribution accumulated onto the first, ordered across the side streams), its updated weights and
    Adam moments (one update, issued when the second contribution has arrived) must equal the oracle's sum.
    Layer 12 and both heads receive a single contribution."""
    cfg = LI.make_config("cfg4")
    print("[case] cfg4 full size", flush=True)
    tr = lpmod.LocalTrainer(cfg, n_streams=lpmod.default_side_streams(cfg))   # the launch configuration bench.py times
    x, y = data_for(cfg)
    xd, yd = tr.stage(x, y)
    names = set()
    for hi in (11, 12):
        names |= set(block_names(cfg, hi)[2])
    P_before = {k: tr.get(k) for k in sorted(names)}
    tr.step(xd, yd)
    got = tr.losses.cpu().numpy().copy()
    contrib = {}
    for hi in (11, 12):
        s, e, _ = block_names(cfg, hi)
        assert (s, e) == (hi - 2, hi)
        t0 = time.time()
        ref_loss, grads, _ = oracle.block_gradients(cfg, P_before, hi, tr.get(f"L{s}.out").astype(np.float64), y)
        print(f"  oracle head {hi} (layers {s + 1}..{e}) took {time.time() - t0:.1f} s", flush=True)
        assert abs(got[hi - 1] - ref_loss) <= 2e-2 * abs(ref_loss), (hi, got[hi - 1], ref_loss)
        contrib[hi] = grads
    total = {}
    for k in P_before:
        if k.startswith("L11."):
            total[k] = contrib[11][k] + contrib[12][k]          # cfg4 combines by summation
        elif k.startswith("L12.") or k.startswith("H12."):
            total[k] = contrib[12][k]
        elif k.startswith("H11."):
            total[k] = contrib[11][k]
    st = oracle.new_state(cfg, {k: P_before[k] for k in total})
    worst = 0.0
    for k, g in total.items():
        err = relerr(tr.get(k + ".grad"), g)
        worst = max(worst, err)
        assert err <= 2e-2, (k, "grad", err)
        newp = OL.optimizer_update(cfg.opt, P_before[k].astype(np.float64), g, st, k, 1)
        assert updated_param_err(tr.get(k), newp, g, cfg.opt.kind) <= 2e-2, (k, "param")
        assert relerr(tr.get(k + ".m"), st["m"][k]) <= 2e-2, (k, "m")
        assert relerr(tr.get(k + ".v"), st["v"][k]) <= 2e-2, (k, "v")
    # the two contributions are of the same size: a lost or doubled one cannot hide inside the tolerance
    k = "L11.w1"
    assert relerr(contrib[12][k], total[k]) > 0.2 and relerr(contrib[11][k], total[k]) > 0.2
    print(f"  layers 11..12, heads 11..12: worst grad rel err {worst:.4f}", flush=True)
    tr.close()


def test_cfg5_full_first_and_last_chunk(lpmod):
    """Chunk 1 (with the token embedding) and chunk 6 (layers 21..24: input gradients chained through four layers,
    no embedding) of the 24-layer configuration, and every chunk head's loss."""
    run_transformer(lpmod, "cfg5", [1, 6])


def test_cfg2_full_step(lpmod):
    """The ResNet configuration at full size against the EXACT float64 oracle (no storage rounding on the oracle's
    side).  End to end (oracle fed only x, y and the initial weights): every head's loss.  Block by block (oracle
    fed the device's stage output): loss and the head's gradients.  Unit by unit (oracle fed the device's own
    unit input, shortcut input and upstream gradient, all of which the method or the chain rule treat as given):
    convolution output, unit output, the three parameter gradients, the input gradient, updated weights and
    momentum of every convolution + normalisation unit, each to 2e-2; the tensors that tie the units together
    are compared bit for bit on the device (see gpu_util.check_resnet_stage_by_unit)."""
    cfg = LI.make_config("cfg2")
    print("[case] cfg2 full size", flush=True)
    from gpu_util import check_resnet_stage_by_unit
    tr = lpmod.LocalTrainer(cfg, n_streams=lpmod.default_side_streams(cfg), debug=True)   # bench.py's launch configuration
    P0 = LI.init_params(cfg)
    tr.set_params(P0)
    x, y = data_for(cfg)
    xd, yd = tr.stage(x, y)
    got = tr.step(xd, yd).cpu().numpy().copy()
    t0 = time.time()
    ref = oracle.eval_loss(cfg, {k: v.astype(np.float64) for k, v in P0.items()}, x, y)
    print(f"  oracle forward took {time.time() - t0:.1f} s; losses {got} vs {ref}", flush=True)
    assert np.all(np.abs(got - ref) <= 2e-2 * np.abs(ref)), (got, ref)
    worst = 0.0
    for hi in range(1, len(cfg.heads) + 1):
        t0 = time.time()
        w = check_resnet_stage_by_unit(tr, cfg, hi, P0, x, y, 2e-2, label="cfg2")
        print(f"  stage {hi}: worst rel err over all unit tensors {w:.4f} ({time.time() - t0:.1f} s)", flush=True)
        worst = max(worst, w)
    print("  worst rel err", worst, flush=True)
    tr.close()


def test_cfg3_full_pipelined_grouped_blocks(lpmod):
    """The pipelined schedule at full size, where the blocks of a call are walked in lockstep and their same-shaped
    products share grouped launches.  Block 4 runs for the first time in call 4, with its initial weights, on the
    activation block 3 produced in call 3 and the labels of minibatch 1, beside blocks 1..3 (already updated, on
    younger minibatches): the oracle, fed that activation as data, must reproduce block 4's loss, gradients,
    updated weights and Adam moments; the same for block 1 on the call's own minibatch."""
    cfg = LI.make_config("cfg3")
    print("[case] cfg3 full size, pipelined", flush=True)
    tr = lpmod.LocalTrainer(cfg, schedule="pipelined_grouped", n_streams=lpmod.default_side_streams(cfg))
    names4 = block_names(cfg, 4)[2]
    P4 = {k: tr.get(k) for k in names4}
    batches = [data_for(cfg, t) for t in range(4)]
    for t in range(3):
        got = tr.step(*tr.stage(*batches[t])).cpu().numpy().copy()
        assert np.all(got[t + 1:] == 0.0) and np.all(got[:t + 1] > 0.0), got
    h3 = tr.get("L3.out").astype(np.float64)            # what block 4 reads in the next call
    names1 = block_names(cfg, 1)[2]
    P1 = {k: tr.get(k) for k in names1}                 # block 1 after three updates
    m1 = {k: tr.get(k + ".m").astype(np.float64) for k in names1}
    v1 = {k: tr.get(k + ".v").astype(np.float64) for k in names1}
    got = tr.step(*tr.stage(*batches[3])).cpu().numpy().copy()
    # block 4: first update, labels of minibatch 1
    y1 = batches[0][1]
    ref_loss, grads, _ = oracle.block_gradients(cfg, P4, 4, h3, y1)
    assert abs(got[3] - ref_loss) <= 2e-2 * abs(ref_loss), (got[3], ref_loss)
    st = oracle.new_state(cfg, P4)
    worst = 0.0
    for k in names4:
        err = relerr(tr.get(k + ".grad"), grads[k])
        worst = max(worst, err)
        assert err <= 2e-2, (k, err)
        newp = OL.optimizer_update(cfg.opt, P4[k].astype(np.float64), grads[k], st, k, 1)
        assert updated_param_err(tr.get(k), newp, grads[k], cfg.opt.kind) <= 2e-2, k
        assert relerr(tr.get(k + ".m"), st["m"][k]) <= 2e-2 and relerr(tr.get(k + ".v"), st["v"][k]) <= 2e-2, k
    # block 1: fourth update, on the call's own minibatch
    x4, y4 = batches[3]
    ref_loss, grads, _ = oracle.block_gradients(cfg, P1, 1, x4, y4)
    assert abs(got[0] - ref_loss) <= 2e-2 * abs(ref_loss), (got[0], ref_loss)
    st = {"t": 3, "m": m1, "v": v1}
    for k in names1:
        err = relerr(tr.get(k + ".grad"), grads[k])
        worst = max(worst, err)
        assert err <= 2e-2, (k, err)
        OL.optimizer_update(cfg.opt, P1[k].astype(np.float64), grads[k], st, k, 4)
        assert relerr(tr.get(k + ".m"), st["m"][k]) <= 2e-2 and relerr(tr.get(k + ".v"), st["v"][k]) <= 2e-2, k
    print(f"  pipelined call 4, blocks 4 and 1: worst grad rel err {worst:.4f}", flush=True)
    tr.close()
