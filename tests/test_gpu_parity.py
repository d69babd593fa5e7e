"""GPU parity: lp_local_step / lp_eval_loss through the C ABI against the CPU oracle, element by
element (per-tensor relative L2 error) on scaled-down forms of the five configurations: sizes the
oracle finishes in seconds, ragged with respect to every kernel tile."""
import dataclasses

import numpy as np
import pytest

import lp_inputs as LI
import oracle

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def lpmod():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2012_03837_amd as lp
    return lp


from gpu_util import (check_resnet_stage_by_unit, compare_step, data_for, generic_params, relerr, stored_for,  # noqa: E402
                      tol_for)


SMALL = ["cfg1_small", "cfg2_small", "cfg3_small", "cfg4_small", "cfg5_small"]


@pytest.mark.parametrize("name", SMALL)
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_local_step_matches_oracle(lpmod, name, dtype):
    if name == "cfg1_small" and dtype == "bf16":
        pytest.skip("the residual-MLP configuration is an fp32 configuration")
    cfg = dataclasses.replace(LI.make_config(name), dtype=dtype)
    print(f"[case] {name} {dtype}", flush=True)
    tr = lpmod.LocalTrainer(cfg)
    x, y = data_for(cfg)
    worst = compare_step(tr, cfg, generic_params(cfg), x, y, n_steps=1, label=f"{name}/{dtype}",
                         stored=stored_for(cfg))
    print("worst rel err", worst, flush=True)
    tr.close()


@pytest.mark.parametrize("name", ["cfg1_small", "cfg3_small", "cfg2_small"])
def test_three_steps_fp32(lpmod, name):
    """Optimizer state carried across steps (Adam bias correction with t > 1, momentum)."""
    cfg = dataclasses.replace(LI.make_config(name), dtype="f32")
    tr = lpmod.LocalTrainer(cfg)
    x, y = data_for(cfg)
    compare_step(tr, cfg, generic_params(cfg), x, y, n_steps=3, label=name)
    tr.close()


@pytest.mark.parametrize("scheme,combine", [("backprop", "sum"), ("last2", "sum"), ("overlap", "mean"),
                                            ("deep_supervision", "sum")])
def test_schemes_fp32(lpmod, scheme, combine):
    """Backprop as one block, the last-K baseline (earlier layers untouched, bit for bit), averaged
    overlapping windows, and full windows from every head."""
    cfg = LI.make_config("cfg3_small", scheme=scheme, combine=combine, n_layers=4, dtype="f32")
    tr = lpmod.LocalTrainer(cfg)
    x, y = data_for(cfg)
    compare_step(tr, cfg, generic_params(cfg), x, y, label=f"{scheme}/{combine}")
    tr.close()


def test_cfg1_full_size_fp32(lpmod):
    """The full residual-MLP configuration (the oracle finishes it in well under a second)."""
    cfg = LI.make_config("cfg1")
    tr = lpmod.LocalTrainer(cfg)
    x, y = data_for(cfg)
    compare_step(tr, cfg, LI.init_params(cfg), x, y, label="cfg1")
    tr.close()


def test_smaller_batch_and_empty_batch(lpmod):
    cfg = dataclasses.replace(LI.make_config("cfg3_small"), dtype="f32")
    tr = lpmod.LocalTrainer(cfg)                     # max_batch 3
    x, y = data_for(cfg, batch=2)
    compare_step(tr, cfg, generic_params(cfg), x, y, label="batch2")
    before = tr.get_params()
    t0 = lpmod.lp_get_step(tr.ctx)
    xd, yd = tr.stage(x, y)
    lpmod.lp_local_step(tr.ctx, xd.data_ptr(), yd.data_ptr(), 0, tr.losses.data_ptr())
    assert lpmod.lp_get_step(tr.ctx) == t0
    assert not np.any(tr.losses.cpu().numpy())
    after = tr.get_params()
    for k in before:
        np.testing.assert_array_equal(before[k], after[k])
    with pytest.raises(lpmod.LpError) as e:
        lpmod.lp_local_step(tr.ctx, xd.data_ptr(), yd.data_ptr(), 4, tr.losses.data_ptr())
    assert e.value.status == 2
    with pytest.raises(lpmod.LpError) as e:
        lpmod.lp_local_step(tr.ctx, 0, yd.data_ptr(), 2, tr.losses.data_ptr())
    assert e.value.status == 1
    with pytest.raises(lpmod.LpError) as e:
        tr.get("L9.nope")
    assert e.value.status == 8
    tr.close()


def test_builtin_init_statistics(lpmod):
    cfg = LI.make_config("cfg3_small")
    tr = lpmod.LocalTrainer(cfg)
    w = tr.get("L2.w1")
    assert abs(w.std() - 0.02) < 0.002 and abs(w.mean()) < 0.002
    assert np.all(tr.get("L1.ln1.g") == 1) and not np.any(tr.get("L1.b1"))
    tr.close()
    cfg = LI.make_config("cfg1")
    tr = lpmod.LocalTrainer(cfg)
    w = tr.get("L2.w1")
    assert abs(w.std() - np.sqrt(2 / 256)) < 0.01
    w2 = tr.get("L3.w1")
    assert abs(np.corrcoef(w.ravel(), w2.ravel())[0, 1]) < 0.02
    tr.close()


def test_repeatable_bitwise(lpmod):
    """Fixed reduction orders: two runs from the same state give identical bits."""
    cfg = LI.make_config("cfg4_small")
    x, y = data_for(cfg)
    outs = []
    for _ in range(2):
        tr = lpmod.LocalTrainer(cfg)
        tr.set_params(generic_params(cfg))
        xd, yd = tr.stage(x, y)
        l = tr.step(xd, yd).cpu().numpy().copy()
        outs.append((l, tr.get("L1.emb"), tr.get("L2.wqkv"), tr.get("H3.w")))
        tr.close()
    for a, b in zip(*outs):
        np.testing.assert_array_equal(a, b)


@pytest.mark.parametrize("name", ["cfg1_small", "cfg2_small", "cfg4_small", "cfg5_small"])
def test_side_streams_bit_identical(lpmod, name):
    """Heads' chains on side streams (forward continues on the caller's stream) give the same bits as
    everything on one stream, over three steps; and parity with the oracle holds."""
    cfg = LI.make_config(name)
    outs = []
    for ns in (0, 3):
        tr = lpmod.LocalTrainer(cfg, n_streams=ns)
        tr.set_params(generic_params(cfg))
        ls = []
        for step in range(3):
            xd, yd = tr.stage(*data_for(cfg, step))
            ls.append(tr.step(xd, yd).cpu().numpy().copy())
        P = tr.get_params()
        G = {k: tr.get(k + ".grad") for k in P}
        outs.append((ls, P, G))
        tr.close()
    for a, b in zip(outs[0][0], outs[1][0]):
        np.testing.assert_array_equal(a, b)
    for k in outs[0][1]:
        np.testing.assert_array_equal(outs[0][1][k], outs[1][1][k])
        np.testing.assert_array_equal(outs[0][2][k], outs[1][2][k])
    tr = lpmod.LocalTrainer(cfg, n_streams=2)
    x, y = data_for(cfg)
    compare_step(tr, cfg, generic_params(cfg), x, y, n_steps=1, label=name + "/streams", stored=stored_for(cfg))
    tr.close()


@pytest.mark.parametrize("name,dtype,tol", [("cfg3_small", "f32", 1e-4), ("cfg1_small", "f32", 1e-4),
                                            ("cfg3_small", "bf16", 2e-2)])
def test_gradient_cosines_local_vs_backprop(lpmod, name, dtype, tol):
    """Section 5, "Gradient Angles": per-layer cosine between greedy-local and backprop gradients on the same
    parameters and minibatch, device reductions against the oracle's; the last layer's is 1."""
    import torch
    g_cfg = dataclasses.replace(LI.make_config(name, scheme="greedy"), dtype=dtype)
    b_cfg = dataclasses.replace(LI.make_config(name, scheme="backprop"), dtype=dtype)
    P = generic_params(g_cfg)
    nh = len(g_cfg.heads)
    Pb = {k: v for k, v in P.items() if not k.startswith("H")}
    Pb.update({"H1." + k.split(".", 1)[1]: v for k, v in P.items() if k.startswith(f"H{nh}.")})
    x, y = data_for(g_cfg)
    ta, tb = lpmod.LocalTrainer(g_cfg), lpmod.LocalTrainer(b_cfg)
    ta.set_params(P)
    tb.set_params(Pb)
    xd, yd = ta.stage(x, y)
    ta.step(xd, yd)
    tb.step(xd, yd)
    out = torch.zeros(g_cfg.n_layers, device="cuda", dtype=torch.float32)
    lpmod.lp_grad_cosine(ta.ctx, tb.ctx, out.data_ptr())
    got = out.cpu().numpy().astype(np.float64)
    Pq = {k: np.asarray(v, np.float64) for k, v in P.items()}
    Pbq = {k: np.asarray(v, np.float64) for k, v in Pb.items()}
    _, gg, _ = oracle.local_gradients(g_cfg, Pq, x, y)
    _, gb, _ = oracle.local_gradients(b_cfg, Pbq, x, y)
    ref = oracle.layer_gradient_cosines(g_cfg, gg, gb)
    assert np.max(np.abs(got - ref)) <= tol, (got, ref)
    assert abs(got[-1] - 1.0) <= (1e-5 if dtype == "f32" else 2e-3)
    # a context against itself: exactly parallel
    lpmod.lp_grad_cosine(ta.ctx, ta.ctx, out.data_ptr())
    np.testing.assert_allclose(out.cpu().numpy(), 1.0, atol=1e-6)
    ta.close()
    tb.close()


@pytest.mark.parametrize("name,dtype,sched", [("cfg1_small", "f32", "pipelined"), ("cfg3_small", "f32", "pipelined"),
                                              ("cfg2_small", "f32", "pipelined"), ("cfg5_small", "f32", "pipelined"),
                                              ("cfg3_small", "bf16", "pipelined"), ("cfg5_small", "bf16", "pipelined"),
                                              ("cfg3_small", "f32", "pipelined_grouped"),
                                              ("cfg3_small", "bf16", "pipelined_grouped"),
                                              ("cfg5_small", "bf16", "pipelined_grouped")])
def test_pipelined_schedule_matches_oracle(lpmod, name, dtype, sched):
    """The pipelined schedule (section 6; labels travel with the activations, section 3) over J + 2 calls with a
    different minibatch each: losses (exactly 0 while a block waits for its first input), every block's
    parameters and optimizer moments after the last call, against the oracle's delay line; and the same
    bits with the blocks spread over side streams.  On the bf16 path (decoders: smooth networks, exact
    oracle) the losses are held to 2e-2 call by call; weights after several Adam steps are compared where the
    accumulated update is well conditioned (see updated_param_err) and the moments in full."""
    cfg = dataclasses.replace(LI.make_config(name), dtype=dtype)
    J = len(cfg.heads)
    P0 = generic_params(cfg)
    ltol, ptol, stol = (1e-4, 1e-4, 1e-4) if dtype == "f32" else (2e-2, 2e-2, 2e-2)
    worst_p = worst_s = 0.0
    finals = []
    for ns in (0, 2):
        tr = lpmod.LocalTrainer(cfg, schedule=sched, n_streams=ns)
        tr.set_params(P0)
        P = {k: v.astype(np.float64) for k, v in P0.items()}
        st, pipe = oracle.new_state(cfg, P), oracle.new_pipeline(cfg)
        for t in range(1, J + 3):
            x, y = data_for(cfg, t)
            xd, yd = tr.stage(x, y)
            got = tr.step(xd, yd).cpu().numpy().copy()
            ref, P = oracle.pipelined_step(cfg, P, st, pipe, x, y)
            for j in range(J):
                if t < j + 1:
                    assert got[j] == 0.0 and ref[j] == 0.0, (t, j)
                else:
                    assert abs(got[j] - ref[j]) <= ltol * abs(ref[j]), (name, t, j, got[j], ref[j])
        got_params = tr.get_params()
        for k in P0:
            worst_p = max(worst_p, relerr(got_params[k], P[k]))
            assert relerr(got_params[k], P[k]) <= ptol, (name, k, relerr(got_params[k], P[k]))
            for sname in ("m", "v"):
                if sname in st:
                    e = relerr(tr.get(k + "." + sname), st[sname][k])
                    worst_s = max(worst_s, e)
                    assert e <= stol, (name, sname, k, e)
        print(f"  pipelined {name}/{dtype} streams {ns}: worst param rel err {worst_p:.2e}, worst moment rel err {worst_s:.2e}", flush=True)
        finals.append(got_params)
        tr.close()
    for k in P0:
        np.testing.assert_array_equal(finals[0][k], finals[1][k])


def test_pipelined_schedule_needs_tiling_windows(lpmod):
    cfg = dataclasses.replace(LI.make_config("cfg4_small"), dtype="f32")      # overlapping windows
    with pytest.raises(lpmod.LpError):
        lpmod.LocalTrainer(cfg, schedule="pipelined")
    with pytest.raises(lpmod.LpError) as e:                                    # the grouped form is for decoder blocks
        lpmod.LocalTrainer(LI.make_config("cfg2_small"), schedule="pipelined_grouped")
    assert e.value.status == 7


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_paper_form_resnet_head(lpmod, dtype):
    """The ResNet auxiliary head of appendix B.3 (batch norm, ReLU, spatial mean, linear) on every stage."""
    cfg = dataclasses.replace(LI.make_config("cfg2_small", head="bn_pool_linear_ce"), dtype=dtype)
    assert cfg.heads[0].kind == "bn_pool_linear_ce"
    tr = lpmod.LocalTrainer(cfg, n_streams=2)
    x, y = data_for(cfg)
    compare_step(tr, cfg, generic_params(cfg), x, y, label="bn head " + dtype, stored=stored_for(cfg))
    tr.close()


@pytest.mark.parametrize("sched", ["pipelined", "pipelined_grouped"])
def test_pipelined_schedule_with_changing_batch_sizes(lpmod, sched):
    """Minibatches of different sizes travel down the pipeline with their own labels; a call with batch 0
    does not advance it."""
    cfg = dataclasses.replace(LI.make_config("cfg3_small"), dtype="f32")
    J = len(cfg.heads)
    tr = lpmod.LocalTrainer(cfg, schedule=sched, n_streams=2)
    P0 = generic_params(cfg)
    tr.set_params(P0)
    P = {k: v.astype(np.float64) for k, v in P0.items()}
    st, pipe = oracle.new_state(cfg, P), oracle.new_pipeline(cfg)
    sizes = [cfg.batch, 1, cfg.batch - 1, 0, cfg.batch, 2, 1][: J + 4]
    for t, b in enumerate(sizes, start=1):
        x, y = data_for(cfg, t, batch=max(b, 1))
        xd, yd = tr.stage(x, y)
        got = tr.step(xd, yd, batch=b).cpu().numpy().copy()
        if b == 0:
            assert not np.any(got)
            continue
        ref, P = oracle.pipelined_step(cfg, P, st, pipe, x, y)
        for j in range(J):
            assert abs(got[j] - ref[j]) <= 1e-4 * max(abs(ref[j]), 1e-30), (t, j, got[j], ref[j])
    got_params = tr.get_params()
    for k in P0:
        assert relerr(got_params[k], P[k]) <= 1e-4, (k, relerr(got_params[k], P[k]))
    tr.close()


@pytest.mark.parametrize("name,ns", [("cfg1_small", 0), ("cfg1_small", 2), ("cfg2_small", 3)])
def test_step_graph_replay_bit_identical(lpmod, name, ns):
    """A step replayed through a HIP graph (first call eager, second captured, later ones replayed; the same
    device buffers refilled between steps, an eager evaluation and a host read between replays) leaves the
    same bits as ordinary steps; a call with other buffers starts over; Adam is refused."""
    import torch
    cfg = LI.make_config(name)
    outs = []
    for graph in (False, True):
        tr = lpmod.LocalTrainer(cfg, n_streams=ns)
        tr.set_params(generic_params(cfg))
        if graph:
            tr.step_graph(True)
        xb, yb = tr.stage(*data_for(cfg, 0))
        ls, ev = [], []
        for step in range(6):
            xd, yd = tr.stage(*data_for(cfg, step))
            if step == 4:                      # other buffers: eager again, then a new capture
                xb, yb = xd.clone(), yd.clone()
            xb.copy_(xd); yb.copy_(yd)
            ls.append(tr.step(xb, yb).cpu().numpy().copy())
            ev.append(tr.eval(xd, yd).cpu().numpy().copy())
            torch.cuda.synchronize()
        P = tr.get_params()
        for k in list(P):       # the running statistics of every batch normalisation travel with the replay too
            if k.endswith(".g") and k.split(".")[-2].startswith("bn"):
                P[k[:-1] + "running_mean"] = tr.get(k[:-1] + "running_mean")
                P[k[:-1] + "running_var"] = tr.get(k[:-1] + "running_var")
        assert lpmod.lp_get_step(tr.ctx) == 6
        outs.append((ls, ev, P))
        tr.close()
    for a, b in zip(outs[0][0] + outs[0][1], outs[1][0] + outs[1][1]):
        np.testing.assert_array_equal(a, b)
    for k in outs[0][2]:
        np.testing.assert_array_equal(outs[0][2][k], outs[1][2][k])
    tr = lpmod.LocalTrainer(LI.make_config("cfg3_small"))
    with pytest.raises(lpmod.LpError):
        tr.step_graph(True)
    tr.close()


def _bn_prefixes(names):
    return [k[:-1] for k in names if k.endswith(".g") and k.split(".")[-2].startswith("bn")]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("sched", ["sync", "pipelined"])
def test_bn_running_statistics_and_evaluation(lpmod, dtype, sched):
    """Running mean / variance of every batch normalisation (stages and appendix-B.3 heads) after three steps
    with batches of different sizes, and the losses of an evaluation that normalises with them, against the
    oracle; momentum 0 freezes them; the default evaluation still uses the batch's own statistics."""
    cfg = dataclasses.replace(LI.make_config("cfg2_small", head="bn_pool_linear_ce"), dtype=dtype)
    tol = tol_for(cfg)
    stored = stored_for(cfg)
    tr = lpmod.LocalTrainer(cfg, n_streams=2, schedule=sched)
    P0 = generic_params(cfg)
    tr.set_params(P0)
    pres = _bn_prefixes(P0)
    assert pres
    for pre in pres:        # start: mean 0, variance 1
        assert not np.any(tr.get(pre + "running_mean"))
        np.testing.assert_array_equal(tr.get(pre + "running_var"), np.ones_like(P0[pre + "g"]))
    tr.bn_running(0.3, eval_with_running=True)
    P = {k: v.astype(np.float64) for k, v in P0.items()}
    st, pipe = oracle.new_state(cfg, P), oracle.new_pipeline(cfg)
    run = oracle.BatchNormRunning(0.3)
    for step, b in enumerate([cfg.batch, cfg.batch - 1, cfg.batch]):
        x, y = data_for(cfg, step, batch=b)
        xd, yd = tr.stage(x, y)
        tr.step(xd, yd)
        if sched == "sync":
            _, P, _ = oracle.local_step(cfg, P, st, x, y, stored=stored, bn=run)
        else:
            _, P = oracle.pipelined_step(cfg, P, st, pipe, x, y, stored=stored, bn=run)
        if dtype == "bf16":     # keep the two weight trajectories together: only the statistics are under test
            tr.set_params({k: v.astype(np.float32) for k, v in P.items()})
            P = {k: v.astype(np.float32).astype(np.float64) for k, v in P.items()}
    for pre in pres:
        if pre not in run.mean:      # a block the pipeline has not reached yet
            assert not np.any(tr.get(pre + "running_mean")), pre
            continue
        assert relerr(tr.get(pre + "running_mean"), run.mean[pre]) <= tol, (pre, "mean")
        assert relerr(tr.get(pre + "running_var"), run.var[pre]) <= tol, (pre, "var")
    x, y = data_for(cfg, 7, batch=3)
    xd, yd = tr.stage(x, y)
    got = tr.eval(xd, yd).cpu().numpy().copy()
    ref = oracle.eval_loss(cfg, P, x, y, stored=stored, bn=run)
    for j in range(len(ref)):
        assert abs(got[j] - ref[j]) <= tol * abs(ref[j]), (j, got[j], ref[j])
    # statistics written through the named tensors are the ones the next evaluation uses
    fake = oracle.BatchNormRunning(0.3)
    rng = np.random.default_rng(5)
    for pre in pres:
        C = P0[pre + "g"].shape[0]
        fake.mean[pre] = rng.normal(0.0, 0.5, C).astype(np.float32).astype(np.float64)
        fake.var[pre] = rng.uniform(0.5, 2.0, C).astype(np.float32).astype(np.float64)
        tr.set(pre + "running_mean", fake.mean[pre].astype(np.float32))
        tr.set(pre + "running_var", fake.var[pre].astype(np.float32))
    got_fake = tr.eval(xd, yd).cpu().numpy().copy()
    ref_fake = oracle.eval_loss(cfg, P, x, y, stored=stored, bn=fake)
    for j in range(len(ref)):
        assert abs(got_fake[j] - ref_fake[j]) <= tol * abs(ref_fake[j]), (j, got_fake[j], ref_fake[j])
    # evaluation changed nothing; momentum 0 freezes the statistics; batch-statistics evaluation is still there
    snap = {pre: (tr.get(pre + "running_mean"), tr.get(pre + "running_var")) for pre in pres}
    tr.bn_running(0.0, eval_with_running=False)
    got_batch = tr.eval(xd, yd).cpu().numpy().copy()
    ref_batch = oracle.eval_loss(cfg, P, x, y, stored=stored)
    for j in range(len(ref)):
        assert abs(got_batch[j] - ref_batch[j]) <= tol * abs(ref_batch[j]), (j, got_batch[j], ref_batch[j])
    assert np.any(got_batch != got)
    tr.step(xd, yd)
    for pre in pres:
        np.testing.assert_array_equal(tr.get(pre + "running_mean"), snap[pre][0])
        np.testing.assert_array_equal(tr.get(pre + "running_var"), snap[pre][1])
    with pytest.raises(lpmod.LpError):
        tr.bn_running(1.5)
    with pytest.raises(lpmod.LpError):
        tr.get("L1.ln1.running_mean")
    tr.close()


def test_convolutions_cut_along_k_match_oracle(lpmod):
    """Few output tiles and a long reduction (4 x 4 images, 128 channels, K = 1152): the forward and data-gradient
    convolutions run cut along k with fp32 partial sums added in a fixed order; same bar as every bf16 step."""
    cfg = LI.configs.resnet_config("t_cut", channels=(128,), in_hw=4, in_ch=3, n_classes=5, batch=8,
                                   n_basic_blocks=1, dtype="bf16")
    tr = lpmod.LocalTrainer(cfg, n_streams=1)
    x, y = data_for(cfg)
    compare_step(tr, cfg, generic_params(cfg), x, y, label="cut conv", stored=stored_for(cfg))
    tr.close()


@pytest.mark.parametrize("name,ns", [("cfg1_small", 2), ("cfg2_small", 3), ("cfg3_small", 2), ("cfg4_small", 2),
                                     ("cfg5_small", 1)])
def test_overlapped_steps_bit_identical(lpmod, name, ns):
    """Six steps issued back to back with lp_overlap_steps on (no join in between: every step has its own input,
    label and loss buffers) leave the same losses, weights and optimizer state, bit for bit, as six ordinary
    steps; an evaluation issued right behind them sees the finished weights; graph replay refuses to combine."""
    import torch
    cfg = LI.make_config(name)
    n = 6
    outs = []
    for overlap in (False, True):
        tr = lpmod.LocalTrainer(cfg, n_streams=ns)
        tr.set_params(generic_params(cfg))
        if overlap:
            tr.overlap_steps(True)
        bufs = [tr.stage(*data_for(cfg, i, batch=cfg.batch - (i % 2))) for i in range(n)]
        loss = [torch.zeros(len(cfg.heads), device=bufs[0][0].device) for _ in range(n)]
        for i in range(n):
            xd, yd = bufs[i]
            lpmod.lp_local_step(tr.ctx, xd.data_ptr(), yd.data_ptr(), xd.shape[0], loss[i].data_ptr())
        ev = tr.eval(*bufs[0]).cpu().numpy().copy()        # any other entry point joins first
        torch.cuda.synchronize()
        P = tr.get_params()
        for k in list(P):
            for sfx in (".m", ".v"):
                try:
                    P[k + sfx] = tr.get(k + sfx)
                except lpmod.LpError:
                    pass
        outs.append(([l.cpu().numpy().copy() for l in loss], ev, P))
        if overlap and cfg.opt.kind != "adam":
            with pytest.raises(lpmod.LpError):
                tr.step_graph(True)
        tr.close()
    for a, b in zip(outs[0][0], outs[1][0]):
        np.testing.assert_array_equal(a, b)
    np.testing.assert_array_equal(outs[0][1], outs[1][1])
    assert outs[0][2].keys() == outs[1][2].keys()
    for k in outs[0][2]:
        np.testing.assert_array_equal(outs[0][2][k], outs[1][2][k])


@pytest.mark.parametrize("joiner", ["bn_running", "get_step", "set_step", "tensor_info", "step_graph_off", "profile_read"])
def test_every_context_call_joins_overlapped_steps(lpmod, joiner):
    """With overlapped steps the chains of the last step run on the library's side streams.  Every entry point that
    takes the context (other than lp_local_step and the three host-only string / count queries) makes the caller's
    stream wait for them: after such a call, synchronising the caller's stream alone must be enough to read the
    losses and the updated weights of the last step."""
    import torch
    cfg = LI.make_config("cfg2_small")
    x, y = data_for(cfg)
    ref = None
    for overlap in (False, True):
        s = torch.cuda.Stream()
        with torch.cuda.stream(s):
            tr = lpmod.LocalTrainer(cfg, n_streams=3, stream=s)
            tr.set_params(generic_params(cfg))
            xd, yd = tr.stage(x, y)
            if overlap:
                tr.overlap_steps(True)
            for _ in range(3):
                tr.step(xd, yd)
            if overlap:
                if joiner == "bn_running":
                    tr.bn_running(0.1, False)
                elif joiner == "get_step":
                    assert lpmod.lp_get_step(tr.ctx) == 3
                elif joiner == "set_step":
                    lpmod.lp_set_step(tr.ctx, 3)
                elif joiner == "tensor_info":
                    lpmod.lp_tensor_info(tr.ctx, "L1.out")
                elif joiner == "step_graph_off":
                    tr.step_graph(False)
                else:
                    lpmod.lp_profile_read(tr.ctx, 0)
            s.synchronize()                      # the caller's stream only
            losses = tr.losses.clone()
            w = tr.params.clone()
        torch.cuda.synchronize()
        got = (losses.cpu().numpy().copy(), w.cpu().numpy().copy())
        tr.close()
        if ref is None:
            ref = got
        else:
            np.testing.assert_array_equal(ref[0], got[0])
            np.testing.assert_array_equal(ref[1], got[1])


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("nbb", [1, 2])
def test_resnet_units_against_exact_oracle(lpmod, dtype, nbb):
    """Every convolution + normalisation unit of a ResNet step against the exact float64 oracle (no storage
    rounding on the oracle's side), fed the device's own unit input, shortcut input and upstream gradient;
    the tensors that tie the units together are compared bit for bit (see check_resnet_stage_by_unit)."""
    cfg = dataclasses.replace(LI.make_config("cfg2_small", n_basic_blocks=nbb), dtype=dtype)
    print(f"[case] resnet units {dtype} blocks/stage {nbb}", flush=True)
    tr = lpmod.LocalTrainer(cfg, n_streams=2, debug=True)
    P0 = generic_params(cfg)
    tr.set_params(P0)
    x, y = data_for(cfg)
    xd, yd = tr.stage(x, y)
    tr.step(xd, yd)
    tol = tol_for(cfg)
    for hi in range(1, len(cfg.heads) + 1):
        w = check_resnet_stage_by_unit(tr, cfg, hi, P0, x, y, tol, label=f"units/{dtype}")
        print(f"  stage {hi}: worst rel err {w:.2e}", flush=True)
    # without the debug flag the gradient copies do not exist
    tr.close()
    tr = lpmod.LocalTrainer(cfg)
    tr.set_params(P0)
    tr.step(*tr.stage(x, y))
    assert tr.get("L1.stem.y").shape == (cfg.batch, 12, 12, 8)
    with pytest.raises(lpmod.LpError) as e:
        tr.get("L1.stem.dy")
    assert e.value.status == 8
    tr.close()
