"""Shared helpers of the GPU parity tests: run the HIP path and the CPU oracle on the same seeded
inputs and compare per tensor."""
import dataclasses

import numpy as np

import lp_inputs as LI
import oracle


def relerr(a, ref):
    a = np.asarray(a, dtype=np.float64).ravel()
    ref = np.asarray(ref, dtype=np.float64).ravel()
    return float(np.linalg.norm(a - ref) / max(np.linalg.norm(ref), 1e-30))


def updated_param_err(p_gpu, p_ref, g_ref, opt_kind):
    """Relative L2 error of an updated tensor.  Adam's update is lr * m_hat / (sqrt(v_hat) + eps), i.e.
    close to lr * sign(g) on the first steps: where a gradient entry is far below the tensor's typical
    magnitude its sign is decided by rounding noise, and for zero-initialised tensors the whole value
    is that update.  Such ill-conditioned entries (|g| < 5 % of the tensor's rms gradient) are left out
    for Adam; the moments m and v, which are linear / quadratic in g, are compared in full."""
    p_gpu = np.asarray(p_gpu, np.float64).ravel()
    p_ref = np.asarray(p_ref, np.float64).ravel()
    if opt_kind == "adam":
        g = np.abs(np.asarray(g_ref, np.float64).ravel())
        rms = np.sqrt(np.mean(g * g))
        keep = g >= 0.05 * rms
        if keep.sum() < 0.8 * g.size:      # mostly-zero gradients (embedding rows never seen): keep nonzero ones
            keep = g > 0.05 * np.sqrt(np.mean(g[g > 0] ** 2)) if np.any(g > 0) else np.ones_like(g, bool)
        untouched = ~keep
        # entries left out must still be within one update of the reference
        assert np.all(np.abs(p_gpu[untouched] - p_ref[untouched]) <= 2.5e-3 + 1e-6), "update out of range"
        p_gpu, p_ref = p_gpu[keep], p_ref[keep]
    return float(np.linalg.norm(p_gpu - p_ref) / max(np.linalg.norm(p_ref), 1e-30))


def bf16_round(x):
    import torch
    return torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).to(torch.bfloat16).to(torch.float32).numpy()


def data_for(cfg, step=0, batch=None):
    x, y = LI.make_batch(cfg, step, batch)
    if cfg.dtype == "bf16" and not np.issubdtype(x.dtype, np.integer):
        x = bf16_round(x)          # the synthetic images are defined as bf16 values
    return x, y


def generic_params(cfg, seed=0):
    """Initial weights with non-trivial biases and gains, so that every term is exercised."""
    P = LI.init_params(cfg, seed=seed)
    rng = np.random.default_rng(seed + 99)
    out = {}
    for k, v in P.items():
        if v.ndim == 1:
            out[k] = (v + 0.1 * rng.standard_normal(v.shape)).astype(np.float32)
        else:
            out[k] = v
    return out


def stored_for(cfg):
    """ReLU networks in bf16: the on/off decision of every ReLU is taken on the stored bf16
    activation on both sides (a flipped unit changes a gradient by O(1), so the two sides must
    decide in the same precision); smooth networks are compared against the exact oracle."""
    return "bf16" if (cfg.dtype == "bf16" and cfg.layers[0].kind != "decoder") else None


def tol_for(cfg):
    # relative error per tensor: 1e-4 on the fp32 path, 2e-2 on the bf16 MFMA path
    return 1e-4 if cfg.dtype == "f32" else 2e-2


def compare_step(tr, cfg, P0, x, y, n_steps=1, check_state=True, label="", stored=None):
    """Runs n_steps local steps on both sides (same batch sequence) and returns the worst relative
    errors; asserts the exact-zero / untouched invariants."""
    import torch
    tol = tol_for(cfg)
    tr.set_params(P0)
    P = {k: v.astype(np.float64) for k, v in P0.items()}
    st = oracle.new_state(cfg, P)
    worst = {"loss": 0.0, "grad": 0.0, "param": 0.0, "state": 0.0}
    for step in range(n_steps):
        xs, ys = (x, y) if step == 0 else data_for(cfg, step, batch=x.shape[0])
        xd, yd = tr.stage(xs, ys)
        ev = tr.eval(xd, yd).cpu().numpy().copy()
        got_l = tr.step(xd, yd).cpu().numpy().copy()
        ref_l, newP, grads = oracle.local_step(cfg, P, st, xs, ys, stored=stored)
        np.testing.assert_array_equal(ev, got_l)       # eval before a step == the losses the step reports
        for j in range(len(ref_l)):
            e = abs(got_l[j] - ref_l[j]) / abs(ref_l[j])
            worst["loss"] = max(worst["loss"], e)
            assert e <= tol, (label, "loss", j, got_l[j], ref_l[j])
        cnt = {}
        for (s, e_) in LI.head_windows(cfg):
            for li in range(s + 1, e_ + 1):
                cnt[li] = cnt.get(li, 0) + 1
        for k in P0:
            g = tr.get(k + ".grad")
            if k in grads:
                ref_g = grads[k]
                if cfg.combine == "mean" and k.startswith("L"):
                    ref_g = ref_g * cnt[int(k.split(".")[0][1:])]   # the device keeps the sum; the mean is applied in the update
                e = relerr(g, ref_g)
                worst["grad"] = max(worst["grad"], e)
                assert e <= tol, (label, "grad", k, e)
            else:
                assert not np.any(g), (label, "gradient leaked outside every window", k)
            p_new = tr.get(k)
            if k in grads:
                e = relerr(p_new, newP[k])
                worst["param"] = max(worst["param"], e)
                assert e <= tol, (label, "param", k, e)
            else:
                np.testing.assert_array_equal(p_new, P0[k])
            if check_state and k in grads:
                for sname in ("m", "v"):
                    if sname in st:
                        e = relerr(tr.get(k + "." + sname), st[sname][k])
                        worst["state"] = max(worst["state"], e)
                        assert e <= tol, (label, sname, k, e)
        P = newP
    return worst


# ----------------------------------------------------------------------------- ResNet: unit by unit
def resnet_units(cfg, li):
    """The convolution + normalisation units of stage li in forward order, as
    (unit name, filter, BN prefix, input (unit name or None = the stage input), stride, pad, relu,
     residual input (unit name, "IN" = the stage input, or None))."""
    l = cfg.layers[li - 1]
    pre = f"L{li}."
    out = []
    prev = None                       # unit whose .y feeds the next block (None: the stage input)
    if l.has_stem:
        out.append((pre + "stem", pre + "stem.w", pre + "stem.bn.", None, 1, 1, True, None))
        prev = pre + "stem"
    shapes = LI.param_shapes(cfg)
    for b in range(l.n_basic_blocks):
        q = pre + f"b{b + 1}."
        stride = l.stride if (b == 0 and not l.has_stem) else 1
        out.append((q + "conv1", q + "conv1.w", q + "bn1.", prev, stride, 1, True, None))
        res = prev if prev is not None else "IN"
        if (q + "proj.w") in shapes:
            out.append((q + "proj", q + "proj.w", q + "proj.bn.", prev, stride, 0, False, None))
            res = q + "proj"
        out.append((q + "conv2", q + "conv2.w", q + "bn2.", q + "conv1", 1, 1, True, res))
        prev = q + "conv2"
    return out


def check_resnet_stage_by_unit(tr, cfg, hi, P_before, x, y, tol, label="", exact_eq=np.testing.assert_array_equal):
    """Stage (= block) hi of a ResNet after one step of a debug context, unit by unit against the EXACT float64
    oracle.  A unit's stored input, its shortcut input and the upstream gradient it was given are read back from
    the device and handed to the oracle as data, so a ReLU that decides differently on the two sides (a bf16
    rounding away from zero) perturbs the one unit it belongs to and cannot spread through the stack.  What is
    compared per unit: the convolution output, the unit's output, the three parameter gradients, the input
    gradient, the updated weights and momentum.  All arithmetic on the oracle's side is exact; only the ReLU
    on/off bits of the backward pass are read off the device's stored activation, after they have been checked
    against the exact pre-activation (a wrong bit is allowed only inside the rounding band of the stored value).  What ties the units together is compared bit for bit on the
    device's own tensors: a unit's upstream gradient IS the input gradient of the unit behind it; and the last
    unit's upstream gradient is the head's, which the oracle reproduces from the device's stage output (the head
    has no ReLU)."""
    from oracle import layers as OLay
    from oracle import local as OL
    s, e = LI.head_windows(cfg)[hi - 1]
    assert e == s + 1, "one stage per block"
    li = e
    P = {k: np.asarray(v, np.float64) for k, v in P_before.items()}
    stage_in = np.asarray(x, np.float64) if s == 0 else tr.get(f"L{s}.out").astype(np.float64)
    units = resnet_units(cfg, li)
    worst = 0.0

    def rel(a, ref, what):
        nonlocal worst
        err = relerr(a, ref)
        worst = max(worst, err)
        assert err <= tol, (label, hi, what, err)

    def val(name):
        return stage_in if name in (None, "IN") else tr.get(name + ".y").astype(np.float64)

    # the head on the device's own stage output: loss, head gradients, and the gradient entering the stage
    h_e = tr.get(f"L{e}.out").astype(np.float64)
    loss, hc = OLay.head_loss(cfg, P, hi, h_e, y)
    dh, hg = OLay.head_bwd(cfg, P, hi, hc)
    got_loss = float(tr.losses.cpu().numpy()[hi - 1])
    assert abs(got_loss - loss) <= tol * abs(loss), (label, hi, "loss", got_loss, loss)
    for k, g in hg.items():
        rel(tr.get(k + ".grad"), g, k + ".grad")
    st = OL.new_state(cfg, P)
    names = [t[0] for t in units]
    by_name = {t[0]: t for t in units}
    # the order of the backward pass: per block conv2, conv1, then the projection (whose kernel adds conv1's share)
    order = []
    for t in reversed(units):
        if t[0].endswith("conv2"):
            blk = t[0].rsplit(".", 1)[0]
            order += [t, by_name[blk + ".conv1"]] + ([by_name[blk + ".proj"]] if blk + ".proj" in by_name else [])
        elif t[0].endswith("stem"):
            order.append(t)
    assert len(order) == len(units)
    eps_store = 2.0 ** -7 if cfg.dtype == "bf16" else 2e-5
    flip_worst = 0.0
    block_in_grad = None             # device tensor: gradient w.r.t. the input of the block handled last
    ds_of, dx_dev = {}, {}           # oracle's ReLU-masked upstream gradient per unit; device input gradients
    for (u, w, bn, inp, stride, pad, relu, res) in order:
        blk = u.rsplit(".", 1)[0]
        has_proj = (blk + ".proj") in by_name
        xin = val(inp)
        # forward: the exact pre-activation v, then the ReLU
        z = oracle.ops.conv2d_fwd(xin, P[w], stride, pad)
        v, cache = OLay._conv_bn(P, w, bn, xin, stride, pad, False, res=None if res is None else val(res))
        rel(tr.get(u + ".z"), z, u + ".z")
        y_dev = tr.get(u + ".y")
        rel(y_dev, np.maximum(v, 0.0) if relu else v, u + ".y")
        if relu:
            # A ReLU's on/off decision is a bit decided by floating point: the backward pass below takes it from
            # the device's stored activation (both sides then decide in the same precision, the kernel's), after
            # checking that the device decided correctly: it may differ from the exact sign of v only where v lies
            # inside the rounding band of the stored convolution output (|gain| * rstd * |z| * eps).
            flips = (y_dev > 0) != (v > 0)
            _, rstd = cache["bn"]
            band = eps_store * np.abs(P[bn + "g"]) * rstd * (np.abs(z) + np.sqrt(np.mean(z * z, axis=(0, 1, 2))))
            assert np.all(np.abs(v[flips]) <= band[flips]), (label, hi, u, "a ReLU decided wrongly outside the rounding band",
                                                             float(np.abs(v[flips]).max()))
            assert flips.mean() <= 2e-3, (label, hi, u, "too many ReLU units inside the rounding band", flips.mean())
            flip_worst = max(flip_worst, float(flips.mean()))
            cache["relu"] = True
            cache["out"] = y_dev.astype(np.float64)
        dy_dev = tr.get(u + ".dy")
        dy = dy_dev.astype(np.float64)
        # where the upstream gradient comes from
        if u == names[-1]:
            rel(dy, dh, u + ".dy (the head's gradient)")
        elif u.endswith("conv2") or u.endswith("stem"):
            exact_eq(dy_dev, block_in_grad)              # = the input gradient of the block behind it
        elif u.endswith("conv1"):
            exact_eq(dy_dev, dx_dev[blk + ".conv2"])     # = conv2's input gradient
        else:
            rel(dy, ds_of[blk + ".conv2"], u + ".dy (the masked gradient of the block output)")
        need_dx = inp is not None                        # a stage's window is the stage: no gradient leaves it
        g = {}
        dx, ds = OLay._conv_bn_bwd(P, w, bn, cache, dy, g, need_dx)
        ds_of[u] = ds
        for k, gv in g.items():
            rel(tr.get(k + ".grad"), gv, k + ".grad")
            newp = OL.optimizer_update(cfg.opt, P[k], gv, st, k, 1)
            rel(tr.get(k), newp, k + " updated")
            if "m" in st:
                rel(tr.get(k + ".m"), st["m"][k], k + ".m")
        if need_dx:
            dx_dev[u] = tr.get(u + ".dx")
            if u.endswith("conv1") and not has_proj:
                dx = dx + ds_of[blk + ".conv2"]          # identity shortcut: its share is added in the same kernel
            if u.endswith("proj"):
                dx = dx + dx_dev[blk + ".conv1"].astype(np.float64)   # a projection's kernel adds conv1's share
            rel(dx_dev[u], dx, u + ".dx")
            if (u.endswith("conv1") and not has_proj) or u.endswith("proj"):
                block_in_grad = dx_dev[u]
    return worst
