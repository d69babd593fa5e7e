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
                        assert e <= 2 * tol, (label, sname, k, e)
        P = newP
    return worst
