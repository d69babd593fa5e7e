"""Host-side checks that need no GPU: the library loads, exports every symbol the header declares,
sizes buffers consistently, and rejects bad specs before touching the device."""
import ctypes as C
import dataclasses
import os
import re

import pytest

import lp_inputs as LI
import paper_2012_03837_amd as lp
from paper_2012_03837_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def header_symbols():
    names = set()
    for fn in sorted(os.listdir(os.path.join(ROOT, "include"))):
        if fn.endswith(".h"):
            txt = open(os.path.join(ROOT, "include", fn)).read()
            txt = re.sub(r"/\*.*?\*/", "", txt, flags=re.S)
            names |= set(re.findall(r"\b(lpk?_[a-z0-9_]+)\s*\(", txt))
    return sorted(names)


def test_library_exports_every_declared_symbol():
    L = lp.lib()
    syms = header_symbols()
    assert "lp_init_blocks" in syms and "lp_local_step" in syms and "lp_eval_loss" in syms
    for s in syms:
        assert hasattr(L, s), s


def test_query_sizes_all_configs():
    import numpy as np
    for name in LI.CONFIG_NAMES:
        cfg = LI.make_config(name)
        spec, keep = lp.make_spec(cfg)
        sz = lp.lp_query_sizes(spec)
        n_par = sum(int(np.prod(s)) for s in LI.param_shapes(cfg).values())
        per = 4 + (2 if cfg.dtype == "bf16" else 0)
        assert sz.param_bytes >= n_par * per
        assert sz.param_bytes < n_par * per * 1.01 + (1 << 20)
        n_state = {"sgd": 0, "sgdm": 1, "adam": 2}[cfg.opt.kind]
        assert sz.state_bytes >= n_par * 4 * n_state
        assert sz.work_bytes > n_par * 4
        assert sz.param_bytes % 256 == 0 and sz.state_bytes % 256 == 0 and sz.work_bytes % 256 == 0
        assert sz.work_bytes < 64 << 30


def _status(fn):
    with pytest.raises(lp.LpError) as e:
        fn()
    return e.value.status, str(e.value)


def test_bad_specs_are_rejected_on_the_host():
    cfg = LI.make_config("cfg3_small")

    def q(c, **kw):
        spec, keep = lp.make_spec(c, **kw)
        return lambda: lp.lp_query_sizes(spec)

    bad_window = dataclasses.replace(cfg, heads=(dataclasses.replace(cfg.heads[0], window=0),) + cfg.heads[1:])
    assert _status(q(bad_window))[0] == B.LP_EINVAL
    unordered = dataclasses.replace(cfg, heads=cfg.heads[::-1])
    assert _status(q(unordered))[0] == B.LP_EINVAL
    bad_heads = dataclasses.replace(cfg, layers=tuple(dataclasses.replace(l, n_heads=3) for l in cfg.layers))
    assert _status(q(bad_heads))[0] == B.LP_ESHAPE
    assert _status(q(cfg, max_batch=0))[0] == B.LP_ESHAPE
    wrong_in = dataclasses.replace(cfg, heads=(dataclasses.replace(cfg.heads[0], in_dim=64),) + cfg.heads[1:])
    st, msg = _status(q(wrong_in))
    assert st == B.LP_ESHAPE and "head 1" in msg
    mlp = LI.make_config("cfg1")
    mixed = dataclasses.replace(mlp, layers=mlp.layers[:1] + cfg.layers[:1])
    assert _status(q(mixed))[0] in (B.LP_EUNSUPPORTED, B.LP_ESHAPE)
    # null spec
    assert lp.lib().lp_query_sizes(None, None) == B.LP_EINVAL


def test_init_rejects_null_and_misaligned_buffers_before_any_device_call():
    cfg = LI.make_config("cfg1")
    spec, keep = lp.make_spec(cfg)
    assert _status(lambda: lp.lp_init_blocks(spec, 0, 0, 0))[0] == B.LP_EINVAL
    assert _status(lambda: lp.lp_init_blocks(spec, 0x1000 + 8, 0x2000, 0x3000))[0] == B.LP_EALIGN
    ctx = C.c_void_p(123)
    bufs = B.lp_buffers(0, 0, 0)
    st = lp.lib().lp_init_blocks(C.byref(spec), C.byref(bufs), None, C.byref(ctx))
    assert st == B.LP_EINVAL and ctx.value is None


def test_null_context_calls_fail_cleanly():
    L = lp.lib()
    assert L.lp_local_step(None, None, None, 1, None) == B.LP_EINVAL
    assert L.lp_eval_loss(None, None, None, 1, None) == B.LP_EINVAL
    assert L.lp_get_tensor(None, b"L1.w1", None, 0) == B.LP_EINVAL
    assert L.lp_num_params(None) == 0
    assert L.lp_step_graph(None, 1) == B.LP_EINVAL
    assert L.lp_bn_running(None, 0.1, 0) == B.LP_EINVAL
    assert L.lp_overlap_steps(None, 1) == B.LP_EINVAL
    assert L.lp_join(None) == B.LP_EINVAL
    L.lp_destroy(None)


def test_bench_refuses_more_than_one_gpu():
    """Every box has one GPU: asking the bench for more ends with a message, before anything touches a device."""
    import os
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode != 0
    assert "--gpus must be 1" in r.stderr
    assert not r.stdout.strip()
