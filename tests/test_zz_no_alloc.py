"""lpk_layernorm_bwd_static (the entry point for callers that cannot allocate: its workspace is an array built
into the library) against lpk_layernorm_bwd with a caller-supplied workspace, through the C ABI: same inputs,
bit-identical outputs, on two calls in a row, the second with a smaller input; and against the CPU oracle."""
import numpy as np
import pytest

from oracle import ops

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def K():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2012_03837_amd import kernels
    return kernels


def _case(K, dtype, rows, d, seed):
    import torch
    print(f"[case] layernorm_bwd_static dtype={dtype} rows={rows} d={d}", flush=True)
    rng = np.random.default_rng(seed)
    tdt = torch.bfloat16 if dtype else torch.float32

    def dev(a, dt):
        t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()
        return t.to(torch.bfloat16) if dt else t

    x = rng.standard_normal((rows, d)).astype(np.float32) * 2.0
    dy = rng.standard_normal((rows, d)).astype(np.float32)
    add = rng.standard_normal((rows, d)).astype(np.float32)
    if dtype:
        x, dy, add = (ops.bf16_round(t).astype(np.float32) for t in (x, dy, add))
    g = rng.standard_normal(d).astype(np.float32)
    b = rng.standard_normal(d).astype(np.float32)
    xd, dyd, addd, gd = dev(x, dtype), dev(dy, dtype), dev(add, dtype), dev(g, 0)
    y = torch.zeros(rows, d, device="cuda", dtype=tdt)
    mean = torch.zeros(rows, device="cuda")
    rstd = torch.zeros(rows, device="cuda")
    K.lpk_layernorm_fwd(dtype, xd, gd, dev(b, 0), y, mean, rstd, rows, d)
    outs = []
    for static in (0, 1):
        dx = torch.zeros(rows, d, device="cuda", dtype=tdt)
        dg = torch.ones(d, device="cuda")
        db = torch.ones(d, device="cuda")
        if static:
            K.lpk_layernorm_bwd_static(dtype, dyd, xd, mean, rstd, gd, addd, dx, dg, db, rows, d, 1)
        else:
            ws = torch.zeros(2 * ((rows + 7) // 8) * d + 16, device="cuda")
            K.lpk_layernorm_bwd(dtype, dyd, xd, mean, rstd, gd, addd, dx, dg, db, rows, d, 1, ws)
        torch.cuda.synchronize()
        outs.append((dx.float().cpu().numpy(), dg.cpu().numpy(), db.cpu().numpy()))
    for a, s in zip(outs[0], outs[1]):
        np.testing.assert_array_equal(a, s)       # same kernels, same order of additions
    # and both against the oracle
    _, cache = ops.layernorm_fwd(x.astype(np.float64), g.astype(np.float64), b.astype(np.float64))
    rdx, rdg, rdb = ops.layernorm_bwd(cache, g.astype(np.float64), dy.astype(np.float64))

    def rel(a, ref):
        return float(np.linalg.norm(a.astype(np.float64).ravel() - ref.ravel()) / np.linalg.norm(ref.ravel()))

    assert rel(outs[1][0], rdx + add) <= (4e-3 if dtype else 2e-6)
    assert rel(outs[1][1], rdg + 1) <= 1e-5 and rel(outs[1][2], rdb + 1) <= 1e-5


@pytest.mark.parametrize("dtype", [1, 0])
def test_static_workspace_matches_caller_workspace(K, dtype):
    _case(K, dtype, 1500, 768, 11)      # several blocks and a ragged tail
    _case(K, dtype, 37, 128, 12)        # smaller input right after: stale partial sums beyond it must not matter


def test_static_workspace_full_size_and_limit(K):
    import torch
    _case(K, 1, 8192, 1024, 13)         # the largest shape the built-in workspace takes
    rows, d = 8200, 1024
    z = torch.zeros(rows, d, device="cuda", dtype=torch.bfloat16)
    v = torch.zeros(rows, device="cuda")
    w = torch.zeros(d, device="cuda")
    with pytest.raises(K.KernelError):
        K.lpk_layernorm_bwd_static(1, z, z, v, v, w, None, z, w, w, rows, d, 0)
