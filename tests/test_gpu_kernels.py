"""Per-kernel GPU parity through the kernel-level C ABI, against the CPU oracle's primitives in
float64 on the same (bf16-representable) inputs.  Shapes span several tiles plus ragged tails."""
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


def zeros(*shape, dtype=None):
    import torch
    return torch.zeros(*shape, device="cuda", dtype=dtype or torch.float32)


def ones(*shape):
    import torch
    return torch.ones(*shape, device="cuda", dtype=torch.float32)


def dev(a, dtype):
    import torch
    t = torch.from_numpy(np.ascontiguousarray(a)).cuda()
    return t.to(torch.bfloat16) if dtype == 1 and t.is_floating_point() else t


def host(t):
    import torch
    return t.detach().to(torch.float32).cpu().numpy().astype(np.float64)


def rnd(rng, shape, dtype, scale=1.0):
    """Random values that are exactly representable in the compute dtype."""
    a = (rng.standard_normal(shape) * scale).astype(np.float32)
    return ops.bf16_round(a).astype(np.float32) if dtype == 1 else a


def relerr(a, ref):
    return float(np.linalg.norm(np.asarray(a, np.float64).ravel() - np.asarray(ref, np.float64).ravel())
                 / max(np.linalg.norm(np.asarray(ref, np.float64).ravel()), 1e-30))


GEMM_SHAPES = [(200, 136, 72), (128, 128, 32), (1, 8, 8), (333, 257, 40), (64, 1000, 128), (600, 128, 600),
               (264, 136, 4104), (520, 264, 2048), (304, 520, 96), (1000, 264, 320), (8, 8, 32),
               (10, 136, 264), (264, 10, 520),        # a 10-class head's weight gradient and forward map (skinny products)
               (5, 24, 77), (24, 3, 100)]             # skinny, reduction not a multiple of 8 or of the waves' shares


@pytest.mark.parametrize("dtype", [0, 1])
@pytest.mark.parametrize("a_kc,b_kc", [(1, 1), (1, 0), (0, 0), (0, 1)])
def test_gemm_layouts_and_epilogues(K, dtype, a_kc, b_kc):
    import torch
    rng = np.random.default_rng(5)
    for (M, N, Kd) in GEMM_SHAPES:
        A = rnd(rng, (M, Kd), dtype)
        B = rnd(rng, (N, Kd), dtype)
        bias = rng.standard_normal(N).astype(np.float32)
        res = rnd(rng, (M, N), dtype)
        dsrc = rnd(rng, (M, N), dtype)
        Am = A if a_kc else np.ascontiguousarray(A.T)
        Bm = B if b_kc else np.ascontiguousarray(B.T)
        dA, dB = dev(Am, dtype), dev(Bm, dtype)
        ref0 = A.astype(np.float64) @ B.astype(np.float64).T
        tol_lo = 4e-3 if dtype == 1 else 2e-6
        # (1) plain product into fp32, with accumulate
        C0 = rng.standard_normal((M, N)).astype(np.float32)
        dC = dev(C0, 0)
        K.lpk_gemm(dtype, dA, Am.shape[1], a_kc, dB, Bm.shape[1], b_kc, dC, N, 1, M, N, Kd, accumulate=1)
        assert relerr(host(dC), ref0 + C0) <= 2e-6, (M, N, Kd, "acc")
        # (2) bias + GELU with saved pre-activation + residual, compute-dtype output
        out = torch.zeros(M, N, device="cuda", dtype=torch.bfloat16 if dtype else torch.float32)
        pre = torch.zeros_like(out)
        K.lpk_gemm(dtype, dA, Am.shape[1], a_kc, dB, Bm.shape[1], b_kc, out, N, 0, M, N, Kd, bias=dev(bias, 0), act=2,
                   pre=pre, res=dev(res, dtype), ldr=N)
        v = ref0 + bias
        assert relerr(host(pre), v) <= tol_lo
        assert relerr(host(out), ops.gelu_fwd(v) + res) <= tol_lo, (M, N, Kd, "gelu")
        # (3) backward-activation epilogues
        for dact, fn in ((1, lambda s, g: g * (s > 0)), (2, ops.gelu_bwd)):
            K.lpk_gemm(dtype, dA, Am.shape[1], a_kc, dB, Bm.shape[1], b_kc, out, N, 0, M, N, Kd, dact_src=dev(dsrc, dtype),
                       dact=dact, ldd=N)
            assert relerr(host(out), fn(dsrc.astype(np.float64), ref0)) <= tol_lo, (M, N, Kd, "dact", dact)
        # (4) split-K with ordered partial sums (long reductions over few tiles)
        if dtype == 1:
            ws = zeros(8 * M * N)
            o3 = zeros(M, N)
            K.lpk_gemm(dtype, dA, Am.shape[1], a_kc, dB, Bm.shape[1], b_kc, o3, N, 1, M, N, Kd, bias=dev(bias, 0),
                       splitk_ws=ws)
            assert relerr(host(o3), ref0 + bias) <= 2e-6, (M, N, Kd, "splitk")
        # (5) the MFMA and plain kernels agree on bf16
        if dtype == 1:
            o2 = torch.zeros(M, N, device="cuda", dtype=torch.float32)
            K.lpk_gemm(dtype, dA, Am.shape[1], a_kc, dB, Bm.shape[1], b_kc, o2, N, 1, M, N, Kd, plain=1)
            assert relerr(host(o2), ref0) <= 2e-6


@pytest.mark.parametrize("causal", [1, 0])
@pytest.mark.parametrize("S", [64, 200, 256, 333])
def test_attention_mfma_vs_oracle(K, S, causal):
    import torch
    rng = np.random.default_rng(S)
    B, H, dh = 2, 3, 64
    d = H * dh
    qkv = rnd(rng, (B * S, 3 * d), 1, scale=1.5)          # sharp softmax: scores of order a few units
    dout = rnd(rng, (B * S, d), 1)
    dq = dev(qkv, 1)
    o = torch.zeros(B * S, d, device="cuda", dtype=torch.bfloat16)
    lse = torch.zeros(B, H, S, device="cuda", dtype=torch.float32)
    K.lpk_attention_fwd(1, dq, o, lse, B, S, H, dh, causal)

    def split(t):
        return t.reshape(B, S, H, dh).transpose(0, 2, 1, 3)
    q64 = qkv.astype(np.float64)
    q, k, v = split(q64[:, :d]), split(q64[:, d:2 * d]), split(q64[:, 2 * d:])
    ro, p = ops.attention_fwd(q, k, v, causal=bool(causal))
    ro2 = ro.transpose(0, 2, 1, 3).reshape(B * S, d)
    assert relerr(host(o), ro2) <= 6e-3
    s = (q @ np.swapaxes(k, -1, -2)) / 8.0
    if causal:
        s = np.where(np.tril(np.ones((S, S), bool)), s, -np.inf)
    ref_lse = np.log(np.exp(s - s.max(-1, keepdims=True)).sum(-1)) + s.max(-1)
    assert np.abs(host(lse) - ref_lse).max() <= 2e-3
    # backward, fed the kernel's own o and lse
    dqkv = torch.zeros(B * S, 3 * d, device="cuda", dtype=torch.bfloat16)
    delta = torch.zeros(B, H, S, device="cuda", dtype=torch.float32)
    K.lpk_attention_bwd(1, dq, o, lse, dev(dout, 1), dqkv, delta, B, S, H, dh, causal)
    rdq, rdk, rdv = ops.attention_bwd(q, k, v, p, split(dout.astype(np.float64)))
    merge = lambda t: t.transpose(0, 2, 1, 3).reshape(B * S, d)
    g = host(dqkv)
    assert relerr(g[:, :d], merge(rdq)) <= 1.5e-2
    assert relerr(g[:, d:2 * d], merge(rdk)) <= 1.5e-2
    assert relerr(g[:, 2 * d:], merge(rdv)) <= 1.5e-2
    # plain kernel on the same inputs
    o2 = torch.zeros_like(o); lse2 = torch.zeros_like(lse); dqkv2 = torch.zeros_like(dqkv)
    K.lpk_attention_fwd(1, dq, o2, lse2, B, S, H, dh, causal, plain=1)
    K.lpk_attention_bwd(1, dq, o2, lse2, dev(dout, 1), dqkv2, delta, B, S, H, dh, causal, plain=1)
    assert relerr(host(o2), ro2) <= 6e-3
    assert relerr(host(dqkv2)[:, :d], merge(rdq)) <= 1.5e-2


@pytest.mark.parametrize("dtype", [0, 1])
@pytest.mark.parametrize("rows,d", [(37, 128), (600, 768), (5, 40), (130, 1024)])
def test_layernorm(K, dtype, rows, d):
    import torch
    rng = np.random.default_rng(rows)
    x = rnd(rng, (rows, d), dtype, 2.0) + (1.0 if dtype == 0 else 0.0)
    x = ops.bf16_round(x).astype(np.float32) if dtype else x
    g = rng.standard_normal(d).astype(np.float32)
    b = rng.standard_normal(d).astype(np.float32)
    dy = rnd(rng, (rows, d), dtype)
    add = rnd(rng, (rows, d), dtype)
    tdt = torch.bfloat16 if dtype else torch.float32
    y = torch.zeros(rows, d, device="cuda", dtype=tdt)
    mean = zeros(rows); rstd = zeros(rows)
    K.lpk_layernorm_fwd(dtype, dev(x, dtype), dev(g, 0), dev(b, 0), y, mean, rstd, rows, d)
    ry, cache = ops.layernorm_fwd(x.astype(np.float64), g.astype(np.float64), b.astype(np.float64))
    tol = 4e-3 if dtype else 2e-6
    assert relerr(host(y), ry) <= tol
    assert relerr(host(mean), x.astype(np.float64).mean(-1)) <= 1e-5
    dx = torch.zeros(rows, d, device="cuda", dtype=tdt)
    dg = ones(d); db = ones(d)
    scratch = zeros(2 * ((rows + 7) // 8) * d + 16)
    K.lpk_layernorm_bwd(dtype, dev(dy, dtype), dev(x, dtype), mean, rstd, dev(g, 0), dev(add, dtype), dx, dg, db, rows, d,
                        1, scratch)
    rdx, rdg, rdb = ops.layernorm_bwd(cache, g.astype(np.float64), dy.astype(np.float64))
    assert relerr(host(dx), rdx + add) <= tol
    assert relerr(host(dg), rdg + 1) <= 1e-5 and relerr(host(db), rdb + 1) <= 1e-5


@pytest.mark.parametrize("dtype", [0, 1])
@pytest.mark.parametrize("rows,n", [(50, 10), (19, 1000), (7, 32000)])
def test_softmax_ce(K, dtype, rows, n):
    import torch
    rng = np.random.default_rng(n)
    z = rnd(rng, (rows, n), dtype, 3.0)
    y = rng.integers(0, n, rows).astype(np.int32)
    dz = dev(z, dtype)
    loss = zeros(rows)
    K.lpk_softmax_ce(dtype, dz, n, dev(y, 0), loss, rows, n, 1, 1.0 / rows)
    z64 = z.astype(np.float64)
    ref_loss, p = ops.softmax_ce_fwd(z64, y)
    rows_ref = np.log(np.exp(z64 - z64.max(-1, keepdims=True)).sum(-1)) + z64.max(-1) - z64[np.arange(rows), y]
    assert np.abs(host(loss) - rows_ref).max() <= 2e-5 * max(1, np.abs(rows_ref).max())
    assert relerr(host(dz), ops.softmax_ce_bwd(p, y)) <= (4e-3 if dtype else 2e-5)


@pytest.mark.parametrize("kind", [0, 1, 2])
def test_optimizer_kernel(K, kind):
    """Identical fp32 inputs, non-zero moments, t > 1."""
    import torch
    import lp_inputs as LI
    from oracle import local as OL
    rng = np.random.default_rng(kind)
    n = 4 * 1237
    p, g = rng.standard_normal(n).astype(np.float32), rng.standard_normal(n).astype(np.float32)
    m = (0.1 * rng.standard_normal(n)).astype(np.float32)
    v = (0.01 * rng.random(n)).astype(np.float32)
    dp, dg, dm, dv = dev(p, 0), dev(g, 0), dev(m, 0), dev(v, 0)
    low = torch.zeros(n, device="cuda", dtype=torch.bfloat16)
    K.lpk_optimizer(kind, 1e-2, 0.9, 0.9, 0.999, 1e-8, 0.0, 7, 0.5, dp, dg, dm, dv, low, n)
    opt = LI.OptCfg(("sgd", "sgdm", "adam")[kind], lr=1e-2)
    st = {"m": {"p": m.astype(np.float64)}, "v": {"p": v.astype(np.float64)}}
    ref = OL.optimizer_update(opt, p.astype(np.float64), 0.5 * g.astype(np.float64), st, "p", 7)
    assert relerr(host(dp), ref) <= 1e-6
    assert np.abs(host(dp) - ref).max() <= 1e-6
    if kind >= 1:
        assert relerr(host(dm), st["m"]["p"]) <= 1e-6
    if kind == 2:
        assert relerr(host(dv), st["v"]["p"]) <= 1e-6
    np.testing.assert_array_equal(host(low), ops.bf16_round(host(dp).astype(np.float32)))


@pytest.mark.parametrize("with_counts", [False, True])
@pytest.mark.parametrize("accumulate", [0, 1])
def test_embed_bwd_repeated_tokens(K, with_counts, accumulate):
    import torch
    rng = np.random.default_rng(0)
    T, V, d = 700, 90, 136
    ids = rng.integers(0, 50, T).astype(np.int32)         # rows 50..89 never occur
    ids[:300] = 3
    ids[5], ids[6] = -4, 1000                              # out of range: counted as rows 0 and V-1
    dh = rnd(rng, (T, d), 1)
    demb = ones(V, d)
    scratch = zeros(4096) if with_counts else None
    K.lpk_embed_bwd(1, dev(ids, 0), dev(dh, 1), demb, T, V, d, accumulate, scratch=scratch)
    ref = ops.embed_bwd(np.clip(ids, 0, V - 1), V, dh.astype(np.float64)) + accumulate
    assert relerr(host(demb), ref) <= 1e-5
    assert np.all(host(demb)[50:89] == accumulate)         # absent rows: exactly zero, or untouched


# Shapes for the persistent direct-to-LDS GEMM: fewer tiles than blocks, exactly one wave of tiles,
# whole waves plus a tail, ragged edges in m and n, reductions shorter than the LDS ring.
DMA_SHAPES = [(520, 264, 4096), (4096, 4096, 64), (4104, 4360, 96), (8192, 776, 768), (2056, 8200, 32),
              (6000, 12000, 160), (264, 136, 16384), (4104, 8200, 256), (8192, 8192, 768)]


_ORACLE_PRODUCTS = {}


def oracle_product(tag, A, B):
    """A B^T by the CPU oracle's linear layer in float64, as a device tensor for the comparison.  The inputs of a
    shape are the same for every kernel variant and layout (same seed, same order), so each product is computed
    once per test session."""
    import torch
    key = (tag,) + A.shape + B.shape + (A.ravel()[:8].tobytes(), B.ravel()[-8:].tobytes())
    if key not in _ORACLE_PRODUCTS:
        _ORACLE_PRODUCTS[key] = torch.from_numpy(ops.linear_fwd(A.astype(np.float64), B.astype(np.float64)))
    return _ORACLE_PRODUCTS[key].cuda()


@pytest.mark.parametrize("variant", [3, 4, 5, 6, 7, 8])
@pytest.mark.parametrize("a_kc,b_kc", [(1, 1), (1, 0), (0, 0), (0, 1)])
def test_gemm_persistent_variants(K, variant, a_kc, b_kc):
    import torch
    rng = np.random.default_rng(11)
    ws = zeros(1 << 25)
    for (M, N, Kd) in DMA_SHAPES:
        A = rnd(rng, (M, Kd), 1, 0.5)
        B = rnd(rng, (N, Kd), 1, 0.5)
        Am = A if a_kc else np.ascontiguousarray(A.T)
        Bm = B if b_kc else np.ascontiguousarray(B.T)
        dA, dB = dev(Am, 1), dev(Bm, 1)
        ref = oracle_product("dma", A, B)
        out = torch.full((M, N), 7.0, device="cuda", dtype=torch.float32)
        K.lpk_gemm(1, dA, Am.shape[1], a_kc, dB, Bm.shape[1], b_kc, out, N, 1, M, N, Kd, variant=variant, splitk_ws=ws)
        err = float((out.double() - ref).norm() / ref.norm())
        assert err <= 2e-6, (M, N, Kd, variant, err)
        # bias + residual epilogue into bf16, applied once even where a tile is summed from pieces
        bias = rng.standard_normal(N).astype(np.float32)
        res = rnd(rng, (M, N), 1)
        outb = torch.zeros(M, N, device="cuda", dtype=torch.bfloat16)
        K.lpk_gemm(1, dA, Am.shape[1], a_kc, dB, Bm.shape[1], b_kc, outb, N, 0, M, N, Kd, bias=dev(bias, 0),
                   res=dev(res, 1), ldr=N, variant=variant, splitk_ws=ws)
        refb = ref + torch.from_numpy(bias).cuda().double() + torch.from_numpy(res).cuda().double()
        errb = float((outb.double() - refb).norm() / refb.norm())
        assert errb <= 4e-3, (M, N, Kd, variant, errb)
        # repeatable bit for bit
        out2 = torch.zeros_like(out)
        K.lpk_gemm(1, dA, Am.shape[1], a_kc, dB, Bm.shape[1], b_kc, out2, N, 1, M, N, Kd, variant=variant, splitk_ws=ws)
        assert torch.equal(out, out2)


# Outputs a few tiles wide over long reductions (the shapes of a vocabulary head's input and weight
# gradients), ragged in every dimension: the panel mode of the persistent kernel.
PANEL_SHAPES = [(8192, 768, 4096), (2056, 520, 2048), (1304, 1000, 6400), (776, 264, 16384)]


@pytest.mark.parametrize("variant", [9, 10, 11])
@pytest.mark.parametrize("a_kc,b_kc", [(1, 0), (0, 0), (1, 1)])
def test_gemm_panel_mode(K, variant, a_kc, b_kc):
    import torch
    rng = np.random.default_rng(13)
    ws = zeros(1 << 25)
    for (M, N, Kd) in PANEL_SHAPES:
        if variant == 9 and N <= 128:
            continue
        A = rnd(rng, (M, Kd), 1, 0.5)
        B = rnd(rng, (N, Kd), 1, 0.5)
        Am = A if a_kc else np.ascontiguousarray(A.T)
        Bm = B if b_kc else np.ascontiguousarray(B.T)
        dA, dB = dev(Am, 1), dev(Bm, 1)
        ref = oracle_product("panel", A, B)
        out = torch.full((M, N), 7.0, device="cuda", dtype=torch.float32)
        K.lpk_gemm(1, dA, Am.shape[1], a_kc, dB, Bm.shape[1], b_kc, out, N, 1, M, N, Kd, variant=variant, splitk_ws=ws)
        err = float((out.double() - ref).norm() / ref.norm())
        assert err <= 2e-6, (M, N, Kd, variant, err)
        bias = rng.standard_normal(N).astype(np.float32)
        outb = torch.zeros(M, N, device="cuda", dtype=torch.bfloat16)
        K.lpk_gemm(1, dA, Am.shape[1], a_kc, dB, Bm.shape[1], b_kc, outb, N, 0, M, N, Kd, bias=dev(bias, 0), act=1,
                   variant=variant, splitk_ws=ws)
        refb = torch.relu(ref + torch.from_numpy(bias).cuda().double())
        errb = float((outb.double() - refb).norm() / refb.norm())
        assert errb <= 4e-3, (M, N, Kd, variant, errb)
        out2 = torch.zeros_like(out)
        K.lpk_gemm(1, dA, Am.shape[1], a_kc, dB, Bm.shape[1], b_kc, out2, N, 1, M, N, Kd, variant=variant, splitk_ws=ws)
        assert torch.equal(out, out2)


def test_gemm_forced_variant_rejects_unsupported_shape(K):
    import torch
    A = torch.zeros(64, 40, device="cuda", dtype=torch.bfloat16)
    out = torch.zeros(64, 64, device="cuda", dtype=torch.float32)
    with pytest.raises(RuntimeError):
        K.lpk_gemm(1, A, 40, 1, A, 40, 1, out, 64, 1, 64, 64, 40, variant=5)      # K % 32 != 0


def test_copy_bit_exact(K):
    import torch
    src = torch.randint(-2**31, 2**31 - 1, ((1 << 20) + 12,), device="cuda", dtype=torch.int32)
    dst = torch.zeros_like(src)
    K.lpk_copy(src, dst, src.numel() * 4)
    assert torch.equal(src, dst)
    with pytest.raises(RuntimeError):
        K.lpk_copy(src, dst, 24)          # not a multiple of 16


@pytest.mark.parametrize("R,C", [(64, 64), (8, 8), (200, 72), (1000, 264), (32000, 768), (72, 4104)])
def test_transpose_bf16_bit_exact(K, R, C):
    """The transposed weight copy is the transpose, bit for bit, also where 64 x 64 tiles are ragged."""
    import torch
    src = torch.randn(R, C, device="cuda").to(torch.bfloat16)
    dst = torch.zeros(C, R, device="cuda", dtype=torch.bfloat16)
    K.lpk_transpose_bf16(src, dst, R, C)
    assert torch.equal(dst, src.t().contiguous())
    with pytest.raises(RuntimeError):
        K.lpk_transpose_bf16(src, dst, R - 1, C)      # not a multiple of 8


@pytest.mark.parametrize("dtype", [0, 1])
@pytest.mark.parametrize("N,H,C,O,R,stride,pad", [(3, 9, 5, 7, 3, 1, 1), (2, 8, 16, 24, 3, 2, 1), (2, 8, 16, 8, 1, 2, 0),
                                                  (4, 12, 3, 64, 3, 1, 1), (3, 10, 3, 64, 3, 2, 1), (5, 14, 64, 136, 3, 1, 1),
                                                  (3, 16, 72, 128, 3, 2, 1), (6, 10, 128, 64, 1, 2, 0)])
def test_conv_and_batchnorm(K, dtype, N, H, C, O, R, stride, pad):
    import torch
    rng = np.random.default_rng(H)
    x = rnd(rng, (N, H, H, C), dtype)
    w = rnd(rng, (O, R, R, C), dtype, 0.3)
    P = (H + 2 * pad - R) // stride + 1
    tdt = torch.bfloat16 if dtype else torch.float32
    out = torch.zeros(N, P, P, O, device="cuda", dtype=tdt)
    K.lpk_conv_fwd(dtype, dev(x, dtype), dev(w, dtype), out, N, H, H, C, O, R, stride, pad)
    ref = ops.conv2d_fwd(x.astype(np.float64), w.astype(np.float64), stride, pad)
    tol = 4e-3 if dtype else 2e-6
    assert relerr(host(out), ref) <= tol
    dout = rnd(rng, (N, P, P, O), dtype)
    dx = torch.zeros(N, H, H, C, device="cuda", dtype=tdt)
    dw = zeros(O, R, R, C)
    K.lpk_conv_bwd_data(dtype, dev(dout, dtype), dev(w, dtype), dx, N, H, H, C, O, R, stride, pad)
    K.lpk_conv_bwd_weight(dtype, dev(dout, dtype), dev(x, dtype), dw, N, H, H, C, O, R, stride, pad)
    rdx, rdw = ops.conv2d_bwd(x.astype(np.float64), w.astype(np.float64), stride, pad, dout.astype(np.float64))
    assert relerr(host(dx), rdx) <= tol
    assert relerr(host(dw), rdw) <= 2e-6
    # the same filter gradient cut along the pixels with workspace (the form a step uses), twice: bit-repeatable
    ws = zeros(max(64 * O * R * R * C, N * O * R * R * C))
    dw2 = torch.full((O, R, R, C), 5.0, device="cuda", dtype=torch.float32)
    dw3 = torch.zeros(O, R, R, C, device="cuda", dtype=torch.float32)
    K.lpk_conv_bwd_weight_ws(dtype, dev(dout, dtype), dev(x, dtype), dw2, N, H, H, C, O, R, stride, pad, ws)
    K.lpk_conv_bwd_weight_ws(dtype, dev(dout, dtype), dev(x, dtype), dw3, N, H, H, C, O, R, stride, pad, ws)
    assert relerr(host(dw2), rdw) <= 2e-6
    assert torch.equal(dw2, dw3)
    # batchnorm + residual + relu on the conv output
    rows = N * P * P
    z = host(out).astype(np.float32)
    g = rng.standard_normal(O).astype(np.float32); b = rng.standard_normal(O).astype(np.float32)
    res = rnd(rng, (N, P, P, O), dtype)
    y = torch.zeros_like(out); mean = zeros(O); rstd = zeros(O)
    scratch = zeros((2 * 1024 + 2) * O + 64)
    K.lpk_batchnorm_fwd(dtype, out, dev(g, 0), dev(b, 0), dev(res, dtype), y, mean, rstd, rows, O, 1, scratch)
    ry, cache = ops.batchnorm_fwd(z.astype(np.float64), g.astype(np.float64), b.astype(np.float64))
    ry = np.maximum(ry + res, 0)
    assert relerr(host(y), ry) <= tol
    dy = rnd(rng, (N, P, P, O), dtype)
    dz = torch.zeros_like(out); dres = torch.zeros_like(out)
    dg = zeros(O); db = zeros(O)
    K.lpk_batchnorm_bwd(dtype, dev(dy, dtype), y, out, mean, rstd, dev(g, 0), dz, dres, dg, db, rows, O, 1, 0, scratch)
    dy_eff = dy.astype(np.float64) * (host(y) > 0)
    rdz, rdg, rdb = ops.batchnorm_bwd(cache, g.astype(np.float64), dy_eff)
    assert relerr(host(dz), rdz) <= (6e-3 if dtype else 2e-5)
    assert relerr(host(dres), dy_eff) <= 1e-7
    assert relerr(host(dg), rdg) <= 2e-5 and relerr(host(db), rdb) <= 2e-5


# Weight gradients of one layer as one grouped launch: products of different sizes over the same rows.
GROUPS = [
    # (K, [(M, N), ...]): a decoder layer's four at width 768 / FFN 3072; ragged sizes; more tiles than blocks
    (8192, [(768, 3072), (3072, 768), (768, 768), (2304, 768)]),
    (2048, [(264, 520), (520, 136), (8, 8), (1000, 264), (136, 776)]),
    (512, [(4096, 4104), (2056, 1032)]),
    (1056, [(520, 264), (264, 776), (2056, 520)]),       # K not a multiple of 64: the 32-deep k-tiles
]


@pytest.mark.parametrize("a_kc,b_kc", [(0, 0), (1, 1), (1, 0)])
@pytest.mark.parametrize("gi", [0, 1, 2, 3])
def test_gemm_grouped(K, gi, a_kc, b_kc):
    """Every product of a grouped launch against the CPU oracle's linear layer in float64, with and without
    accumulation onto existing outputs; bit-repeatable; and the same bits as each product launched alone where the
    two cut the reduction identically is not required (different cuts add partial sums in a different order)."""
    import torch
    Kd, shapes = GROUPS[gi]
    rng = np.random.default_rng(17 + gi)
    ws = zeros(1 << 25)
    As, Bs, refs = [], [], []
    for (M, N) in shapes:
        A = rnd(rng, (M, Kd), 1, 0.5)
        B = rnd(rng, (N, Kd), 1, 0.5)
        As.append(dev(A if a_kc else np.ascontiguousarray(A.T), 1))
        Bs.append(dev(B if b_kc else np.ascontiguousarray(B.T), 1))
        refs.append(oracle_product(f"grp{gi}", A, B))
    Ms, Ns = [m for m, _ in shapes], [n for _, n in shapes]
    outs = [torch.full((m, n), 3.0, device="cuda", dtype=torch.float32) for m, n in shapes]
    K.lpk_gemm_grouped(As, Bs, outs, Ms, Ns, Kd, a_kc, b_kc, 0, ws)
    for o, r, sh in zip(outs, refs, shapes):
        err = float((o.double() - r).norm() / r.norm())
        assert err <= 2e-6, (sh, err)
    again = [torch.zeros_like(o) for o in outs]
    K.lpk_gemm_grouped(As, Bs, again, Ms, Ns, Kd, a_kc, b_kc, 0, ws)
    for o, a in zip(outs, again):
        assert torch.equal(o, a)
    acc = [torch.full((m, n), 0.5, device="cuda", dtype=torch.float32) for m, n in shapes]
    K.lpk_gemm_grouped(As, Bs, acc, Ms, Ns, Kd, a_kc, b_kc, 1, ws)
    for o, r, sh in zip(acc, refs, shapes):
        err = float((o.double() - (r + 0.5)).norm() / r.norm())
        assert err <= 2e-6, (sh, "accumulate", err)


def test_gemm_grouped_with_epilogues(K):
    """Twelve same-shaped forward products of independent blocks in one launch (the pipelined schedule's layer
    GEMMs): bf16 outputs through each problem's own fused epilogue (bias, ReLU, residual), ragged row counts."""
    import torch
    rng = np.random.default_rng(23)
    ws = zeros(1 << 25)
    Kd, N = 256, 520
    Ms = [1304, 1304, 776, 8, 1304, 2056, 1304, 1304, 600, 1304, 1304, 1304]
    W = [rnd(rng, (N, Kd), 1, 0.5) for _ in Ms]
    X = [rnd(rng, (m, Kd), 1, 0.5) for m in Ms]
    bias = [rng.standard_normal(N).astype(np.float32) for _ in Ms]
    res = [rnd(rng, (m, N), 1) for m in Ms]
    outs = [torch.zeros(m, N, device="cuda", dtype=torch.bfloat16) for m in Ms]
    K.lpk_gemm_grouped([dev(x, 1) for x in X], [dev(w, 1) for w in W], outs, Ms, [N] * len(Ms), Kd, 1, 1, 0, ws,
                       biases=[dev(b, 0) for b in bias], act=1, ress=[dev(r, 1) for r in res])
    for i, m in enumerate(Ms):
        ref = np.maximum(ops.linear_fwd(X[i].astype(np.float64), W[i].astype(np.float64), bias[i].astype(np.float64)), 0.0) + res[i]
        assert relerr(host(outs[i]), ref) <= 4e-3, (i, m)


def test_gemm_grouped_rejects_mixed_reductions(K):
    import torch
    ws = zeros(1 << 25)
    a = torch.zeros(64, 64, device="cuda", dtype=torch.bfloat16)
    o = torch.zeros(64, 64, device="cuda", dtype=torch.float32)
    with pytest.raises(RuntimeError):
        K.lpk_gemm_grouped([a], [a], [o], [64], [64], 64, 1, 1, 0, ws)            # a single product is not a group
    with pytest.raises(RuntimeError):
        K.lpk_gemm_grouped([a, a], [a, a], [o, o], [64, 64], [64, 64], 40, 1, 1, 0, ws)   # K not a multiple of 32


@pytest.mark.parametrize("variant", [20, 21, 22])
@pytest.mark.parametrize("a_kc,b_kc", [(1, 1), (1, 0), (0, 0), (0, 1)])
def test_gemm_persistent_64_deep_k_tiles(K, variant, a_kc, b_kc):
    """The direct-to-LDS kernel with 64-deep k-tiles (K a multiple of 64), tail whole / cut along k / panel mode:
    against the CPU oracle's linear layer, with a fused epilogue, and bit-repeatable."""
    import torch
    rng = np.random.default_rng(11 if variant != 22 else 13)
    ws = zeros(1 << 25)
    for (M, N, Kd) in (DMA_SHAPES if variant != 22 else PANEL_SHAPES):
        A = rnd(rng, (M, Kd), 1, 0.5)
        B = rnd(rng, (N, Kd), 1, 0.5)
        if Kd % 64:
            continue
        Am = A if a_kc else np.ascontiguousarray(A.T)
        Bm = B if b_kc else np.ascontiguousarray(B.T)
        dA, dB = dev(Am, 1), dev(Bm, 1)
        ref = oracle_product("dma" if variant != 22 else "panel", A, B)
        out = torch.full((M, N), 7.0, device="cuda", dtype=torch.float32)
        K.lpk_gemm(1, dA, Am.shape[1], a_kc, dB, Bm.shape[1], b_kc, out, N, 1, M, N, Kd, variant=variant, splitk_ws=ws)
        err = float((out.double() - ref).norm() / ref.norm())
        assert err <= 2e-6, (M, N, Kd, variant, err)
        bias = rng.standard_normal(N).astype(np.float32)
        res = rnd(rng, (M, N), 1)
        outb = torch.zeros(M, N, device="cuda", dtype=torch.bfloat16)
        K.lpk_gemm(1, dA, Am.shape[1], a_kc, dB, Bm.shape[1], b_kc, outb, N, 0, M, N, Kd, bias=dev(bias, 0), res=dev(res, 1),
                   ldr=N, variant=variant, splitk_ws=ws)
        refb = ref + torch.from_numpy(bias).cuda().double() + torch.from_numpy(res).cuda().double()
        errb = float((outb.double() - refb).norm() / refb.norm())
        assert errb <= 4e-3, (M, N, Kd, variant, errb)
        out2 = torch.zeros_like(out)
        K.lpk_gemm(1, dA, Am.shape[1], a_kc, dB, Bm.shape[1], b_kc, out2, N, 1, M, N, Kd, variant=variant, splitk_ws=ws)
        assert torch.equal(out, out2)


@pytest.mark.parametrize("variant", [5, 6, 20, 21])
@pytest.mark.parametrize("a_kc,b_kc", [(1, 1), (1, 0)])
def test_gemm_persistent_fused_epilogues(K, variant, a_kc, b_kc):
    """Every fused epilogue of the direct-to-LDS kernel (whole sub-tiles through the row-layout path, ragged edges
    through the element path): bias + GELU / ReLU with the stored pre-activation and a residual, and the backward
    forms (activation derivative from a stored source, residual added), against float64 from the CPU oracle's ops."""
    import torch
    rng = np.random.default_rng(17)
    ws = zeros(1 << 25)
    for (M, N, Kd) in [(520, 264, 256), (2056, 776, 128), (4096, 1024, 64)]:
        A = rnd(rng, (M, Kd), 1, 0.5)
        B = rnd(rng, (N, Kd), 1, 0.5)
        bias = rng.standard_normal(N).astype(np.float32)
        ldr, ldd = N + 8, N + 16                                   # strided residual and derivative source
        res = rnd(rng, (M, ldr), 1)
        dsrc = rnd(rng, (M, ldd), 1)
        Am = A if a_kc else np.ascontiguousarray(A.T)
        Bm = B if b_kc else np.ascontiguousarray(B.T)
        dA, dB, dres, dds, dbias = dev(Am, 1), dev(Bm, 1), dev(res, 1), dev(dsrc, 1), dev(bias, 0)
        ref0 = A.astype(np.float64) @ B.astype(np.float64).T
        v = ref0 + bias
        for act, fwd in ((2, ops.gelu_fwd), (1, lambda z: np.maximum(z, 0.0))):
            out = torch.full((M, N), 3.0, device="cuda", dtype=torch.bfloat16)
            pre = torch.full((M, N), 3.0, device="cuda", dtype=torch.bfloat16)
            K.lpk_gemm(1, dA, Am.shape[1], a_kc, dB, Bm.shape[1], b_kc, out, N, 0, M, N, Kd, bias=dbias, act=act, pre=pre,
                       res=dres, ldr=ldr, variant=variant, splitk_ws=ws)
            want = fwd(v) + res[:, :N]
            assert relerr(host(pre), v) <= 4e-3, (M, N, Kd, variant, "pre")
            assert relerr(host(out), want) <= 4e-3, (M, N, Kd, variant, "act", act)
            assert np.max(np.abs(host(out).astype(np.float64) - want)) <= 0.02 * max(1.0, np.max(np.abs(want)))
        for dact, fn in ((1, lambda s, g: g * (s > 0)), (2, ops.gelu_bwd)):
            out = torch.full((M, N), 3.0, device="cuda", dtype=torch.bfloat16)
            K.lpk_gemm(1, dA, Am.shape[1], a_kc, dB, Bm.shape[1], b_kc, out, N, 0, M, N, Kd, dact_src=dds, dact=dact, ldd=ldd,
                       res=dres, ldr=ldr, variant=variant, splitk_ws=ws)
            want = fn(dsrc[:, :N].astype(np.float64), ref0) + res[:, :N]
            assert relerr(host(out), want) <= 4e-3, (M, N, Kd, variant, "dact", dact)
            assert np.max(np.abs(host(out).astype(np.float64) - want)) <= 0.02 * max(1.0, np.max(np.abs(want)))


@pytest.mark.parametrize("N,H,C,O,R,stride,pad", [(4, 16, 16, 64, 3, 1, 1), (8, 16, 32, 128, 3, 1, 1), (16, 16, 64, 256, 3, 2, 1),
                                                  (64, 8, 16, 64, 1, 2, 0), (100, 32, 8, 64, 3, 1, 1), (2, 32, 8, 192, 3, 1, 1),
                                                  (3, 10, 16, 64, 3, 1, 1), (5, 12, 24, 72, 3, 1, 1)])
def test_conv_bn_unit_forward(K, N, H, C, O, R, stride, pad):
    """A convolution + normalisation unit in one call (the convolution leaves the normalisation's column sums where its
    output is whole tiles, 128- and 256-row tiles, 64 and 128 columns wide: the first five shapes; the others fall back
    to the separate statistics pass): z, the batch
    mean and 1 / sqrt(var + eps), and y against the CPU oracle's convolution and batch normalisation, and the same
    bits as the two separate calls for z; twice: bit-repeatable."""
    import torch
    rng = np.random.default_rng(N * 100 + H)
    x = rnd(rng, (N, H, H, C), 1)
    w = rnd(rng, (O, R, R, C), 1, 0.3)
    P = (H + 2 * pad - R) // stride + 1
    g = rng.standard_normal(O).astype(np.float32); b = rng.standard_normal(O).astype(np.float32)
    res = rnd(rng, (N, P, P, O), 1)
    scratch = zeros(max(3 * (N * P * P // 32 + O), (2 * 1024 + 2) * O) + 64)
    outs = []
    for rep in range(2):
        z = torch.zeros(N, P, P, O, device="cuda", dtype=torch.bfloat16)
        y = torch.zeros_like(z); mean = zeros(O); rstd = zeros(O)
        K.lpk_conv_bn_fwd(1, dev(x, 1), dev(w, 1), z, dev(g, 0), dev(b, 0), dev(res, 1), y, mean, rstd, N, H, H, C, O, R,
                          stride, pad, 1, scratch)
        outs.append((z, y, mean, rstd))
    z, y, mean, rstd = outs[0]
    for a_, b_ in zip(outs[0], outs[1]):
        assert torch.equal(a_, b_)
    z2 = torch.zeros_like(z)
    K.lpk_conv_fwd(1, dev(x, 1), dev(w, 1), z2, N, H, H, C, O, R, stride, pad)
    assert torch.equal(z, z2)
    ref = ops.conv2d_fwd(x.astype(np.float64), w.astype(np.float64), stride, pad)
    assert relerr(host(z), ref) <= 4e-3
    # statistics of the stored (rounded) convolution output, exactly
    zs = host(z).astype(np.float64).reshape(-1, O)
    mu = zs.mean(0); var = zs.var(0)
    assert np.max(np.abs(host(mean) - mu)) <= 1e-5 * max(1.0, np.max(np.abs(mu)))
    assert relerr(host(rstd), 1.0 / np.sqrt(var + 1e-5)) <= 1e-5
    ry, _ = ops.batchnorm_fwd(zs.reshape(N, P, P, O), g.astype(np.float64), b.astype(np.float64))
    ry = np.maximum(ry + res, 0)
    assert relerr(host(y), ry) <= 4e-3
