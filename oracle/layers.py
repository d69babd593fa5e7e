"""Atomic layers and auxiliary heads of the CPU oracle (test infrastructure only).

A layer is a pair forward(params, x) -> (out, cache) and backward(params, cache, dout, need_dx)
-> (dx, grads).  A head is loss(params, h, y) -> (loss, cache) and backward(...) -> (dh, grads).
Layer forms: residual MLP block (appendix A, "MLP"), pre-LN causal decoder layer (appendix B.2),
ResNet stage of BasicBlocks (appendix B.3).  Head forms follow the same appendices: a linear
classifier, spatial mean + linear classifier, and LayerNorm + linear projection to the vocabulary,
each under softmax cross-entropy (section 3: auxiliary objectives take the form of the global one).
"""
from __future__ import annotations

import numpy as np

from . import ops


# ============================================================================= residual MLP
def resmlp_fwd(P, pre, l, x, q=ops.identity):
    cache = {"x": x}
    if l.in_dim != l.width:
        p = q(ops.linear_fwd(x, P[pre + "win"], P[pre + "bin"]))
    else:
        p = x
    a = ops.linear_fwd(p, P[pre + "w1"], P[pre + "b1"])
    r = q(ops.relu_fwd(a))
    out = q(p + ops.linear_fwd(r, P[pre + "w2"], P[pre + "b2"]))
    cache.update(p=p, a=a, r=r)
    return out, cache


def resmlp_bwd(P, pre, l, cache, dout, need_dx=True):
    g = {}
    dr, g[pre + "w2"], g[pre + "b2"] = ops.linear_bwd(cache["r"], P[pre + "w2"], dout)
    da = ops.relu_bwd(cache["r"], dr)          # r > 0 exactly where a > 0
    dp, g[pre + "w1"], g[pre + "b1"] = ops.linear_bwd(cache["p"], P[pre + "w1"], da)
    dp = dp + dout
    if l.in_dim != l.width:
        dx, g[pre + "win"], g[pre + "bin"] = ops.linear_bwd(cache["x"], P[pre + "win"], dp)
    else:
        dx = dp
    return (dx if need_dx else None), g


# ============================================================================= decoder layer
def _split_heads(t, B, S, H):
    d = t.shape[-1]
    return t.reshape(B, S, H, d // H).transpose(0, 2, 1, 3)


def _merge_heads(t):
    B, H, S, dh = t.shape
    return t.transpose(0, 2, 1, 3).reshape(B * S, H * dh)


def decoder_fwd(P, pre, l, x, first, vocab, q=ops.identity):
    """x: token ids [B, S] if this is layer 1 of a model with an embedding, else h [B*S, d]."""
    S, d, H = l.seq_len, l.width, l.n_heads
    cache = {}
    if first and vocab > 0:
        ids = x
        B = ids.shape[0]
        emb = P[pre + "emb"]
        pe = ops.sinusoid_positions(S, d, emb.dtype)
        h = q(ops.embed_fwd(ids, emb, pe).reshape(B * S, d))
        cache["ids"] = ids
    else:
        h = x
        B = h.shape[0] // S
    a, c_ln1 = ops.layernorm_fwd(h, P[pre + "ln1.g"], P[pre + "ln1.b"])
    a = q(a)
    qkv = q(ops.linear_fwd(a, P[pre + "wqkv"], P[pre + "bqkv"]))
    qh = _split_heads(qkv[:, :d], B, S, H)
    k = _split_heads(qkv[:, d:2 * d], B, S, H)
    v = _split_heads(qkv[:, 2 * d:], B, S, H)
    o4, p = ops.attention_fwd(qh, k, v, causal=bool(l.causal))
    o = q(_merge_heads(o4))
    u = q(h + ops.linear_fwd(o, P[pre + "wo"], P[pre + "bo"]))
    c, c_ln2 = ops.layernorm_fwd(u, P[pre + "ln2.g"], P[pre + "ln2.b"])
    c = q(c)
    f_exact = ops.linear_fwd(c, P[pre + "w1"], P[pre + "b1"])
    f = q(ops.gelu_fwd(f_exact) if l.act == "gelu" else ops.relu_fwd(f_exact))
    f_pre = q(f_exact)
    out = q(u + ops.linear_fwd(f, P[pre + "w2"], P[pre + "b2"]))
    cache.update(B=B, a=a, c_ln1=c_ln1, q=qh, k=k, v=v, p=p, o=o, c=c, c_ln2=c_ln2, f_pre=f_pre, f=f)
    return out, cache


def decoder_bwd(P, pre, l, cache, dout, need_dx, first, vocab):
    S, d, H = l.seq_len, l.width, l.n_heads
    B = cache["B"]
    g = {}
    df, g[pre + "w2"], g[pre + "b2"] = ops.linear_bwd(cache["f"], P[pre + "w2"], dout)
    dpre = ops.gelu_bwd(cache["f_pre"], df) if l.act == "gelu" else ops.relu_bwd(cache["f_pre"], df)
    dc, g[pre + "w1"], g[pre + "b1"] = ops.linear_bwd(cache["c"], P[pre + "w1"], dpre)
    du_ln, g[pre + "ln2.g"], g[pre + "ln2.b"] = ops.layernorm_bwd(cache["c_ln2"], P[pre + "ln2.g"], dc)
    du = dout + du_ln
    do, g[pre + "wo"], g[pre + "bo"] = ops.linear_bwd(cache["o"], P[pre + "wo"], du)
    do4 = _split_heads(do, B, S, H)
    dq, dk, dv = ops.attention_bwd(cache["q"], cache["k"], cache["v"], cache["p"], do4)
    dqkv = np.concatenate([_merge_heads(dq), _merge_heads(dk), _merge_heads(dv)], axis=1)
    da, g[pre + "wqkv"], g[pre + "bqkv"] = ops.linear_bwd(cache["a"], P[pre + "wqkv"], dqkv)
    dh_ln, g[pre + "ln1.g"], g[pre + "ln1.b"] = ops.layernorm_bwd(cache["c_ln1"], P[pre + "ln1.g"], da)
    dh = du + dh_ln
    if first and vocab > 0:
        g[pre + "emb"] = ops.embed_bwd(cache["ids"], vocab, dh.reshape(B, S, d))
        return None, g
    return (dh if need_dx else None), g


# ============================================================================= ResNet stage
def _conv_bn(P, wname, bnpre, x, stride, pad, relu, res=None, q=ops.identity, bn=None):
    """out = [relu]( BN(conv(x)) [+ res] ); the conv output and the result are stored activations."""
    z = q(ops.conv2d_fwd(x, P[wname], stride, pad))
    y, bnc = ops.batchnorm(z, P[bnpre + "g"], P[bnpre + "b"], bn, bnpre)
    if res is not None:
        y = y + res
    out = q(ops.relu_fwd(y) if relu else y)
    return out, {"x": x, "bn": bnc, "out": out, "stride": stride, "pad": pad, "relu": relu}


def _conv_bn_bwd(P, wname, bnpre, c, dout, g, need_dx=True):
    """Returns (dx, dy) where dy is dout masked by the unit's ReLU (= gradient of the residual input)."""
    dy = ops.relu_bwd(c["out"], dout) if c["relu"] else dout     # out > 0 exactly where the pre-ReLU value is
    dz, g[bnpre + "g"], g[bnpre + "b"] = ops.batchnorm_bwd(c["bn"], P[bnpre + "g"], dy)
    dx, g[wname] = ops.conv2d_bwd(c["x"], P[wname], c["stride"], c["pad"], dz, need_dx)
    return dx, dy


def resnet_stage_fwd(P, pre, l, x, q=ops.identity, bn=None):
    """stem (optional) then n BasicBlocks: relu(bn2(conv2(relu(bn1(conv1 x)))) + shortcut(x))."""
    cache = {"blocks": []}
    h = x
    if l.has_stem:
        h, cache["stem"] = _conv_bn(P, pre + "stem.w", pre + "stem.bn.", h, 1, 1, True, q=q, bn=bn)
    for b in range(l.n_basic_blocks):
        n = pre + f"b{b + 1}."
        stride = l.stride if (b == 0 and not l.has_stem) else 1
        bc = {"in": h}
        t, bc["c1"] = _conv_bn(P, n + "conv1.w", n + "bn1.", h, stride, 1, True, q=q, bn=bn)
        if (n + "proj.w") in P:
            sc, bc["proj"] = _conv_bn(P, n + "proj.w", n + "proj.bn.", h, stride, 0, False, q=q, bn=bn)
        else:
            sc = h
        h, bc["c2"] = _conv_bn(P, n + "conv2.w", n + "bn2.", t, 1, 1, True, res=sc, q=q, bn=bn)
        cache["blocks"].append(bc)
    return h, cache


def resnet_stage_bwd(P, pre, l, cache, dout, need_dx=True):
    g = {}
    dh = dout
    for b in reversed(range(l.n_basic_blocks)):
        q = pre + f"b{b + 1}."
        bc = cache["blocks"][b]
        first_op = (b == 0 and not l.has_stem)
        dt, ds = _conv_bn_bwd(P, q + "conv2.w", q + "bn2.", bc["c2"], dh, g)
        want_dx = need_dx or not first_op
        dx_main, _ = _conv_bn_bwd(P, q + "conv1.w", q + "bn1.", bc["c1"], dt, g, want_dx)
        if "proj" in bc:
            dx_sc, _ = _conv_bn_bwd(P, q + "proj.w", q + "proj.bn.", bc["proj"], ds, g, want_dx)
        else:
            dx_sc = ds
        dh = (dx_main + dx_sc) if want_dx else None
    if l.has_stem:
        dh, _ = _conv_bn_bwd(P, pre + "stem.w", pre + "stem.bn.", cache["stem"], dh, g, need_dx)
    return (dh if need_dx else None), g


# ============================================================================= dispatch
def layer_fwd(cfg, P, li, x, q=ops.identity, bn=None):
    l = cfg.layers[li - 1]
    pre = f"L{li}."
    if l.kind == "resmlp":
        return resmlp_fwd(P, pre, l, x, q)
    if l.kind == "decoder":
        return decoder_fwd(P, pre, l, x, li == 1, cfg.vocab, q)
    if l.kind == "resnet_stage":
        return resnet_stage_fwd(P, pre, l, x, q, bn)
    raise ValueError(l.kind)


def layer_bwd(cfg, P, li, cache, dout, need_dx):
    l = cfg.layers[li - 1]
    pre = f"L{li}."
    if l.kind == "resmlp":
        return resmlp_bwd(P, pre, l, cache, dout, need_dx)
    if l.kind == "decoder":
        return decoder_bwd(P, pre, l, cache, dout, need_dx, li == 1, cfg.vocab)
    if l.kind == "resnet_stage":
        return resnet_stage_bwd(P, pre, l, cache, dout, need_dx)
    raise ValueError(l.kind)


# ============================================================================= heads
def head_loss(cfg, P, hi, h, y, q=ops.identity, bn=None):
    """Auxiliary objective of head hi on activation h with labels y.  Returns (loss, cache)."""
    hd = cfg.heads[hi - 1]
    pre = f"H{hi}."
    cache = {}
    if hd.kind == "pool_linear_ce":
        feat = q(h.mean(axis=(1, 2)))
        cache["hw_shape"] = h.shape
    elif hd.kind == "bn_pool_linear_ce":
        # appendix B.3: batch normalisation, ReLU, mean over the spatial dimensions, then the linear projection
        a, cache["bn"] = ops.batchnorm(h, P[pre + "bn.g"], P[pre + "bn.b"], bn, pre + "bn.")
        a = q(ops.relu_fwd(a))
        cache["a"] = a
        feat = q(a.mean(axis=(1, 2)))
        cache["hw_shape"] = h.shape
    elif hd.kind == "ln_linear_ce":
        feat, cache["ln"] = ops.layernorm_fwd(h, P[pre + "ln.g"], P[pre + "ln.b"])
        feat = q(feat)
    elif hd.kind == "linear_ce":
        feat = h
    else:
        raise ValueError(hd.kind)
    z = q(ops.linear_fwd(feat, P[pre + "w"], P[pre + "b"] if hd.bias else None))
    yy = y.reshape(-1)
    loss, p = ops.softmax_ce_fwd(z, yy)
    cache.update(feat=feat, p=p, y=yy)
    return loss, cache


def head_bwd(cfg, P, hi, cache):
    """Returns (d loss / d h, grads of the head's own parameters)."""
    hd = cfg.heads[hi - 1]
    pre = f"H{hi}."
    g = {}
    dz = ops.softmax_ce_bwd(cache["p"], cache["y"])
    dfeat, g[pre + "w"], db = ops.linear_bwd(cache["feat"], P[pre + "w"], dz, bool(hd.bias))
    if hd.bias:
        g[pre + "b"] = db
    if hd.kind == "pool_linear_ce":
        N, Hh, Ww, C = cache["hw_shape"]
        dh = np.broadcast_to(dfeat[:, None, None, :] / (Hh * Ww), (N, Hh, Ww, C)).copy()
    elif hd.kind == "bn_pool_linear_ce":
        N, Hh, Ww, C = cache["hw_shape"]
        da = np.broadcast_to(dfeat[:, None, None, :] / (Hh * Ww), (N, Hh, Ww, C))
        da = ops.relu_bwd(cache["a"], da)            # the stored post-ReLU activation decides
        dh, g[pre + "bn.g"], g[pre + "bn.b"] = ops.batchnorm_bwd(cache["bn"], P[pre + "bn.g"], da)
    elif hd.kind == "ln_linear_ce":
        dh, g[pre + "ln.g"], g[pre + "ln.b"] = ops.layernorm_bwd(cache["ln"], P[pre + "ln.g"], dfeat)
    else:
        dh = dfeat
    return dh, g
