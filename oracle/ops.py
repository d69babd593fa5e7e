"""Primitive operations of the CPU oracle, each as a forward/backward pair in plain numpy.

TEST INFRASTRUCTURE ONLY.  Nothing in the product path may import this package; it exists so
that tests, the smoke check and the bench's CPU-baseline leg have an independent, slow and
obviously-correct statement of what the local-update step computes.  It shares no code with the
HIP kernels.

Every function here is the textbook definition written out (the paper names these operations
but does not define them: section 3 for the auxiliary objective "of the same form as the global
objective", appendix B for the per-model layers and heads).  Arithmetic runs in the dtype of the
inputs: float64 for parity, float32 when the bench times it.
"""
from __future__ import annotations

import numpy as np

LN_EPS = 1e-5
BN_EPS = 1e-5


# ----------------------------------------------------------------------------- storage precision
def bf16_round(x):
    """Round to the nearest bfloat16 (ties to even) and return in the input's float type.

    Used only in the "stored-activation precision" mode of the oracle: a configuration that says
    "bf16 compute" stores every forward activation and every matrix weight operand as bf16, and the
    ReLU on/off decisions are then taken on those stored values.  Arithmetic stays in float64."""
    a = np.asarray(x, dtype=np.float32)
    u = a.view(np.uint32).astype(np.uint64)
    r = ((u + 0x7FFF + ((u >> 16) & 1)) >> 16) << 16
    out = r.astype(np.uint32).view(np.float32)
    out = np.where(np.isfinite(a), out, a)
    return out.astype(np.asarray(x).dtype if np.asarray(x).dtype.kind == "f" else np.float64)


def identity(x):
    return x


# ----------------------------------------------------------------------------- linear
def linear_fwd(x, w, b=None):
    """y[n, o] = sum_i x[n, i] w[o, i] (+ b[o]);  w is [out, in]."""
    y = x @ w.T
    if b is not None:
        y = y + b
    return y


def linear_bwd(x, w, dy, has_bias=True):
    """Returns (dx, dw, db) for y = x w^T + b."""
    dx = dy @ w
    dw = dy.T @ x
    db = dy.sum(axis=0) if has_bias else None
    return dx, dw, db


# ----------------------------------------------------------------------------- activations
def relu_fwd(x):
    return np.maximum(x, 0)


def relu_bwd(x, dy):
    return dy * (x > 0)


_GELU_C = 0.7978845608028654  # sqrt(2/pi)
_GELU_A = 0.044715


def gelu_fwd(x):
    """tanh-form GELU: 0.5 x (1 + tanh(sqrt(2/pi) (x + 0.044715 x^3)))."""
    return 0.5 * x * (1.0 + np.tanh(_GELU_C * (x + _GELU_A * x ** 3)))


def gelu_bwd(x, dy):
    t = np.tanh(_GELU_C * (x + _GELU_A * x ** 3))
    dt = (1.0 - t * t) * _GELU_C * (1.0 + 3.0 * _GELU_A * x * x)
    return dy * (0.5 * (1.0 + t) + 0.5 * x * dt)


# ----------------------------------------------------------------------------- normalisation
def layernorm_fwd(x, g, b):
    """Over the last dim, biased variance, eps 1e-5, affine.  Returns (y, cache)."""
    mu = x.mean(axis=-1, keepdims=True)
    xc = x - mu
    var = (xc * xc).mean(axis=-1, keepdims=True)
    rstd = 1.0 / np.sqrt(var + LN_EPS)
    xhat = xc * rstd
    return xhat * g + b, (xhat, rstd)


def layernorm_bwd(cache, g, dy):
    xhat, rstd = cache
    dg = (dy * xhat).reshape(-1, xhat.shape[-1]).sum(axis=0)
    db = dy.reshape(-1, xhat.shape[-1]).sum(axis=0)
    dxhat = dy * g
    m1 = dxhat.mean(axis=-1, keepdims=True)
    m2 = (dxhat * xhat).mean(axis=-1, keepdims=True)
    dx = (dxhat - m1 - xhat * m2) * rstd
    return dx, dg, db


def batchnorm_fwd(x, g, b):
    """x is [N, H, W, C]; statistics of the current batch over (N, H, W); biased variance."""
    C = x.shape[-1]
    x2 = x.reshape(-1, C)
    mu = x2.mean(axis=0)
    xc = x2 - mu
    var = (xc * xc).mean(axis=0)
    rstd = 1.0 / np.sqrt(var + BN_EPS)
    xhat = xc * rstd
    return (xhat * g + b).reshape(x.shape), (xhat, rstd)


def batchnorm_running_fwd(x, g, b, run_mean, run_var):
    """Normalisation with fixed per-channel statistics (evaluation form of Ioffe & Szegedy's batch
    normalisation, which appendix B.3 cites): y = (x - run_mean) / sqrt(run_var + eps) * g + b."""
    return (x - run_mean) / np.sqrt(run_var + BN_EPS) * g + b


class BatchNormRunning:
    """Running per-channel statistics of every batch normalisation, keyed by the parameter prefix.

    The paper does not say how its ResNets normalise at evaluation time; this takes the usual convention
    of the method it cites: an exponential moving average with weight ``momentum`` on the newest batch,
        run_mean <- (1 - momentum) run_mean + momentum * mean_B
        run_var  <- (1 - momentum) run_var  + momentum * var_B * n / (n - 1)    (unbiased batch variance)
    started from mean 0, variance 1.  ``mode`` selects what a forward pass does with it:
    "update" normalises with the statistics of the batch and folds them in, "use" normalises with the
    running ones, "batch" ignores it."""

    def __init__(self, momentum=0.1, mode="update"):
        self.momentum = float(momentum)
        self.mode = mode
        self.mean = {}
        self.var = {}

    def ensure(self, name, C):
        if name not in self.mean:
            self.mean[name] = np.zeros(C)
            self.var[name] = np.ones(C)

    def observe(self, name, x):
        C = x.shape[-1]
        x2 = np.asarray(x, dtype=np.float64).reshape(-1, C)
        n = x2.shape[0]
        mu = x2.mean(axis=0)
        var = ((x2 - mu) ** 2).mean(axis=0)
        if n > 1:
            var = var * n / (n - 1)
        self.ensure(name, C)
        m = self.momentum
        self.mean[name] = (1.0 - m) * self.mean[name] + m * mu
        self.var[name] = (1.0 - m) * self.var[name] + m * var


def batchnorm(x, g, b, running=None, name=None):
    """Batch normalisation as a forward pass sees it: (y, cache for batchnorm_bwd or None)."""
    if running is None or running.mode == "batch":
        return batchnorm_fwd(x, g, b)
    running.ensure(name, x.shape[-1])
    if running.mode == "use":
        return batchnorm_running_fwd(x, g, b, running.mean[name], running.var[name]), None
    if running.mode == "update":
        running.observe(name, x)
        return batchnorm_fwd(x, g, b)
    raise ValueError(running.mode)


def batchnorm_bwd(cache, g, dy):
    xhat, rstd = cache
    C = xhat.shape[-1]
    dy2 = dy.reshape(-1, C)
    dg = (dy2 * xhat).sum(axis=0)
    db = dy2.sum(axis=0)
    dxhat = dy2 * g
    m1 = dxhat.mean(axis=0)
    m2 = (dxhat * xhat).mean(axis=0)
    dx = (dxhat - m1 - xhat * m2) * rstd
    return dx.reshape(dy.shape), dg, db


# ----------------------------------------------------------------------------- convolution
def conv2d_fwd(x, w, stride, pad):
    """out[n,p,q,o] = sum_{r,s,c} xpad[n, p*stride+r, q*stride+s, c] * w[o,r,s,c].

    x [N,H,W,C] (NHWC), w [O,R,S,C], zero padding ``pad`` on each side, no bias.
    """
    N, H, W, C = x.shape
    O, R, S, _ = w.shape
    P = (H + 2 * pad - R) // stride + 1
    Q = (W + 2 * pad - S) // stride + 1
    xp = np.zeros((N, H + 2 * pad, W + 2 * pad, C), dtype=x.dtype)
    xp[:, pad:pad + H, pad:pad + W, :] = x
    out = np.zeros((N, P, Q, O), dtype=x.dtype)
    for r in range(R):
        for s in range(S):
            patch = xp[:, r:r + (P - 1) * stride + 1:stride, s:s + (Q - 1) * stride + 1:stride, :]
            out += patch @ w[:, r, s, :].T
    return out


def conv2d_bwd(x, w, stride, pad, dout, need_dx=True):
    """Returns (dx, dw) of conv2d_fwd."""
    N, H, W, C = x.shape
    O, R, S, _ = w.shape
    P, Q = dout.shape[1], dout.shape[2]
    xp = np.zeros((N, H + 2 * pad, W + 2 * pad, C), dtype=x.dtype)
    xp[:, pad:pad + H, pad:pad + W, :] = x
    dxp = np.zeros_like(xp)
    dw = np.zeros_like(w)
    d2 = dout.reshape(-1, O)
    for r in range(R):
        for s in range(S):
            sl = (slice(None), slice(r, r + (P - 1) * stride + 1, stride),
                  slice(s, s + (Q - 1) * stride + 1, stride), slice(None))
            dw[:, r, s, :] = d2.T @ xp[sl].reshape(-1, C)
            if need_dx:
                dxp[sl] += dout @ w[:, r, s, :]
    dx = dxp[:, pad:pad + H, pad:pad + W, :] if need_dx else None
    return dx, dw


# ----------------------------------------------------------------------------- attention
def attention_fwd(q, k, v, causal=True):
    """q, k, v: [B, H, S, dh].  o = softmax(q k^T / sqrt(dh) + mask) v, mask = -inf above diagonal."""
    dh = q.shape[-1]
    s = (q @ np.swapaxes(k, -1, -2)) / np.sqrt(dh)
    if causal:
        S = q.shape[-2]
        s = np.where(np.tril(np.ones((S, S), dtype=bool)), s, -np.inf)
    s = s - s.max(axis=-1, keepdims=True)
    p = np.exp(s)
    p = p / p.sum(axis=-1, keepdims=True)
    return p @ v, p


def attention_bwd(q, k, v, p, do):
    dh = q.shape[-1]
    dv = np.swapaxes(p, -1, -2) @ do
    dp = do @ np.swapaxes(v, -1, -2)
    ds = p * (dp - (dp * p).sum(axis=-1, keepdims=True))
    dq = (ds @ k) / np.sqrt(dh)
    dk = (np.swapaxes(ds, -1, -2) @ q) / np.sqrt(dh)
    return dq, dk, dv


# ----------------------------------------------------------------------------- loss
def softmax_ce_fwd(z, y):
    """mean_n( logsumexp(z_n) - z[n, y_n] ), max-subtracted.  Returns (loss, softmax probs)."""
    zm = z - z.max(axis=-1, keepdims=True)
    e = np.exp(zm)
    se = e.sum(axis=-1, keepdims=True)
    lse = np.log(se)
    n = z.shape[0]
    loss = (lse[:, 0] - zm[np.arange(n), y]).mean()
    return loss, e / se


def softmax_ce_bwd(p, y):
    """dz = (softmax(z) - onehot(y)) / N."""
    n = p.shape[0]
    dz = p.copy()
    dz[np.arange(n), y] -= 1.0
    return dz / n


# ----------------------------------------------------------------------------- embedding
def sinusoid_positions(S, d, dtype=np.float64):
    """PE[s, 2i] = sin(s / 10000^(2i/d)),  PE[s, 2i+1] = cos(s / 10000^(2i/d))."""
    pos = np.arange(S, dtype=np.float64)[:, None]
    i2 = (np.arange(d) // 2 * 2).astype(np.float64)[None, :]
    ang = pos / np.power(10000.0, i2 / d)
    pe = np.where(np.arange(d)[None, :] % 2 == 0, np.sin(ang), np.cos(ang))
    return pe.astype(dtype)


def embed_fwd(ids, emb, pe):
    """h[b, s, :] = emb[ids[b, s], :] + pe[s, :]."""
    return emb[ids] + pe[None, :, :]


def embed_bwd(ids, vocab, dh):
    demb = np.zeros((vocab, dh.shape[-1]), dtype=dh.dtype)
    np.add.at(demb, ids.reshape(-1), dh.reshape(-1, dh.shape[-1]))
    return demb
