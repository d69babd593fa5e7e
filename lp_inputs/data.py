"""Seeded synthetic minibatches and initial weights (no training arithmetic here).

The paper trains on CIFAR-10, ImageNet and LM1B; none of those is available, so inputs with the
same shapes and value structure stand in: Gaussian vectors / images with teacher or uniform
labels, and token streams drawn from a truncated Zipf law over the vocabulary.
"""
from __future__ import annotations

import numpy as np

from .configs import ModelCfg, param_shapes


def zipf_pmf(vocab: int, s: float = 1.1) -> np.ndarray:
    """Truncated Zipf law on ranks 1..vocab: p(r) proportional to r**-s."""
    r = np.arange(1, vocab + 1, dtype=np.float64)
    w = r ** (-s)
    return w / w.sum()


def zipf_tokens(rng: np.random.Generator, shape, vocab: int, s: float = 1.1) -> np.ndarray:
    """Token ids (= rank-1) by inverse-CDF sampling of the truncated Zipf law."""
    cdf = np.cumsum(zipf_pmf(vocab, s))
    u = rng.random(size=shape)
    ids = np.searchsorted(cdf, u, side="right")
    return np.minimum(ids, vocab - 1).astype(np.int32)


def make_batch(cfg: ModelCfg, step: int = 0, batch: int | None = None):
    """(x, y) for minibatch number ``step``.  Seeds: 1000+step for data, cfg.seed for the teacher.

    resmlp : x [B, in_dim] f32 ~ N(0,1); y = argmax of a fixed random linear teacher on x.
    resnet : x [B, H, W, C] f32 ~ N(0,1) (NHWC); y uniform over the classes.
    decoder: ids [B, S+1] Zipf(1.1); x = ids[:, :S], y = ids[:, 1:] (next-token targets).
    """
    B = cfg.batch if batch is None else batch
    rng = np.random.default_rng(1000 + step)
    kind = cfg.layers[0].kind
    if kind == "resmlp":
        d_in = cfg.layers[0].in_dim
        x = rng.standard_normal((B, d_in)).astype(np.float32)
        teacher = np.random.default_rng(cfg.seed + 7919).standard_normal((d_in, cfg.heads[0].n_classes))
        y = np.argmax(x.astype(np.float64) @ teacher, axis=1).astype(np.int32)
        return x, y
    if kind == "resnet_stage":
        l0 = cfg.layers[0]
        x = rng.standard_normal((B, l0.in_hw, l0.in_hw, l0.in_ch)).astype(np.float32)
        y = rng.integers(0, cfg.heads[0].n_classes, size=(B,)).astype(np.int32)
        return x, y
    if kind == "decoder":
        S = cfg.layers[0].seq_len
        ids = zipf_tokens(rng, (B, S + 1), cfg.vocab)
        return np.ascontiguousarray(ids[:, :S]), np.ascontiguousarray(ids[:, 1:])
    raise ValueError(kind)


def init_params(cfg: ModelCfg, seed: int | None = None, head_scale: float = 1.0) -> dict:
    """Initial fp32 weights by name.

    resmlp / conv / 10-class heads: Kaiming-normal, std = sqrt(2 / fan_in); biases 0.
    decoder and vocabulary heads: N(0, 0.02); LayerNorm / BatchNorm gain 1, shift 0.
    """
    rng = np.random.default_rng(cfg.seed if seed is None else seed)
    out = {}
    is_dec = cfg.layers[0].kind == "decoder"
    for name, shape in param_shapes(cfg).items():
        leaf = name.split(".")[-1]
        if leaf == "g":
            out[name] = np.ones(shape, np.float32)
        elif leaf in ("b", "b1", "b2", "bin", "bqkv", "bo"):
            out[name] = np.zeros(shape, np.float32)
        else:
            if is_dec:
                std = 0.02
            else:
                fan_in = int(np.prod(shape[1:]))
                std = np.sqrt(2.0 / fan_in)
            if name.startswith("H"):
                std *= head_scale
            out[name] = (rng.standard_normal(shape) * std).astype(np.float32)
    return out


def perturb_params(params: dict, seed: int, scale: float = 0.05) -> dict:
    """Make biases/gains generic (non-zero, non-one) so tests exercise every term."""
    rng = np.random.default_rng(seed)
    out = {}
    for k, v in params.items():
        out[k] = (v + scale * rng.standard_normal(v.shape)).astype(np.float32)
    return out
