"""Plain-data descriptions of the networks and local-training schemes.

A network is a list of atomic layers; a local-training scheme is a list of
auxiliary heads, each attached after layer ``after_layer`` (1-based) whose
loss is backpropagated through the last ``window`` layers ending there
(paper section 3: greedy = every layer, window 1; overlapping = every layer,
window 2; chunked = every K-th layer, window K; backprop = one head, window L).
"""
from __future__ import annotations

from dataclasses import dataclass, field, replace
from typing import List, Tuple, Dict


@dataclass(frozen=True)
class LayerCfg:
    kind: str                 # "resmlp" | "decoder" | "resnet_stage"
    in_dim: int = 0           # resmlp: input width (a projection is added if != width)
    width: int = 0            # resmlp / decoder: model width d
    hidden: int = 0           # resmlp hidden width / decoder FFN width F
    n_heads: int = 0          # decoder attention heads
    seq_len: int = 0          # decoder sequence length S
    causal: int = 1
    act: str = "gelu"         # decoder FFN activation: "gelu" (tanh form) | "relu"
    in_ch: int = 0            # resnet stage
    out_ch: int = 0
    stride: int = 1           # stride of the stage's first conv (and 1x1 projection)
    n_basic_blocks: int = 2
    has_stem: int = 0         # stage starts with conv3x3(in_ch->out_ch)+BN+ReLU
    in_hw: int = 0            # input spatial size (square)


@dataclass(frozen=True)
class HeadCfg:
    kind: str                 # "linear_ce" | "pool_linear_ce" | "ln_linear_ce" | "bn_pool_linear_ce"
    after_layer: int          # e_j, 1-based
    window: int               # w_j >= 1 (clamped to e_j)
    in_dim: int
    n_classes: int
    bias: int = 1


@dataclass(frozen=True)
class OptCfg:
    kind: str = "sgd"         # "sgd" | "sgdm" | "adam"
    lr: float = 0.1
    momentum: float = 0.9
    beta1: float = 0.9
    beta2: float = 0.999
    eps: float = 1e-8
    weight_decay: float = 0.0


@dataclass(frozen=True)
class ModelCfg:
    name: str
    layers: Tuple[LayerCfg, ...]
    heads: Tuple[HeadCfg, ...]
    opt: OptCfg
    combine: str = "sum"      # "sum" | "mean" over heads whose window covers a layer
    dtype: str = "f32"        # "f32" | "bf16" compute dtype (master weights always f32)
    batch: int = 1
    vocab: int = 0            # >0: layer 1 owns a token embedding [vocab, width]
    seed: int = 0

    @property
    def n_layers(self) -> int:
        return len(self.layers)


def head_windows(cfg: ModelCfg) -> List[Tuple[int, int]]:
    """(s_j, e_j) per head: the loss of head j reaches layers s_j+1 .. e_j."""
    out = []
    for h in cfg.heads:
        e = h.after_layer
        out.append((max(e - h.window, 0), e))
    return out


def _scheme_heads(kind: str, n_layers: int, scheme: str, in_dim_of, n_classes: int,
                  bias: int, chunk: int = 1) -> Tuple[HeadCfg, ...]:
    L = n_layers
    if scheme == "greedy":
        pos = [(k, 1) for k in range(1, L + 1)]
    elif scheme == "overlap":
        pos = [(k, 2) for k in range(1, L + 1)]
    elif scheme == "chunk":
        pos = [(k, chunk) for k in range(chunk, L + 1, chunk)]
        if L % chunk:
            pos.append((L, L % chunk))
    elif scheme == "backprop":
        pos = [(L, L)]
    elif scheme == "deep_supervision":   # every head sees everything below it (test pin)
        pos = [(k, k) for k in range(1, L + 1)]
    elif scheme.startswith("last"):
        pos = [(L, int(scheme[4:]))]
    else:
        raise ValueError(scheme)
    return tuple(HeadCfg(kind, e, w, in_dim_of(e), n_classes, bias) for e, w in pos)


def mlp_config(name, n_layers=4, in_dim=64, width=256, hidden=256, n_classes=10, batch=128,
               scheme="greedy", chunk=1, opt=None, combine="sum", seed=0) -> ModelCfg:
    layers = tuple(LayerCfg("resmlp", in_dim=(in_dim if l == 0 else width), width=width, hidden=hidden)
                   for l in range(n_layers))
    heads = _scheme_heads("linear_ce", n_layers, scheme, lambda e: width, n_classes, 1, chunk)
    return ModelCfg(name, layers, heads, opt or OptCfg("sgd", lr=0.1), combine, "f32", batch, 0, seed)


def decoder_config(name, n_layers, width, n_heads, hidden, seq_len, batch, vocab, scheme="greedy",
                   chunk=1, opt=None, combine="sum", dtype="bf16", act="gelu", seed=0) -> ModelCfg:
    layers = tuple(LayerCfg("decoder", width=width, hidden=hidden, n_heads=n_heads, seq_len=seq_len,
                            causal=1, act=act) for _ in range(n_layers))
    heads = _scheme_heads("ln_linear_ce", n_layers, scheme, lambda e: width, vocab, 0, chunk)
    return ModelCfg(name, layers, heads, opt or OptCfg("adam", lr=1e-3), combine, dtype, batch, vocab, seed)


def resnet_config(name, channels=(64, 128, 256, 512), in_hw=32, in_ch=3, n_classes=10, batch=256,
                  n_basic_blocks=2, scheme="greedy", chunk=1, opt=None, combine="sum", dtype="bf16",
                  seed=0, head="pool_linear_ce") -> ModelCfg:
    layers = []
    hw, cin = in_hw, in_ch
    for i, c in enumerate(channels):
        stride = 1 if i == 0 else 2
        layers.append(LayerCfg("resnet_stage", in_ch=cin, out_ch=c, stride=stride,
                               n_basic_blocks=n_basic_blocks, has_stem=int(i == 0), in_hw=hw))
        hw = hw // stride
        cin = c
    layers = tuple(layers)
    heads = _scheme_heads(head, len(layers), scheme, lambda e: layers[e - 1].out_ch,
                          n_classes, 1, chunk)
    return ModelCfg(name, layers, heads, opt or OptCfg("sgdm", lr=0.1, momentum=0.9), combine, dtype,
                    batch, 0, seed)


CONFIG_NAMES = ("cfg1", "cfg2", "cfg3", "cfg4", "cfg5")


def make_config(name: str, **over) -> ModelCfg:
    """The five benchmark configurations, plus scaled-down ``*_small`` forms for tests.

    cfg1: 4-block residual MLP, greedy, fp32, SGD 0.1, batch 128.
    cfg2: 4-stage ResNet-18-style CNN on 32x32x3, greedy per stage, bf16, SGD-momentum.
    cfg3: 12-layer decoder (d 768, 12 heads, FFN 3072, seq 1024, batch 8, vocab 32000), greedy, Adam.
    cfg4: cfg3 with overlapping windows of 2 layers, contributions summed.
    cfg5: 24-layer decoder (d 1024, 16 heads, FFN 4096, seq 2048, batch 4), 6 chunks of 4 layers.
    """
    if name == "cfg1":
        return mlp_config("cfg1", **over)
    if name == "cfg2":
        return resnet_config("cfg2", **over)
    if name == "cfg3":
        kw = dict(n_layers=12, width=768, n_heads=12, hidden=3072, seq_len=1024, batch=8, vocab=32000,
                  scheme="greedy")
        kw.update(over)
        return decoder_config("cfg3", **kw)
    if name == "cfg4":
        kw = dict(n_layers=12, width=768, n_heads=12, hidden=3072, seq_len=1024, batch=8, vocab=32000,
                  scheme="overlap", combine="sum")
        kw.update(over)
        return decoder_config("cfg4", **kw)
    if name == "cfg5":
        kw = dict(n_layers=24, width=1024, n_heads=16, hidden=4096, seq_len=2048, batch=4, vocab=32000,
                  scheme="chunk", chunk=4)
        kw.update(over)
        return decoder_config("cfg5", **kw)
    # scaled-down versions: same structure, sizes the oracle finishes in seconds; deliberately
    # ragged (vocab, tokens and widths that are not multiples of the kernels' tiles).
    if name == "cfg1_small":
        kw = dict(n_layers=3, in_dim=24, width=40, hidden=56, batch=19)
        kw.update(over)
        return mlp_config("cfg1_small", **kw)
    if name == "cfg2_small":
        kw = dict(channels=(8, 16, 24), in_hw=12, batch=6, n_basic_blocks=1)
        kw.update(over)
        return resnet_config("cfg2_small", **kw)
    if name == "cfg3_small":
        kw = dict(n_layers=3, width=128, n_heads=2, hidden=320, seq_len=200, batch=3, vocab=1000,
                  scheme="greedy")
        kw.update(over)
        return decoder_config("cfg3_small", **kw)
    if name == "cfg4_small":
        kw = dict(n_layers=4, width=128, n_heads=2, hidden=320, seq_len=200, batch=3, vocab=1000,
                  scheme="overlap", combine="sum")
        kw.update(over)
        return decoder_config("cfg4_small", **kw)
    if name == "cfg5_small":
        kw = dict(n_layers=6, width=128, n_heads=2, hidden=320, seq_len=200, batch=2, vocab=1000,
                  scheme="chunk", chunk=3)
        kw.update(over)
        return decoder_config("cfg5_small", **kw)
    raise KeyError(name)


def param_shapes(cfg: ModelCfg) -> Dict[str, Tuple[int, ...]]:
    """Name -> shape of every trainable tensor, in storage order (layers, then heads).

    Linear weights are [out, in]; conv weights are [C_out, KH, KW, C_in]; the token embedding is
    [vocab, d] and belongs to layer 1.
    """
    shapes: Dict[str, Tuple[int, ...]] = {}
    for li, l in enumerate(cfg.layers, start=1):
        p = f"L{li}."
        if l.kind == "resmlp":
            if l.in_dim != l.width:
                shapes[p + "win"] = (l.width, l.in_dim)
                shapes[p + "bin"] = (l.width,)
            shapes[p + "w1"] = (l.hidden, l.width)
            shapes[p + "b1"] = (l.hidden,)
            shapes[p + "w2"] = (l.width, l.hidden)
            shapes[p + "b2"] = (l.width,)
        elif l.kind == "decoder":
            d, F = l.width, l.hidden
            if li == 1 and cfg.vocab > 0:
                shapes[p + "emb"] = (cfg.vocab, d)
            shapes[p + "ln1.g"] = (d,)
            shapes[p + "ln1.b"] = (d,)
            shapes[p + "wqkv"] = (3 * d, d)
            shapes[p + "bqkv"] = (3 * d,)
            shapes[p + "wo"] = (d, d)
            shapes[p + "bo"] = (d,)
            shapes[p + "ln2.g"] = (d,)
            shapes[p + "ln2.b"] = (d,)
            shapes[p + "w1"] = (F, d)
            shapes[p + "b1"] = (F,)
            shapes[p + "w2"] = (d, F)
            shapes[p + "b2"] = (d,)
        elif l.kind == "resnet_stage":
            c = l.out_ch
            if l.has_stem:
                shapes[p + "stem.w"] = (c, 3, 3, l.in_ch)
                shapes[p + "stem.bn.g"] = (c,)
                shapes[p + "stem.bn.b"] = (c,)
            for b in range(l.n_basic_blocks):
                q = p + f"b{b + 1}."
                cin = c if (l.has_stem or b > 0) else l.in_ch
                shapes[q + "conv1.w"] = (c, 3, 3, cin)
                shapes[q + "bn1.g"] = (c,)
                shapes[q + "bn1.b"] = (c,)
                shapes[q + "conv2.w"] = (c, 3, 3, c)
                shapes[q + "bn2.g"] = (c,)
                shapes[q + "bn2.b"] = (c,)
                if b == 0 and not l.has_stem and (l.stride != 1 or cin != c):
                    shapes[q + "proj.w"] = (c, 1, 1, cin)
                    shapes[q + "proj.bn.g"] = (c,)
                    shapes[q + "proj.bn.b"] = (c,)
        else:
            raise ValueError(l.kind)
    for hi, h in enumerate(cfg.heads, start=1):
        p = f"H{hi}."
        if h.kind == "ln_linear_ce":
            shapes[p + "ln.g"] = (h.in_dim,)
            shapes[p + "ln.b"] = (h.in_dim,)
        if h.kind == "bn_pool_linear_ce":
            shapes[p + "bn.g"] = (h.in_dim,)
            shapes[p + "bn.b"] = (h.in_dim,)
        shapes[p + "w"] = (h.n_classes, h.in_dim)
        if h.bias:
            shapes[p + "b"] = (h.n_classes,)
    return shapes
