"""ctypes binding of liblp.so: argument marshalling only.

Every function mirrors an entry point of include/lp.h under the same name.  PyTorch supplies
device memory and the HIP stream; nothing is computed here.  There is no CPU fallback: if the
library is missing, loading raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Dict, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "liblp.so")

LP_OK, LP_EINVAL, LP_ESHAPE, LP_EALIGN, LP_ENOMEM, LP_EDEVICE, LP_ESTATE, LP_EUNSUPPORTED, LP_ENOTFOUND = range(9)
LP_F32, LP_BF16, LP_I32 = 0, 1, 2
LAYER_KINDS = {"resmlp": 0, "decoder": 1, "resnet_stage": 2}
HEAD_KINDS = {"linear_ce": 0, "pool_linear_ce": 1, "ln_linear_ce": 2, "bn_pool_linear_ce": 3}
OPT_KINDS = {"sgd": 0, "sgdm": 1, "adam": 2}
COMBINE = {"sum": 0, "mean": 1}
ACTS = {"gelu": 0, "relu": 1}
DTYPES = {"f32": LP_F32, "bf16": LP_BF16}


class LpError(RuntimeError):
    def __init__(self, status: int, msg: str):
        super().__init__(f"lp status {status}: {msg}")
        self.status = status


class lp_layer_spec(C.Structure):
    _fields_ = [(n, C.c_int) for n in ("kind", "in_dim", "width", "hidden", "n_heads", "seq_len", "causal", "act",
                                        "in_ch", "out_ch", "stride", "n_basic_blocks", "has_stem", "in_hw")]


class lp_head_spec(C.Structure):
    _fields_ = [(n, C.c_int) for n in ("kind", "after_layer", "window", "in_dim", "n_classes", "bias")]


class lp_opt_spec(C.Structure):
    _fields_ = [("kind", C.c_int)] + [(n, C.c_float) for n in ("lr", "momentum", "beta1", "beta2", "eps",
                                                                "weight_decay")]


class lp_model_spec(C.Structure):
    _fields_ = [("n_layers", C.c_int), ("layers", C.POINTER(lp_layer_spec)), ("n_heads", C.c_int),
                ("heads", C.POINTER(lp_head_spec)), ("opt", lp_opt_spec), ("combine", C.c_int), ("dtype", C.c_int),
                ("max_batch", C.c_int), ("vocab", C.c_int), ("seed", C.c_uint64), ("n_streams", C.c_int),
                ("schedule", C.c_int), ("debug", C.c_int)]


class lp_sizes(C.Structure):
    _fields_ = [("param_bytes", C.c_size_t), ("state_bytes", C.c_size_t), ("work_bytes", C.c_size_t)]


class lp_buffers(C.Structure):
    _fields_ = [("params_dev", C.c_void_p), ("state_dev", C.c_void_p), ("work_dev", C.c_void_p)]


class lp_cost_inputs(C.Structure):
    _fields_ = [("forward_cost", C.c_double), ("aux_cost", C.c_double), ("backward_multiplier", C.c_double),
                ("parameters", C.c_double), ("layers", C.c_int)]


class lp_cost(C.Structure):
    _fields_ = [("cost_per_example", C.c_double), ("cost", C.c_double), ("time", C.c_double),
                ("parallelism", C.c_double)]


_lib = None


def lib() -> C.CDLL:
    """Loads liblp.so (built by `python -m paper_2012_03837_amd.build`); raises if absent."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(f"{LIB_PATH} not built: run `python -m paper_2012_03837_amd.build`")
        L = C.CDLL(LIB_PATH)
        vp, ip, sz = C.c_void_p, C.c_int, C.c_size_t
        L.lp_query_sizes.argtypes = [C.POINTER(lp_model_spec), C.POINTER(lp_sizes)]
        L.lp_init_blocks.argtypes = [C.POINTER(lp_model_spec), C.POINTER(lp_buffers), vp, C.POINTER(vp)]
        L.lp_local_step.argtypes = [vp, vp, vp, ip, vp]
        L.lp_eval_loss.argtypes = [vp, vp, vp, ip, vp]
        L.lp_tensor_info.argtypes = [vp, C.c_char_p, C.POINTER(C.c_int64), C.POINTER(ip), C.POINTER(ip), C.POINTER(sz)]
        L.lp_get_tensor.argtypes = [vp, C.c_char_p, vp, sz]
        L.lp_set_tensor.argtypes = [vp, C.c_char_p, vp, sz]
        L.lp_num_params.argtypes = [vp]
        L.lp_param_name.argtypes = [vp, ip]
        L.lp_param_name.restype = C.c_char_p
        L.lp_get_step.argtypes = [vp]
        L.lp_set_step.argtypes = [vp, ip]
        L.lp_last_error.argtypes = [vp]
        L.lp_last_error.restype = C.c_char_p
        L.lp_profile_enable.argtypes = [vp, ip]
        L.lp_profile_read.argtypes = [vp, ip, C.POINTER(C.c_double), C.POINTER(C.c_longlong), C.POINTER(C.c_double)]
        L.lp_profile_gemm_shapes.argtypes = [vp, C.c_char_p, sz]
        L.lp_profile_gemm_kernels.argtypes = [vp, C.c_char_p, sz]
        L.lp_cost_model.argtypes = [C.POINTER(lp_cost_inputs), ip, ip, C.c_double, C.c_double, C.POINTER(lp_cost)]
        L.lp_mlp_flops.argtypes = [ip, ip, ip, C.POINTER(C.c_double), C.POINTER(C.c_double)]
        L.lp_grad_cosine.argtypes = [vp, vp, vp]
        L.lp_step_graph.argtypes = [vp, C.c_int]
        L.lp_bn_running.argtypes = [vp, C.c_float, C.c_int]
        L.lp_overlap_steps.argtypes = [vp, C.c_int]
        L.lp_join.argtypes = [vp]
        L.lp_destroy.argtypes = [vp]
        L.lp_destroy.restype = None
        _lib = L
    return _lib


SCHEDULES = {"sync": 0, "pipelined": 1, "pipelined_grouped": 2}


def make_spec(cfg, max_batch: int | None = None, n_streams: int = 0, schedule: str = "sync", debug: bool = False):
    """lp_model_spec from a plain-data model description (fields as in lp_inputs.ModelCfg).
    Returns (spec, keepalive): the arrays the spec points into must outlive its use."""
    layers = (lp_layer_spec * len(cfg.layers))()
    for i, l in enumerate(cfg.layers):
        layers[i] = lp_layer_spec(LAYER_KINDS[l.kind], l.in_dim, l.width, l.hidden, l.n_heads, l.seq_len, l.causal,
                                  ACTS[l.act], l.in_ch, l.out_ch, l.stride, l.n_basic_blocks, l.has_stem, l.in_hw)
    heads = (lp_head_spec * len(cfg.heads))()
    for i, h in enumerate(cfg.heads):
        heads[i] = lp_head_spec(HEAD_KINDS[h.kind], h.after_layer, h.window, h.in_dim, h.n_classes, h.bias)
    o = cfg.opt
    opt = lp_opt_spec(OPT_KINDS[o.kind], o.lr, o.momentum, o.beta1, o.beta2, o.eps, o.weight_decay)
    spec = lp_model_spec(len(cfg.layers), layers, len(cfg.heads), heads, opt, COMBINE[cfg.combine],
                         DTYPES[cfg.dtype], cfg.batch if max_batch is None else max_batch, cfg.vocab, cfg.seed,
                         n_streams, SCHEDULES[schedule], 1 if debug else 0)
    return spec, (layers, heads)


def _check(status: int, ctx=None):
    if status != LP_OK:
        msg = lib().lp_last_error(ctx)
        raise LpError(status, msg.decode() if msg else "")


def lp_query_sizes(spec: lp_model_spec) -> lp_sizes:
    out = lp_sizes()
    _check(lib().lp_query_sizes(C.byref(spec), C.byref(out)))
    return out


def lp_init_blocks(spec: lp_model_spec, params_ptr: int, state_ptr: int, work_ptr: int, stream: int = 0) -> int:
    bufs = lp_buffers(params_ptr, state_ptr, work_ptr)
    ctx = C.c_void_p()
    _check(lib().lp_init_blocks(C.byref(spec), C.byref(bufs), C.c_void_p(stream), C.byref(ctx)))
    return ctx.value


def lp_local_step(ctx: int, x_ptr: int, y_ptr: int, batch: int, losses_ptr: int) -> None:
    _check(lib().lp_local_step(ctx, x_ptr, y_ptr, batch, losses_ptr), ctx)


def lp_eval_loss(ctx: int, x_ptr: int, y_ptr: int, batch: int, losses_ptr: int) -> None:
    _check(lib().lp_eval_loss(ctx, x_ptr, y_ptr, batch, losses_ptr), ctx)


def lp_tensor_info(ctx: int, name: str):
    shape = (C.c_int64 * 4)()
    ndim, dtype, nbytes = C.c_int(), C.c_int(), C.c_size_t()
    _check(lib().lp_tensor_info(ctx, name.encode(), shape, C.byref(ndim), C.byref(dtype), C.byref(nbytes)), ctx)
    return tuple(shape[i] for i in range(ndim.value)), dtype.value, nbytes.value


def _bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    return (bits.astype(np.uint32) << 16).view(np.float32)


def lp_get_tensor(ctx: int, name: str) -> np.ndarray:
    """Copies a named tensor to the host; bf16 tensors are widened to float32 (exactly)."""
    shape, dtype, nbytes = lp_tensor_info(ctx, name)
    raw = np.empty(nbytes, dtype=np.uint8)
    _check(lib().lp_get_tensor(ctx, name.encode(), raw.ctypes.data, nbytes), ctx)
    if dtype == LP_BF16:
        return _bf16_bits_to_f32(raw.view(np.uint16)).reshape(shape)
    return raw.view(np.float32 if dtype == LP_F32 else np.int32).reshape(shape)


def lp_set_tensor(ctx: int, name: str, value: np.ndarray) -> None:
    shape, dtype, nbytes = lp_tensor_info(ctx, name)
    if dtype != LP_F32:
        raise LpError(LP_EUNSUPPORTED, "only fp32 tensors can be set")
    v = np.ascontiguousarray(value, dtype=np.float32)
    if tuple(v.shape) != tuple(shape):
        raise LpError(LP_ESHAPE, f"{name}: shape {v.shape} != {shape}")
    _check(lib().lp_set_tensor(ctx, name.encode(), v.ctypes.data, nbytes), ctx)


def lp_param_names(ctx: int):
    L = lib()
    return [L.lp_param_name(ctx, i).decode() for i in range(L.lp_num_params(ctx))]


def lp_get_step(ctx: int) -> int:
    return lib().lp_get_step(ctx)


def lp_set_step(ctx: int, t: int) -> None:
    _check(lib().lp_set_step(ctx, t), ctx)


KERNEL_CLASSES = ("gemm", "attn_fwd", "attn_bwd", "layernorm", "softmax_ce", "optimizer", "embed", "colsum", "conv",
                  "batchnorm", "other", "gemm_kernel")


def lp_profile_enable(ctx: int, on: bool) -> None:
    _check(lib().lp_profile_enable(ctx, int(on)), ctx)


def lp_profile_read(ctx: int, kernel_class: int):
    """(total event ms, ops launched, FLOPs launched) of one kernel class since profiling was enabled."""
    ms, n, fl = C.c_double(), C.c_longlong(), C.c_double()
    _check(lib().lp_profile_read(ctx, kernel_class, C.byref(ms), C.byref(n), C.byref(fl)), ctx)
    return ms.value, n.value, fl.value


def lp_profile_gemm_shapes(ctx: int):
    """GEMM ops by shape since profiling was enabled: dicts with M, N, K, a_kc, b_kc, c_f32, count, ms."""
    buf = C.create_string_buffer(1 << 16)
    _check(lib().lp_profile_gemm_shapes(ctx, buf, len(buf)), ctx)
    rows = []
    for line in buf.value.decode().splitlines():
        M, N, K, a, b, f, n, ms = line.split()
        rows.append({"M": int(M), "N": int(N), "K": int(K), "a_kc": int(a), "b_kc": int(b), "c_f32": int(f),
                     "count": int(n), "ms": float(ms)})
    return rows


def lp_profile_gemm_kernels(ctx: int):
    """The main kernel of every bf16 GEMM op since profiling was enabled, by kernel instance: dicts with name,
    launches, ms, flops."""
    buf = C.create_string_buffer(1 << 16)
    _check(lib().lp_profile_gemm_kernels(ctx, buf, len(buf)), ctx)
    rows = []
    for line in buf.value.decode().splitlines():
        name, n, ms, fl = line.split("\t")
        rows.append({"name": name, "launches": int(n), "ms": float(ms), "flops": float(fl)})
    return rows


def lp_step_graph(ctx: int, on: bool) -> None:
    _check(lib().lp_step_graph(ctx, 1 if on else 0), ctx)


def lp_overlap_steps(ctx: int, on: bool) -> None:
    _check(lib().lp_overlap_steps(ctx, 1 if on else 0), ctx)


def lp_join(ctx: int) -> None:
    _check(lib().lp_join(ctx), ctx)


def lp_bn_running(ctx: int, momentum: float = 0.1, eval_with_running: bool = False) -> None:
    _check(lib().lp_bn_running(ctx, float(momentum), 1 if eval_with_running else 0), ctx)


def lp_grad_cosine(ctx_a: int, ctx_b: int, out_dev_ptr: int) -> None:
    _check(lib().lp_grad_cosine(ctx_a, ctx_b, out_dev_ptr), ctx_a)


METHODS = {"backprop": 0, "greedy": 1, "overlap": 2, "chunk": 3, "last_k": 4}


def lp_cost_model(forward_cost, aux_cost, backward_multiplier, layers, parameters, method, steps, batch_size, K=1):
    """(cost_per_example, cost, time, parallelism) of the appendix-A cost model; method is a METHODS key."""
    inp = lp_cost_inputs(float(forward_cost), float(aux_cost), float(backward_multiplier), float(parameters), int(layers))
    out = lp_cost()
    rc = lib().lp_cost_model(C.byref(inp), METHODS[method] if isinstance(method, str) else int(method), int(K),
                             float(steps), float(batch_size), C.byref(out))
    if rc != 0:
        raise LpError(rc, "lp_cost_model: invalid argument")
    return out.cost_per_example, out.cost, out.time, out.parallelism


def lp_mlp_flops(input_size, hidden, layers):
    f, a = C.c_double(), C.c_double()
    rc = lib().lp_mlp_flops(int(input_size), int(hidden), int(layers), C.byref(f), C.byref(a))
    if rc != 0:
        raise LpError(rc, "lp_mlp_flops: invalid argument")
    return f.value, a.value


def lp_destroy(ctx: int) -> None:
    lib().lp_destroy(ctx)


def default_side_streams(cfg) -> int:
    """Side streams for the heads' chains that the benchmark times each workload with (the fastest measured on
    one MI355X): two for the decoders, three for the residual MLP, one per stage (at most four) for the ResNets,
    whose chains are short enough to run side by side."""
    kind0 = cfg.layers[0].kind
    if kind0 == "resnet_stage":
        return min(4, len(cfg.heads))
    return 2 if kind0 == "decoder" else 3


class LocalTrainer:
    """Owns the three device buffers (torch tensors) and a context over them."""

    def __init__(self, cfg, device="cuda:0", max_batch: int | None = None, stream=None, n_streams: int = 0,
                 schedule: str = "sync", debug: bool = False):
        import torch
        if not torch.cuda.is_available():
            raise RuntimeError("no GPU: the local-update step runs only on the HIP device")
        self.torch = torch
        self.cfg = cfg
        self.device = torch.device(device)
        self.spec, self._keep = make_spec(cfg, max_batch, n_streams, schedule, debug)
        sz = lp_query_sizes(self.spec)
        self.sizes = sz
        with torch.cuda.device(self.device):
            self.params = torch.empty(sz.param_bytes, dtype=torch.uint8, device=self.device)
            self.state = torch.empty(sz.state_bytes, dtype=torch.uint8, device=self.device)
            self.work = torch.empty(sz.work_bytes, dtype=torch.uint8, device=self.device)
            self.losses = torch.zeros(len(cfg.heads), dtype=torch.float32, device=self.device)
            self.stream = stream if stream is not None else torch.cuda.current_stream(self.device)
            torch.cuda.synchronize(self.device)
            self.ctx = lp_init_blocks(self.spec, self.params.data_ptr(), self.state.data_ptr(), self.work.data_ptr(),
                                      self.stream.cuda_stream)

    # ---- data staging (host numpy -> device tensors in the layout lp.h asks for)
    def stage(self, x: np.ndarray, y: np.ndarray):
        torch = self.torch
        if np.issubdtype(x.dtype, np.integer):
            xd = torch.from_numpy(np.ascontiguousarray(x, dtype=np.int32)).to(self.device)
        else:
            xd = torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).to(self.device)
            if self.cfg.dtype == "bf16":
                xd = xd.to(torch.bfloat16)
        yd = torch.from_numpy(np.ascontiguousarray(y, dtype=np.int32)).to(self.device)
        return xd.contiguous(), yd.contiguous()

    def step(self, xd, yd, batch: int | None = None):
        b = xd.shape[0] if batch is None else batch
        lp_local_step(self.ctx, xd.data_ptr(), yd.data_ptr(), b, self.losses.data_ptr())
        return self.losses

    def step_graph(self, on: bool = True) -> None:
        lp_step_graph(self.ctx, on)

    def overlap_steps(self, on: bool = True) -> None:
        lp_overlap_steps(self.ctx, on)

    def join(self) -> None:
        lp_join(self.ctx)

    def bn_running(self, momentum: float = 0.1, eval_with_running: bool = False) -> None:
        lp_bn_running(self.ctx, momentum, eval_with_running)

    def eval(self, xd, yd, batch: int | None = None):
        b = xd.shape[0] if batch is None else batch
        lp_eval_loss(self.ctx, xd.data_ptr(), yd.data_ptr(), b, self.losses.data_ptr())
        return self.losses

    def get(self, name: str) -> np.ndarray:
        return lp_get_tensor(self.ctx, name)

    def set(self, name: str, value: np.ndarray) -> None:
        lp_set_tensor(self.ctx, name, value)

    def names(self):
        return lp_param_names(self.ctx)

    def set_params(self, params: Dict[str, np.ndarray]) -> None:
        for k, v in params.items():
            self.set(k, v)

    def get_params(self) -> Dict[str, np.ndarray]:
        return {k: self.get(k) for k in self.names()}

    def close(self):
        if getattr(self, "ctx", None):
            self.torch.cuda.synchronize(self.device)
            lp_destroy(self.ctx)
            self.ctx = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
