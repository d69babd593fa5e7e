"""ctypes binding of the kernel-level ABI (include/lp_kernels.h): argument marshalling only.
Arguments are torch CUDA tensors (or None); every function enqueues on torch's current stream."""
from __future__ import annotations

import ctypes as C

from .binding import lib


class KernelError(RuntimeError):
    pass


def _p(t):
    return C.c_void_p(0 if t is None else t.data_ptr())


def _stream():
    import torch
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _ck(rc, what):
    if rc != 0:
        raise KernelError(f"{what} failed with hipError {rc}")


_i, _i64, _f, _sz = C.c_int, C.c_int64, C.c_float, C.c_size_t


def lpk_gemm(dtype, A, lda, a_kc, B, ldb, b_kc, Cout, ldc, c_f32, M, N, K, bias=None, act=0, pre=None, dact_src=None,
             dact=0, ldd=0, res=None, ldr=0, accumulate=0, plain=0, splitk_ws=None, variant=None):
    variant = (1 if plain else 0) if variant is None else variant
    _ck(lib().lpk_gemm(_i(dtype), _p(A), _i64(lda), _i(a_kc), _p(B), _i64(ldb), _i(b_kc), _p(Cout), _i64(ldc),
                       _i(c_f32), _i(M), _i(N), _i(K), _p(bias), _i(act), _p(pre), _p(dact_src), _i(dact), _i64(ldd),
                       _p(res), _i64(ldr), _i(accumulate), _i(variant), _p(splitk_ws),
                       _sz(0 if splitk_ws is None else splitk_ws.numel()), _stream()), "lpk_gemm")


def lpk_gemm_grouped(As, Bs, Cs, Ms, Ns, K, a_kc, b_kc, accumulate, splitk_ws, biases=None, act=0, ress=None):
    """As, Bs, Cs: lists of torch CUDA tensors (bf16 operands as stored; outputs [M_i, N_i], all fp32 or all bf16);
    biases / ress: optional lists of fp32 [N_i] / bf16 [M_i, N_i] tensors."""
    import torch
    n = len(As)
    vp = (C.c_void_p * n)
    i64 = (C.c_int64 * n)
    ia = (C.c_int * n)
    c_f32 = 1 if Cs[0].dtype == torch.float32 else 0
    bias = vp(*[b.data_ptr() for b in biases]) if biases is not None else None
    res = vp(*[r.data_ptr() for r in ress]) if ress is not None else None
    _ck(lib().lpk_gemm_grouped(_i(n), vp(*[a.data_ptr() for a in As]), i64(*[a.shape[1] for a in As]),
                               vp(*[b.data_ptr() for b in Bs]), i64(*[b.shape[1] for b in Bs]),
                               vp(*[c.data_ptr() for c in Cs]), i64(*[c.shape[1] for c in Cs]), _i(c_f32), ia(*Ms), ia(*Ns),
                               _i(K), _i(a_kc), _i(b_kc), bias, _i(act), res, _i(accumulate), _p(splitk_ws),
                               _sz(splitk_ws.numel()), _stream()),
        "lpk_gemm_grouped")


def lpk_attention_fwd(dtype, qkv, o, lse, B, S, H, dh, causal=1, plain=0):
    _ck(lib().lpk_attention_fwd(_i(dtype), _p(qkv), _p(o), _p(lse), _i(B), _i(S), _i(H), _i(dh), _i(causal), _i(plain),
                                _stream()), "lpk_attention_fwd")


def lpk_attention_bwd(dtype, qkv, o, lse, dout, dqkv, delta, B, S, H, dh, causal=1, plain=0):
    _ck(lib().lpk_attention_bwd(_i(dtype), _p(qkv), _p(o), _p(lse), _p(dout), _p(dqkv), _p(delta), _i(B), _i(S), _i(H),
                                _i(dh), _i(causal), _i(plain), _stream()), "lpk_attention_bwd")


def lpk_layernorm_fwd(dtype, x, g, b, y, mean, rstd, rows, d):
    _ck(lib().lpk_layernorm_fwd(_i(dtype), _p(x), _p(g), _p(b), _p(y), _p(mean), _p(rstd), _i(rows), _i(d), _stream()),
        "lpk_layernorm_fwd")


def lpk_layernorm_bwd_static(dtype, dy, x, mean, rstd, g, add, dx, dg, db, rows, d, accumulate):
    rc = lib().lpk_layernorm_bwd_static(_i(dtype), _p(dy), _p(x), _p(mean), _p(rstd), _p(g), _p(add), _p(dx), _p(dg),
                                        _p(db), _i(rows), _i(d), _i(accumulate), _stream())
    if rc == 1:
        raise KernelError(f"lpk_layernorm_bwd_static: rows={rows}, d={d} exceed the built-in workspace "
                          f"(((rows + 7) // 8) * d * 2 must be <= {1 << 21})")
    _ck(rc, "lpk_layernorm_bwd_static")


def lpk_layernorm_bwd(dtype, dy, x, mean, rstd, g, add, dx, dg, db, rows, d, accumulate, scratch):
    _ck(lib().lpk_layernorm_bwd(_i(dtype), _p(dy), _p(x), _p(mean), _p(rstd), _p(g), _p(add), _p(dx), _p(dg), _p(db),
                                _i(rows), _i(d), _i(accumulate), _p(scratch), _sz(scratch.numel()), _stream()),
        "lpk_layernorm_bwd")


def lpk_softmax_ce(dtype, z, ld, y, loss_rows, rows, n, write_grad, inv_rows):
    _ck(lib().lpk_softmax_ce(_i(dtype), _p(z), _i64(ld), _p(y), _p(loss_rows), _i(rows), _i(n), _i(write_grad),
                             _f(inv_rows), _stream()), "lpk_softmax_ce")


def lpk_optimizer(kind, lr, momentum, beta1, beta2, eps, weight_decay, t, grad_scale, p, g, m, v, p_bf16, n):
    _ck(lib().lpk_optimizer(_i(kind), _f(lr), _f(momentum), _f(beta1), _f(beta2), _f(eps), _f(weight_decay), _i(t),
                            _f(grad_scale), _p(p), _p(g), _p(m), _p(v), _p(p_bf16), _sz(n), _stream()),
        "lpk_optimizer")


def lpk_copy(src, dst, nbytes):
    _ck(lib().lpk_copy(_p(src), _p(dst), _sz(nbytes), _stream()), "lpk_copy")


def lpk_transpose_bf16(src, dst, R, C):
    _ck(lib().lpk_transpose_bf16(_p(src), _p(dst), _i(R), _i(C), _stream()), "lpk_transpose_bf16")


def lpk_embed_bwd(dtype, ids, dh, demb, T, V, d, accumulate=0, scratch=None):
    _ck(lib().lpk_embed_bwd(_i(dtype), _p(ids), _p(dh), _p(demb), _i(T), _i(V), _i(d), _i(accumulate), _p(scratch),
                            _sz(0 if scratch is None else scratch.numel()), _stream()), "lpk_embed_bwd")


def lpk_conv_fwd(dtype, x, w, out, N, H, W, Cin, O, R, stride, pad):
    _ck(lib().lpk_conv_fwd(_i(dtype), _p(x), _p(w), _p(out), _i(N), _i(H), _i(W), _i(Cin), _i(O), _i(R), _i(stride),
                           _i(pad), _stream()), "lpk_conv_fwd")


def lpk_conv_bwd_data(dtype, dout, w, dx, N, H, W, Cin, O, R, stride, pad):
    _ck(lib().lpk_conv_bwd_data(_i(dtype), _p(dout), _p(w), _p(dx), _i(N), _i(H), _i(W), _i(Cin), _i(O), _i(R),
                                _i(stride), _i(pad), _stream()), "lpk_conv_bwd_data")


def lpk_conv_bwd_weight(dtype, dout, x, dw, N, H, W, Cin, O, R, stride, pad, accumulate=0):
    _ck(lib().lpk_conv_bwd_weight(_i(dtype), _p(dout), _p(x), _p(dw), _i(N), _i(H), _i(W), _i(Cin), _i(O), _i(R),
                                  _i(stride), _i(pad), _i(accumulate), _stream()), "lpk_conv_bwd_weight")


def lpk_conv_bwd_weight_ws(dtype, dout, x, dw, N, H, W, Cin, O, R, stride, pad, splitk_ws, accumulate=0):
    _ck(lib().lpk_conv_bwd_weight_ws(_i(dtype), _p(dout), _p(x), _p(dw), _i(N), _i(H), _i(W), _i(Cin), _i(O), _i(R),
                                     _i(stride), _i(pad), _i(accumulate), _p(splitk_ws), _sz(splitk_ws.numel()),
                                     _stream()), "lpk_conv_bwd_weight_ws")


def lpk_conv_bn_fwd(dtype, x, w, z, g, b, res, y, mean, rstd, N, H, W, Cin, O, R, stride, pad, relu, scratch):
    _ck(lib().lpk_conv_bn_fwd(_i(dtype), _p(x), _p(w), _p(z), _p(g), _p(b), _p(res), _p(y), _p(mean), _p(rstd), _i(N),
                              _i(H), _i(W), _i(Cin), _i(O), _i(R), _i(stride), _i(pad), _i(relu), _p(scratch),
                              _sz(scratch.numel()), _stream()), "lpk_conv_bn_fwd")


def lpk_batchnorm_fwd(dtype, z, g, b, res, y, mean, rstd, rows, Cc, relu, scratch):
    _ck(lib().lpk_batchnorm_fwd(_i(dtype), _p(z), _p(g), _p(b), _p(res), _p(y), _p(mean), _p(rstd), _i(rows), _i(Cc),
                                _i(relu), _p(scratch), _sz(scratch.numel()), _stream()), "lpk_batchnorm_fwd")


def lpk_batchnorm_bwd(dtype, dy, y, z, mean, rstd, g, dz, dres, dg, db, rows, Cc, relu, accumulate, scratch):
    _ck(lib().lpk_batchnorm_bwd(_i(dtype), _p(dy), _p(y), _p(z), _p(mean), _p(rstd), _p(g), _p(dz), _p(dres), _p(dg),
                                _p(db), _i(rows), _i(Cc), _i(relu), _i(accumulate), _p(scratch), _sz(scratch.numel()),
                                _stream()), "lpk_batchnorm_bwd")
