"""Thin ctypes binding of liboptimus.so: same names as the C ABI, argument marshalling only.

Tensors are torch tensors used purely as device-memory handles (``data_ptr()``); the stream is torch's
current HIP stream unless one is passed.  Nothing here computes.
"""
from __future__ import annotations

import ctypes as C
import os

import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "liboptimus.so")

OK, EINVAL, ESHAPE, ECOORD, EDTYPE, EWORKSPACE, EHIP = range(7)
FP32, BF16 = 0, 1
FORM_AB, FORM_ABT, FORM_ATB = 0, 1, 2
ALL = -1
STATIC_SCRATCH_BYTES = 4 << 20   # OPTIMUS_STATIC_SCRATCH_BYTES: the most scratch optimus_attention_fused_bwd_static can serve
FORMS = {"ab": FORM_AB, "abt": FORM_ABT, "atb": FORM_ATB}


class OptimusError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__(f"{where}: error {code}: {error_string(code)}")


class Epilogue(C.Structure):
    _fields_ = [("bias", C.c_void_p), ("pre_act", C.c_void_p), ("act", C.c_int),
                ("gelu_grad_of", C.c_void_p), ("residual", C.c_void_p), ("out_fp32", C.c_int)]


class LayerCfg(C.Structure):
    _fields_ = [("b", C.c_int), ("s", C.c_int), ("h", C.c_int), ("n", C.c_int), ("q", C.c_int),
                ("eps", C.c_float), ("causal", C.c_int), ("dtype", C.c_int), ("fused_attention", C.c_int)]


LAYER_TENSOR_FIELDS = [
    "x", "ln1_g", "ln1_b", "w_qkv", "b_qkv", "w_o", "b_o", "ln2_g", "ln2_b", "w1", "b1", "w2", "b2",
    "ln1_out", "xhat1", "rstd1", "stats1", "qkv", "probs", "attn", "h_mid",
    "ln2_out", "xhat2", "rstd2", "stats2", "pre_gelu", "gelu", "out",
    "d_out", "d_pre_gelu", "d_ln2_out", "d_h_mid", "d_attn", "d_qkv", "d_ln1_out", "d_x",
    "bstats1", "bstats2", "d_w_qkv", "d_w_o", "d_w1", "d_w2", "d_b_qkv", "d_b_o", "d_b1", "d_b2",
    "d_ln1_g", "d_ln1_b", "d_ln2_g", "d_ln2_b",
    "lse",
]


class LayerTensors(C.Structure):
    _fields_ = [(name, C.c_void_p) for name in LAYER_TENSOR_FIELDS]


LAYER_PARAM_FIELDS = ["ln1_g", "ln1_b", "w_qkv", "b_qkv", "w_o", "b_o", "ln2_g", "ln2_b", "w1", "b1", "w2", "b2"]
LAYER_GRAD_FIELDS = ["d_w_qkv", "d_w_o", "d_w1", "d_w2", "d_b_qkv", "d_b_o", "d_b1", "d_b2",
                     "d_ln1_g", "d_ln1_b", "d_ln2_g", "d_ln2_b"]


class LayerParams(C.Structure):
    _fields_ = [(name, C.c_void_p) for name in LAYER_PARAM_FIELDS]


class LayerGrads(C.Structure):
    _fields_ = [(name, C.c_void_p) for name in LAYER_GRAD_FIELDS]


class StackSizes(C.Structure):
    _fields_ = [(name, C.c_size_t) for name in ("workspace", "forward", "backward", "param_grad", "conjunction", "checkpoint")]


class StackBuffers(C.Structure):
    _fields_ = [(name, C.c_void_p) for name in ("workspace", "forward", "backward", "conjunction", "checkpoint")]


LAYER_DONE_FN = C.CFUNCTYPE(None, C.c_int, C.c_void_p)


_lib = None

_I64, _INT, _P, _SZ, _F = C.c_int64, C.c_int, C.c_void_p, C.c_size_t, C.c_float
_SUMMA_ARGS = [_P, _P, _P, _I64, _I64, _I64, _INT, _INT, _INT, _INT, _P, _SZ, _P]
SIGNATURES = {
    "optimus_error_string": (C.c_char_p, [_INT]),
    "optimus_abi_version": (_INT, []),
    "optimus_pack_blocks": (_INT, [_P, _P, _I64, _I64, _INT, _INT, _P]),
    "optimus_unpack_blocks": (_INT, [_P, _P, _I64, _I64, _INT, _INT, _P]),
    "optimus_summa_ab": (_INT, _SUMMA_ARGS),
    "optimus_summa_abt": (_INT, _SUMMA_ARGS),
    "optimus_summa_atb": (_INT, _SUMMA_ARGS),
    "optimus_summa_workspace_bytes": (_SZ, [_INT, _I64, _I64, _I64, _INT, _INT, _INT, _INT]),
    "optimus_summa_ex": (_INT, [_INT, _P, _P, _P, _I64, _I64, _I64, _INT, _INT, _INT, _INT, C.POINTER(Epilogue), _P, _SZ, _P]),
    "optimus_summa_step": (_INT, [_INT, _P, _P, _P, _I64, _I64, _I64, _INT, _INT, _INT, _INT, _INT, _P]),
    "optimus_summa_reduce": (_INT, [_P, _INT, _P, _I64, _I64, _INT, _INT, _INT, _INT, _P]),
    "optimus_bias_grad": (_INT, [_P, _P, _I64, _I64, _INT, _INT, _INT, _INT, _P]),
    "optimus_layernorm2d_stats": (_INT, [_P, _P, _I64, _I64, _INT, _INT, _INT, _INT, _P]),
    "optimus_layernorm2d": (_INT, [_P, _P, _P, _P, _P, _P, _P, _I64, _I64, _INT, _INT, _INT, _F, _INT, _P]),
    "optimus_layernorm2d_bwd_stats": (_INT, [_P, _P, _P, _P, _I64, _I64, _INT, _INT, _INT, _INT, _P]),
    "optimus_layernorm2d_bwd": (_INT, [_P, _P, _P, _P, _P, _P, _P, _P, _P, _I64, _I64, _INT, _INT, _INT, _INT, _P]),
    "optimus_attention_fwd": (_INT, [_P, _P, _P, _INT, _INT, _INT, _INT, _INT, _INT, _INT, _INT, _INT, _P, _SZ, _P]),
    "optimus_attention_bwd": (_INT, [_P, _P, _P, _P, _INT, _INT, _INT, _INT, _INT, _INT, _INT, _INT, _INT, _P, _SZ, _P]),
    "optimus_attention_workspace_bytes": (_SZ, [_INT, _INT, _INT, _INT, _INT]),
    "optimus_softmax_rows": (_INT, [_P, _P, _I64, _INT, _INT, _P]),
    "optimus_softmax_rows_bwd": (_INT, [_P, _P, _P, _I64, _INT, _INT, _P]),
    "optimus_attention_fused_fwd": (_INT, [_P, _P, _P, _INT, _INT, _INT, _INT, _INT, _INT, _INT, _INT, _INT, _P]),
    "optimus_attention_fused_bwd": (_INT, [_P, _P, _P, _P, _P, _INT, _INT, _INT, _INT, _INT, _INT, _INT, _INT, _INT, _P, _SZ, _P]),
    "optimus_attention_fused_workspace_bytes": (_SZ, [_INT, _INT, _INT, _INT, _INT]),
    "optimus_attention_fused_bwd_static": (_INT, [_P, _P, _P, _P, _P, _INT, _INT, _INT, _INT, _INT, _INT, _INT, _INT, _INT, _P]),
    "optimus_embedding_fwd": (_INT, [_P, _P, _P, _I64, _I64, _I64, _INT, _INT, _INT, _INT, _P]),
    "optimus_embedding_bwd": (_INT, [_P, _P, _P, _I64, _I64, _I64, _INT, _INT, _INT, _INT, _P]),
    "optimus_cross_entropy2d_stats": (_INT, [_P, _P, _I64, _I64, _INT, _INT, _INT, _INT, _P]),
    "optimus_cross_entropy2d": (_INT, [_P, _P, _P, _P, _P, _I64, _I64, _INT, _INT, _INT, _INT, _P]),
    "optimus_cross_entropy2d_bwd": (_INT, [_P, _P, _P, _P, _F, _I64, _I64, _INT, _INT, _INT, _INT, _P]),
    "optimus_stack_sizes_of": (_INT, [C.POINTER(LayerCfg), _INT, C.POINTER(StackSizes)]),
    "optimus_layer_grads_in": (_INT, [C.POINTER(LayerCfg), _P, C.POINTER(LayerGrads)]),
    "optimus_stack_fwd": (_INT, [C.POINTER(LayerCfg), _INT, C.POINTER(LayerParams), _P, C.POINTER(StackBuffers), _P, _P]),
    "optimus_stack_bwd": (_INT, [C.POINTER(LayerCfg), _INT, C.POINTER(LayerParams), C.POINTER(LayerGrads), _P,
                                 C.POINTER(StackBuffers), _P, LAYER_DONE_FN, _P, _P]),
    "optimus_layer_workspace_bytes": (_SZ, [C.POINTER(LayerCfg)]),
    "optimus_layer_workspace_bytes_grid": (_SZ, [C.POINTER(LayerCfg)]),
    "optimus_layer_fwd": (_INT, [C.POINTER(LayerCfg), C.POINTER(LayerTensors), _INT, _INT, _P, _SZ, _P]),
    "optimus_layer_bwd": (_INT, [C.POINTER(LayerCfg), C.POINTER(LayerTensors), _INT, _INT, _P, _SZ, _P]),
    "optimus_gemm_flops": (_I64, [_I64, _I64, _I64, _INT]),
    "optimus_layer_flops": (_I64, [C.POINTER(LayerCfg), _INT]),
    "optimus_debug_set_gemm_variant": (None, [_INT]),
    "optimus_debug_set_corun_variants": (None, [_INT, _INT]),
    "optimus_debug_last_gemm_plan": (_INT, []),
    "optimus_debug_plan_summa": (_INT, [_INT, _I64, _I64, _I64, _INT, _INT, _INT, _INT, _INT, C.POINTER(C.c_int)]),
    "optimus_debug_mfma_rate": (_INT, [_P, _INT, _INT, _INT, _P]),
}


def lib():
    """Load liboptimus.so (once).  Raises if it has not been built: there is no fallback path."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} not found: build it with `python -c 'import __graft_entry__ as g; g.build()'`")
        L = C.CDLL(LIB_PATH)
        for name, (res, args) in SIGNATURES.items():
            fn = getattr(L, name)
            fn.restype = res
            fn.argtypes = args
        _lib = L
    return _lib


def _ptr(t):
    if t is None:
        return None
    if isinstance(t, int):
        return t
    return t.data_ptr()


def _stream(stream):
    if stream is None:
        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream


def _ws(ws):
    if ws is None:
        return None, 0
    return ws.data_ptr(), ws.numel() * ws.element_size()


def _check(rc, where):
    if rc != OK:
        raise OptimusError(rc, where)


def error_string(code: int) -> str:
    return lib().optimus_error_string(code).decode()


def abi_version() -> int:
    return lib().optimus_abi_version()


def pack_blocks(src, dst, R, C_, q, elem_bytes, stream=None):
    _check(lib().optimus_pack_blocks(_ptr(src), _ptr(dst), R, C_, q, elem_bytes, _stream(stream)), "optimus_pack_blocks")


def unpack_blocks(src, dst, R, C_, q, elem_bytes, stream=None):
    _check(lib().optimus_unpack_blocks(_ptr(src), _ptr(dst), R, C_, q, elem_bytes, _stream(stream)), "optimus_unpack_blocks")


def _summa(name, A, B, Cm, M, K, N, q, i, j, dtype, ws, stream):
    p, n = _ws(ws)
    _check(getattr(lib(), name)(_ptr(A), _ptr(B), _ptr(Cm), M, K, N, q, i, j, dtype, p, n, _stream(stream)), name)


def summa_ab(A, B, Cm, M, K, N, q, i, j, dtype, ws=None, stream=None):
    _summa("optimus_summa_ab", A, B, Cm, M, K, N, q, i, j, dtype, ws, stream)


def summa_abt(A, B, Cm, M, K, N, q, i, j, dtype, ws=None, stream=None):
    _summa("optimus_summa_abt", A, B, Cm, M, K, N, q, i, j, dtype, ws, stream)


def summa_atb(A, B, Cm, M, K, N, q, i, j, dtype, ws=None, stream=None):
    _summa("optimus_summa_atb", A, B, Cm, M, K, N, q, i, j, dtype, ws, stream)


def summa(form, *args, **kw):
    return {"ab": summa_ab, "abt": summa_abt, "atb": summa_atb}[form](*args, **kw)


def summa_workspace_bytes(form, M, K, N, q, i, j, dtype) -> int:
    return lib().optimus_summa_workspace_bytes(FORMS[form] if isinstance(form, str) else form, M, K, N, q, i, j, dtype)


def summa_ex(form, A, B, Cm, M, K, N, q, i, j, dtype, bias=None, pre_act=None, act=0, gelu_grad_of=None,
             residual=None, out_fp32=False, ws=None, stream=None):
    e = Epilogue(_ptr(bias), _ptr(pre_act), act, _ptr(gelu_grad_of), _ptr(residual), 1 if out_fp32 else 0)
    p, n = _ws(ws)
    f = FORMS[form] if isinstance(form, str) else form
    _check(lib().optimus_summa_ex(f, _ptr(A), _ptr(B), _ptr(Cm), M, K, N, q, i, j, dtype, C.byref(e), p, n, _stream(stream)),
           "optimus_summa_ex")


def bias_grad(dY, dbias_part, M, N, q, i, j, dtype, stream=None):
    _check(lib().optimus_bias_grad(_ptr(dY), _ptr(dbias_part), M, N, q, i, j, dtype, _stream(stream)), "optimus_bias_grad")


def layernorm2d_stats(X, stats, M, H, q, i, l, dtype, stream=None):
    _check(lib().optimus_layernorm2d_stats(_ptr(X), _ptr(stats), M, H, q, i, l, dtype, _stream(stream)), "optimus_layernorm2d_stats")


def layernorm2d(X, gamma, beta, Y, xhat, rstd, stats, M, H, q, i, j, eps, dtype, stream=None):
    _check(lib().optimus_layernorm2d(_ptr(X), _ptr(gamma), _ptr(beta), _ptr(Y), _ptr(xhat), _ptr(rstd), _ptr(stats), M, H, q, i, j,
                                     eps, dtype, _stream(stream)), "optimus_layernorm2d")


def layernorm2d_bwd_stats(dY, xhat, gamma, stats, M, H, q, i, l, dtype, stream=None):
    _check(lib().optimus_layernorm2d_bwd_stats(_ptr(dY), _ptr(xhat), _ptr(gamma), _ptr(stats), M, H, q, i, l, dtype, _stream(stream)),
           "optimus_layernorm2d_bwd_stats")


def layernorm2d_bwd(dY, xhat, rstd, gamma, dres, dX, dgamma_part, dbeta_part, stats, M, H, q, i, j, dtype, stream=None):
    _check(lib().optimus_layernorm2d_bwd(_ptr(dY), _ptr(xhat), _ptr(rstd), _ptr(gamma), _ptr(dres), _ptr(dX), _ptr(dgamma_part),
                                         _ptr(dbeta_part), _ptr(stats), M, H, q, i, j, dtype, _stream(stream)),
           "optimus_layernorm2d_bwd")


def summa_step(form, A, B, c_temp, M, K, N, q, i, j, l, dtype, stream=None):
    """form: 'ab' | 'abt' | 'atb' or the OPTIMUS_FORM_* code."""
    f = {"ab": 0, "abt": 1, "atb": 2}.get(form, form)
    _check(lib().optimus_summa_step(f, _ptr(A), _ptr(B), _ptr(c_temp), M, K, N, q, i, j, l, dtype, _stream(stream)),
           "optimus_summa_step")


def summa_reduce(c_temps, count, Cmat, M, N, q, root_i, root_j, dtype, stream=None):
    _check(lib().optimus_summa_reduce(_ptr(c_temps), count, _ptr(Cmat), M, N, q, root_i, root_j, dtype, _stream(stream)),
           "optimus_summa_reduce")


def attention_workspace_bytes(b, s, h, n, q) -> int:
    return lib().optimus_attention_workspace_bytes(b, s, h, n, q)


def attention_fwd(qkv, probs, attn, b, s, h, n, q, i, j, causal, dtype, ws, stream=None):
    p, nb = _ws(ws)
    _check(lib().optimus_attention_fwd(_ptr(qkv), _ptr(probs), _ptr(attn), b, s, h, n, q, i, j, int(causal), dtype, p, nb,
                                       _stream(stream)), "optimus_attention_fwd")


def attention_bwd(qkv, probs, d_attn, d_qkv, b, s, h, n, q, i, j, causal, dtype, ws, stream=None):
    p, nb = _ws(ws)
    _check(lib().optimus_attention_bwd(_ptr(qkv), _ptr(probs), _ptr(d_attn), _ptr(d_qkv), b, s, h, n, q, i, j, int(causal), dtype,
                                       p, nb, _stream(stream)), "optimus_attention_bwd")


def attention_fused_bwd_static(qkv, attn, lse, d_attn, d_qkv, b, s, h, n, q, i, j, causal, dtype, stream=None):
    _check(lib().optimus_attention_fused_bwd_static(_ptr(qkv), _ptr(attn), _ptr(lse), _ptr(d_attn), _ptr(d_qkv), b, s, h, n, q, i, j,
                                                    int(causal), dtype, _stream(stream)), "optimus_attention_fused_bwd_static")


def softmax_rows(scores, probs, nmat, s, causal, stream=None):
    _check(lib().optimus_softmax_rows(_ptr(scores), _ptr(probs), nmat, s, int(causal), _stream(stream)), "optimus_softmax_rows")


def softmax_rows_bwd(d_probs, probs, d_scores, nmat, s, causal, stream=None):
    _check(lib().optimus_softmax_rows_bwd(_ptr(d_probs), _ptr(probs), _ptr(d_scores), nmat, s, int(causal), _stream(stream)),
           "optimus_softmax_rows_bwd")


def attention_fused_workspace_bytes(b, s, h, n, q) -> int:
    return lib().optimus_attention_fused_workspace_bytes(b, s, h, n, q)


def attention_fused_fwd(qkv, attn, lse, b, s, h, n, q, i, j, causal, dtype, stream=None):
    _check(lib().optimus_attention_fused_fwd(_ptr(qkv), _ptr(attn), _ptr(lse), b, s, h, n, q, i, j, int(causal), dtype,
                                             _stream(stream)), "optimus_attention_fused_fwd")


def attention_fused_bwd(qkv, attn, lse, d_attn, d_qkv, b, s, h, n, q, i, j, causal, dtype, ws, stream=None):
    p, nb = _ws(ws)
    _check(lib().optimus_attention_fused_bwd(_ptr(qkv), _ptr(attn), _ptr(lse), _ptr(d_attn), _ptr(d_qkv), b, s, h, n, q, i, j,
                                             int(causal), dtype, p, nb, _stream(stream)), "optimus_attention_fused_bwd")


def layer_workspace_bytes(cfg: LayerCfg) -> int:
    return lib().optimus_layer_workspace_bytes(C.byref(cfg))


def layer_workspace_bytes_grid(cfg: LayerCfg) -> int:
    return lib().optimus_layer_workspace_bytes_grid(C.byref(cfg))


def make_layer_tensors(tensors: dict) -> LayerTensors:
    """tensors: name -> torch tensor (or None) for every field of optimus_layer_tensors."""
    t = LayerTensors()
    for name in LAYER_TENSOR_FIELDS:
        setattr(t, name, _ptr(tensors.get(name)))
    return t


def layer_fwd(cfg: LayerCfg, t: LayerTensors, i, j, ws, stream=None):
    p, nb = _ws(ws)
    _check(lib().optimus_layer_fwd(C.byref(cfg), C.byref(t), i, j, p, nb, _stream(stream)), "optimus_layer_fwd")


def layer_bwd(cfg: LayerCfg, t: LayerTensors, i, j, ws, stream=None):
    p, nb = _ws(ws)
    _check(lib().optimus_layer_bwd(C.byref(cfg), C.byref(t), i, j, p, nb, _stream(stream)), "optimus_layer_bwd")


def embedding_fwd(tokens, table, x, M, v, h, q, i, j, dtype, stream=None):
    _check(lib().optimus_embedding_fwd(_ptr(tokens), _ptr(table), _ptr(x), M, v, h, q, i, j, dtype, _stream(stream)),
           "optimus_embedding_fwd")


def embedding_bwd(tokens, d_x, d_table, M, v, h, q, l, j, dtype, stream=None):
    _check(lib().optimus_embedding_bwd(_ptr(tokens), _ptr(d_x), _ptr(d_table), M, v, h, q, l, j, dtype, _stream(stream)),
           "optimus_embedding_bwd")


def cross_entropy2d_stats(logits, stats, M, v, q, i, l, dtype, stream=None):
    _check(lib().optimus_cross_entropy2d_stats(_ptr(logits), _ptr(stats), M, v, q, i, l, dtype, _stream(stream)),
           "optimus_cross_entropy2d_stats")


def cross_entropy2d(logits, labels, loss, lse, stats, M, v, q, i, j, dtype, stream=None):
    _check(lib().optimus_cross_entropy2d(_ptr(logits), _ptr(labels), _ptr(loss), _ptr(lse), _ptr(stats), M, v, q, i, j, dtype,
                                         _stream(stream)), "optimus_cross_entropy2d")


def cross_entropy2d_bwd(logits, labels, lse, d_logits, scale, M, v, q, i, j, dtype, stream=None):
    _check(lib().optimus_cross_entropy2d_bwd(_ptr(logits), _ptr(labels), _ptr(lse), _ptr(d_logits), float(scale), M, v, q, i, j,
                                             dtype, _stream(stream)), "optimus_cross_entropy2d_bwd")


def stack_sizes(cfg: LayerCfg, n_layers: int) -> StackSizes:
    out = StackSizes()
    _check(lib().optimus_stack_sizes_of(C.byref(cfg), n_layers, C.byref(out)), "optimus_stack_sizes_of")
    return out


def layer_grads_in(cfg: LayerCfg, param_grad) -> LayerGrads:
    out = LayerGrads()
    _check(lib().optimus_layer_grads_in(C.byref(cfg), _ptr(param_grad), C.byref(out)), "optimus_layer_grads_in")
    return out


def make_layer_params(tensors: dict) -> LayerParams:
    p = LayerParams()
    for name in LAYER_PARAM_FIELDS:
        setattr(p, name, _ptr(tensors[name]))
    return p


def make_layer_grads(tensors: dict) -> LayerGrads:
    g = LayerGrads()
    for name in LAYER_GRAD_FIELDS:
        setattr(g, name, _ptr(tensors[name]))
    return g


def make_stack_buffers(workspace, forward, backward, conjunction, checkpoint) -> StackBuffers:
    return StackBuffers(_ptr(workspace), _ptr(forward), _ptr(backward), _ptr(conjunction), _ptr(checkpoint))


def stack_fwd(cfg: LayerCfg, params, x, buf: StackBuffers, out, stream=None):
    """params: list of LayerParams, one per layer."""
    arr = (LayerParams * len(params))(*params)
    _check(lib().optimus_stack_fwd(C.byref(cfg), len(params), arr, _ptr(x), C.byref(buf), _ptr(out), _stream(stream)),
           "optimus_stack_fwd")


def stack_bwd(cfg: LayerCfg, params, grads, d_out, buf: StackBuffers, d_x, done=None, stream=None):
    """params / grads: lists of LayerParams / LayerGrads, one per layer; done(layer) is called on the host after each
    layer's backward kernels have been enqueued."""
    pa = (LayerParams * len(params))(*params)
    ga = (LayerGrads * len(grads))(*grads)
    cb = LAYER_DONE_FN((lambda layer, user: done(layer)) if done is not None else 0)
    _check(lib().optimus_stack_bwd(C.byref(cfg), len(params), pa, ga, _ptr(d_out), C.byref(buf), _ptr(d_x), cb, None,
                                   _stream(stream)), "optimus_stack_bwd")


def gemm_flops(M, K, N, q) -> int:
    return lib().optimus_gemm_flops(M, K, N, q)


def layer_flops(cfg: LayerCfg, what: int) -> int:
    return lib().optimus_layer_flops(C.byref(cfg), what)


def debug_set_gemm_variant(v: int):
    lib().optimus_debug_set_gemm_variant(v)


def debug_set_corun_variants(chain_v: int, branch_v: int) -> None:
    lib().optimus_debug_set_corun_variants(chain_v, branch_v)


def debug_mfma_rate(out, workgroups, iters, random_data, stream=None):
    _check(lib().optimus_debug_mfma_rate(_ptr(out), workgroups, iters, int(random_data), _stream(stream)), "optimus_debug_mfma_rate")


def debug_plan_summa(form, M, K, N, q, i, j, corun=0, have_ws=True):
    """(variant, panel splits, walked inside the workgroups) a bf16 product of this shape would be launched with; host
    arithmetic only (works without a GPU)."""
    out = (C.c_int * 3)()
    f = FORMS[form] if isinstance(form, str) else form
    _check(lib().optimus_debug_plan_summa(f, M, K, N, q, i, j, corun, 1 if have_ws else 0, out), "optimus_debug_plan_summa")
    return out[0], out[1], out[2]


def debug_last_gemm_plan():
    """(variant, panel splits, 1 if the split is emulated inside each workgroup) of the most recent matrix-core product."""
    p = lib().optimus_debug_last_gemm_plan()
    return (p & 0xFF, (p >> 8) & 0xFF, p >> 16) if p >= 0 else None
