"""Thin ctypes binding of libmtnlg.so (same names as include/mtnlg.h).

Argument marshalling only: torch tensors give device pointers and the current
stream; every step of the layer runs in the library's HIP kernels.  If the
library is not built this module raises -- there is no fallback.
"""
import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libmtnlg.so")

PARAM_NAMES = ("ln1_g", "ln1_b", "w_qkv", "b_qkv", "w_o", "b_o",
               "ln2_g", "ln2_b", "w_fc1", "b_fc1", "w_fc2", "b_fc2")

F32, BF16 = 0, 1
GELU_TANH, GELU_ERF = 0, 1
RECOMPUTE, ACCUMULATE_WGRAD, WGRAD_FP32 = 1, 2, 4
GEMM_NT, GEMM_NN, GEMM_TN = 0, 1, 2
EPI_BIAS, EPI_GELU, EPI_RESIDUAL, EPI_ACCUMULATE, EPI_OUT_F32, EPI_GELU_ERF, EPI_GELU_GRAD = 1, 2, 4, 8, 16, 32, 64
KERNEL_CLASSES = ("gemm_nt", "gemm_nn", "gemm_tn", "attn_fwd", "attn_bwd", "ln_fwd", "ln_bwd",
                  "gelu", "colsum", "elementwise")


class MtnlgError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        super().__init__(f"{where}: {status_string(status)} ({status})")


class LayerDesc(ctypes.Structure):
    _fields_ = [("hidden", ctypes.c_int32), ("heads_local", ctypes.c_int32),
                ("head_dim", ctypes.c_int32), ("ffn_local", ctypes.c_int32),
                ("seq", ctypes.c_int32), ("micro_batch", ctypes.c_int32),
                ("tp_size", ctypes.c_int32), ("tp_rank", ctypes.c_int32),
                ("dtype", ctypes.c_int32), ("gelu", ctypes.c_int32),
                ("ln_eps", ctypes.c_float), ("softmax_scale", ctypes.c_float),
                ("flags", ctypes.c_uint32)]


class AdamDesc(ctypes.Structure):
    _fields_ = [("lr", ctypes.c_float), ("beta1", ctypes.c_float), ("beta2", ctypes.c_float), ("eps", ctypes.c_float),
                ("weight_decay", ctypes.c_float), ("max_grad_norm", ctypes.c_float), ("step", ctypes.c_int32)]


class HeadDesc(ctypes.Structure):
    _fields_ = [("hidden", ctypes.c_int32), ("vocab_local", ctypes.c_int32), ("vocab_start", ctypes.c_int32),
                ("seq", ctypes.c_int32), ("micro_batch", ctypes.c_int32), ("dtype", ctypes.c_int32),
                ("ln_eps", ctypes.c_float)]


REDUCE_OP_FN = ctypes.CFUNCTYPE(ctypes.c_int, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int, ctypes.c_int,
                                ctypes.c_void_p, ctypes.c_void_p)
REDUCE_SUM, REDUCE_MAX = 0, 1


class _Ptrs12(ctypes.Structure):
    _fields_ = [(n, ctypes.c_void_p) for n in PARAM_NAMES]


class SavedLayout(ctypes.Structure):
    _fields_ = [(n, ctypes.c_size_t) for n in
                ("u1", "qkv", "a", "x1", "u2", "z", "g", "mu1", "rs1", "mu2", "rs2", "lse", "total")]


REDUCE_FN = ctypes.CFUNCTYPE(ctypes.c_int, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int,
                             ctypes.c_void_p, ctypes.c_void_p)

_lib = None


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is not built; run `python -m paper_2201_11990_amd.build` "
                               "(there is no CPU fallback)")
        L = ctypes.CDLL(LIB_PATH)
        vp, sz, i32, i64, u32, f32 = (ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int32, ctypes.c_int64,
                                      ctypes.c_uint32, ctypes.c_float)
        dp = ctypes.POINTER(LayerDesc)
        pp = ctypes.POINTER(_Ptrs12)
        sigs = {
            "mtnlg_version": (ctypes.c_int, []),
            "mtnlg_status_string": (ctypes.c_char_p, [ctypes.c_int]),
            "mtnlg_layer_desc_check": (ctypes.c_int, [dp]),
            "mtnlg_saved_layout_get": (ctypes.c_int, [dp, ctypes.POINTER(SavedLayout)]),
            "mtnlg_saved_bytes": (sz, [dp]),
            "mtnlg_stage_saved_bytes": (sz, [dp, ctypes.c_int]),
            "mtnlg_workspace_bytes": (sz, [dp]),
            "mtnlg_layer_fwd": (ctypes.c_int, [dp, pp, vp, vp, vp, vp, sz, REDUCE_FN, vp, vp]),
            "mtnlg_layer_bwd": (ctypes.c_int, [dp, pp, vp, vp, vp, vp, pp, vp, sz, REDUCE_FN, vp, vp]),
            "mtnlg_stage_step": (ctypes.c_int, [dp, ctypes.c_int, pp, vp, vp, vp, vp, pp, vp, sz, vp, sz,
                                                REDUCE_FN, vp, vp]),
            "mtnlg_stage_step_accumulate": (ctypes.c_int, [dp, ctypes.c_int, pp, ctypes.c_int, vp, vp, vp, vp, pp, vp,
                                                           sz, vp, sz, REDUCE_FN, vp, vp]),
            "mtnlg_lm_head_workspace": (sz, [ctypes.POINTER(HeadDesc)]),
            "mtnlg_embedding_fwd": (ctypes.c_int, [ctypes.POINTER(HeadDesc), vp, vp, vp, vp, REDUCE_OP_FN, vp, vp]),
            "mtnlg_embedding_bwd": (ctypes.c_int, [ctypes.POINTER(HeadDesc), vp, vp, vp, vp, vp]),
            "mtnlg_lm_head_step": (ctypes.c_int, [ctypes.POINTER(HeadDesc), vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp,
                                                  vp, sz, REDUCE_OP_FN, vp, vp]),
            "mtnlg_grad_sqnorm_workspace": (sz, []),
            "mtnlg_grad_sqnorm": (ctypes.c_int, [i64, vp, vp, vp, ctypes.c_int, vp]),
            "mtnlg_adam_step": (ctypes.c_int, [ctypes.POINTER(AdamDesc), i64, vp, vp, vp, vp, vp, vp, vp]),
            "mtnlg_gemm_workspace": (sz, [ctypes.c_int, ctypes.c_int, i64, i64, i64]),
            "mtnlg_gemm": (ctypes.c_int, [ctypes.c_int, ctypes.c_int, i64, i64, i64, vp, vp, vp, vp, vp, u32, vp, sz, vp]),
            "mtnlg_layernorm_fwd": (ctypes.c_int, [ctypes.c_int, i64, i64, vp, vp, vp, vp, vp, f32, vp, vp, vp, vp, vp]),
            "mtnlg_layernorm_bwd_workspace": (sz, [i64, i64]),
            "mtnlg_layernorm_bwd": (ctypes.c_int, [ctypes.c_int, i64, i64, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp,
                                                   ctypes.c_int, ctypes.c_int, vp, vp]),
            "mtnlg_attention_fwd": (ctypes.c_int, [ctypes.c_int, i32, i32, i32, i32, f32, vp, vp, vp, vp]),
            "mtnlg_attention_bwd_workspace": (sz, [i32, i32, i32, i32]),
            "mtnlg_attention_bwd": (ctypes.c_int, [ctypes.c_int, i32, i32, i32, i32, f32, vp, vp, vp, vp, vp, vp, vp]),
            "mtnlg_gelu_fwd": (ctypes.c_int, [ctypes.c_int, ctypes.c_int, i64, vp, vp, vp]),
            "mtnlg_gelu_bwd": (ctypes.c_int, [ctypes.c_int, ctypes.c_int, i64, vp, vp, vp, vp]),
            "mtnlg_colsum_workspace": (sz, [i64, i64]),
            "mtnlg_colsum": (ctypes.c_int, [ctypes.c_int, i64, i64, vp, vp, ctypes.c_int, ctypes.c_int, vp, vp]),
            "mtnlg_colsum_static_max_columns": (i64, []),
            "mtnlg_colsum_static": (ctypes.c_int, [ctypes.c_int, i64, i64, vp, vp, ctypes.c_int, ctypes.c_int, vp]),
            "mtnlg_bias_residual": (ctypes.c_int, [ctypes.c_int, i64, i64, vp, vp, vp, vp, vp]),
            "mtnlg_calibrate_mfma_operand_bytes": (sz, [ctypes.c_int]),
            "mtnlg_calibrate_mfma_flops": (i64, [ctypes.c_int, ctypes.c_int]),
            "mtnlg_calibrate_mfma": (ctypes.c_int, [ctypes.c_int, ctypes.c_int, vp, vp, vp]),
            "mtnlg_calibrate_copy": (ctypes.c_int, [vp, vp, i64, vp]),
            "mtnlg_profile_enable": (ctypes.c_int, [ctypes.c_int]),
            "mtnlg_profile_pause": (ctypes.c_int, [ctypes.c_int]),
            "mtnlg_profile_read": (ctypes.c_int, [ctypes.POINTER(ctypes.c_int32), ctypes.POINTER(ctypes.c_float)]),
        }
        for name, (res, args) in sigs.items():
            fn = getattr(L, name)
            fn.restype, fn.argtypes = res, args
        _lib = L
    return _lib


EXPORTED = ("mtnlg_version", "mtnlg_status_string", "mtnlg_layer_desc_check", "mtnlg_saved_layout_get",
            "mtnlg_saved_bytes", "mtnlg_stage_saved_bytes", "mtnlg_workspace_bytes", "mtnlg_layer_fwd",
            "mtnlg_layer_bwd", "mtnlg_stage_step", "mtnlg_stage_step_accumulate", "mtnlg_gemm_workspace", "mtnlg_gemm", "mtnlg_layernorm_fwd",
            "mtnlg_layernorm_bwd_workspace", "mtnlg_layernorm_bwd", "mtnlg_attention_fwd",
            "mtnlg_attention_bwd_workspace", "mtnlg_attention_bwd", "mtnlg_gelu_fwd", "mtnlg_gelu_bwd",
            "mtnlg_colsum_workspace", "mtnlg_colsum", "mtnlg_colsum_static_max_columns", "mtnlg_colsum_static",
            "mtnlg_bias_residual", "mtnlg_grad_sqnorm_workspace", "mtnlg_grad_sqnorm", "mtnlg_adam_step",
            "mtnlg_lm_head_workspace", "mtnlg_embedding_fwd", "mtnlg_embedding_bwd", "mtnlg_lm_head_step",
            "mtnlg_calibrate_mfma_operand_bytes", "mtnlg_calibrate_mfma_flops", "mtnlg_calibrate_mfma",
            "mtnlg_calibrate_copy", "mtnlg_profile_enable", "mtnlg_profile_pause", "mtnlg_profile_read")


def status_string(status):
    return lib().mtnlg_status_string(int(status)).decode()


def _check(status, where):
    if status != 0:
        raise MtnlgError(status, where)


def _dtype_code(t):
    if t.dtype == torch.float32:
        return F32
    if t.dtype == torch.bfloat16:
        return BF16
    raise TypeError(f"unsupported dtype {t.dtype}")


def _p(t):
    """Device pointer of a contiguous CUDA tensor (None -> NULL)."""
    if t is None:
        return None
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError("tensors handed to the library must be contiguous device tensors")
    return ctypes.c_void_p(t.data_ptr())


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def make_desc(hidden, heads_local, head_dim, ffn_local, seq, micro_batch, dtype, tp_size=1, tp_rank=0,
              gelu=GELU_TANH, ln_eps=0.0, softmax_scale=0.0, flags=0):
    code = dtype if isinstance(dtype, int) else {"fp32": F32, "bf16": BF16,
                                                 torch.float32: F32, torch.bfloat16: BF16}[dtype]
    return LayerDesc(hidden, heads_local, head_dim, ffn_local, seq, micro_batch, tp_size, tp_rank, code,
                     gelu, ln_eps, softmax_scale, flags)


def desc_from_workload(wl, flags=0, **kw):
    return make_desc(wl.hidden, wl.heads, wl.head_dim, wl.ffn, wl.seq, wl.micro_batch, wl.dtype,
                     tp_size=wl.tp_size, flags=flags | (RECOMPUTE if wl.recompute else 0), **kw)


def mtnlg_version():
    return lib().mtnlg_version()


def mtnlg_layer_desc_check(desc):
    return lib().mtnlg_layer_desc_check(ctypes.byref(desc))


def mtnlg_saved_layout_get(desc):
    out = SavedLayout()
    _check(lib().mtnlg_saved_layout_get(ctypes.byref(desc), ctypes.byref(out)), "mtnlg_saved_layout_get")
    return out


def mtnlg_saved_bytes(desc):
    return lib().mtnlg_saved_bytes(ctypes.byref(desc))


def mtnlg_stage_saved_bytes(desc, n_layers):
    return lib().mtnlg_stage_saved_bytes(ctypes.byref(desc), n_layers)


def mtnlg_workspace_bytes(desc):
    return lib().mtnlg_workspace_bytes(ctypes.byref(desc))


def _table(tensors):
    st = _Ptrs12()
    for n in PARAM_NAMES:
        setattr(st, n, _p(tensors[n]))
    return st


def _tables(list_of_dicts):
    arr = (_Ptrs12 * len(list_of_dicts))()
    for i, d in enumerate(list_of_dicts):
        for n in PARAM_NAMES:
            setattr(arr[i], n, _p(d[n]))
    return arr


def _hook(reduce):
    """reduce(ptr:int, count:int, dtype:int, stream:int) -> None, or None."""
    if reduce is None:
        return ctypes.cast(None, REDUCE_FN)

    def cb(buf, count, dtype, stream, _user):
        try:
            reduce(buf, count, dtype, stream)
            return 0
        except Exception:  # noqa: BLE001 - must not unwind through C
            return 1

    return REDUCE_FN(cb)


def _nbytes(t):
    return t.numel() * t.element_size()


def mtnlg_layer_fwd(desc, weights, x, y, saved, workspace, reduce=None):
    hook = _hook(reduce)
    _check(lib().mtnlg_layer_fwd(ctypes.byref(desc), ctypes.byref(_table(weights)), _p(x), _p(y), _p(saved),
                                 _p(workspace), _nbytes(workspace), hook, None, _stream()), "mtnlg_layer_fwd")


def mtnlg_layer_bwd(desc, weights, x, saved, dy, dx, grads, workspace, reduce=None):
    hook = _hook(reduce)
    _check(lib().mtnlg_layer_bwd(ctypes.byref(desc), ctypes.byref(_table(weights)), _p(x), _p(saved), _p(dy),
                                 _p(dx), ctypes.byref(_table(grads)), _p(workspace), _nbytes(workspace), hook,
                                 None, _stream()), "mtnlg_layer_bwd")


class StageArgs:
    """Marshalled argument tables of mtnlg_stage_step, built once and reused per call."""

    def __init__(self, desc, weights, grads):
        self.desc, self.n_layers = desc, len(weights)
        self.w, self.g = _tables(weights), _tables(grads)
        self._keep = (weights, grads)


def mtnlg_stage_step(desc, weights, x_in, dy_out, y_out, dx_in, grads, saved, workspace, reduce=None,
                     args=None):
    a = args if args is not None else StageArgs(desc, weights, grads)
    hook = _hook(reduce)
    _check(lib().mtnlg_stage_step(ctypes.byref(a.desc), a.n_layers, a.w, _p(x_in), _p(dy_out), _p(y_out),
                                  _p(dx_in), a.g, _p(saved), _nbytes(saved), _p(workspace),
                                  _nbytes(workspace), hook, None, _stream()), "mtnlg_stage_step")


def mtnlg_stage_step_accumulate(desc, weights, x_in, dy_out, y_out, dx_in, grads, saved, workspace, reduce=None,
                                args=None):
    """x_in, dy_out, y_out, dx_in: [n_micro, b, s, h] contiguous."""
    a = args if args is not None else StageArgs(desc, weights, grads)
    hook = _hook(reduce)
    n_micro = x_in.shape[0]
    assert x_in.is_contiguous() and dy_out.is_contiguous() and y_out.is_contiguous() and dx_in.is_contiguous()
    assert dy_out.shape[0] == n_micro and y_out.shape[0] == n_micro and dx_in.shape[0] == n_micro
    _check(lib().mtnlg_stage_step_accumulate(ctypes.byref(a.desc), a.n_layers, a.w, n_micro, _p(x_in), _p(dy_out),
                                             _p(y_out), _p(dx_in), a.g, _p(saved), _nbytes(saved), _p(workspace),
                                             _nbytes(workspace), hook, None, _stream()),
           "mtnlg_stage_step_accumulate")


def mtnlg_gemm_workspace(dtype, layout, M, N, K):
    return lib().mtnlg_gemm_workspace(dtype, layout, M, N, K)


def mtnlg_gemm(layout, A, B, C, bias=None, aux=None, epilogue=0, workspace=None):
    if layout == GEMM_NT:
        (M, K), N = A.shape, B.shape[0]
        assert B.shape == (N, K)
    elif layout == GEMM_NN:
        (M, K), N = A.shape, B.shape[1]
        assert B.shape == (K, N)
    else:
        (K, M), N = A.shape, B.shape[1]
        assert B.shape == (K, N)
    assert C.shape == (M, N)
    _check(lib().mtnlg_gemm(_dtype_code(A), layout, M, N, K, _p(A), _p(B), _p(C), _p(bias), _p(aux), epilogue,
                            _p(workspace), _nbytes(workspace) if workspace is not None else 0, _stream()),
           "mtnlg_gemm")


def mtnlg_layernorm_fwd(x, gamma, beta, eps, out, mean, rstd, partial=None, bias=None, xsum=None):
    T, h = x.shape
    _check(lib().mtnlg_layernorm_fwd(_dtype_code(x), T, h, _p(x), _p(partial), _p(bias), _p(gamma), _p(beta),
                                     eps, _p(xsum), _p(out), _p(mean), _p(rstd), _stream()),
           "mtnlg_layernorm_fwd")


def mtnlg_layernorm_bwd_workspace(T, h):
    return lib().mtnlg_layernorm_bwd_workspace(T, h)


def mtnlg_layernorm_bwd(x, gamma, mean, rstd, dout, dx, dgamma, dbeta, workspace, dres=None, colsum_dx=None,
                        grad_f32=False, accumulate=False):
    T, h = x.shape
    _check(lib().mtnlg_layernorm_bwd(_dtype_code(x), T, h, _p(x), _p(gamma), _p(mean), _p(rstd), _p(dout),
                                     _p(dres), _p(dx), _p(dgamma), _p(dbeta), _p(colsum_dx), int(grad_f32),
                                     int(accumulate), _p(workspace), _stream()), "mtnlg_layernorm_bwd")


def mtnlg_attention_fwd(b, s, n, d, scale, qkv, a, lse):
    _check(lib().mtnlg_attention_fwd(_dtype_code(qkv), b, s, n, d, scale, _p(qkv), _p(a), _p(lse), _stream()),
           "mtnlg_attention_fwd")


def mtnlg_attention_bwd_workspace(b, s, n, d):
    return lib().mtnlg_attention_bwd_workspace(b, s, n, d)


def mtnlg_attention_bwd(b, s, n, d, scale, qkv, a, lse, da, dqkv, workspace):
    _check(lib().mtnlg_attention_bwd(_dtype_code(qkv), b, s, n, d, scale, _p(qkv), _p(a), _p(lse), _p(da),
                                     _p(dqkv), _p(workspace), _stream()), "mtnlg_attention_bwd")


def mtnlg_gelu_fwd(z, g, gelu=GELU_TANH):
    _check(lib().mtnlg_gelu_fwd(_dtype_code(z), gelu, z.numel(), _p(z), _p(g), _stream()), "mtnlg_gelu_fwd")


def mtnlg_gelu_bwd(z, dg, dz, gelu=GELU_TANH):
    _check(lib().mtnlg_gelu_bwd(_dtype_code(z), gelu, z.numel(), _p(z), _p(dg), _p(dz), _stream()),
           "mtnlg_gelu_bwd")


def mtnlg_colsum_workspace(T, C):
    return lib().mtnlg_colsum_workspace(T, C)


def mtnlg_colsum(x, out, workspace, accumulate=False):
    T, C = x.shape
    _check(lib().mtnlg_colsum(_dtype_code(x), T, C, _p(x), _p(out), int(out.dtype == torch.float32),
                              int(accumulate), _p(workspace), _stream()), "mtnlg_colsum")


def mtnlg_colsum_static_max_columns():
    return lib().mtnlg_colsum_static_max_columns()


def mtnlg_colsum_static(x, out, accumulate=False):
    T, C = x.shape
    _check(lib().mtnlg_colsum_static(_dtype_code(x), T, C, _p(x), _p(out), int(out.dtype == torch.float32),
                                     int(accumulate), _stream()), "mtnlg_colsum_static")


def mtnlg_bias_residual(res, partial, bias, out):
    T, h = res.shape
    _check(lib().mtnlg_bias_residual(_dtype_code(res), T, h, _p(res), _p(partial), _p(bias), _p(out), _stream()),
           "mtnlg_bias_residual")


def head_desc(hidden, vocab_local, vocab_start, seq, micro_batch, dtype, ln_eps=1e-5):
    return HeadDesc(hidden, vocab_local, vocab_start, seq, micro_batch, {"fp32": F32, "bf16": BF16}[dtype], ln_eps)


def _op_hook(reduce):
    """reduce(ptr:int, count:int, dtype:int, op:int, stream:int) -> None, or None."""
    if reduce is None:
        return ctypes.cast(None, REDUCE_OP_FN)

    def cb(buf, count, dtype, op, stream, _user):
        try:
            reduce(buf, count, dtype, op, stream)
            return 0
        except Exception:  # noqa: BLE001 - must not unwind through C
            return 1

    return REDUCE_OP_FN(cb)


def mtnlg_lm_head_workspace(desc):
    return lib().mtnlg_lm_head_workspace(ctypes.byref(desc))


def mtnlg_embedding_fwd(desc, tokens, emb, pos, x, reduce=None):
    assert tokens.dtype == torch.int32
    _check(lib().mtnlg_embedding_fwd(ctypes.byref(desc), _p(tokens), _p(emb), _p(pos), _p(x), _op_hook(reduce), None,
                                     _stream()), "mtnlg_embedding_fwd")


def mtnlg_embedding_bwd(desc, tokens, dx, demb, dpos):
    assert tokens.dtype == torch.int32
    _check(lib().mtnlg_embedding_bwd(ctypes.byref(desc), _p(tokens), _p(dx), _p(demb), _p(dpos), _stream()),
           "mtnlg_embedding_bwd")


def mtnlg_lm_head_step(desc, x, ln_g, ln_b, emb, targets, dloss, loss, dx, d_ln_g, d_ln_b, demb, workspace, reduce=None):
    assert targets.dtype == torch.int32 and loss.dtype == torch.float32
    assert dloss is None or dloss.dtype == torch.float32
    _check(lib().mtnlg_lm_head_step(ctypes.byref(desc), _p(x), _p(ln_g), _p(ln_b), _p(emb), _p(targets), _p(dloss),
                                    _p(loss), _p(dx), _p(d_ln_g), _p(d_ln_b), _p(demb), _p(workspace),
                                    _nbytes(workspace), _op_hook(reduce), None, _stream()), "mtnlg_lm_head_step")


def mtnlg_grad_sqnorm_workspace():
    return lib().mtnlg_grad_sqnorm_workspace()


def mtnlg_grad_sqnorm(grad, workspace, sqnorm, accumulate=False):
    """grad: fp32 tensor (any shape, contiguous); sqnorm: fp32 device tensor of one element."""
    assert grad.dtype == torch.float32 and grad.is_contiguous() and sqnorm.dtype == torch.float32
    _check(lib().mtnlg_grad_sqnorm(grad.numel(), _p(grad), _p(workspace), _p(sqnorm), int(bool(accumulate)), _stream()),
           "mtnlg_grad_sqnorm")


def mtnlg_adam_step(master, m, v, grad, weight_bf16=None, sqnorm=None, *, lr, step, beta1=0.9, beta2=0.95, eps=1e-8,
                    weight_decay=0.1, max_grad_norm=1.0):
    """In-place Adam update of fp32 tensors master, m, v from fp32 grad; weight_bf16 receives the rounded weight."""
    for t in (master, m, v, grad):
        assert t.dtype == torch.float32 and t.is_contiguous() and t.numel() == master.numel()
    if weight_bf16 is not None:
        assert weight_bf16.dtype == torch.bfloat16 and weight_bf16.is_contiguous() and weight_bf16.numel() == master.numel()
    d = AdamDesc(lr, beta1, beta2, eps, weight_decay, max_grad_norm, step)
    _check(lib().mtnlg_adam_step(ctypes.byref(d), master.numel(), _p(master), _p(m), _p(v), _p(grad), _p(weight_bf16),
                                 _p(sqnorm), _stream()), "mtnlg_adam_step")


def mtnlg_calibrate_mfma_operand_bytes(workgroups):
    return lib().mtnlg_calibrate_mfma_operand_bytes(workgroups)


def mtnlg_calibrate_mfma_flops(workgroups, iters):
    return lib().mtnlg_calibrate_mfma_flops(workgroups, iters)


def mtnlg_calibrate_mfma(workgroups, iters, operands, out):
    assert operands.dtype == torch.bfloat16 and _nbytes(operands) >= mtnlg_calibrate_mfma_operand_bytes(workgroups)
    assert out.dtype == torch.float32 and out.numel() >= workgroups * 512
    _check(lib().mtnlg_calibrate_mfma(workgroups, iters, _p(operands), _p(out), _stream()), "mtnlg_calibrate_mfma")


def mtnlg_calibrate_copy(dst, src):
    assert _nbytes(dst) == _nbytes(src)
    _check(lib().mtnlg_calibrate_copy(_p(dst), _p(src), _nbytes(src), _stream()), "mtnlg_calibrate_copy")


def mtnlg_profile_enable(on):
    _check(lib().mtnlg_profile_enable(int(bool(on))), "mtnlg_profile_enable")


def mtnlg_profile_pause(paused):
    _check(lib().mtnlg_profile_pause(int(bool(paused))), "mtnlg_profile_pause")


def mtnlg_profile_read():
    n = len(KERNEL_CLASSES)
    launches, ms = (ctypes.c_int32 * n)(), (ctypes.c_float * n)()
    _check(lib().mtnlg_profile_read(launches, ms), "mtnlg_profile_read")
    return {k: (launches[i], ms[i]) for i, k in enumerate(KERNEL_CLASSES)}
