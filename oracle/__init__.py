"""fp64 CPU oracle for one tensor-parallel slice of a GPT decoder layer.

TEST INFRASTRUCTURE.  Only ``tests/``, ``__graft_entry__.smoke()`` and the
``cpu_baseline`` leg of ``bench.py`` may import this package; the GPU library
and its Python binding never do.  The arithmetic lives in ``mtnlg_oracle.c``
(plain loops, fp64); this module only marshals numpy arrays through ctypes.

Model definition followed: Section 3.2 of the paper (GPT-2 style decoder, layer
count, hidden size, heads, sequence length, 8-way tensor slicing) and the
tensor-slicing paragraph of Section 2.1; the per-operation readings are listed
in the C file's header.
"""
import ctypes
import os

import numpy as np

from . import build as _build
from .optimizer import adam_step, clip_coefficient, grad_sqnorm  # noqa: F401  (optimizer step, numpy)

_PARAM_NAMES = ("ln1_g", "ln1_b", "w_qkv", "b_qkv", "w_o", "b_o",
                "ln2_g", "ln2_b", "w_fc1", "b_fc1", "w_fc2", "b_fc2")
_SAVED_NAMES = ("u1", "mu1", "rs1", "qkv", "a", "A_r", "x1", "u2", "mu2", "rs2", "z", "g", "M_r")

_dp = ctypes.POINTER(ctypes.c_double)


class _Dims(ctypes.Structure):
    _fields_ = [("hidden", ctypes.c_int32), ("heads", ctypes.c_int32),
                ("head_dim", ctypes.c_int32), ("ffn", ctypes.c_int32),
                ("seq", ctypes.c_int32), ("batch", ctypes.c_int32),
                ("gelu_exact", ctypes.c_int32), ("pad_", ctypes.c_int32),
                ("ln_eps", ctypes.c_double), ("softmax_scale", ctypes.c_double)]


class _Ptrs12(ctypes.Structure):
    _fields_ = [(n, _dp) for n in _PARAM_NAMES]


class _Saved(ctypes.Structure):
    _fields_ = [(n, _dp) for n in _SAVED_NAMES]


REDUCE_FN = ctypes.CFUNCTYPE(None, _dp, ctypes.c_size_t, ctypes.c_void_p)

_lib = None


def lib():
    global _lib
    if _lib is None:
        path = _build.build(force=False)
        _lib = ctypes.CDLL(path)
        _lib.orc_gelu.restype = ctypes.c_double
        _lib.orc_gelu.argtypes = [ctypes.c_double, ctypes.c_int]
        _lib.orc_gelu_grad.restype = ctypes.c_double
        _lib.orc_gelu_grad.argtypes = [ctypes.c_double, ctypes.c_int]
    return _lib


class Dims:
    """Shape of one slice: hidden h, local heads n, head dim d, local FFN F, seq s, batch b."""

    def __init__(self, hidden, heads, head_dim, ffn, seq, batch, gelu_exact=False,
                 ln_eps=1e-5, softmax_scale=0.0):
        self.hidden, self.heads, self.head_dim, self.ffn = hidden, heads, head_dim, ffn
        self.seq, self.batch = seq, batch
        self.gelu_exact, self.ln_eps, self.softmax_scale = bool(gelu_exact), ln_eps, softmax_scale

    @property
    def tokens(self):
        return self.batch * self.seq

    @property
    def proj(self):
        return self.heads * self.head_dim

    def c(self):
        return _Dims(self.hidden, self.heads, self.head_dim, self.ffn, self.seq, self.batch,
                     int(self.gelu_exact), 0, self.ln_eps, self.softmax_scale)

    def param_shapes(self):
        h, p, F = self.hidden, self.proj, self.ffn
        return {"ln1_g": (h,), "ln1_b": (h,), "w_qkv": (3 * p, h), "b_qkv": (3 * p,),
                "w_o": (h, p), "b_o": (h,), "ln2_g": (h,), "ln2_b": (h,),
                "w_fc1": (F, h), "b_fc1": (F,), "w_fc2": (h, F), "b_fc2": (h,)}

    def saved_shapes(self):
        T, h, p, F = self.tokens, self.hidden, self.proj, self.ffn
        return {"u1": (T, h), "mu1": (T,), "rs1": (T,), "qkv": (T, 3 * p), "a": (T, p),
                "A_r": (T, h), "x1": (T, h), "u2": (T, h), "mu2": (T,), "rs2": (T,),
                "z": (T, F), "g": (T, F), "M_r": (T, h)}


def _f64(a):
    return np.ascontiguousarray(a, dtype=np.float64)


def _ptr(a):
    return a.ctypes.data_as(_dp)


def _weights_struct(dims, w):
    keep = {}
    st = _Ptrs12()
    for name, shape in dims.param_shapes().items():
        arr = _f64(w[name])
        assert arr.shape == shape, (name, arr.shape, shape)
        keep[name] = arr
        setattr(st, name, _ptr(arr))
    return st, keep


def _alloc_struct(shapes, cls):
    arrs = {k: np.zeros(v, dtype=np.float64) for k, v in shapes.items()}
    st = cls()
    for k, a in arrs.items():
        setattr(st, k, _ptr(a))
    return st, arrs


def _saved_struct(dims, saved):
    st = _Saved()
    keep = {}
    for k, shape in dims.saved_shapes().items():
        arr = _f64(saved[k])
        assert arr.shape == shape, (k, arr.shape, shape)
        keep[k] = arr
        setattr(st, k, _ptr(arr))
    return st, keep


def _wrap_reduce(reduce):
    if reduce is None:
        return ctypes.cast(None, REDUCE_FN), None

    def cb(buf, count, _user):
        view = np.ctypeslib.as_array(buf, shape=(count,))
        reduce(view)

    fn = REDUCE_FN(cb)
    return fn, fn


# ---------------------------------------------------------------- pieces
def gelu(z, exact=False):
    z = _f64(z)
    f = lib().orc_gelu
    return np.array([f(float(v), int(exact)) for v in z.ravel()]).reshape(z.shape)


def gelu_grad(z, exact=False):
    z = _f64(z)
    f = lib().orc_gelu_grad
    return np.array([f(float(v), int(exact)) for v in z.ravel()]).reshape(z.shape)


def layernorm_fwd(x, gamma, beta, eps=1e-5):
    x, gamma, beta = _f64(x), _f64(gamma), _f64(beta)
    T, h = x.shape
    out, mean, rstd = np.empty_like(x), np.empty(T), np.empty(T)
    lib().orc_layernorm_fwd(_ptr(x), _ptr(gamma), _ptr(beta), ctypes.c_int64(T), ctypes.c_int64(h),
                            ctypes.c_double(eps), _ptr(out), _ptr(mean), _ptr(rstd))
    return out, mean, rstd


def layernorm_bwd(x, gamma, mean, rstd, dout):
    x, gamma, mean, rstd, dout = map(_f64, (x, gamma, mean, rstd, dout))
    T, h = x.shape
    dx, dg, db = np.empty_like(x), np.empty(h), np.empty(h)
    lib().orc_layernorm_bwd(_ptr(x), _ptr(gamma), _ptr(mean), _ptr(rstd), _ptr(dout),
                            ctypes.c_int64(T), ctypes.c_int64(h), _ptr(dx), _ptr(dg), _ptr(db))
    return dx, dg, db


def linear_fwd(x, W, bias=None):
    x, W = _f64(x), _f64(W)
    T, K = x.shape
    N = W.shape[0]
    assert W.shape == (N, K)
    out = np.empty((T, N))
    b = _f64(bias) if bias is not None else None
    lib().orc_linear_fwd(_ptr(x), _ptr(W), _ptr(b) if b is not None else None,
                         ctypes.c_int64(T), ctypes.c_int64(N), ctypes.c_int64(K), _ptr(out))
    return out


def linear_dgrad(dout, W):
    dout, W = _f64(dout), _f64(W)
    T, N = dout.shape
    K = W.shape[1]
    dx = np.empty((T, K))
    lib().orc_linear_dgrad(_ptr(dout), _ptr(W), ctypes.c_int64(T), ctypes.c_int64(N),
                           ctypes.c_int64(K), _ptr(dx))
    return dx


def linear_wgrad(dout, x):
    dout, x = _f64(dout), _f64(x)
    T, N = dout.shape
    K = x.shape[1]
    dW, db = np.empty((N, K)), np.empty(N)
    lib().orc_linear_wgrad(_ptr(dout), _ptr(x), ctypes.c_int64(T), ctypes.c_int64(N),
                           ctypes.c_int64(K), _ptr(dW), _ptr(db))
    return dW, db


def attention_fwd(dims, qkv, return_probs=False):
    qkv = _f64(qkv)
    T, p = dims.tokens, dims.proj
    assert qkv.shape == (T, 3 * p)
    a = np.empty((T, p))
    P = np.empty((dims.batch, dims.heads, dims.seq, dims.seq)) if return_probs else None
    d = dims.c()
    lib().orc_attention_fwd(ctypes.byref(d), _ptr(qkv), _ptr(a), _ptr(P) if P is not None else None)
    return (a, P) if return_probs else a


def attention_bwd(dims, qkv, da):
    qkv, da = _f64(qkv), _f64(da)
    dqkv = np.empty_like(qkv)
    d = dims.c()
    lib().orc_attention_bwd(ctypes.byref(d), _ptr(qkv), _ptr(da), _ptr(dqkv))
    return dqkv


# ---------------------------------------------------------------- layer
def layer_fwd(dims, w, x, reduce=None):
    """Forward of one slice.  ``reduce(view)`` sums a partial in place across ranks
    (None: a tensor-parallel group of one).  Returns (y, saved)."""
    x = _f64(x).reshape(dims.tokens, dims.hidden)
    wst, _keep = _weights_struct(dims, w)
    sst, saved = _alloc_struct(dims.saved_shapes(), _Saved)
    y = np.empty_like(x)
    d = dims.c()
    fn, _keepfn = _wrap_reduce(reduce)
    lib().orc_layer_fwd(ctypes.byref(d), ctypes.byref(wst), _ptr(x), _ptr(y), ctypes.byref(sst),
                        fn, None)
    return y, saved


def layer_bwd(dims, w, x, saved, dy, reduce=None):
    """Backward of one slice.  Returns (dx, grads dict over the 12 parameters)."""
    x = _f64(x).reshape(dims.tokens, dims.hidden)
    dy = _f64(dy).reshape(dims.tokens, dims.hidden)
    wst, _keep = _weights_struct(dims, w)
    sst, _keeps = _saved_struct(dims, saved)
    gst, grads = _alloc_struct(dims.param_shapes(), _Ptrs12)
    dx = np.empty_like(x)
    d = dims.c()
    fn, _keepfn = _wrap_reduce(reduce)
    lib().orc_layer_bwd(ctypes.byref(d), ctypes.byref(wst), _ptr(x), ctypes.byref(sst), _ptr(dy),
                        _ptr(dx), ctypes.byref(gst), fn, None)
    return dx, grads


def attn_half_fwd(dims, w, x):
    """LN1 -> QKV -> attention -> projection (no bias).  Returns the saved dict; A_r is the partial."""
    x = _f64(x).reshape(dims.tokens, dims.hidden)
    wst, _keep = _weights_struct(dims, w)
    sst, saved = _alloc_struct(dims.saved_shapes(), _Saved)
    d = dims.c()
    lib().orc_attn_half_fwd(ctypes.byref(d), ctypes.byref(wst), _ptr(x), ctypes.byref(sst))
    return saved


def mlp_half_fwd(dims, w, saved):
    """LN2 -> FC1 -> GeLU -> FC2 (no bias) from saved['x1']; fills u2, z, g, M_r in place."""
    wst, _keep = _weights_struct(dims, w)
    sst, keep = _saved_struct(dims, saved)
    d = dims.c()
    lib().orc_mlp_half_fwd(ctypes.byref(d), ctypes.byref(wst), ctypes.byref(sst))
    saved.update(keep)
    return saved


def mlp_half_bwd(dims, w, saved, dy):
    dy = _f64(dy).reshape(dims.tokens, dims.hidden)
    wst, _keep = _weights_struct(dims, w)
    sst, _keeps = _saved_struct(dims, saved)
    gst, grads = _alloc_struct(dims.param_shapes(), _Ptrs12)
    du = np.empty_like(dy)
    d = dims.c()
    lib().orc_mlp_half_bwd(ctypes.byref(d), ctypes.byref(wst), ctypes.byref(sst), _ptr(dy), _ptr(du),
                           ctypes.byref(gst))
    return du, {k: grads[k] for k in ("w_fc2", "w_fc1", "b_fc1")}


def attn_half_bwd(dims, w, saved, dA):
    dA = _f64(dA).reshape(dims.tokens, dims.hidden)
    wst, _keep = _weights_struct(dims, w)
    sst, _keeps = _saved_struct(dims, saved)
    gst, grads = _alloc_struct(dims.param_shapes(), _Ptrs12)
    du = np.empty_like(dA)
    d = dims.c()
    lib().orc_attn_half_bwd(ctypes.byref(d), ctypes.byref(wst), ctypes.byref(sst), _ptr(dA), _ptr(du),
                            ctypes.byref(gst))
    return du, {k: grads[k] for k in ("w_o", "w_qkv", "b_qkv")}


def num_threads():
    """OpenMP threads the oracle's loops use."""
    return int(lib().orc_num_threads())


def stage_step(dims, weights, x, dy):
    """n_layers slices stacked (identity at the reduce points): forward through all
    layers, backward in reverse.  Returns (y, dx, [grads per layer])."""
    xs, saves = [_f64(x).reshape(dims.tokens, dims.hidden)], []
    for w in weights:
        y, sv = layer_fwd(dims, w, xs[-1])
        xs.append(y)
        saves.append(sv)
    g = _f64(dy).reshape(dims.tokens, dims.hidden)
    grads = [None] * len(weights)
    for l in reversed(range(len(weights))):
        g, grads[l] = layer_bwd(dims, weights[l], xs[l], saves[l], g)
    return xs[-1], g, grads


from .head import (cross_entropy_bwd, cross_entropy_fwd, embedding_bwd, embedding_fwd,  # noqa: E402,F401
                   lm_head_step)
