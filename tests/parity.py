"""Shared helpers of the GPU parity tests: conversions between device tensors and the oracle's
fp64 numpy arrays, and the error measure (relative Frobenius error per output tensor)."""
import numpy as np
import torch

import oracle

# spec tolerances: relative Frobenius error per output tensor
TOL = {"fp32": 1e-5, "bf16": 1e-2}


def to_np(t):
    return t.detach().to("cpu", torch.float64).numpy()


def rel_fro(got, want):
    got = to_np(got) if isinstance(got, torch.Tensor) else np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64).reshape(got.shape)
    den = np.linalg.norm(want)
    num = np.linalg.norm(got - want)
    if den == 0.0:
        return 0.0 if num == 0.0 else float("inf")
    return float(num / den)


def assert_close(got, want, tol, what):
    assert torch.isfinite(got.float()).all() if isinstance(got, torch.Tensor) else True, f"{what}: non-finite"
    err = rel_fro(got, want)
    assert err <= tol, f"{what}: relative Frobenius error {err:.3e} > {tol:.1e}"
    return err


def oracle_dims(wl, gelu_exact=False, softmax_scale=0.0, ln_eps=1e-5):
    return oracle.Dims(wl.hidden, wl.heads, wl.head_dim, wl.ffn, wl.seq, wl.micro_batch,
                       gelu_exact=gelu_exact, ln_eps=ln_eps, softmax_scale=softmax_scale)


def params_np(w):
    return {k: to_np(v) for k, v in w.items()}


def dev(t):
    return t.to("cuda").contiguous()
