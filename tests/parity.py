"""Shared helpers of the GPU parity tests: conversions between device tensors and the oracle's
fp64 numpy arrays, and the two error measures every compared tensor has to pass.

1. Relative Frobenius error per output tensor, ||got - want||_F / ||want||_F <= tol, with tol = 1e-2 on the
   bf16 path and 1e-5 on the fp32 path (the stated bar; TOL below).
2. An element-wise complement, because one norm per tensor cannot see a small wrong region (one wrong 16 x 16
   block of a 2048 x 20480 output moves the norm by 2.5e-3): every element must satisfy
       |got - want| <= ELEM_SIGMAS * tol * (scale + |want|),
   scale = the largest of the tensor's rms, the rms of the element's row and the rms of its column (a matrix is
   taken as [everything else, last axis]).  An error field at the bar has an additive part (accumulated roundings
   of the operands: standard deviation tol * scale -- an element of a product inherits the size of the row and of
   the column it is contracted from, and the rows of a weight gradient differ in size by an order of magnitude) and
   a part proportional to the element (roundings of the element itself and of factors it is proportional to:
   relative standard deviation tol).  Were they Gaussian, none of up to 1e9 compared elements would leave 6
   standard deviations of either; they are sums of products of roundings and values, heavier-tailed than that,
   so the allowance is 8.  A misplaced tile or a bad edge row is wrong by about the local rms per element:
   six times the allowance at the bf16 bar.

Every comparison is recorded (test id, tensor, both measures); conftest.py prints the worst ones at the end of a
run and writes the whole table to $MTNLG_PARITY_LOG when that is set.
"""
import os

import numpy as np
import torch

import oracle

# spec tolerances: relative Frobenius error per output tensor
TOL = {"fp32": 1e-5, "bf16": 1e-2}
ELEM_SIGMAS = 8.0

RECORDS = []   # (test id, what, rel_fro, tol, elementwise ratio: worst |diff| / allowance, elements)


def to_np(t):
    return t.detach().to("cpu", torch.float64).numpy()


def _as_rows(a):
    """[everything else, last axis] view of a tensor (a vector is one row)."""
    return a.reshape(1, -1) if a.dim() < 2 else a.reshape(-1, a.shape[-1])


def compare(got, want, tol):
    """(relative Frobenius error, element-wise ratio) of got against want in one chunked pass: the reference is
    fp64 already, the device tensor is widened a block of rows at a time (the largest compared tensors have 1.3e9
    elements); the arithmetic is fp64 on the host's cores.  The ratio is
    max |got - want| / (ELEM_SIGMAS * tol * (scale + |want|)) with scale the largest of the global, row and column
    rms of want; <= 1 passes."""
    g_all = got.detach().cpu() if isinstance(got, torch.Tensor) else torch.from_numpy(np.asarray(got, dtype=np.float64))
    w = torch.from_numpy(np.ascontiguousarray(np.asarray(want, dtype=np.float64).reshape(tuple(g_all.shape))))
    g_all, w = _as_rows(g_all), _as_rows(w)
    if w.numel() == 0:
        return 0.0, 0.0
    R, C = w.shape
    step = max(1, (1 << 23) // C)
    col_sq = torch.zeros(C, dtype=torch.float64)
    row_sq = torch.empty(R, dtype=torch.float64)
    for r0 in range(0, R, step):
        sq = w[r0:r0 + step] ** 2
        col_sq += sq.sum(0)
        row_sq[r0:r0 + step] = sq.sum(1)
    total = float(col_sq.sum())
    rms = (total / w.numel()) ** 0.5
    matrix = R > 1 and C > 1
    col = torch.sqrt(col_sq / R)[None, :] if matrix else torch.zeros((1, C), dtype=torch.float64)
    row = torch.sqrt(row_sq / C)[:, None] if matrix else torch.zeros((R, 1), dtype=torch.float64)
    num, worst = 0.0, 0.0
    for r0 in range(0, R, step):
        sl = slice(r0, r0 + step)
        d = (g_all[sl].to(torch.float64) - w[sl]).abs_()
        num += float((d * d).sum())
        if rms > 0.0:
            local = torch.maximum(torch.maximum(row[sl], col), torch.tensor(rms, dtype=torch.float64))
            d /= (local + w[sl].abs()) * (ELEM_SIGMAS * tol)
            worst = max(worst, float(d.max()))
    if total == 0.0:
        return (0.0, 0.0) if num == 0.0 else (float("inf"), float("inf"))
    return (num / total) ** 0.5, worst


def rel_fro(got, want):
    return compare(got, want, 1.0)[0]


def elementwise_ratio(got, want, tol):
    return compare(got, want, tol)[1]


def assert_close(got, want, tol, what, elementwise=True):
    assert torch.isfinite(got.float()).all() if isinstance(got, torch.Tensor) else True, f"{what}: non-finite"
    err, ratio = compare(got, want, tol)
    if not elementwise:
        ratio = float("nan")
    test = os.environ.get("PYTEST_CURRENT_TEST", "?").split(" ")[0]
    RECORDS.append((test, what, err, tol, ratio, int(np.asarray(want).size)))
    assert err <= tol, f"{what}: relative Frobenius error {err:.3e} > {tol:.1e}"
    if elementwise:
        assert ratio <= 1.0, f"{what}: an element is off by {ratio:.2f} x its allowance (tol {tol:.1e})"
    return err


def poison(run):
    """NaN (all-ones words) in every byte the library writes before it reads -- saved activations, workspace,
    outputs of a LayerRunner / StageRunner: a kernel that reads scratch it has not filled, or leaves a hole in an
    output, then shows up as a non-finite result."""
    for buf in (run.saved, run.workspace):
        buf.view(torch.int32).fill_(-1)      # sizes are multiples of 256 bytes; 0xFFFFFFFF is NaN as bf16 and as float
    run.y.fill_(float("nan"))
    run.dx.fill_(float("nan"))
    return run


def copy_into_pointer(ptr, src):
    """Copy a contiguous device tensor over the device memory at address `ptr` (what an exchange hook does with the
    group's value) and wait for it: src may be freed by the caller right after."""
    import ctypes
    hip = ctypes.CDLL("libamdhip64.so")
    hip.hipMemcpyAsync.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int, ctypes.c_void_p]
    stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    rc = hip.hipMemcpyAsync(ctypes.c_void_p(ptr), ctypes.c_void_p(src.data_ptr()), src.numel() * src.element_size(),
                            3, stream)
    if rc != 0:
        raise RuntimeError(f"hipMemcpyAsync failed: {rc}")
    torch.cuda.current_stream().synchronize()


def oracle_dims(wl, gelu_exact=False, softmax_scale=0.0, ln_eps=1e-5):
    return oracle.Dims(wl.hidden, wl.heads, wl.head_dim, wl.ffn, wl.seq, wl.micro_batch,
                       gelu_exact=gelu_exact, ln_eps=ln_eps, softmax_scale=softmax_scale)


def params_np(w):
    return {k: to_np(v) for k, v in w.items()}


def dev(t):
    return t.to("cuda").contiguous()
