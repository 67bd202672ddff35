"""Kernel-level parity on the GPU: each exported operation against the oracle's matching piece,
element by element, on shapes that span several tiles and leave a ragged tail."""
import math

import numpy as np
import pytest
import torch

import oracle
import paper_2201_11990_amd as M
from paper_2201_11990_amd import binding as B
from parity import TOL, assert_close, dev, rel_fro, to_np

pytestmark = pytest.mark.gpu
DT = {"fp32": torch.float32, "bf16": torch.bfloat16}


def randn(shape, dtype, seed, scale=1.0):
    g = torch.Generator().manual_seed(seed)
    return (torch.randn(shape, generator=g) * scale).to(DT[dtype])


def gemm_oracle(layout, A, Bm, bias=None):
    A, Bm = to_np(A), to_np(Bm)
    if layout == B.GEMM_NT:
        return oracle.linear_fwd(A, Bm, to_np(bias) if bias is not None else None)
    if layout == B.GEMM_NN:
        return oracle.linear_dgrad(A, Bm)
    return oracle.linear_wgrad(A, Bm)[0]


GEMM_SHAPES = [(64, 64, 64), (200, 136, 88), (264, 520, 328), (37, 53, 29), (8, 8, 8), (1000, 24, 4104),
               (520, 776, 2056)]


@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
@pytest.mark.parametrize("layout", [B.GEMM_NT, B.GEMM_NN, B.GEMM_TN])
@pytest.mark.parametrize("shape", GEMM_SHAPES)
def test_gemm_plain(dtype, layout, shape):
    Mm, N, K = shape
    a_shape = (Mm, K) if layout != B.GEMM_TN else (K, Mm)
    b_shape = (N, K) if layout == B.GEMM_NT else (K, N)
    A, Bm = randn(a_shape, dtype, 1), randn(b_shape, dtype, 2)
    C = torch.full((Mm, N), float("nan"), dtype=DT[dtype], device="cuda")
    M.mtnlg_gemm(layout, dev(A), dev(Bm), C)
    assert_close(C, gemm_oracle(layout, A, Bm), TOL[dtype], f"gemm {layout} {shape}")


# Aligned shapes that take the streaming kernel whole, every element against the oracle: one and several slabs of K
# (the DMA ring's prologue and its clamped look-ahead), one and several tiles of both tile widths (N a multiple of
# 320 takes the 256 x 320 tile in all three forms), several row tiles.
STREAM_SHAPES = [(256, 320, 64), (256, 640, 128), (512, 320, 192), (256, 256, 64), (512, 512, 128), (768, 960, 256)]


@pytest.mark.parametrize("layout", [B.GEMM_NT, B.GEMM_NN, B.GEMM_TN])
@pytest.mark.parametrize("shape", STREAM_SHAPES)
def test_gemm_streaming_kernel_small_aligned_shapes(layout, shape):
    Mm, N, K = shape
    a_shape = (Mm, K) if layout != B.GEMM_TN else (K, Mm)
    b_shape = (N, K) if layout == B.GEMM_NT else (K, N)
    A, Bm = randn(a_shape, "bf16", 11), randn(b_shape, "bf16", 12, 0.3)
    bias, res = randn((N,), "bf16", 13), randn((Mm, N), "bf16", 14)
    want = gemm_oracle(layout, A, Bm)
    C = torch.full((Mm, N), float("nan"), dtype=torch.bfloat16, device="cuda")
    M.mtnlg_gemm(layout, dev(A), dev(Bm), C)
    assert_close(C, want, TOL["bf16"], f"stream {layout} {shape}")
    # the epilogue that goes through fp32 (bias + residual), and fp32 output
    C.fill_(float("nan"))
    M.mtnlg_gemm(layout, dev(A), dev(Bm), C, bias=dev(bias), aux=dev(res), epilogue=B.EPI_BIAS | B.EPI_RESIDUAL)
    assert_close(C, want + to_np(bias) + to_np(res), TOL["bf16"], f"stream {layout} {shape} bias+residual")
    C32 = torch.full((Mm, N), float("nan"), dtype=torch.float32, device="cuda")
    M.mtnlg_gemm(layout, dev(A), dev(Bm), C32, epilogue=B.EPI_OUT_F32)
    assert_close(C32, want, TOL["fp32"], f"stream {layout} {shape} f32 out")


@pytest.mark.parametrize("shape", [(256, 320, 128), (512, 256, 64), (264, 520, 328)])
def test_gemm_fused_activation_backward_at_fp32_accuracy(shape):
    """The MFMA GEMMs evaluate GeLU and GeLU' through the hardware exp2 and reciprocal (s = 1 / (1 + exp(-2u))) rather
    than the library tanh.  With fp32 output nothing is rounded to bf16 after the activation's derivative, so the
    product times GeLU'(aux) has to meet the fp32 bar: that pins the fast form to a few 1e-7, four orders below
    what the bf16 cases can see.  aux spans the whole range, including very negative values where 1 + tanh cancels."""
    Mm, N, K = shape
    A, W = randn((Mm, K), "bf16", 91), randn((N, K), "bf16", 92, 0.2)
    z = (torch.linspace(-14.0, 14.0, Mm * N).reshape(Mm, N) + randn((Mm, N), "bf16", 93, 0.5).float()).bfloat16()
    C32 = torch.full((Mm, N), float("nan"), dtype=torch.float32, device="cuda")
    M.mtnlg_gemm(B.GEMM_NT, dev(A), dev(W), C32, aux=dev(z), epilogue=B.EPI_GELU_GRAD | B.EPI_OUT_F32)
    want = gemm_oracle(B.GEMM_NT, A, W) * oracle.gelu_grad(to_np(z))
    assert_close(C32, want, TOL["fp32"], f"gelu grad f32 out {shape}")


@pytest.mark.parametrize("layout", [B.GEMM_NT, B.GEMM_NN, B.GEMM_TN])
@pytest.mark.parametrize("shape", [(520, 776, 4104), (256, 512, 2048)])
def test_gemm_split_k_tail_with_workspace(layout, shape):
    """Few output tiles and a long K: with workspace the tiles are split along K and summed by a
    second kernel; the result must match the oracle and, bit for bit in bf16 terms, stay within
    tolerance of the unsplit run."""
    Mm, N, K = shape
    a_shape = (Mm, K) if layout != B.GEMM_TN else (K, Mm)
    b_shape = (N, K) if layout == B.GEMM_NT else (K, N)
    A, Bm = randn(a_shape, "bf16", 40), randn(b_shape, "bf16", 41, 0.1)
    bias, res = randn((N,), "bf16", 42), randn((Mm, N), "bf16", 43)
    need = M.mtnlg_gemm_workspace(B.BF16, layout, Mm, N, K)
    assert need > 0
    ws = torch.empty(need, dtype=torch.uint8, device="cuda")
    want = gemm_oracle(layout, A, Bm) + to_np(bias) + to_np(res)
    for workspace in (ws, None):
        C = torch.full((Mm, N), float("nan"), dtype=torch.bfloat16, device="cuda")
        M.mtnlg_gemm(layout, dev(A), dev(Bm), C, bias=dev(bias), aux=dev(res), epilogue=B.EPI_BIAS | B.EPI_RESIDUAL,
                     workspace=workspace)
        assert_close(C, want, TOL["bf16"], f"split-k {layout} {shape} ws={workspace is not None}")
    # fp32 accumulate into an existing buffer through the split path
    C32 = dev(res).float().contiguous()
    M.mtnlg_gemm(layout, dev(A), dev(Bm), C32, epilogue=B.EPI_ACCUMULATE | B.EPI_OUT_F32, workspace=ws)
    assert_close(C32, gemm_oracle(layout, A, Bm) + to_np(res), TOL["fp32"], "split-k fp32 accumulate")   # fp32 out of exact bf16 products


@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
@pytest.mark.parametrize("shape", [(200, 136, 88), (264, 520, 328), (45, 27, 19)])
def test_gemm_epilogues(dtype, shape):
    Mm, N, K = shape
    tol = TOL[dtype]
    A, W, bias, res = randn((Mm, K), dtype, 3), randn((N, K), dtype, 4, 0.2), randn((N,), dtype, 5), randn((Mm, N), dtype, 6)
    want = gemm_oracle(B.GEMM_NT, A, W, bias)
    dA, dW, dbias, dres = map(dev, (A, W, bias, res))
    # bias
    C = torch.empty((Mm, N), dtype=DT[dtype], device="cuda")
    M.mtnlg_gemm(B.GEMM_NT, dA, dW, C, bias=dbias, epilogue=B.EPI_BIAS)
    assert_close(C, want, tol, "bias")
    # bias + GeLU (both forms): C = GeLU(z), aux = z
    for erf_form in (False, True):
        Z = torch.empty_like(C)
        M.mtnlg_gemm(B.GEMM_NT, dA, dW, C, bias=dbias, aux=Z,
                     epilogue=B.EPI_BIAS | B.EPI_GELU | (B.EPI_GELU_ERF if erf_form else 0))
        assert_close(Z, want, tol, "pre-activation")
        assert_close(C, oracle.gelu(want, exact=erf_form), tol, f"gelu erf={erf_form}")
    # the activation's backward fused into the product: C = (A W^T) o GeLU'(aux), both forms, aux untouched
    for erf_form in (False, True):
        Z = dres.clone()
        M.mtnlg_gemm(B.GEMM_NT, dA, dW, C, aux=Z, epilogue=B.EPI_GELU_GRAD | (B.EPI_GELU_ERF if erf_form else 0))
        assert torch.equal(Z, dres)
        assert_close(C, gemm_oracle(B.GEMM_NT, A, W) * oracle.gelu_grad(to_np(res), exact=erf_form), tol,
                     f"gelu grad erf={erf_form}")
    with pytest.raises(B.MtnlgError):
        M.mtnlg_gemm(B.GEMM_NT, dA, dW, C, bias=dbias, aux=dres, epilogue=B.EPI_GELU_GRAD | B.EPI_BIAS)
    # bias + residual
    M.mtnlg_gemm(B.GEMM_NT, dA, dW, C, bias=dbias, aux=dres, epilogue=B.EPI_BIAS | B.EPI_RESIDUAL)
    assert_close(C, want + to_np(res), tol, "bias+residual")
    # accumulate into an existing buffer, and fp32 output from bf16 inputs
    C.copy_(dres)
    M.mtnlg_gemm(B.GEMM_NT, dA, dW, C, epilogue=B.EPI_ACCUMULATE)
    assert_close(C, gemm_oracle(B.GEMM_NT, A, W) + to_np(res), tol, "accumulate")
    C32 = dres.float().contiguous()
    M.mtnlg_gemm(B.GEMM_NT, dA, dW, C32, epilogue=B.EPI_ACCUMULATE | B.EPI_OUT_F32)
    assert_close(C32, gemm_oracle(B.GEMM_NT, A, W) + to_np(res), TOL["fp32"], "acc f32")   # fp32 output of exact products: the fp32 bar on both paths
    C32.fill_(float("nan"))
    M.mtnlg_gemm(B.GEMM_TN, dev(randn((K, Mm), dtype, 7)), dev(randn((K, N), dtype, 8)), C32, epilogue=B.EPI_OUT_F32)
    assert_close(C32, gemm_oracle(B.GEMM_TN, randn((K, Mm), dtype, 7), randn((K, N), dtype, 8)), 1e-5, "tn f32 out")


@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
@pytest.mark.parametrize("T,h", [(5, 256), (33, 2056), (7, 20480), (3, 8)])
def test_layernorm_fwd_bwd(dtype, T, h):
    tol = TOL[dtype]
    x = randn((T, h), dtype, 10, 2.0) + 0.5
    x = x.to(DT[dtype])
    gamma, beta = (1 + randn((h,), dtype, 11, 0.2).float()).to(DT[dtype]), randn((h,), dtype, 12, 0.2)
    dout, dres = randn((T, h), dtype, 13), randn((T, h), dtype, 14)
    out = torch.empty((T, h), dtype=DT[dtype], device="cuda")
    mean, rstd = torch.empty(T, device="cuda"), torch.empty(T, device="cuda")
    M.mtnlg_layernorm_fwd(dev(x), dev(gamma), dev(beta), 1e-5, out, mean, rstd)
    o_out, o_mean, o_rstd = oracle.layernorm_fwd(to_np(x), to_np(gamma), to_np(beta), 1e-5)
    assert_close(out, o_out, tol, "ln out")
    assert_close(mean, o_mean, 1e-5, "ln mean")
    assert_close(rstd, o_rstd, 1e-5, "ln rstd")
    # fused x + partial + bias
    partial, bias = randn((T, h), dtype, 15), randn((h,), dtype, 16)
    xsum = torch.empty_like(out)
    M.mtnlg_layernorm_fwd(dev(x), dev(gamma), dev(beta), 1e-5, out, mean, rstd, partial=dev(partial), bias=dev(bias), xsum=xsum)
    s = to_np(x) + to_np(partial) + to_np(bias)
    assert_close(xsum, s, tol, "xsum")
    assert_close(out, oracle.layernorm_fwd(s, to_np(gamma), to_np(beta), 1e-5)[0], tol, "ln(xsum)")
    # backward with the oracle's stats on the original x
    ws = torch.empty(M.mtnlg_layernorm_bwd_workspace(T, h), dtype=torch.uint8, device="cuda")
    dx = torch.empty_like(out)
    gdt = torch.float32
    dgamma, dbeta, cs = (torch.full((h,), float("nan"), dtype=gdt, device="cuda") for _ in range(3))
    M.mtnlg_layernorm_bwd(dev(x), dev(gamma), dev(torch.tensor(o_mean, dtype=torch.float32)),
                          dev(torch.tensor(o_rstd, dtype=torch.float32)), dev(dout), dx, dgamma, dbeta, ws,
                          dres=dev(dres), colsum_dx=cs, grad_f32=True)
    o_dx, o_dg, o_db = oracle.layernorm_bwd(to_np(x), to_np(gamma), o_mean, o_rstd, to_np(dout))
    assert_close(dx, o_dx + to_np(dres), tol, "ln dx")
    assert_close(dgamma, o_dg, tol, "ln dgamma")
    assert_close(dbeta, o_db, tol, "ln dbeta")
    assert_close(cs, to_np(dx).sum(0), tol, "colsum dx")
    # accumulate on top
    M.mtnlg_layernorm_bwd(dev(x), dev(gamma), dev(torch.tensor(o_mean, dtype=torch.float32)),
                          dev(torch.tensor(o_rstd, dtype=torch.float32)), dev(dout), dx, dgamma, dbeta, ws,
                          grad_f32=True, accumulate=True)
    assert_close(dgamma, 2 * o_dg, tol, "ln dgamma accumulated")
    assert_close(dx, o_dx, tol, "ln dx without residual")


@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
def test_layernorm_rows_with_large_mean_or_no_spread(dtype):
    """Rows whose mean is a hundred times their spread (a sum-of-squares variance would lose them in fp32), a row
    of tiny values (eps dominates the variance) and a constant row (variance exactly 0: the output is beta)."""
    T, h = 6, 2056
    g = torch.Generator().manual_seed(91)
    x = torch.randn((T, h), generator=g)
    x[0] = 6.0 + 0.05 * x[0]
    x[1] = -40.0 + 0.3 * x[1]
    x[2] = 1e-4 * x[2]
    x[3] = 3.25
    x = x.to(DT[dtype])
    gamma, beta = (1 + randn((h,), dtype, 92, 0.2).float()).to(DT[dtype]), randn((h,), dtype, 93, 0.2)
    out = torch.empty((T, h), dtype=DT[dtype], device="cuda")
    mean, rstd = torch.empty(T, device="cuda"), torch.empty(T, device="cuda")
    M.mtnlg_layernorm_fwd(dev(x), dev(gamma), dev(beta), 1e-5, out, mean, rstd)
    o_out, o_mean, o_rstd = oracle.layernorm_fwd(to_np(x), to_np(gamma), to_np(beta), 1e-5)
    for t in range(T):
        assert_close(out[t], o_out[t], TOL[dtype], f"row {t} out")
    assert np.abs(to_np(rstd) / o_rstd - 1).max() <= 2e-5
    assert torch.equal(out[3].cpu(), beta.to(DT[dtype])), "a constant row normalises to beta exactly"
    dout = randn((T, h), dtype, 94)
    ws = torch.empty(M.mtnlg_layernorm_bwd_workspace(T, h), dtype=torch.uint8, device="cuda")
    dx = torch.empty_like(out)
    dgamma, dbeta = (torch.full((h,), float("nan"), dtype=torch.float32, device="cuda") for _ in range(2))
    M.mtnlg_layernorm_bwd(dev(x), dev(gamma), mean, rstd, dev(dout), dx, dgamma, dbeta, ws, grad_f32=True)
    o_dx, o_dg, o_db = oracle.layernorm_bwd(to_np(x), to_np(gamma), o_mean, o_rstd, to_np(dout))
    # backward runs on the GPU's own fp32 statistics: the mean of the row around -40 carries ~2e-6 of absolute
    # rounding error against a spread of 0.3, i.e. ~1e-5 in xhat, hence three times the fp32 bar
    for t in range(T):
        assert_close(dx[t], o_dx[t], TOL[dtype], f"row {t} dx")
    assert_close(dgamma, o_dg, TOL[dtype], "dgamma")
    assert_close(dbeta, o_db, TOL[dtype], "dbeta")


ATT_CASES = [(2, 40, 3, 64), (1, 130, 2, 128), (2, 77, 2, 160), (1, 1, 1, 8), (1, 300, 1, 32), (1, 257, 2, 160),
             (1, 700, 2, 160), (1, 520, 1, 64), (2, 390, 1, 128)]   # many streamed tiles: the three-stage ring wraps


@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
@pytest.mark.parametrize("b,s,n,d", ATT_CASES)
def test_attention_fwd_bwd(dtype, b, s, n, d):
    tol = TOL[dtype]
    dims = oracle.Dims(hidden=8, heads=n, head_dim=d, ffn=8, seq=s, batch=b)
    qkv = randn((b * s, 3 * n * d), dtype, 20, 1.0)
    da = randn((b * s, n * d), dtype, 21)
    scale = 1.0 / math.sqrt(d)
    a = torch.full((b * s, n * d), float("nan"), dtype=DT[dtype], device="cuda")
    lse = torch.empty((b, n, s), device="cuda")
    M.mtnlg_attention_fwd(b, s, n, d, scale, dev(qkv), a, lse)
    o_a, P = oracle.attention_fwd(dims, to_np(qkv), return_probs=True)
    assert_close(a, o_a, tol, "attention out")
    # log-sum-exp of the scaled masked scores, from the definition
    q = to_np(qkv).reshape(b, s, n, 3, d)
    S = np.einsum("bsnd,btnd->bnst", q[:, :, :, 0], q[:, :, :, 1]) * scale
    S = np.where(np.tril(np.ones((s, s), bool)), S, -np.inf)
    want_lse = np.log(np.exp(S - S.max(-1, keepdims=True)).sum(-1)) + S.max(-1)
    assert np.abs(to_np(lse) - want_lse).max() < 1e-3 + 2e-3 * (dtype == "bf16")
    ws = torch.empty(M.mtnlg_attention_bwd_workspace(b, s, n, d), dtype=torch.uint8, device="cuda")
    dqkv = torch.full(qkv.shape, float("nan"), dtype=DT[dtype], device="cuda")
    M.mtnlg_attention_bwd(b, s, n, d, scale, dev(qkv), a, lse, dev(da), dqkv, ws)
    o_dqkv = oracle.attention_bwd(dims, to_np(qkv), to_np(da))
    assert_close(dqkv, o_dqkv, tol, "attention dqkv")
    got = to_np(dqkv).reshape(b, s, n, 3, d)
    want = o_dqkv.reshape(b, s, n, 3, d)
    for i, nm in enumerate("qkv"):
        assert rel_fro(got[:, :, :, i], want[:, :, :, i]) <= tol, f"d{nm}"


# Enough (sequence block, head, batch) workgroups for the forward kernel to take its 256-rows-per-workgroup shape
# (32 rows per wave) at head sizes 128 and 160: an odd number of 64-row tiles whose last block hangs over the end
# (s 150), an odd number of 128-row blocks, i.e. a middle block alone in its workgroup (s 257, 700 -> 3 and 6 blocks),
# one block only (s 64, s 1), several tiles per block with a ragged end (s 1000).
ATT_WIDE_CASES = [(8, 150, 64, 128), (4, 257, 64, 160), (2, 700, 64, 128), (16, 64, 16, 160), (8, 1, 32, 128),
                  (2, 1000, 32, 160)]


@pytest.mark.parametrize("b,s,n,d", ATT_WIDE_CASES)
def test_attention_forward_with_32_rows_per_wave(b, s, n, d):
    dims = oracle.Dims(hidden=8, heads=n, head_dim=d, ffn=8, seq=s, batch=b)
    qkv = randn((b * s, 3 * n * d), "bf16", 30, 1.0)
    scale = 1.0 / math.sqrt(d)
    a = torch.full((b * s, n * d), float("nan"), dtype=torch.bfloat16, device="cuda")
    lse = torch.full((b, n, s), float("nan"), device="cuda")
    M.mtnlg_attention_fwd(b, s, n, d, scale, dev(qkv), a, lse)
    assert_close(a, oracle.attention_fwd(dims, to_np(qkv)), TOL["bf16"], "attention out")
    q = to_np(qkv).reshape(b, s, n, 3, d)
    S = np.einsum("bsnd,btnd->bnst", q[:, :, :, 0], q[:, :, :, 1]) * scale
    S = np.where(np.tril(np.ones((s, s), bool)), S, -np.inf)
    want_lse = np.log(np.exp(S - S.max(-1, keepdims=True)).sum(-1)) + S.max(-1)
    assert np.abs(to_np(lse) - want_lse).max() < 3e-3
    # the backward kernels read what this forward wrote
    da = randn((b * s, n * d), "bf16", 31)
    ws = torch.empty(M.mtnlg_attention_bwd_workspace(b, s, n, d), dtype=torch.uint8, device="cuda")
    dqkv = torch.full(qkv.shape, float("nan"), dtype=torch.bfloat16, device="cuda")
    M.mtnlg_attention_bwd(b, s, n, d, scale, dev(qkv), a, lse, dev(da), dqkv, ws)
    assert_close(dqkv, oracle.attention_bwd(dims, to_np(qkv), to_np(da)), TOL["bf16"], "attention dqkv")


@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
@pytest.mark.parametrize("kind", ["sharp", "rising", "falling", "constant"])
def test_attention_with_hard_score_patterns(dtype, kind):
    """Score rows that stress the running-maximum bookkeeping of a streamed softmax over several 64-key tiles:
    sharp (scores of std 8: nearly one-hot rows), rising (each later key scores higher: the reference maximum
    moves in every tile), falling (the first key dominates: everything after it underflows towards zero), constant
    (all scores equal: the running mean of v)."""
    b, s, n, d = 1, 330, 2, 64 if dtype == "bf16" else 16
    g = torch.Generator().manual_seed(77)
    q = torch.randn((s, n, d), generator=g)
    k = torch.randn((s, n, d), generator=g)
    v = torch.randn((s, n, d), generator=g)
    ramp = torch.arange(s, dtype=torch.float32)[:, None, None] / 8.0
    if kind == "sharp":
        q, k = q * 2.8, k * 2.8
    elif kind in ("rising", "falling"):
        q = torch.ones((s, n, d)) + 0.1 * q
        k = (ramp if kind == "rising" else -ramp) * torch.ones((s, n, d)) / math.sqrt(d) + 0.1 * k
    else:
        k = torch.zeros((s, n, d))
    qkv = torch.stack([q, k, v], dim=2).reshape(s, 3 * n * d).to(DT[dtype])
    da = randn((s, n * d), dtype, 78)
    dims = oracle.Dims(hidden=8, heads=n, head_dim=d, ffn=8, seq=s, batch=b)
    scale = 1.0 / math.sqrt(d)
    a = torch.full((s, n * d), float("nan"), dtype=DT[dtype], device="cuda")
    lse = torch.empty((b, n, s), device="cuda")
    M.mtnlg_attention_fwd(b, s, n, d, scale, dev(qkv), a, lse)
    assert torch.isfinite(lse).all()
    assert_close(a, oracle.attention_fwd(dims, to_np(qkv)), TOL[dtype], f"{kind} attention out")
    ws = torch.empty(M.mtnlg_attention_bwd_workspace(b, s, n, d), dtype=torch.uint8, device="cuda")
    dqkv = torch.full(qkv.shape, float("nan"), dtype=DT[dtype], device="cuda")
    M.mtnlg_attention_bwd(b, s, n, d, scale, dev(qkv), a, lse, dev(da), dqkv, ws)
    want = oracle.attention_bwd(dims, to_np(qkv), to_np(da)).reshape(s, n, 3, d)
    got = dqkv.reshape(s, n, 3, d)
    # dv is as well conditioned as the output; dq and dk are differences of nearly equal terms when the rows are
    # nearly one-hot, so they are held to the tolerance relative to dv's size as well
    assert_close(got[:, :, 2], want[:, :, 2], TOL[dtype], f"{kind} dv")
    ref = np.linalg.norm(want[:, :, 2])
    for i, nm in ((0, "dq"), (1, "dk")):
        err = np.linalg.norm(to_np(got[:, :, i]) - want[:, :, i])
        assert err <= TOL[dtype] * max(np.linalg.norm(want[:, :, i]), ref), f"{kind} {nm}: {err:.3e}"


@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
def test_gelu_colsum_bias_residual(dtype):
    tol = TOL[dtype]
    z = randn((70, 264), dtype, 30, 2.0)
    dg = randn((70, 264), dtype, 31)
    for form, exact in ((B.GELU_TANH, False), (B.GELU_ERF, True)):
        g = torch.empty(z.shape, dtype=DT[dtype], device="cuda")
        M.mtnlg_gelu_fwd(dev(z), g, gelu=form)
        assert_close(g, oracle.gelu(to_np(z), exact), tol, "gelu")
        dz = torch.empty_like(g)
        M.mtnlg_gelu_bwd(dev(z), dev(dg), dz, gelu=form)
        assert_close(dz, to_np(dg) * oracle.gelu_grad(to_np(z), exact), tol, "gelu bwd")
    for T, C in ((70, 264), (1, 8), (3000, 520), (257, 10240)):
        x = randn((T, C), dtype, 32)
        ws = torch.empty(M.mtnlg_colsum_workspace(T, C), dtype=torch.uint8, device="cuda")
        for odt in (torch.float32, DT[dtype]):
            out = torch.full((C,), float("nan"), dtype=odt, device="cuda")
            M.mtnlg_colsum(dev(x), out, ws)
            assert_close(out, to_np(x).sum(0), tol, f"colsum {T}x{C}")
            M.mtnlg_colsum(dev(x), out, ws, accumulate=True)
            assert_close(out, 2 * to_np(x).sum(0), tol, "colsum accumulate")
    res, part, bias = randn((70, 264), dtype, 33), randn((70, 264), dtype, 34), randn((264,), dtype, 35)
    out = torch.empty((70, 264), dtype=DT[dtype], device="cuda")
    M.mtnlg_bias_residual(dev(res), dev(part), dev(bias), out)
    assert_close(out, to_np(res) + to_np(part) + to_np(bias), tol, "bias_residual")
    M.mtnlg_bias_residual(dev(res), dev(part), None, out)
    assert_close(out, to_np(res) + to_np(part), tol, "residual")




# ---- optimizer step (Section 3.2: Adam, clipping, weight decay; Section 2.1: fp32 copies and states) ----------

@pytest.mark.parametrize("count", [1, 1023, 4096 + 3, 3_000_001])
def test_adam_step_against_the_oracle(count):
    """Three updates of a slice: squared gradient norm (two tensors summed into one scalar), clipped and
    unclipped steps, decaying and non-decaying tensors.  fp32 arithmetic against the fp64 oracle: 2e-6 relative
    on weights and moments; the bf16 weight is exactly the rounded fp32 weight."""
    g = torch.Generator(device="cuda").manual_seed(count)
    p = (torch.randn(count, generator=g, device="cuda") * 0.02).contiguous()
    m, v = torch.zeros_like(p), torch.zeros_like(p)
    w16 = torch.empty(count, dtype=torch.bfloat16, device="cuda")
    other = torch.randn(777, generator=g, device="cuda") * 0.01      # a second tensor of the "model"
    ws = torch.empty(M.mtnlg_grad_sqnorm_workspace(), dtype=torch.uint8, device="cuda")
    sq = torch.full((1,), float("nan"), device="cuda")
    po, mo, vo = to_np(p), to_np(m), to_np(v)
    for step in range(1, 4):
        scale = 5.0 if step != 2 else 1e-3 / math.sqrt(count)          # steps 1, 3 clip; step 2 does not
        grad = (torch.randn(count, generator=g, device="cuda") * scale).contiguous()
        wd = 0.1 if step != 3 else 0.0
        M.mtnlg_grad_sqnorm(grad, ws, sq)
        M.mtnlg_grad_sqnorm(other, ws, sq, accumulate=True)
        want_sq = oracle.grad_sqnorm([to_np(grad), to_np(other)])
        assert abs(float(sq) - want_sq) <= 1e-6 * want_sq
        coef = oracle.clip_coefficient(want_sq, 1.0)
        assert (coef < 1.0) == (step != 2)
        M.mtnlg_adam_step(p, m, v, grad, w16, sq, lr=5e-3, step=step, weight_decay=wd)
        po, mo, vo = oracle.adam_step(po, mo, vo, to_np(grad), lr=5e-3, beta1=0.9, beta2=0.95, eps=1e-8,
                                      weight_decay=wd, step=step, clip_coef=coef)
        for name, got, want in (("weight", p, po), ("m", m, mo), ("v", v, vo)):
            err = np.abs(to_np(got) - want).max()
            assert err <= 2e-6 * np.abs(want).max() + 1e-30, (name, step, err)
        assert torch.equal(w16, p.to(torch.bfloat16)), "bf16 weight is the rounded fp32 weight"
    # without the scalar (or with max_grad_norm <= 0) nothing is clipped
    p2, m2, v2 = p.clone(), m.clone(), v.clone()
    big = torch.full((count,), 100.0, device="cuda")
    M.mtnlg_adam_step(p2, m2, v2, big, None, None, lr=1e-3, step=4)
    pw, mw, vw = oracle.adam_step(to_np(p), to_np(m), to_np(v), to_np(big), lr=1e-3, step=4)
    assert np.abs(to_np(m2) - mw).max() <= 2e-6 * np.abs(mw).max()
    assert np.abs(to_np(p2) - pw).max() <= 2e-6 * np.abs(pw).max()


def test_adam_step_rejects_bad_arguments():
    p = torch.zeros(64, device="cuda")
    with pytest.raises(B.MtnlgError):
        M.mtnlg_adam_step(p, p.clone(), p.clone(), p.clone(), lr=1e-3, step=0)
    with pytest.raises(B.MtnlgError):
        M.mtnlg_adam_step(p, p.clone(), p.clone(), p.clone(), lr=1e-3, step=1, beta2=1.0)
    with pytest.raises(B.MtnlgError):   # misaligned fp32 pointer
        M.mtnlg_adam_step(torch.zeros(33, device="cuda")[1:], torch.zeros(32, device="cuda"),
                          torch.zeros(32, device="cuda"), torch.zeros(32, device="cuda"), lr=1e-3, step=1)
