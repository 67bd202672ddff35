"""Parity at the benchmark's full sizes (MT-NLG per-GPU slice: h 20480, 16 heads x 160, FFN 10240,
seq 2048), in the launch configuration bench.py times.

The fp64 oracle cannot run the full problem in seconds, so:
* the whole layer is checked on a causal prefix: with the upstream gradient zero beyond the first n0
  tokens, rows < n0 of y, all of dx and every weight gradient equal the n0-token problem with the
  full-width weights (causality), which the oracle computes exactly;
* every kernel is checked at its full launch shape on sampled outputs the oracle computes one by one
  from the GPU's own inputs (rows and columns chosen to fall in first / interior / last tiles);
* the 3-layer stage step is checked for determinism and against chained single-layer calls.
"""
import math

import numpy as np
import pytest
import torch

import oracle
import paper_2201_11990_amd as M
from paper_2201_11990_amd import binding as B
from paper_2201_11990_amd.inputs import PARAM_NAMES, WORKLOADS, make_activations, make_layer_params
from paper_2201_11990_amd.runner import LayerRunner, StageRunner
from parity import TOL, assert_close, oracle_dims, rel_fro, to_np

pytestmark = pytest.mark.gpu

WL = WORKLOADS["mtnlg_tp8_stage"]
ROWS = [0, 31, 32, 255, 256, 1023, 1500, 2047]


def test_slice_layer_on_a_causal_prefix():
    wl = WL.with_(n_layers=1)
    n0 = 48
    w = make_layer_params(wl, 0, seed=0, device="cuda", affine="random")
    x, dy = make_activations(wl, seed=0, device="cuda")
    dy[:, n0:] = 0
    run = LayerRunner(wl, w)
    y = run.forward(x)
    dx, grads = run.backward(x, dy)
    torch.cuda.synchronize()
    small = oracle_dims(wl.with_(seq=n0))
    wn = {k: to_np(v) for k, v in w.items()}
    xs, dys = to_np(x[:, :n0]).reshape(n0, -1), to_np(dy[:, :n0]).reshape(n0, -1)
    y_o, saved = oracle.layer_fwd(small, wn, xs)
    dx_o, g_o = oracle.layer_bwd(small, wn, xs, saved, dys)
    tol = TOL["bf16"]
    assert_close(y[:, :n0], y_o, tol, "y[:n0]")
    assert_close(dx[:, :n0], dx_o, tol, "dx[:n0]")
    assert (dx[:, n0:] == 0).all(), "tokens after the prefix must get exactly zero gradient"
    for name in PARAM_NAMES:
        assert_close(grads[name], g_o[name], tol, f"grad {name}")


def _gemm_case(layout, Mm, N, K, epi=0, seed=0):
    g = torch.Generator(device="cuda").manual_seed(seed)
    a_shape = (Mm, K) if layout != B.GEMM_TN else (K, Mm)
    b_shape = (N, K) if layout == B.GEMM_NT else (K, N)
    A = torch.randn(a_shape, generator=g, device="cuda").bfloat16()
    Bm = (torch.randn(b_shape, generator=g, device="cuda") * 0.05).bfloat16()
    bias = torch.randn((N,), generator=g, device="cuda").bfloat16() if epi & B.EPI_BIAS else None
    aux = (torch.randn((Mm, N), generator=g, device="cuda").bfloat16()
           if epi & (B.EPI_RESIDUAL | B.EPI_GELU | B.EPI_GELU_GRAD) else None)
    if epi & B.EPI_ACCUMULATE:  # the micro-batch loop's weight-gradient form: fp32 buffer, added to
        C = torch.randn((Mm, N), generator=g, device="cuda", dtype=torch.float32 if epi & B.EPI_OUT_F32 else torch.bfloat16)
        before = C.clone()
    else:
        C = torch.full((Mm, N), float("nan"), dtype=torch.bfloat16, device="cuda")
    res = aux.clone() if epi & (B.EPI_RESIDUAL | B.EPI_GELU_GRAD) else None
    need = M.mtnlg_gemm_workspace(B.BF16, layout, Mm, N, K)
    ws = torch.empty(need, dtype=torch.uint8, device="cuda") if need else None
    M.mtnlg_gemm(layout, A, Bm, C, bias=bias, aux=aux, epilogue=epi, workspace=ws)
    # first / interior / last tiles, and both sides of the 64-, 80-, 256- and 320-column seams of the tile shapes
    rows = sorted({r for r in (0, 1, 127, 128, 255, 256, Mm // 2 + 3, Mm - 129, Mm - 1)})
    cols = sorted({c for c in (0, 7, 63, 64, 79, 80, 255, 256, 319, 320, 639, 640, N // 2 + 5, N - 321, N - 257, N - 1)})
    # operand rows / columns of the samples are picked on the device: the whole operands need not cross to the host
    if layout == B.GEMM_NT:
        want = oracle.linear_fwd(to_np(A[rows]), to_np(Bm[cols]), to_np(bias)[cols] if bias is not None else None)
    elif layout == B.GEMM_NN:
        want = oracle.linear_dgrad(to_np(A[rows]), to_np(Bm[:, cols]))
    else:
        want = oracle.linear_wgrad(to_np(A[:, rows]), to_np(Bm[:, cols]))[0]
    if epi & B.EPI_GELU:
        assert_close(aux[rows][:, cols], want, TOL["bf16"], "pre-activation samples")
        want = oracle.gelu(want)
    if epi & B.EPI_RESIDUAL:
        want = want + to_np(res)[np.ix_(rows, cols)]
    if epi & B.EPI_GELU_GRAD:
        want = want * oracle.gelu_grad(to_np(res)[np.ix_(rows, cols)])
    if epi & B.EPI_ACCUMULATE:
        want = want + to_np(before)[np.ix_(rows, cols)]
    assert_close(C[rows][:, cols], want, TOL["bf16"], f"gemm {layout} {Mm}x{N}x{K} samples")
    assert torch.isfinite(C.float()).all()


T, H, P, F = WL.tokens, WL.hidden, WL.proj, WL.ffn
FULL_GEMMS = [
    ("qkv", B.GEMM_NT, T, 3 * P, H, B.EPI_BIAS), ("proj", B.GEMM_NT, T, H, P, B.EPI_BIAS | B.EPI_RESIDUAL),
    ("fc1", B.GEMM_NT, T, F, H, B.EPI_BIAS | B.EPI_GELU), ("fc2", B.GEMM_NT, T, H, F, B.EPI_BIAS | B.EPI_RESIDUAL),
    ("dfc2", B.GEMM_NN, T, F, H, 0), ("dfc2_gelu_grad", B.GEMM_NN, T, F, H, B.EPI_GELU_GRAD), ("dfc1", B.GEMM_NN, T, H, F, 0), ("dproj", B.GEMM_NN, T, P, H, 0),
    ("dqkv", B.GEMM_NN, T, H, 3 * P, 0),
    ("wfc2", B.GEMM_TN, H, F, T, 0), ("wfc1", B.GEMM_TN, F, H, T, 0), ("wproj", B.GEMM_TN, H, P, T, 0),
    ("wqkv", B.GEMM_TN, 3 * P, H, T, 0),
    ("wfc1_accumulate_fp32", B.GEMM_TN, F, H, T, B.EPI_ACCUMULATE | B.EPI_OUT_F32),
    # the slice at micro-batch 4 (8192 tokens: four times the rows forward, four times the depth of the weight gradients)
    ("mb4_fc1", B.GEMM_NT, 4 * T, F, H, B.EPI_BIAS | B.EPI_GELU), ("mb4_dqkv", B.GEMM_NN, 4 * T, H, 3 * P, 0),
    ("mb4_wfc2", B.GEMM_TN, H, F, 4 * T, 0), ("mb4_wproj", B.GEMM_TN, H, P, 4 * T, 0),
    # the whole unsliced layer (61440 QKV columns, FFN 81920: operands and outputs beyond 2^31 bytes)
    ("full_qkv", B.GEMM_NT, T, 8 * 3 * P, H, B.EPI_BIAS), ("full_fc2", B.GEMM_NT, T, H, 8 * F, B.EPI_BIAS | B.EPI_RESIDUAL),
    ("full_dfc2", B.GEMM_NN, T, 8 * F, H, 0), ("full_wfc1", B.GEMM_TN, 8 * F, H, T, 0),
    # the 1.3B-shaped layer (h 2048, FFN 8192, 8192 tokens)
    ("1p3b_qkv", B.GEMM_NT, 8192, 6144, 2048, B.EPI_BIAS), ("1p3b_dfc1", B.GEMM_NN, 8192, 2048, 8192, 0),
    ("1p3b_wfc1", B.GEMM_TN, 8192, 2048, 8192, 0),
]


@pytest.mark.parametrize("name,layout,Mm,N,K,epi", FULL_GEMMS, ids=[g[0] for g in FULL_GEMMS])
def test_gemm_at_full_launch_shape_on_sampled_outputs(name, layout, Mm, N, K, epi):
    _gemm_case(layout, Mm, N, K, epi, seed=sum(map(ord, name)))


# (b, s, n, d, heads checked): the benchmark slice; the 1.3B-shaped layer (micro-batch 4, head size 128); the
# whole unsliced layer's 128 heads; a long ragged sequence with an odd number of 64-row blocks at head size 64
FULL_ATTENTION = [(WL.micro_batch, WL.seq, WL.heads, WL.head_dim, (0, 11)), (4, 2048, 16, 128, (5,)),
                  (1, 2048, 128, 160, (127,)), (2, 1990, 3, 64, (2,))]


@pytest.mark.parametrize("b,s,n,d,heads", FULL_ATTENTION, ids=[f"b{c[0]}-s{c[1]}-n{c[2]}-d{c[3]}" for c in FULL_ATTENTION])
def test_attention_at_full_sequence_length_on_sampled_heads(b, s, n, d, heads):
    g = torch.Generator(device="cuda").manual_seed(5)
    qkv = torch.randn((b * s, 3 * n * d), generator=g, device="cuda").bfloat16()
    da = torch.randn((b * s, n * d), generator=g, device="cuda").bfloat16()
    a = torch.full((b * s, n * d), float("nan"), dtype=torch.bfloat16, device="cuda")
    lse = torch.empty((b, n, s), device="cuda")
    scale = 1 / math.sqrt(d)
    M.mtnlg_attention_fwd(b, s, n, d, scale, qkv, a, lse)
    ws = torch.empty(M.mtnlg_attention_bwd_workspace(b, s, n, d), dtype=torch.uint8, device="cuda")
    dqkv = torch.full(qkv.shape, float("nan"), dtype=torch.bfloat16, device="cuda")
    M.mtnlg_attention_bwd(b, s, n, d, scale, qkv, a, lse, da, dqkv, ws)
    assert torch.isfinite(a.float()).all() and torch.isfinite(dqkv.float()).all()
    one = oracle.Dims(hidden=8, heads=1, head_dim=d, ffn=8, seq=s, batch=b)
    for head in heads:
        q1 = to_np(qkv[:, head * 3 * d:(head + 1) * 3 * d])
        da1 = to_np(da[:, head * d:(head + 1) * d])
        assert_close(a[:, head * d:(head + 1) * d], oracle.attention_fwd(one, q1), TOL["bf16"], f"head {head} out")
        want = oracle.attention_bwd(one, q1, da1)
        got = dqkv[:, head * 3 * d:(head + 1) * 3 * d]
        for i, nm in enumerate("qkv"):
            assert_close(got[:, i * d:(i + 1) * d], want[:, i * d:(i + 1) * d], TOL["bf16"], f"head {head} d{nm}")


def test_rowwise_kernels_at_full_width_on_sampled_rows():
    g = torch.Generator(device="cuda").manual_seed(6)
    x = (torch.randn((T, H), generator=g, device="cuda") * 1.5 + 0.2).bfloat16()
    gamma = (1 + 0.1 * torch.randn((H,), generator=g, device="cuda")).bfloat16()
    beta = (0.1 * torch.randn((H,), generator=g, device="cuda")).bfloat16()
    dout = torch.randn((T, H), generator=g, device="cuda").bfloat16()
    out = torch.empty_like(x)
    mean, rstd = torch.empty(T, device="cuda"), torch.empty(T, device="cuda")
    M.mtnlg_layernorm_fwd(x, gamma, beta, 1e-5, out, mean, rstd)
    o_out, o_mean, o_rstd = oracle.layernorm_fwd(to_np(x[ROWS]), to_np(gamma), to_np(beta), 1e-5)
    assert_close(out[ROWS], o_out, TOL["bf16"], "ln rows")
    assert_close(mean[ROWS], o_mean, 1e-5, "ln mean")
    ws = torch.empty(M.mtnlg_layernorm_bwd_workspace(T, H), dtype=torch.uint8, device="cuda")
    dx = torch.empty_like(x)
    dgm, dbt, cs = (torch.empty(H, device="cuda") for _ in range(3))
    M.mtnlg_layernorm_bwd(x, gamma, mean, rstd, dout, dx, dgm, dbt, ws, colsum_dx=cs, grad_f32=True)
    o_dx, _, _ = oracle.layernorm_bwd(to_np(x[ROWS]), to_np(gamma), to_np(mean[ROWS]), to_np(rstd[ROWS]), to_np(dout[ROWS]))
    assert_close(dx[ROWS], o_dx, TOL["bf16"], "ln bwd rows")
    cols = [0, 7, 511, 512, 10000, H - 1]
    xhat = (to_np(x[:, cols]) - to_np(mean)[:, None]) * to_np(rstd)[:, None]
    assert_close(dgm[cols], (to_np(dout[:, cols]) * xhat).sum(0), TOL["bf16"], "dgamma cols")
    assert_close(dbt[cols], to_np(dout[:, cols]).sum(0), TOL["bf16"], "dbeta cols")
    assert_close(cs[cols], to_np(dx[:, cols]).sum(0), TOL["bf16"], "colsum(dx) cols")
    z = torch.randn((T, F), generator=g, device="cuda").bfloat16()
    dz = torch.empty_like(z)
    M.mtnlg_gelu_bwd(z, dout[:, :F].contiguous(), dz)
    assert_close(dz[ROWS], to_np(dout[ROWS][:, :F]) * oracle.gelu_grad(to_np(z[ROWS])), TOL["bf16"], "gelu bwd rows")


def test_stage_step_in_the_benchmark_configuration_is_deterministic_and_chains_layers():
    wl = WL
    ws = [make_layer_params(wl, l, seed=0, device="cuda") for l in range(wl.n_layers)]
    x, dy = make_activations(wl, seed=0, device="cuda")
    run = StageRunner(wl, ws)
    y, dx, grads = run.step(x, dy)
    y1, dx1 = y.clone(), dx.clone()
    g1 = [{k: v.clone() for k, v in g.items()} for g in grads]
    y2, dx2, grads2 = run.step(x, dy)
    assert torch.isfinite(y2.float()).all() and torch.isfinite(dx2.float()).all()
    assert torch.equal(y1, y2) and torch.equal(dx1, dx2)
    for l in range(wl.n_layers):
        for k in PARAM_NAMES:
            assert torch.equal(g1[l][k], grads2[l][k]), (l, k)
            assert torch.isfinite(grads2[l][k].float()).all()
    del run, grads, grads2
    # chained single-layer calls give the same bits
    cur, inputs = x, []
    runners = []
    for l in range(wl.n_layers):
        r = LayerRunner(wl, ws[l])
        inputs.append(cur)
        cur = r.forward(cur).clone()
        runners.append(r)
    assert torch.equal(cur, y1)
    gcur = dy
    for l in reversed(range(wl.n_layers)):
        d, g = runners[l].backward(inputs[l], gcur)
        gcur = d.clone()
        for k in ("w_qkv", "w_fc2", "ln1_g", "b_fc1"):
            assert torch.equal(g[k], g1[l][k]), (l, k)
    assert torch.equal(gcur, dx1)
    # a recomputing step returns the same bits as well
    rec = StageRunner(wl, ws, flags=B.RECOMPUTE)
    y3, dx3, g3 = rec.step(x, dy)
    assert torch.equal(y3, y1) and torch.equal(dx3, dx1)
    assert all(torch.equal(g3[0][k], g1[0][k]) for k in PARAM_NAMES)


VOCAB_LOCAL = 6400   # GPT-2's 50257-entry vocabulary padded to 51200, one of 8 slices (the paper gives no size)


def test_lm_head_at_full_width_on_a_token_prefix():
    """With the loss weights zero beyond the first n0 tokens, loss[:n0], dx[:n0], the LayerNorm gradients and dE are
    exactly those of the n0-token problem (token rows are independent up to the sums over tokens), which the oracle
    computes with the full-width E slice; the GPU runs all T = 2048 tokens in the shape bench.py times."""
    n0, T, h, Vl = 24, WL.tokens, WL.hidden, VOCAB_LOCAL
    g = torch.Generator(device="cuda").manual_seed(7)
    x = torch.randn((T, h), generator=g, device="cuda").bfloat16()
    gamma = (torch.randn(h, generator=g, device="cuda") * 0.2 + 1.0).bfloat16()
    beta = (torch.randn(h, generator=g, device="cuda") * 0.1).bfloat16()
    E = (torch.randn((Vl, h), generator=g, device="cuda") * 0.004).bfloat16()
    targets = torch.randint(0, Vl, (T,), generator=g, device="cuda", dtype=torch.int32)
    dloss = torch.zeros(T, device="cuda")
    dloss[:n0] = torch.rand(n0, generator=g, device="cuda") + 0.5
    desc = B.head_desc(h, Vl, 0, WL.seq, WL.micro_batch, "bf16")
    ws = torch.empty(M.mtnlg_lm_head_workspace(desc), dtype=torch.uint8, device="cuda")
    loss = torch.empty(T, device="cuda")
    dx, dg, db, dE = torch.empty_like(x), torch.empty_like(gamma), torch.empty_like(beta), torch.empty_like(E)
    M.mtnlg_lm_head_step(desc, x, gamma, beta, E, targets, dloss, loss, dx, dg, db, dE, ws)
    torch.cuda.synchronize()
    want = oracle.lm_head_step(to_np(x[:n0]), to_np(gamma), to_np(beta), to_np(E), targets[:n0].cpu().numpy(),
                               to_np(dloss[:n0]))
    assert np.abs(to_np(loss[:n0]) - want[0]).max() <= 3e-2
    assert torch.isfinite(loss).all() and (loss > 0).all()
    tol = TOL["bf16"]
    assert_close(dx[:n0], want[1], tol, "dx[:n0]")
    assert (dx[n0:] == 0).all(), "tokens with zero loss weight get exactly zero gradient"
    assert_close(dg, want[2], tol, "dgamma")
    assert_close(db, want[3], tol, "dbeta")
    assert_close(dE, want[4], tol, "dE")


# ---- the other named workloads at their full sizes ---------------------------------------------------------------

def _prefix_inputs(wl, n0, seed=0):
    x, dy = make_activations(wl, seed=seed, device="cuda")
    dy[:, n0:] = 0
    return x, dy


def _prefix_np(t, n0):
    """First n0 tokens of every sequence, as the oracle's [b * n0, h] fp64 array."""
    return to_np(t[:, :n0]).reshape(t.shape[0] * n0, -1)


def test_gpt1p3b_layer_on_causal_prefixes_of_four_sequences():
    """1.3B-shaped unsliced layer, micro-batch 4 (T = 8192): each of the four sequences keeps only its first n0
    upstream-gradient rows, so the oracle's b = 4, s = n0 problem fixes y[:, :n0], all of dx and every parameter
    gradient of the full launch."""
    wl, n0 = WORKLOADS["gpt1p3b_layer"], 96
    w = make_layer_params(wl, 0, seed=0, device="cuda", affine="random")
    x, dy = _prefix_inputs(wl, n0)
    run = LayerRunner(wl, w)
    y = run.forward(x)
    dx, grads = run.backward(x, dy)
    torch.cuda.synchronize()
    small = oracle_dims(wl.with_(seq=n0))
    wn = {k: to_np(v) for k, v in w.items()}
    xs = _prefix_np(x, n0)
    y_o, saved = oracle.layer_fwd(small, wn, xs)
    dx_o, g_o = oracle.layer_bwd(small, wn, xs, saved, _prefix_np(dy, n0))
    tol = TOL["bf16"]
    assert_close(y[:, :n0], y_o, tol, "y[:, :n0]")
    assert_close(dx[:, :n0], dx_o, tol, "dx[:, :n0]")
    assert (dx[:, n0:] == 0).all()
    for name in PARAM_NAMES:
        assert_close(grads[name], g_o[name], tol, f"grad {name}")


def test_recomputing_stage_at_micro_batch_four_on_causal_prefixes():
    """Three slice layers, micro-batch 4, activations recomputed inside backward: the stage step's y, dx and the
    36 parameter gradients against the oracle's three-layer stack on the prefixes, and bit for bit against the
    same step with all activations kept."""
    wl, n0 = WORKLOADS["mtnlg_tp8_stage_mb4_recompute"], 12
    assert wl.recompute and wl.micro_batch == 4
    ws = [make_layer_params(wl, l, seed=0, device="cuda", affine="random") for l in range(wl.n_layers)]
    x, dy = _prefix_inputs(wl, n0)
    rec = StageRunner(wl, ws)
    assert rec.desc.flags & B.RECOMPUTE
    y, dx, grads = rec.step(x, dy)
    torch.cuda.synchronize()
    y_o, dx_o, g_o = oracle.stage_step(oracle_dims(wl.with_(seq=n0)), [{k: to_np(v) for k, v in w.items()} for w in ws],
                                       _prefix_np(x, n0), _prefix_np(dy, n0))
    tol = TOL["bf16"]
    assert_close(y[:, :n0], y_o, tol, "y[:, :n0]")
    assert_close(dx[:, :n0], dx_o, tol, "dx[:, :n0]")
    assert (dx[:, n0:] == 0).all()
    for l in range(wl.n_layers):
        for name in PARAM_NAMES:
            assert_close(grads[l][name], g_o[l][name], tol, f"layer {l} grad {name}")
    del y_o, dx_o, g_o
    keep = StageRunner(wl.with_(recompute=False), ws)
    assert keep.saved.numel() > rec.saved.numel()
    y2, dx2, grads2 = keep.step(x, dy)
    assert torch.equal(y, y2) and torch.equal(dx, dx2)
    for l in range(wl.n_layers):
        for name in PARAM_NAMES:
            assert torch.equal(grads[l][name], grads2[l][name]), (l, name)


@pytest.mark.timeout(900)
def test_whole_unsliced_mtnlg_layer_on_a_causal_prefix():
    """One full layer (h 20480, 128 heads x 160, FFN 81920: 5.0e9 parameters, 10 GB in bf16) on one GPU.  The oracle
    takes the same weights in fp64 on the first n0 tokens; tensors are compared and released one at a time to bound
    host memory (the fp64 weights alone are 40 GB)."""
    wl, n0 = WORKLOADS["mtnlg_full_layer"], 16
    w = make_layer_params(wl, 0, seed=0, device="cuda", affine="random")
    x, dy = _prefix_inputs(wl, n0)
    run = LayerRunner(wl, w)
    y = run.forward(x)
    dx, grads = run.backward(x, dy)
    torch.cuda.synchronize()
    small = oracle_dims(wl.with_(seq=n0))
    wn = {k: to_np(v) for k, v in w.items()}
    xs = _prefix_np(x, n0)
    y_o, saved = oracle.layer_fwd(small, wn, xs)
    dx_o, g_o = oracle.layer_bwd(small, wn, xs, saved, _prefix_np(dy, n0))
    del wn, saved
    tol = TOL["bf16"]
    assert_close(y[:, :n0], y_o, tol, "y[:n0]")
    assert_close(dx[:, :n0], dx_o, tol, "dx[:n0]")
    assert (dx[:, n0:] == 0).all()
    for name in PARAM_NAMES:
        assert_close(grads[name], g_o.pop(name), tol, f"grad {name}")


@pytest.mark.parametrize("count", [WL.ffn * WL.hidden, (1 << 31) + 7], ids=["fc1_slice", "beyond_2_31_elements"])
def test_optimizer_step_at_full_tensor_sizes(count):
    """The squared norm over the whole tensor against the oracle (converted in chunks) and one clipped Adam update
    on sampled elements (the update is elementwise): first and last elements, the 2^31 boundary, 200000 at random."""
    g = torch.Generator(device="cuda").manual_seed(11)
    p = torch.randn(count, generator=g, device="cuda") * 0.004
    m = torch.randn(count, generator=g, device="cuda") * 1e-3
    v = torch.rand(count, generator=g, device="cuda") * 1e-6
    grad = torch.randn(count, generator=g, device="cuda") * 0.01
    w16 = torch.empty(count, dtype=torch.bfloat16, device="cuda")
    near = torch.arange(-8, 8, device="cuda") + min(count - 9, 1 << 31)
    idx = torch.cat([torch.arange(0, 1024, device="cuda"), torch.arange(count - 1031, count, device="cuda"), near,
                     torch.randint(0, count, (200000,), generator=g, device="cuda")])
    before = [to_np(t[idx]) for t in (p, m, v, grad)]
    ws = torch.empty(M.mtnlg_grad_sqnorm_workspace(), dtype=torch.uint8, device="cuda")
    sq = torch.full((1,), float("nan"), device="cuda")
    M.mtnlg_grad_sqnorm(grad, ws, sq)
    want_sq = sum(oracle.grad_sqnorm([to_np(c)]) for c in grad.split(1 << 26))
    assert abs(float(sq) - want_sq) <= 1e-6 * want_sq
    coef = oracle.clip_coefficient(want_sq, 1.0)
    assert coef < 1.0
    M.mtnlg_adam_step(p, m, v, grad, w16, sq, lr=1e-3, step=3, weight_decay=0.1)
    want = oracle.adam_step(*before, lr=1e-3, beta1=0.9, beta2=0.95, eps=1e-8, weight_decay=0.1, step=3, clip_coef=coef)
    for name, got, ref in zip(("weight", "m", "v"), (p, m, v), want):
        err = np.abs(to_np(got[idx]) - ref).max()
        assert err <= 2e-6 * np.abs(ref).max(), (name, err)
    for lo in range(0, count, 1 << 28):   # every bf16 weight is the rounded fp32 weight
        assert torch.equal(w16[lo:lo + (1 << 28)], p[lo:lo + (1 << 28)].to(torch.bfloat16))


@pytest.mark.parametrize("b", [1, 4], ids=["micro_batch_1", "micro_batch_4"])
def test_embedding_at_full_width(b):
    """Token and position embedding of the first stage at h 20480, 6400 vocabulary rows of this slice (block 3 of 8),
    sequence 2048; about one token in eight belongs to the slice, a few ids repeat many times."""
    s, h, Vl, vs = WL.seq, WL.hidden, VOCAB_LOCAL, 3 * VOCAB_LOCAL
    T = b * s
    g = torch.Generator(device="cuda").manual_seed(13 + b)
    E = (torch.randn((Vl, h), generator=g, device="cuda") * 0.02).bfloat16()
    P = (torch.randn((s, h), generator=g, device="cuda") * 0.02).bfloat16()
    tokens = torch.randint(0, 8 * Vl, (T,), generator=g, device="cuda", dtype=torch.int32)
    tokens[::37] = vs + 5          # a frequent token of this slice
    tokens[-1], tokens[0] = vs, vs + Vl - 1   # the first and the last row of the block
    desc = B.head_desc(h, Vl, vs, s, b, "bf16")
    x = torch.full((T, h), float("nan"), dtype=torch.bfloat16, device="cuda")
    M.mtnlg_embedding_fwd(desc, tokens, E, P, x)
    tok = tokens.cpu().numpy()
    assert_close(x, oracle.embedding_fwd(tok, to_np(E), to_np(P), s, vs), TOL["bf16"], "embedding")
    dx = torch.randn((T, h), generator=g, device="cuda").bfloat16()
    dE = torch.full((Vl, h), float("nan"), dtype=torch.bfloat16, device="cuda")
    dP = torch.full((s, h), float("nan"), dtype=torch.bfloat16, device="cuda")
    M.mtnlg_embedding_bwd(desc, tokens, dx, dE, dP)
    dE_o, dP_o = oracle.embedding_bwd(tok, to_np(dx), Vl, s, vs)
    assert_close(dE, dE_o, TOL["bf16"], "dE")
    assert_close(dP, dP_o, TOL["bf16"], "dP")
    untouched = torch.ones(Vl, dtype=torch.bool, device="cuda")
    mine = tokens[(tokens >= vs) & (tokens < vs + Vl)].long() - vs
    untouched[mine] = False
    assert (dE[untouched] == 0).all(), "rows of tokens that do not occur get exactly zero gradient"


def test_micro_batch_loop_at_full_size_on_causal_prefixes():
    """Two micro-batches through the 3-layer slice with fp32 gradient buffers (mtnlg_stage_step_accumulate, the
    shape bench.py --micro-batches times): each micro-batch's y and dx and the gradients summed over both against
    the oracle's prefix problems."""
    wl, n0, k = WL, 12, 2
    ws = [make_layer_params(wl, l, seed=0, device="cuda", affine="random") for l in range(wl.n_layers)]
    acts = [_prefix_inputs(wl, n0, seed=20 + m) for m in range(k)]
    xs, dys = torch.stack([a[0] for a in acts]), torch.stack([a[1] for a in acts])
    run = StageRunner(wl, ws, flags=B.WGRAD_FP32)
    ys, dxs, grads = run.step_accumulate(xs, dys)
    torch.cuda.synchronize()
    assert grads[0]["w_fc1"].dtype == torch.float32
    dims = oracle_dims(wl.with_(seq=n0))
    wn = [{name: to_np(v) for name, v in w.items()} for w in ws]
    tol = TOL["bf16"]
    total = None
    for m in range(k):
        y_o, dx_o, g_o = oracle.stage_step(dims, wn, _prefix_np(xs[m], n0), _prefix_np(dys[m], n0))
        assert_close(ys[m][:, :n0], y_o, tol, f"micro-batch {m} y[:, :n0]")
        assert_close(dxs[m][:, :n0], dx_o, tol, f"micro-batch {m} dx[:, :n0]")
        assert (dxs[m][:, n0:] == 0).all()
        total = g_o if total is None else [{name: a[name] + b_[name] for name in PARAM_NAMES} for a, b_ in zip(total, g_o)]
    for l in range(wl.n_layers):
        for name in PARAM_NAMES:
            assert_close(grads[l][name], total[l][name], tol, f"layer {l} summed grad {name}")
