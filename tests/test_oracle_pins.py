"""Pins for the fp64 CPU oracle: it is checked against things other than itself.

* central finite differences of every gradient (non-trivial biases / gamma / beta);
* an independent autograd composition of torch library ops in fp64;
* invariants: softmax rows, causal mask, LayerNorm moments, residual identity;
* causal invariance to future tokens and its dual;
* the tensor-parallel sum identity with 8 slices;
* textbook special cases.
All CPU, no GPU library involved.
"""
import math

import numpy as np
import pytest
import torch
import torch.nn.functional as Fnn

import oracle

PARAMS = ("ln1_g", "ln1_b", "w_qkv", "b_qkv", "w_o", "b_o",
          "ln2_g", "ln2_b", "w_fc1", "b_fc1", "w_fc2", "b_fc2")


def rand_params(dims, rng, w_std=0.2):
    w = {}
    for name, shape in dims.param_shapes().items():
        if name.startswith("w_"):
            w[name] = rng.standard_normal(shape) * w_std
        elif name.endswith("_g"):
            w[name] = 1.0 + 0.3 * rng.standard_normal(shape)
        else:
            w[name] = 0.3 * rng.standard_normal(shape)
    return w


TINY = dict(hidden=32, heads=2, head_dim=16, ffn=64, seq=8, batch=2)


# ------------------------------------------------------------ finite differences
@pytest.mark.parametrize("gelu_exact", [False, True])
def test_gradients_match_central_finite_differences(gelu_exact):
    rng = np.random.default_rng(0)
    dims = oracle.Dims(**TINY, gelu_exact=gelu_exact)
    w = rand_params(dims, rng)
    x = rng.standard_normal((dims.tokens, dims.hidden))
    dy = rng.standard_normal((dims.tokens, dims.hidden))

    def loss(w_, x_):
        y, _ = oracle.layer_fwd(dims, w_, x_)
        return float((y * dy).sum())

    y, saved = oracle.layer_fwd(dims, w, x)
    dx, grads = oracle.layer_bwd(dims, w, x, saved, dy)

    eps = 1e-5
    checked = 0
    for name in ("x",) + PARAMS:
        base = x if name == "x" else w[name]
        analytic = dx if name == "x" else grads[name]
        flat_idx = rng.choice(base.size, size=min(12, base.size), replace=False)
        for fi in flat_idx:
            idx = np.unravel_index(fi, base.shape)
            plus, minus = base.copy(), base.copy()
            plus[idx] += eps
            minus[idx] -= eps
            if name == "x":
                fd = (loss(w, plus) - loss(w, minus)) / (2 * eps)
            else:
                fd = (loss({**w, name: plus}, x) - loss({**w, name: minus}, x)) / (2 * eps)
            an = analytic[idx]
            assert abs(fd - an) <= 1e-6 * max(1.0, abs(an)), (name, idx, fd, an)
            checked += 1
    assert checked >= 13 * 10


# ------------------------------------------------------------ library composition
def torch_layer(dims, w, x, gelu_exact=False):
    """The same layer built from torch library ops (fp64).  Written independently of
    the oracle's loops: layer_norm, linear, softmax and gelu are torch's own."""
    b, s, h, n, d = dims.batch, dims.seq, dims.hidden, dims.heads, dims.head_dim
    X = x.reshape(b, s, h)
    u1 = Fnn.layer_norm(X, (h,), w["ln1_g"], w["ln1_b"], dims.ln_eps)
    qkv = Fnn.linear(u1, w["w_qkv"], w["b_qkv"]).reshape(b, s, n, 3, d)
    q, k, v = (qkv[:, :, :, i, :].permute(0, 2, 1, 3) for i in range(3))  # [b,n,s,d]
    scores = q @ k.transpose(-1, -2) / math.sqrt(d)
    mask = torch.ones(s, s, dtype=torch.bool).tril()
    scores = scores.masked_fill(~mask, float("-inf"))
    a = (torch.softmax(scores, -1) @ v).permute(0, 2, 1, 3).reshape(b, s, n * d)
    x1 = X + Fnn.linear(a, w["w_o"], w["b_o"])
    u2 = Fnn.layer_norm(x1, (h,), w["ln2_g"], w["ln2_b"], dims.ln_eps)
    g = Fnn.gelu(Fnn.linear(u2, w["w_fc1"], w["b_fc1"]), approximate="none" if gelu_exact else "tanh")
    return (x1 + Fnn.linear(g, w["w_fc2"], w["b_fc2"])).reshape(b * s, h)


@pytest.mark.parametrize("gelu_exact", [False, True])
def test_forward_and_backward_match_torch_autograd(gelu_exact):
    rng = np.random.default_rng(1)
    dims = oracle.Dims(hidden=48, heads=3, head_dim=8, ffn=80, seq=13, batch=2, gelu_exact=gelu_exact)
    w = rand_params(dims, rng)
    x = rng.standard_normal((dims.tokens, dims.hidden))
    dy = rng.standard_normal((dims.tokens, dims.hidden))
    y, saved = oracle.layer_fwd(dims, w, x)
    dx, grads = oracle.layer_bwd(dims, w, x, saved, dy)

    tw = {k: torch.tensor(v, dtype=torch.float64, requires_grad=True) for k, v in w.items()}
    tx = torch.tensor(x, dtype=torch.float64, requires_grad=True)
    ty = torch_layer(dims, tw, tx, gelu_exact)
    ty.backward(torch.tensor(dy))
    np.testing.assert_allclose(y, ty.detach().numpy(), rtol=1e-11, atol=1e-11)
    np.testing.assert_allclose(dx, tx.grad.numpy(), rtol=1e-10, atol=1e-10)
    for name in PARAMS:
        np.testing.assert_allclose(grads[name], tw[name].grad.numpy(), rtol=1e-10, atol=1e-10,
                                   err_msg=name)


def test_stage_step_is_composition_of_layers_vs_torch():
    rng = np.random.default_rng(2)
    dims = oracle.Dims(hidden=24, heads=2, head_dim=4, ffn=40, seq=6, batch=1)
    ws = [rand_params(dims, rng) for _ in range(3)]
    x = rng.standard_normal((dims.tokens, dims.hidden))
    dy = rng.standard_normal((dims.tokens, dims.hidden))
    y, dx, grads = oracle.stage_step(dims, ws, x, dy)
    tws = [{k: torch.tensor(v, requires_grad=True) for k, v in w.items()} for w in ws]
    tx = torch.tensor(x, requires_grad=True)
    cur = tx
    for tw in tws:
        cur = torch_layer(dims, tw, cur)
    cur.backward(torch.tensor(dy))
    np.testing.assert_allclose(y, cur.detach().numpy(), rtol=1e-10, atol=1e-10)
    np.testing.assert_allclose(dx, tx.grad.numpy(), rtol=1e-9, atol=1e-9)
    for l in range(3):
        for name in PARAMS:
            np.testing.assert_allclose(grads[l][name], tws[l][name].grad.numpy(), rtol=1e-9,
                                       atol=1e-9, err_msg=f"{l}:{name}")


# ------------------------------------------------------------ invariants
def test_softmax_rows_sum_to_one_and_mask_is_exact_zero():
    rng = np.random.default_rng(3)
    dims = oracle.Dims(hidden=16, heads=2, head_dim=8, ffn=16, seq=17, batch=2)
    qkv = rng.standard_normal((dims.tokens, 3 * dims.proj)) * 3.0
    _, P = oracle.attention_fwd(dims, qkv, return_probs=True)
    assert np.abs(P.sum(-1) - 1.0).max() <= 1e-14
    iu = np.triu_indices(dims.seq, k=1)
    assert (P[:, :, iu[0], iu[1]] == 0.0).all()
    assert (P[:, :, np.arange(dims.seq), np.arange(dims.seq)] > 0).all()  # diagonal attends


def test_layernorm_moments():
    rng = np.random.default_rng(4)
    x = rng.standard_normal((5, 64)) * 2.5 + 1.0
    eps = 1e-5
    out, mean, rstd = oracle.layernorm_fwd(x, np.ones(64), np.zeros(64), eps)
    var = x.var(axis=1)  # biased
    assert np.abs(out.mean(axis=1)).max() <= 1e-14
    np.testing.assert_allclose(out.var(axis=1), var / (var + eps), rtol=1e-12)
    np.testing.assert_allclose(mean, x.mean(axis=1), rtol=1e-13)
    np.testing.assert_allclose(rstd, 1 / np.sqrt(var + eps), rtol=1e-13)
    # constant row -> beta
    beta = rng.standard_normal(64)
    out, _, _ = oracle.layernorm_fwd(np.full((1, 64), 3.25), rng.standard_normal(64), beta, eps)
    np.testing.assert_allclose(out[0], beta, atol=1e-12)


def test_layernorm_matches_torch_library_and_its_autograd():
    rng = np.random.default_rng(5)
    x, g, b, do = (rng.standard_normal(s) for s in ((7, 40), (40,), (40,), (7, 40)))
    out, mean, rstd = oracle.layernorm_fwd(x, g, b, 1e-5)
    dx, dg, db = oracle.layernorm_bwd(x, g, mean, rstd, do)
    tx, tg, tb = (torch.tensor(a, requires_grad=True) for a in (x, g, b))
    to = Fnn.layer_norm(tx, (40,), tg, tb, 1e-5)
    to.backward(torch.tensor(do))
    np.testing.assert_allclose(out, to.detach().numpy(), rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(dx, tx.grad.numpy(), rtol=1e-11, atol=1e-11)
    np.testing.assert_allclose(dg, tg.grad.numpy(), rtol=1e-11, atol=1e-11)
    np.testing.assert_allclose(db, tb.grad.numpy(), rtol=1e-11, atol=1e-11)


def test_zero_weights_give_residual_plus_biases():
    rng = np.random.default_rng(6)
    dims = oracle.Dims(**TINY)
    w = rand_params(dims, rng)
    for k in ("w_qkv", "w_o", "w_fc1", "w_fc2"):
        w[k] = np.zeros_like(w[k])
    w["b_fc1"] = np.zeros_like(w["b_fc1"])  # GeLU(0) = 0 so the MLP contributes b_fc2 only
    x = rng.standard_normal((dims.tokens, dims.hidden))
    y, _ = oracle.layer_fwd(dims, w, x)
    np.testing.assert_allclose(y, x + w["b_o"] + w["b_fc2"], atol=1e-14)


# ------------------------------------------------------------ causality
def test_future_tokens_do_not_change_past_outputs_and_dual():
    rng = np.random.default_rng(7)
    dims = oracle.Dims(**TINY)
    w = rand_params(dims, rng)
    b, s, h = dims.batch, dims.seq, dims.hidden
    t0 = 5
    x = rng.standard_normal((b, s, h))
    x2 = x.copy()
    x2[:, t0:, :] += rng.standard_normal((b, s - t0, h))
    y, saved = oracle.layer_fwd(dims, w, x.reshape(-1, h))
    y2, _ = oracle.layer_fwd(dims, w, x2.reshape(-1, h))
    assert (y.reshape(b, s, h)[:, :t0] == y2.reshape(b, s, h)[:, :t0]).all()  # bitwise
    assert not np.allclose(y.reshape(b, s, h)[:, t0:], y2.reshape(b, s, h)[:, t0:])
    dy = rng.standard_normal((b, s, h))
    dy[:, t0:, :] = 0.0
    dx, _ = oracle.layer_bwd(dims, w, x.reshape(-1, h), saved, dy.reshape(-1, h))
    assert (dx.reshape(b, s, h)[:, t0:] == 0.0).all()
    assert np.abs(dx.reshape(b, s, h)[:, :t0]).min() > 0


def test_prefix_problem_equals_truncated_problem():
    """A causal prefix with zero upstream gradient beyond it is the n-token problem."""
    rng = np.random.default_rng(8)
    dims = oracle.Dims(**TINY)
    w = rand_params(dims, rng)
    b, s, h, n0 = dims.batch, dims.seq, dims.hidden, 3
    x = rng.standard_normal((b, s, h))
    dy = rng.standard_normal((b, s, h))
    dy[:, n0:] = 0
    y, saved = oracle.layer_fwd(dims, w, x.reshape(-1, h))
    dx, grads = oracle.layer_bwd(dims, w, x.reshape(-1, h), saved, dy.reshape(-1, h))
    small = oracle.Dims(**{**TINY, "seq": n0})
    ys, ssaved = oracle.layer_fwd(small, w, x[:, :n0].reshape(-1, h))
    dxs, gs = oracle.layer_bwd(small, w, x[:, :n0].reshape(-1, h), ssaved, dy[:, :n0].reshape(-1, h))
    np.testing.assert_allclose(y.reshape(b, s, h)[:, :n0].reshape(-1, h), ys, rtol=1e-13, atol=1e-13)
    np.testing.assert_allclose(dx.reshape(b, s, h)[:, :n0].reshape(-1, h), dxs, rtol=1e-12, atol=1e-12)
    for name in PARAMS:
        np.testing.assert_allclose(grads[name], gs[name], rtol=1e-12, atol=1e-12, err_msg=name)


# ------------------------------------------------------------ tensor-parallel sum
def slice_params(w, r, R, heads, d, ffn):
    """Rank r's dense local copy under Megatron-style slicing: QKV / FC1 by output rows
    (whole heads, columns ordered [head][q|k|v][d]), Wo / FC2 by input columns;
    LayerNorms and row-parallel biases replicated."""
    nl, Fl = heads // R, ffn // R
    p_l = nl * d
    out = dict(w)
    out["w_qkv"] = w["w_qkv"][r * 3 * p_l:(r + 1) * 3 * p_l]
    out["b_qkv"] = w["b_qkv"][r * 3 * p_l:(r + 1) * 3 * p_l]
    out["w_o"] = w["w_o"][:, r * p_l:(r + 1) * p_l]
    out["w_fc1"] = w["w_fc1"][r * Fl:(r + 1) * Fl]
    out["b_fc1"] = w["b_fc1"][r * Fl:(r + 1) * Fl]
    out["w_fc2"] = w["w_fc2"][:, r * Fl:(r + 1) * Fl]
    return out


def test_sum_of_eight_slices_equals_unsliced_layer():
    rng = np.random.default_rng(9)
    R, heads, d, h, F, s, b = 8, 8, 16, 128, 512, 6, 2
    full = oracle.Dims(hidden=h, heads=heads, head_dim=d, ffn=F, seq=s, batch=b)
    loc = oracle.Dims(hidden=h, heads=heads // R, head_dim=d, ffn=F // R, seq=s, batch=b)
    w = rand_params(full, rng, w_std=0.1)
    x = rng.standard_normal((full.tokens, h))
    dy = rng.standard_normal((full.tokens, h))
    y, saved = oracle.layer_fwd(full, w, x)
    dx, grads = oracle.layer_bwd(full, w, x, saved, dy)

    ws = [slice_params(w, r, R, heads, d, F) for r in range(R)]
    # forward, phase by phase, with a host-side sum standing in for the all-reduce
    sv = [oracle.attn_half_fwd(loc, ws[r], x) for r in range(R)]
    A = sum(s_["A_r"] for s_ in sv)
    np.testing.assert_allclose(A, saved["A_r"], rtol=1e-12, atol=1e-12)
    x1 = x + A + w["b_o"]
    for r in range(R):
        sv[r]["x1"] = x1.copy()
        oracle.mlp_half_fwd(loc, ws[r], sv[r])
    M = sum(s_["M_r"] for s_ in sv)
    np.testing.assert_allclose(M, saved["M_r"], rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(x1 + M + w["b_fc2"], y, rtol=1e-12, atol=1e-12)

    # backward
    mb = [oracle.mlp_half_bwd(loc, ws[r], sv[r], dy) for r in range(R)]
    du2 = sum(m[0] for m in mb)
    dln2, dg2, db2 = oracle.layernorm_bwd(x1, w["ln2_g"], sv[0]["mu2"], sv[0]["rs2"], du2)
    dx1 = dy + dln2
    ab = [oracle.attn_half_bwd(loc, ws[r], sv[r], dx1) for r in range(R)]
    du1 = sum(a_[0] for a_ in ab)
    dln1, dg1, db1 = oracle.layernorm_bwd(x, w["ln1_g"], sv[0]["mu1"], sv[0]["rs1"], du1)
    np.testing.assert_allclose(dx1 + dln1, dx, rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(dg2, grads["ln2_g"], rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(db1, grads["ln1_b"], rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(np.concatenate([m[1]["w_fc1"] for m in mb], 0), grads["w_fc1"], rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(np.concatenate([m[1]["b_fc1"] for m in mb], 0), grads["b_fc1"], rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(np.concatenate([m[1]["w_fc2"] for m in mb], 1), grads["w_fc2"], rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(np.concatenate([a_[1]["w_qkv"] for a_ in ab], 0), grads["w_qkv"], rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(np.concatenate([a_[1]["b_qkv"] for a_ in ab], 0), grads["b_qkv"], rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(np.concatenate([a_[1]["w_o"] for a_ in ab], 1), grads["w_o"], rtol=1e-11, atol=1e-12)


def test_reduce_hook_sums_partials_inside_layer_fwd():
    """With the hook adding the other ranks' partials, a slice's layer_fwd returns the unsliced y."""
    rng = np.random.default_rng(10)
    R, heads, d, h, F, s, b = 2, 4, 8, 32, 64, 5, 1
    full = oracle.Dims(hidden=h, heads=heads, head_dim=d, ffn=F, seq=s, batch=b)
    loc = oracle.Dims(hidden=h, heads=heads // R, head_dim=d, ffn=F // R, seq=s, batch=b)
    w = rand_params(full, rng)
    x = rng.standard_normal((full.tokens, h))
    y, saved = oracle.layer_fwd(full, w, x)
    ws = [slice_params(w, r, R, heads, d, F) for r in range(R)]
    other = oracle.attn_half_fwd(loc, ws[1], x)
    other["x1"] = saved["x1"].copy()
    oracle.mlp_half_fwd(loc, ws[1], other)
    calls = []

    def reduce(view):
        view += (other["A_r"] if not calls else other["M_r"]).ravel()
        calls.append(1)

    y0, _ = oracle.layer_fwd(loc, ws[0], x, reduce=reduce)
    assert len(calls) == 2
    np.testing.assert_allclose(y0, y, rtol=1e-12, atol=1e-12)


# ------------------------------------------------------------ special cases
def test_attention_special_cases():
    rng = np.random.default_rng(11)
    # s = 1: a = v
    dims = oracle.Dims(hidden=8, heads=2, head_dim=4, ffn=8, seq=1, batch=3)
    qkv = rng.standard_normal((3, 24))
    a = oracle.attention_fwd(dims, qkv)
    v = qkv.reshape(3, 2, 3, 4)[:, :, 2, :].reshape(3, 8)
    np.testing.assert_allclose(a, v, atol=1e-15)
    # all keys equal: P[t, u] = 1/(t+1), a = causal running mean of v
    dims = oracle.Dims(hidden=8, heads=1, head_dim=4, ffn=8, seq=9, batch=1)
    qkv = rng.standard_normal((9, 12))
    qkv[:, 4:8] = qkv[0, 4:8]
    a, P = oracle.attention_fwd(dims, qkv, return_probs=True)
    for t in range(9):
        np.testing.assert_allclose(P[0, 0, t, :t + 1], 1.0 / (t + 1), rtol=1e-13)
    np.testing.assert_allclose(a, np.cumsum(qkv[:, 8:], 0) / np.arange(1, 10)[:, None], rtol=1e-12)


def test_attention_matches_torch_sdpa_and_explicit_scale():
    rng = np.random.default_rng(12)
    dims = oracle.Dims(hidden=8, heads=3, head_dim=5, ffn=8, seq=11, batch=2)
    qkv = rng.standard_normal((dims.tokens, 45))
    a = oracle.attention_fwd(dims, qkv)
    t = torch.tensor(qkv).reshape(2, 11, 3, 3, 5)
    q, k, v = (t[:, :, :, i].permute(0, 2, 1, 3) for i in range(3))
    ref = Fnn.scaled_dot_product_attention(q, k, v, is_causal=True).permute(0, 2, 1, 3).reshape(22, 15)
    np.testing.assert_allclose(a, ref.numpy(), rtol=1e-12, atol=1e-12)
    dims2 = oracle.Dims(hidden=8, heads=3, head_dim=5, ffn=8, seq=11, batch=2, softmax_scale=0.37)
    a2 = oracle.attention_fwd(dims2, qkv)
    ref2 = Fnn.scaled_dot_product_attention(q, k, v, is_causal=True, scale=0.37).permute(0, 2, 1, 3).reshape(22, 15)
    np.testing.assert_allclose(a2, ref2.numpy(), rtol=1e-12, atol=1e-12)


def test_attention_bwd_matches_torch_autograd():
    rng = np.random.default_rng(13)
    dims = oracle.Dims(hidden=8, heads=2, head_dim=6, ffn=8, seq=10, batch=2)
    qkv = rng.standard_normal((dims.tokens, 36))
    da = rng.standard_normal((dims.tokens, 12))
    dqkv = oracle.attention_bwd(dims, qkv, da)
    tq = torch.tensor(qkv, requires_grad=True)
    t = tq.reshape(2, 10, 2, 3, 6)
    q, k, v = (t[:, :, :, i].permute(0, 2, 1, 3) for i in range(3))
    out = Fnn.scaled_dot_product_attention(q, k, v, is_causal=True).permute(0, 2, 1, 3).reshape(20, 12)
    out.backward(torch.tensor(da))
    np.testing.assert_allclose(dqkv, tq.grad.numpy(), rtol=1e-11, atol=1e-12)


def test_gelu_values_and_derivative():
    assert oracle.gelu(np.array([0.0]))[0] == 0.0
    assert oracle.gelu_grad(np.array([0.0]))[0] == 0.5
    assert oracle.gelu_grad(np.array([0.0]), exact=True)[0] == 0.5
    big = np.array([12.0, 30.0])
    np.testing.assert_allclose(oracle.gelu(big), big, rtol=1e-12)
    np.testing.assert_allclose(oracle.gelu(-big), 0.0, atol=1e-12)
    z = np.linspace(-6, 6, 241)
    # library forms
    np.testing.assert_allclose(oracle.gelu(z), Fnn.gelu(torch.tensor(z), approximate="tanh").numpy(), rtol=1e-13, atol=1e-15)
    np.testing.assert_allclose(oracle.gelu(z, exact=True), Fnn.gelu(torch.tensor(z)).numpy(), rtol=1e-13, atol=1e-15)
    # the two forms differ by a known small amount (max about 5e-4 near |z| ~ 2.3)
    diff = np.abs(oracle.gelu(z) - oracle.gelu(z, exact=True)).max()
    assert 1e-4 < diff < 1e-3
    # derivative against central differences of the function itself
    for exact in (False, True):
        e = 1e-6
        fd = (oracle.gelu(z + e, exact) - oracle.gelu(z - e, exact)) / (2 * e)
        np.testing.assert_allclose(oracle.gelu_grad(z, exact), fd, rtol=1e-8, atol=1e-9)


def test_linear_pieces_match_numpy_matmul():
    rng = np.random.default_rng(14)
    x, W, b, do = rng.standard_normal((9, 21)), rng.standard_normal((13, 21)), rng.standard_normal(13), rng.standard_normal((9, 13))
    np.testing.assert_allclose(oracle.linear_fwd(x, W, b), x @ W.T + b, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(oracle.linear_fwd(x, W), x @ W.T, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(oracle.linear_dgrad(do, W), do @ W, rtol=1e-12, atol=1e-12)
    dW, db = oracle.linear_wgrad(do, x)
    np.testing.assert_allclose(dW, do.T @ x, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(db, do.sum(0), rtol=1e-12, atol=1e-12)


# ---- optimizer step (Section 3.2: Adam, beta2 = 0.95, clipping at 1.0, weight decay 0.1) ----------------

def test_adam_oracle_against_the_library_adamw_and_clip():
    """Five steps of the oracle against torch.optim.AdamW / clip_grad_norm_ in fp64 (an independent
    implementation of the same published algorithm): weights and both moments."""
    rng = np.random.default_rng(5)
    shapes = [(7, 13), (31,), (4, 5, 3)]
    p0 = [rng.standard_normal(s) * 0.02 for s in shapes]
    tp = [torch.tensor(a.copy(), dtype=torch.float64, requires_grad=True) for a in p0]
    opt = torch.optim.AdamW(tp, lr=5e-3, betas=(0.9, 0.95), eps=1e-8, weight_decay=0.1)
    p = [a.copy() for a in p0]
    m = [np.zeros_like(a) for a in p0]
    v = [np.zeros_like(a) for a in p0]
    for step in range(1, 6):
        g = [rng.standard_normal(s) * (3.0 if step % 2 else 0.01) for s in shapes]   # clipped and unclipped steps
        for t, gi in zip(tp, g):
            t.grad = torch.tensor(gi.copy(), dtype=torch.float64)
        total = torch.nn.utils.clip_grad_norm_(tp, 1.0)
        opt.step()
        sq = oracle.grad_sqnorm(g)
        assert abs(np.sqrt(sq) - float(total)) < 1e-12 * float(total)
        coef = oracle.clip_coefficient(sq, 1.0)
        assert (coef < 1.0) == (np.sqrt(sq) > 1.0)
        for i in range(len(p)):
            p[i], m[i], v[i] = oracle.adam_step(p[i], m[i], v[i], g[i], lr=5e-3, beta1=0.9, beta2=0.95, eps=1e-8,
                                                weight_decay=0.1, step=step, clip_coef=coef)
            st = opt.state[tp[i]]
            np.testing.assert_allclose(p[i], tp[i].detach().numpy(), rtol=1e-12, atol=1e-15)
            np.testing.assert_allclose(m[i], st["exp_avg"].numpy(), rtol=1e-12, atol=1e-18)
            np.testing.assert_allclose(v[i], st["exp_avg_sq"].numpy(), rtol=1e-12, atol=1e-18)


def test_adam_oracle_closed_forms():
    g = np.array([3.0, -0.5, 1e-3, -2e-6])
    p = np.array([0.1, -0.2, 0.3, 0.4])
    z = np.zeros(4)
    # first step from zero moments, no decay: the bias corrections cancel, the step is lr * g / (|g| + eps)
    p1, m1, v1 = oracle.adam_step(p, z, z, g, lr=1e-2, beta1=0.9, beta2=0.95, eps=1e-8, weight_decay=0.0, step=1)
    np.testing.assert_allclose(p1, p - 1e-2 * g / (np.abs(g) + 1e-8), rtol=1e-13)
    np.testing.assert_allclose(m1, 0.1 * g, rtol=1e-13)
    np.testing.assert_allclose(v1, 0.05 * g * g, rtol=1e-13)
    # zero gradient: only the decoupled decay acts, p shrinks by the factor 1 - lr * wd, moments stay zero
    p2, m2, v2 = oracle.adam_step(p, z, z, z, lr=1e-2, weight_decay=0.1, step=7)
    np.testing.assert_allclose(p2, p * (1 - 1e-3), rtol=1e-13)
    assert not m2.any() and not v2.any()
    # a constant gradient held for many steps: both corrected moments tend to g and g^2
    pm, mm, vm = p, z, z
    for t in range(1, 400):
        pm, mm, vm = oracle.adam_step(pm, mm, vm, g, lr=0.0, weight_decay=0.0, step=t)
    np.testing.assert_allclose(mm, g, rtol=1e-10)
    np.testing.assert_allclose(vm, g * g, rtol=1e-8)
    # clipping: below the threshold nothing changes, above it the clipped gradients have norm max_norm
    assert oracle.clip_coefficient(0.25, 1.0) == 1.0 and oracle.clip_coefficient(123.0, 0.0) == 1.0
    big = np.array([3.0, 4.0])
    c = oracle.clip_coefficient(oracle.grad_sqnorm([big]), 1.0)
    assert abs(np.linalg.norm(big * c) - 1.0) < 1e-6


# ---- first / last stage extras (GPT-2 readings: tied embedding, final LayerNorm, next-token cross-entropy) --------

def _head_case(rng, T=24, h=16, V=40, seq=8):
    x = rng.standard_normal((T, h))
    gamma, beta = rng.standard_normal(h) * 0.5 + 1.0, rng.standard_normal(h) * 0.1
    E = rng.standard_normal((V, h)) * 0.3
    targets = rng.integers(0, V, T)
    dloss = rng.uniform(0.2, 1.5, T)
    return x, gamma, beta, E, targets, dloss


def test_lm_head_oracle_against_library_autograd():
    rng = np.random.default_rng(11)
    x, gamma, beta, E, targets, dloss = _head_case(rng)
    loss, dx, dg, db, dE = oracle.lm_head_step(x, gamma, beta, E, targets, dloss)
    tx, tg, tb, tE = (torch.tensor(a, dtype=torch.float64, requires_grad=True) for a in (x, gamma, beta, E))
    u = Fnn.layer_norm(tx, (x.shape[1],), tg, tb, 1e-5)
    tl = Fnn.cross_entropy(u @ tE.T, torch.tensor(targets), reduction="none")
    (tl * torch.tensor(dloss)).sum().backward()
    np.testing.assert_allclose(loss, tl.detach().numpy(), rtol=1e-12)
    for got, want in ((dx, tx.grad), (dg, tg.grad), (db, tb.grad), (dE, tE.grad)):
        np.testing.assert_allclose(got, want.numpy(), rtol=1e-9, atol=1e-13)
    # a uniform row: loss = log V whatever the target
    l0, _, _ = oracle.cross_entropy_fwd(np.zeros((3, 40)), [0, 7, 39])
    np.testing.assert_allclose(l0, np.log(40.0), rtol=1e-14)
    # softmax minus one-hot: every gradient row of the unsliced loss sums to zero
    lg = rng.standard_normal((5, 9))
    tg5 = [1, 2, 3, 4, 8]
    _, m5, s5 = oracle.cross_entropy_fwd(lg, tg5)
    d = oracle.cross_entropy_bwd(lg, tg5, m5, s5, np.ones(5))
    assert np.abs(d.sum(axis=1)).max() < 1e-14 and all(d[t, tg5[t]] < 0 for t in range(5))


def test_vocabulary_slices_reproduce_the_unsliced_head_and_embedding():
    """Four ranks, each with a quarter of E's rows, exchanging one maximum and three sums, give the unsliced loss,
    dx and LayerNorm gradients, and each its own rows of dE; likewise for the embedding lookup."""
    rng = np.random.default_rng(12)
    x, gamma, beta, E, targets, dloss = _head_case(rng)
    V, R = E.shape[0], 4
    Vl = V // R
    want = oracle.lm_head_step(x, gamma, beta, E, targets, dloss)

    # lock-step emulation of the exchanges: run every rank up to each exchange point by re-running with recorded values
    logits = [oracle.linear_fwd(oracle.layernorm_fwd(x, gamma, beta)[0], E[r * Vl:(r + 1) * Vl]) for r in range(R)]
    m = np.max([l.max(1) for l in logits], axis=0)
    s = sum(np.exp(l - m[:, None]).sum(1) for l in logits)
    tl = sum(np.array([l[t, targets[t] - r * Vl] if r * Vl <= targets[t] < (r + 1) * Vl else 0.0
                       for t in range(len(targets))]) for r, l in enumerate(logits))
    dus = [oracle.linear_dgrad(oracle.cross_entropy_bwd(logits[r], targets, m, s, dloss, r * Vl), E[r * Vl:(r + 1) * Vl])
           for r in range(R)]
    du = sum(dus)

    def make_reduce(state):
        def reduce(a, op):
            state["n"] += 1
            return {1: m, 2: s, 3: tl, 4: du}[state["n"]]
        return reduce
    for r in range(R):
        got = oracle.lm_head_step(x, gamma, beta, E[r * Vl:(r + 1) * Vl], targets, dloss, vocab_start=r * Vl,
                                  reduce=make_reduce({"n": 0}))
        for g, w in zip(got[:4], want[:4]):
            np.testing.assert_allclose(g, w, rtol=1e-10, atol=1e-13)
        np.testing.assert_allclose(got[4], want[4][r * Vl:(r + 1) * Vl], rtol=1e-10, atol=1e-13)

    # embedding: lookup against the library routine, slices sum to it, gradients against autograd
    seq, T, h = 8, 24, E.shape[1]
    tokens = rng.integers(0, V, T)
    P = rng.standard_normal((seq, h))
    xe = oracle.embedding_fwd(tokens, E, P, seq)
    tE, tP = torch.tensor(E, requires_grad=True), torch.tensor(P, requires_grad=True)
    te = Fnn.embedding(torch.tensor(tokens), tE) + tP.repeat(T // seq, 1)
    np.testing.assert_allclose(xe, te.detach().numpy(), rtol=1e-15)
    parts = [oracle.embedding_fwd(tokens, E[r * Vl:(r + 1) * Vl], np.zeros_like(P), seq, r * Vl) for r in range(R)]
    np.testing.assert_allclose(sum(parts) + np.tile(P, (T // seq, 1)), xe, rtol=1e-15)
    dxe = rng.standard_normal((T, h))
    (te * torch.tensor(dxe)).sum().backward()
    for r in range(R):
        dE_r, dP = oracle.embedding_bwd(tokens, dxe, Vl, seq, r * Vl)
        np.testing.assert_allclose(dE_r, tE.grad.numpy()[r * Vl:(r + 1) * Vl], rtol=1e-12, atol=1e-15)
        np.testing.assert_allclose(dP, tP.grad.numpy(), rtol=1e-12, atol=1e-15)
