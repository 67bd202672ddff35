"""Do the oracle's pins have teeth?  Plausible mistakes are planted in copies of the oracle's C source
(a dropped term, a wrong sign, constant or operand, a missing scale), each copy is compiled on the CPU
and put in the oracle's place, and the pin battery of test_oracle_pins.py has to reject every one of
them, while the source as committed passes.  The numpy references of the optimizer step and of the
first / last stage's extras get the same treatment further down.  Nothing here touches the GPU library.
"""
import ctypes
import os
import subprocess

import pytest

import oracle
import test_oracle_pins as pins

SRC = os.path.join(os.path.dirname(os.path.abspath(oracle.__file__)), "mtnlg_oracle.c")

# (name, text as committed, planted mistake, which occurrence)
MUTANTS = [
    ("gelu_cubic_term_squared", "kSqrt2OverPi * (z + kGeluC * z * z * z)));", "kSqrt2OverPi * (z + kGeluC * z * z)));", 0),
    ("gelu_derivative_factor", "(1.0 + 3.0 * kGeluC * z * z)", "(1.0 + 2.0 * kGeluC * z * z)", 0),
    ("gelu_erf_derivative_without_density", "return cdf + z * pdf;", "return cdf;", 0),
    ("layernorm_unbiased_variance", "var /= (double)h; /* biased variance */", "var /= (double)(h - 1);", 0),
    ("layernorm_bwd_mean_term_dropped", "rs * (dxh - m1 - xhat * m2)", "rs * (dxh - xhat * m2)", 0),
    ("layernorm_bwd_sign", "rs * (dxh - m1 - xhat * m2)", "rs * (dxh - m1 + xhat * m2)", 0),
    ("layernorm_dgamma_without_xhat", "sg += dout[t * h + i] * xhat;", "sg += dout[t * h + i];", 0),
    ("linear_bias_dropped", "out[t * N + n] = acc + (bias ? bias[n] : 0.0);", "out[t * N + n] = acc;", 0),
    ("bias_gradient_dropped", "sb += go;", "sb += 0.0 * go;", 0),
    ("softmax_scale_one_over_d", "1.0 / sqrt((double)D->head_dim)", "1.0 / (double)D->head_dim", 0),
    ("attention_reads_keys_as_values",
     "const double *v = qkv + (bi * s + u) * ld + j * 3 * d + 2 * d;\n          for (int64_t e = 0; e < d; ++e) ar[e] += P[u] * v[e];",
     "const double *v = qkv + (bi * s + u) * ld + j * 3 * d + d;\n          for (int64_t e = 0; e < d; ++e) ar[e] += P[u] * v[e];", 0),
    ("softmax_jacobian_term_dropped", "double dS = P[u] * (dP[u] - dot);", "double dS = P[u] * dP[u];", 0),
    ("dk_without_scale", "dk[e] += sc * dS * q[e];", "dk[e] += dS * q[e];", 0),
    ("dq_from_queries", "dq[e] += sc * dS * k[e];", "dq[e] += sc * dS * q[e];", 0),
    ("second_residual_dropped", "y[t * h + i] = S->x1[t * h + i] + S->M_r[t * h + i] + W->b_fc2[i];",
     "y[t * h + i] = S->M_r[t * h + i] + W->b_fc2[i];", 0),
    ("projection_bias_dropped", "S->x1[t * h + i] = x[t * h + i] + S->A_r[t * h + i] + W->b_o[i];",
     "S->x1[t * h + i] = x[t * h + i] + S->A_r[t * h + i];", 0),
    ("residual_gradient_dropped", "dx1[i] = dy[i] + tmp[i];", "dx1[i] = tmp[i];", 0),
    ("fc2_weight_gradient_from_preactivation", "orc_linear_wgrad(dy, S->g, T, h, F, G->w_fc2, NULL);",
     "orc_linear_wgrad(dy, S->z, T, h, F, G->w_fc2, NULL);", 0),
    ("projection_bias_gradient_from_dy", "for (int64_t t = 0; t < T; ++t) sb += dx1[t * h + i];",
     "for (int64_t t = 0; t < T; ++t) sb += dy[t * h + i];", 0),
    ("layernorm2_backward_on_layer_input", "orc_layernorm_bwd(S->x1, W->ln2_g, S->mu2, S->rs2, du,",
     "orc_layernorm_bwd(x, W->ln2_g, S->mu2, S->rs2, du,", 0),
]


def battery():
    """The pins that look at the C oracle's arithmetic (each raises AssertionError on a mismatch)."""
    for exact in (False, True):
        pins.test_gradients_match_central_finite_differences(exact)
        pins.test_forward_and_backward_match_torch_autograd(exact)
    pins.test_layernorm_moments()
    pins.test_layernorm_matches_torch_library_and_its_autograd()
    pins.test_zero_weights_give_residual_plus_biases()
    pins.test_attention_special_cases()
    pins.test_attention_matches_torch_sdpa_and_explicit_scale()
    pins.test_attention_bwd_matches_torch_autograd()
    pins.test_gelu_values_and_derivative()
    pins.test_linear_pieces_match_numpy_matmul()


def load(path):
    lib = ctypes.CDLL(path)
    lib.orc_gelu.restype = ctypes.c_double
    lib.orc_gelu.argtypes = [ctypes.c_double, ctypes.c_int]
    lib.orc_gelu_grad.restype = ctypes.c_double
    lib.orc_gelu_grad.argtypes = [ctypes.c_double, ctypes.c_int]
    return lib


def compile_variant(text, workdir, name):
    src = os.path.join(workdir, name + ".c")
    out = os.path.join(workdir, "lib" + name + ".so")
    with open(src, "w") as f:
        f.write(text)
    subprocess.check_call(["gcc", "-O1", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-o", out, src, "-lm"])
    return out


@pytest.fixture()
def in_place_of_the_oracle():
    genuine = oracle.lib()

    def swap(lib):
        oracle._lib = lib
    yield swap
    oracle._lib = genuine


def test_the_committed_source_passes_the_battery(tmp_path, in_place_of_the_oracle):
    in_place_of_the_oracle(load(compile_variant(open(SRC).read(), str(tmp_path), "as_committed")))
    battery()


@pytest.mark.parametrize("name,old,new,which", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_a_planted_mistake_is_caught(name, old, new, which, tmp_path, in_place_of_the_oracle):
    text = open(SRC).read()
    start = -1
    for _ in range(which + 1):
        start = text.find(old, start + 1)
        assert start >= 0, f"mutation site of {name} not found: the oracle's source changed, update this list"
    mutated = text[:start] + new + text[start + len(old):]
    in_place_of_the_oracle(load(compile_variant(mutated, str(tmp_path), name)))
    with pytest.raises(AssertionError):
        battery()


# ---- the numpy references of the optimizer step and of the first / last stage's extras ------------------------

PY_MUTANTS = [
    ("optimizer", "adam_without_bias_correction", "m_hat = m / (1.0 - beta1 ** step)", "m_hat = m"),
    ("optimizer", "second_moment_of_the_gradient_itself", "v = beta2 * v + (1.0 - beta2) * g * g", "v = beta2 * v + (1.0 - beta2) * g"),
    ("optimizer", "epsilon_under_the_root", "(np.sqrt(v_hat) + eps)", "np.sqrt(v_hat + eps)"),
    ("optimizer", "decay_not_scaled_by_the_rate", "p = p - lr * (m_hat / (np.sqrt(v_hat) + eps) + weight_decay * p)",
     "p = p - lr * (m_hat / (np.sqrt(v_hat) + eps)) - weight_decay * p"),
    ("optimizer", "clipping_also_scales_up", "return min(1.0, max_norm / (np.sqrt(sqnorm) + 1e-6))",
     "return max_norm / (np.sqrt(sqnorm) + 1e-6)"),
    ("optimizer", "norm_of_absolute_values", "np.sum(np.asarray(g, dtype=np.float64) ** 2)", "np.sum(np.abs(np.asarray(g, dtype=np.float64)))"),
    ("head", "positions_indexed_by_sequence_number", "x[t] += P[t % seq]", "x[t] += P[t // seq]"),
    ("head", "first_row_of_a_block_skipped", "if 0 <= v < Vl:\n            x[t] = E[v]", "if 0 < v < Vl:\n            x[t] = E[v]"),
    ("head", "maximum_not_added_back", "return np.log(s) + m - tl, m, s", "return np.log(s) - tl, m, s"),
    ("head", "one_hot_not_subtracted", "d[t, v] -= 1.0", "d[t, v] -= 0.0"),
    ("head", "embedding_gradient_from_the_unnormalised_input", "dE, _ = linear_wgrad(dlogits, u)", "dE, _ = linear_wgrad(dlogits, x)"),
    ("head", "position_gradient_overwritten", "dP[t % seq] += dx[t]", "dP[t % seq] = dx[t]"),
    ("head", "token_gradient_overwritten", "dE[v] += dx[t]", "dE[v] = dx[t]"),
]
PY_NAMES = {"optimizer": ("grad_sqnorm", "clip_coefficient", "adam_step"),
            "head": ("embedding_fwd", "embedding_bwd", "cross_entropy_fwd", "cross_entropy_bwd", "lm_head_step")}


def py_battery():
    pins.test_adam_oracle_against_the_library_adamw_and_clip()
    pins.test_adam_oracle_closed_forms()
    pins.test_lm_head_oracle_against_library_autograd()
    pins.test_vocabulary_slices_reproduce_the_unsliced_head_and_embedding()


def module_from_text(which, text):
    import types
    mod = types.ModuleType(f"oracle._variant_of_{which}")
    mod.__package__ = "oracle"
    exec(compile(text, f"<variant of oracle/{which}.py>", "exec"), mod.__dict__)
    return mod


def test_the_committed_numpy_references_pass_their_battery():
    py_battery()


@pytest.mark.parametrize("which,name,old,new", PY_MUTANTS, ids=[m[1] for m in PY_MUTANTS])
def test_a_mistake_planted_in_a_numpy_reference_is_caught(which, name, old, new, monkeypatch):
    path = os.path.join(os.path.dirname(SRC), which + ".py")
    text = open(path).read()
    assert text.count(old) == 1, f"mutation site of {name} not found once: the source changed, update this list"
    mod = module_from_text(which, text.replace(old, new))
    for fn in PY_NAMES[which]:
        monkeypatch.setattr(oracle, fn, getattr(mod, fn))
    with pytest.raises(AssertionError):
        py_battery()
