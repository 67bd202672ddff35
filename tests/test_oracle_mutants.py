"""Do the oracle's pins have teeth?  Plausible mistakes are planted in copies of the oracle's C source
(a dropped term, a wrong sign, constant or operand, a missing scale), each copy is compiled on the CPU
and put in the oracle's place, and the pin battery of test_oracle_pins.py has to reject every one of
them, while the source as committed passes.  Nothing here touches the GPU library.
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
