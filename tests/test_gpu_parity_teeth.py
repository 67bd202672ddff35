"""Are the GPU parity tolerances tight enough to notice a mistake?  The GPU path is left alone; the mistakes of
test_oracle_mutants.py are planted in compiled copies of the CPU oracle, one at a time, and the layer parity check
(HIP path against that oracle, same seeded inputs, same tolerances as the real parity tests) has to fail for each,
on the fp32 path (1e-5) and on the bf16 path (1e-2).  Three of the twenty mistakes change a bf16 result by less
than the 1e-2 that bf16 storage needs (a 0.045 z^2 term of the GeLU derivative, the h / (h - 1) of an unbiased
variance, the mean term of the LayerNorm gradient, which is ~h^-1/2 of a term that the residual path dilutes): those
are left to the fp32 path, which runs the same LayerNorm / GeLU kernels and the same orchestration."""
import pytest

import test_gpu_layer as layer_tests
import test_oracle_mutants as mutants
from test_oracle_mutants import in_place_of_the_oracle  # noqa: F401  (fixture)

pytestmark = pytest.mark.gpu


def both_gelu_forms(wl):
    layer_tests.check_layer(wl, "random")
    layer_tests.check_layer(wl, "random", gelu_exact=True)


def test_parity_holds_against_the_oracle_as_committed():
    both_gelu_forms(layer_tests.TINY)
    both_gelu_forms(layer_tests.SMALL_BF16)


BELOW_THE_BF16_BAR = {"gelu_derivative_factor", "layernorm_unbiased_variance", "layernorm_bwd_mean_term_dropped"}
CASES = [(layer_tests.TINY, m) for m in mutants.MUTANTS] + \
        [(layer_tests.SMALL_BF16, m) for m in mutants.MUTANTS if m[0] not in BELOW_THE_BF16_BAR]


@pytest.mark.parametrize("wl,name,old,new,which", [(w,) + m for w, m in CASES], ids=[f"{m[0]}-{w.dtype}" for w, m in CASES])
def test_parity_fails_against_an_oracle_with_a_planted_mistake(name, old, new, which, wl, tmp_path,
                                                               in_place_of_the_oracle):  # noqa: F811
    text = open(mutants.SRC).read()
    start = -1
    for _ in range(which + 1):
        start = text.find(old, start + 1)
        assert start >= 0, f"mutation site of {name} not found"
    mutated = text[:start] + new + text[start + len(old):]
    in_place_of_the_oracle(mutants.load(mutants.compile_variant(mutated, str(tmp_path), name)))
    with pytest.raises(AssertionError):
        both_gelu_forms(wl)
