"""The parity measures themselves (CPU): the element-wise complement must reject what the Frobenius bar alone lets
through (a misplaced 16 x 16 block, a bad ragged tail, one wrong element) and must accept honest rounding noise of
the size the bar allows, on Gaussian and on heavy-tailed tensors."""
import numpy as np
import pytest

from parity import TOL, assert_close, elementwise_ratio, rel_fro


def bf16_round(a):
    import torch
    return torch.tensor(a, dtype=torch.float32).bfloat16().double().numpy()


@pytest.fixture(scope="module")
def want():
    return np.random.default_rng(0).standard_normal((2048, 4096))


def test_rounding_noise_at_half_the_bar_passes(want):
    rng = np.random.default_rng(1)
    got = want * (1 + 3e-3 * rng.standard_normal(want.shape)) + 3e-3 * rng.standard_normal(want.shape)
    assert rel_fro(got, want) < TOL["bf16"]
    assert elementwise_ratio(got, want, TOL["bf16"]) < 1.0
    assert_close(got, want, TOL["bf16"], "noise")
    # plain bf16 storage of a heavy-tailed tensor (a few elements 50 x the rms)
    heavy = want.copy()
    heavy[::97, ::89] *= 50.0
    assert_close(bf16_round(heavy), heavy, TOL["bf16"], "bf16 storage, heavy tails")


@pytest.mark.parametrize("damage", ["block", "edge_row", "one_element", "swapped_tiles"])
def test_local_damage_below_the_norm_bar_is_caught(want, damage):
    got = bf16_round(want)
    if damage == "block":          # a 16 x 16 block taken from somewhere else
        got[512:528, 1024:1040] = got[0:16, 0:16]
    elif damage == "edge_row":     # the ragged tail of the last row never written (zeros)
        got[-1, -200:] = 0.0
    elif damage == "one_element":  # a single wrong value of ordinary size
        got[7, 9] = -got[7, 9] + 1.0
    else:                          # two neighbouring 16-column strips of an 8-row block swapped
        got[64:72, 32:48], got[64:72, 48:64] = got[64:72, 48:64].copy(), got[64:72, 32:48].copy()
    assert rel_fro(got, want) < TOL["bf16"], "the norm alone does not see it"
    with pytest.raises(AssertionError, match="allowance"):
        assert_close(got, want, TOL["bf16"], damage)


def test_rows_of_very_different_size():
    """A weight-gradient-like matrix (outer-product structure: row i scaled by a_i, column j by b_j, scales over an
    order of magnitude): errors proportional to the local size pass, damage in a small-valued region is still seen."""
    rng = np.random.default_rng(3)
    a = np.exp(rng.uniform(-1.5, 1.5, (1024, 1)))
    b = np.exp(rng.uniform(-1.0, 1.0, (1, 2048)))
    want = a * b * rng.standard_normal((1024, 2048))
    got = want + 4e-3 * a * b * rng.standard_normal(want.shape)
    assert_close(got, want, TOL["bf16"], "noise proportional to row and column size")
    small_rows = np.argsort(a[:, 0])[:16]
    got2 = bf16_round(want)
    got2[small_rows[:, None], np.arange(64, 80)[None, :]] = 0.0     # a 16 x 16 hole where values are smallest
    assert rel_fro(got2, want) < TOL["bf16"]
    with pytest.raises(AssertionError, match="allowance"):
        assert_close(got2, want, TOL["bf16"], "hole in the smallest rows")


def test_fp32_bar_and_degenerate_inputs():
    rng = np.random.default_rng(2)
    w = rng.standard_normal((300, 300))
    assert_close(w.astype(np.float32).astype(np.float64), w, TOL["fp32"], "float storage")
    with pytest.raises(AssertionError):
        assert_close(w * (1 + 1e-4), w, TOL["fp32"], "1e-4 relative")
    z = np.zeros((4, 4))
    assert_close(z, z, TOL["bf16"], "zeros")
    with pytest.raises(AssertionError):
        assert_close(z + 1e-30, z, TOL["bf16"], "non-zero against zero")
