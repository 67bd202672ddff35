"""mtnlg_colsum_static (the entry point that allocates nothing: its partial sums go through a static device
array) against mtnlg_colsum (the same kernels with a caller's workspace), through the C ABI: bit-equal outputs
on two calls in a row, the second with a smaller input, both dtypes, overwrite and accumulate; and the limit."""
import ctypes

import pytest
import torch

import paper_2201_11990_amd as M
from paper_2201_11990_amd import binding as B

pytestmark = pytest.mark.gpu


def both(x, out_dtype, accumulate, seed):
    T, C = x.shape
    g = torch.Generator(device="cuda").manual_seed(seed)
    start = torch.randn(C, device="cuda", generator=g).to(out_dtype)
    want, got = start.clone(), start.clone()
    ws = torch.full((M.mtnlg_colsum_workspace(T, C),), 0xFF, dtype=torch.uint8, device="cuda")
    M.mtnlg_colsum(x, want, ws, accumulate=accumulate)
    M.mtnlg_colsum_static(x, got, accumulate=accumulate)
    torch.cuda.synchronize()
    return want, got


@pytest.mark.parametrize("dtype,out_dtype", [(torch.bfloat16, torch.bfloat16), (torch.bfloat16, torch.float32),
                                             (torch.float32, torch.float32)], ids=["bf16", "bf16-f32out", "fp32"])
def test_two_calls_in_a_row_the_second_smaller(dtype, out_dtype):
    g = torch.Generator(device="cuda").manual_seed(11)
    # the first call leaves 32 x 20480 partials in the static array; the second uses fewer rows of fewer columns
    for i, (T, C) in enumerate([(2048, 20480), (333, 520), (70, 32768), (5, 8)]):
        x = torch.randn((T, C), device="cuda", generator=g).to(dtype)
        for accumulate in (False, True):
            want, got = both(x, out_dtype, accumulate, seed=100 + i)
            assert torch.isfinite(got.float()).all()
            assert torch.equal(want, got), (T, C, accumulate)
        # and against the definition (fp64 column sums of the stored values), to the parity bar
        ref = x.double().sum(0)
        out = torch.zeros(C, dtype=out_dtype, device="cuda")
        M.mtnlg_colsum_static(x, out)
        err = ((out.double() - ref).norm() / ref.norm()).item()
        assert err <= (1e-2 if out_dtype == torch.bfloat16 else 1e-5), (T, C, err)


def test_limit_and_argument_errors():
    cmax = M.mtnlg_colsum_static_max_columns()
    assert cmax == 32768
    x = torch.zeros((2, cmax + 8), dtype=torch.bfloat16, device="cuda")
    out = torch.zeros(cmax + 8, dtype=torch.bfloat16, device="cuda")
    with pytest.raises(B.MtnlgError) as ei:
        M.mtnlg_colsum_static(x, out)
    assert ei.value.status == -4
    L = B.lib()
    assert L.mtnlg_colsum_static(B.BF16, 4, 16, None, ctypes.c_void_p(out.data_ptr()), 0, 0, None) == -2
    assert L.mtnlg_colsum_static(B.BF16, 0, 16, ctypes.c_void_p(x.data_ptr()), ctypes.c_void_p(out.data_ptr()), 0, 0, None) == -1
    assert L.mtnlg_colsum_static(B.BF16, 4, 12, ctypes.c_void_p(x.data_ptr()), ctypes.c_void_p(out.data_ptr()), 0, 0, None) == -3
    torch.cuda.synchronize()
