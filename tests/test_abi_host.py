"""Host-side checks of the C ABI that need no GPU: the library loads, exports every function the
header declares, validates descriptors and pointers before touching the device."""
import ctypes
import os
import re

import pytest

import paper_2201_11990_amd as M
from paper_2201_11990_amd import binding as B
from paper_2201_11990_amd.inputs import WORKLOADS

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def header_functions():
    src = open(os.path.join(ROOT, "include", "mtnlg.h")).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(mtnlg_[a-z0-9_]+)\s*\(", src)) - {"mtnlg_reduce_fn"})


def test_library_exports_every_declared_function():
    names = header_functions()
    assert len(names) >= 20
    L = B.lib()
    for n in names:
        assert hasattr(L, n), n
    assert sorted(B.EXPORTED) == names


def test_version_and_status_strings():
    assert M.mtnlg_version() == 1
    assert B.status_string(0) == "ok"
    for code in range(-6, 0):
        assert B.status_string(code) not in ("ok", "unknown status")
    assert B.status_string(-99) == "unknown status"


def test_descriptor_validation():
    for wl in WORKLOADS.values():
        assert M.mtnlg_layer_desc_check(B.desc_from_workload(wl)) == 0, wl.name
    ok = dict(hidden=256, heads_local=4, head_dim=64, ffn_local=1024, seq=128, micro_batch=2, dtype="fp32")
    assert M.mtnlg_layer_desc_check(B.make_desc(**ok)) == 0
    bad = [dict(hidden=0), dict(seq=-1), dict(tp_size=0), dict(tp_size=2, tp_rank=2), dict(dtype=7),
           dict(gelu=3), dict(flags=64), dict(ln_eps=-1.0)]
    for b in bad:
        assert M.mtnlg_layer_desc_check(B.make_desc(**{**ok, **b})) == -1, b
    for b in [dict(hidden=260), dict(head_dim=60), dict(ffn_local=1001), dict(hidden=65536), dict(head_dim=512)]:
        assert M.mtnlg_layer_desc_check(B.make_desc(**{**ok, **b})) == -3, b
    assert B.lib().mtnlg_layer_desc_check(None) == -2


def test_size_queries():
    wl = WORKLOADS["mtnlg_tp8_stage"]
    d = B.desc_from_workload(wl)
    L = M.mtnlg_saved_layout_get(d)
    T, h, p, F = wl.tokens, wl.hidden, wl.proj, wl.ffn
    payload = 2 * (3 * T * h + 3 * T * p + T * p + 2 * T * F) + 4 * (4 * T + wl.heads * T)
    assert payload <= L.total == M.mtnlg_saved_bytes(d) < payload + 13 * 256
    offs = [getattr(L, n) for n, _ in B.SavedLayout._fields_][:-1]
    assert all(o % 256 == 0 for o in offs) and len(set(offs)) == len(offs)
    slot = T * h * 2
    assert M.mtnlg_stage_saved_bytes(d, 3) == 3 * slot + 3 * L.total
    dr = B.desc_from_workload(wl, flags=B.RECOMPUTE)
    assert M.mtnlg_stage_saved_bytes(dr, 3) == 3 * slot + L.total
    assert M.mtnlg_workspace_bytes(d) >= 2 * (3 * T * h + T * F + 4 * T * p)
    assert M.mtnlg_saved_bytes(B.make_desc(0, 1, 8, 8, 8, 1, "bf16")) == 0
    assert M.mtnlg_stage_saved_bytes(d, 0) == 0


def test_null_pointers_and_small_workspace_are_reported_before_any_gpu_work():
    L = B.lib()
    d = B.desc_from_workload(WORKLOADS["tiny_fp32"])
    nohook = ctypes.cast(None, B.REDUCE_FN)
    one = ctypes.c_void_p(256)  # never dereferenced: argument checks come first
    assert L.mtnlg_layer_fwd(ctypes.byref(d), None, one, one, one, one, 1 << 40, nohook, None, None) == -2
    tbl = B._Ptrs12(*([256] * 12))
    assert L.mtnlg_layer_fwd(ctypes.byref(d), ctypes.byref(tbl), None, one, one, one, 1 << 40, nohook, None, None) == -2
    assert L.mtnlg_layer_fwd(ctypes.byref(d), ctypes.byref(tbl), one, one, one, one, 1 << 40, nohook, None, None) == -1  # y aliases x
    two = ctypes.c_void_p(512)
    assert L.mtnlg_layer_fwd(ctypes.byref(d), ctypes.byref(tbl), one, two, one, one, 16, nohook, None, None) == -4
    assert L.mtnlg_layer_bwd(ctypes.byref(d), ctypes.byref(tbl), one, one, one, two, None, one, 1 << 40, nohook, None, None) == -2
    assert L.mtnlg_layer_bwd(ctypes.byref(d), ctypes.byref(tbl), one, one, one, one, ctypes.byref(tbl), one, 1 << 40, nohook, None, None) == -1
    assert L.mtnlg_stage_step(ctypes.byref(d), 0, ctypes.byref(tbl), one, one, two, two, ctypes.byref(tbl), one, 1 << 40, one, 1 << 40, nohook, None, None) == -1
    assert L.mtnlg_stage_step(ctypes.byref(d), 1, ctypes.byref(tbl), one, one, two, two, ctypes.byref(tbl), one, 8, one, 1 << 40, nohook, None, None) == -4
    assert L.mtnlg_gemm(1, 0, 8, 8, 8, None, one, one, None, None, 0, None, 0, None) == -2
    assert L.mtnlg_gemm(1, 5, 8, 8, 8, one, one, one, None, None, 0, None, 0, None) == -1
    assert L.mtnlg_gemm(1, 0, 8, 8, 8, one, one, one, None, None, B.EPI_BIAS, None, 0, None) == -2
    assert L.mtnlg_layernorm_fwd(1, 4, 12, one, None, None, one, one, 1e-5, None, one, one, one, None) == -3
    assert L.mtnlg_attention_fwd(1, 1, 8, 1, 8, 0.0, one, one, one, None) == -1
    assert L.mtnlg_colsum(1, 4, 12, one, one, 0, 0, one, None) == -3


def test_empty_problems_are_rejected_before_any_gpu_work():
    """A size of zero anywhere is an argument error (MTNLG_INVALID_ARG), never a launch; size queries answer 0."""
    L = B.lib()
    one, two = ctypes.c_void_p(256), ctypes.c_void_p(512)
    f = ctypes.c_float
    i64 = ctypes.c_int64
    for M_, N_, K_ in ((0, 8, 8), (8, 0, 8), (8, 8, 0)):
        assert L.mtnlg_gemm(1, 0, i64(M_), i64(N_), i64(K_), one, one, two, None, None, 0, None, 0, None) == -1
    assert L.mtnlg_layernorm_fwd(1, i64(0), i64(16), one, None, None, one, one, f(1e-5), None, two, one, one, None) == -1
    assert L.mtnlg_layernorm_bwd(1, i64(0), i64(16), one, one, one, one, one, None, two, one, one, None, 1, 0, one, None) == -1
    assert L.mtnlg_attention_fwd(1, 1, 0, 1, 64, f(0.125), one, two, one, None) == -1
    assert L.mtnlg_attention_bwd(1, 0, 8, 1, 64, f(0.125), one, one, one, one, two, one, None) == -1
    assert L.mtnlg_attention_bwd_workspace(1, 0, 1, 64) == 0
    assert L.mtnlg_gelu_fwd(1, 0, i64(0), one, two, None) == -1
    assert L.mtnlg_gelu_bwd(1, 0, i64(0), one, one, two, None) == -1
    assert L.mtnlg_colsum(1, i64(0), i64(16), one, two, 0, 0, one, None) == -1
    assert L.mtnlg_bias_residual(1, i64(0), i64(16), one, one, None, two, None) == -1
    assert L.mtnlg_grad_sqnorm(i64(0), one, one, one, 0, None) == -1
    adam = B.AdamDesc(1e-3, 0.9, 0.95, 1e-8, 0.1, 1.0, 1)
    assert L.mtnlg_adam_step(ctypes.byref(adam), i64(0), one, one, one, one, None, None, None) == -1
    d = B.desc_from_workload(WORKLOADS["tiny_fp32"])
    tbl = B._Ptrs12(*([256] * 12))
    nohook = ctypes.cast(None, B.REDUCE_FN)
    assert L.mtnlg_stage_step_accumulate(ctypes.byref(d), 1, ctypes.byref(tbl), 0, one, one, two, two, ctypes.byref(tbl),
                                         one, 1 << 40, one, 1 << 40, nohook, None, None) == -1
    for field in ("seq", "micro_batch", "hidden", "heads_local", "ffn_local"):
        bad = B.desc_from_workload(WORKLOADS["tiny_fp32"])
        setattr(bad, field, 0)
        assert L.mtnlg_layer_desc_check(ctypes.byref(bad)) == -1, field
        assert L.mtnlg_saved_bytes(ctypes.byref(bad)) == 0 and L.mtnlg_workspace_bytes(ctypes.byref(bad)) == 0
    head = B.head_desc(64, 0, 0, 8, 1, "fp32")
    assert L.mtnlg_lm_head_workspace(ctypes.byref(head)) == 0
    assert L.mtnlg_embedding_fwd(ctypes.byref(head), one, one, one, two, ctypes.cast(None, B.REDUCE_OP_FN), None, None) == -1
