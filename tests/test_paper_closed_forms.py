"""Host-side accounting (shapes, FLOPs, bytes) pinned to numbers the paper prints.
The fixture tests/golden/paper_closed_forms.json carries the values and where they are printed."""
import json
import math
import os

import torch

from paper_2201_11990_amd import flops, inputs

G = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "paper_closed_forms.json")))
M = G["model"]


def test_parameter_count_fixes_ffn_width_at_4h():
    per_layer = flops.layer_param_count(M["hidden"], 4 * M["hidden"])
    total = M["layers"] * per_layer
    assert abs(total / 1e9 - M["params_billion_stated"]) < 2.0          # 528.5 B + embeddings
    assert abs(per_layer / 1e9 - 5.03) < 0.01
    # a 2h or 8h FFN would miss "530 billion" by far
    for mult in (2, 8):
        assert abs(M["layers"] * flops.layer_param_count(M["hidden"], mult * M["hidden"]) / 1e9 - 530) > 100


def test_memory_closed_forms():
    mem = G["memory"]
    assert M["params_billion_stated"] * 1e9 * mem["bytes_per_param"] > mem["state_terabytes_lower_bound"] * 1e12
    act = flops.boundary_activation_bytes(M["global_batch"], M["layers"], M["seq"], M["hidden"])
    assert round(act / 1e12, 1) == mem["boundary_activation_terabytes"]
    assert round(act / M["global_batch"] / 1e9, 1) == mem["boundary_activation_gigabytes_mb1"]


def test_flop_convention_reproduces_printed_throughput():
    t = G["throughput"]
    F = flops.paper_iteration_flops(M["global_batch"], M["seq"], M["layers"], M["hidden"], 51200)
    for gpus, secs, tf in zip(t["gpus"], t["iteration_seconds"], t["tflops_per_gpu"]):
        assert abs(F / secs / gpus / 1e12 - tf) < 1.0
    # per-layer: 4x our full-attention forward count equals the formula's per-layer part
    fwd = flops.layer_forward_flops(M["hidden"], M["heads"], M["hidden"] // M["heads"], 4 * M["hidden"],
                                    M["seq"], 1, attention="full")
    per_layer_formula = 96 * M["seq"] * M["hidden"] ** 2 * (1 + M["seq"] / (6 * M["hidden"]))
    assert abs(4 * fwd / per_layer_formula - 1) < 1e-12


def test_pipeline_efficiency_formula():
    pe = G["pipeline_efficiency"]
    for ratio, pct in zip(pe["ratios"], pe["efficiency_percent"]):
        mb = ratio * M["pipeline_parallel"]
        assert abs(100 * mb / (mb + M["pipeline_parallel"] - 1) - pct) < 1.0


def test_named_workloads_follow_the_paper_shapes():
    wl = inputs.WORKLOADS["mtnlg_tp8_stage"]
    assert wl.hidden == M["hidden"] and wl.seq == M["seq"]
    assert wl.heads == M["heads"] // M["tensor_parallel"]
    assert wl.head_dim == M["hidden"] // M["heads"] == 160
    assert wl.ffn == 4 * M["hidden"] // M["tensor_parallel"]
    assert wl.n_layers == M["layers"] // M["pipeline_parallel"] == 3
    assert 3 * wl.proj == 7680
    assert abs(wl.w_std - M["init_std"]) < 1e-12
    assert abs(math.sqrt(1 / (3 * M["hidden"])) - M["init_std"]) < 1e-4
    full = inputs.WORKLOADS["mtnlg_full_layer"]
    assert full.heads == M["heads"] and full.ffn == 4 * M["hidden"]
    # layer I/O tensor of one sequence: s*h*2 bytes = 83.9 MB
    assert wl.seq * wl.hidden * 2 == 83886080
    # step FLOPs (3x forward, causal count) of the benchmark workload
    assert abs(flops.step_model_flops(wl) / 2.339e13 - 1) < 1e-3
    assert abs(flops.step_model_flops(wl, "full") / 2.358e13 - 1) < 1e-3
    assert abs(flops.step_model_flops(inputs.WORKLOADS["gpt1p3b_layer"]) / 2.680e12 - 1) < 1e-3
    assert abs(flops.step_model_flops(inputs.WORKLOADS["tiny_fp32"]) / 1.259e9 - 1) < 1e-3


def test_generators_are_seeded_and_storage_rounded():
    wl = inputs.WORKLOADS["tiny_fp32"].with_(dtype="bf16")
    a = inputs.make_layer_params(wl, 0, seed=0)
    b = inputs.make_layer_params(wl, 0, seed=0)
    c = inputs.make_layer_params(wl, 1, seed=0)
    assert all(torch.equal(a[k], b[k]) for k in a)
    assert not torch.equal(a["w_qkv"], c["w_qkv"])
    assert a["w_qkv"].dtype == torch.bfloat16 and a["w_qkv"].shape == (768, 256)
    assert abs(a["w_fc1"].float().std().item() - 0.02) < 1e-3
    assert (a["ln1_g"] == 1).all() and (a["b_qkv"] == 0).all()
    r = inputs.make_layer_params(wl, 0, seed=0, affine="random")
    assert r["b_qkv"].float().abs().max() > 0 and torch.equal(r["w_qkv"], a["w_qkv"])
    x, dy = inputs.make_activations(wl, seed=0)
    assert x.shape == (2, 128, 256) and not torch.equal(x, dy)
    assert abs(x.float().std().item() - 1.0) < 0.02
