"""Seeded synthetic inputs and the named workload shapes.

This module holds none of the layer's arithmetic: it only names shapes and draws
random tensors.  Both the GPU path's callers (tests, benchmark) and the CPU
oracle's callers take their inputs from here, so both sides see the same values,
already rounded to the storage dtype.

Shapes come from Section 3.2 of the paper ("Model and Training Process": 105
layers, hidden 20480, 128 heads, sequence 2048, 8-way tensor and 35-way pipeline
parallelism, weight init N(0, 4.0e-3)); an FFN width of 4x hidden is the only
width consistent with the stated 530 billion parameters.
"""
from dataclasses import dataclass, replace

import torch


@dataclass(frozen=True)
class Workload:
    name: str
    hidden: int        # h
    heads: int         # n, local heads of the slice
    head_dim: int      # d
    ffn: int           # F, local FFN width of the slice
    seq: int           # s
    micro_batch: int   # b
    n_layers: int
    dtype: str         # "fp32" or "bf16" (storage; accumulation is fp32 on the GPU)
    w_std: float
    tp_size: int = 1
    recompute: bool = False

    @property
    def tokens(self):
        return self.seq * self.micro_batch

    @property
    def proj(self):
        return self.heads * self.head_dim

    def param_shapes(self):
        h, p, F = self.hidden, self.proj, self.ffn
        return {"ln1_g": (h,), "ln1_b": (h,), "w_qkv": (3 * p, h), "b_qkv": (3 * p,),
                "w_o": (h, p), "b_o": (h,), "ln2_g": (h,), "ln2_b": (h,),
                "w_fc1": (F, h), "b_fc1": (F,), "w_fc2": (h, F), "b_fc2": (h,)}

    def with_(self, **kw):
        return replace(self, **kw)


PARAM_NAMES = ("ln1_g", "ln1_b", "w_qkv", "b_qkv", "w_o", "b_o",
               "ln2_g", "ln2_b", "w_fc1", "b_fc1", "w_fc2", "b_fc2")

WORKLOADS = {
    # tiny unsliced layer, fp32 path
    "tiny_fp32": Workload("tiny_fp32", 256, 4, 64, 1024, 128, 2, 1, "fp32", 0.02),
    # GPT 1.3B-shaped unsliced layer
    "gpt1p3b_layer": Workload("gpt1p3b_layer", 2048, 16, 128, 8192, 2048, 4, 1, "bf16", 0.02),
    # MT-NLG: one GPU's share under 8-way tensor slicing and 35 pipeline stages (3 layers)
    "mtnlg_tp8_stage": Workload("mtnlg_tp8_stage", 20480, 16, 160, 10240, 2048, 1, 3, "bf16",
                                0.004, tp_size=8),
    # same, micro-batch 4, activations recomputed inside backward
    "mtnlg_tp8_stage_mb4_recompute": Workload("mtnlg_tp8_stage_mb4_recompute", 20480, 16, 160,
                                              10240, 2048, 4, 3, "bf16", 0.004, tp_size=8,
                                              recompute=True),
    # one whole MT-NLG layer, unsliced
    "mtnlg_full_layer": Workload("mtnlg_full_layer", 20480, 128, 160, 81920, 2048, 1, 1, "bf16",
                                 0.004),
}


def torch_dtype(name):
    return {"fp32": torch.float32, "bf16": torch.bfloat16}[name]


def _gen(device, seed, *stream):
    g = torch.Generator(device=device)
    key = seed
    for s in stream:
        key = (key * 1000003 + int(s) + 12345) % (2 ** 62)
    g.manual_seed(key)
    return g


_STREAM_ID = {n: i for i, n in enumerate(PARAM_NAMES)}


def make_layer_params(wl, layer, seed=0, device="cpu", affine="config"):
    """Parameters of layer ``layer`` in the storage dtype.

    affine="config": biases 0, LayerNorm gamma 1 / beta 0 (what the workloads state).
    affine="random": biases, gamma, beta drawn at random so that those paths carry signal.
    """
    dt = torch_dtype(wl.dtype)
    out = {}
    for name, shape in wl.param_shapes().items():
        g = _gen(device, seed, 1, layer, _STREAM_ID[name])
        if name.startswith("w_"):
            t = torch.randn(shape, generator=g, device=device, dtype=torch.float32) * wl.w_std
        elif affine == "random":
            t = torch.randn(shape, generator=g, device=device, dtype=torch.float32) * 0.1
            if name.endswith("_g"):
                t = t + 1.0
        else:
            t = torch.ones(shape, device=device) if name.endswith("_g") else torch.zeros(shape, device=device)
        out[name] = t.to(dt).contiguous()
    return out


def make_activations(wl, seed=0, device="cpu"):
    """Input hidden states x and upstream gradient dy, [b, s, h], N(0,1), storage dtype."""
    dt = torch_dtype(wl.dtype)
    shape = (wl.micro_batch, wl.seq, wl.hidden)
    x = torch.randn(shape, generator=_gen(device, seed, 2, 0), device=device, dtype=torch.float32)
    dy = torch.randn(shape, generator=_gen(device, seed, 2, 1), device=device, dtype=torch.float32)
    return x.to(dt).contiguous(), dy.to(dt).contiguous()
