"""Buffer allocation around mtnlg_stage_step / mtnlg_layer_fwd / mtnlg_layer_bwd.

Holds no arithmetic: it sizes and allocates the device buffers the C ABI asks the
caller to own (grads, saved activations, workspace) with torch.empty and passes
them through the binding.
"""
import torch

from . import binding as B
from .inputs import torch_dtype


class StageRunner:
    """Owns grads / saved / workspace for n_layers slices of workload ``wl`` on ``device``."""

    def __init__(self, wl, weights, flags=0, device="cuda", gelu=B.GELU_TANH):
        self.wl, self.weights = wl, weights
        self.desc = B.desc_from_workload(wl, flags=flags, gelu=gelu)
        st = B.mtnlg_layer_desc_check(self.desc)
        if st != 0:
            raise B.MtnlgError(st, "mtnlg_layer_desc_check")
        dt = torch_dtype(wl.dtype)
        gdt = torch.float32 if (flags & B.WGRAD_FP32) else dt
        self.grads = [{k: torch.zeros_like(v, dtype=gdt) for k, v in w.items()} for w in weights]
        self.saved = torch.empty(B.mtnlg_stage_saved_bytes(self.desc, len(weights)), dtype=torch.uint8,
                                 device=device)
        self.workspace = torch.empty(B.mtnlg_workspace_bytes(self.desc), dtype=torch.uint8, device=device)
        shape = (wl.micro_batch, wl.seq, wl.hidden)
        self.y = torch.empty(shape, dtype=dt, device=device)
        self.dx = torch.empty(shape, dtype=dt, device=device)
        self.args = B.StageArgs(self.desc, weights, self.grads)

    def step(self, x, dy, reduce=None):
        B.mtnlg_stage_step(self.desc, self.weights, x, dy, self.y, self.dx, self.grads, self.saved,
                           self.workspace, reduce=reduce, args=self.args)
        return self.y, self.dx, self.grads

    def step_accumulate(self, xs, dys, reduce=None):
        """xs, dys: [n_micro, b, s, h]; returns per-micro-batch y and dx and the summed grads."""
        ys, dxs = torch.empty_like(xs), torch.empty_like(xs)
        B.mtnlg_stage_step_accumulate(self.desc, self.weights, xs, dys, ys, dxs, self.grads, self.saved,
                                      self.workspace, reduce=reduce, args=self.args)
        return ys, dxs, self.grads


class LayerRunner:
    """Owns the buffers of a single layer's forward and backward."""

    def __init__(self, wl, weights, flags=0, device="cuda", gelu=B.GELU_TANH):
        self.wl, self.weights = wl, weights
        self.desc = B.desc_from_workload(wl, flags=flags, gelu=gelu)
        st = B.mtnlg_layer_desc_check(self.desc)
        if st != 0:
            raise B.MtnlgError(st, "mtnlg_layer_desc_check")
        dt = torch_dtype(wl.dtype)
        gdt = torch.float32 if (flags & B.WGRAD_FP32) else dt
        self.grads = {k: torch.zeros_like(v, dtype=gdt) for k, v in weights.items()}
        self.saved = torch.empty(B.mtnlg_saved_bytes(self.desc), dtype=torch.uint8, device=device)
        self.workspace = torch.empty(B.mtnlg_workspace_bytes(self.desc), dtype=torch.uint8, device=device)
        shape = (wl.micro_batch, wl.seq, wl.hidden)
        self.y = torch.empty(shape, dtype=dt, device=device)
        self.dx = torch.empty(shape, dtype=dt, device=device)

    def forward(self, x, reduce=None):
        B.mtnlg_layer_fwd(self.desc, self.weights, x, self.y, self.saved, self.workspace, reduce=reduce)
        return self.y

    def backward(self, x, dy, reduce=None):
        B.mtnlg_layer_bwd(self.desc, self.weights, x, self.saved, dy, self.dx, self.grads, self.workspace,
                          reduce=reduce)
        return self.dx, self.grads

    def saved_tensor(self, name):
        """View of one saved activation (for kernel-level checks)."""
        wl, L = self.wl, B.mtnlg_saved_layout_get(self.desc)
        T, h, p, F = wl.tokens, wl.hidden, wl.proj, wl.ffn
        dt = torch_dtype(wl.dtype)
        shapes = {"u1": (T, h), "qkv": (T, 3 * p), "a": (T, p), "x1": (T, h), "u2": (T, h), "z": (T, F),
                  "g": (T, F), "mu1": (T,), "rs1": (T,), "mu2": (T,), "rs2": (T,),
                  "lse": (wl.micro_batch, wl.heads, wl.seq)}
        edt = torch.float32 if name in ("mu1", "rs1", "mu2", "rs2", "lse") else dt
        shape = shapes[name]
        n = 1
        for v in shape:
            n *= v
        off = getattr(L, name)
        nbytes = n * torch.empty((), dtype=edt).element_size()
        return self.saved[off:off + nbytes].view(edt).view(shape)
