"""MI355X (gfx950) implementation of one GPU's tensor-parallel slice of a pre-LayerNorm GPT
decoder layer stack, forward and backward: a C-ABI library of hand-written HIP kernels
(include/mtnlg.h) and this thin ctypes binding.  PyTorch only provides device memory and streams."""
from .binding import *  # noqa: F401,F403
from . import binding, flops, inputs  # noqa: F401
