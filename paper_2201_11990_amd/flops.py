"""FLOP and byte accounting for the layer slice (host arithmetic only).

A multiply-add counts as 2.  Forward of one layer over T = b*s tokens:
  GEMMs      2*T*h*(3p) + 2*T*p*h + 2*T*h*F + 2*T*F*h
  attention  4*b*p*s*(s+1)/2   ("causal": only the unmasked half is counted)
             4*b*p*s*s         ("full":   the whole s x s square)
Backward is counted as twice the forward, so a training step's model FLOPs are
3x forward; a recomputed forward adds a 4th that only "hardware FLOPs" count.

The paper's per-GPU throughput figures (Section 2.4, "System Performance
Evaluation": 126 / 121 / 113 TFLOP/s at 60.1 / 50.2 / 44.4 s per iteration on
2240 / 2800 / 3360 GPUs) are reproduced by the whole-model count
  96*B*s*L*h^2 * (1 + s/(6h) + V/(16*L*h)),
i.e. 4x forward with the full attention square; ``paper_iteration_flops`` is
that formula and is pinned against those printed figures in the tests.
"""


def layer_forward_flops(hidden, heads, head_dim, ffn, seq, micro_batch, attention="causal"):
    T, p = seq * micro_batch, heads * head_dim
    gemm = 2 * T * hidden * 3 * p + 2 * T * p * hidden + 2 * T * hidden * ffn + 2 * T * ffn * hidden
    if attention == "causal":
        attn = 4 * micro_batch * p * seq * (seq + 1) // 2
    elif attention == "full":
        attn = 4 * micro_batch * p * seq * seq
    else:
        raise ValueError(attention)
    return gemm + attn


def step_model_flops(wl, attention="causal"):
    """fwd + bwd model FLOPs of a stage step on workload ``wl`` (3x forward)."""
    return 3 * wl.n_layers * layer_forward_flops(wl.hidden, wl.heads, wl.head_dim, wl.ffn, wl.seq,
                                                 wl.micro_batch, attention)


def step_hardware_flops(wl, attention="causal"):
    """As step_model_flops, plus the recomputed forward when the workload recomputes."""
    mult = 4 if wl.recompute else 3
    return mult * wl.n_layers * layer_forward_flops(wl.hidden, wl.heads, wl.head_dim, wl.ffn,
                                                    wl.seq, wl.micro_batch, attention)


def layer_param_count(hidden, ffn):
    """Parameters of one unsliced layer: 4 h*h attention matrices, 2 h*F FFN matrices,
    their biases and the two LayerNorms."""
    return 4 * hidden * hidden + 2 * hidden * ffn + (3 * hidden + hidden + ffn + hidden) + 4 * hidden


def paper_iteration_flops(batch, seq, layers, hidden, vocab):
    return 96 * batch * seq * layers * hidden ** 2 * (1 + seq / (6 * hidden) + vocab / (16 * layers * hidden))


def boundary_activation_bytes(batch, layers, seq, hidden, bytes_per=2):
    """Section 2.1, "Memory Efficiency": batch x layers x seq x hidden x 2 bytes."""
    return batch * layers * seq * hidden * bytes_per


def hbm_bytes_per_launch(wl, bytes_per=2):
    """Algorithmic HBM bytes of one launch of each bandwidth-bound kernel class on workload ``wl`` (every operand
    read once, every result written once; statistics, gains and biases are negligible and not counted):
      LayerNorm forward   x in, LN(x) out                              2 T h
      LayerNorm backward  x, d(out), residual gradient in, dx out      4 T h   (its column sums are by-products)
      GeLU backward       z, dg in, dz out                             3 T F
      column sums         the matrix in; three per layer (T x h, T x F, T x 3p), averaged over a layer's launches
    in elements, times ``bytes_per``."""
    T, h, p, F = wl.tokens, wl.hidden, wl.heads * wl.head_dim, wl.ffn
    return {"ln_fwd": 2 * T * h * bytes_per, "ln_bwd": 4 * T * h * bytes_per, "gelu": 3 * T * F * bytes_per,
            "colsum": T * (h + F + 3 * p) * bytes_per / 3.0}
