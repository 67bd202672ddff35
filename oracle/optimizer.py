"""fp64 reference of the optimizer step on one rank's parameter slice (plain numpy, elementwise).

TEST INFRASTRUCTURE: only ``tests/`` may import this; the GPU library and its binding never do.

What the paper fixes (Section 3.2, model and training process): the Adam optimizer with
beta1 = 0.9, beta2 = 0.95, epsilon = 1e-8, the gradient norm clipped at 1.0, weight decay 0.1;
and (Section 2.1, memory efficiency) that weights and gradients exist in half precision for
forward/backward and as full-precision copies, next to the two Adam states, for the optimizer:
2 + 4 + 2 + 4 + 4 + 4 = 20 bytes per parameter.

Readings (the paper names the optimizer and its constants, not its equations):
  * Adam as published (Kingma and Ba): exponential moving averages of the gradient and of its
    square, both bias-corrected by 1 - beta^t with t counted from 1.
  * Weight decay in the decoupled form: lr * wd * p is subtracted from the full-precision
    weight next to the Adam update and does not enter the moments.  Which tensors decay is the
    caller's choice (the rate is an argument; the paper lists no exemptions).
  * Clipping: every gradient is multiplied by min(1, max_norm / (norm + 1e-6)) where norm is the
    L2 norm over ALL parameters of the model; a rank computes the squared norm of its own slice
    and the squared norms are summed over ranks before the square root (replicated tensors are
    the caller's business).
  * The half-precision weight used by the next forward pass is the full-precision weight rounded
    to nearest even.
"""
import numpy as np


def grad_sqnorm(grads):
    """Sum of squares over a list of gradient arrays (this rank's share of the global norm)."""
    return float(sum(np.sum(np.asarray(g, dtype=np.float64) ** 2) for g in grads))


def clip_coefficient(sqnorm, max_norm):
    """Factor applied to every gradient; max_norm <= 0 means no clipping."""
    if max_norm <= 0:
        return 1.0
    return min(1.0, max_norm / (np.sqrt(sqnorm) + 1e-6))


def adam_step(p, m, v, g, *, lr, beta1=0.9, beta2=0.95, eps=1e-8, weight_decay=0.1, step=1, clip_coef=1.0):
    """One update of full-precision weight p with moments m, v from gradient g (all fp64 arrays).
    Returns the new (p, m, v)."""
    p, m, v, g = (np.asarray(a, dtype=np.float64) for a in (p, m, v, g))
    g = g * clip_coef
    m = beta1 * m + (1.0 - beta1) * g
    v = beta2 * v + (1.0 - beta2) * g * g
    m_hat = m / (1.0 - beta1 ** step)
    v_hat = v / (1.0 - beta2 ** step)
    p = p - lr * (m_hat / (np.sqrt(v_hat) + eps) + weight_decay * p)
    return p, m, v
