"""fp64 reference of the first and last pipeline stage's extras (plain numpy; the matrix products and the
LayerNorm go through the same plain-loop C routines as the layer oracle).

TEST INFRASTRUCTURE: only ``tests/`` may import this; the GPU library and its binding never do.

The paper (Section 3.2) only says that the model is the GPT-2 transformer decoder, a left-to-right
autoregressive language model; it prints no equations and no vocabulary size.  Readings:
  * first stage: x[t] = E[token[t]] + P[position(t)], E the token embedding [V, h], P the learned
    position embedding [s, h] (GPT-2);
  * last stage: u = LayerNorm(x); logits = u E^T with the output projection tied to the token
    embedding (GPT-2); per-token loss = cross-entropy of softmax(logits) against the next token;
  * under tensor slicing (Section 2.1) the vocabulary is split in contiguous row blocks of E: a rank
    looks up only its own rows (zero elsewhere, summed over ranks, P added once after the sum) and
    computes logits for its own block; the softmax needs a maximum and two sums over ranks
    (sum of exponentials, the target's logit), the gradient of u one more sum.
``reduce(array, op)`` with op "sum" or "max" stands for those exchanges; None = a group of one.
"""
import numpy as np

from . import layernorm_bwd, layernorm_fwd, linear_dgrad, linear_fwd, linear_wgrad


def embedding_fwd(tokens, E, P, seq, vocab_start=0, reduce=None):
    """tokens [T] global ids (T = batch * seq, token-major); E [Vl, h] this rank's rows; P [seq, h]."""
    tokens = np.asarray(tokens, dtype=np.int64)
    E, P = np.asarray(E, dtype=np.float64), np.asarray(P, dtype=np.float64)
    T, (Vl, h) = tokens.shape[0], E.shape
    x = np.zeros((T, h))
    for t in range(T):
        v = tokens[t] - vocab_start
        if 0 <= v < Vl:
            x[t] = E[v]
    if reduce is not None:
        x = reduce(x, "sum")
    for t in range(T):
        x[t] += P[t % seq]
    return x


def embedding_bwd(tokens, dx, vocab_local, seq, vocab_start=0):
    """dE [Vl, h]: rows of dx summed per token id of this rank's block; dP [seq, h]: summed over the batch."""
    tokens = np.asarray(tokens, dtype=np.int64)
    dx = np.asarray(dx, dtype=np.float64)
    T, h = dx.shape
    dE, dP = np.zeros((vocab_local, h)), np.zeros((seq, h))
    for t in range(T):
        v = tokens[t] - vocab_start
        if 0 <= v < vocab_local:
            dE[v] += dx[t]
        dP[t % seq] += dx[t]
    return dE, dP


def cross_entropy_fwd(logits, targets, vocab_start=0, reduce=None):
    """Per-token loss from this rank's block of logits [T, Vl]; returns (loss [T], row maximum, sum of exponentials)."""
    logits = np.asarray(logits, dtype=np.float64)
    targets = np.asarray(targets, dtype=np.int64)
    T, Vl = logits.shape
    m = logits.max(axis=1)
    if reduce is not None:
        m = reduce(m, "max")
    s = np.exp(logits - m[:, None]).sum(axis=1)
    tl = np.zeros(T)
    for t in range(T):
        v = targets[t] - vocab_start
        if 0 <= v < Vl:
            tl[t] = logits[t, v]
    if reduce is not None:
        s, tl = reduce(s, "sum"), reduce(tl, "sum")
    return np.log(s) + m - tl, m, s


def cross_entropy_bwd(logits, targets, m, s, dloss, vocab_start=0):
    """Gradient of sum_t dloss[t] * loss[t] with respect to this rank's block of logits."""
    logits = np.asarray(logits, dtype=np.float64)
    targets = np.asarray(targets, dtype=np.int64)
    T, Vl = logits.shape
    d = np.exp(logits - m[:, None]) / s[:, None]
    for t in range(T):
        v = targets[t] - vocab_start
        if 0 <= v < Vl:
            d[t, v] -= 1.0
    return d * np.asarray(dloss, dtype=np.float64)[:, None]


def lm_head_step(x, gamma, beta, E, targets, dloss, vocab_start=0, eps=1e-5, reduce=None):
    """Final LayerNorm, tied output projection, cross-entropy, and the whole way back.
    Returns loss [T], dx [T, h], dgamma, dbeta, dE [Vl, h]."""
    u, mean, rstd = layernorm_fwd(x, gamma, beta, eps)
    logits = linear_fwd(u, E)
    loss, m, s = cross_entropy_fwd(logits, targets, vocab_start, reduce)
    dlogits = cross_entropy_bwd(logits, targets, m, s, dloss, vocab_start)
    du = linear_dgrad(dlogits, E)
    if reduce is not None:
        du = reduce(du, "sum")
    dE, _ = linear_wgrad(dlogits, u)
    dx, dgamma, dbeta = layernorm_bwd(x, gamma, mean, rstd, du)
    return loss, dx, dgamma, dbeta, dE
