"""Transformer primitives in fp64 numpy.  Test infrastructure only.

The paper fixes none of these (it says "stacked transformer decoder", Section
3.2); they are the standard definitions for the block the workloads name:
pre-norm residual block, LayerNorm or RMSNorm, exact-erf GELU or SwiGLU,
learned absolute positions or rotary embedding.
"""

import numpy as np
from scipy.special import erf

F = np.float64


def layer_norm(x, gain, bias, eps):
    """LayerNorm over the last axis with the population variance."""
    mu = x.mean(axis=-1, keepdims=True)
    var = ((x - mu) ** 2).mean(axis=-1, keepdims=True)
    return (x - mu) / np.sqrt(var + eps) * gain + bias


def rms_norm(x, gain, eps):
    """RMSNorm over the last axis: x / sqrt(mean(x^2) + eps) * gain."""
    ms = (x * x).mean(axis=-1, keepdims=True)
    return x / np.sqrt(ms + eps) * gain


def gelu(x):
    """Exact GELU: x * Phi(x) with the Gaussian CDF written through erf."""
    return 0.5 * x * (1.0 + erf(x / np.sqrt(2.0)))


def silu(x):
    return x / (1.0 + np.exp(-x))


def rope(x, pos, base):
    """Rotary embedding, rotate-half pairing.

    x: [..., hd]; pos: scalar or array broadcastable to x[..., 0].
    Pair (j, j + hd/2) is rotated by the angle pos * base**(-2j/hd).
    """
    hd = x.shape[-1]
    half = hd // 2
    j = np.arange(half, dtype=F)
    theta = np.asarray(pos, dtype=F)[..., None] * base ** (-2.0 * j / hd)
    c, s = np.cos(theta), np.sin(theta)
    x1, x2 = x[..., :half], x[..., half:]
    return np.concatenate([x1 * c - x2 * s, x2 * c + x1 * s], axis=-1)


def softmax(s, axis=-1):
    m = s.max(axis=axis, keepdims=True)
    e = np.exp(s - m)
    return e / e.sum(axis=axis, keepdims=True)


def argmax_lowest(v):
    """Index of the maximum; the lowest index wins ties (Eq. 4: the most probable
    token; softmax is monotone so logits are compared directly)."""
    return int(np.argmax(v))  # numpy returns the first occurrence
