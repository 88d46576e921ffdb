"""Softmax attention over a key set from partial results over a partition of it.
Test infrastructure only.

For a chunk c of the keys let m_c = max score, l_c = sum exp(s - m_c),
o_c = sum exp(s - m_c) * v.  With m = max_c m_c the attention output over the
union is  sum_c exp(m_c - m) o_c  /  sum_c exp(m_c - m) l_c.  An empty chunk has
m_c = -inf, l_c = 0, o_c = 0 and drops out.  This is an exact identity of the
softmax, not an approximation.
"""

import numpy as np

F = np.float64


def partial(q, K, V, scale):
    """q [hd], K [n, hd], V [n, hd] -> (m, l, o)."""
    if K.shape[0] == 0:
        return -np.inf, 0.0, np.zeros(V.shape[1], dtype=F)
    s = (K @ q) * scale
    m = s.max()
    e = np.exp(s - m)
    return m, e.sum(), e @ V


def merge(parts):
    """parts: iterable of (m, l, o) -> attention output [hd]."""
    parts = list(parts)
    m = max(p[0] for p in parts)
    num = sum(np.exp(p[0] - m) * p[2] for p in parts if p[1] > 0)
    den = sum(np.exp(p[0] - m) * p[1] for p in parts if p[1] > 0)
    return num / den


def attention(q, K, V, scale):
    """Direct definition: softmax(K q * scale) V."""
    s = (K @ q) * scale
    e = np.exp(s - s.max())
    return (e / e.sum()) @ V
