"""TEST INFRASTRUCTURE -- partial attention statistics and the softmax
re-scaling operator of Section 4.1, in fp64 numpy.

A partial is the triple ``(O~, m, l)`` of the un-scaled output, the row
maximum and the row sum of exponentials over one block of the context.  The
operator ``f`` merges two partials; ``finalize`` divides by ``l``.
Test support only: it lets the exact definition be checked by splitting the
context arbitrarily and merging in any bracketing.
"""
from __future__ import annotations

import numpy as np


def identity(D: int):
    """Initial state of Algorithm 1: O = 0, m = -inf, l = 0 (the unit of f)."""
    return np.zeros(D, dtype=np.float64), -np.inf, 0.0


def partial(q, k_block, v_block, scale):
    """Statistics of one context block (first display of Section 4.1).

    The paper's display omits the 1/sqrt(d) of Eq. 1; the scale is applied to
    the scores before the max and the exponential.
    """
    q = np.asarray(q, dtype=np.float64)
    k_block = np.asarray(k_block, dtype=np.float64)
    v_block = np.asarray(v_block, dtype=np.float64)
    if k_block.shape[0] == 0:
        return identity(q.shape[0])
    s = scale * (k_block @ q)          # S = Q K^T, one row
    m = float(np.max(s))               # m = rowmax(S)
    a = np.exp(s - m)                  # A = exp(S - m)
    l = float(np.sum(a))               # l = rowsum(A)
    o = a @ v_block                    # O~ = A V
    return o, m, l


def _weight(m_part: float, m_new: float) -> float:
    # e^{m_part - m_new}; a block that saw no score (m = -inf) weighs nothing,
    # including against another empty block where -inf - (-inf) is undefined.
    if m_part == -np.inf:
        return 0.0
    return float(np.exp(m_part - m_new))


def f(x, y):
    """Softmax re-scaling operator: merge two partials (second display, Section 4.1)."""
    ox, mx, lx = x
    oy, my, ly = y
    m = max(mx, my)
    wx, wy = _weight(mx, m), _weight(my, m)
    l = wx * lx + wy * ly
    o = wx * np.asarray(ox, dtype=np.float64) + wy * np.asarray(oy, dtype=np.float64)
    return o, m, l


def finalize(x):
    """O = diag(l)^-1 O~ and L = m + log(l)."""
    o, m, l = x
    if l == 0.0:
        return np.zeros_like(o), -np.inf
    return o / l, m + float(np.log(l))
