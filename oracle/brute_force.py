"""Element-by-element brute force of the DEF step for tiny d (d <= 64).

TEST INFRASTRUCTURE ONLY (part of the CPU oracle).

Written straight from the definitions of arXiv 2004.05298, Algorithm 1 and the
"Momentum Variant" of Sec. 3.2, with Python loops and dense vectors, as a
witness for the vectorised oracle: the kept index set is enumerated as
{(s + j) mod d : j = 0..B-1} (Sec. 1, RBGS: one start, one contiguous block),
C(p_k) is built as a dense d-vector, e_k <- p_k - C(p_k) is evaluated as a
subtraction, the all-reduce is a dense average of the C(p_k), and x <- x - C(p)
touches all d entries.  Scalars are numpy float32 (or float64) values so every
operation rounds once in that precision.
"""
from __future__ import annotations

import numpy as np


def brute_force_step(x, e, m, g, s, B, lr, mu, wd, dtype=np.float32):
    """One iteration on Python lists.  x: d values; e, m, g: W lists of d values.
    Returns (x_new, e_new, m_new, cbar_dense) as lists of `dtype` scalars."""
    ft = np.dtype(dtype).type
    d = len(x)
    W = len(g)
    lr, mu, wd = ft(lr), ft(mu), ft(wd)
    kept = set()
    for j in range(B):
        kept.add((s + j) % d)
    assert len(kept) == B
    e_new = [[None] * d for _ in range(W)]
    m_new = [[None] * d for _ in range(W)]
    compressed = [[None] * d for _ in range(W)]
    for k in range(W):
        for i in range(d):
            gi = ft(g[k][i])
            if wd != ft(0):
                gi = gi + wd * ft(x[i])
            if mu != ft(0):
                mi = mu * ft(m[k][i]) + gi
                m_new[k][i] = mi
            else:
                mi = gi
                m_new[k][i] = ft(m[k][i])
            p = lr * mi + ft(e[k][i])
            c = p if i in kept else ft(0)
            compressed[k][i] = c
            # p - C(p): p - p inside the block, p - 0 outside.  For finite p the
            # difference p - p is +0 under round-to-nearest.
            e_new[k][i] = p - c
    cbar = []
    for i in range(d):
        acc = ft(0)
        for k in range(W):
            acc = acc + compressed[k][i]
        cbar.append(acc / ft(W))
    x_new = [ft(x[i]) - cbar[i] for i in range(d)]
    return x_new, e_new, m_new, cbar
