"""Fixed-uniform-grid comparator (App. A, "Fixed Grid"; Prop. 1).  TEST INFRASTRUCTURE ONLY.

A plain GPTQ-style sweep whose per-(row, group) levels are lo + s*{0,..,2^k-1}:
the shape-invariant grid the paper's feasible-set argument compares against.
Written on its own (round-to-nearest on the integer grid, no level enumeration)
so that the variable-grid sweep of `bpdq_oracle` with coefficients frozen to
(lo, s, 2s, 4s, ...) can be checked against it bit for bit.
"""
from __future__ import annotations

import numpy as np


def uniform_grid(T, k):
    """Per-row asymmetric min/max grid of a group block: (lo, s), s = (hi-lo)/(2^k-1);
    a flat row gets s = 1 (every weight then rounds to code 0)."""
    T = np.asarray(T, dtype=np.float64)
    lo = T.min(axis=1)
    hi = T.max(axis=1)
    s = (hi - lo) / float((1 << k) - 1)
    s = np.where(s == 0.0, 1.0, s)
    return lo, s


def uniform_group(T, UL, k):
    """Column sweep of one group on the fixed uniform grid with error compensation
    (Eq. 3-4).  Returns dict(code, coef, What, E, it) like the BPDQ group solver;
    coef = (lo, s, 2s, ..., 2^(k-1) s) is the bit-plane form of the same grid."""
    T = np.asarray(T, dtype=np.float64)
    rows, g = T.shape
    lo, s = uniform_grid(T, k)
    qmax = (1 << k) - 1
    Wg = T.copy()
    code = np.zeros((rows, g), dtype=np.uint8)
    What = np.zeros((rows, g))
    E = np.zeros((rows, g))
    for l in range(g):
        z = np.clip(np.rint((Wg[:, l] - lo) / s), 0, qmax)
        code[:, l] = z.astype(np.uint8)
        What[:, l] = lo + s * z
        E[:, l] = (Wg[:, l] - What[:, l]) / UL[l, l]
        for j in range(l + 1, g):
            Wg[:, j] -= E[:, l] * UL[l, j]
    coef = np.stack([lo] + [s * (1 << i) for i in range(k)], axis=1)
    return dict(code=code, coef=coef, What=What, E=E, it=np.zeros(rows, dtype=np.int32))
