"""Pure-Python brute force of the RS-DGC sparsifier for tiny matrices.

A second, independent statement of the paper's definitions (Eqs. 6-12 and the
ranking of Algorithm 1), written with Python floats (IEEE double), lists and
``sorted`` only.  numpy is used solely to round to float32.  It exists to pin
the C oracle; it is far too slow for anything above ~32 x 32.
"""
import math

import numpy as np


def f32(x):
    return float(np.float32(x))


def brute_compress(g, r, p, alpha, rho):
    """g, r: lists of lists (R x C) of float32-representable floats."""
    R, C = len(g), len(g[0])
    h = (p - 1) // 2
    # Eq. 12 (u = g): v = r + g in float32
    v = [[f32(np.float32(r[x][y]) + np.float32(g[x][y])) for y in range(C)] for x in range(R)]

    def window(x0, y0):
        out = []
        for x in range(x0 - h, x0 + h + 1):
            for y in range(y0 - h, y0 + h + 1):
                out.append(v[x][y] if 0 <= x < R and 0 <= y < C else 0.0)
        assert len(out) == p * p
        return out

    nsi = []
    for x0 in range(R):
        for y0 in range(C):
            w = window(x0, y0)
            mean_abs = sum(abs(t) for t in w) / (p * p)          # Eq. 9
            mean = sum(w) / (p * p)
            std = math.sqrt(sum((t - mean) ** 2 for t in w) / (p * p))  # Eq. 10
            nsi.append(f32(alpha * mean_abs + (1.0 - alpha) * std))     # Eq. 8
    G = R * C
    k = math.ceil(G / (p * p) * rho)                             # Eq. 11
    k = max(0, min(G, k))
    order = sorted(range(G), key=lambda i: (-nsi[i], i))         # ranking, ties -> low index
    centres = sorted(order[:k])
    mask = [False] * G
    for c in centres:
        x0, y0 = divmod(c, C)
        for x in range(max(0, x0 - h), min(R, x0 + h + 1)):
            for y in range(max(0, y0 - h), min(C, y0 + h + 1)):
                mask[x * C + y] = True
    flat_v = [v[x][y] for x in range(R) for y in range(C)]
    idx = [i for i in range(G) if mask[i]]
    val = [flat_v[i] for i in idx]
    r_new = [0.0 if mask[i] else flat_v[i] for i in range(G)]
    return dict(v=flat_v, nsi=nsi, k=k, centres=centres, idx=idx, val=val, r_new=r_new,
                tau=(nsi[order[k - 1]] if k > 0 else None))
