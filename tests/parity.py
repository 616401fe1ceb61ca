"""GPU-versus-oracle comparison rule for one layer of one iteration.

Scores: the GPU evaluates the window statistics in double like the oracle but in a
different order, so float32 scores may differ in the last place.  The tolerance is
EPS = 1e-5 relative and nothing else (two zeros count as equal).

Selection: let tau be the oracle's k-th largest score, BAND the centres whose oracle
score is within EPS*tau of tau and HIGH the centres above the band.  The GPU must
select exactly k centres, all of HIGH, the rest from BAND.  Everything downstream is
then checked exactly: kept mask == dilation of the GPU's own centres, indices strictly
ascending, values bit-equal to v, residual bit-exact.  If the GPU's centres equal the
oracle's, every output must equal the oracle's byte for byte.
"""
from __future__ import annotations

import numpy as np
from scipy import ndimage

EPS = 1e-5


def nsi_close(gpu: np.ndarray, ref: np.ndarray):
    """Boolean map of scores within EPS relative of each other."""
    a = gpu.astype(np.float64)
    b = ref.astype(np.float64)
    return np.abs(a - b) <= EPS * np.maximum(np.abs(a), np.abs(b))


def dilate_np(centres: np.ndarray, R: int, C: int, p: int) -> np.ndarray:
    seed = np.zeros(R * C, dtype=bool)
    seed[centres] = True
    return ndimage.binary_dilation(seed.reshape(R, C), structure=np.ones((p, p), bool)).reshape(-1)


def check_layer(name, shape, p, k, tau, ref_nsi, ref_centres, ref_idx, ref_val, ref_r_new, v,
                gpu_idx, gpu_val, gpu_centres, gpu_ncentres, gpu_r_new):
    """Asserts the parity rule; returns True when the GPU output equals the oracle's exactly."""
    R, C = shape
    G = R * C
    v = np.asarray(v, dtype=np.float32).reshape(-1)
    gpu_r_new = np.asarray(gpu_r_new, dtype=np.float32).reshape(-1)
    # selection
    assert gpu_ncentres == k, f"{name}: selected {gpu_ncentres} centres, Eq. 11 gives {k}"
    assert len(gpu_centres) == k
    if k:
        assert np.all(np.diff(gpu_centres.astype(np.int64)) > 0), f"{name}: centres not ascending"
        assert int(gpu_centres[-1]) < G
    exact = np.array_equal(gpu_centres, ref_centres)
    if not exact:
        s = ref_nsi.reshape(-1).astype(np.float64)
        t = float(tau)
        band = np.abs(s - t) <= EPS * t
        high = s > t * (1.0 + EPS)
        sel = np.zeros(G, dtype=bool)
        sel[gpu_centres] = True
        assert np.all(sel[high]), f"{name}: a centre above the tolerance band was not selected"
        assert np.all((high | band)[sel]), f"{name}: a centre below the tolerance band was selected"
    # kept elements = dilation of the GPU's own centres
    mask = dilate_np(gpu_centres, R, C, p) if k else np.zeros(G, dtype=bool)
    want_idx = np.flatnonzero(mask).astype(np.uint32)
    assert np.array_equal(gpu_idx, want_idx), f"{name}: kept indices are not the dilation of the centres"
    assert np.array_equal(gpu_val.view(np.uint32), v[want_idx].view(np.uint32)), f"{name}: values differ from v"
    assert k <= len(gpu_idx) <= min(k * p * p, G) or k == 0
    # residual: +0 where sent, v elsewhere (bitwise)
    want_r = v.copy()
    want_r[want_idx] = 0.0
    assert np.array_equal(gpu_r_new.view(np.uint32), want_r.view(np.uint32)), f"{name}: residual differs"
    if exact:
        assert np.array_equal(gpu_idx, ref_idx)
        assert np.array_equal(gpu_val.view(np.uint32), ref_val.view(np.uint32))
        assert np.array_equal(gpu_r_new.view(np.uint32), ref_r_new.reshape(-1).view(np.uint32))
    return exact
