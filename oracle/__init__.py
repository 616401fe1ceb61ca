"""CPU oracle for the RS-DGC local gradient compressor -- TEST INFRASTRUCTURE.

Thin ctypes layer over ``rsdgc_oracle.c`` (plain C, double-precision window
statistics, full-sort ranking).  Only the tests, the smoke check and the
benchmark's CPU-baseline leg may import this package; the GPU library and its
Python binding never do, and share no code with it.

Step numbering (used in the function names' docstrings) follows the paper:
Eq. 12 (accumulate), Eqs. 6-10 (NSI), Eq. 11 (k), Algorithm 1 (ranking),
Section III-C (keep whole neighbourhoods, emit indices), Eq. 12 (residual,
decompression).
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import List, NamedTuple, Optional, Sequence, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "rsdgc_oracle.c")
_LIB = os.path.join(_HERE, "librsdgc_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (no fast-math, no contraction)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c99", "-fPIC", "-shared", "-ffp-contract=off",
               "-fno-fast-math", "-Wall", "-Wextra", _SRC, "-o", _LIB, "-lm"]
        subprocess.check_call(cmd)
    return _LIB


def _load():
    global _lib
    if _lib is not None:
        return _lib
    build()
    lib = ctypes.CDLL(_LIB)
    i64, f64, c_int = ctypes.c_int64, ctypes.c_double, ctypes.c_int
    fp = ctypes.POINTER(ctypes.c_float)
    u32p = ctypes.POINTER(ctypes.c_uint32)
    u8p = ctypes.POINTER(ctypes.c_uint8)
    i64p = ctypes.POINTER(ctypes.c_int64)
    lib.rsdgc_oracle_accumulate.argtypes = [fp, fp, fp, i64]
    lib.rsdgc_oracle_accumulate.restype = None
    lib.rsdgc_oracle_nsi_at.argtypes = [fp, i64, i64, c_int, f64, i64, i64]
    lib.rsdgc_oracle_nsi_at.restype = f64
    lib.rsdgc_oracle_nsi.argtypes = [fp, i64, i64, c_int, f64, fp]
    lib.rsdgc_oracle_nsi.restype = None
    lib.rsdgc_oracle_k.argtypes = [i64, c_int, f64]
    lib.rsdgc_oracle_k.restype = i64
    lib.rsdgc_oracle_select.argtypes = [fp, i64, i64, u32p, fp]
    lib.rsdgc_oracle_select.restype = c_int
    lib.rsdgc_oracle_dilate.argtypes = [u32p, i64, i64, i64, c_int, u8p]
    lib.rsdgc_oracle_dilate.restype = None
    lib.rsdgc_oracle_emit.argtypes = [fp, u8p, i64, u32p, fp]
    lib.rsdgc_oracle_emit.restype = i64
    lib.rsdgc_oracle_residual.argtypes = [fp, u8p, i64, fp]
    lib.rsdgc_oracle_residual.restype = None
    lib.rsdgc_oracle_decompress.argtypes = [u32p, fp, i64, fp, i64, c_int]
    lib.rsdgc_oracle_decompress.restype = None
    lib.rsdgc_oracle_compress_layer.argtypes = [fp, fp, i64, i64, c_int, f64, f64,
                                                u32p, fp, u32p, i64p, fp, fp, fp]
    lib.rsdgc_oracle_compress_layer.restype = i64
    c_float = ctypes.c_float
    lib.rsdgc_oracle_momentum.argtypes = [fp, fp, fp, c_float, fp, fp, i64]
    lib.rsdgc_oracle_momentum.restype = None
    lib.rsdgc_oracle_mask_momentum.argtypes = [fp, u8p, i64, fp]
    lib.rsdgc_oracle_mask_momentum.restype = None
    lib.rsdgc_oracle_compress_layer_momentum.argtypes = [fp, fp, fp, c_float, i64, i64, c_int, f64, f64,
                                                         u32p, fp, u32p, ctypes.POINTER(i64),
                                                         ctypes.POINTER(c_float), fp, fp]
    lib.rsdgc_oracle_compress_layer_momentum.restype = i64
    lib.rsdgc_oracle_dynamic_ratios.argtypes = [fp, ctypes.POINTER(i64), ctypes.c_int32, f64,
                                                ctypes.POINTER(f64)]
    lib.rsdgc_oracle_dynamic_ratios.restype = c_int
    lib.rsdgc_oracle_apply.argtypes = [fp, i64, ctypes.c_int32, ctypes.POINTER(u32p), ctypes.POINTER(fp),
                                       ctypes.POINTER(i64), c_float]
    lib.rsdgc_oracle_apply.restype = c_int
    lib.rsdgc_oracle_apply_blocks.argtypes = [fp, i64, i64, c_int, ctypes.c_int32, ctypes.POINTER(u32p),
                                              ctypes.POINTER(fp), ctypes.POINTER(i64), c_float]
    lib.rsdgc_oracle_apply_blocks.restype = c_int
    lib.rsdgc_oracle_block_nsi.argtypes = [fp, i64, i64, c_int, f64, fp]
    lib.rsdgc_oracle_block_nsi.restype = None
    lib.rsdgc_oracle_compress_layer_blocks.argtypes = [fp, fp, i64, i64, c_int, f64, f64, u32p, fp,
                                                       ctypes.POINTER(c_float), fp, fp]
    lib.rsdgc_oracle_compress_layer_blocks.restype = i64
    lib.rsdgc_oracle_compress_layer_blocks_momentum.argtypes = [fp, fp, fp, c_float, i64, i64, c_int, f64, f64,
                                                                u32p, fp, ctypes.POINTER(c_float), fp, fp]
    lib.rsdgc_oracle_compress_layer_blocks_momentum.restype = i64
    lib.rsdgc_oracle_decompress_blocks.argtypes = [u32p, fp, i64, i64, i64, c_int, fp, c_int]
    lib.rsdgc_oracle_decompress_blocks.restype = None
    _lib = lib
    return lib


def _f32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float32)


def _p(a: np.ndarray, ctype):
    return a.ctypes.data_as(ctypes.POINTER(ctype))


def _check_p(p: int) -> None:
    if p < 1 or p % 2 == 0:
        raise ValueError("neighbourhood side p must be odd and >= 1")


# ------------------------------------------------------------------ steps
def accumulate(r, g) -> np.ndarray:
    """Eq. 12 line 2 (u = g): v = r + g, one float32 add per element."""
    r, g = _f32(r), _f32(g)
    assert r.shape == g.shape
    v = np.empty_like(r)
    _load().rsdgc_oracle_accumulate(_p(r, ctypes.c_float), _p(g, ctypes.c_float),
                                    _p(v, ctypes.c_float), r.size)
    return v


def nsi_at(v, p: int, alpha: float, x0: int, y0: int) -> float:
    """Eqs. 8-10 at one centre, in double (not rounded to float32)."""
    _check_p(p)
    v = _f32(v)
    R, C = v.shape
    return float(_load().rsdgc_oracle_nsi_at(_p(v, ctypes.c_float), R, C, p, float(alpha),
                                             int(x0), int(y0)))


def nsi(v, p: int, alpha: float) -> np.ndarray:
    """NSI map (float32) of one R x C layer."""
    _check_p(p)
    v = _f32(v)
    R, C = v.shape
    out = np.empty((R, C), dtype=np.float32)
    _load().rsdgc_oracle_nsi(_p(v, ctypes.c_float), R, C, p, float(alpha),
                             _p(out, ctypes.c_float))
    return out


def keep_count(G: int, p: int, rho: float) -> int:
    """Eq. 11: number of neighbourhoods kept in a layer of G elements."""
    _check_p(p)
    return int(_load().rsdgc_oracle_k(int(G), p, float(rho)))


def select(nsi_map, k: int) -> Tuple[np.ndarray, Optional[float]]:
    """Algorithm 1 ranking: indices (ascending) of the k top-ranked centres and
    the k-th largest score (None when k == 0)."""
    s = _f32(nsi_map).reshape(-1)
    k = int(k)
    centres = np.empty(max(k, 0), dtype=np.uint32)
    tau = ctypes.c_float(0.0)
    rc = _load().rsdgc_oracle_select(_p(s, ctypes.c_float), s.size, k,
                                     _p(centres, ctypes.c_uint32), ctypes.byref(tau))
    if rc != 0:
        raise MemoryError("oracle ranking ran out of memory")
    return centres, (float(tau.value) if k > 0 else None)


def dilate(centres, R: int, C: int, p: int) -> np.ndarray:
    """Mask (uint8, R x C) of all elements inside a selected neighbourhood."""
    _check_p(p)
    c = np.ascontiguousarray(centres, dtype=np.uint32)
    mask = np.empty((R, C), dtype=np.uint8)
    _load().rsdgc_oracle_dilate(_p(c, ctypes.c_uint32), c.size, R, C, p,
                                _p(mask, ctypes.c_uint8))
    return mask


def emit(v, mask) -> Tuple[np.ndarray, np.ndarray]:
    """Kept (index, value) pairs in ascending flat index."""
    v = _f32(v).reshape(-1)
    m = np.ascontiguousarray(mask, dtype=np.uint8).reshape(-1)
    cap = int(m.astype(bool).sum())
    idx = np.empty(cap, dtype=np.uint32)
    val = np.empty(cap, dtype=np.float32)
    n = _load().rsdgc_oracle_emit(_p(v, ctypes.c_float), _p(m, ctypes.c_uint8), v.size,
                                  _p(idx, ctypes.c_uint32), _p(val, ctypes.c_float))
    assert n == cap
    return idx, val


def residual(v, mask) -> np.ndarray:
    """r_new = 0 where sent, v elsewhere."""
    vv = _f32(v)
    m = np.ascontiguousarray(mask, dtype=np.uint8).reshape(-1)
    out = np.empty(vv.size, dtype=np.float32)
    _load().rsdgc_oracle_residual(_p(vv.reshape(-1), ctypes.c_float), _p(m, ctypes.c_uint8),
                                  vv.size, _p(out, ctypes.c_float))
    return out.reshape(vv.shape)


def decompress(idx, val, G: int, dense: Optional[np.ndarray] = None,
               accumulate_into: bool = False) -> np.ndarray:
    """Scatter pairs into a dense float32 vector of G elements."""
    idx = np.ascontiguousarray(idx, dtype=np.uint32)
    val = _f32(val)
    if dense is None:
        dense = np.zeros(G, dtype=np.float32)
    assert dense.dtype == np.float32 and dense.size == G and dense.flags.c_contiguous
    _load().rsdgc_oracle_decompress(_p(idx, ctypes.c_uint32), _p(val, ctypes.c_float),
                                    idx.size, _p(dense.reshape(-1), ctypes.c_float), G,
                                    1 if accumulate_into else 0)
    return dense


# ------------------------------------------------------------ whole layers
class LayerResult(NamedTuple):
    idx: np.ndarray       # uint32, ascending flat indices of kept elements
    val: np.ndarray       # float32, v at those indices
    centres: np.ndarray   # uint32, ascending flat indices of selected centres
    k: int                # Eq. 11
    tau: Optional[float]  # k-th largest NSI (float32 value), None if k == 0
    nsi: np.ndarray       # float32 R x C
    v: np.ndarray         # float32 R x C, accumulated gradient
    r_new: np.ndarray     # float32 R x C


def compress_layer(g, r, p: int, alpha: float, rho: float) -> LayerResult:
    """Steps 1-7 for one layer.  g, r: R x C float32; r is NOT modified."""
    _check_p(p)
    g = _f32(g)
    r_new = _f32(r).copy()
    assert g.ndim == 2 and g.shape == r_new.shape
    R, C = g.shape
    G = R * C
    k = keep_count(G, p, rho)
    cap = min(k * p * p, G)
    idx = np.empty(max(cap, 1), dtype=np.uint32)
    val = np.empty(max(cap, 1), dtype=np.float32)
    centres = np.empty(max(k, 1), dtype=np.uint32)
    k_out = ctypes.c_int64(0)
    tau = ctypes.c_float(0.0)
    nsi_map = np.empty((R, C), dtype=np.float32)
    v = np.empty((R, C), dtype=np.float32)
    n = _load().rsdgc_oracle_compress_layer(
        _p(g, ctypes.c_float), _p(r_new, ctypes.c_float), R, C, p, float(alpha), float(rho),
        _p(idx, ctypes.c_uint32), _p(val, ctypes.c_float), _p(centres, ctypes.c_uint32),
        ctypes.byref(k_out), ctypes.byref(tau), _p(nsi_map, ctypes.c_float),
        _p(v, ctypes.c_float))
    if n < 0:
        raise MemoryError("oracle ran out of memory")
    assert k_out.value == k
    return LayerResult(idx[:n].copy(), val[:n].copy(), centres[:k].copy(), k,
                       float(tau.value) if k > 0 else None, nsi_map, v, r_new)


def momentum_accumulate(u, g, r, m: float) -> Tuple[np.ndarray, np.ndarray]:
    """Eq. 12, lines 1-2: (u_new, v) with u_new = m*u + g and v = r + u_new, in float32."""
    u, g, r = _f32(u), _f32(g), _f32(r)
    assert u.shape == g.shape == r.shape
    u_new = np.empty_like(g)
    v = np.empty_like(g)
    _load().rsdgc_oracle_momentum(_p(u, ctypes.c_float), _p(g, ctypes.c_float), _p(r, ctypes.c_float),
                                  float(m), _p(u_new, ctypes.c_float), _p(v, ctypes.c_float), g.size)
    return u_new, v


def mask_momentum(u_new, mask) -> np.ndarray:
    """Momentum restarts from +0 where the accumulated gradient was sent."""
    u_new = _f32(u_new)
    mask = np.ascontiguousarray(mask, dtype=np.uint8)
    assert mask.size == u_new.size
    out = np.empty_like(u_new)
    _load().rsdgc_oracle_mask_momentum(_p(u_new, ctypes.c_float), _p(mask, ctypes.c_uint8), u_new.size,
                                       _p(out, ctypes.c_float))
    return out


class MomentumLayerResult(NamedTuple):
    layer: LayerResult    # as compress_layer (v is the momentum-corrected accumulation)
    u_new: np.ndarray     # float32 R x C, momentum after masking


def compress_layer_momentum(g, u, r, m: float, p: int, alpha: float, rho: float) -> MomentumLayerResult:
    """Steps 1m, 2-7 for one layer (Eq. 12 in full).  g, u, r: R x C float32; none is modified."""
    _check_p(p)
    g = _f32(g)
    u_new = _f32(u).copy()
    r_new = _f32(r).copy()
    assert g.ndim == 2 and g.shape == r_new.shape == u_new.shape
    R, C = g.shape
    G = R * C
    k = keep_count(G, p, rho)
    cap = min(k * p * p, G)
    idx = np.empty(max(cap, 1), dtype=np.uint32)
    val = np.empty(max(cap, 1), dtype=np.float32)
    centres = np.empty(max(k, 1), dtype=np.uint32)
    k_out = ctypes.c_int64(0)
    tau = ctypes.c_float(0.0)
    nsi_map = np.empty((R, C), dtype=np.float32)
    v = np.empty((R, C), dtype=np.float32)
    n = _load().rsdgc_oracle_compress_layer_momentum(
        _p(g, ctypes.c_float), _p(u_new, ctypes.c_float), _p(r_new, ctypes.c_float), float(m), R, C, p,
        float(alpha), float(rho), _p(idx, ctypes.c_uint32), _p(val, ctypes.c_float),
        _p(centres, ctypes.c_uint32), ctypes.byref(k_out), ctypes.byref(tau),
        _p(nsi_map, ctypes.c_float), _p(v, ctypes.c_float))
    if n < 0:
        raise MemoryError("oracle ran out of memory")
    assert k_out.value == k
    return MomentumLayerResult(
        LayerResult(idx[:n].copy(), val[:n].copy(), centres[:k].copy(), k,
                    float(tau.value) if k > 0 else None, nsi_map, v, r_new), u_new)


def dynamic_ratios(weights: Sequence[np.ndarray], rho: float) -> List[float]:
    """Eqs. 3-5: per-layer keep ratios from one ranking of |w| over all layers; rho is the global
    keep fraction, ceil(rho * G) weights survive, equal |w| rank by layer, then by index."""
    flat = [_f32(w).reshape(-1) for w in weights]
    off = np.zeros(len(flat) + 1, dtype=np.int64)
    off[1:] = np.cumsum([f.size for f in flat])
    w_all = np.concatenate(flat) if flat else np.zeros(0, dtype=np.float32)
    if w_all.size == 0:
        w_all = np.zeros(1, dtype=np.float32)
    out = (ctypes.c_double * len(flat))()
    rc = _load().rsdgc_oracle_dynamic_ratios(_p(w_all, ctypes.c_float),
                                             off.ctypes.data_as(ctypes.POINTER(ctypes.c_int64)),
                                             len(flat), float(rho), out)
    if rc != 0:
        raise MemoryError("oracle ran out of memory")
    return [float(x) for x in out]


def apply_messages(w, messages: Sequence[Tuple[np.ndarray, np.ndarray]], eta: float) -> np.ndarray:
    """Eq. 12, third line, for one layer: w - eta * (sum of the messages, first message first).
    messages: (idx uint32, val float32) per node.  Returns the new weights; w is not modified."""
    w_new = _f32(w).copy()
    flat = w_new.reshape(-1)
    n = len(messages)
    idxs = [np.ascontiguousarray(m[0], dtype=np.uint32) for m in messages]
    vals = [np.ascontiguousarray(m[1], dtype=np.float32) for m in messages]
    for i, v in zip(idxs, vals):
        assert i.size == v.size and (i.size == 0 or int(i.max()) < flat.size)
    pad_i, pad_v = np.zeros(1, np.uint32), np.zeros(1, np.float32)
    ip = (ctypes.POINTER(ctypes.c_uint32) * max(n, 1))(*[_p(i if i.size else pad_i, ctypes.c_uint32) for i in idxs])
    vp = (ctypes.POINTER(ctypes.c_float) * max(n, 1))(*[_p(v if v.size else pad_v, ctypes.c_float) for v in vals])
    cnt = (ctypes.c_int64 * max(n, 1))(*[i.size for i in idxs])
    rc = _load().rsdgc_oracle_apply(_p(flat, ctypes.c_float), flat.size, n, ip, vp, cnt, float(eta))
    if rc != 0:
        raise MemoryError("oracle ran out of memory")
    return w_new


# ------------------------------------------------ the block reading of Section III-C
def block_nsi(v, p: int, alpha: float) -> np.ndarray:
    """NSI of every non-overlapping p x p block: a ceil(R/p) x ceil(C/p) float32 map."""
    _check_p(p)
    v = _f32(v)
    R, C = v.shape
    out = np.empty(((R + p - 1) // p, (C + p - 1) // p), dtype=np.float32)
    _load().rsdgc_oracle_block_nsi(_p(v, ctypes.c_float), R, C, p, float(alpha), _p(out, ctypes.c_float))
    return out


def block_keep_count(G: int, p: int, rho: float, n_blocks: int) -> int:
    return min(keep_count(G, p, rho), n_blocks)


class BlockLayerResult(NamedTuple):
    blocks: np.ndarray    # uint32, ascending indices of the kept blocks (row-major over the block grid)
    val: np.ndarray       # float32, p*p values per kept block, row-major inside the block
    k: int
    tau: Optional[float]
    nsi: np.ndarray       # float32 block map
    v: np.ndarray
    r_new: np.ndarray


def compress_layer_blocks(g, r, p: int, alpha: float, rho: float) -> BlockLayerResult:
    """One layer under the block reading.  g, r: R x C float32; r is NOT modified."""
    _check_p(p)
    g = _f32(g)
    r_new = _f32(r).copy()
    R, C = g.shape
    BR, BC = (R + p - 1) // p, (C + p - 1) // p
    k = block_keep_count(R * C, p, rho, BR * BC)
    blocks = np.empty(max(k, 1), dtype=np.uint32)
    val = np.empty(max(k * p * p, 1), dtype=np.float32)
    tau = ctypes.c_float(0.0)
    nsi_map = np.empty((BR, BC), dtype=np.float32)
    v = np.empty((R, C), dtype=np.float32)
    n = _load().rsdgc_oracle_compress_layer_blocks(
        _p(g, ctypes.c_float), _p(r_new, ctypes.c_float), R, C, p, float(alpha), float(rho),
        _p(blocks, ctypes.c_uint32), _p(val, ctypes.c_float), ctypes.byref(tau),
        _p(nsi_map, ctypes.c_float), _p(v, ctypes.c_float))
    if n < 0:
        raise MemoryError("oracle ran out of memory")
    assert n == k
    return BlockLayerResult(blocks[:k].copy(), val[:k * p * p].copy(), k,
                            float(tau.value) if k > 0 else None, nsi_map, v, r_new)


class MomentumBlockLayerResult(NamedTuple):
    layer: BlockLayerResult   # v = r + u_new; everything else as in the plain block reading
    u_new: np.ndarray         # m*u + g, then +0 on every slot of a kept block


def compress_layer_blocks_momentum(g, u, r, m: float, p: int, alpha: float, rho: float) -> MomentumBlockLayerResult:
    """One layer under the block reading with Eq. 12's momentum.  g, u, r: R x C float32; none is modified."""
    _check_p(p)
    g = _f32(g)
    u_new = _f32(u).copy()
    r_new = _f32(r).copy()
    R, C = g.shape
    BR, BC = (R + p - 1) // p, (C + p - 1) // p
    k = block_keep_count(R * C, p, rho, BR * BC)
    blocks = np.empty(max(k, 1), dtype=np.uint32)
    val = np.empty(max(k * p * p, 1), dtype=np.float32)
    tau = ctypes.c_float(0.0)
    nsi_map = np.empty((BR, BC), dtype=np.float32)
    v = np.empty((R, C), dtype=np.float32)
    n = _load().rsdgc_oracle_compress_layer_blocks_momentum(
        _p(g, ctypes.c_float), _p(u_new, ctypes.c_float), _p(r_new, ctypes.c_float), ctypes.c_float(m),
        R, C, p, float(alpha), float(rho), _p(blocks, ctypes.c_uint32), _p(val, ctypes.c_float),
        ctypes.byref(tau), _p(nsi_map, ctypes.c_float), _p(v, ctypes.c_float))
    if n < 0:
        raise MemoryError("oracle ran out of memory")
    assert n == k
    return MomentumBlockLayerResult(
        BlockLayerResult(blocks[:k].copy(), val[:k * p * p].copy(), k, float(tau.value) if k > 0 else None,
                         nsi_map, v, r_new), u_new)


def decompress_blocks(blocks, val, R: int, C: int, p: int, dense: Optional[np.ndarray] = None,
                      accumulate_into: bool = False) -> np.ndarray:
    blocks = np.ascontiguousarray(blocks, dtype=np.uint32)
    val = np.ascontiguousarray(val, dtype=np.float32)
    assert val.size == blocks.size * p * p
    if dense is None:
        dense = np.zeros((R, C), dtype=np.float32)
    assert dense.dtype == np.float32 and dense.size == R * C and dense.flags.c_contiguous
    pad_b, pad_v = np.zeros(1, np.uint32), np.zeros(1, np.float32)
    _load().rsdgc_oracle_decompress_blocks(_p(blocks if blocks.size else pad_b, ctypes.c_uint32),
                                           _p(val if val.size else pad_v, ctypes.c_float), blocks.size,
                                           R, C, p, _p(dense.reshape(-1), ctypes.c_float),
                                           1 if accumulate_into else 0)
    return dense


def compress_model(grads: Sequence[np.ndarray], residuals: Sequence[np.ndarray], p: int,
                   alpha: float, ratios: Sequence[float]) -> List[LayerResult]:
    """All layers of one iteration, each independently (per-layer selection)."""
    assert len(grads) == len(residuals) == len(ratios)
    return [compress_layer(g, r, p, alpha, rho) for g, r, rho in zip(grads, residuals, ratios)]


def apply_block_messages(w, messages: Sequence[Tuple[np.ndarray, np.ndarray]], p: int, eta: float) -> np.ndarray:
    """Eq. 12, third line, for one layer and block messages: w - eta * (sum of the messages,
    first message first).  messages: (block indices uint32, p*p float32 values per block) per
    node.  Returns the new weights; w is not modified."""
    _check_p(p)
    w_new = _f32(w).copy()
    R, C = w_new.shape
    n_blocks = ((R + p - 1) // p) * ((C + p - 1) // p)
    n = len(messages)
    bs = [np.ascontiguousarray(m[0], dtype=np.uint32) for m in messages]
    vs = [np.ascontiguousarray(m[1], dtype=np.float32) for m in messages]
    for b, v in zip(bs, vs):
        assert v.size == b.size * p * p and (b.size == 0 or int(b.max()) < n_blocks)
    pad_b, pad_v = np.zeros(1, np.uint32), np.zeros(1, np.float32)
    bp = (ctypes.POINTER(ctypes.c_uint32) * max(n, 1))(*[_p(b if b.size else pad_b, ctypes.c_uint32) for b in bs])
    vp = (ctypes.POINTER(ctypes.c_float) * max(n, 1))(*[_p(v if v.size else pad_v, ctypes.c_float) for v in vs])
    cnt = (ctypes.c_int64 * max(n, 1))(*[b.size for b in bs])
    rc = _load().rsdgc_oracle_apply_blocks(_p(w_new.reshape(-1), ctypes.c_float), R, C, p, n, bp, vp, cnt,
                                           float(eta))
    if rc != 0:
        raise MemoryError("oracle ran out of memory")
    return w_new
