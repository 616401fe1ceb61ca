"""Pins for the CPU oracle: what the paper and the mathematics fix.

No GPU, no GPU library.  Each test states which definition it pins:
Eqs. 6-10 (NSI), Eq. 11 (k), Algorithm 1 (ranking), Section III-C (whole
neighbourhoods kept, indices transmitted), Eq. 12 (accumulation / residual).
"""
import math
import os
from fractions import Fraction

import hypothesis
import hypothesis.strategies as st
import numpy as np
import pytest
from scipy import ndimage

import oracle
from tests.brute import brute_compress

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _rows(name):
    with open(os.path.join(GOLDEN, name)) as f:
        return [ln.split() for ln in f if ln.strip() and not ln.startswith("#")]


# ---------------------------------------------------------------- Eq. 11
def test_keep_count_golden():
    for G, p, rho, k in _rows("eq11_keep_counts.txt"):
        assert oracle.keep_count(int(G), int(p), float(rho)) == int(k)


def test_keep_count_matches_exact_rational_away_from_integers():
    rng = np.random.default_rng(11)
    for _ in range(500):
        G = int(rng.integers(1, 10 ** 8))
        p = int(rng.choice([1, 3, 5, 7]))
        rho = float(rng.choice([1e-3, 0.01, 0.02, 0.05, 0.37, 1.0]))
        exact = Fraction(G, p * p) * Fraction(rho)
        if abs(exact - round(exact)) < Fraction(1, 10 ** 6):
            continue  # borderline: double rounding may legitimately decide
        want = min(G, max(0, math.ceil(exact)))
        assert oracle.keep_count(G, p, rho) == want


def test_keep_count_clamps():
    assert oracle.keep_count(100, 3, 0.0) == 0
    assert oracle.keep_count(5, 1, 1.0) == 5
    assert oracle.keep_count(4, 3, 1.0) == 1          # ceil(4/9)
    with pytest.raises(ValueError):
        oracle.keep_count(100, 2, 0.5)                # even p rejected


# ------------------------------------------------------------ Eq. 12 add
def test_accumulate_is_one_float32_add():
    rng = np.random.default_rng(0)
    r = rng.standard_normal(10000).astype(np.float32)
    g = (rng.standard_normal(10000) * 1e-3).astype(np.float32)
    v = oracle.accumulate(r, g)
    assert v.dtype == np.float32
    assert np.array_equal(v, r + g)                   # numpy float32 add
    # round-to-nearest-even cases with known answers
    one, ulp = np.float32(1.0), np.float32(2.0 ** -23)
    r2 = np.array([1.0, 1.0, 1.0], dtype=np.float32)
    g2 = np.array([2.0 ** -24, 3 * 2.0 ** -25, 2.0 ** -25], dtype=np.float32)
    got = oracle.accumulate(r2, g2)
    assert got[0] == one                               # tie -> even
    assert got[1] == one + ulp                         # above the tie
    assert got[2] == one                               # below the tie


# --------------------------------------------------- Eqs. 8-10 closed forms
@pytest.mark.parametrize("alpha", [0.0, 0.25, 0.5, 1.0])
@pytest.mark.parametrize("c", [1.0, -3.5, 2.0 ** -10])
def test_nsi_constant_matrix_closed_forms(alpha, c):
    forms = {r[0]: (float(r[2]), float(r[3])) for r in _rows("nsi_closed_forms.txt") if r[1] == "3"}
    v = np.full((7, 9), c, dtype=np.float32)
    m = oracle.nsi(v, 3, alpha).astype(np.float64)

    def want(case):
        A, S = forms[case]
        return abs(c) * (alpha * A + (1 - alpha) * S)

    assert np.allclose(m[1:-1, 1:-1], want("constant_interior"), rtol=1e-6, atol=1e-12)
    for (x, y) in [(0, 0), (0, 8), (6, 0), (6, 8)]:
        assert m[x, y] == pytest.approx(want("constant_corner"), rel=1e-6)
    assert np.allclose(m[0, 1:-1], want("constant_edge"), rtol=1e-6)
    assert np.allclose(m[-1, 1:-1], want("constant_edge"), rtol=1e-6)
    assert np.allclose(m[1:-1, 0], want("constant_edge"), rtol=1e-6)
    assert np.allclose(m[1:-1, -1], want("constant_edge"), rtol=1e-6)
    # all centres of one class tie exactly
    assert len(set(m[1:-1, 1:-1].ravel().tolist())) == 1
    assert len(set(m[0, 1:-1].tolist())) == 1


@pytest.mark.parametrize("p", [3, 5, 7])
@pytest.mark.parametrize("alpha", [0.0, 0.5, 1.0])
def test_nsi_single_impulse(p, alpha):
    forms = {int(r[1]): (float(r[2]), float(r[3])) for r in _rows("nsi_closed_forms.txt")
             if r[0] == "impulse"}
    a, R, C = -0.75, 23, 29
    h = (p - 1) // 2
    x0, y0 = 11, 14
    v = np.zeros((R, C), dtype=np.float32)
    v[x0, y0] = a
    m = oracle.nsi(v, p, alpha).astype(np.float64)
    A, S = forms[p]
    want = abs(a) * (alpha * A + (1 - alpha) * S)
    inside = np.zeros((R, C), bool)
    inside[x0 - h:x0 + h + 1, y0 - h:y0 + h + 1] = True
    assert inside.sum() == p * p
    assert np.allclose(m[inside], want, rtol=1e-6)
    assert np.all(m[~inside] == 0.0)
    # k = 1 keeps the top-left centre whose window holds the impulse; p*p pairs out
    rho = 1.0 * p * p / (R * C) * 0.999
    res = oracle.compress_layer(v, np.zeros_like(v), p, alpha, rho)
    if want > 0:
        assert res.k == 1
        assert res.centres.tolist() == [(x0 - h) * C + (y0 - h)]
        assert len(res.idx) == p * p
        assert (x0 * C + y0) in res.idx.tolist()
        assert np.all(res.r_new == 0.0)


@pytest.mark.parametrize("alpha", [0.0, 0.5, 1.0])
def test_nsi_checkerboard_interior(alpha):
    forms = {r[0]: (float(r[2]), float(r[3])) for r in _rows("nsi_closed_forms.txt")}
    c = 0.125
    xs, ys = np.meshgrid(np.arange(10), np.arange(12), indexing="ij")
    v = np.where((xs + ys) % 2 == 0, c, -c).astype(np.float32)
    m = oracle.nsi(v, 3, alpha).astype(np.float64)
    A, S = forms["checker_interior"]
    assert np.allclose(m[1:-1, 1:-1], c * (alpha * A + (1 - alpha) * S), rtol=1e-6)


# ---------------------------- alpha = 1 / alpha = 0 against library box filters
@pytest.mark.parametrize("p", [1, 3, 5, 9])
@pytest.mark.parametrize("shape", [(37, 53), (5, 64), (64, 3), (1, 40), (2, 2)])
def test_nsi_alpha_extremes_against_uniform_filter(p, shape):
    rng = np.random.default_rng(hash((p,) + shape) % 2 ** 32)
    v = (rng.standard_normal(shape) + 0.7).astype(np.float32)
    v64 = v.astype(np.float64)
    box_abs = ndimage.uniform_filter(np.abs(v64), size=p, mode="constant", cval=0.0)
    box = ndimage.uniform_filter(v64, size=p, mode="constant", cval=0.0)
    box_sq = ndimage.uniform_filter(v64 * v64, size=p, mode="constant", cval=0.0)
    std = np.sqrt(np.maximum(box_sq - box * box, 0.0))
    got1 = oracle.nsi(v, p, 1.0).astype(np.float64)
    got0 = oracle.nsi(v, p, 0.0).astype(np.float64)
    assert np.allclose(got1, box_abs, rtol=2e-7, atol=1e-30)
    assert np.allclose(got0, std, rtol=1e-6, atol=1e-7)
    mix = oracle.nsi(v, p, 0.3).astype(np.float64)
    assert np.allclose(mix, 0.3 * box_abs + 0.7 * std, rtol=1e-6, atol=1e-7)


def test_nsi_at_agrees_with_map_and_is_double():
    rng = np.random.default_rng(5)
    v = rng.standard_normal((19, 23)).astype(np.float32)
    m = oracle.nsi(v, 5, 0.4)
    for (x, y) in [(0, 0), (18, 22), (7, 0), (9, 11)]:
        d = oracle.nsi_at(v, 5, 0.4, x, y)
        assert np.float32(d) == m[x, y]


# ------------------------------------------------------------- symmetries
def test_nsi_symmetries():
    rng = np.random.default_rng(8)
    v = (rng.standard_normal((31, 17)) * 1e-3).astype(np.float32)
    base = oracle.nsi(v, 3, 0.5)
    assert np.array_equal(oracle.nsi(v * np.float32(8.0), 3, 0.5), base * np.float32(8.0))
    assert np.array_equal(oracle.nsi(v * np.float32(2.0 ** -7), 3, 0.5), base * np.float32(2.0 ** -7))
    assert np.allclose(oracle.nsi(-v, 3, 0.5), base, rtol=1e-6)
    assert np.allclose(oracle.nsi(np.ascontiguousarray(v.T), 3, 0.5), base.T, rtol=1e-6)
    # power-of-two scaling leaves the selection unchanged
    a = oracle.compress_layer(v, np.zeros_like(v), 3, 0.5, 0.1)
    b = oracle.compress_layer(v * np.float32(4.0), np.zeros_like(v), 3, 0.5, 0.1)
    assert np.array_equal(a.centres, b.centres) and np.array_equal(a.idx, b.idx)


# ------------------------------------------- p = 1: plain magnitude top-k
@pytest.mark.parametrize("alpha", [1.0, 0.5])
def test_p1_is_magnitude_topk(alpha):
    rng = np.random.default_rng(3)
    v = rng.standard_normal((40, 50)).astype(np.float32)
    v[3, 4] = v[20, 1] = v[39, 49] = np.float32(9.0)      # exact ties at the top
    v[10, 10] = np.float32(-9.0)
    rho = 0.013
    res = oracle.compress_layer(v, np.zeros_like(v), 1, alpha, rho)
    G = v.size
    k = math.ceil(G * rho)
    assert res.k == k
    order = np.argsort(-np.abs(v.ravel()), kind="stable")   # library sort, stable
    want = np.sort(order[:k]).astype(np.uint32)
    assert np.array_equal(res.centres, want)
    assert np.array_equal(res.idx, want)                     # window = the element itself
    assert np.array_equal(res.val, v.ravel()[want])


def test_ranking_ties_go_to_lower_index_and_count_is_exact():
    v = np.full((6, 6), 2.0, dtype=np.float32)
    # alpha = 1: interior (4x4 = 16 centres) ranks above edges and corners
    res = oracle.compress_layer(v, np.zeros_like(v), 3, 1.0, 9 * 5 / 36.0)   # k = 5
    assert res.k == 5
    interior = [x * 6 + y for x in range(1, 5) for y in range(1, 5)]
    assert res.centres.tolist() == interior[:5]
    # all-zero matrix: every score ties at 0; the first k indices win
    z = np.zeros((5, 7), dtype=np.float32)
    res = oracle.compress_layer(z, z, 3, 0.5, 0.5)
    assert res.centres.tolist() == list(range(res.k)) and res.k == math.ceil(35 / 9 * 0.5)


def test_select_against_full_sort():
    rng = np.random.default_rng(21)
    s = rng.integers(0, 50, size=5000).astype(np.float32)    # many ties
    for k in [0, 1, 17, 500, 5000]:
        centres, tau = oracle.select(s, k)
        order = sorted(range(s.size), key=lambda i: (-float(s[i]), i))
        assert centres.tolist() == sorted(order[:k])
        if k:
            assert tau == float(s[order[k - 1]])
        else:
            assert tau is None


# --------------------------------------------------------------- dilation
@pytest.mark.parametrize("p", [1, 3, 5])
def test_dilate_against_library_binary_dilation(p):
    rng = np.random.default_rng(p)
    R, C = 33, 47
    centres = np.sort(rng.choice(R * C, size=25, replace=False)).astype(np.uint32)
    seed = np.zeros((R, C), bool)
    seed.ravel()[centres] = True
    want = ndimage.binary_dilation(seed, structure=np.ones((p, p), bool))
    got = oracle.dilate(centres, R, C, p).astype(bool)
    assert np.array_equal(got, want)


def test_isolated_centres_emit_exactly_k_p_squared():
    # impulses >= p apart and away from the border: each selected window is whole
    R, C, p = 40, 40, 3
    v = np.zeros((R, C), dtype=np.float32)
    pts = [(5, 5), (5, 20), (20, 9), (30, 30)]
    for i, (x, y) in enumerate(pts):
        v[x, y] = 1.0 + i
    # each impulse yields p*p tied centres; k = 4 picks the 4 largest-impulse windows'
    # top-left centres one impulse at a time only if k walks down the impulses:
    res = oracle.compress_layer(v, np.zeros_like(v), p, 0.5, 1 * 9 / 1600.0 * 0.999)  # k = 1
    assert res.k == 1 and len(res.idx) == 9
    # k <= n <= min(k p^2, G) in general
    rng = np.random.default_rng(0)
    g = rng.standard_normal((R, C)).astype(np.float32)
    res = oracle.compress_layer(g, np.zeros_like(g), p, 0.5, 0.05)
    assert res.k <= len(res.idx) <= min(res.k * 9, R * C)


# ------------------------------------------------ invariants of one iteration
@pytest.mark.parametrize("p,alpha,rho", [(3, 0.5, 0.02), (5, 0.25, 0.1), (1, 1.0, 0.3), (3, 0.0, 1.0)])
def test_sent_plus_residual_is_accumulated_gradient(p, alpha, rho):
    rng = np.random.default_rng(17)
    g = (rng.standard_normal((45, 61)) * 1e-3).astype(np.float32)
    r = (rng.standard_normal((45, 61)) * 1e-3).astype(np.float32)
    res = oracle.compress_layer(g, r, p, alpha, rho)
    v = r + g
    assert np.array_equal(res.v, v)
    dense = oracle.decompress(res.idx, res.val, v.size).reshape(v.shape)
    assert np.array_equal((dense + res.r_new).view(np.uint32), v.view(np.uint32)) or \
        np.array_equal(dense + res.r_new, v)
    assert np.all(res.r_new.ravel()[res.idx] == 0.0)
    assert not np.any(np.signbit(res.r_new.ravel()[res.idx]))        # +0, not -0
    assert np.all(np.diff(res.idx.astype(np.int64)) > 0)
    assert np.array_equal(res.val, v.ravel()[res.idx])
    assert len(res.centres) == res.k == oracle.keep_count(v.size, p, rho)
    # mask is exactly the dilation of the centres
    mask = oracle.dilate(res.centres, 45, 61, p).astype(bool).ravel()
    assert np.array_equal(np.flatnonzero(mask).astype(np.uint32), res.idx)
    # every selected centre ranks at or above tau, every other at or below
    s = res.nsi.ravel()
    sel = np.zeros(v.size, bool)
    sel[res.centres] = True
    if res.k:
        assert s[sel].min() == np.float32(res.tau)
        if (~sel).any():
            assert s[~sel].max() <= np.float32(res.tau)


def test_zero_ratio_sends_nothing():
    rng = np.random.default_rng(1)
    g = rng.standard_normal((9, 9)).astype(np.float32)
    res = oracle.compress_layer(g, np.zeros_like(g), 3, 0.5, 0.0)
    assert res.k == 0 and len(res.idx) == 0 and res.tau is None
    assert np.array_equal(res.r_new, g)


def test_decompress_overwrite_and_accumulate():
    idx = np.array([1, 4, 7], dtype=np.uint32)
    val = np.array([0.5, -2.0, 3.0], dtype=np.float32)
    d = oracle.decompress(idx, val, 10)
    assert d.tolist() == [0, 0.5, 0, 0, -2.0, 0, 0, 3.0, 0, 0]
    d = oracle.decompress(idx, val, 10, dense=d, accumulate_into=True)
    assert d.tolist() == [0, 1.0, 0, 0, -4.0, 0, 0, 6.0, 0, 0]
    d2 = np.full(10, 7.0, dtype=np.float32)
    oracle.decompress(idx, val, 10, dense=d2, accumulate_into=False)   # overwrite clears
    assert d2.tolist() == [0, 0.5, 0, 0, -2.0, 0, 0, 3.0, 0, 0]


def test_two_iterations_carry_the_residual():
    rng = np.random.default_rng(4)
    g0 = (rng.standard_normal((24, 24)) * 1e-3).astype(np.float32)
    g1 = (rng.standard_normal((24, 24)) * 1e-3).astype(np.float32)
    a = oracle.compress_layer(g0, np.zeros_like(g0), 3, 0.5, 0.05)
    b = oracle.compress_layer(g1, a.r_new, 3, 0.5, 0.05)
    assert np.array_equal(b.v, a.r_new + g1)
    sent = oracle.decompress(a.idx, a.val, g0.size) + oracle.decompress(b.idx, b.val, g0.size)
    total = (g0.astype(np.float64) + g1.astype(np.float64)).ravel()
    assert np.allclose(sent.astype(np.float64) + b.r_new.ravel(), total, atol=4 * 2.0 ** -23 * np.abs(total).max())


# ------------------------------------------------------------ brute force
@pytest.mark.parametrize("R,C,p,alpha,rho,seed", [
    (8, 8, 3, 0.5, 0.2, 0), (13, 7, 3, 0.25, 0.5, 1), (5, 16, 5, 0.5, 0.3, 2),
    (16, 5, 5, 0.75, 1.0, 3), (1, 20, 3, 0.5, 0.4, 4), (20, 1, 3, 0.5, 0.4, 5),
    (2, 2, 5, 0.5, 1.0, 6), (12, 12, 1, 0.5, 0.1, 7), (24, 31, 3, 0.0, 0.05, 8),
    (32, 32, 7, 0.5, 0.05, 9),
])
def test_oracle_against_pure_python_brute_force(R, C, p, alpha, rho, seed):
    rng = np.random.default_rng(seed)
    g = (rng.standard_normal((R, C)) * 1e-2).astype(np.float32)
    r = (rng.standard_normal((R, C)) * 1e-2).astype(np.float32)
    if seed % 2:                       # plant exact ties and zeros
        g[0, :] = 0.0
        r[0, :] = 0.0
        g[-1, :] = g[-1, 0]
        r[-1, :] = r[-1, 0]
    b = brute_compress(g.tolist(), r.tolist(), p, alpha, rho)
    o = oracle.compress_layer(g, r, p, alpha, rho)
    assert o.k == b["k"]
    assert o.v.ravel().tolist() == b["v"]
    # scores: both are double evaluations rounded to float32; summation order inside the
    # window is the same (row-major), so they agree to the last bit or one ulp
    assert np.allclose(o.nsi.ravel(), np.array(b["nsi"], dtype=np.float32), rtol=2e-7, atol=1e-30)
    if np.array_equal(o.nsi.ravel(), np.array(b["nsi"], dtype=np.float32)):
        assert o.centres.tolist() == b["centres"]
        assert o.idx.tolist() == b["idx"]
        assert o.val.tolist() == b["val"]
        assert o.r_new.ravel().tolist() == b["r_new"]
        if b["k"]:
            assert o.tau == b["tau"]
    else:  # pragma: no cover - only if the two double evaluations round differently
        pytest.skip("score rounding differed between C and Python doubles")


@hypothesis.settings(max_examples=60, deadline=None, derandomize=True)
@hypothesis.given(R=st.integers(1, 12), C=st.integers(1, 12), p=st.sampled_from([1, 3, 5, 7]),
                  alpha=st.sampled_from([0.0, 0.25, 0.5, 1.0]), rho=st.sampled_from([0.0, 0.01, 0.1, 0.3, 0.7, 1.0]),
                  few_values=st.booleans(), seed=st.integers(0, 2 ** 16))
def test_oracle_against_brute_force_on_drawn_cases(R, C, p, alpha, rho, few_values, seed):
    """The same comparison on drawn shapes, neighbourhood sides, mixes and ratios; half of the
    inputs take only five distinct values, so equal scores (and the index tie rule) are common."""
    rng = np.random.default_rng(seed)
    if few_values:
        g = rng.integers(-2, 3, size=(R, C)).astype(np.float32) * np.float32(0.125)
        r = rng.integers(-1, 2, size=(R, C)).astype(np.float32) * np.float32(0.25)
    else:
        g = (rng.standard_normal((R, C)) * 1e-2).astype(np.float32)
        r = (rng.standard_normal((R, C)) * 1e-2).astype(np.float32)
    b = brute_compress(g.tolist(), r.tolist(), p, alpha, rho)
    o = oracle.compress_layer(g, r, p, alpha, rho)
    assert o.k == b["k"]
    assert o.v.ravel().tolist() == b["v"]
    assert np.allclose(o.nsi.ravel(), np.array(b["nsi"], dtype=np.float32), rtol=2e-7, atol=1e-30)
    hypothesis.assume(np.array_equal(o.nsi.ravel(), np.array(b["nsi"], dtype=np.float32)))
    assert o.centres.tolist() == b["centres"]
    assert o.idx.tolist() == b["idx"]
    assert o.val.tolist() == b["val"]
    assert o.r_new.ravel().tolist() == b["r_new"]


# ------------------------------------------------- momentum correction (Eq. 12 in full)
def test_momentum_is_one_rounded_multiply_then_one_rounded_add():
    rng = np.random.default_rng(21)
    u = rng.standard_normal(20000).astype(np.float32)
    g = rng.standard_normal(20000).astype(np.float32)
    r = rng.standard_normal(20000).astype(np.float32)
    m = np.float32(0.9)
    u_new, v = oracle.momentum_accumulate(u, g, r, 0.9)
    assert np.array_equal(u_new, m * u + g)                  # numpy rounds the product, then the sum
    assert np.array_equal(v, r + u_new)
    fused = (np.float64(m) * u.astype(np.float64) + g.astype(np.float64)).astype(np.float32)
    assert np.any(fused != u_new), "the inputs must tell a fused multiply-add from two roundings"


def test_momentum_closed_form_constant_gradient_nothing_sent():
    # g = 1, m = 1/2, rho = 0: u_t = 2 - 2^(1-t), v_t = sum of u; every value is exact in float32
    g = np.ones((6, 7), dtype=np.float32)
    u = np.zeros_like(g)
    r = np.zeros_like(g)
    want_u, want_v = 0.0, 0.0
    for t in range(1, 12):
        res = oracle.compress_layer_momentum(g, u, r, 0.5, 3, 0.5, 0.0)
        want_u = 0.5 * want_u + 1.0
        want_v += want_u
        assert want_u == 2.0 - 2.0 ** (1 - t)
        assert len(res.layer.idx) == 0
        assert np.all(res.u_new == np.float32(want_u)) and np.all(res.layer.r_new == np.float32(want_v))
        u, r = res.u_new, res.layer.r_new


def test_momentum_zero_is_the_plain_path_and_selection_runs_on_r_plus_u():
    rng = np.random.default_rng(22)
    g = (rng.standard_normal((19, 23)) * 1e-2).astype(np.float32)
    u = (rng.standard_normal((19, 23)) * 1e-2).astype(np.float32)
    r = (rng.standard_normal((19, 23)) * 1e-2).astype(np.float32)
    a = oracle.compress_layer_momentum(g, u, r, 0.0, 3, 0.5, 0.2).layer
    b = oracle.compress_layer(g, r, 3, 0.5, 0.2)
    for x, y in zip(a[:3] + (a.nsi, a.v, a.r_new), b[:3] + (b.nsi, b.v, b.r_new)):
        assert np.array_equal(x, y)
    # general m: the same as the plain path fed with u_new = m*u + g (formed here in numpy)
    m = np.float32(0.9)
    un = m * u + g
    c = oracle.compress_layer_momentum(g, u, r, 0.9, 3, 0.5, 0.2)
    d = oracle.compress_layer(un, r, 3, 0.5, 0.2)
    assert np.array_equal(c.layer.idx, d.idx) and np.array_equal(c.layer.val, d.val)
    assert np.array_equal(c.layer.centres, d.centres) and np.array_equal(c.layer.r_new, d.r_new)
    # masking: momentum and residual restart from +0 exactly where something was sent
    sent = np.zeros(g.size, dtype=bool)
    sent[c.layer.idx] = True
    want_u = un.ravel().copy()
    want_u[sent] = 0.0
    assert np.array_equal(c.u_new.ravel().view(np.uint32), want_u.view(np.uint32))
    assert np.array_equal(oracle.mask_momentum(un, sent).ravel(), want_u)
    dense = oracle.decompress(c.layer.idx, c.layer.val, g.size)
    assert np.array_equal(dense + c.layer.r_new.ravel(), c.layer.v.ravel())


def test_momentum_against_pure_python_brute_force():
    rng = np.random.default_rng(23)
    for R, C, p, rho in ((9, 11, 3, 0.3), (7, 16, 5, 0.5)):
        g = (rng.standard_normal((R, C)) * 1e-2).astype(np.float32)
        u = (rng.standard_normal((R, C)) * 1e-2).astype(np.float32)
        r = (rng.standard_normal((R, C)) * 1e-2).astype(np.float32)
        m = np.float32(0.9)
        un = [[float(np.float32(np.float32(m * np.float32(u[x, y])) + np.float32(g[x, y]))) for y in range(C)]
              for x in range(R)]
        b = brute_compress(un, r.tolist(), p, 0.5, rho)        # Eq. 12: v = r + u_new
        o = oracle.compress_layer_momentum(g, u, r, 0.9, p, 0.5, rho)
        assert o.layer.v.ravel().tolist() == b["v"]
        if np.array_equal(o.layer.nsi.ravel(), np.array(b["nsi"], dtype=np.float32)):
            assert o.layer.idx.tolist() == b["idx"] and o.layer.r_new.ravel().tolist() == b["r_new"]
            kept = set(b["idx"])
            flat = [x for row in un for x in row]
            assert o.u_new.ravel().tolist() == [0.0 if i in kept else flat[i] for i in range(R * C)]


# ------------------------------------------------- dynamic per-layer ratios (Eqs. 3-5)
def test_dynamic_ratios_against_a_library_sort():
    rng = np.random.default_rng(31)
    shapes = [(9, 11), (40, 3), (1, 57), (16, 16)]
    ws = [(rng.standard_normal(sh) * s).astype(np.float32) for sh, s in zip(shapes, (1.0, 0.2, 5.0, 1.0))]
    for rho in (0.0, 0.001, 0.013, 0.25, 0.5, 0.999, 1.0):
        got = oracle.dynamic_ratios(ws, rho)
        mu = np.concatenate([np.abs(w).ravel() for w in ws])
        layer = np.concatenate([np.full(w.size, l) for l, w in enumerate(ws)])
        K = int(math.ceil(rho * mu.size))
        order = np.argsort(-mu.astype(np.float64), kind="stable")        # stable: ties keep layer/index order
        kept = np.bincount(layer[order[:K]], minlength=len(ws))
        assert got == [kept[l] / ws[l].size for l in range(len(ws))]
        assert sum(round(r * w.size) for r, w in zip(got, ws)) == K      # Eq. 5 over all layers: the survivors


def test_dynamic_ratios_closed_forms_and_tie_order():
    big = np.full((4, 5), -2.0, dtype=np.float32)         # |w| = 2 everywhere (sign must not matter)
    small = np.full((10, 3), 1.0, dtype=np.float32)
    assert oracle.dynamic_ratios([big, small], 20 / 50) == [1.0, 0.0]
    assert oracle.dynamic_ratios([small, big], 20 / 50) == [0.0, 1.0]
    assert oracle.dynamic_ratios([big, small], 35 / 50) == [1.0, 0.5]
    # all weights equal: the ranking falls back to layer order, then index order
    a = np.ones((2, 5), dtype=np.float32)
    b = -np.ones((3, 4), dtype=np.float32)
    assert oracle.dynamic_ratios([a, b], 13 / 22) == [1.0, 3 / 12]
    assert oracle.dynamic_ratios([a, b], 1.0) == [1.0, 1.0]
    assert oracle.dynamic_ratios([a, b], 0.0) == [0.0, 0.0]
    # scaling one layer up moves the budget towards it (the paper's premise), monotonically
    rng = np.random.default_rng(32)
    x = rng.standard_normal((30, 30)).astype(np.float32)
    y = rng.standard_normal((30, 30)).astype(np.float32)
    prev = -1.0
    for s in (0.25, 0.5, 1.0, 2.0, 4.0):
        r0, r1 = oracle.dynamic_ratios([x * np.float32(s), y], 0.1)
        assert r0 >= prev and abs(r0 * 900 + r1 * 900 - 180) < 1e-9
        prev = r0
    assert oracle.dynamic_ratios([x, y * np.float32(1.0)], 0.1)[0] == oracle.dynamic_ratios([x, y], 0.1)[0]


# ------------------------------------------------- receiving side (Eq. 12, third line)
def test_apply_messages_is_w_minus_eta_times_the_ordered_sum():
    rng = np.random.default_rng(51)
    G = 5000
    w = rng.standard_normal(G).astype(np.float32)
    msgs = []
    for k in range(4):
        idx = np.sort(rng.choice(G, size=3000, replace=False)).astype(np.uint32)   # most positions get 2-3 messages
        msgs.append((idx, (rng.standard_normal(3000) * 10.0 ** rng.uniform(-1, 1)).astype(np.float32)))
    eta = np.float32(0.1)
    got = oracle.apply_messages(w, msgs, 0.1)
    total = np.zeros(G, dtype=np.float32)
    for idx, val in msgs:                                  # numpy float32: one rounded add per message
        total[idx] = total[idx] + val
    assert np.array_equal(got, w - eta * total)            # one rounded product, one rounded difference
    touched = np.zeros(G, dtype=bool)
    for idx, _ in msgs:
        touched[idx] = True
    assert np.array_equal(got[~touched].view(np.uint32), w[~touched].view(np.uint32))   # untouched bits survive
    # the order of the messages is the order of the float32 adds
    rev = oracle.apply_messages(w, msgs[::-1], 0.1)
    both = np.zeros(G, dtype=np.float32)
    for idx, val in msgs[::-1]:
        both[idx] = both[idx] + val
    assert np.array_equal(rev, w - eta * both)
    assert np.any(rev != got), "the data must tell the two summation orders apart"


def test_apply_messages_small_cases():
    w = np.arange(10, dtype=np.float32)
    m1 = (np.array([1, 3], np.uint32), np.array([1.0, 2.0], np.float32))
    m2 = (np.array([3, 9], np.uint32), np.array([0.5, -4.0], np.float32))
    assert oracle.apply_messages(w, [m1, m2], 0.5).tolist() == [0, 0.5, 2, 1.75, 4, 5, 6, 7, 8, 11]
    assert oracle.apply_messages(w, [], 0.5).tolist() == w.tolist()
    assert oracle.apply_messages(w, [m1], 0.0).tolist() == w.tolist()
    neg0 = np.array([-0.0, 1.0], np.float32)
    out = oracle.apply_messages(neg0, [(np.array([1], np.uint32), np.array([0.0], np.float32))], 1.0)
    assert np.array_equal(out.view(np.uint32), neg0.view(np.uint32))
    # one iteration end to end on one layer, two nodes: what is applied is what the nodes sent
    rng = np.random.default_rng(52)
    ww = rng.standard_normal((20, 30)).astype(np.float32)
    sent = []
    dense = np.zeros(600, np.float32)
    for k in range(2):
        g = (rng.standard_normal((20, 30)) * 1e-2).astype(np.float32)
        res = oracle.compress_layer(g, np.zeros_like(g), 3, 0.5, 0.1)
        sent.append((res.idx, res.val))
        dense = oracle.decompress(res.idx, res.val, 600, dense=dense, accumulate_into=True)
    assert np.array_equal(oracle.apply_messages(ww, sent, 0.25).ravel(), ww.ravel() - np.float32(0.25) * dense)


# ------------------------------------------------- the block reading (non-overlapping p x p neighbourhoods)
def _numpy_block_nsi(v, p, alpha):
    """Zero-pad to multiples of p, cut into blocks with a reshape, statistics with numpy in double."""
    R, C = v.shape
    BR, BC = -(-R // p), -(-C // p)
    pad = np.zeros((BR * p, BC * p), dtype=np.float64)
    pad[:R, :C] = v
    blk = pad.reshape(BR, p, BC, p).transpose(0, 2, 1, 3).reshape(BR, BC, p * p)
    return alpha * np.abs(blk).mean(axis=2) + (1.0 - alpha) * blk.std(axis=2)       # population std


@pytest.mark.parametrize("R,C,p", [(12, 15, 3), (13, 17, 3), (10, 10, 5), (11, 23, 5), (7, 7, 7), (4, 9, 1), (2, 2, 3)])
def test_block_nsi_against_numpy_reshape(R, C, p):
    rng = np.random.default_rng(R * 100 + C)
    v = (rng.standard_normal((R, C)) + 0.3).astype(np.float32)
    for alpha in (0.0, 0.3, 1.0):
        got = oracle.block_nsi(v, p, alpha)
        want = _numpy_block_nsi(v, p, alpha)
        assert got.shape == want.shape
        assert np.allclose(got, want, rtol=1e-6, atol=1e-7)


def test_block_nsi_equals_the_window_nsi_at_block_centres():
    # a full interior block is exactly the window of its centre element
    rng = np.random.default_rng(71)
    v = rng.standard_normal((15, 21)).astype(np.float32)
    for p in (3, 5):
        full = oracle.nsi(v, p, 0.4)
        blk = oracle.block_nsi(v, p, 0.4)
        h = (p - 1) // 2
        for bx in range(15 // p):
            for by in range(21 // p):
                assert blk[bx, by] == full[bx * p + h, by * p + h]


def test_block_compress_invariants_counts_and_order():
    rng = np.random.default_rng(72)
    for R, C, p, rho in ((20, 31, 3, 0.2), (9, 9, 5, 1.0), (30, 7, 3, 0.05), (8, 8, 1, 0.1), (6, 40, 7, 0.5)):
        g = (rng.standard_normal((R, C)) * 1e-2).astype(np.float32)
        r = (rng.standard_normal((R, C)) * 1e-2).astype(np.float32)
        res = oracle.compress_layer_blocks(g, r, p, 0.5, rho)
        BR, BC = -(-R // p), -(-C // p)
        assert res.k == min(math.ceil(R * C / (p * p) * rho), BR * BC)           # Eq. 11, at most all blocks
        assert np.array_equal(res.v, r + g)
        # ranking: the k best blocks by (score desc, index asc), listed ascending
        s = res.nsi.ravel()
        order = sorted(range(s.size), key=lambda i: (-float(s[i]), i))
        assert res.blocks.tolist() == sorted(order[:res.k])
        if res.k:
            assert res.tau == float(s[order[res.k - 1]])
        # wire format: p*p values per kept block, row-major, zero outside the matrix
        for j, b in enumerate(res.blocks):
            bx, by = divmod(int(b), BC)
            for dx in range(p):
                for dy in range(p):
                    x, y = bx * p + dx, by * p + dy
                    want = res.v[x, y] if x < R and y < C else np.float32(0.0)
                    assert res.val[j * p * p + dx * p + dy] == want
        # what was sent plus what stays is the accumulated gradient, bit for bit
        dense = oracle.decompress_blocks(res.blocks, res.val, R, C, p)
        assert np.array_equal(dense + res.r_new, res.v)
        kept = dense != 0
        assert np.all(res.r_new[kept] == 0)
        acc = oracle.decompress_blocks(res.blocks, res.val, R, C, p, dense=np.ones((R, C), np.float32), accumulate_into=True)
        assert np.array_equal(acc, np.float32(1.0) + dense)


def test_block_reading_with_p1_is_the_element_reading():
    rng = np.random.default_rng(73)
    g = (rng.standard_normal((12, 19)) * 1e-2).astype(np.float32)
    r = (rng.standard_normal((12, 19)) * 1e-2).astype(np.float32)
    a = oracle.compress_layer_blocks(g, r, 1, 0.5, 0.1)
    b = oracle.compress_layer(g, r, 1, 0.5, 0.1)
    assert np.array_equal(a.blocks, b.idx) and np.array_equal(a.val, b.val) and np.array_equal(a.r_new, b.r_new)


# ------------------------------------------------- block reading with momentum (Eq. 12 in full)
def test_block_momentum_zero_is_the_plain_block_reading():
    rng = np.random.default_rng(74)
    g = (rng.standard_normal((19, 23)) * 1e-2).astype(np.float32)
    u = (rng.standard_normal((19, 23)) * 1e-2).astype(np.float32)
    r = (rng.standard_normal((19, 23)) * 1e-2).astype(np.float32)
    a = oracle.compress_layer_blocks_momentum(g, u, r, 0.0, 3, 0.5, 0.2)
    b = oracle.compress_layer_blocks(g, r, 3, 0.5, 0.2)
    for x, y in zip(a.layer, b):
        assert np.array_equal(x, y)
    kept = oracle.decompress_blocks(b.blocks, np.ones(b.k * 9, np.float32), 19, 23, 3) != 0
    assert np.array_equal(a.u_new, np.where(kept, np.float32(0), g))


def test_block_momentum_is_the_plain_block_reading_fed_with_m_u_plus_g():
    rng = np.random.default_rng(75)
    for (R, C), p, rho in (((19, 23), 3, 0.2), ((10, 31), 5, 0.6), ((7, 7), 7, 1.0), ((9, 40), 1, 0.1)):
        g = (rng.standard_normal((R, C)) * 1e-2).astype(np.float32)
        u = (rng.standard_normal((R, C)) * 1e-2).astype(np.float32)
        r = (rng.standard_normal((R, C)) * 1e-2).astype(np.float32)
        un = np.float32(0.9) * u + g                         # one rounded multiply, one rounded add (numpy)
        c = oracle.compress_layer_blocks_momentum(g, u, r, 0.9, p, 0.5, rho)
        d = oracle.compress_layer_blocks(un, r, p, 0.5, rho)
        assert np.array_equal(c.layer.v, r + un)
        assert np.array_equal(c.layer.blocks, d.blocks) and np.array_equal(c.layer.val, d.val)
        assert np.array_equal(c.layer.nsi, d.nsi) and np.array_equal(c.layer.r_new, d.r_new)
        # momentum and residual restart from +0 on exactly the slots of the kept blocks
        kept = np.zeros((R, C), bool)
        BC = -(-C // p)
        for b in c.layer.blocks.tolist():
            bx, by = divmod(b, BC)
            kept[bx * p:bx * p + p, by * p:by * p + p] = True
        want_u = np.where(kept, np.float32(0), un)
        assert np.array_equal(c.u_new.view(np.uint32), want_u.view(np.uint32))
        assert np.array_equal(c.layer.r_new.view(np.uint32), np.where(kept, np.float32(0), r + un).view(np.uint32))
        dense = oracle.decompress_blocks(c.layer.blocks, c.layer.val, R, C, p)
        assert np.array_equal(dense + c.layer.r_new, c.layer.v)


def test_block_momentum_closed_form_constant_gradient_nothing_sent_then_all_sent():
    # g = 1, m = 1/2, rho = 0: u_t = 2 - 2^(1-t), v_t = sum of u (all exact in float32); then one
    # call with rho = 1 sends every block and both u and r restart from zero
    g = np.ones((6, 7), dtype=np.float32)
    u = np.zeros_like(g)
    r = np.zeros_like(g)
    want_u, want_v = 0.0, 0.0
    for t in range(1, 10):
        res = oracle.compress_layer_blocks_momentum(g, u, r, 0.5, 3, 0.5, 0.0)
        want_u = 0.5 * want_u + 1.0
        want_v += want_u
        assert res.layer.k == 0 and res.layer.blocks.size == 0
        assert np.all(res.u_new == np.float32(want_u)) and np.all(res.layer.r_new == np.float32(want_v))
        u, r = res.u_new, res.layer.r_new
    res = oracle.compress_layer_blocks_momentum(g, u, r, 0.5, 3, 0.5, 1.0)
    assert res.layer.k == 5 and res.layer.blocks.tolist() == [0, 1, 2, 3, 4]     # ceil(42/9) of 6 blocks
    sent = np.float32(want_v + 0.5 * want_u + 1.0)
    # the block not sent is one with the lowest score: the right-hand blocks are cut by the edge
    # (one column of three inside), equal scores tie towards the lower index
    assert res.layer.nsi[0, 2] == res.layer.nsi[1, 2] < res.layer.nsi[0, 0]
    assert np.all(res.layer.val.reshape(5, 3, 3)[[0, 1, 3, 4]] == sent)
    assert np.all(res.u_new[:, :6] == 0) and np.all(res.layer.r_new[:, :6] == 0)
    assert np.all(res.u_new[0:3, 6] == 0) and np.all(res.u_new[3:6, 6] == np.float32(0.5 * want_u + 1.0))
    assert np.all(res.layer.r_new[3:6, 6] == sent)


def test_block_momentum_with_p1_is_the_element_reading_with_momentum():
    rng = np.random.default_rng(76)
    g = (rng.standard_normal((12, 19)) * 1e-2).astype(np.float32)
    u = (rng.standard_normal((12, 19)) * 1e-2).astype(np.float32)
    r = (rng.standard_normal((12, 19)) * 1e-2).astype(np.float32)
    a = oracle.compress_layer_blocks_momentum(g, u, r, 0.7, 1, 0.5, 0.1)
    b = oracle.compress_layer_momentum(g, u, r, 0.7, 1, 0.5, 0.1)
    assert np.array_equal(a.layer.blocks, b.layer.idx) and np.array_equal(a.layer.val, b.layer.val)
    assert np.array_equal(a.layer.r_new, b.layer.r_new) and np.array_equal(a.u_new, b.u_new)


def test_block_momentum_against_pure_python_brute_force():
    rng = np.random.default_rng(77)
    for R, C, p, rho in ((9, 11, 3, 0.3), (7, 16, 5, 0.5)):
        g = (rng.standard_normal((R, C)) * 1e-2).astype(np.float32)
        u = (rng.standard_normal((R, C)) * 1e-2).astype(np.float32)
        r = (rng.standard_normal((R, C)) * 1e-2).astype(np.float32)
        m = np.float32(0.9)
        un = [[float(np.float32(np.float32(m * u[x, y]) + g[x, y])) for y in range(C)] for x in range(R)]
        v = [[float(np.float32(np.float32(r[x, y]) + np.float32(un[x][y]))) for y in range(C)] for x in range(R)]
        BR, BC = -(-R // p), -(-C // p)
        score = []
        for bx in range(BR):
            for by in range(BC):
                w = [v[x][y] if x < R and y < C else 0.0
                     for x in range(bx * p, bx * p + p) for y in range(by * p, by * p + p)]
                mean = sum(w) / (p * p)
                std = math.sqrt(sum((t - mean) ** 2 for t in w) / (p * p))               # Eq. 10
                score.append(float(np.float32(0.5 * sum(abs(t) for t in w) / (p * p) + 0.5 * std)))   # Eqs. 8, 9
        k = min(math.ceil(R * C / (p * p) * rho), BR * BC)                                # Eq. 11
        kept_blocks = sorted(sorted(range(BR * BC), key=lambda i: (-score[i], i))[:k])
        o = oracle.compress_layer_blocks_momentum(g, u, r, 0.9, p, 0.5, rho)
        assert o.layer.v.tolist() == v
        if o.layer.nsi.ravel().tolist() == score:
            assert o.layer.blocks.tolist() == kept_blocks
            for x in range(R):
                for y in range(C):
                    kept = (x // p) * BC + y // p in kept_blocks
                    assert o.u_new[x, y] == (0.0 if kept else un[x][y])
                    assert o.layer.r_new[x, y] == (0.0 if kept else v[x][y])


def _blocks_as_pairs(blocks, val, R, C, p):
    """A block message written out as (flat index, value) pairs of the slots inside the matrix."""
    BC = (C + p - 1) // p
    idx, out = [], []
    for j, b in enumerate(blocks.tolist()):
        bx, by = divmod(b, BC)
        for dx in range(p):
            for dy in range(p):
                x, y = bx * p + dx, by * p + dy
                if x < R and y < C:
                    idx.append(x * C + y)
                    out.append(val[j * p * p + dx * p + dy])
    return np.array(idx, np.uint32), np.array(out, np.float32)


def test_apply_block_messages_small_case_by_hand():
    # 4 x 5 matrix, p = 3: blocks 0 1 / 2 3; blocks 1 and 3 are cut by the right edge, 2 and 3 by the lower one
    w = np.arange(20, dtype=np.float32).reshape(4, 5)
    m1 = (np.array([0, 3], np.uint32),
          np.array([1, 2, 3, 4, 5, 6, 7, 8, 9] + [10, 20, 99, 99, 99, 99, 99, 99, 99], np.float32))
    m2 = (np.array([0], np.uint32), np.array([0.5, 0, 0, 0, -4, 0, 0, 0, 0], np.float32))
    got = oracle.apply_block_messages(w, [m1, m2], 3, 0.5)
    want = w.copy()
    want[0:3, 0:3] -= np.float32(0.5) * np.array([[1.5, 2, 3], [4, 1, 6], [7, 8, 9]], np.float32)
    want[3, 3] -= 0.5 * 10
    want[3, 4] -= 0.5 * 20
    assert got.tolist() == want.tolist()
    assert oracle.apply_block_messages(w, [], 3, 0.5).tolist() == w.tolist()
    assert oracle.apply_block_messages(w, [m1], 3, 0.0).tolist() == w.tolist()


def test_apply_block_messages_is_the_element_form_on_the_blocks_slots():
    rng = np.random.default_rng(53)
    order_seen = False
    for (R, C), p in [((20, 31), 3), ((17, 17), 5), ((9, 40), 1), ((14, 10), 7)]:
        BR, BC = (R + p - 1) // p, (C + p - 1) // p
        w = rng.standard_normal((R, C)).astype(np.float32)
        msgs = []
        for k in range(3):
            blocks = np.sort(rng.choice(BR * BC, size=max(1, 3 * BR * BC // 4), replace=False)).astype(np.uint32)
            msgs.append((blocks, (rng.standard_normal(blocks.size * p * p) * 10.0 ** rng.uniform(-1, 1)).astype(np.float32)))
        got = oracle.apply_block_messages(w, msgs, p, 0.3)
        pairs = [_blocks_as_pairs(b, v, R, C, p) for b, v in msgs]
        assert np.array_equal(got.view(np.uint32), oracle.apply_messages(w, pairs, 0.3).view(np.uint32)), (R, C, p)
        # and numpy's float32 arithmetic: one rounded add per message, one product, one difference
        total = np.zeros(R * C, dtype=np.float32)
        for idx, val in pairs:
            total[idx] = total[idx] + val
        assert np.array_equal(got.ravel(), w.ravel() - np.float32(0.3) * total)
        order_seen = order_seen or bool(np.any(oracle.apply_block_messages(w, msgs[::-1], p, 0.3) != got))
    assert order_seen, "the data must tell the two summation orders apart"


def test_apply_block_messages_applies_what_the_nodes_sent():
    rng = np.random.default_rng(54)
    R, C, p = 26, 35, 3
    w = rng.standard_normal((R, C)).astype(np.float32)
    dense = np.zeros((R, C), np.float32)
    sent = []
    for k in range(2):
        g = (rng.standard_normal((R, C)) * 1e-2).astype(np.float32)
        res = oracle.compress_layer_blocks(g, np.zeros_like(g), p, 0.5, 0.2)
        sent.append((res.blocks, res.val))
        dense = oracle.decompress_blocks(res.blocks, res.val, R, C, p, dense=dense, accumulate_into=True)
    assert np.array_equal(oracle.apply_block_messages(w, sent, p, 0.25), w - np.float32(0.25) * dense)
