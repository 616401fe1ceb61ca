"""The float32 test with which the main pass rules out centres below a layer's candidate bound
(before the evaluation in full), replayed in numpy float32 on hard windows and compared with exact
arithmetic: with the slacks the kernel's comment derives, no centre whose exact score reaches the
bound is ever ruled out; without them, many are.  This checks the error bounds (the constants are
typed in here as they stand in the kernel source), not the kernel -- the GPU parity tests do that.
NSI of a window: alpha * mean|w| + (1 - alpha) * std w (Eqs. 8-10)."""
import numpy as np
import pytest

f32 = np.float32
U = 5.9604645e-8          # 2^-24


def _fma32(a, b, c):
    # round32(a * b + c): the product of two float32 is exact in double
    return (a.astype(np.float64) * b.astype(np.float64) + c.astype(np.float64)).astype(f32)


def _round_down32(x):
    y = x.astype(f32)
    return np.where(y.astype(np.float64) > x, np.nextafter(y, f32(-np.inf)), y).astype(f32)


def _kept(P, alpha, W, bound, slack_factor=1.3, bound_terms=2.04):
    """The test as the main pass applies it: True where the centre stays (queued for evaluation)."""
    n = P * P
    ca, cb = alpha / n, (1.0 - alpha) / n
    caf, cb2f = f32(ca), f32(cb * cb)
    kslack = f32(f32(slack_factor) * f32(3.0 * n + 3.0) * f32(U))
    bound_lof = _round_down32(bound.astype(np.float64) * (1.0 - 2.0 ** -22 - bound_terms * n * U))
    ra, rs, rq = np.abs(W[:, :, 0]), W[:, :, 0].copy(), (W[:, :, 0] * W[:, :, 0]).astype(f32)
    for j in range(1, P):                         # row sums, left to right
        ra = (ra + np.abs(W[:, :, j])).astype(f32)
        rs = (rs + W[:, :, j]).astype(f32)
        rq = _fma32(W[:, :, j], W[:, :, j], rq)
    sa, ss, sq = ra[:, 0], rs[:, 0], rq[:, 0]
    for i in range(1, P):                         # window sums, top to bottom
        sa, ss, sq = (sa + ra[:, i]).astype(f32), (ss + rs[:, i]).astype(f32), (sq + rq[:, i]).astype(f32)
    with np.errstate(all="ignore"):
        nsq = (f32(n) * sq).astype(f32)
        d_hi = _fma32(np.full_like(nsq, kslack), nsq, _fma32(-ss, ss, nsq))
        rest = _fma32(np.full_like(sa, -caf), sa, bound_lof)
        lhs = (cb2f * d_hi).astype(f32)
        rhs = ((rest * rest).astype(f32) * f32(1.0 - 1e-6)).astype(f32)
        return (rest <= 0) | ~(lhs < rhs)


def _must_stay(P, alpha, W, bound):
    """Exact: the score reaches what rounds to the bound in float32 (with the evaluation's own 1e-9)."""
    n = P * P
    Wd = W.astype(np.longdouble)
    SA, SS, SQ = np.abs(Wd).sum(axis=(1, 2)), Wd.sum(axis=(1, 2)), (Wd * Wd).sum(axis=(1, 2))
    D = np.maximum(n * SQ - SS * SS, 0)
    S = np.longdouble(alpha / n) * SA + np.longdouble((1.0 - alpha) / n) * np.sqrt(D)
    return S >= bound.astype(np.longdouble) * (np.longdouble(1) - np.longdouble(2.0) ** -22)


def _windows(rng, P, N):
    n = P * P
    c = rng.standard_normal((N, 1, 1)).astype(f32)
    one_large = rng.standard_normal((N, P, P)).astype(f32) * f32(1e-4)
    one_large[:, 0, 0] = rng.standard_normal(N).astype(f32)
    signs = np.where((np.arange(n).reshape(P, P) % 2) == 0, 1, -1).astype(f32)
    return {
        "noise": rng.standard_normal((N, P, P)).astype(f32),
        "near-constant": (c * (1 + rng.integers(-4, 5, (N, P, P)) * 2.0 ** -23)).astype(f32),
        "constant": np.broadcast_to(c, (N, P, P)).astype(f32).copy(),
        "one large value": one_large,
        "alternating signs": np.abs(rng.standard_normal((N, P, P))).astype(f32) * signs,
        "six decades": (rng.standard_normal((N, P, P)) * 10.0 ** rng.uniform(-6, 0, (N, P, P))).astype(f32),
        "ramp on an offset": (c * (1 + np.arange(n).reshape(1, P, P) * 2.0 ** -20)).astype(f32),
    }


def _sweep(P, seed, N, **kw):
    rng = np.random.default_rng(seed)
    n = P * P
    wrong = clear = kept_clear = 0      # clear: noise windows whose score lies 10 % below the bound
    for alpha in (0.5, 0.0, 1.0, 0.25, 0.9):
        for name, W in _windows(rng, P, N).items():
            for scale in (1.0, 2.0 ** -38, 2.0 ** 38, 1e-3):
                Ws = (W * f32(scale)).astype(f32)
                Wd = Ws.astype(np.float64)
                SA, SS, SQ = np.abs(Wd).sum(axis=(1, 2)), Wd.sum(axis=(1, 2)), (Wd * Wd).sum(axis=(1, 2))
                S = alpha / n * SA + (1 - alpha) / n * np.sqrt(np.maximum(n * SQ - SS * SS, 0))
                # bounds right at the score, a hair to either side, and well away from it
                eps = rng.choice([0.0, 1e-8, -1e-8, 1e-7, -1e-7, 3e-7, -3e-7, 1e-6, -1e-6, 1e-5, 1e-3, -1e-3, 0.1, -0.1], size=N)
                b = (S * (1 + eps)).astype(f32)
                ok = np.isfinite(b) & (b >= 2.0 ** -40) & (b <= 2.0 ** 40)     # the range bounds are handed out in
                if not ok.any():
                    continue
                kept, must = _kept(P, alpha, Ws[ok], b[ok], **kw), _must_stay(P, alpha, Ws[ok], b[ok])
                wrong += int((must & ~kept).sum())
                if name == "noise":
                    far = eps[ok] >= 0.1
                    clear += int(far.sum())
                    kept_clear += int((kept & far).sum())
    return wrong, clear, kept_clear


@pytest.mark.parametrize("P", [1, 3, 5, 7])
def test_no_centre_that_reaches_the_bound_is_ruled_out(P):
    wrong, clear, kept_clear = _sweep(P, seed=100 + P, N=6000)
    assert wrong == 0
    assert clear > 5000 and kept_clear == 0      # and what lies clearly below the bound is still ruled out


@pytest.mark.parametrize("P", [3, 7])
def test_without_the_slacks_centres_are_lost(P):
    """The same replay with the slack on d and the extra terms of the bound's factor taken out: the
    sweep above has the power to see a bound that is too tight."""
    wrong, _, _ = _sweep(P, seed=200 + P, N=3000, slack_factor=0.0, bound_terms=0.0)
    assert wrong > 100
