"""The error bound the nearest-centroid shortlist relies on, checked on the CPU with numpy's fp16.

The device pass approximates |q - c|^2 by |q|^2 + |c|^2 - 2 <hi(q), hi(c)>, where hi(x) is x scaled by
a power of two (largest magnitude of the row, or of the whole centroid table, into [2^14, 2^15)) and
rounded to fp16, and keeps every centroid whose approximation minus eps is not above the smallest
approximation plus eps seen, with

    eps(q, c) = 2^-9 (|q|^2 + |c|^2) + 2^-30 (|q|^2 + D gmax^2).

That is only sound if the exact distance always lies within eps of the approximation.  Here the
approximation is rebuilt from its definition (numpy float16 rounding, exact fp64 arithmetic otherwise)
for inputs chosen to stress it: rows of very different magnitude under one table-wide scale, elements
far below the row's largest, and vectors sitting on fp16 rounding midpoints, where the bound is
nearly attained.
"""
import numpy as np

KAPPA = 2.0 ** -9


def _scale(m):
    """2^(14 - floor(log2 m)): the largest magnitude m lands in [2^14, 2^15)."""
    e = np.floor(np.log2(m))
    return np.exp2(14 - e)


def _hi(x, s):
    with np.errstate(over="raise"):
        return (x.astype(np.float64) * s).astype(np.float32).astype(np.float16).astype(np.float64) / s


def _approx_and_exact(Q, C):
    q64, c64 = Q.astype(np.float64), C.astype(np.float64)
    sq = _scale(np.abs(q64).max(1, keepdims=True))       # one scale per query row
    sc = _scale(np.abs(c64).max())                        # one scale for the centroid table
    qh, ch = _hi(Q, sq), _hi(C, sc)
    qn, cn = (q64 ** 2).sum(1), (c64 ** 2).sum(1)
    approx = qn[:, None] + cn[None, :] - 2.0 * qh @ ch.T
    exact = ((q64[:, None, :] - c64[None, :, :]) ** 2).sum(-1)
    eps = KAPPA * (qn[:, None] + cn[None, :]) + 2.0 ** -30 * (qn[:, None] + Q.shape[1] * np.abs(c64).max() ** 2)
    return approx, exact, eps


def test_bound_holds_for_rows_of_very_different_magnitude():
    rng = np.random.default_rng(3)
    D = 96
    C = (rng.standard_normal((400, D)) * np.exp2(rng.integers(-30, 1, size=(400, 1)))).astype(np.float32)
    Q = (rng.standard_normal((300, D)) * np.exp2(rng.integers(-20, 12, size=(300, 1)))).astype(np.float32)
    Q[:50] *= np.exp2(rng.integers(-24, 1, size=(50, D)))          # elements far below the row's largest
    C[:50] *= np.exp2(rng.integers(-24, 1, size=(50, D))).astype(np.float32)
    approx, exact, eps = _approx_and_exact(Q, C)
    assert (np.abs(approx - exact) <= eps).all(), float((np.abs(approx - exact) / eps).max())


def test_bound_is_nearly_attained_on_rounding_midpoints():
    """Every element (1 + 2^-11) 2^k sits halfway between two fp16 numbers: rounding to even moves q and c
    the same way, the inner product is off by almost 2^-10 |q||c|, the distance by almost 2^-10 (|q|^2+|c|^2)
    when q = c: half of eps.  A bound with a quarter of the constant would fail here."""
    D = 64
    k = np.arange(D) % 3
    x = ((1.0 + 2.0 ** -11) * np.exp2(-k)).astype(np.float32)[None, :]
    approx, exact, eps = _approx_and_exact(x, x)
    err = abs(float(approx[0, 0] - exact[0, 0]))
    assert err <= float(eps[0, 0])
    assert err >= 0.24 * float(eps[0, 0])


def test_bound_holds_for_unit_vectors_and_sift_like_integers():
    rng = np.random.default_rng(4)
    for D, gen in ((96, lambda n: rng.standard_normal((n, 96))), (128, lambda n: rng.gamma(0.5, 20.0, size=(n, 128)).round().clip(0, 255))):
        C = gen(500)
        Q = gen(200)
        if D == 96:
            C /= np.linalg.norm(C, axis=1, keepdims=True)
            Q /= np.linalg.norm(Q, axis=1, keepdims=True)
        approx, exact, eps = _approx_and_exact(Q.astype(np.float32), C.astype(np.float32))
        assert (np.abs(approx - exact) <= eps).all()
        # and the shortlist it defines contains the exact nearest centroid of every query
        lo, up = approx - eps, approx + eps
        keep = lo <= up.min(1, keepdims=True)
        assert keep[np.arange(len(Q)), exact.argmin(1)].all()
        assert keep.sum(1).max() < 100                    # ... and stays short on such data
