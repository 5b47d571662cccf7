"""Pins of the oracle's index-construction steps (Section 3.2): neighbours, alpha,
subregion assignment, PQ, the per-point constant and the grouped layout."""
import numpy as np
import pytest

from oracle import ivf_oracle as orc
from test_oracle_query import read_golden


def test_neighbours_bruteforce_excluding_self(rng):
    Cn = rng.standard_normal((30, 4)).astype(np.float32)
    Cn[11] = Cn[2]                                   # a duplicate centroid is a neighbour at distance 0
    nbr, cs = orc.neighbours(Cn, 6)
    d = ((Cn.astype(np.float64)[:, None] - Cn.astype(np.float64)[None]) ** 2).sum(-1)
    for r in range(30):
        others = [j for j in range(30) if j != r]
        ref = sorted(others, key=lambda j: (d[r, j], j))[:6]
        assert nbr[r].tolist() == ref
        assert (cs[r] == d[r, ref].astype(np.float32)).all()
    assert nbr[2, 0] == 11 and nbr[11, 0] == 2 and cs[2, 0] == 0


def test_alpha_hand_example():
    g = read_golden("alpha_hand_example.txt")
    Cn = np.stack([g["c"][0], g["s1"][0], g["s2"][0]]).astype(np.float32)
    X = np.stack(g["x"]).astype(np.float32)
    nbr = np.array([[1, 2], [0, 2], [0, 1]], np.int32)
    a = orc.learn_alpha(X, np.zeros(3, np.int32), Cn, nbr)
    assert a[0] == pytest.approx(g["alpha"][0][0], abs=1e-6)
    # regions 1 and 2 have no training points: they get the pooled ratio, which here is the same
    assert a[1] == pytest.approx(0.3, abs=1e-6) and a[2] == pytest.approx(0.3, abs=1e-6)


def test_alpha_recovers_planted_factor_and_minimises_objective(rng):
    D, K, L = 8, 20, 5
    Cn = rng.standard_normal((K, D)).astype(np.float32)
    nbr, _ = orc.neighbours(Cn, L)
    n = 4000
    reg = rng.integers(0, K, n).astype(np.int32)
    l = rng.integers(0, L, n)
    c = Cn[reg].astype(np.float64)
    s = Cn[nbr[reg, l]].astype(np.float64)
    X = (c + 0.3 * (s - c) + 1e-3 * rng.standard_normal((n, D))).astype(np.float32)
    a = orc.learn_alpha(X, reg, Cn, nbr)
    assert np.abs(a - 0.3).max() < 5e-3
    # Eq. (12) is the exact minimiser of sum ||x - c - a (s* - c)||^2 for the s* of step 1:
    # with planted data s* is the planted neighbour, so a fine grid cannot beat it
    for r in range(3):
        m = reg == r
        xc = X[m].astype(np.float64) - c[m]
        u = s[m] - c[m]
        obj = lambda al: ((xc - al * u) ** 2).sum()
        grid = np.linspace(0.25, 0.35, 2001)
        best = grid[np.argmin([obj(al) for al in grid])]
        assert abs(best - a[r]) <= 1e-4
        assert obj(float(a[r])) <= min(obj(al) for al in grid) + 1e-9


def test_alpha_clamped_and_degenerate(rng):
    Cn = np.array([[0, 0], [1, 0], [0, 0]], np.float32)        # centroid 2 duplicates centroid 0
    nbr = np.array([[2, 1], [0, 2], [0, 1]], np.int32)
    X = np.array([[3, 0], [4, 0]], np.float32)                  # far beyond s: unconstrained ratio is 3.5
    a = orc.learn_alpha(X, np.zeros(2, np.int32), Cn, nbr)
    assert a[0] == 1.0
    X = np.array([[-3, 0.0]], np.float32)                       # behind c: every a_l clamps to 0
    a = orc.learn_alpha(X, np.zeros(1, np.int32), Cn, nbr)
    assert 0.0 <= a[0] <= 1.0


def test_sub_assign_and_encode_against_numpy_bruteforce(tiny):
    spec, ix, Q, X = tiny
    n = 400
    x = X[:n]
    enc = orc.encode(x, ix.centroids, ix.nbr, ix.alpha, ix.pq_codebook, ix.const_table)
    c = ix.centroids.astype(np.float64)
    x64 = x.astype(np.float64)
    d = ((x64[:, None] - c[None]) ** 2).sum(-1)
    assert (enc.region == d.argmin(1)).all()
    ds = ix.D // ix.M
    for i in range(n):
        r = enc.region[i]
        mus = c[r][None] + float(ix.alpha[r]) * (c[ix.nbr[r]] - c[r][None])
        l = int(((x64[i][None] - mus) ** 2).sum(1).argmin())
        assert enc.sub[i] == l
        np.testing.assert_allclose(enc.mu[i], mus[l], rtol=0, atol=1e-15)
        e = x64[i] - mus[l]
        for m in range(ix.M):
            dd = ((e[m * ds:(m + 1) * ds][None] - ix.pq_codebook[m].astype(np.float64)) ** 2).sum(1)
            assert enc.codes[i, m] == dd.argmin()
        dec = orc.pq_decode(enc.codes[i:i + 1], ix.pq_codebook)[0]
        assert enc.t[i] == pytest.approx(2 * mus[l] @ dec + dec @ dec, abs=1e-12)
        assert enc.const_byte[i] == np.abs(ix.const_table.astype(np.float64) - enc.t[i]).argmin()


def test_grouped_layout(tiny):
    spec, ix, Q, X = tiny
    off = ix.sub_offsets.astype(np.int64)
    assert off[0] == 0 and off[-1] == ix.N and (np.diff(off) >= 0).all()
    assert sorted(ix.ids.tolist()) == list(range(ix.N))          # every point stored exactly once
    enc = orc.encode(X[ix.ids[:3000]], ix.centroids, ix.nbr, ix.alpha, ix.pq_codebook, ix.const_table)
    bucket = enc.region.astype(np.int64) * ix.L + enc.sub
    pos = np.arange(3000)
    assert ((off[bucket] <= pos) & (pos < off[bucket + 1])).all()  # stored inside its own subregion
    assert (enc.codes == ix.codes[:3000]).all() and (enc.const_byte == ix.const_byte[:3000]).all()
    # ascending original id inside every subregion
    same = np.repeat(np.arange(ix.K * ix.L), np.diff(off))
    inside = same[1:] == same[:-1]
    assert (np.diff(ix.ids.astype(np.int64))[inside] > 0).all()


def test_kmeans_objective_and_exact_special_case(rng):
    X = rng.standard_normal((3000, 5)).astype(np.float32)
    cent, obj = orc.kmeans(X, 16, 8, np.arange(16))
    assert (np.diff(obj) <= 1e-9).all() and obj[-1] < obj[0]
    # as many well-separated distinct values as centroids: each centroid lands on one value exactly
    vals = np.arange(256, dtype=np.float32)[:, None] * 3.0
    Xs = np.repeat(vals, 4, axis=0)[rng.permutation(1024)]
    init = np.array([int(np.flatnonzero(Xs[:, 0] == v)[0]) for v in vals[:, 0]])
    cent, obj = orc.kmeans(Xs, 256, 3, init)
    assert sorted(cent[:, 0].tolist()) == vals[:, 0].tolist() and obj[-1] == 0.0
    # PQ with one dimension per block over such values reproduces the input exactly
    E = np.stack([Xs[:, 0], Xs[::-1, 0]], axis=1).astype(np.float64)
    cb = np.stack([cent, cent])                                  # [M=2, 256, 1]
    codes = orc.pq_encode(E, cb)
    assert (orc.pq_decode(codes, cb) == E).all()


def test_pq_training_objective_non_increasing(tiny, rng):
    spec, ix, Q, X = tiny
    E = rng.standard_normal((4000, 16)) * 0.1
    cb, objs = orc.pq_train(E, 4, 6, np.arange(256))
    assert cb.shape == (4, 256, 4) and (np.diff(objs, axis=1) <= 1e-9).all()


def test_scalar_quantiser(rng):
    t = rng.standard_normal(20000) * 0.2 + 1.0
    table = orc.lloyd_1d(t, 20)
    assert (np.diff(table) >= 0).all() and table[0] >= t.min() - 1e-6 and table[-1] <= t.max() + 1e-6
    b = orc.quantize_1d(t, table)
    assert (b == np.abs(t[:, None] - table.astype(np.float64)[None]).argmin(1)).all()
    # Lloyd iterations never increase the training error (started from the quantile table)
    mses = []
    for it in (0, 1, 5, 20):
        tab = orc.lloyd_1d(t, it).astype(np.float64)
        mses.append(((tab[orc.quantize_1d(t, tab)] - t) ** 2).mean())
    assert all(b2 <= a2 + 1e-15 for a2, b2 in zip(mses, mses[1:])) and mses[-1] < 0.5 * mses[0]
    # iteration 0 is the (j + 1/2)/256 quantile table
    q0 = np.sort(t)[((np.arange(256) + 0.5) / 256 * t.shape[0]).astype(np.int64)].astype(np.float32)
    assert (orc.lloyd_1d(t, 0) == q0).all()
    # exact tie between two levels resolves to the lower index
    tab = np.arange(256, dtype=np.float32)
    assert orc.quantize_1d(np.array([3.5, 0.5, 254.5]), tab).tolist() == [3, 0, 254]
