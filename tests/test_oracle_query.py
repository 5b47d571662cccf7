"""Pins of the oracle's query path (stages 1-6) against things other than itself:
the definitions written out with explicit subcentroids / decoded vectors,
brute-force sorts, special cases, and hand-worked numbers."""
import os

import numpy as np
import pytest

from oracle import ivf_oracle as orc

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def read_golden(name):
    out = {}
    for line in open(os.path.join(GOLD, name)):
        if line.startswith("#") or not line.strip():
            continue
        key, *vals = line.split()
        out.setdefault(key, []).append(np.array([float(v) for v in vals]))
    return out


def tiny_index(D=2, K=2, L=1, M=1, **kw):
    z = dict(centroids=np.zeros((K, D), np.float32), nbr=np.zeros((K, L), np.int32),
             alpha=np.zeros(K, np.float32), cs_dist2=np.zeros((K, L), np.float32),
             pq_codebook=np.zeros((M, 256, D // M), np.float32), const_table=np.zeros(256, np.float32),
             sub_offsets=np.zeros(K * L + 1, np.uint32), codes=np.zeros((0, M), np.uint8),
             const_byte=np.zeros(0, np.uint8), ids=np.zeros(0, np.int32))
    z.update(kw)
    N = z["codes"].shape[0]
    return orc.Index(D, M, L, K, N, **z)


# ------------------------------------------------------------------ stage 1


def test_coarse_distances_match_expansion_and_direct(rng):
    Q = rng.standard_normal((7, 13)).astype(np.float32)
    Cn = rng.standard_normal((29, 13)).astype(np.float32)
    d = orc.coarse_dist(Q, Cn)
    Q64, C64 = Q.astype(np.float64), Cn.astype(np.float64)
    direct = ((Q64[:, None, :] - C64[None, :, :]) ** 2).sum(-1)
    expand = (Q64 ** 2).sum(1)[:, None] - 2 * Q64 @ C64.T + (C64 ** 2).sum(1)[None, :]
    np.testing.assert_allclose(d, direct, rtol=1e-14)
    np.testing.assert_allclose(d, expand, rtol=1e-12, atol=1e-12)


def test_probe_is_bruteforce_knn_with_id_tiebreak(rng):
    Q = rng.standard_normal((9, 5)).astype(np.float32)
    Cn = rng.standard_normal((40, 5)).astype(np.float32)
    Cn[17] = Cn[3]          # exact duplicates: ties must resolve to the lower id
    Cn[30] = Cn[3]
    pid, pd = orc.probe(Q, Cn, 11)
    d = ((Q.astype(np.float64)[:, None] - Cn.astype(np.float64)[None]) ** 2).sum(-1)
    for q in range(9):
        order = np.lexsort((np.arange(40), d[q]))[:11]
        assert (pid[q] == order).all()
        np.testing.assert_allclose(pd[q], d[q][order], rtol=1e-14)
    # the duplicate triple, when selected, appears in id order
    for q in range(9):
        got = [j for j in pid[q] if j in (3, 17, 30)]
        assert got == sorted(got)


def test_smallest_against_python_sort(rng):
    v = rng.integers(0, 6, 200).astype(np.float64)        # many exact ties
    tie = rng.permutation(200)
    pos, val = orc.smallest(v, 50, tie)
    ref = sorted(range(200), key=lambda i: (v[i], tie[i]))[:50]
    assert list(pos) == ref
    assert (val == v[ref]).all()


# ------------------------------------------------------------------ stage 2


def test_scores_equal_distance_to_explicit_subcentroid(tiny, rng):
    spec, ix, Q, _ = tiny
    pid, _ = orc.probe(Q[:20], ix.centroids, spec.nprobe)
    sc = orc.scores(Q[:20], ix, pid)
    c = ix.centroids.astype(np.float64)
    for q in range(20):
        for p in range(spec.nprobe):
            r = pid[q, p]
            mu = c[r][None] + float(ix.alpha[r]) * (c[ix.nbr[r]] - c[r][None])       # [L, D]
            direct = ((Q[q].astype(np.float64)[None] - mu) ** 2).sum(1)
            # cs_dist2 is stored in fp32, which bounds the agreement
            np.testing.assert_allclose(sc[q, p], direct, rtol=0, atol=2e-7)


def test_scores_alpha_zero_and_one(rng):
    D, K, L = 6, 12, 4
    Cn = rng.standard_normal((K, D)).astype(np.float32)
    nbr, cs = orc.neighbours(Cn, L)
    Q = rng.standard_normal((3, D)).astype(np.float32)
    pid, pd = orc.probe(Q, Cn, 5)
    d = orc.coarse_dist(Q, Cn)
    ix0 = tiny_index(D, K, L, 1, centroids=Cn, nbr=nbr, cs_dist2=cs, alpha=np.zeros(K, np.float32))
    sc0 = orc.scores(Q, ix0, pid)
    assert (sc0 == pd[:, :, None]).all()                       # alpha = 0: subcentroid = c for every l
    ix1 = tiny_index(D, K, L, 1, centroids=Cn, nbr=nbr, cs_dist2=cs, alpha=np.ones(K, np.float32))
    sc1 = orc.scores(Q, ix1, pid)
    for q in range(3):
        assert (sc1[q] == d[q][nbr[pid[q]]]).all()             # alpha = 1: subcentroid = s_l


def test_hand_example_eq7_eq6():
    g = read_golden("eq6_eq7_hand_example.txt")
    q, c, s, r = (g[k][0].astype(np.float32) for k in ("q", "c", "s", "r"))
    a = np.float32(g["alpha"][0][0])
    # two regions: region 0 = c with neighbour 1 = s (and vice versa); one PQ block of 2 dims whose
    # codeword 5 is r; a single stored point in subregion (0, 0) with id 42.
    cb = np.zeros((1, 256, 2), np.float32)
    cb[0, 5] = r
    table = np.linspace(-1, 1, 256).astype(np.float32)
    table[100] = np.float32(g["const_t"][0][0])
    table.sort()
    byte = int(np.argmin(np.abs(table.astype(np.float64) - g["const_t"][0][0])))
    ix = tiny_index(2, 2, 1, 1, centroids=np.stack([c, s]), nbr=np.array([[1], [0]], np.int32),
                    alpha=np.array([a, a]), cs_dist2=np.array([[8.0], [8.0]], np.float32), pq_codebook=cb,
                    const_table=table, sub_offsets=np.array([0, 1, 1], np.uint32),
                    codes=np.array([[5]], np.uint8), const_byte=np.array([byte], np.uint8),
                    ids=np.array([42], np.int32))
    st = orc.search_staged(ix, q[None], nprobe=1, prune_frac=1.0, k=2)
    assert st["probe_id"][0, 0] == 0
    assert st["scores"][0, 0, 0] == pytest.approx(g["dist_q_mu"][0][0], abs=1e-12)
    assert st["ids"][0].tolist() == [42, -1]
    assert st["dists"][0, 0] == pytest.approx(g["dist_q_point"][0][0], abs=1e-7)   # fp32 codeword / table
    assert np.isinf(st["dists"][0, 1])


# ------------------------------------------------------------------ stage 3


def test_prune_is_global_bruteforce_sort(rng):
    nq, P, L = 4, 6, 5
    sc = rng.integers(0, 9, (nq, P, L)).astype(np.float64)     # ties on purpose
    pid = np.stack([rng.permutation(50)[:P] for _ in range(nq)]).astype(np.int32)
    for tau, S_expect in ((0.5, 15), (0.34, 11), (1.0, 30), (1e-9, 1), (0.3, 9)):
        kept, ks = orc.prune(sc, pid, tau)
        assert kept.shape[1] == S_expect == orc.num_kept(tau, P, L)
        for q in range(nq):
            sid = (pid[q].astype(np.int64)[:, None] * L + np.arange(L)[None]).ravel()
            flat = sc[q].ravel()
            ref = sorted(range(P * L), key=lambda i: (flat[i], sid[i]))[:S_expect]
            assert kept[q].tolist() == [int(sid[i]) for i in ref]
            assert ks[q].tolist() == [flat[i] for i in ref]
    kept, _ = orc.prune(sc, pid, 1.0)                          # tau = 1 keeps every scored subregion
    for q in range(nq):
        sid = (pid[q].astype(np.int64)[:, None] * L + np.arange(L)[None]).ravel()
        assert sorted(kept[q].tolist()) == sorted(sid.tolist())


# -------------------------------------------------------------- stages 4 + 5


def explicit_points(ix, region_of_pos, sub_of_pos):
    """mu + decode(code) for every stored point, built from the definitions in numpy."""
    c = ix.centroids.astype(np.float64)
    s = c[ix.nbr[region_of_pos, sub_of_pos]]
    mu = c[region_of_pos] + ix.alpha[region_of_pos].astype(np.float64)[:, None] * (s - c[region_of_pos])
    ds = ix.D // ix.M
    dec = np.concatenate([ix.pq_codebook[m][ix.codes[:, m]].astype(np.float64) for m in range(ix.M)], axis=1)
    assert dec.shape[1] == ds * ix.M
    return mu, dec


def pos_to_bucket(ix):
    sizes = np.diff(ix.sub_offsets.astype(np.int64))
    bucket = np.repeat(np.arange(ix.K * ix.L), sizes)
    return bucket // ix.L, bucket % ix.L


def test_lut_is_inner_product_table(tiny):
    spec, ix, Q, _ = tiny
    T = orc.lut(Q[:5], ix)
    ds = ix.D // ix.M
    for m in range(ix.M):
        ref = -2.0 * Q[:5, m * ds:(m + 1) * ds].astype(np.float64) @ ix.pq_codebook[m].astype(np.float64).T
        np.testing.assert_allclose(T[:, m, :], ref, rtol=1e-13, atol=1e-15)


def test_scan_equals_distance_to_explicitly_decoded_points(tiny):
    """Eq. (6) with the unquantised per-point term reproduces ||q - (mu + decode(code))||^2."""
    spec, ix, Q, _ = tiny
    reg, sub = pos_to_bucket(ix)
    mu, dec = explicit_points(ix, reg, sub)
    t_exact = 2.0 * (mu * dec).sum(1) + (dec * dec).sum(1)
    nq = 15
    pid, _ = orc.probe(Q[:nq], ix.centroids, spec.nprobe)
    sc = orc.scores(Q[:nq], ix, pid)
    kept, ks = orc.prune(sc, pid, spec.prune_frac)
    T = orc.lut(Q[:nq], ix)
    start, pos, dist = orc.scan(ix, kept, ks, T, const_exact=t_exact)
    assert start[-1] == pos.shape[0] > 0
    for q in range(nq):
        p = pos[start[q]:start[q + 1]]
        direct = ((Q[q].astype(np.float64)[None] - mu[p] - dec[p]) ** 2).sum(1)
        np.testing.assert_allclose(dist[start[q]:start[q + 1]], direct, rtol=0, atol=3e-7)
        # candidates are exactly the members of the kept subregions
        members = np.concatenate([np.arange(ix.sub_offsets[b], ix.sub_offsets[b + 1]) for b in kept[q]])
        assert (p == members).all()
    # with the stored byte the estimate moves by exactly the byte's quantisation error
    start2, pos2, dist2 = orc.scan(ix, kept, ks, T)
    assert (pos2 == pos).all()
    err = ix.const_table[ix.const_byte[pos]].astype(np.float64) - t_exact[pos]
    np.testing.assert_allclose(dist2 - dist, err, rtol=0, atol=1e-12)
    gaps = np.diff(ix.const_table.astype(np.float64))
    inside = (t_exact[pos] >= ix.const_table[0]) & (t_exact[pos] <= ix.const_table[-1])
    assert (np.abs(err[inside]) <= gaps.max() / 2 + 1e-6).all()


# ------------------------------------------------------------------ stage 6


def test_select_bruteforce_and_padding(rng):
    ids = rng.permutation(500).astype(np.int32)
    ix = tiny_index(ids=ids)
    pos = rng.permutation(500)[:60].astype(np.int64)
    dist = rng.integers(0, 5, 60).astype(np.float64)
    oi, od = orc.select(ix, pos, dist, 25)
    ref = sorted(range(60), key=lambda i: (dist[i], ids[pos[i]]))[:25]
    assert oi.tolist() == [int(ids[pos[i]]) for i in ref]
    assert od.tolist() == [dist[i] for i in ref]
    oi, od = orc.select(ix, pos[:3], dist[:3], 5)
    assert oi[3:].tolist() == [-1, -1] and np.isinf(od[3:]).all() and (oi[:3] >= 0).all()
    oi, od = orc.select(ix, pos[:0], dist[:0], 4)
    assert oi.tolist() == [-1] * 4 and np.isinf(od).all()


# --------------------------------------------------------------- whole path


def test_full_probe_no_pruning_is_exhaustive_adc(tiny):
    """nprobe = K and tau = 1 visits every stored point: the result must be the plain
    exhaustive PQ scan over explicitly decoded points (plus each byte's quantisation error)."""
    spec, ix, Q, _ = tiny
    reg, sub = pos_to_bucket(ix)
    mu, dec = explicit_points(ix, reg, sub)
    t_exact = 2.0 * (mu * dec).sum(1) + (dec * dec).sum(1)
    shift = ix.const_table[ix.const_byte].astype(np.float64) - t_exact
    nq, k = 6, 20
    oi, od, ns = orc.search(ix, Q[:nq], ix.K, 1.0, k)
    assert (ns == ix.N).all()
    for q in range(nq):
        full = ((Q[q].astype(np.float64)[None] - mu - dec) ** 2).sum(1) + shift
        order = np.lexsort((ix.ids, full))[:k]
        # fp32-stored cs_dist2 perturbs estimates by < 1e-6: compare as sets unless gaps are clear
        assert set(oi[q].tolist()) == set(ix.ids[order].tolist())
        np.testing.assert_allclose(od[q], full[order], rtol=0, atol=1e-6)


def test_search_equals_staged_composition(tiny):
    spec, ix, Q, _ = tiny
    oi, od, ns = orc.search(ix, Q, spec.nprobe, spec.prune_frac, spec.k)
    st = orc.search_staged(ix, Q, spec.nprobe, spec.prune_frac, spec.k)
    assert (oi == st["ids"]).all() and (od == st["dists"]).all()
    assert (ns == np.diff(st["cand_start"])).all()


def test_recall_against_exact_knn_grows_with_nprobe(tiny):
    """With tau = 1 the candidate sets are nested in nprobe, so recall@k against the exact
    fp64 nearest neighbours cannot decrease."""
    spec, ix, Q, X = tiny
    k = 10
    X64 = X.astype(np.float64)
    exact = np.stack([np.lexsort((np.arange(X.shape[0]), ((X64 - q.astype(np.float64)) ** 2).sum(1)))[:k]
                      for q in Q])
    recalls, nn_in_cands = [], []
    for P in (1, 2, 4, 8, 16, 64):
        st = orc.search_staged(ix, Q, P, 1.0, k)
        recalls.append(np.mean([len(set(st["ids"][q]) & set(exact[q])) / k for q in range(Q.shape[0])]))
        nn_in_cands.append(np.mean([exact[q, 0] in ix.ids[st["cand_pos"][st["cand_start"][q]:st["cand_start"][q + 1]]]
                                    for q in range(Q.shape[0])]))
    assert all(b >= a for a, b in zip(nn_in_cands, nn_in_cands[1:]))     # nested candidate sets: exact
    assert all(b >= a - 0.02 for a, b in zip(recalls, recalls[1:]))      # reranked by compressed distances: trend
    assert nn_in_cands[-1] >= 0.95 and recalls[-1] >= recalls[0]


# ---------------------------------------------------------- candidate budget


def _walk(sub, score, sizes, R):
    """The traversal written out: ascending (score, subregion id), stop once R points are in."""
    order = sorted(range(len(sub)), key=lambda j: (score[j], sub[j]))
    flags, collected = [0] * len(sub), 0
    for j in order:
        if collected >= R:
            break
        flags[j] = 1
        collected += sizes[sub[j]]
    return flags, collected


def test_budget_walk_against_python_traversal(rng):
    """Planted ties in the scores, empty subregions, budgets below, at and above what is there."""
    nsub, nq, S = 40, 5, 17
    sizes = rng.integers(0, 6, nsub)
    sizes[rng.permutation(nsub)[:8]] = 0
    off = np.zeros(nsub + 1, np.uint32)
    off[1:] = np.cumsum(sizes)
    ix = tiny_index(K=nsub, L=1, sub_offsets=off, codes=np.zeros((int(off[-1]), 1), np.uint8),
                    const_byte=np.zeros(int(off[-1]), np.uint8), ids=np.arange(int(off[-1]), dtype=np.int32))
    sub = np.stack([rng.permutation(nsub)[:S] for _ in range(nq)]).astype(np.int64)
    score = rng.integers(0, 5, (nq, S)).astype(np.float64)
    for R in (1, 2, 7, 20, 10 ** 6):
        vis = orc.budget_visit(ix, sub, score, R)
        for q in range(nq):
            flags, collected = _walk(sub[q].tolist(), score[q].tolist(), sizes, R)
            assert vis[q].tolist() == flags, (R, q)
            total = int(sizes[sub[q]].sum())
            got = int(sizes[sub[q]][vis[q] == 1].sum())
            assert got == collected and got >= min(R, total)
            if got > R:                                   # only the subregion that crosses R overshoots
                last = max((j for j in range(S) if flags[j]), key=lambda j: (score[q, j], sub[q, j]))
                assert got - sizes[sub[q, last]] < R


def test_budget_nested_and_unbounded_budget_is_plain_search(tiny):
    spec, ix, Q, X = tiny
    Qs = Q[:12]
    ids_all, d_all, ns_all = orc.search(ix, Qs, spec.nprobe, 0.5, 10)
    ids_b, d_b, ns_b, st = orc.search_budget(ix, Qs, spec.nprobe, 0.5, 10 ** 9, 10)
    assert (ids_b == ids_all).all() and (d_b == d_all).all() and (ns_b == ns_all).all()
    assert (st["visit"] == 1).all()
    prev = None
    for R in (1, 50, 300, 1000):
        ids_r, d_r, ns_r, st = orc.search_budget(ix, Qs, spec.nprobe, 0.5, R, 10)
        assert (ns_r >= np.minimum(R, ns_all)).all() and (ns_r <= ns_all).all()
        if prev is not None:
            assert (st["visit"] >= prev).all()            # a larger budget visits a superset
        prev = st["visit"]
        # the result is the plain top-k over exactly the visited subregions' points
        for q in range(len(Qs)):
            cp = st["cand_pos"][st["cand_start"][q]:st["cand_start"][q + 1]]
            cd = st["cand_dist"][st["cand_start"][q]:st["cand_start"][q + 1]]
            sizes = np.diff(ix.sub_offsets.astype(np.int64))[st["scan_sub"][q]]
            assert len(cp) == int(sizes[st["visit"][q] == 1].sum())
            ref = sorted(zip(cd.tolist(), ix.ids[cp].tolist()))[:10]
            got = [(d, i) for d, i in zip(d_r[q].tolist(), ids_r[q].tolist()) if i >= 0]
            assert got == ref


# ------------------------------------------------- rotation in front of the PQ


def random_rotation(D, rng):
    q, r = np.linalg.qr(rng.standard_normal((D, D)))
    return (q * np.sign(np.diag(r))[None, :]).astype(np.float32)


def test_rotate_is_the_matrix_product(rng):
    X = rng.standard_normal((7, 5))
    R = rng.standard_normal((5, 5)).astype(np.float32)          # not symmetric: a transposed operand shows
    np.testing.assert_allclose(orc.rotate(X, R), X @ R.astype(np.float64).T, rtol=0, atol=1e-14)
    np.testing.assert_allclose(orc.rotate(X, np.eye(5, dtype=np.float32)), X, rtol=0, atol=0)


def rotated_tiny(tiny, rng):
    """The tiny index re-encoded with a random orthogonal rotation in front of its (unchanged) PQ."""
    spec, ix, Q, X = tiny
    R = random_rotation(spec.D, rng)
    enc = orc.encode(X, ix.centroids, ix.nbr, ix.alpha, ix.pq_codebook, ix.const_table, rotation=R)
    perm, off = orc.group(enc.region, enc.sub, spec.L, spec.K)
    ixr = orc.Index(spec.D, spec.M, spec.L, spec.K, spec.N, ix.centroids, ix.nbr, ix.alpha, ix.cs_dist2,
                    ix.pq_codebook, ix.const_table, off, np.ascontiguousarray(enc.codes[perm]),
                    np.ascontiguousarray(enc.const_byte[perm]), np.arange(spec.N, dtype=np.int32)[perm].copy(), R)
    return ixr, R


def test_rotation_identity_changes_nothing(tiny):
    spec, ix, Q, X = tiny
    eye = np.eye(spec.D, dtype=np.float32)
    a = orc.encode(X[:3000], ix.centroids, ix.nbr, ix.alpha, ix.pq_codebook, ix.const_table)
    b = orc.encode(X[:3000], ix.centroids, ix.nbr, ix.alpha, ix.pq_codebook, ix.const_table, rotation=eye)
    assert (a.codes == b.codes).all() and (a.const_byte == b.const_byte).all() and (a.t == b.t).all()
    import dataclasses
    ixe = dataclasses.replace(ix, rotation=eye)
    r0, r1 = orc.search(ix, Q[:20], spec.nprobe, spec.prune_frac, spec.k), orc.search(ixe, Q[:20], spec.nprobe, spec.prune_frac, spec.k)
    assert (r0[0] == r1[0]).all() and (r0[1] == r1[1]).all()


def test_rotated_scan_equals_distance_to_points_decoded_in_the_original_space(tiny, rng):
    """With an orthogonal R the stored point is mu + R^T decode(code); Eq. (6) with the table of the
    rotated query and the unquantised constant of the rotated subcentroid must give the plain
    distance to that point."""
    spec, _, Q, X = tiny
    ixr, R = rotated_tiny(tiny, rng)
    reg, sub = pos_to_bucket(ixr)
    mu, dec = explicit_points(ixr, reg, sub)                   # dec lives in the rotated space
    back = dec @ R.astype(np.float64)                          # R^T dec, row-wise
    mu_rot = mu @ R.astype(np.float64).T
    t_exact = 2.0 * (mu_rot * dec).sum(1) + (dec * dec).sum(1)
    # the encoder minimised the error of R (x - mu): decoding lands near the original points
    xg = X[ixr.ids].astype(np.float64)
    assert ((xg - mu - back) ** 2).sum(1).mean() < 0.7 * ((xg - mu) ** 2).sum(1).mean()   # (the codebook was trained without the rotation)
    nq = 10
    pid, _ = orc.probe(Q[:nq], ixr.centroids, spec.nprobe)
    kept, ks = orc.prune(orc.scores(Q[:nq], ixr, pid), pid, spec.prune_frac)
    start, pos, dist = orc.scan(ixr, kept, ks, orc.lut(Q[:nq], ixr), const_exact=t_exact)
    for q in range(nq):
        p = pos[start[q]:start[q + 1]]
        direct = ((Q[q].astype(np.float64)[None] - mu[p] - back[p]) ** 2).sum(1)
        np.testing.assert_allclose(dist[start[q]:start[q + 1]], direct, rtol=0, atol=2e-6)
    # the stored constant byte is the nearest table entry to that t
    np.testing.assert_array_equal(ixr.const_byte, orc.quantize_1d(t_exact, ixr.const_table))
    # and the one-call search is the staged composition
    oi, od, _ = orc.search(ixr, Q[:nq], spec.nprobe, spec.prune_frac, spec.k)
    st = orc.search_staged(ixr, Q[:nq], spec.nprobe, spec.prune_frac, spec.k)
    assert (oi == st["ids"]).all() and (od == st["dists"]).all()
