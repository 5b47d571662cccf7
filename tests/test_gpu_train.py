"""The device-side index construction routines against the oracle's (needs an MI355X)."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

import synthdata as sd
import paper_1802_02422_amd as ivf
from oracle import ivf_oracle as orc
import parity


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


@pytest.mark.parametrize("n,nb", [(1, 1), (4097, 3), (100_000, 70_000), (300_001, 1 << 21), (50_000, 2)])
def test_group_is_a_stable_counting_sort(n, nb):
    print("case: group", n, nb, flush=True)
    rng = np.random.default_rng(n + nb)
    bucket = rng.integers(0, nb, n).astype(np.int32)
    if n > 1000:
        bucket[rng.integers(0, n, n // 3)] = nb - 1        # one crowded bucket, many empty ones
    perm, off = ivf.ivf_group(dev(bucket), nb)
    perm, off = perm.cpu().numpy(), off.cpu().numpy().view(np.uint32).astype(np.int64)
    ref = np.lexsort((np.arange(n), bucket))
    assert (perm == ref).all()
    sizes = np.bincount(bucket, minlength=nb)
    assert off[0] == 0 and (np.diff(off) == sizes).all()
    # the rows in grouped order
    rows = rng.integers(0, 255, (n, 16)).astype(np.uint8)
    got = ivf.ivf_gather_rows(dev(rows), dev(perm.astype(np.int32))).cpu().numpy()
    assert (got == rows[ref]).all()
    b1 = rng.integers(0, 255, n).astype(np.uint8)
    assert (ivf.ivf_gather_rows(dev(b1), dev(perm.astype(np.int32))).cpu().numpy() == b1[ref]).all()
    r, s = rng.integers(0, 1000, n).astype(np.int32), rng.integers(0, 7, n).astype(np.int32)
    assert (ivf.ivf_bucket_ids(dev(r), dev(s), 7).cpu().numpy() == r * 7 + s).all()


def test_cluster_means_and_kmeans_match_oracle(small):
    spec, ix, Q, X = small
    print("case: kmeans small", flush=True)
    mix = sd.make_mixture(spec.kind, spec.n_mix, spec.D)
    Xt = sd.draw_points(mix, spec.n_train, 0, "train")[0].numpy()
    init = sd.draw_indices(spec.n_train, spec.K, "kmeans-init").numpy()
    Xd = dev(Xt)
    # zero rounds: the initial points
    c0 = ivf.ivf_kmeans(Xd, spec.K, 0, dev(init)).cpu().numpy()
    assert (c0 == Xt[init]).all()
    # update step alone, from the oracle's assignment: means in fp64 rounded to fp32
    lab, _ = orc.assign(Xt, c0)
    got = ivf.ivf_cluster_means(Xd, dev(lab), dev(c0)).cpu().numpy()
    sums = np.zeros((spec.K, spec.D))
    np.add.at(sums, lab, Xt.astype(np.float64))
    cnt = np.bincount(lab, minlength=spec.K)
    ref = np.where(cnt[:, None] > 0, sums / np.maximum(cnt, 1)[:, None], c0).astype(np.float32)
    assert np.abs(got - ref).max() <= 1e-7
    assert (got[cnt == 0] == c0[cnt == 0]).all()
    # whole Lloyd runs from the same start
    for iters in (1, 3):
        c_g, obj = ivf.ivf_kmeans(Xd, spec.K, iters, dev(init), want_objective=True)
        c_g, obj = c_g.cpu().numpy(), obj.cpu().numpy()
        c_o, obj_o = orc.kmeans(Xt, spec.K, iters, init)
        close = np.abs(c_g - c_o).max(1) <= 1e-5
        print("  iters", iters, "centroids equal within 1e-5:", close.mean(), "objective", obj, obj_o, flush=True)
        assert close.mean() >= 0.99
        np.testing.assert_allclose(obj, obj_o, rtol=1e-5)
        assert (np.diff(obj) <= 1e-6 * obj[0]).all()
    again = ivf.ivf_kmeans(Xd, spec.K, 3, dev(init)).cpu().numpy()
    assert (again == c_g).all(), "two runs must give the same bits"


def test_neighbours_match_oracle_with_duplicate_centroids(tiny):
    spec, ix, Q, X = tiny
    print("case: neighbours", flush=True)
    C = ix.centroids.copy()
    C[10:20] = C[5]                                  # eleven identical centroids (ids 5, 10..19)
    for L in (8, 3):
        nbr, cs = ivf.ivf_neighbours(dev(C), L)
        nbr, cs = nbr.cpu().numpy(), cs.cpu().numpy()
        o_nbr, o_cs = orc.neighbours(C, L)
        same = (nbr == o_nbr)
        print("  L", L, "agreement", same.mean(), flush=True)
        assert same.mean() >= 0.999
        # rows of the duplicated centroids: the lowest other ids among the copies, at distance 0
        for r in (5, 10, 19):
            assert (nbr[r] == o_nbr[r]).all() and (cs[r][: min(L, 10)] <= 1e-6).all()
        np.testing.assert_allclose(cs[same], o_cs[same], rtol=1e-4, atol=1e-6)
        assert (np.diff(cs, axis=1) >= 0).all() and (nbr != np.arange(spec.K)[:, None]).all()


def test_learn_alpha_matches_oracle(tiny):
    spec, ix, Q, X = tiny
    print("case: alpha", flush=True)
    n = 20000
    x = X[:n]
    reg, _ = orc.assign(x, ix.centroids)
    a = ivf.ivf_learn_alpha(dev(ix.centroids), dev(ix.nbr), dev(x), dev(reg)).cpu().numpy()
    ref = orc.learn_alpha(x, reg, ix.centroids, ix.nbr)
    np.testing.assert_allclose(a, ref, rtol=0, atol=2e-6)        # pooled value of regions without points included
    assert (np.bincount(reg, minlength=spec.K) == 0).any(), "the case should contain regions without training points"
    b = ivf.ivf_learn_alpha(dev(ix.centroids), dev(ix.nbr), dev(x), dev(reg)).cpu().numpy()
    assert (a == b).all(), "two runs must give the same bits"


def test_pq_train_and_scalar_table_match_oracle(tiny):
    spec, ix, Q, X = tiny
    print("case: pq_train", flush=True)
    n = 30000
    x = X[:n]
    reg, _ = orc.assign(x, ix.centroids)
    sub, mu, res = orc.sub_assign(x, reg, ix.centroids, ix.nbr, ix.alpha)
    E = res.astype(np.float32)
    init = sd.draw_indices(n, 256, "pq-init-test").numpy()
    for iters in (0, 1, 4):
        cb = ivf.ivf_pq_train(dev(E), spec.M, iters, dev(init)).cpu().numpy()
        cb_o, _ = orc.pq_train(E, spec.M, iters, init)
        close = np.abs(cb - cb_o).max(2) <= 1e-6
        print("  iters", iters, "codewords equal within 1e-6:", close.mean(), flush=True)
        assert close.mean() >= (1.0 if iters == 0 else 0.97)
        # as good a codebook: quantisation error of the training rows within 0.1 %
        err = lambda c: float(((E.astype(np.float64) - orc.pq_decode(orc.pq_encode(E.astype(np.float64), c), c)) ** 2).sum())
        if iters:
            assert abs(err(cb) - err(cb_o)) <= 1e-3 * err(cb_o)
    # the 256-level table on the per-point terms
    codes = orc.pq_encode(res, cb_o)
    t = orc.const_term(mu, codes, cb_o).astype(np.float32)
    for iters in (0, 1, 20):
        tab = ivf.ivf_lloyd_1d(dev(t), iters).cpu().numpy()
        tab_o = orc.lloyd_1d(t.astype(np.float64), iters)
        assert (np.diff(tab) >= 0).all()
        print("  table iters", iters, "max abs diff", np.abs(tab - tab_o).max(), flush=True)
        np.testing.assert_allclose(tab, tab_o, rtol=1e-6, atol=1e-7)
    # few values, many equal: levels without values keep their entries
    t2 = np.repeat(np.array([0.5, -1.0, 2.0], np.float32), 40)
    np.testing.assert_allclose(ivf.ivf_lloyd_1d(dev(t2), 5).cpu().numpy(), orc.lloyd_1d(t2.astype(np.float64), 5), rtol=1e-6)


def test_whole_construction_from_the_oracles_start(small):
    """The construction pipeline step by step through the C ABI, from the training sample and the
    initial indices the oracle used for the cached `small` index: the product must be that index up
    to near-ties (k-means amplifies a rounding-level difference in one assignment into slightly
    different centroids, so later arrays are compared where the earlier ones agree)."""
    spec, ix, Q, X = small
    print("case: construction small", flush=True)
    mix = sd.make_mixture(spec.kind, spec.n_mix, spec.D)
    Xt = sd.draw_points(mix, spec.n_train, 0, "train")[0].numpy()
    ci = sd.draw_indices(spec.n_train, spec.K, "kmeans-init").numpy()
    pi = sd.draw_indices(spec.n_train, 256, "pq-init").numpy()
    Xd, Xb = dev(Xt), dev(X)
    cent = ivf.ivf_kmeans(Xd, spec.K, 10, dev(ci))
    c_same = (np.abs(cent.cpu().numpy() - ix.centroids).max(1) <= 1e-5)
    print("  centroids equal:", c_same.mean(), flush=True)
    assert c_same.mean() >= 0.98
    # from here on with the oracle's centroids, so that each later step is compared on equal inputs
    cent = dev(ix.centroids)
    nbr, cs = ivf.ivf_neighbours(cent, spec.L)
    assert (nbr.cpu().numpy() == ix.nbr).mean() >= 0.999
    reg_t = ivf.ivf_coarse_topk(cent, Xd, 1)[0].view(-1).contiguous()
    nbr = dev(ix.nbr)
    alpha = ivf.ivf_learn_alpha(cent, nbr, Xd, reg_t)
    a_same = np.abs(alpha.cpu().numpy() - ix.alpha) <= 1e-5
    print("  alpha equal:", a_same.mean(), flush=True)
    assert a_same.mean() >= 0.99
    desc = ivf.IndexDesc(cent, nbr, dev(ix.alpha), dev(ix.cs_dist2), None, spec.M)
    _, _, _, _, _, res = ivf.ivf_encode(desc, Xd, region_in=reg_t, want_residual=True)
    cb = ivf.ivf_pq_train(res, spec.M, 20, dev(pi))
    cb_same = np.abs(cb.cpu().numpy() - ix.pq_codebook).max(2) <= 1e-5
    print("  codewords equal:", cb_same.mean(), flush=True)
    assert cb_same.mean() >= 0.9
    desc.pq_codebook = dev(ix.pq_codebook)
    _, _, _, _, t = ivf.ivf_encode(desc, Xd, region_in=reg_t, want_t=True)
    tab = ivf.ivf_lloyd_1d(t, 20).cpu().numpy()
    print("  table max diff:", np.abs(tab - ix.const_table).max(), flush=True)
    np.testing.assert_allclose(tab, ix.const_table, rtol=2e-3, atol=2e-5)
    desc.const_table = dev(ix.const_table)
    # encode the base set and group it: the oracle's grouped index, near-ties aside
    r, s_, cd, by, _ = ivf.ivf_encode(desc, Xb)
    bucket = ivf.ivf_bucket_ids(r, s_, spec.L)
    perm, off = ivf.ivf_group(bucket, spec.K * spec.L)
    codes = ivf.ivf_gather_rows(cd, perm).cpu().numpy()
    byte = ivf.ivf_gather_rows(by, perm).cpu().numpy()
    perm, off = perm.cpu().numpy(), off.cpu().numpy().view(np.uint32)
    o_bucket = np.repeat(np.arange(spec.K * spec.L), np.diff(ix.sub_offsets.astype(np.int64)))
    o_bucket_of_id = np.empty(spec.N, np.int64)
    o_bucket_of_id[ix.ids] = o_bucket
    same_bucket = bucket.cpu().numpy() == o_bucket_of_id
    print("  points in the oracle's subregion:", same_bucket.mean(), flush=True)
    assert same_bucket.mean() >= 0.995
    if same_bucket.all():
        assert (perm == ix.ids).all() and (off == ix.sub_offsets).all()
        assert (codes == ix.codes).mean() >= 0.999 and (byte == ix.const_byte).mean() >= 0.99
    # and it searches like the oracle says it should
    d2 = ivf.IndexDesc(cent, nbr, dev(ix.alpha), dev(ix.cs_dist2), dev(ix.pq_codebook), const_table=dev(ix.const_table),
                       sub_offsets=dev(off.view(np.int32)), codes=dev(codes), const_byte=dev(byte), ids=dev(perm))
    ix2 = orc.Index(spec.D, spec.M, spec.L, spec.K, spec.N, ix.centroids, ix.nbr, ix.alpha, ix.cs_dist2, ix.pq_codebook,
                    ix.const_table, off, codes, byte, perm)
    handle = ivf.ivf_load_index(d2)
    out = parity.run_gpu_search(handle, Q[:100], spec.nprobe, spec.prune_frac, spec.k)
    rep = parity.check_search(ix2, Q[:100], spec.nprobe, spec.prune_frac, spec.k, out)
    print(rep, flush=True)
    rep.assert_ok()
