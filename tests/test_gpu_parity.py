"""HIP library vs oracle through the C ABI (needs an MI355X)."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

import paper_1802_02422_amd as ivf
from oracle import ivf_oracle as orc
import parity


@pytest.fixture(scope="module")
def tiny_gpu(tiny):
    spec, ix, Q, X = tiny
    handle = ivf.ivf_load_index(parity.to_device(ix))
    return spec, ix, Q, X, handle


def test_library_is_loaded():
    assert ivf.load_library() is not None and torch.cuda.is_available()


def test_coarse_topk_matches_bruteforce(tiny):
    spec, ix, Q, X = tiny
    print("case: coarse_topk tiny", flush=True)
    C = torch.from_numpy(ix.centroids).cuda()
    for nq, P in ((100, 16), (1, 1), (77, 1), (100, 1024)):
        gid, gd = ivf.ivf_coarse_topk(C, torch.from_numpy(Q[:nq]).cuda(), P)
        gid, gd = gid.cpu().numpy(), gd.cpu().numpy()
        oid, od = orc.probe(Q[:nq], ix.centroids, P)
        at = parity.abs_term(ix, Q[:nq])
        c64 = ix.centroids.astype(np.float64)
        near = 0
        for q in range(nq):
            dist = lambda j: float(((Q[q].astype(np.float64) - c64[j]) ** 2).sum())
            kind, gap = parity.compare_selection(gid[q], oid[q], dist, od[q, -1], max(1e-5 * od[q, -1], at[q]))
            assert kind != "mismatch", (nq, P, q, gap)
            near += kind == "near"
        assert near <= 2
        d_true = ((Q[:nq].astype(np.float64)[:, None] - c64[gid]) ** 2).sum(-1)
        assert (np.abs(gd - d_true) <= np.maximum(1e-4 * d_true, at[:, None])).all()


@pytest.mark.parametrize("D,K,nq", [(20, 300, 1), (96, 1280, 65), (100, 1000, 128), (128, 1024, 200), (96, 2560, 300),
                                    (96, 1152, 200), (96, 384, 130), (128, 9 * 128, 70)])
def test_coarse_distances_within_fp32_bound_for_all_kernel_variants(D, K, nq):
    """Shapes that reach every variant of the coarse kernel (small batch, generic tile with a
    padded width, swept tiles with a partial last query tile, with fewer tiles than one write-out
    of the block minima covers and with rows of block minima that are not 16-byte aligned), rows of very different
    magnitude (centroid rows up to 2^16 apart under the one scale of the table), exact duplicates: every returned distance is within 16 u (|q|^2 + max |c|^2) of
    the fp64 value, and the P returned regions are the exact ones up to ties inside that bound."""
    print("case: coarse variants", D, K, nq, flush=True)
    rng = np.random.default_rng(1000 * D + K + nq)
    C = rng.standard_normal((K, D)) * np.exp2(rng.integers(-16, 1, size=(K, 1)))     # rows 2^-16 .. 2^0 apart
    Q = rng.standard_normal((nq, D)) * np.exp2(rng.integers(-8, 9, size=(nq, 1)))
    Q[0] = C[K // 2]                                     # a query that is a centroid: distance 0
    C, Q = C.astype(np.float32), Q.astype(np.float32)
    P = min(K, 64)
    gid, gd = ivf.ivf_coarse_topk(torch.from_numpy(C).cuda(), torch.from_numpy(Q).cuda(), P)
    gid, gd = gid.cpu().numpy(), gd.cpu().numpy()
    c64, q64 = C.astype(np.float64), Q.astype(np.float64)
    exact = (q64 ** 2).sum(1)[:, None] + (c64 ** 2).sum(1)[None, :] - 2.0 * q64 @ c64.T
    exact = np.maximum(exact, 0.0)
    u = 2.0 ** -24
    tol = 16 * u * ((q64 ** 2).sum(1) + (c64 ** 2).sum(1).max())
    err = np.abs(gd - np.take_along_axis(exact, gid.astype(np.int64), axis=1))
    print("  max error / tolerance: %.3f" % (err / tol[:, None]).max(), flush=True)
    assert (err <= tol[:, None]).all()
    assert gd[0].min() <= tol[0] and (gd >= 0).all()
    kth = np.sort(exact, axis=1)[:, P - 1]
    for q in range(nq):
        assert len(set(gid[q].tolist())) == P and (np.diff(gid[q]) > 0).all()      # distinct, ascending ids
        assert (exact[q, gid[q]] <= kth[q] + 2 * tol[q]).all()                       # nothing beyond the boundary
        must = np.nonzero(exact[q] < kth[q] - 2 * tol[q])[0]                         # clearly inside: all present
        assert np.isin(must, gid[q]).all()


def test_coarse_topk_beyond_the_lds_selection_limits():
    """More than 2^20 centroids (block minima no longer fit LDS) and more than 256 probes: the
    global-memory selection kernels, checked against brute force."""
    print("case: coarse_topk K = 1 100 003", flush=True)
    rng = np.random.default_rng(77)
    K, D = 1_100_003, 32
    C = rng.standard_normal((K, D)).astype(np.float32)
    Q = rng.standard_normal((70, D)).astype(np.float32)
    Cg = torch.from_numpy(C).cuda()
    c64 = C.astype(np.float64)
    cn = (c64 ** 2).sum(1)
    u = 2.0 ** -24
    for nq, P in ((3, 16), (70, 300)):
        gid, gd = ivf.ivf_coarse_topk(Cg, torch.from_numpy(Q[:nq]).cuda(), P)
        gid, gd = gid.cpu().numpy(), gd.cpu().numpy()
        for q in range(nq):
            q64 = Q[q].astype(np.float64)
            exact = np.maximum((q64 ** 2).sum() + cn - 2.0 * (c64 @ q64), 0.0)
            tol = 16 * u * ((q64 ** 2).sum() + cn.max())
            kth = np.partition(exact, P - 1)[P - 1]
            assert len(set(gid[q].tolist())) == P and (np.diff(gid[q]) > 0).all()
            assert (np.abs(gd[q] - exact[gid[q]]) <= tol).all()
            assert (exact[gid[q]] <= kth + 2 * tol).all()
            assert np.isin(np.nonzero(exact < kth - 2 * tol)[0], gid[q]).all()


def test_coarse_topk_with_thousands_of_tied_centroids():
    """6000 exact copies of one centroid closer to the queries than everything else: every copy ties
    at the block threshold, more survivors than the LDS selection holds, so the kernel takes its
    global-memory pass; the P results are the P lowest ids among the copies (ties by id)."""
    print("case: coarse_topk tied duplicates", flush=True)
    rng = np.random.default_rng(5)
    K, D, P = 16384, 96, 64
    C = rng.standard_normal((K, D)).astype(np.float32)
    dup = np.sort(rng.choice(K, size=6000, replace=False))
    C[dup] = C[dup[0]]
    Q = (C[dup[0]][None, :] + 0.01 * rng.standard_normal((130, D))).astype(np.float32)
    gid, gd = ivf.ivf_coarse_topk(torch.from_numpy(C).cuda(), torch.from_numpy(Q).cuda(), P)
    gid, gd = gid.cpu().numpy(), gd.cpu().numpy()
    assert (gid == dup[:P][None, :]).all()
    d_true = ((Q.astype(np.float64) - C[dup[0]].astype(np.float64)[None, :]) ** 2).sum(1)
    u = 2.0 ** -24
    tol = 16 * u * ((Q.astype(np.float64) ** 2).sum(1) + (C.astype(np.float64) ** 2).sum(1).max())
    assert (np.abs(gd - d_true[:, None]) <= tol[:, None]).all()
    assert (gd == gd[:, :1]).all()                       # identical operands give identical distances
    # the same with fewer copies than the limit: the LDS pass
    C2 = rng.standard_normal((K, D)).astype(np.float32)
    dup2 = np.sort(rng.choice(K, size=3000, replace=False))
    C2[dup2] = C[dup[0]]
    gid2, _ = ivf.ivf_coarse_topk(torch.from_numpy(C2).cuda(), torch.from_numpy(Q).cuda(), P)
    assert (gid2.cpu().numpy() == dup2[:P][None, :]).all()


def test_search_tiny_all_stages(tiny_gpu):
    spec, ix, Q, X, handle = tiny_gpu
    print("case: search tiny", spec, flush=True)
    out = parity.run_gpu_search(handle, Q, spec.nprobe, spec.prune_frac, spec.k)
    rep = parity.check_search(ix, Q, spec.nprobe, spec.prune_frac, spec.k, out)
    print(rep)
    rep.assert_ok()


@pytest.mark.parametrize("nprobe,tau,k,nq", [(1, 1.0, 1, 5), (16, 0.5, 10, 1), (64, 0.25, 100, 33),
                                             (1024, 1.0, 20, 3), (7, 0.01, 1024, 4), (3, 0.3, 100, 100)])
def test_search_tiny_parameter_corners(tiny_gpu, nprobe, tau, k, nq):
    spec, ix, Q, X, handle = tiny_gpu
    print("case: corners", nprobe, tau, k, nq, flush=True)
    out = parity.run_gpu_search(handle, Q[:nq], nprobe, tau, k)
    rep = parity.check_search(ix, Q[:nq], nprobe, tau, k, out)
    print(rep)
    rep.assert_ok(max_near_frac=0.2)


def test_search_is_deterministic_and_matches_plain_entry(tiny_gpu):
    spec, ix, Q, X, handle = tiny_gpu
    Qd = torch.from_numpy(Q).cuda()
    a = ivf.ivf_search_stages(handle, Qd, spec.nprobe, spec.prune_frac, spec.k)
    ids, d = ivf.ivf_search(handle, Qd, spec.nprobe, spec.prune_frac, spec.k)
    b = ivf.ivf_search_stages(handle, Qd, spec.nprobe, spec.prune_frac, spec.k)
    torch.cuda.synchronize()
    for n in a:
        assert torch.equal(a[n], b[n]), n
    assert torch.equal(ids, a["ids"]) and torch.equal(d, a["dists"])


def test_search_replays_from_a_captured_graph(tiny_gpu):
    """Once its scratch buffers exist a search neither allocates nor clears memory with memset nodes:
    it can be captured into a HIP graph.  Every replay, with eager searches of other shapes in
    between, returns the bits of the eager call."""
    spec, ix, Q, X, handle = tiny_gpu
    print("case: graph capture", flush=True)
    Qd = torch.from_numpy(Q).cuda()
    ids = torch.empty((len(Q), spec.k), dtype=torch.int32, device="cuda")
    d = torch.empty((len(Q), spec.k), dtype=torch.float32, device="cuda")
    ivf.ivf_search(handle, Qd, spec.nprobe, spec.prune_frac, spec.k, ids, d)      # sizes the scratch buffers
    torch.cuda.synchronize()
    ref_ids, ref_d = ids.clone(), d.clone()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        ivf.ivf_search(handle, Qd, spec.nprobe, spec.prune_frac, spec.k, ids, d)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        ivf.ivf_search(handle, Qd, spec.nprobe, spec.prune_frac, spec.k, ids, d)
    for rep in range(4):
        ids.fill_(-7)
        d.fill_(-7.0)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(ids, ref_ids) and torch.equal(d, ref_d), rep
        ivf.ivf_search(handle, Qd[: 3 + rep].contiguous(), 5 + rep, 1.0, 7)     # the program's own eager work in between
        torch.cuda.synchronize()
    del graph


def test_query_tiling_gives_identical_results(tiny_gpu):
    spec, ix, Q, X, handle = tiny_gpu
    Qd = torch.from_numpy(Q).cuda()
    a = ivf.ivf_search_stages(handle, Qd, spec.nprobe, spec.prune_frac, spec.k)
    h2 = ivf.ivf_load_index(parity.to_device(ix))
    ivf.ivf_set_scratch_limit(h2, 37 * ix.K * 4)          # distance tile of 37 queries: 3 passes, ragged tail
    b = ivf.ivf_search_stages(h2, Qd, spec.nprobe, spec.prune_frac, spec.k)
    torch.cuda.synchronize()
    for n in a:
        assert torch.equal(a[n], b[n]), n


def test_empty_and_invalid_arguments(tiny_gpu):
    spec, ix, Q, X, handle = tiny_gpu
    Qd = torch.from_numpy(Q).cuda()
    ids, d = ivf.ivf_search(handle, Qd[:0], 4, 0.5, 3)
    assert ids.shape == (0, 3)
    for bad in (dict(nprobe=0), dict(nprobe=ix.K + 1), dict(prune_frac=0.0), dict(prune_frac=1.5),
                dict(k=0), dict(k=5000)):
        args = dict(nprobe=4, prune_frac=0.5, k=3)
        args.update(bad)
        with pytest.raises(ivf.IvfError):
            ivf.ivf_search(handle, Qd, args["nprobe"], args["prune_frac"], args["k"])
    assert "must be" in ivf.ivf_last_error()


def test_encode_matches_oracle(tiny):
    spec, ix, Q, X = tiny
    print("case: encode tiny", flush=True)
    n = 5000
    x = X[:n]
    desc = parity.to_device(ix, with_codes=False)
    region, sub, codes, byte, t = ivf.ivf_encode(desc, torch.from_numpy(x).cuda(), want_t=True)
    region, sub, codes, byte, t = (v.cpu().numpy() for v in (region, sub, codes, byte, t))
    enc = orc.encode(x, ix.centroids, ix.nbr, ix.alpha, ix.pq_codebook, ix.const_table)
    assert (region == enc.region).mean() >= 0.999
    same = (region == enc.region) & (sub == enc.sub)
    assert same.mean() >= 0.995, same.mean()
    code_same = (codes[same] == enc.codes[same])
    assert code_same.mean() >= 0.999, code_same.mean()
    full = same & (codes == enc.codes).all(1)
    np.testing.assert_allclose(t[full], enc.t[full], rtol=1e-4, atol=2e-6)
    assert (byte[full] == enc.const_byte[full]).mean() >= 0.99
    # every disagreement must be a near-tie of the oracle's own fp64 decision
    c64 = ix.centroids.astype(np.float64)
    for i in np.flatnonzero(region != enc.region):
        d = ((x[i].astype(np.float64) - c64[[region[i], enc.region[i]]]) ** 2).sum(1)
        assert abs(d[0] - d[1]) <= 1e-5 * d[1]
    for i in np.flatnonzero((region == enc.region) & (sub != enc.sub)):
        r = region[i]
        mus = c64[r][None] + float(ix.alpha[r]) * (c64[ix.nbr[r]] - c64[r][None])
        d = ((x[i].astype(np.float64)[None] - mus) ** 2).sum(1)
        assert abs(d[sub[i]] - d[enc.sub[i]]) <= 1e-5 * max(d[enc.sub[i]], 1.0)
    ds = ix.D // ix.M
    for i in np.flatnonzero(same & ~(codes == enc.codes).all(1)):
        e = x[i].astype(np.float64) - enc.mu[i]
        for m in np.flatnonzero(codes[i] != enc.codes[i]):
            dd = ((e[m * ds:(m + 1) * ds][None] - ix.pq_codebook[m].astype(np.float64)) ** 2).sum(1)
            assert abs(dd[codes[i, m]] - dd[enc.codes[i, m]]) <= 1e-5 * max(dd[enc.codes[i, m]], 1e-3)
    tab = ix.const_table.astype(np.float64)
    for i in np.flatnonzero(full & (byte != enc.const_byte)):
        assert abs(abs(tab[byte[i]] - enc.t[i]) - abs(tab[enc.const_byte[i]] - enc.t[i])) <= 4e-6


def test_encode_with_given_regions(tiny):
    spec, ix, Q, X = tiny
    n = 1000
    desc = parity.to_device(ix, with_codes=False)
    xd = torch.from_numpy(X[:n]).cuda()
    r1, s1, c1, b1, _ = ivf.ivf_encode(desc, xd)
    r2, s2, c2, b2, _ = ivf.ivf_encode(desc, xd, region_in=r1)
    assert torch.equal(r1, r2) and torch.equal(s1, s2) and torch.equal(c1, c2) and torch.equal(b1, b2)
