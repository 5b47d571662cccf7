"""Candidate-budget search (candidate lists of a given length, Section 4) against the oracle, and
the largest score count one query may have (needs an MI355X)."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

import synthdata as sd
import paper_1802_02422_amd as ivf
from oracle import ivf_oracle as orc
import parity


def run_budget(handle, ix, Q, nprobe, tau, R, k, max_near_frac=0.05):
    Qd = torch.from_numpy(Q).cuda()
    so = ivf.ivf_search_stages(handle, Qd, nprobe, tau, k)
    bo = ivf.ivf_search_budget(handle, Qd, nprobe, tau, R, k)
    torch.cuda.synchronize()
    so = {n: v.cpu().numpy() for n, v in so.items()}
    bo = {n: v.cpu().numpy() for n, v in bo.items()}
    rep = parity.check_search_budget(ix, Q, nprobe, tau, R, k, so, bo)
    print("R =", R, rep, flush=True)
    rep.assert_ok(max_near_frac=max_near_frac)
    return so, bo


def test_budget_tiny(tiny):
    spec, ix, Q, X = tiny
    handle = ivf.ivf_load_index(parity.to_device(ix))
    print("case: budget tiny", flush=True)
    for R in (1, 17, 200, 700, 10 ** 7):
        so, bo = run_budget(handle, ix, Q, spec.nprobe, spec.prune_frac, R, spec.k)
        if R == 10 ** 7:                                  # more than there is: the plain search
            assert (bo["visited"] == 1).all()
            assert (bo["ids"] == so["ids"]).all() and (bo["dists"] == so["dists"]).all()
        else:
            assert (bo["n_scanned"] >= np.minimum(R, so["n_scanned"])).all()
    run_budget(handle, ix, Q[:9], 64, 1.0, 300, 20)      # without pruning
    with pytest.raises(ivf.IvfError):
        ivf.ivf_search_budget(handle, torch.from_numpy(Q).cuda(), 4, 0.5, 0, 3)
    ivf.ivf_free_index(handle)


def test_budget_small_many_tiles(small):
    spec, ix, Q, X = small
    handle = ivf.ivf_load_index(parity.to_device(ix))
    print("case: budget small", flush=True)
    for R in (100, 3000):
        run_budget(handle, ix, Q[:120], spec.nprobe, spec.prune_frac, R, spec.k)
    ivf.ivf_free_index(handle)


def test_budget_with_exactly_tied_scores_and_long_lists():
    """alpha = 0 everywhere: the L scores of a region tie exactly, so the crossing subregion is
    decided by the subregion id among equal scores; few regions, lists of thousands of points."""
    mix = sd.make_mixture("deep", 6, 32, name="degenerate")
    X = sd.draw_points(mix, 30000, 0, "deg-base")[0].numpy()
    Xt = sd.draw_points(mix, 5000, 0, "deg-train")[0].numpy()
    Q = sd.draw_queries(mix, 30, "deg-query").numpy()
    ix = orc.build_index(Xt, X, 12, 3, 16, sd.draw_indices(5000, 12, "deg-k").numpy(),
                         sd.draw_indices(5000, 256, "deg-pq").numpy(), kmeans_iters=3, pq_iters=3)
    alpha = np.zeros(12, np.float32)
    enc = orc.encode(X, ix.centroids, ix.nbr, alpha, ix.pq_codebook, ix.const_table)
    perm, off = orc.group(enc.region, enc.sub, 3, 12)
    ix0 = orc.Index(32, 16, 3, 12, 30000, ix.centroids, ix.nbr, alpha, ix.cs_dist2, ix.pq_codebook, ix.const_table,
                    off, np.ascontiguousarray(enc.codes[perm]), np.ascontiguousarray(enc.const_byte[perm]),
                    np.arange(30000, dtype=np.int32)[perm].copy())
    print("case: budget, tied scores", flush=True)
    for index in (ix, ix0):
        handle = ivf.ivf_load_index(parity.to_device(index))
        for R in (1, 2500, 9000):
            run_budget(handle, index, Q, 5, 0.8, R, 50, max_near_frac=1.0)
        ivf.ivf_free_index(handle)


def test_largest_score_count_per_query():
    """nprobe * L = 32768 (L = 128, nprobe = 256: the largest table of the paper's ablation over L)."""
    mix = sd.make_mixture("deep", 300, 32, name="wide")
    X = sd.draw_points(mix, 40000, 0, "wide-base")[0].numpy()
    Xt = sd.draw_points(mix, 8000, 0, "wide-train")[0].numpy()
    Q = sd.draw_queries(mix, 6, "wide-query").numpy()
    ix = orc.build_index(Xt, X, 400, 128, 8, sd.draw_indices(8000, 400, "wide-k").numpy(),
                         sd.draw_indices(8000, 256, "wide-pq").numpy(), kmeans_iters=3, pq_iters=3)
    handle = ivf.ivf_load_index(parity.to_device(ix))
    print("case: nprobe*L = 32768", flush=True)
    out = parity.run_gpu_search(handle, Q, 256, 0.2, 10)
    rep = parity.check_search(ix, Q, 256, 0.2, 10, out)
    print(rep, flush=True)
    rep.assert_ok(max_near_frac=0.2)
    run_budget(handle, ix, Q, 256, 0.5, 500, 10, max_near_frac=0.2)
    with pytest.raises(ivf.IvfError):
        ivf.ivf_search(handle, torch.from_numpy(Q).cuda(), 257, 0.2, 10)
    ivf.ivf_free_index(handle)
