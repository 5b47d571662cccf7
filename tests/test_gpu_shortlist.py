"""Nearest-centroid assignment through the certified shortlist (reduced-precision pass with an error
bound, exact decision among the listed pairs) against fp64 brute force: the returned centroid must be
the exact nearest one, whatever the magnitudes, however many ties there are, and also where the list
overflows and the one-pass kernel takes over."""
import os

import numpy as np
import pytest
import torch

import paper_1802_02422_amd as ivf

pytestmark = pytest.mark.gpu

U = 2.0 ** -24


def _exact(C, Q):
    c64, q64 = C.astype(np.float64), Q.astype(np.float64)
    d = (q64 ** 2).sum(1)[:, None] + (c64 ** 2).sum(1)[None, :] - 2.0 * q64 @ c64.T
    return np.maximum(d, 0.0)


def _assign(C, Q):
    gid, gd = ivf.ivf_coarse_topk(torch.from_numpy(C).cuda(), torch.from_numpy(Q).cuda(), 1)
    return gid.cpu().numpy()[:, 0].astype(np.int64), gd.cpu().numpy()[:, 0].astype(np.float64)


def _check(C, Q, gid, gd):
    """ids: the fp64 nearest, or within the fp32 rounding of the exact pass of it; distances within that rounding."""
    d = _exact(C, Q)
    best = d.min(1)
    tol = 16 * U * ((Q.astype(np.float64) ** 2).sum(1) + (C.astype(np.float64) ** 2).sum(1).max())
    got = d[np.arange(len(Q)), gid]
    assert (got <= best + tol).all(), float(((got - best) / tol).max())
    assert (np.abs(gd - got) <= tol).all()
    # clear winners must be returned exactly, and among exact duplicates of the winner the smallest id
    first = d.argmin(1)                                   # numpy: the first minimum = the smallest id
    second = np.partition(d, 1, axis=1)[:, 1] if d.shape[1] > 1 else np.full(len(Q), np.inf)
    clear = second - best > 2 * tol
    assert (gid[clear] == first[clear]).all()
    return int((~clear).sum())


@pytest.mark.parametrize("D,K,nq", [(96, 4096, 3000), (128, 1000, 700), (20, 300, 1), (100, 2500, 129), (64, 64, 50),
                                    (96, 1000, 300), (96, 50, 40), (96, 20000, 500), (128, 128, 128)])
def test_shortlist_assignment_is_the_exact_nearest(D, K, nq):
    """Widths that take the swept kernel (96, 128, 100 -> 128) and the tile kernel (20, 64); whole and partial
    last centroid tiles, fewer centroids than a tile, more tiles than one workgroup sweeps, one row."""
    print("case: shortlist", D, K, nq, flush=True)
    rng = np.random.default_rng(7 * D + K + nq)
    # clustered points around the centroids, rows of very different magnitude, a point that is a centroid
    C = rng.standard_normal((K, D)) * np.exp2(rng.integers(-12, 1, size=(K, 1)))
    own = rng.integers(0, K, size=nq)
    Q = C[own] + 0.3 * rng.standard_normal((nq, D)) * np.linalg.norm(C[own], axis=1, keepdims=True) / np.sqrt(D)
    Q[0] = C[K // 2]
    C, Q = C.astype(np.float32), Q.astype(np.float32)
    before = ivf.ivf_assign_stats()
    gid, gd = _assign(C, Q)
    after = ivf.ivf_assign_stats()
    assert after[0] == before[0] + 1 and after[1] == before[1]      # decided by the shortlist, no fallback
    _check(C, Q, gid, gd)
    assert gid[0] == K // 2 and gd[0] <= 16 * U * 2 * float((Q[0].astype(np.float64) ** 2).sum())


def test_shortlist_with_many_near_ties_and_duplicates():
    """Unit vectors in few dimensions: thousands of centroids at almost the same distance from every
    query, a quarter of them exact duplicates.  Still the exact nearest, the smallest id among duplicates."""
    print("case: shortlist near-ties", flush=True)
    rng = np.random.default_rng(11)
    D, K, nq = 8, 4096, 600
    C = rng.standard_normal((K, D))
    C /= np.linalg.norm(C, axis=1, keepdims=True)
    C[K // 4 * 3:] = C[:K // 4]                                      # duplicates with larger ids
    Q = rng.standard_normal((nq, D))
    Q /= np.linalg.norm(Q, axis=1, keepdims=True)
    C, Q = C.astype(np.float32), Q.astype(np.float32)
    gid, gd = _assign(C, Q)
    _check(C, Q, gid, gd)
    assert (gid < K // 4 * 3).all()                                  # never the larger id of a duplicate pair


def test_list_overflow_falls_back_to_the_one_pass_kernel():
    """Every centroid the same vector: every pair is a candidate, the list overflows, the exact kernel decides
    and returns id 0 for every row."""
    print("case: shortlist overflow", flush=True)
    rng = np.random.default_rng(12)
    D, K, nq = 32, 2048, 4096
    C = np.tile(rng.standard_normal((1, D)), (K, 1)).astype(np.float32)
    Q = rng.standard_normal((nq, D)).astype(np.float32)
    before = ivf.ivf_assign_stats()
    gid, gd = _assign(C, Q)
    after = ivf.ivf_assign_stats()
    assert after[1] == before[1] + 1 and after[0] == before[0]      # the fallback ran
    assert (gid == 0).all()
    d = _exact(C, Q)[:, 0]
    assert (np.abs(gd - d) <= 16 * U * ((Q.astype(np.float64) ** 2).sum(1) + float((C[0].astype(np.float64) ** 2).sum()))).all()


def test_shortlist_and_one_pass_kernel_agree(small):
    """The two ways of deciding a chunk on a real workload: the same region for every point that has a
    clear nearest centroid, and both within rounding of the fp64 minimum everywhere."""
    spec, ix, Q, X = small
    print("case: shortlist vs one-pass on the small workload", flush=True)
    C = ix.centroids
    P = X[:20000]
    a_id, a_d = _assign(C, P)
    os.environ["IVF_GP_EXACT_ASSIGN"] = "1"
    try:
        b_id, b_d = _assign(C, P)
    finally:
        del os.environ["IVF_GP_EXACT_ASSIGN"]
    unclear = _check(C, P, a_id, a_d)
    _check(C, P, b_id, b_d)
    assert (a_id != b_id).sum() <= unclear
