"""The device-side index builder: its product must be a valid grouped index that the
oracle, given the same arrays, searches to the same results."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

import synthdata as sd
import paper_1802_02422_amd as ivf
from paper_1802_02422_amd import index_builder
from oracle import ivf_oracle as orc
import parity
from bench import download_index


@pytest.mark.parametrize("mode", ["kmeans", "mixture"])
def test_builder_product_is_searchable_and_matches_oracle(mode):
    print("case: builder", mode, flush=True)
    spec = sd.WORKLOADS["tiny"]
    dev = torch.device("cuda:0")
    mix = sd.make_mixture(spec.kind, spec.n_mix, spec.D, dev)
    desc, stats = index_builder.build(spec, mix, mode=mode, chunk=30_000, n_pq_train=20_000, kmeans_iters=4,
                                      pq_iters=5)
    ix = download_index(desc, spec)
    off = ix.sub_offsets.astype(np.int64)
    assert off[0] == 0 and off[-1] == spec.N and (np.diff(off) >= 0).all()
    assert sorted(ix.ids.tolist()) == list(range(spec.N))
    assert (np.diff(ix.const_table) >= 0).all() and ((ix.alpha >= 0) & (ix.alpha <= 1)).all()
    # neighbour table against the oracle's definition (Eq. (2)); cs_dist2 against direct distances
    nbr_o, cs_o = orc.neighbours(ix.centroids, spec.L)
    agree = (nbr_o == ix.nbr).mean()
    assert agree >= 0.999, agree
    np.testing.assert_allclose(ix.cs_dist2[nbr_o == ix.nbr], cs_o[nbr_o == ix.nbr], rtol=1e-4, atol=1e-6)
    # stored points sit in the subregion the oracle's encoder chooses (sample; near-ties aside)
    X = torch.cat([sd.draw_points(mix, min(30_000, spec.N - c * 30_000), c, "base",
                                  sorted_labels=(mode == "mixture"))[0] for c in range((spec.N + 29_999) // 30_000)])
    X = X.cpu().numpy()
    pos = np.random.default_rng(1).integers(0, spec.N, 3000)
    region_given = None
    if mode == "mixture":
        bucket = np.repeat(np.arange(spec.K * spec.L), np.diff(off))
        region_given = (bucket[pos] // spec.L).astype(np.int32)
    enc = orc.encode(X[ix.ids[pos]], ix.centroids, ix.nbr, ix.alpha, ix.pq_codebook, ix.const_table,
                     region=region_given)
    b = enc.region.astype(np.int64) * spec.L + enc.sub
    inside = (off[b] <= pos) & (pos < off[b + 1])
    assert inside.mean() >= 0.995, inside.mean()
    same = inside & (ix.codes[pos] == enc.codes).all(1)
    assert same.mean() >= 0.99
    if mode == "mixture":
        assert stats["label_vs_exact_assignment"] >= 0.99
    # search parity on the GPU-built index
    Q = sd.draw_queries(mix, spec.nq).cpu().numpy()
    handle = ivf.ivf_load_index(desc)
    out = parity.run_gpu_search(handle, Q, spec.nprobe, spec.prune_frac, spec.k)
    rep = parity.check_search(ix, Q, spec.nprobe, spec.prune_frac, spec.k, out)
    print(rep)
    rep.assert_ok()


def test_builder_with_a_rotation_matches_oracle():
    """The builder with a seeded random rotation in front of the PQ: its product searches to the
    oracle's results, and the codes are the oracle's encoder's with that rotation."""
    print("case: builder with rotation", flush=True)
    spec = sd.WORKLOADS["tiny"]
    dev = torch.device("cuda:0")
    mix = sd.make_mixture(spec.kind, spec.n_mix, spec.D, dev)
    R = sd.random_rotation(spec.D, device=dev)
    assert torch.allclose(R @ R.T, torch.eye(spec.D, device=dev), atol=1e-5)
    desc, stats = index_builder.build(spec, mix, mode="kmeans", chunk=30_000, n_pq_train=20_000, kmeans_iters=4,
                                      pq_iters=5, rotation=R)
    ix = download_index(desc, spec)
    assert ix.rotation is not None
    Q = sd.draw_queries(mix, spec.nq).cpu().numpy()
    handle = ivf.ivf_load_index(desc)
    out = parity.run_gpu_search(handle, Q, spec.nprobe, spec.prune_frac, spec.k)
    rep = parity.check_search(ix, Q, spec.nprobe, spec.prune_frac, spec.k, out)
    print(rep)
    rep.assert_ok()
    X = torch.cat([sd.draw_points(mix, min(30_000, spec.N - c * 30_000), c, "base")[0]
                   for c in range((spec.N + 29_999) // 30_000)]).cpu().numpy()
    pos = np.random.default_rng(2).integers(0, spec.N, 2000)
    enc = orc.encode(X[ix.ids[pos]], ix.centroids, ix.nbr, ix.alpha, ix.pq_codebook, ix.const_table, rotation=ix.rotation)
    off = ix.sub_offsets.astype(np.int64)
    b = enc.region.astype(np.int64) * spec.L + enc.sub
    inside = (off[b] <= pos) & (pos < off[b + 1])
    same = inside & (ix.codes[pos] == enc.codes).all(1)
    assert inside.mean() >= 0.995 and same.mean() >= 0.99
