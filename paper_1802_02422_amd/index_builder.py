"""Device-side construction of a trained + encoded index for the large synthetic workloads.

Every step of the construction runs in the library's kernels, called through the C ABI:
``ivf_kmeans`` (region codebook), ``ivf_neighbours`` (Eq. (2)), ``ivf_learn_alpha`` (Eqs. (8)-(12)),
``ivf_encode`` (region, subregion by Eq. (3), displacement by Eq. (4), PQ code, constant byte),
``ivf_pq_train`` (PQ codebooks), ``ivf_lloyd_1d`` (the 256-level table), ``ivf_group`` and
``ivf_gather_rows`` (grouped order).  This module only draws the synthetic data chunk by chunk,
allocates the device buffers and passes them on; nothing here is on the query path.  Its product
is the flat ``IndexDesc`` that ``ivf_load_index`` consumes.

Two ways of obtaining the coarse codebook (Section 3.1 uses an approximate nearest-centroid search
both for k-means and for assigning the base set):
  "kmeans"   Lloyd iterations from a seeded sample, exact assignment by the fused nearest-centroid
             kernel; the base set is assigned exactly.
  "mixture"  for K equal to the number of mixture components: the codebook is one Lloyd update of
             the generating means on the training sample with the component labels as the
             assignment, and a base point's region is its component; the agreement of that
             assignment with the exact nearest centroid is measured on a sample and returned.
"""
from __future__ import annotations

import time
from typing import Callable, Optional

import torch

import synthdata as sd
from . import binding as B


def neighbour_table(centroids: torch.Tensor, L: int):
    """NN_L of every centroid among the others (Eq. (2)), ordered by (distance, id)."""
    return B.ivf_neighbours(centroids, L)


def build(spec: sd.WorkloadSpec, mix: sd.Mixture, mode: str = "kmeans", chunk: int = 10_000_000,
          n_pq_train: int = 1_000_000, kmeans_iters: int = 10, pq_iters: int = 20, const_iters: int = 20,
          log: Optional[Callable[[str], None]] = None, centroids: Optional[torch.Tensor] = None,
          alpha_override: Optional[float] = None, rotation: Optional[torch.Tensor] = None):
    """Returns (IndexDesc of flat device tensors, stats dict).

    ``centroids`` reuses a region codebook trained earlier (the ablation over L builds several
    indexes on one codebook); ``alpha_override`` forces one scaling factor for every region
    (0 gives the variant without grouping); ``rotation`` ([D, D], orthogonal) is put in front of
    the product quantiser (Section 4: OPQ-compressed displacements; learning the rotation itself is
    not part of this build, any orthogonal matrix may be given)."""
    dev = mix.means.device
    say = log or (lambda s: None)
    stats = {}
    t0 = time.time()
    K, L, M, D = spec.K, spec.L, spec.M, spec.D
    Xt, lab_t = sd.draw_points(mix, spec.n_train, 0, "train")

    if mode == "mixture":
        assert K == spec.n_mix, "mixture mode needs one region per mixture component"
        reg_t = lab_t.int().contiguous()
        if centroids is None:
            # one Lloyd update with the component labels as the assignment: the members of every
            # component listed by ivf_group, averaged by the k-means update kernel (zero rounds of
            # assignment: ivf_kmeans is not used here because the assignment is given)
            cent = B.ivf_cluster_means(Xt, reg_t, mix.means.contiguous())
        else:
            cent = centroids
    elif mode == "kmeans":
        if centroids is None:
            init = sd.draw_indices(spec.n_train, K, "kmeans-init", dev)
            cent = B.ivf_kmeans(Xt, K, kmeans_iters, init)
        else:
            cent = centroids
        reg_t = B.ivf_coarse_topk(cent, Xt, 1)[0].view(-1).contiguous()
    else:
        raise ValueError(mode)
    cent = cent.contiguous()
    torch.cuda.synchronize()
    say(f"centroids ({mode}) {time.time() - t0:.1f}s")

    nbr, cs = neighbour_table(cent, L)
    say(f"neighbour table {time.time() - t0:.1f}s")

    if alpha_override is None:
        alpha = B.ivf_learn_alpha(cent, nbr, Xt, reg_t)
    else:
        alpha = torch.full((K,), float(alpha_override), dtype=torch.float32, device=dev)
    say(f"alpha (mean {alpha.mean().item():.4f}) {time.time() - t0:.1f}s")

    # PQ codebooks on the displacements of a training subsample, then the scalar table
    n_pq = min(n_pq_train, spec.n_train)
    desc = B.IndexDesc(cent, nbr, alpha, cs, None, M, rotation=rotation)
    Xp, rp = Xt[:n_pq].contiguous(), reg_t[:n_pq].contiguous()
    _, _, _, _, _, res = B.ivf_encode(desc, Xp, region_in=rp, want_residual=True)
    init_pq = sd.draw_indices(n_pq, 256, "pq-init", dev)
    if rotation is not None:
        res = B.ivf_rotate(res, rotation)
    desc.pq_codebook = B.ivf_pq_train(res, M, pq_iters, init_pq)
    _, _, _, _, t = B.ivf_encode(desc, Xp, region_in=rp, want_t=True)
    desc.const_table = B.ivf_lloyd_1d(t, const_iters)
    del Xt, Xp, res, t
    say(f"pq codebooks + constant table {time.time() - t0:.1f}s")

    # encode the base set chunk by chunk; raw vectors are discarded
    N = spec.N
    codes = torch.empty((N, M), dtype=torch.uint8, device=dev)
    byte = torch.empty(N, dtype=torch.uint8, device=dev)
    bucket = torch.empty(N, dtype=torch.int32, device=dev)
    done, c = 0, 0
    while done < N:
        n = min(chunk, N - done)
        X, lab = sd.draw_points(mix, n, c, "base", sorted_labels=(mode == "mixture"))
        rin = lab.int().contiguous() if mode == "mixture" else None
        r, s_, cd, by, _ = B.ivf_encode(desc, X, region_in=rin)
        if c == 0 and mode == "mixture":
            ns = min(1_000_000, n)
            pick = sd.draw_indices(n, ns, "assign-check", dev)
            exact = B.ivf_coarse_topk(cent, X[pick].contiguous(), 1)[0].view(-1)
            stats["label_vs_exact_assignment"] = (exact == r[pick]).float().mean().item()
        B.ivf_bucket_ids(r, s_, L, bucket[done:done + n])
        codes[done:done + n] = cd
        byte[done:done + n] = by
        done += n
        c += 1
        del X, lab, r, s_, cd, by
    torch.cuda.synchronize()
    say(f"encoded {N} points {time.time() - t0:.1f}s")

    # grouped order: by (region, subregion), then id
    perm, off = B.ivf_group(bucket, K * L)
    del bucket
    desc.sub_offsets = off
    desc.codes = B.ivf_gather_rows(codes, perm)
    del codes
    desc.const_byte = B.ivf_gather_rows(byte, perm)
    del byte
    desc.ids = perm
    torch.cuda.synchronize()
    stats["build_seconds"] = time.time() - t0
    say(f"grouped {time.time() - t0:.1f}s")
    return desc, stats
