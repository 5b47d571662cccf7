"""Device-side construction of a trained + encoded index for the large synthetic workloads.

The heavy steps run in the library's kernels (``ivf_coarse_topk`` for
assignment and the neighbour table, ``ivf_alpha_stats`` for the alpha sums,
``ivf_encode`` for subregion / PQ code / constant byte).  torch is used for
plumbing around them: drawing the data, averaging points per cluster, the
small k-means of the PQ sub-codebooks and of the 256-level scalar table, and
sorting the encoded points into grouped order.  Nothing here is on the query
path; the product of this module is the flat ``IndexDesc`` that
``ivf_load_index`` consumes.

Two ways of obtaining the coarse codebook (Section 3.1 uses an approximate
nearest-centroid search both for k-means and for assigning the base set):
  "kmeans"   Lloyd iterations from a seeded sample, exact assignment by the
             fused nearest-centroid kernel; the base set is assigned exactly.
  "mixture"  for K equal to the number of mixture components: centroids are
             the per-component means of the training sample (one Lloyd update
             from the generating means) and a point's region is its
             component; the agreement of that assignment with the exact
             nearest centroid is measured on a sample and returned.
"""
from __future__ import annotations

import time
from typing import Callable, Optional

import torch

import synthdata as sd
from . import binding as B


def _kmeans_small(X: torch.Tensor, k: int, iters: int, init_idx: torch.Tensor) -> torch.Tensor:
    """Plain Lloyd on a small codebook (PQ sub-codebooks): nearest by (distance, index)."""
    cent = X[init_idx].clone()
    n = X.shape[0]
    step = max(1, (1 << 26) // max(k, 1))
    for _ in range(iters):
        lab = torch.empty(n, dtype=torch.int64, device=X.device)
        for s in range(0, n, step):
            lab[s:s + step] = torch.cdist(X[s:s + step], cent).argmin(dim=1)
        sums = torch.zeros_like(cent).index_add_(0, lab, X)
        cnt = torch.bincount(lab, minlength=k).to(X.dtype)
        cent = torch.where(cnt[:, None] > 0, sums / cnt.clamp(min=1)[:, None], cent)
    return cent


def _lloyd_1d(t: torch.Tensor, iters: int) -> torch.Tensor:
    """256-level scalar quantiser: quantile start, Lloyd iterations, ascending fp32 table."""
    s, _ = torch.sort(t.double())
    n = s.shape[0]
    pos = ((torch.arange(256, device=t.device, dtype=torch.float64) + 0.5) / 256.0 * n).long().clamp(max=n - 1)
    table = s[pos].float()
    for _ in range(iters):
        tb = table.double()
        mid = (tb[1:] + tb[:-1]) / 2
        idx = torch.bucketize(s, mid, right=False)
        sums = torch.zeros(256, dtype=torch.float64, device=t.device).index_add_(0, idx, s)
        cnt = torch.bincount(idx, minlength=256).double()
        lev = torch.where(cnt > 0, sums / cnt.clamp(min=1), tb)
        table = torch.sort(lev)[0].float()
    return table


def neighbour_table(centroids: torch.Tensor, L: int):
    """NN_L of every centroid among the others (Eq. (2)), ordered by (distance, id)."""
    K = centroids.shape[0]
    ids, d = B.ivf_coarse_topk(centroids, centroids, L + 1)
    torch.cuda.synchronize()
    me = torch.arange(K, device=centroids.device, dtype=torch.int32)[:, None]
    is_self = ids == me
    # drop the centroid itself; if it is not in its own list (exact duplicates), drop the farthest
    none = ~is_self.any(dim=1)
    far = d.argmax(dim=1)
    is_self[none, far[none]] = True
    d = d.masked_fill(is_self, float("inf"))
    # order every row by (distance, id) with ONE flat stable radix sort: key = row << 32 | bits(distance)
    # (non-negative floats order like their bit patterns; ids already ascend inside a row)
    rows = torch.arange(K, device=centroids.device, dtype=torch.int64)[:, None]
    key = (rows << 32) | d.contiguous().view(torch.int32).to(torch.int64)
    order = torch.sort(key.view(-1), stable=True)[1].view(K, L + 1)[:, :L]
    del key
    nbr = ids.view(-1)[order].contiguous()
    cs = d.view(-1)[order].contiguous()
    return nbr, cs


def build(spec: sd.WorkloadSpec, mix: sd.Mixture, mode: str = "kmeans", chunk: int = 10_000_000,
          n_pq_train: int = 1_000_000, kmeans_iters: int = 10, pq_iters: int = 20, const_iters: int = 20,
          log: Optional[Callable[[str], None]] = None):
    """Returns (IndexDesc of flat device tensors, stats dict)."""
    dev = mix.means.device
    say = log or (lambda s: None)
    stats = {}
    t0 = time.time()
    K, L, M, D = spec.K, spec.L, spec.M, spec.D
    Xt, lab_t = sd.draw_points(mix, spec.n_train, 0, "train")

    if mode == "mixture":
        assert K == spec.n_mix, "mixture mode needs one region per mixture component"
        sums = torch.zeros(K, D, device=dev).index_add_(0, lab_t, Xt)
        cnt = torch.bincount(lab_t, minlength=K).float()
        cent = torch.where(cnt[:, None] > 0, sums / cnt.clamp(min=1)[:, None], mix.means)
        reg_t = lab_t.int()
        del sums
    elif mode == "kmeans":
        init = sd.draw_indices(spec.n_train, K, "kmeans-init", dev)
        cent = Xt[init].clone()
        for it in range(kmeans_iters):
            reg, _ = B.ivf_coarse_topk(cent, Xt, 1)
            lab = reg.view(-1).long()
            sums = torch.zeros(K, D, device=dev).index_add_(0, lab, Xt)
            cnt = torch.bincount(lab, minlength=K).float()
            cent = torch.where(cnt[:, None] > 0, sums / cnt.clamp(min=1)[:, None], cent)
        reg_t = B.ivf_coarse_topk(cent, Xt, 1)[0].view(-1).contiguous()
    else:
        raise ValueError(mode)
    cent = cent.contiguous()
    torch.cuda.synchronize()
    say(f"centroids ({mode}) {time.time() - t0:.1f}s")

    nbr, cs = neighbour_table(cent, L)
    say(f"neighbour table {time.time() - t0:.1f}s")

    num = torch.zeros(K, dtype=torch.float64, device=dev)
    den = torch.zeros(K, dtype=torch.float64, device=dev)
    B.ivf_alpha_stats(cent, nbr, Xt, reg_t, num, den)
    torch.cuda.synchronize()
    pooled = (num.sum() / den.sum()).clamp(0, 1) if den.sum() > 0 else torch.zeros((), dtype=torch.float64, device=dev)
    alpha = torch.where(den > 0, num / den.clamp(min=1e-300), pooled).clamp(0, 1).float().contiguous()
    say(f"alpha (mean {alpha.mean().item():.4f}) {time.time() - t0:.1f}s")

    # PQ codebooks on the displacements of a training subsample, then the scalar table
    n_pq = min(n_pq_train, spec.n_train)
    desc = B.IndexDesc(cent, nbr, alpha, cs, None, M)
    _, _, _, _, _, res = B.ivf_encode(desc, Xt[:n_pq], region_in=reg_t[:n_pq].contiguous(), want_residual=True)
    init_pq = sd.draw_indices(n_pq, 256, "pq-init", dev)
    ds = D // M
    cb = torch.stack([_kmeans_small(res[:, m * ds:(m + 1) * ds].contiguous(), 256, pq_iters, init_pq)
                      for m in range(M)]).contiguous()
    desc.pq_codebook = cb
    _, _, _, _, t = B.ivf_encode(desc, Xt[:n_pq], region_in=reg_t[:n_pq].contiguous(), want_t=True)
    desc.const_table = _lloyd_1d(t, const_iters).contiguous()
    del Xt, res, t
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
            ns = min(100_000, n)
            pick = sd.draw_indices(n, ns, "assign-check", dev)
            exact = B.ivf_coarse_topk(cent, X[pick].contiguous(), 1)[0].view(-1)
            stats["label_vs_exact_assignment"] = (exact == r[pick]).float().mean().item()
        bucket[done:done + n] = r * L + s_
        codes[done:done + n] = cd
        byte[done:done + n] = by
        done += n
        c += 1
        del X, lab, r, s_, cd, by
    torch.cuda.synchronize()
    say(f"encoded {N} points {time.time() - t0:.1f}s")

    # grouped order: by (region, subregion), then id
    _, perm = torch.sort(bucket, stable=True)
    sizes = torch.bincount(bucket, minlength=K * L)
    off = torch.zeros(K * L + 1, dtype=torch.int64, device=dev)
    off[1:] = torch.cumsum(sizes, 0)
    del bucket, sizes
    desc.sub_offsets = off.to(torch.int32).contiguous()     # N < 2^31: same bits as uint32
    desc.codes = codes[perm].contiguous()
    del codes
    desc.const_byte = byte[perm].contiguous()
    del byte
    desc.ids = perm.to(torch.int32).contiguous()
    del perm
    torch.cuda.synchronize()
    stats["build_seconds"] = time.time() - t0
    say(f"grouped {time.time() - t0:.1f}s")
    return desc, stats
