#!/usr/bin/env python3
"""Recall-versus-time tables of the candidate-budget search on the synthetic workloads.

Synthetic analogue of the paper's ablations (Section 4: candidate lists of length R; Table 3-left:
L in {32, 64, 128} at R = 30 000; the variant without grouping, alpha = 0; the variant without
pruning, tau = 1).  For every index variant and every R the script runs ``ivf_search_budget`` over
the workload's whole query batch and reports
  list   Recall@R of the candidate list itself: the share of queries whose true nearest neighbour
         lies in a visited subregion (no reranking), as in the paper's indexing-quality experiment
  R@1 / R@10 / R@100   the share of queries whose true nearest neighbour is among the first
         1 / 10 / 100 results after ranking the candidates by the compressed-domain distance
  us/query   wall time of the whole path per query (batch time / batch size, HIP events)
against the exact nearest neighbour of every query, computed here in fp64 from the regenerated
base vectors.  Needs the GPU; prints one markdown table per workload and writes the rows as JSON.
"""
import argparse
import dataclasses
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)


def exact_nn(mix, spec, Q, mode, chunk=10_000_000, tile=1 << 18):
    """Index (generation order = id) of the exact nearest base vector of every query, in fp64."""
    import torch
    import synthdata as sd
    nq = Q.shape[0]
    best_d = torch.full((nq,), float("inf"), dtype=torch.float64, device=Q.device)
    best_i = torch.zeros(nq, dtype=torch.int64, device=Q.device)
    Q64 = Q.double()
    qn = (Q64 * Q64).sum(1)
    done, c = 0, 0
    while done < spec.N:
        n = min(chunk, spec.N - done)
        X, _ = sd.draw_points(mix, n, c, "base", sorted_labels=(mode == "mixture"))
        for s in range(0, n, tile):
            xb = X[s:s + tile].double()
            d = qn[:, None] + (xb * xb).sum(1)[None, :] - 2.0 * (Q64 @ xb.T)
            dm, im = d.min(dim=1)
            upd = dm < best_d
            best_d = torch.where(upd, dm, best_d)
            best_i = torch.where(upd, im + done + s, best_i)
        done += n
        c += 1
        del X
    return best_i


def evaluate(handle, desc, spec, Q, nn, nprobe, tau, R, k, reps):
    import torch
    import paper_1802_02422_amd as ivf
    out = ivf.ivf_search_budget(handle, Q, nprobe, tau, R, k)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        ivf.ivf_search_budget(handle, Q, nprobe, tau, R, k)
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / reps
    ids = out["ids"].long()
    hit = ids == nn[:, None]
    # candidate list: is the true neighbour's subregion among the visited ones?
    pos = desc["pos_of_id"][nn].long()
    bucket = torch.searchsorted(desc["off"], pos, right=True) - 1
    in_list = ((out["kept_sub"] == bucket[:, None]) & (out["visited"] == 1)).any(1)
    return {"R": R, "candidates_mean": out["n_scanned"].double().mean().item(),
            "list": in_list.double().mean().item(),
            "R@1": hit[:, :1].any(1).double().mean().item(),
            "R@10": hit[:, :10].any(1).double().mean().item(),
            "R@100": hit[:, :100].any(1).double().mean().item(),
            "us_per_query": ms * 1e3 / Q.shape[0]}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", default="deep10m")
    ap.add_argument("--Ls", default="32,64,128")
    ap.add_argument("--Rs", default="1000,3000,10000,30000,100000")
    ap.add_argument("--nprobe", type=int, default=256)
    ap.add_argument("--reps", type=int, default=3)
    ap.add_argument("--out", default=None)
    args = ap.parse_args()

    import torch
    import synthdata as sd
    import paper_1802_02422_amd as ivf
    from paper_1802_02422_amd import index_builder

    dev = torch.device("cuda:0")
    base = sd.WORKLOADS[args.workload]
    mix = sd.make_mixture(base.kind, base.n_mix, base.D, dev)
    mode = "mixture" if base.K >= (1 << 18) else "kmeans"
    Q = sd.draw_queries(mix, base.nq).contiguous()
    t0 = time.time()
    nn = exact_nn(mix, base, Q, mode)
    print(f"[ablation] exact nearest neighbours of {base.nq} queries in {time.time() - t0:.1f}s", file=sys.stderr, flush=True)
    Ls = [int(v) for v in args.Ls.split(",")]
    Rs = [int(v) for v in args.Rs.split(",")]
    k = 100
    rows, cent = [], None
    variants = [(L, None, 0.5, f"grouping + pruning, L={L}, tau=0.5") for L in Ls]
    Lref = Ls[len(Ls) // 2]
    variants.append((Lref, None, 1.0, f"grouping, no pruning, L={Lref}, tau=1"))
    variants.append((Lref, 0.0, 1.0, "no grouping (alpha=0), tau=1"))
    built = {}
    for L, a_over, tau, name in variants:
        key = (L, a_over)
        if key not in built:
            spec = dataclasses.replace(base, L=L)
            desc, stats = index_builder.build(spec, mix, mode=mode, centroids=cent, alpha_override=a_over)
            cent = desc.centroids
            aux = {"off": desc.sub_offsets.long(),
                   "pos_of_id": torch.empty(spec.N, dtype=torch.int32, device=dev)}
            aux["pos_of_id"][desc.ids.long()] = torch.arange(spec.N, dtype=torch.int32, device=dev)
            handle = ivf.ivf_load_index(desc)
            desc.codes = desc.const_byte = desc.ids = None
            built = {key: (handle, aux, spec)}            # keep one index resident at a time
            torch.cuda.empty_cache()
        handle, aux, spec = built[key]
        nprobe = min(args.nprobe, spec.K, ivf_max_probe(L))
        for R in Rs:
            r = evaluate(handle, aux, spec, Q, nn, nprobe, tau, R, k, args.reps)
            r.update({"workload": base.name, "variant": name, "L": L, "tau": tau, "nprobe": nprobe})
            rows.append(r)
            print(json.dumps(r), flush=True)
    print(f"\n### {base.name}: N={base.N}, D={base.D}, K={base.K}, M={base.M}, {base.nq} queries, k={k}\n")
    print("| variant | nprobe | R | candidates | list | R@1 | R@10 | R@100 | us/query |")
    print("|---|---|---|---|---|---|---|---|---|")
    for r in rows:
        print(f"| {r['variant']} | {r['nprobe']} | {r['R']} | {r['candidates_mean']:.0f} | {r['list']:.3f} | "
              f"{r['R@1']:.3f} | {r['R@10']:.3f} | {r['R@100']:.3f} | {r['us_per_query']:.2f} |")
    if args.out:
        with open(args.out, "w") as f:
            json.dump(rows, f, indent=1)


def ivf_max_probe(L):
    """Largest nprobe whose nprobe * L scores one workgroup holds (the library's limit)."""
    return min(32768 // L, 39424 // (L + 3))


if __name__ == "__main__":
    main()
