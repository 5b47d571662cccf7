#!/usr/bin/env python3
"""Nearest-centroid assignment (the index-time use of stage 1, P = 1): the certified shortlist against the
one-pass full-precision kernel, on synthetic data of a workload's shape.

    python assign_bench.py --workload deep1b --rows 1048576

Prints one JSON line per timed call (two rounds per mode) and a last line that compares the assignments.
The centroids are the generating means where the workload has one component per region, else one Lloyd
round from sampled points.  The one-pass kernel is selected with IVF_GP_EXACT_ASSIGN=1, which the library
reads at every call.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", default="deep1b")
    ap.add_argument("--rows", type=int, default=1 << 20)
    args = ap.parse_args()
    import torch
    import synthdata as sd
    import paper_1802_02422_amd as ivf
    spec = sd.WORKLOADS[args.workload]
    dev = torch.device("cuda:0")
    mix = sd.make_mixture(spec.kind, spec.n_mix, spec.D, dev)
    X, _ = sd.draw_points(mix, args.rows, 0, "train")
    if spec.n_mix == spec.K:
        C = mix.means.contiguous()
    else:
        C = ivf.ivf_kmeans(X, spec.K, 1, sd.draw_indices(args.rows, spec.K, "kmeans-init", dev))
    out = {}
    for mode in ("shortlist", "one-pass", "shortlist", "one-pass"):
        if mode == "one-pass":
            os.environ["IVF_GP_EXACT_ASSIGN"] = "1"
        else:
            os.environ.pop("IVF_GP_EXACT_ASSIGN", None)
        s0 = ivf.ivf_assign_stats()
        torch.cuda.synchronize()
        t = time.time()
        out[mode] = ivf.ivf_coarse_topk(C, X, 1)
        torch.cuda.synchronize()
        dt = time.time() - t
        s1 = ivf.ivf_assign_stats()
        print(json.dumps({"mode": mode, "K": spec.K, "D": spec.D, "rows": args.rows, "seconds": round(dt, 4),
                          "useful_tflops": round(2.0 * args.rows * spec.K * spec.D / dt / 1e12, 1),
                          "chunks_by_shortlist": s1[0] - s0[0], "chunks_by_one_pass": s1[1] - s0[1]}), flush=True)
    a, b = out["shortlist"], out["one-pass"]
    print(json.dumps({"assignments_that_differ": int((a[0] != b[0]).sum()), "rows": args.rows,
                      "max_abs_distance_difference": float((a[1] - b[1]).abs().max())}), flush=True)


if __name__ == "__main__":
    main()
