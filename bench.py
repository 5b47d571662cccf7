#!/usr/bin/env python3
"""Throughput of the batched query path on one MI355X.

A "step" is one pass of the whole path (coarse distances + top-nprobe, subcentroid
scoring, pruning, lookup tables, ADC scan, k-select) over the workload's full
query batch, with queries and index resident in HBM when the timed region
starts.  Prints one JSON line with queries/s, the roofline of the dominant
kernel (the ADC scan, timed with HIP events on its own stream inside the
library) and the CPU oracle timed on the host cores on a bounded sample of the
same queries.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
DESC_BYTES = 16          # one kept-subregion descriptor read by the scan

# HBM bytes per launch from rocprofv3 hardware counters (FETCH_SIZE and WRITE_SIZE in KiB per dispatch, each
# scaled by what the same counter reads for the library's plain 1 GiB copy kernel: 2.0 and 1.0).  These are
# readings of separate counter runs of this same command (two `rocprofv3 --pmc` passes cannot run inside a
# timed benchmark); the profile summary each comes from is named beside it and holds the full commands.
# None where no counter run has been made for the workload.
MEASURED_TRAFFIC = {
    ("scan_kernel", "deep1b"): ((5_050_370 * 2.0 + 31_683 * 1.0) * 1024, "profiles/scan_kernel_deep1b.md"),
    ("coarse_gemm_sweep_kernel", "deep1b"): ((3_475_044 * 2.0 + 42_069_101 * 1.0) * 1024, "profiles/coarse_gemm_deep1b.md"),
}


def measured_traffic(kernel, workload):
    return MEASURED_TRAFFIC.get((kernel, workload), (None, None))


def log(msg):
    print(f"[bench] {msg}", file=sys.stderr, flush=True)


def download_index(desc, spec):
    """Flat device index -> the oracle's Index of numpy arrays (host)."""
    import numpy as np
    from oracle import ivf_oracle as orc
    h = lambda t: t.cpu().numpy()
    return orc.Index(spec.D, spec.M, spec.L, spec.K, spec.N, h(desc.centroids), h(desc.nbr), h(desc.alpha),
                     h(desc.cs_dist2), h(desc.pq_codebook), h(desc.const_table),
                     h(desc.sub_offsets).view(np.uint32), h(desc.codes), h(desc.const_byte), h(desc.ids),
                     None if desc.rotation is None else h(desc.rotation))


def _omp_threads(n):
    """Team size of the process's OpenMP runtime (the oracle's loops take the runtime's default)."""
    import ctypes
    try:
        ctypes.CDLL("libgomp.so.1").omp_set_num_threads(int(n))
        return True
    except (OSError, AttributeError):
        return False


def cpu_baseline(ix, Q, spec, budget_s=20.0):
    """The oracle's whole-path search on the host cores, on as many of the same queries as fit the budget."""
    import numpy as np
    from oracle import ivf_oracle as orc
    cores = len(os.sched_getaffinity(0))
    omp = int(os.environ.get("OMP_NUM_THREADS", cores))
    cores = min(cores, omp)
    tau = float(np.float32(spec.prune_frac))
    n0 = min(Q.shape[0], max(2, cores))
    t = time.time()
    orc.search(ix, Q[:n0], spec.nprobe, tau, spec.k)
    per_q = (time.time() - t) / n0
    n = int(min(Q.shape[0], max(n0, budget_s / max(per_q, 1e-9))))
    t = time.time()
    _, _, ns = orc.search(ix, Q[:n], spec.nprobe, tau, spec.k)
    dt = time.time() - t
    out = {"value": n / dt, "unit": "queries/s", "cores": cores, "kind": "oracle",
           "sample": f"first {n} of {Q.shape[0]} queries of the same workload, full index, {dt:.1f} s wall",
           "codes_per_s": float(ns.sum()) / dt}
    # the same on one thread (the kind of figure the paper's timings are), on a few seconds' worth of queries
    if cores > 1 and _omp_threads(1):
        n1 = int(min(n, max(2, 4.0 / max(dt / n * cores, 1e-9))))
        t = time.time()
        orc.search(ix, Q[:n1], spec.nprobe, tau, spec.k)
        d1 = time.time() - t
        _omp_threads(omp)
        out["single_thread"] = {"value": n1 / d1, "unit": "queries/s", "cores": 1,
                                "sample": f"first {n1} queries, {d1:.1f} s wall"}
    return out


def check_sample(ix, Q, spec, ids, dists, n_check=64):
    """The results that were just timed, on a sample of the queries, against the oracle's whole-path search:
    counts for the JSON line (selections differ only where the oracle's own fp64 values nearly tie)."""
    import numpy as np
    from oracle import ivf_oracle as orc
    sample = np.unique(np.linspace(0, Q.shape[0] - 1, min(n_check, Q.shape[0])).astype(np.int64))
    tau = float(np.float32(spec.prune_frac))
    oi, od, _ = orc.search(ix, Q[sample], spec.nprobe, tau, spec.k)
    gi, gd = ids[sample], dists[sample]
    rows_same = int((gi == oi).all(1).sum())
    # slots holding the same id: compare the distances there
    same = (gi == oi) & (oi >= 0)
    rel = np.abs(gd[same].astype(np.float64) - od[same]) / np.maximum(np.abs(od[same]), 1e-30)
    # ids returned by one side only, per query
    only = sum(len(set(a.tolist()) ^ set(b.tolist())) // 2 for a, b in zip(gi, oi))
    return {"queries_checked": int(len(sample)), "rows_identical": rows_same,
            "slots_identical": int(same.sum()), "slots_total": int((oi >= 0).sum()),
            "ids_in_one_result_only": int(only),
            "max_rel_dist_err_on_identical_slots": float(rel.max()) if rel.size else 0.0}


def measure(args, workload, nq=0, with_oracle=True, with_cpu_baseline=True, calibrate=False):
    """Builds the workload's index on the device, times `args.steps` passes and returns the result object."""
    import torch
    import synthdata as sd
    import paper_1802_02422_amd as ivf
    from paper_1802_02422_amd import index_builder

    assert torch.cuda.is_available(), "bench.py needs the GPU"
    dev = torch.device("cuda:0")
    spec = sd.WORKLOADS[workload]
    if nq:
        import dataclasses
        spec = dataclasses.replace(spec, nq=min(nq, spec.nq))
    ivf.load_library()

    t0 = time.time()
    mix = sd.make_mixture(spec.kind, spec.n_mix, spec.D, dev)
    mode = "mixture" if spec.K >= (1 << 18) else "kmeans"
    desc, stats = index_builder.build(spec, mix, mode=mode, log=log)
    Q = sd.draw_queries(mix, spec.nq).contiguous()
    log(f"index built in {time.time() - t0:.1f}s ({mode}); stats {stats}")

    host_ix = None
    if with_oracle:
        host_ix = download_index(desc, spec)
        log(f"index downloaded to host {time.time() - t0:.1f}s")
    handle = ivf.ivf_load_index(desc)
    desc.codes = desc.const_byte = desc.ids = None      # the handle owns its own copy
    torch.cuda.empty_cache()
    ivf.ivf_set_scratch_limit(handle, int(args.scratch_gib * (1 << 30)))
    log(f"index loaded {time.time() - t0:.1f}s")

    out_ids = torch.empty((spec.nq, spec.k), dtype=torch.int32, device=dev)
    out_d = torch.empty((spec.nq, spec.k), dtype=torch.float32, device=dev)
    st = ivf.ivf_search_stages(handle, Q, spec.nprobe, spec.prune_frac, spec.k)
    torch.cuda.synchronize()
    codes_scanned = int(st["n_scanned"].sum().item())
    S = ivf.ivf_num_kept(spec.nprobe, spec.L, spec.prune_frac)
    del st

    for _ in range(args.warmup):
        ivf.ivf_search(handle, Q, spec.nprobe, spec.prune_frac, spec.k, out_ids, out_d)
    torch.cuda.synchronize()
    # the headline time: exactly `steps` passes, nothing but the library's launches in the timed region
    t1 = time.perf_counter()
    for _ in range(args.steps):
        ivf.ivf_search(handle, Q, spec.nprobe, spec.prune_frac, spec.k, out_ids, out_d)
    torch.cuda.synchronize()
    t2 = time.perf_counter()
    # the per-stage and per-kernel times: the same `steps` passes again with HIP events recorded on the stream
    # around every stage inside the library (the events cost a few microseconds per stage, which matters only
    # for the latency workloads)
    ivf.ivf_profile_enable(handle, True)
    ivf.ivf_profile_read(handle)
    for _ in range(args.steps):
        ivf.ivf_search(handle, Q, spec.nprobe, spec.prune_frac, spec.k, out_ids, out_d)
    torch.cuda.synchronize()
    stage_ms, passes = ivf.ivf_profile_read(handle)
    ivf.ivf_profile_enable(handle, False)

    ms_per_step = (t2 - t1) * 1e3 / args.steps
    qps = spec.nq / (ms_per_step * 1e-3)
    scan_launches = passes                      # one scan launch per pass over a tile of queries
    scan_ms = stage_ms["scan"] / max(scan_launches, 1)
    algo_bytes = (codes_scanned * (spec.M + 1) + spec.nq * S * DESC_BYTES) * args.steps / max(scan_launches, 1)
    achieved = algo_bytes / (scan_ms * 1e-3) / 1e9 if scan_ms > 0 else 0.0
    coarse_tflops = 2.0 * spec.nq * spec.K * spec.D * args.steps / (stage_ms["coarse_gemm"] * 1e-3) / 1e12
    # stage 1 must write the distance matrix (reused by the scoring stage) and the block minima, and read the
    # packed centroid table (4 bytes per component, hi + lo fp16) and the queries once
    nb = (spec.K + 63) // 64
    gemm_ms = stage_ms["coarse_gemm"] / max(passes, 1)
    gemm_bytes = spec.nq * args.steps / max(passes, 1) * (spec.K + nb + spec.D) * 4 + spec.K * spec.D * 4   # per launch
    gemm_kernel = ("coarse_gemm_skinny_kernel" if spec.nq <= 64 else
                   "coarse_gemm_sweep_kernel" if spec.K % 128 == 0 and -(-spec.D // 32) * 2 in (6, 8) else "coarse_gemm_kernel")
    gemm_achieved = gemm_bytes / (gemm_ms * 1e-3) / 1e9 if gemm_ms > 0 else 0.0

    copy_gbs = None
    if calibrate:
        a = torch.empty(1 << 28, dtype=torch.float32, device=dev).normal_()
        b = torch.empty_like(a)
        ivf.ivf_copy_bytes(b, a)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(3):
            ivf.ivf_copy_bytes(b, a)
        e1.record()
        torch.cuda.synchronize()
        copy_gbs = 3 * 2 * a.numel() * 4 / (e0.elapsed_time(e1) * 1e-3) / 1e9     # read + write
        log(f"copy kernel: {copy_gbs:.0f} GB/s (read+write) on 1 GiB")
        del a, b

    result = {
        "metric": "queries/s at fixed nprobe/prune budget; ADC codes scanned/s (HBM GB/s)",
        "value": qps, "unit": "queries/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": spec.name, "N": spec.N, "D": spec.D, "K": spec.K, "L": spec.L, "M": spec.M,
                   "nq": spec.nq, "nprobe": spec.nprobe, "prune_frac": spec.prune_frac, "k": spec.k,
                   "kept_subregions": S, "codes_scanned_per_query": codes_scanned / spec.nq,
                   "index_build": mode, **{k_: v for k_, v in stats.items()}},
        "codes_scanned_per_s": codes_scanned * args.steps / (stage_ms["scan"] * 1e-3) if stage_ms["scan"] > 0 else 0.0,
        "stage_ms_per_step": {k_: v / args.steps for k_, v in stage_ms.items()},
        "coarse_gemm_tflops": coarse_tflops,     # useful 2*nq*K*D flop; each is three fp16 matrix-core products
        "arithmetic": "fp32 results throughout; stage-1 inner products as fp16 hi/lo split operands (22 bits) "
                      "accumulated in fp32 on the matrix cores, same accuracy as fp32",
        "roofline": {"kernel": "scan_kernel", "bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
                     "traffic": measured_traffic("scan_kernel", spec.name)[0],
                     "traffic_source": measured_traffic("scan_kernel", spec.name)[1],
                     "launches": scan_launches, "avg_launch_ms": scan_ms, "algorithmic_bytes_per_launch": algo_bytes,
                     # the same with 12 instead of this library's 16 bytes counted per descriptor
                     "frac_at_12B_per_descriptor": (algo_bytes - 4 * spec.nq * S * args.steps / max(scan_launches, 1))
                                                   / (scan_ms * 1e-3) / 1e9 / HBM_PEAK_GBS if scan_ms > 0 else 0.0},
        # the longest stage, bound by its stores; timed by events around packing + GEMM (packing: a few us)
        "roofline_coarse_gemm": {"kernel": gemm_kernel, "bound": "hbm", "achieved": gemm_achieved,
                                 "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": gemm_achieved / HBM_PEAK_GBS,
                                 "traffic": measured_traffic(gemm_kernel, spec.name)[0],
                                 "traffic_source": measured_traffic(gemm_kernel, spec.name)[1],
                                 "launches": passes, "avg_launch_ms": gemm_ms,
                                 "algorithmic_bytes_per_launch": gemm_bytes},
    }
    if copy_gbs is not None:
        result["copy_kernel_gbs_read_plus_write"] = copy_gbs
    if host_ix is not None:
        Qh = Q.cpu().numpy()
        result["checked_against_oracle"] = check_sample(host_ix, Qh, spec, out_ids.cpu().numpy(), out_d.cpu().numpy())
        log(f"sample check: {result['checked_against_oracle']}")
        if with_cpu_baseline:
            result["cpu_baseline"] = cpu_baseline(host_ix, Qh, spec)
    ivf.ivf_free_index(handle)
    del handle, desc
    torch.cuda.empty_cache()
    return result


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default=os.environ.get("IVF_BENCH_WORKLOAD", "deep1b"))
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--scratch-gib", type=float, default=48.0)
    ap.add_argument("--nq", type=int, default=0, help="use only the first NQ queries of the workload (latency runs)")
    ap.add_argument("--all", action="store_true",
                    help="after the headline workload also measure the other workloads of the benchmark definition "
                         "(reported inside the same JSON line as other_workloads)")
    ap.add_argument("--calibrate", action="store_true",
                    help="also run the plain 1 GiB copy kernel (reference for rocprofv3 HBM counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no sharding or collectives); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    result = measure(args, args.workload, args.nq, with_oracle=not args.no_cpu_baseline,
                     with_cpu_baseline=not args.no_cpu_baseline, calibrate=args.calibrate)
    if args.all:
        # the other workloads of the benchmark definition, each with its stage split and the scan's roofline
        # fraction (no CPU baseline; the sample check against the oracle stays on)
        others = []
        for name, nq in (("deep10m", 0), ("sift10m", 0), ("deep100m", 1), ("deep100m", 64), ("tiny", 0)):
            if name == args.workload and nq == args.nq:
                continue
            r = measure(args, name, nq, with_oracle=not args.no_cpu_baseline, with_cpu_baseline=False)
            others.append({k_: r[k_] for k_ in ("value", "unit", "ms_per_step", "config", "codes_scanned_per_s",
                                                "stage_ms_per_step", "roofline", "checked_against_oracle") if k_ in r})
        result["other_workloads"] = others
    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
