"""Shared fixtures: seeded workloads and oracle-built indices.

Markers: ``gpu`` = needs an MI355X (parity of the HIP library against the
oracle through the C ABI); everything else runs on the CPU.
"""
import os
import sys

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X GPU")


def make_workload(name, scale_nq=None):
    """Generate the named workload on the CPU and build its index with the oracle.

    Returns (spec, index, queries, base vectors).  Results are cached in
    ``tests/_cache`` keyed by the workload name (the generators are seeded, so
    the cache only saves time).
    """
    import torch
    import synthdata as sd
    from oracle import ivf_oracle as orc

    spec = sd.WORKLOADS[name]
    cache = os.path.join(ROOT, "tests", "_cache", f"{name}_v1.npz")
    mix = sd.make_mixture(spec.kind, spec.n_mix, spec.D)
    Q = sd.draw_queries(mix, spec.nq).numpy()
    X, _ = sd.draw_points(mix, spec.N, 0, "base")
    X = X.numpy()
    fields = ["centroids", "nbr", "alpha", "cs_dist2", "pq_codebook", "const_table", "sub_offsets",
              "codes", "const_byte", "ids"]
    if os.path.exists(cache):
        z = np.load(cache)
        ix = orc.Index(spec.D, spec.M, spec.L, spec.K, spec.N, *[z[f] for f in fields])
    else:
        Xt, _ = sd.draw_points(mix, spec.n_train, 0, "train")
        Xt = Xt.numpy()
        ci = sd.draw_indices(spec.n_train, spec.K, "kmeans-init").numpy()
        pi = sd.draw_indices(spec.n_train, 256, "pq-init").numpy()
        ix = orc.build_index(Xt, X, spec.K, spec.L, spec.M, ci, pi)
        os.makedirs(os.path.dirname(cache), exist_ok=True)
        np.savez(cache, **{f: getattr(ix, f) for f in fields})
    return spec, ix, Q, X


@pytest.fixture(scope="session")
def tiny():
    return make_workload("tiny")


@pytest.fixture
def rng():
    return np.random.default_rng(20180207)


@pytest.fixture(scope="session")
def small():
    return make_workload("small")


@pytest.fixture(scope="session")
def small_sift():
    return make_workload("small_sift")
