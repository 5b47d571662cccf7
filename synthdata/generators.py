"""Seeded generators for the synthetic retrieval workloads.

Every array is a pure function of (MASTER_SEED, stream name, chunk number,
device type): the same call on the same device type returns the same bytes.
Draws on "cpu" and on "cuda" use different random streams, so a workload is
always generated once and the *same tensors* are handed to both the oracle
and the HIP path.

Recipes
-------
deep-like   mixture of ``n_mix`` Gaussians in D dims.  Component j has a mean
            m_j (uniform random unit vector) and a D-vector of standard
            deviations sigma_j ~ U(0.02, 0.1) per dimension.  A point picks a
            component uniformly at random and is
            normalise(m_j + sigma_j * N(0, I)).
sift-like   m_j ~ Gamma(shape 0.5, scale 20) per dimension, sigma_j ~ U(2, 10)
            per dimension, a point is
            uint8(clip(round(m_j + sigma_j * N(0, I)), 0, 255)) cast to fp32.
Queries come from the same mixture through a separate stream.
"""
from __future__ import annotations

import hashlib
from dataclasses import dataclass

import torch

MASTER_SEED = 180202422


def stream_seed(name: str, chunk: int = 0) -> int:
    """63-bit seed for the named stream and chunk."""
    h = hashlib.sha256(f"{MASTER_SEED}/{name}/{chunk}".encode()).digest()
    return int.from_bytes(h[:8], "little") & ((1 << 63) - 1)


def _gen(name: str, chunk: int, device) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(stream_seed(name, chunk))
    return g


@dataclass(frozen=True)
class WorkloadSpec:
    name: str
    kind: str        # "deep" or "sift"
    N: int           # database size
    D: int           # dimensionality
    n_mix: int       # mixture components
    K: int           # coarse centroids (regions)
    L: int           # neighbour subregions per region
    M: int           # PQ bytes per vector
    nq: int          # queries
    nprobe: int      # regions visited per query
    prune_frac: float  # fraction of the nprobe*L subregions kept
    k: int           # results per query
    n_train: int     # size of the training sample


WORKLOADS = {
    # the five configurations of the benchmark definition, in order
    "tiny": WorkloadSpec("tiny", "deep", 100_000, 96, 1024, 1024, 8, 8, 100, 16, 0.5, 10, 50_000),
    "deep10m": WorkloadSpec("deep10m", "deep", 10_000_000, 96, 65_536, 65_536, 64, 16, 10_000, 64, 0.25, 100, 2_000_000),
    "sift10m": WorkloadSpec("sift10m", "sift", 10_000_000, 128, 65_536, 65_536, 64, 16, 10_000, 64, 0.25, 100, 2_000_000),
    "deep100m": WorkloadSpec("deep100m", "deep", 100_000_000, 96, 1 << 20, 1 << 20, 64, 8, 64, 128, 0.2, 10, 20_000_000),
    "deep1b": WorkloadSpec("deep1b", "deep", 1_000_000_000, 96, 1 << 20, 1 << 20, 64, 16, 10_000, 256, 0.2, 100, 20_000_000),
    # an intermediate size the CPU oracle can still train and encode in about
    # a minute, spanning many kernel tiles with ragged tails
    "small": WorkloadSpec("small", "deep", 300_000, 96, 2048, 2000, 24, 16, 333, 40, 0.3, 100, 60_000),
    "small_sift": WorkloadSpec("small_sift", "sift", 200_000, 128, 1024, 1000, 16, 16, 150, 24, 0.25, 50, 50_000),
}


@dataclass
class Mixture:
    kind: str
    means: torch.Tensor   # [n_mix, D] fp32
    sigmas: torch.Tensor  # [n_mix, D] fp32


def make_mixture(kind: str, n_mix: int, D: int, device="cpu", name: str = "mixture") -> Mixture:
    dev = torch.device(device)
    g = _gen(f"{name}/{kind}/{n_mix}/{D}", 0, dev)
    if kind == "deep":
        m = torch.randn(n_mix, D, generator=g, device=dev, dtype=torch.float32)
        m /= m.norm(dim=1, keepdim=True)
        s = torch.rand(n_mix, D, generator=g, device=dev, dtype=torch.float32) * 0.08 + 0.02
    elif kind == "sift":
        # Gamma(shape 1/2, scale 20) is 10 * chi-square(1) = 10 * z^2
        z = torch.randn(n_mix, D, generator=g, device=dev, dtype=torch.float32)
        m = 10.0 * z * z
        s = torch.rand(n_mix, D, generator=g, device=dev, dtype=torch.float32) * 8.0 + 2.0
    else:
        raise ValueError(f"unknown mixture kind {kind!r}")
    return Mixture(kind, m, s)


def _draw(mix: Mixture, n: int, g: torch.Generator, sorted_labels: bool):
    dev = mix.means.device
    n_mix, D = mix.means.shape
    labels = torch.randint(0, n_mix, (n,), generator=g, device=dev, dtype=torch.int64)
    if sorted_labels:
        labels, _ = torch.sort(labels)
    x = torch.randn(n, D, generator=g, device=dev, dtype=torch.float32)
    x.mul_(mix.sigmas[labels]).add_(mix.means[labels])
    if mix.kind == "deep":
        x /= x.norm(dim=1, keepdim=True)
    else:
        x = x.round_().clamp_(0.0, 255.0).to(torch.uint8).to(torch.float32)
    return x, labels


def draw_points(mix: Mixture, n: int, chunk: int = 0, stream: str = "base", sorted_labels: bool = False):
    """n points of chunk ``chunk`` of the named stream: (x [n, D] fp32, component labels [n] int64).

    With ``sorted_labels`` the labels of the chunk are drawn first and sorted, so
    that points of one component are adjacent; the multiset of the chunk is
    distributed exactly as without sorting.
    """
    g = _gen(f"{stream}/{mix.kind}/{mix.means.shape[0]}", chunk, mix.means.device)
    return _draw(mix, n, g, sorted_labels)


def draw_queries(mix: Mixture, nq: int, stream: str = "query"):
    """nq query vectors [nq, D] fp32 from the same mixture, separate stream."""
    x, _ = draw_points(mix, nq, 0, stream)
    return x


def draw_indices(n_from: int, n: int, stream: str, device="cpu") -> torch.Tensor:
    """n distinct indices out of range(n_from), int64 (initial centroids, codewords)."""
    dev = torch.device(device)
    g = _gen(f"{stream}/{n_from}", 0, dev)
    return torch.randperm(n_from, generator=g, device=dev)[:n].contiguous()


def random_rotation(D: int, stream: str = "rotation", device="cpu") -> torch.Tensor:
    """A seeded random orthogonal D x D matrix (Q of the QR factorisation of a Gaussian matrix,
    columns signed so that R's diagonal is positive), fp32."""
    dev = torch.device(device)
    g = _gen(f"{stream}/{D}", 0, "cpu")
    a = torch.randn(D, D, generator=g, dtype=torch.float64)
    q, r = torch.linalg.qr(a)
    q = q * torch.sign(torch.diagonal(r))[None, :]
    return q.to(torch.float32).contiguous().to(dev)
