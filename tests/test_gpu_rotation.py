"""Indexes with a global rotation in front of the product quantiser (Section 4, OPQ-compressed
displacements) against the oracle (needs an MI355X)."""
import dataclasses

import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

import paper_1802_02422_amd as ivf
from oracle import ivf_oracle as orc
import parity
from test_oracle_query import random_rotation, rotated_tiny


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def test_rotate_rows_matches_oracle(rng):
    print("case: ivf_rotate", flush=True)
    for n, D in ((1, 4), (37, 96), (1000, 128), (19, 260)):
        X = rng.standard_normal((n, D)).astype(np.float32)
        R = rng.standard_normal((D, D)).astype(np.float32)            # any matrix: checks the operand order
        got = ivf.ivf_rotate(dev(X), dev(R)).cpu().numpy()
        ref = orc.rotate(X.astype(np.float64), R)
        scale = np.abs(R).astype(np.float64) @ np.abs(X).astype(np.float64).T
        assert (np.abs(got - ref) <= D * 2.0 ** -24 * scale.T + 1e-30).all()      # a chain of D fused multiply-adds in fp32
    eye = np.eye(96, dtype=np.float32)
    X = rng.standard_normal((50, 96)).astype(np.float32)
    assert (ivf.ivf_rotate(dev(X), dev(eye)).cpu().numpy() == X).all()


def test_search_and_encode_with_rotation(tiny, rng):
    spec, ix, Q, X = tiny
    ixr, R = rotated_tiny(tiny, rng)
    print("case: rotated tiny", flush=True)
    handle = ivf.ivf_load_index(parity.to_device(ixr))
    out = parity.run_gpu_search(handle, Q, spec.nprobe, spec.prune_frac, spec.k)
    rep = parity.check_search(ixr, Q, spec.nprobe, spec.prune_frac, spec.k, out)
    print(rep, flush=True)
    rep.assert_ok()
    # without the rotation the same codes would be read wrongly: the results must differ
    plain = ivf.ivf_load_index(parity.to_device(dataclasses.replace(ixr, rotation=None)))
    out2 = parity.run_gpu_search(plain, Q, spec.nprobe, spec.prune_frac, spec.k)
    assert (out2["ids"] != out["ids"]).mean() > 0.2
    # the static-scratch entry point takes the same path
    Qd = dev(Q[:9])
    ids = torch.empty((9, spec.k), dtype=torch.int32, device="cuda")
    d = torch.empty((9, spec.k), dtype=torch.float32, device="cuda")
    ivf.ivf_search_noalloc(handle, Qd, spec.nprobe, spec.prune_frac, spec.k, ids, d)
    torch.cuda.synchronize()
    assert (ids.cpu().numpy() == out["ids"][:9]).all() and (d.cpu().numpy() == out["dists"][:9]).all()
    # the encoder
    n = 4000
    desc = parity.to_device(ixr, with_codes=False)
    region, sub, codes, byte, t = ivf.ivf_encode(desc, dev(X[:n]), want_t=True)
    region, sub, codes, byte, t = (v.cpu().numpy() for v in (region, sub, codes, byte, t))
    enc = orc.encode(X[:n], ixr.centroids, ixr.nbr, ixr.alpha, ixr.pq_codebook, ixr.const_table, rotation=R)
    same = (region == enc.region) & (sub == enc.sub)
    assert same.mean() >= 0.995
    full = same & (codes == enc.codes).all(1)
    print("  codes identical:", full.mean(), flush=True)
    assert full.mean() >= 0.99
    np.testing.assert_allclose(t[full], enc.t[full], rtol=1e-4, atol=3e-6)
    assert (byte[full] == enc.const_byte[full]).mean() >= 0.99
    # the residual output stays the plain displacement x - mu
    _, _, _, _, _, res = ivf.ivf_encode(desc, dev(X[:200]), want_residual=True)
    np.testing.assert_allclose(res.cpu().numpy(), (X[:200].astype(np.float64) - enc.mu[:200]), rtol=0, atol=1e-6)


def test_identity_rotation_is_bit_identical(tiny):
    spec, ix, Q, X = tiny
    print("case: identity rotation", flush=True)
    a = ivf.ivf_load_index(parity.to_device(ix))
    b = ivf.ivf_load_index(parity.to_device(dataclasses.replace(ix, rotation=np.eye(spec.D, dtype=np.float32))))
    oa = parity.run_gpu_search(a, Q, spec.nprobe, spec.prune_frac, spec.k)
    ob = parity.run_gpu_search(b, Q, spec.nprobe, spec.prune_frac, spec.k)
    for n in oa:
        assert (oa[n] == ob[n]).all(), n
