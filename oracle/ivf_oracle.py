"""ctypes loader and numpy-level driver of the CPU oracle (``ivf_oracle.c``).

TEST INFRASTRUCTURE: only tests, the smoke check and the benchmark's CPU
baseline leg may import this.  The product (the HIP library and its binding)
never does, and nothing here imports the product.

Everything of substance is in the C file; this module marshals numpy arrays,
strings the index-construction steps together in the order the paper gives
them (Section 3.2) and lays the encoded points out in grouped order.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from dataclasses import dataclass
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "ivf_oracle.c")
_LIB = os.path.join(_HERE, "libivf_oracle.so")


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (-O2, OpenMP over independent items)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-o", _LIB, _SRC, "-lm"])
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        _lib.orc_num_kept.restype = C.c_int64
        _lib.orc_num_kept.argtypes = [C.c_double, C.c_int64, C.c_int]
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _f32(a):
    return np.ascontiguousarray(a, dtype=np.float32)


def _i32(a):
    return np.ascontiguousarray(a, dtype=np.int32)


def _i64(a):
    return np.ascontiguousarray(a, dtype=np.int64)


def _f64(a):
    return np.ascontiguousarray(a, dtype=np.float64)


def _u8(a):
    return np.ascontiguousarray(a, dtype=np.uint8)


I64 = C.c_int64
INT = C.c_int

# ----------------------------------------------------------------- stages ---


def coarse_dist(Q, Cn):
    Q, Cn = _f32(Q), _f32(Cn)
    nq, D = Q.shape
    K = Cn.shape[0]
    out = np.empty((nq, K), np.float64)
    lib().orc_coarse_dist(_p(Q), I64(nq), _p(Cn), I64(K), INT(D), _p(out))
    return out


def smallest(v, nsel, tie=None):
    v = _f64(v)
    n = v.shape[0]
    nsel = min(nsel, n)
    pos = np.empty(nsel, np.int64)
    val = np.empty(nsel, np.float64)
    t = None if tie is None else _i64(tie)
    lib().orc_smallest(_p(v), _p(t), I64(n), I64(nsel), _p(pos), _p(val))
    return pos, val


def probe(Q, Cn, P):
    Q, Cn = _f32(Q), _f32(Cn)
    nq, D = Q.shape
    K = Cn.shape[0]
    pid = np.empty((nq, P), np.int32)
    pd = np.empty((nq, P), np.float64)
    lib().orc_probe(_p(Q), I64(nq), _p(Cn), I64(K), INT(D), I64(P), _p(pid), _p(pd))
    return pid, pd


def scores(Q, ix, probe_id):
    Q = _f32(Q)
    probe_id = _i32(probe_id)
    nq, D = Q.shape
    P = probe_id.shape[1]
    out = np.empty((nq, P, ix.L), np.float64)
    lib().orc_scores(_p(Q), I64(nq), _p(ix.centroids), INT(D), _p(ix.nbr), INT(ix.L), _p(ix.alpha),
                     _p(ix.cs_dist2), _p(probe_id), I64(P), _p(out))
    return out


def num_kept(prune_frac, P, L):
    return int(lib().orc_num_kept(C.c_double(prune_frac), I64(P), INT(L)))


def prune(sc, probe_id, prune_frac):
    sc = _f64(sc)
    probe_id = _i32(probe_id)
    nq, P, L = sc.shape
    S = num_kept(prune_frac, P, L)
    kept = np.empty((nq, S), np.int64)
    ks = np.empty((nq, S), np.float64)
    lib().orc_prune(_p(sc), I64(nq), I64(P), INT(L), _p(probe_id), I64(S), _p(kept), _p(ks))
    return kept, ks


def rotate(X, R):
    """Rows of X (fp64) multiplied by the D x D matrix R: out[i] = R x[i]."""
    X, R = _f64(X), _f32(R)
    n, D = X.shape
    out = np.empty((n, D), np.float64)
    lib().orc_rotate(_p(X), I64(n), INT(D), _p(R), _p(out))
    return out


def lut(Q, ix):
    Q = _f32(Q)
    nq, D = Q.shape
    T = np.empty((nq, ix.M, 256), np.float64)
    rot = None if ix.rotation is None else _f32(ix.rotation)
    lib().orc_lut(_p(Q), I64(nq), INT(D), INT(ix.M), _p(ix.pq_codebook), _p(rot), _p(T))
    return T


def budget_visit(ix, kept_sub, kept_score, R):
    """Candidate budget: flags [nq, S] of the kept subregions that are visited before R points are collected."""
    kept_sub, kept_score = _i64(kept_sub), _f64(kept_score)
    nq, S = kept_sub.shape
    visit = np.empty((nq, S), np.uint8)
    lib().orc_budget_visit(_p(kept_sub), _p(kept_score), I64(nq), I64(S), _p(ix.sub_offsets), I64(R), _p(visit))
    return visit


def scan(ix, kept_sub, kept_score, T, const_exact=None, visit=None):
    """Candidates of every query: (start offsets [nq+1], positions, distances)."""
    kept_sub, kept_score, T = _i64(kept_sub), _f64(kept_score), _f64(T)
    nq, S = kept_sub.shape
    cnt = np.empty(nq, np.int64)
    vis = None if visit is None else _u8(visit)
    lib().orc_scan_count(_p(kept_sub), _p(vis), I64(nq), I64(S), _p(ix.sub_offsets), _p(cnt))
    start = np.zeros(nq + 1, np.int64)
    np.cumsum(cnt, out=start[1:])
    tot = int(start[-1])
    pos = np.empty(max(tot, 1), np.int64)
    dist = np.empty(max(tot, 1), np.float64)
    ce = None if const_exact is None else _f64(const_exact)
    lib().orc_scan(_p(kept_sub), _p(kept_score), _p(vis), I64(nq), I64(S), _p(ix.sub_offsets), _p(ix.codes),
                   INT(ix.M), _p(ix.const_byte), _p(ix.const_table), _p(ce), _p(T), _p(start),
                   _p(pos), _p(dist))
    return start, pos[:tot], dist[:tot]


def select(ix, cand_pos, cand_dist, k):
    cand_pos, cand_dist = _i64(cand_pos), _f64(cand_dist)
    oi = np.empty(k, np.int32)
    od = np.empty(k, np.float64)
    lib().orc_select(_p(cand_pos), _p(cand_dist), I64(cand_pos.shape[0]), _p(ix.ids), I64(k), _p(oi), _p(od))
    return oi, od


class _CIndex(C.Structure):
    _fields_ = [("D", C.c_int32), ("M", C.c_int32), ("L", C.c_int32), ("K", C.c_int64), ("N", C.c_int64),
                ("centroids", C.c_void_p), ("nbr", C.c_void_p), ("alpha", C.c_void_p),
                ("cs_dist2", C.c_void_p), ("pq_codebook", C.c_void_p), ("const_table", C.c_void_p),
                ("sub_offsets", C.c_void_p), ("codes", C.c_void_p), ("const_byte", C.c_void_p),
                ("ids", C.c_void_p), ("rotation", C.c_void_p)]


def search(ix, Q, nprobe, prune_frac, k):
    """Whole query path: (ids [nq,k] int32, dists [nq,k] fp64, codes scanned [nq])."""
    Q = _f32(Q)
    nq = Q.shape[0]
    rot = None if ix.rotation is None else _f32(ix.rotation)     # kept alive until the call returns
    ci = _CIndex(ix.D, ix.M, ix.L, ix.K, ix.N, *[a.ctypes.data for a in (
        ix.centroids, ix.nbr, ix.alpha, ix.cs_dist2, ix.pq_codebook, ix.const_table, ix.sub_offsets,
        ix.codes, ix.const_byte, ix.ids)], None if rot is None else rot.ctypes.data)
    oi = np.empty((nq, k), np.int32)
    od = np.empty((nq, k), np.float64)
    ns = np.empty(nq, np.int64)
    lib().orc_search(C.byref(ci), _p(Q), I64(nq), I64(nprobe), C.c_double(prune_frac), I64(k),
                     _p(oi), _p(od), _p(ns))
    return oi, od, ns


def search_budget(ix, Q, nprobe, prune_frac, R, k):
    """Whole query path with a candidate budget R: (ids, dists, codes scanned [nq], staged intermediates)."""
    st = search_staged(ix, Q, nprobe, prune_frac, k, budget=R)
    return st["ids"], st["dists"], np.diff(st["cand_start"]), st


def search_staged(ix, Q, nprobe, prune_frac, k, probe_id=None, kept=None, budget=None, visit=None):
    """Stages 1-6 one after another, returning every intermediate.

    ``probe_id`` ([nq, P]) or ``kept`` ([nq, S] subregion ids) replace the
    oracle's own selection of that stage (used to carry on after a reported
    near-tie); all values are still recomputed here in fp64.  ``budget`` = R
    switches the candidate budget on (``out["visit"]`` are the flags of the
    subregions in ``out["scan_sub"]``); ``visit`` replaces the oracle's flags.
    """
    Q = _f32(Q)
    out = {}
    pid, pd = probe(Q, ix.centroids, nprobe)
    out["probe_id"], out["probe_d"] = pid, pd
    if probe_id is not None:
        pid = _i32(probe_id)
    sc = scores(Q, ix, pid)
    out["scores"] = sc
    ksub, kscore = prune(sc, pid, prune_frac)
    out["kept_sub"], out["kept_score"] = ksub, kscore
    if kept is not None:
        ksub = _i64(kept)
        # look the injected subregions' scores up among the scored ones
        L = ix.L
        kscore = np.empty(ksub.shape, np.float64)
        for q in range(Q.shape[0]):
            sid = (pid[q].astype(np.int64)[:, None] * L + np.arange(L)[None, :]).ravel()
            order = np.argsort(sid)
            where = order[np.searchsorted(sid[order], ksub[q])]
            kscore[q] = sc[q].ravel()[where]
    T = lut(Q, ix)
    out["lut"] = T
    out["scan_sub"], out["scan_score"] = ksub, kscore
    vis = None
    if budget is not None:
        vis = budget_visit(ix, ksub, kscore, budget)
        out["visit"] = vis
        if visit is not None:
            vis = _u8(visit)
    start, cpos, cdist = scan(ix, ksub, kscore, T, visit=vis)
    out["cand_start"], out["cand_pos"], out["cand_dist"] = start, cpos, cdist
    oi = np.empty((Q.shape[0], k), np.int32)
    od = np.empty((Q.shape[0], k), np.float64)
    for q in range(Q.shape[0]):
        oi[q], od[q] = select(ix, cpos[start[q]:start[q + 1]], cdist[start[q]:start[q + 1]], k)
    out["ids"], out["dists"] = oi, od
    return out


# ------------------------------------------------------ index construction ---


def assign(X, Cn):
    X, Cn = _f32(X), _f32(Cn)
    n, D = X.shape
    reg = np.empty(n, np.int32)
    d = np.empty(n, np.float64)
    lib().orc_assign(_p(X), I64(n), _p(Cn), I64(Cn.shape[0]), INT(D), _p(reg), _p(d))
    return reg, d


def kmeans(X, k, iters, init_idx):
    X = _f32(X)
    n, d = X.shape
    init_idx = _i64(init_idx)
    assert init_idx.shape[0] == k
    cent = np.empty((k, d), np.float32)
    obj = np.empty(iters, np.float64)
    lib().orc_kmeans(_p(X), I64(n), INT(d), I64(k), INT(iters), _p(init_idx), _p(cent), _p(obj))
    return cent, obj


def neighbours(Cn, L):
    Cn = _f32(Cn)
    K, D = Cn.shape
    nbr = np.empty((K, L), np.int32)
    cs = np.empty((K, L), np.float32)
    lib().orc_neighbours(_p(Cn), I64(K), INT(D), INT(L), _p(nbr), _p(cs))
    return nbr, cs


def learn_alpha(X, region, Cn, nbr):
    X, Cn, region, nbr = _f32(X), _f32(Cn), _i32(region), _i32(nbr)
    K, D = Cn.shape
    alpha = np.empty(K, np.float32)
    lib().orc_learn_alpha(_p(X), I64(X.shape[0]), _p(region), _p(Cn), I64(K), INT(D), _p(nbr),
                          INT(nbr.shape[1]), _p(alpha))
    return alpha


def sub_assign(X, region, Cn, nbr, alpha, want_mu=True, want_res=True):
    X, Cn, region, nbr, alpha = _f32(X), _f32(Cn), _i32(region), _i32(nbr), _f32(alpha)
    n, D = X.shape
    sub = np.empty(n, np.int32)
    mu = np.empty((n, D), np.float64) if want_mu else None
    res = np.empty((n, D), np.float64) if want_res else None
    lib().orc_sub_assign(_p(X), I64(n), _p(region), _p(Cn), INT(D), _p(nbr), INT(nbr.shape[1]),
                         _p(alpha), _p(sub), _p(mu), _p(res))
    return sub, mu, res


def pq_encode(E, codebook):
    E, codebook = _f64(E), _f32(codebook)
    n, D = E.shape
    M = codebook.shape[0]
    codes = np.empty((n, M), np.uint8)
    lib().orc_pq_encode(_p(E), I64(n), INT(D), INT(M), _p(codebook), _p(codes))
    return codes


def pq_decode(codes, codebook):
    codes, codebook = _u8(codes), _f32(codebook)
    n, M = codes.shape
    D = M * codebook.shape[2]
    out = np.empty((n, D), np.float64)
    lib().orc_pq_decode(_p(codes), I64(n), INT(D), INT(M), _p(codebook), _p(out))
    return out


def const_term(mu, codes, codebook):
    mu, codes, codebook = _f64(mu), _u8(codes), _f32(codebook)
    n, D = mu.shape
    t = np.empty(n, np.float64)
    lib().orc_const_term(_p(mu), _p(codes), I64(n), INT(D), INT(codes.shape[1]), _p(codebook), _p(t))
    return t


def lloyd_1d(t, iters=20):
    t = _f64(t)
    table = np.empty(256, np.float32)
    lib().orc_lloyd_1d(_p(t), I64(t.shape[0]), INT(iters), _p(table))
    return table


def quantize_1d(t, table):
    t, table = _f64(t), _f32(table)
    b = np.empty(t.shape[0], np.uint8)
    lib().orc_quantize_1d(_p(t), I64(t.shape[0]), _p(table), _p(b))
    return b


def pq_train(E, M, iters, init_idx):
    """One k-means (256 codewords) per block of D/M dims of the displacements."""
    E = np.asarray(E)
    n, D = E.shape
    ds = D // M
    cb = np.empty((M, 256, ds), np.float32)
    objs = []
    for m in range(M):
        cb[m], obj = kmeans(E[:, m * ds:(m + 1) * ds].astype(np.float32), 256, iters, init_idx)
        objs.append(obj)
    return cb, np.array(objs)


@dataclass
class Index:
    """The trained and encoded index: exactly the arrays the search consumes."""
    D: int
    M: int
    L: int
    K: int
    N: int
    centroids: np.ndarray    # [K, D] fp32
    nbr: np.ndarray          # [K, L] int32, neighbours of each centroid, self excluded
    alpha: np.ndarray        # [K] fp32
    cs_dist2: np.ndarray     # [K, L] fp32, ||c - s_l||^2
    pq_codebook: np.ndarray  # [M, 256, D/M] fp32
    const_table: np.ndarray  # [256] fp32 ascending
    sub_offsets: np.ndarray  # [K*L + 1] uint32, start of each subregion in grouped order
    codes: np.ndarray        # [N, M] uint8, grouped order
    const_byte: np.ndarray   # [N] uint8, grouped order
    ids: np.ndarray          # [N] int32, original id of each grouped position
    rotation: Optional[np.ndarray] = None   # [D, D] fp32 or None: rotation in front of the PQ


@dataclass
class Encoded:
    region: np.ndarray
    sub: np.ndarray
    codes: np.ndarray
    t: np.ndarray
    const_byte: np.ndarray
    mu: np.ndarray


def encode(X, Cn, nbr, alpha, codebook, const_table=None, region=None, rotation=None) -> Encoded:
    """Index-time encoding of points: region, subregion (Eq. 3), PQ code of the
    displacement (Eq. 4), per-point constant t and its byte.  With a rotation the
    PQ sees R (x - mu) and the constant is taken with R mu."""
    if region is None:
        region, _ = assign(X, Cn)
    sub, mu, res = sub_assign(X, region, Cn, nbr, alpha)
    if rotation is not None:
        codes = pq_encode(rotate(res, rotation), codebook)
        t = const_term(rotate(mu, rotation), codes, codebook)
    else:
        codes = pq_encode(res, codebook)
        t = const_term(mu, codes, codebook)
    byte = quantize_1d(t, const_table) if const_table is not None else None
    return Encoded(region, sub, codes, t, byte, mu)


def group(region, sub, L, K):
    """Grouped layout: points ordered by (region, subregion, id); returns the
    permutation (grouped position -> original index) and the K*L+1 offsets."""
    bucket = region.astype(np.int64) * L + sub.astype(np.int64)
    perm = np.lexsort((np.arange(bucket.shape[0]), bucket))
    sizes = np.bincount(bucket, minlength=K * L)
    off = np.zeros(K * L + 1, np.uint32)
    off[1:] = np.cumsum(sizes).astype(np.uint32)
    return perm, off


def build_index(X_train, X_base, K, L, M, init_centroids_idx, init_pq_idx, kmeans_iters=10, pq_iters=20,
                const_iters=20, ids=None, rotation=None) -> Index:
    """Train on the hold-out sample, then encode and group the base set
    (Section 3.2; all trainable parameters come from the learning set, Section 4)."""
    X_train, X_base = _f32(X_train), _f32(X_base)
    D = X_train.shape[1]
    cent, _ = kmeans(X_train, K, kmeans_iters, init_centroids_idx)
    nbr, cs = neighbours(cent, L)
    reg_t, _ = assign(X_train, cent)
    alpha = learn_alpha(X_train, reg_t, cent, nbr)
    _, mu_t, res_t = sub_assign(X_train, reg_t, cent, nbr, alpha)
    if rotation is not None:
        mu_t, res_t = rotate(mu_t, rotation), rotate(res_t, rotation)
    cb, _ = pq_train(res_t, M, pq_iters, init_pq_idx)
    codes_t = pq_encode(res_t, cb)
    t_t = const_term(mu_t, codes_t, cb)
    table = lloyd_1d(t_t, const_iters)
    enc = encode(X_base, cent, nbr, alpha, cb, table, rotation=rotation)
    perm, off = group(enc.region, enc.sub, L, K)
    N = X_base.shape[0]
    ids = np.arange(N, dtype=np.int32) if ids is None else _i32(ids)
    return Index(D, M, L, K, N, cent, nbr, alpha, cs, cb, table, off,
                 np.ascontiguousarray(enc.codes[perm]), np.ascontiguousarray(enc.const_byte[perm]),
                 np.ascontiguousarray(ids[perm]), None if rotation is None else _f32(rotation))
