"""ctypes binding with the same names as the C ABI (``include/ivf_gp.h``).

Tensors are torch CUDA(HIP) tensors used purely as device buffers: the binding
checks dtype / device / contiguity, passes ``data_ptr()`` and the current
stream handle, and allocates output tensors.  Every step of the method runs in
the library's kernels.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libivf_gp.so")
_lib = None


class IvfError(RuntimeError):
    pass


class _Desc(C.Structure):
    _fields_ = [("D", C.c_int32), ("M", C.c_int32), ("L", C.c_int32), ("K", C.c_int64), ("N", C.c_int64),
                ("centroids", C.c_void_p), ("nbr", C.c_void_p), ("alpha", C.c_void_p),
                ("cs_dist2", C.c_void_p), ("pq_codebook", C.c_void_p), ("const_table", C.c_void_p),
                ("sub_offsets", C.c_void_p), ("codes", C.c_void_p), ("const_byte", C.c_void_p),
                ("ids", C.c_void_p), ("rotation", C.c_void_p)]


def library_path() -> str:
    return _LIB_PATH


def load_library():
    """Load the built HIP library; raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise IvfError(f"{_LIB_PATH} is missing: build it first (python -m paper_1802_02422_amd.build); "
                       "there is no fallback path")
    lib = C.CDLL(_LIB_PATH)
    vp, i64, i32, f32 = C.c_void_p, C.c_int64, C.c_int, C.c_float
    lib.ivf_load_index.argtypes = [C.POINTER(_Desc), vp, C.POINTER(vp)]
    lib.ivf_free_index.argtypes = [vp]
    lib.ivf_free_index.restype = None
    lib.ivf_set_scratch_limit.argtypes = [vp, i64]
    lib.ivf_search.argtypes = [vp, vp, i64, i32, f32, i32, vp, vp, vp]
    lib.ivf_search_noalloc.argtypes = [vp, vp, i64, i32, f32, i32, vp, vp, vp]
    lib.ivf_search_budget.argtypes = [vp, vp, i64, i32, f32, i64, i32, vp, vp, vp, vp, vp, vp]
    lib.ivf_search_stages.argtypes = [vp, vp, i64, i32, f32, i32, vp, vp, vp, vp, vp, vp, vp]
    lib.ivf_num_kept.argtypes = [i32, i32, f32]
    lib.ivf_num_kept.restype = i64
    lib.ivf_coarse_topk.argtypes = [vp, i64, i32, vp, i64, i32, vp, vp, vp]
    lib.ivf_assign_stats.argtypes = [C.POINTER(C.c_int64)]
    lib.ivf_assign_stats.restype = None
    lib.ivf_encode.argtypes = [C.POINTER(_Desc), vp, i64, vp, vp, vp, vp, vp, vp, vp, vp]
    lib.ivf_rotate.argtypes = [vp, i64, i32, vp, vp, vp]
    lib.ivf_kmeans.argtypes = [vp, i64, i32, i64, i32, vp, vp, vp, vp]
    lib.ivf_cluster_means.argtypes = [vp, i64, i32, vp, i64, vp, vp]
    lib.ivf_bucket_ids.argtypes = [vp, vp, i64, i32, vp, vp]
    lib.ivf_neighbours.argtypes = [vp, i64, i32, i32, vp, vp, vp]
    lib.ivf_learn_alpha.argtypes = [vp, i64, i32, vp, i32, vp, i64, vp, vp, vp]
    lib.ivf_pq_train.argtypes = [vp, i64, i32, i32, i32, vp, vp, vp]
    lib.ivf_lloyd_1d.argtypes = [vp, i64, i32, vp, vp]
    lib.ivf_group.argtypes = [vp, i64, i64, vp, vp, vp]
    lib.ivf_gather_rows.argtypes = [vp, i64, vp, i64, vp, vp]
    lib.ivf_profile_enable.argtypes = [vp, i32]
    lib.ivf_profile_read.argtypes = [vp, C.POINTER(C.c_double), C.POINTER(i64)]
    lib.ivf_copy_bytes.argtypes = [vp, vp, i64, vp]
    lib.ivf_last_error.restype = C.c_char_p
    _lib = lib
    return lib


def ivf_last_error() -> str:
    return load_library().ivf_last_error().decode()


def _check(rc: int):
    if rc != 0:
        raise IvfError(f"ivf error {rc}: {ivf_last_error()}")


def _dev(t: Optional[torch.Tensor], dtype, name: str, shape=None):
    if t is None:
        return None
    if not isinstance(t, torch.Tensor) or not t.is_cuda:
        raise IvfError(f"{name} must be a device tensor")
    if t.dtype != dtype or not t.is_contiguous():
        raise IvfError(f"{name} must be contiguous {dtype}, got {t.dtype}")
    if shape is not None and tuple(t.shape) != tuple(shape):
        raise IvfError(f"{name} has shape {tuple(t.shape)}, expected {tuple(shape)}")
    return t


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


@dataclass
class IndexDesc:
    """Device tensors of the trained (+ optionally encoded) index, mirroring ``ivf_index_desc``."""
    centroids: torch.Tensor                      # [K, D] fp32
    nbr: torch.Tensor                            # [K, L] int32
    alpha: torch.Tensor                          # [K] fp32
    cs_dist2: torch.Tensor                       # [K, L] fp32
    pq_codebook: Optional[torch.Tensor] = None   # [M, 256, D/M] fp32
    M: int = 0                                   # only needed while pq_codebook is None
    const_table: Optional[torch.Tensor] = None   # [256] fp32
    sub_offsets: Optional[torch.Tensor] = None   # [K*L+1] uint32 bit patterns (int32 / int64 accepted)
    codes: Optional[torch.Tensor] = None         # [N, M] uint8
    const_byte: Optional[torch.Tensor] = None    # [N] uint8
    ids: Optional[torch.Tensor] = None           # [N] int32
    rotation: Optional[torch.Tensor] = None      # [D, D] fp32 rotation in front of the PQ

    def _c(self) -> _Desc:
        K, D = self.centroids.shape
        L = self.nbr.shape[1]
        M = self.pq_codebook.shape[0] if self.pq_codebook is not None else (self.M or 8)
        _dev(self.centroids, torch.float32, "centroids")
        _dev(self.nbr, torch.int32, "nbr", (K, L))
        _dev(self.alpha, torch.float32, "alpha", (K,))
        _dev(self.cs_dist2, torch.float32, "cs_dist2", (K, L))
        _dev(self.pq_codebook, torch.float32, "pq_codebook", (M, 256, D // M))
        _dev(self.const_table, torch.float32, "const_table", (256,))
        N = 0
        if self.codes is not None:
            N = self.codes.shape[0]
            _dev(self.codes, torch.uint8, "codes", (N, M))
            _dev(self.const_byte, torch.uint8, "const_byte", (N,))
            _dev(self.ids, torch.int32, "ids", (N,))
            if self.sub_offsets is None or self.sub_offsets.dtype not in (torch.int32, torch.uint32):
                raise IvfError("sub_offsets must be a 32-bit tensor of K*L+1 entries")
            _dev(self.sub_offsets, self.sub_offsets.dtype, "sub_offsets", (K * L + 1,))
        return _Desc(D, M, L, K, N, *[None if t is None else t.data_ptr() for t in (
            self.centroids, self.nbr, self.alpha, self.cs_dist2, self.pq_codebook, self.const_table,
            self.sub_offsets, self.codes, self.const_byte, self.ids, _dev(self.rotation, torch.float32, "rotation", (D, D)))])


class IndexHandle:
    def __init__(self, ptr, desc: IndexDesc):
        self.ptr = ptr
        self.K, self.D = desc.centroids.shape
        self.L = desc.nbr.shape[1]
        self.M = desc.pq_codebook.shape[0]
        self.N = desc.codes.shape[0]

    def __del__(self):
        try:
            ivf_free_index(self)
        except Exception:
            pass


def ivf_load_index(desc: IndexDesc) -> IndexHandle:
    lib = load_library()
    out = C.c_void_p()
    _check(lib.ivf_load_index(C.byref(desc._c()), _stream(), C.byref(out)))
    return IndexHandle(out, desc)


def ivf_free_index(index: IndexHandle) -> None:
    if index.ptr is not None:
        load_library().ivf_free_index(index.ptr)
        index.ptr = None


def ivf_set_scratch_limit(index: IndexHandle, nbytes: int) -> None:
    _check(load_library().ivf_set_scratch_limit(index.ptr, nbytes))


def ivf_num_kept(nprobe: int, L: int, prune_frac: float) -> int:
    return int(load_library().ivf_num_kept(nprobe, L, prune_frac))


def ivf_search(index: IndexHandle, queries: torch.Tensor, nprobe: int, prune_frac: float, k: int,
               out_ids: Optional[torch.Tensor] = None, out_dists: Optional[torch.Tensor] = None):
    """(ids [nq, k] int32, dists [nq, k] fp32); asynchronous on the current stream."""
    nq = queries.shape[0]
    _dev(queries, torch.float32, "queries", (nq, index.D))
    if out_ids is None:
        out_ids = torch.empty((nq, k), dtype=torch.int32, device=queries.device)
    if out_dists is None:
        out_dists = torch.empty((nq, k), dtype=torch.float32, device=queries.device)
    _dev(out_ids, torch.int32, "out_ids", (nq, k))
    _dev(out_dists, torch.float32, "out_dists", (nq, k))
    _check(load_library().ivf_search(index.ptr, _ptr(queries), nq, nprobe, prune_frac, k,
                                     _ptr(out_ids), _ptr(out_dists), _stream()))
    return out_ids, out_dists


def ivf_search_noalloc(index: IndexHandle, queries: torch.Tensor, nprobe: int, prune_frac: float, k: int,
                       out_ids: torch.Tensor, out_dists: torch.Tensor):
    """ivf_search on the library's static scratch array: the call allocates nothing (outputs are the caller's)."""
    nq = queries.shape[0]
    _dev(queries, torch.float32, "queries", (nq, index.D))
    _dev(out_ids, torch.int32, "out_ids", (nq, k))
    _dev(out_dists, torch.float32, "out_dists", (nq, k))
    _check(load_library().ivf_search_noalloc(index.ptr, _ptr(queries), nq, nprobe, prune_frac, k,
                                             _ptr(out_ids), _ptr(out_dists), _stream()))
    return out_ids, out_dists


def ivf_search_stages(index: IndexHandle, queries: torch.Tensor, nprobe: int, prune_frac: float, k: int):
    """ivf_search plus the stage-1 probes, the kept subregions and the scanned-record counts."""
    nq = queries.shape[0]
    _dev(queries, torch.float32, "queries", (nq, index.D))
    dev = queries.device
    S = ivf_num_kept(nprobe, index.L, prune_frac)
    out = {
        "ids": torch.empty((nq, k), dtype=torch.int32, device=dev),
        "dists": torch.empty((nq, k), dtype=torch.float32, device=dev),
        "probe_id": torch.empty((nq, nprobe), dtype=torch.int32, device=dev),
        "probe_d": torch.empty((nq, nprobe), dtype=torch.float32, device=dev),
        "kept_sub": torch.empty((nq, S), dtype=torch.int64, device=dev),
        "n_scanned": torch.empty((nq,), dtype=torch.int64, device=dev),
    }
    _check(load_library().ivf_search_stages(
        index.ptr, _ptr(queries), nq, nprobe, prune_frac, k, _ptr(out["ids"]), _ptr(out["dists"]),
        _ptr(out["probe_id"]), _ptr(out["probe_d"]), _ptr(out["kept_sub"]), _ptr(out["n_scanned"]),
        _stream()))
    return out


def ivf_search_budget(index: IndexHandle, queries: torch.Tensor, nprobe: int, prune_frac: float,
                      max_candidates: int, k: int):
    """Search that stops collecting candidates after ``max_candidates`` points: ids, dists, the kept
    subregions, the flags of the visited ones and the number of records read per query."""
    nq = queries.shape[0]
    _dev(queries, torch.float32, "queries", (nq, index.D))
    dev = queries.device
    S = ivf_num_kept(nprobe, index.L, prune_frac)
    out = {
        "ids": torch.empty((nq, k), dtype=torch.int32, device=dev),
        "dists": torch.empty((nq, k), dtype=torch.float32, device=dev),
        "kept_sub": torch.empty((nq, S), dtype=torch.int64, device=dev),
        "visited": torch.empty((nq, S), dtype=torch.uint8, device=dev),
        "n_scanned": torch.empty((nq,), dtype=torch.int64, device=dev),
    }
    _check(load_library().ivf_search_budget(
        index.ptr, _ptr(queries), nq, nprobe, prune_frac, max_candidates, k, _ptr(out["ids"]), _ptr(out["dists"]),
        _ptr(out["kept_sub"]), _ptr(out["visited"]), _ptr(out["n_scanned"]), _stream()))
    return out


def ivf_assign_stats():
    """(chunks decided by the shortlist, chunks decided by the one-pass exact kernel) so far in this process."""
    out = (C.c_int64 * 2)()
    load_library().ivf_assign_stats(out)
    return int(out[0]), int(out[1])


def ivf_coarse_topk(centroids: torch.Tensor, x: torch.Tensor, P: int):
    """(ids [n, P] int32 ascending centroid id, squared distances [n, P] fp32)."""
    K, D = centroids.shape
    n = x.shape[0]
    _dev(centroids, torch.float32, "centroids")
    _dev(x, torch.float32, "x", (n, D))
    oid = torch.empty((n, P), dtype=torch.int32, device=x.device)
    od = torch.empty((n, P), dtype=torch.float32, device=x.device)
    _check(load_library().ivf_coarse_topk(_ptr(centroids), K, D, _ptr(x), n, P, _ptr(oid), _ptr(od), _stream()))
    return oid, od


def ivf_encode(trained: IndexDesc, x: torch.Tensor, region_in: Optional[torch.Tensor] = None,
               want_t: bool = False, want_residual: bool = False):
    """(region, sub, codes, const_byte, t[, residual]) for the points x [n, D]."""
    n = x.shape[0]
    c = trained._c()
    _dev(x, torch.float32, "x", (n, c.D))
    _dev(region_in, torch.int32, "region_in", (n,))
    dev = x.device
    region = torch.empty(n, dtype=torch.int32, device=dev)
    sub = torch.empty(n, dtype=torch.int32, device=dev)
    has_pq = trained.pq_codebook is not None
    codes = torch.empty((n, c.M), dtype=torch.uint8, device=dev) if has_pq else None
    byte = torch.empty(n, dtype=torch.uint8, device=dev) if has_pq and trained.const_table is not None else None
    t = torch.empty(n, dtype=torch.float32, device=dev) if want_t and has_pq else None
    res = torch.empty((n, c.D), dtype=torch.float32, device=dev) if want_residual else None
    _check(load_library().ivf_encode(C.byref(c), _ptr(x), n, _ptr(region_in), _ptr(region), _ptr(sub),
                                     _ptr(codes), _ptr(byte), _ptr(t), _ptr(res), _stream()))
    if want_residual:
        return region, sub, codes, byte, t, res
    return region, sub, codes, byte, t


def ivf_rotate(x: torch.Tensor, rotation: torch.Tensor):
    """Rows of x multiplied by the D x D rotation: out[i] = R x[i]."""
    n, D = x.shape
    _dev(x, torch.float32, "x", (n, D))
    _dev(rotation, torch.float32, "rotation", (D, D))
    out = torch.empty_like(x)
    _check(load_library().ivf_rotate(_ptr(x), n, D, _ptr(rotation), _ptr(out), _stream()))
    return out


def ivf_kmeans(x: torch.Tensor, K: int, iters: int, init_idx: torch.Tensor, want_objective: bool = False):
    """Region codebook [K, D] by Lloyd's k-means from the rows init_idx of x (and the objective per round)."""
    n, D = x.shape
    _dev(x, torch.float32, "x", (n, D))
    _dev(init_idx, torch.int64, "init_idx", (K,))
    cent = torch.empty((K, D), dtype=torch.float32, device=x.device)
    obj = torch.zeros(max(iters, 1), dtype=torch.float64, device=x.device) if want_objective else None
    _check(load_library().ivf_kmeans(_ptr(x), n, D, K, iters, _ptr(init_idx), _ptr(cent), _ptr(obj), _stream()))
    return (cent, obj[:iters]) if want_objective else cent


def ivf_cluster_means(x: torch.Tensor, assign: torch.Tensor, centroids: torch.Tensor):
    """One k-means update with a given assignment; returns a new [K, D] tensor (empty clusters keep `centroids`)."""
    n, D = x.shape
    K = centroids.shape[0]
    _dev(x, torch.float32, "x", (n, D))
    _dev(assign, torch.int32, "assign", (n,))
    _dev(centroids, torch.float32, "centroids", (K, D))
    out = centroids.clone()
    _check(load_library().ivf_cluster_means(_ptr(x), n, D, _ptr(assign), K, _ptr(out), _stream()))
    return out


def ivf_bucket_ids(region: torch.Tensor, sub: torch.Tensor, L: int, out: Optional[torch.Tensor] = None):
    """bucket = region * L + sub (int32), optionally into a slice of a larger tensor."""
    n = region.shape[0]
    _dev(region, torch.int32, "region", (n,))
    _dev(sub, torch.int32, "sub", (n,))
    if out is None:
        out = torch.empty(n, dtype=torch.int32, device=region.device)
    _dev(out, torch.int32, "bucket", (n,))
    _check(load_library().ivf_bucket_ids(_ptr(region), _ptr(sub), n, L, _ptr(out), _stream()))
    return out


def ivf_neighbours(centroids: torch.Tensor, L: int):
    """(nbr [K, L] int32, cs_dist2 [K, L] fp32): the L nearest other centroids of each centroid, by (distance, id)."""
    K, D = centroids.shape
    _dev(centroids, torch.float32, "centroids")
    nbr = torch.empty((K, L), dtype=torch.int32, device=centroids.device)
    cs = torch.empty((K, L), dtype=torch.float32, device=centroids.device)
    _check(load_library().ivf_neighbours(_ptr(centroids), K, D, L, _ptr(nbr), _ptr(cs), _stream()))
    return nbr, cs


def ivf_learn_alpha(centroids: torch.Tensor, nbr: torch.Tensor, x: torch.Tensor, region: torch.Tensor):
    """alpha [K] fp32 from the training points x with their regions."""
    K, D = centroids.shape
    L = nbr.shape[1]
    n = x.shape[0]
    _dev(centroids, torch.float32, "centroids")
    _dev(nbr, torch.int32, "nbr", (K, L))
    _dev(x, torch.float32, "x", (n, D))
    _dev(region, torch.int32, "region", (n,))
    alpha = torch.empty(K, dtype=torch.float32, device=x.device)
    _check(load_library().ivf_learn_alpha(_ptr(centroids), K, D, _ptr(nbr), L, _ptr(x), n, _ptr(region),
                                          _ptr(alpha), _stream()))
    return alpha


def ivf_pq_train(E: torch.Tensor, M: int, iters: int, init_idx: torch.Tensor):
    """PQ codebooks [M, 256, D/M] trained on the displacements E [n, D]."""
    n, D = E.shape
    _dev(E, torch.float32, "E", (n, D))
    _dev(init_idx, torch.int64, "init_idx", (256,))
    cb = torch.empty((M, 256, D // M), dtype=torch.float32, device=E.device)
    _check(load_library().ivf_pq_train(_ptr(E), n, D, M, iters, _ptr(init_idx), _ptr(cb), _stream()))
    return cb


def ivf_lloyd_1d(t: torch.Tensor, iters: int):
    """256-level scalar quantiser table (ascending fp32) for the values t."""
    n = t.shape[0]
    _dev(t, torch.float32, "t", (n,))
    table = torch.empty(256, dtype=torch.float32, device=t.device)
    _check(load_library().ivf_lloyd_1d(_ptr(t), n, iters, _ptr(table), _stream()))
    return table


def ivf_group(bucket: torch.Tensor, nbuckets: int):
    """(perm [n] int32, offsets [nbuckets + 1] uint32 bit patterns as int32): items listed bucket by bucket, stable."""
    n = bucket.shape[0]
    _dev(bucket, torch.int32, "bucket", (n,))
    perm = torch.empty(n, dtype=torch.int32, device=bucket.device)
    off = torch.empty(nbuckets + 1, dtype=torch.int32, device=bucket.device)
    _check(load_library().ivf_group(_ptr(bucket), n, nbuckets, _ptr(perm), _ptr(off), _stream()))
    return perm, off


def ivf_gather_rows(src: torch.Tensor, perm: torch.Tensor, out: Optional[torch.Tensor] = None):
    """out[j] = src[perm[j]] along dim 0 (rows copied byte for byte)."""
    n = perm.shape[0]
    if not (src.is_cuda and src.is_contiguous()):
        raise IvfError("src must be a contiguous device tensor")
    _dev(perm, torch.int32, "perm", (n,))
    row_bytes = src.element_size() * (src.numel() // max(src.shape[0], 1))
    if out is None:
        out = torch.empty((n,) + tuple(src.shape[1:]), dtype=src.dtype, device=src.device)
    _check(load_library().ivf_gather_rows(_ptr(src), row_bytes, _ptr(perm), n, _ptr(out), _stream()))
    return out


STAGE_NAMES = ("coarse_gemm", "probe_select", "score_prune", "lut", "scan", "merge")


def ivf_profile_enable(index: IndexHandle, on: bool) -> None:
    _check(load_library().ivf_profile_enable(index.ptr, 1 if on else 0))


def ivf_profile_read(index: IndexHandle):
    """({stage name: summed milliseconds}, number of query-tile passes) since the last read."""
    ms = (C.c_double * len(STAGE_NAMES))()
    n = C.c_int64()
    _check(load_library().ivf_profile_read(index.ptr, ms, C.byref(n)))
    return dict(zip(STAGE_NAMES, list(ms))), n.value


def ivf_copy_bytes(dst: torch.Tensor, src: torch.Tensor) -> None:
    """Streaming copy of src's bytes into dst (same byte size, multiple of 16)."""
    nbytes = src.numel() * src.element_size()
    if dst.numel() * dst.element_size() != nbytes or not (src.is_cuda and dst.is_cuda):
        raise IvfError("ivf_copy_bytes: device tensors of equal byte size expected")
    _check(load_library().ivf_copy_bytes(_ptr(dst), _ptr(src), nbytes, _stream()))
