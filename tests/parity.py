"""Comparison of the HIP library's results with the oracle's, stage by stage.

Selections (probed regions, kept subregions, returned ids) must be identical.
Where they differ, the oracle's fp64 values of the items in the symmetric
difference are inspected: if every one lies within ``tol`` of the selection
boundary the query is counted as a *near-tie* (fp32 rounding decided between
values the oracle sees as almost equal), the GPU's selection is injected into
the oracle for the following stages, and the comparison carries on; anything
else is a mismatch.

Tolerances (derived from the arithmetic, fp32 unit roundoff u = 2^-24):
  selection   max(1e-5 * |boundary value|, 16 u (||q||^2 + max ||c||^2))
              — the expansion ||q||^2 - 2<q,c> + ||c||^2 carries an absolute
              error proportional to the size of its terms, not of the result
  distances   1e-4 relative (plus the same absolute term)
"""
import numpy as np
import torch

from oracle import ivf_oracle as orc
import paper_1802_02422_amd as ivf

U = 2.0 ** -24


def to_device(ix, with_codes=True):
    dev = torch.device("cuda:0")
    t = lambda a, dt=None: torch.from_numpy(np.ascontiguousarray(a)).to(dev)
    d = ivf.IndexDesc(t(ix.centroids), t(ix.nbr), t(ix.alpha), t(ix.cs_dist2), t(ix.pq_codebook),
                      const_table=t(ix.const_table))
    if with_codes:
        d.sub_offsets = t(ix.sub_offsets.view(np.int32))
        d.codes = t(ix.codes)
        d.const_byte = t(ix.const_byte)
        d.ids = t(ix.ids)
    if getattr(ix, "rotation", None) is not None:
        d.rotation = t(ix.rotation)
    return d


def abs_term(ix, Q):
    qn = (Q.astype(np.float64) ** 2).sum(1)
    cn = (ix.centroids.astype(np.float64) ** 2).sum(1).max()
    return 16 * U * (qn + cn)


def compare_selection(gpu_sel, orc_sel, value_of, boundary, tol):
    """Returns 'exact', 'near' or 'mismatch' for one query's selected sets."""
    g, o = set(int(v) for v in gpu_sel), set(int(v) for v in orc_sel)
    if g == o:
        return "exact", 0.0
    if len(g) != len(o):
        return "mismatch", np.inf
    gap = max(abs(value_of(i) - boundary) for i in (g ^ o))
    return ("near", gap) if gap <= tol else ("mismatch", gap)


class Report:
    def __init__(self):
        self.counts = {}
        self.max_gap = {}
        self.max_rel = 0.0       # beyond the absolute floor of the tolerance (what the bar applies to)
        self.max_rel_raw = 0.0   # plain |gpu - oracle| / |oracle| wherever |oracle| exceeds 1e4 x the absolute floor

    def add(self, stage, kind, gap=0.0):
        self.counts.setdefault(stage, {"exact": 0, "near": 0, "mismatch": 0})[kind] += 1
        self.max_gap[stage] = max(self.max_gap.get(stage, 0.0), gap if np.isfinite(gap) else 0.0)

    def __str__(self):
        parts = [f"{s}: {c} max-gap {self.max_gap[s]:.3g}" for s, c in self.counts.items()]
        return "; ".join(parts) + f"; max rel dist err {self.max_rel:.3g} (raw {self.max_rel_raw:.3g})"

    def assert_ok(self, max_near_frac=0.05):
        for s, c in self.counts.items():
            assert c["mismatch"] == 0, f"{s}: {c}  [{self}]"
            n = sum(c.values())
            assert c["near"] <= max(2, max_near_frac * n), f"{s}: too many near-ties {c}"
        assert self.max_rel <= 1e-4, f"distance error {self.max_rel}"
        assert self.max_rel_raw <= 1e-4, f"raw relative distance error {self.max_rel_raw}"
        print("near-ties per stage:", {s: c["near"] for s, c in self.counts.items()}, flush=True)


def check_search(ix, Q, nprobe, prune_frac, k, out, rep=None):
    """Compare the stage outputs `out` of ivf_search_stages (CPU numpy arrays) with the oracle."""
    rep = rep or Report()
    nq = Q.shape[0]
    L = ix.L
    tau = float(np.float32(prune_frac))
    at = abs_term(ix, Q)
    # stage 1
    o_pid, o_pd = orc.probe(Q, ix.centroids, nprobe)
    g_pid = out["probe_id"]
    assert (np.diff(g_pid, axis=1) > 0).all(), "probe ids must be ascending and distinct"
    c64 = ix.centroids.astype(np.float64)
    for q in range(nq):
        dist = lambda j, q=q: float(((Q[q].astype(np.float64) - c64[j]) ** 2).sum())
        b = o_pd[q, -1]
        kind, gap = compare_selection(g_pid[q], o_pid[q], dist, b, max(1e-5 * abs(b), at[q]))
        rep.add("probe", kind, gap)
    d_true = ((Q.astype(np.float64)[:, None, :] - c64[g_pid]) ** 2).sum(-1)
    err = np.abs(out["probe_d"] - d_true) / np.maximum(d_true, 1e-30)
    ok = np.abs(out["probe_d"] - d_true) <= np.maximum(1e-4 * d_true, at[:, None])
    assert ok.all(), f"stage-1 distances off: rel {err.max()}"
    # stage 2+3 on the GPU's probes
    sc = orc.scores(Q, ix, g_pid)
    o_kept, o_ks = orc.prune(sc, g_pid, tau)
    g_kept = out["kept_sub"]
    assert g_kept.shape == o_kept.shape, (g_kept.shape, o_kept.shape)
    assert (np.diff(g_kept, axis=1) > 0).all(), "kept subregions must be ascending and distinct"
    for q in range(nq):
        sid = (g_pid[q].astype(np.int64)[:, None] * L + np.arange(L)[None]).ravel()
        look = dict(zip(sid.tolist(), sc[q].ravel().tolist()))
        assert set(g_kept[q].tolist()) <= set(look), "kept a subregion that was not scored"
        b = o_ks[q, -1]
        kind, gap = compare_selection(g_kept[q], o_kept[q], lambda s: look[s], b, max(1e-5 * abs(b), at[q]))
        rep.add("prune", kind, gap)
    # stages 4-6 on the GPU's kept subregions
    st = orc.search_staged(ix, Q, nprobe, tau, k, probe_id=g_pid, kept=g_kept)
    check_topk(ix, st, out, at, rep)
    return rep


def check_topk(ix, st, out, at, rep):
    """Stages 5-6: scanned-record counts, returned ids and distances against the oracle's staged
    result `st` (computed on the GPU's own kept / visited subregions)."""
    nq = out["ids"].shape[0]
    assert (np.diff(st["cand_start"]) == out["n_scanned"]).all(), "scanned-record counts differ"
    g_ids, g_d = out["ids"], out["dists"]
    for q in range(nq):
        cpos = st["cand_pos"][st["cand_start"][q]:st["cand_start"][q + 1]]
        cd = dict(zip(ix.ids[cpos].tolist(), st["cand_dist"][st["cand_start"][q]:st["cand_start"][q + 1]].tolist()))
        o_ids, o_d = st["ids"][q], st["dists"][q]
        n_valid = int((o_ids >= 0).sum())
        assert (g_ids[q, n_valid:] == -1).all() and np.isinf(g_d[q, n_valid:]).all(), "padding"
        gi = g_ids[q, :n_valid]
        assert len(set(gi.tolist())) == n_valid and set(gi.tolist()) <= set(cd), "returned id not a candidate / repeated"
        tol = max(1e-5 * abs(o_d[n_valid - 1]), at[q]) if n_valid else 0.0
        if (gi == o_ids[:n_valid]).all():
            rep.add("topk", "exact")
        else:
            dg = np.array([cd[i] for i in gi.tolist()])
            set_ok = all(abs(cd[i] - o_d[n_valid - 1]) <= tol for i in set(gi.tolist()) ^ set(o_ids[:n_valid].tolist()))
            order_ok = (np.diff(dg) >= -tol).all()
            rep.add("topk", "near" if (set_ok and order_ok) else "mismatch",
                    float(np.abs(np.sort(dg) - o_d[:n_valid]).max()))
        if n_valid:
            dg = np.array([cd[i] for i in gi.tolist()])
            e = np.abs(g_d[q, :n_valid].astype(np.float64) - dg)
            rel = (np.maximum(e - at[q], 0) / np.maximum(np.abs(dg), 1e-30)).max()
            rep.max_rel = max(rep.max_rel, float(rel))
            # the plain bar, 1e-4 relative with no allowance, wherever it is attainable in fp32: the estimate
            # is a sum of O(||q||^2 + ||c||^2) terms and carries an absolute error of the order of the floor
            # `at`, so it can be 1e-4-relative only for distances above 1e4 * at (every distance of the
            # benchmark workloads is: they are ~5e5 * at); below that the bar above (with the floor) applies
            clear = np.abs(dg) > 1e4 * at[q]
            if clear.any():
                rep.max_rel_raw = max(rep.max_rel_raw, float((e[clear] / np.abs(dg[clear])).max()))
            assert (np.diff(g_d[q, :n_valid]) >= 0).all(), "returned distances not ascending"


def check_search_budget(ix, Q, nprobe, prune_frac, R, k, stages_out, budget_out, rep=None):
    """The candidate-budget search against the oracle.  `stages_out` is ivf_search_stages on the same
    queries and parameters (its probes and kept subregions are checked as usual and must be the ones
    the budget call reports); `budget_out` is ivf_search_budget's output."""
    rep = check_search(ix, Q, nprobe, prune_frac, k, stages_out, rep)
    tau = float(np.float32(prune_frac))
    at = abs_term(ix, Q)
    g_pid, g_kept, g_vis = stages_out["probe_id"], budget_out["kept_sub"], budget_out["visited"]
    assert (g_kept == stages_out["kept_sub"]).all(), "the budget call kept other subregions than the plain call"
    st = orc.search_staged(ix, Q, nprobe, tau, k, probe_id=g_pid, kept=g_kept, budget=R)
    o_vis, score = st["visit"], st["scan_score"]
    sizes = np.diff(ix.sub_offsets.astype(np.int64))
    for q in range(Q.shape[0]):
        if (g_vis[q] == o_vis[q]).all():
            rep.add("budget", "exact")
            continue
        # boundary: the last subregion the oracle visits, in (score, id) order
        vis_idx = np.flatnonzero(o_vis[q])
        last = max(vis_idx.tolist(), key=lambda j: (score[q, j], g_kept[q, j]))
        b = score[q, last]
        diff = np.flatnonzero(g_vis[q] != o_vis[q])
        gap = float(np.abs(score[q, diff] - b).max())
        got = int(sizes[g_kept[q]][g_vis[q] == 1].sum())
        total = int(sizes[g_kept[q]].sum())
        ok = gap <= max(1e-5 * abs(b), at[q]) and got >= min(R, total)
        rep.add("budget", "near" if ok else "mismatch", gap)
    st = orc.search_staged(ix, Q, nprobe, tau, k, probe_id=g_pid, kept=g_kept, budget=R, visit=g_vis)
    check_topk(ix, st, budget_out, at, rep)
    return rep


def run_gpu_search(handle, Q, nprobe, prune_frac, k):
    Qd = torch.from_numpy(Q).cuda()
    out = ivf.ivf_search_stages(handle, Qd, nprobe, prune_frac, k)
    torch.cuda.synchronize()
    return {n: v.cpu().numpy() for n, v in out.items()}
