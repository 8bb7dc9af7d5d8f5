"""Helpers shared by the GPU parity tests, smoke() and bench.py's checks.

run_gpu()      drives the HIP library through its C ABI (via the ctypes binding) on cuda:0.
check_parity() compares every stage with the CPU oracle.

Near-threshold protocol.  Cluster maps must be bit-identical to the oracle's, except that a decision
whose fp64 similarity lies within BAND = 1e-5 of the threshold may fall either way (the GPU accumulates
in fp32).  The oracle is authoritative outside the band; inside it, and only there, it is told which way
the GPU decided (a hook it consults only when |sigma64 - tau| <= BAND), and the number of such decisions
is reported.  All other oracle inputs are the seeded synthetic features and thresholds.
"""
from __future__ import annotations

import math
from typing import Optional

import numpy as np

from oracle import sttm_oracle as O

BAND = O.BAND
SIM_TOL = 1e-5          # |sigma_gpu(fp32) - sigma_oracle(fp64)|
TOL_F32 = 1e-3          # merged features, fp32 in / fp32 out
TOL_BF16 = 2e-2         # bf16 in, fp32 accumulate
TOL_F16 = 5e-3          # fp16 in / out: half an ulp of the output, 2^-11 |x| <= 3.9e-3 for |x| < 8, plus fp32 sums


class GpuResult:
    pass


def _to_dev(feats: np.ndarray):
    import torch
    if feats.dtype == np.uint16:
        return torch.from_numpy(feats.view(np.int16)).cuda().view(torch.bfloat16)
    return torch.from_numpy(feats).cuda()


def lib_dtype(lib, feats: np.ndarray) -> int:
    return {np.dtype(np.uint16): lib.STTM_BF16, np.dtype(np.float16): lib.STTM_F16}.get(feats.dtype, lib.STTM_F32)


MODES = {"first_passing": 0, "topleft_only": 1, "most_similar": 2}
ORDERS = {"raster": 0, "zscan": 1}


CANARY_BYTES = 4096
CANARY_FILL = 0xA5


class Guarded:
    """Caller buffers with a band of CANARY_BYTES known bytes on either side: a kernel that stores outside a buffer
    it was handed changes a band, and check() says which one. The second band starts at the buffer's last byte."""

    def __init__(self, dev="cuda:0"):
        self.dev = dev
        self.items = []

    def alloc(self, name, n_elems, dtype, zero=False):
        import torch
        nbytes = int(n_elems) * torch.empty(0, dtype=dtype).element_size()
        raw = torch.full((2 * CANARY_BYTES + nbytes,), CANARY_FILL, dtype=torch.uint8, device=self.dev)
        view = raw[CANARY_BYTES:CANARY_BYTES + nbytes].view(dtype)
        if zero:
            view.zero_()
        self.items.append((name, raw, nbytes))
        return view

    def check(self, after: str):
        for name, raw, nbytes in self.items:
            lo = bool((raw[:CANARY_BYTES] == CANARY_FILL).all().item())
            hi = bool((raw[CANARY_BYTES + nbytes:] == CANARY_FILL).all().item())
            assert lo and hi, f"bytes {'before' if not lo else 'after'} buffer '{name}' were overwritten by {after}"


def run_gpu(lib, feats: np.ndarray, *, tau_s=None, tau_t=None, keep=None, root_grid: int = 1,
            out_dtype: Optional[int] = None, node_map_override=None, ctx=None, feats_dev=None,
            use_nodes: bool = True, mode: str = "first_passing", order: str = "raster",
            positions: bool = False, cell_dots: int = 1) -> GpuResult:
    """Whole path through the C ABI. Fixed thresholds, or `keep` (budget mode). Every buffer the library writes
    for the caller sits between canary bands, which are checked after every call."""
    import torch
    B, T, H, W, D = feats.shape
    dt = lib_dtype(lib, feats)
    if out_dtype is None:
        out_dtype = dt
    x = _to_dev(feats) if feats_dev is None else feats_dev
    s = ctx or lib.Sttm(0)
    s.sttm_set_match_mode(MODES[mode])
    s.sttm_set_output_order(ORDERS[order])
    s.sttm_set_cell_dots(cell_dots)
    s.ensure_workspace(B, T, H, W, D, dt, root_grid)
    N = B * T * H * W
    NN = lib.sttm_nodes_per_frame(H, W, root_grid)
    dev = "cuda:0"
    r = GpuResult()
    gd = Guarded(dev)
    node_map = gd.alloc("node_map", N, torch.int32)
    node_level = gd.alloc("node_level", N, torch.uint8)
    cluster = gd.alloc("cluster_ids", N, torch.int32)
    r.tau_s = r.tau_t = None
    if tau_s is None:
        s.sttm_spatial_stats(x, dt, B, T, H, W, D, root_grid)
        r.tau_s = s.sttm_budget_threshold(lib.STTM_STAGE_SPATIAL, keep)
        s.sttm_spatial_quadtree(x, dt, B, T, H, W, D, root_grid, None, node_map, node_level)
    else:
        s.sttm_spatial_quadtree(x, dt, B, T, H, W, D, root_grid, tau_s, node_map, node_level)
    gd.check("the spatial stage")
    tbl = gd.alloc("export table", B * T * NN, torch.float32)
    s.sttm_export(lib.STTM_TBL_CHILD_SIM, tbl)
    r.child_sim = tbl.cpu().numpy().reshape(B * T, NN)
    s.sttm_export(lib.STTM_TBL_MIN_SIM, tbl)
    r.min_sim = tbl.cpu().numpy().reshape(B * T, NN)
    r.node_map = node_map.cpu().numpy().reshape(B, T, H, W)
    r.node_level = node_level.cpu().numpy().reshape(B, T, H, W)
    if node_map_override is not None:
        node_map.copy_(torch.from_numpy(node_map_override[0].reshape(-1)).cuda())
        node_level.copy_(torch.from_numpy(node_map_override[1].reshape(-1)).cuda())
    if tau_t is None:
        s.sttm_temporal_stats(x, node_map, node_level)
        r.tau_t = s.sttm_budget_threshold(lib.STTM_STAGE_TEMPORAL, keep)
        s.sttm_temporal_merge(x, node_map, node_level, None, cluster)
    else:
        s.sttm_temporal_merge(x, node_map, node_level, tau_t, cluster)
    gd.check("the temporal stage")
    t32 = gd.alloc("export table (cells)", N, torch.float32)
    s.sttm_export(lib.STTM_TBL_PAIR_SIM, t32)
    r.pair_sim = t32.cpu().numpy()
    s.sttm_export(lib.STTM_TBL_BEST_SIM, t32)
    r.best_sim = t32.cpu().numpy()
    ti = gd.alloc("export table (parent)", N, torch.int32)
    s.sttm_export(lib.STTM_TBL_PARENT, ti)
    r.parent = ti.cpu().numpy().reshape(B, T, H, W)
    r.cluster_ids = cluster.cpu().numpy().reshape(B, T, H, W)
    odt = {lib.STTM_BF16: torch.bfloat16, lib.STTM_F16: torch.float16}.get(out_dtype, torch.float32)
    merged = gd.alloc("merged", N * D, odt, zero=True).view(N, D)
    counts = gd.alloc("counts", N, torch.int32, zero=True)
    out_ids = gd.alloc("out_ids", N, torch.int32, zero=True)
    offsets = gd.alloc("offsets", B + 1, torch.int64, zero=True)
    K = s.sttm_reduce(x, cluster, node_map if use_nodes else None, node_level if use_nodes else None, out_dtype, N,
                      merged, counts, out_ids, offsets)
    gd.check("the reduce stage")
    r.K = K
    r.merged = merged[:K].float().cpu().numpy()
    r.counts = counts[:K].cpu().numpy()
    r.out_ids = out_ids[:K].cpu().numpy()
    r.offsets = offsets.cpu().numpy()
    if positions:
        sv = gd.alloc("survived", N, torch.int32, zero=True)
        ra = gd.alloc("reassigned", N, torch.int32, zero=True)
        mp = gd.alloc("merged_pos", N, torch.float32, zero=True)
        rt = gd.alloc("root_tyxl", 4 * N, torch.int32, zero=True).view(N, 4)
        s.sttm_positions(cluster, node_map if use_nodes else None, node_level, offsets, N, sv, ra, mp, rt)
        gd.check("the position indices")
        r.survived, r.reassigned = sv[:K].cpu().numpy(), ra[:K].cpu().numpy()
        r.merged_pos, r.root_tyxl = mp[:K].cpu().numpy(), rt[:K].cpu().numpy()
    r.ctx = s
    r.feats_dev = x
    return r


def check_spatial(lib, feats, r: GpuResult, tau_s, root_grid=1, stats=None):
    """Similarity tables within SIM_TOL, node map identical under the near-threshold protocol."""
    B, T, H, W, D = feats.shape
    HW = H * W
    stats = stats or O.spatial_stats(feats, root_grid, keep_means=False)
    grid = stats[0]
    worst = 0.0
    for f, (_, cnt, sims, m) in enumerate(stats[1]):
        for lvl in range(1, grid.L + 1):
            g = grid.side(lvl)
            for by in range(g):
                for bx in range(g):
                    if cnt[lvl][by, bx] == 0:
                        continue
                    for k in range(4):
                        cy, cx = 2 * by + (k >> 1), 2 * bx + (k & 1)
                        if cnt[lvl - 1][cy, cx] == 0:
                            continue
                        got = float(r.child_sim[f, lib.sttm_node_index(H, W, root_grid, lvl - 1, cy, cx)])
                        want = float(sims[lvl][by, bx, k])
                        assert (got != got) == (want != want), "undefined similarity on one side only"
                        if want == want:
                            worst = max(worst, abs(got - want))
                    gm = float(r.min_sim[f, lib.sttm_node_index(H, W, root_grid, lvl, by, bx)])
                    wm = float(m[lvl][by, bx])
                    assert (gm != gm) == (wm != wm), "undefined minimum similarity on one side only"
                    if wm == wm:
                        worst = max(worst, abs(gm - wm))
    assert worst <= SIM_TOL, f"spatial similarity error {worst}"

    def decide(b, t, lvl, by, bx, val):
        y0, x0 = by << lvl, bx << lvl
        return bool(r.node_level[b, t, y0, x0] == lvl and r.node_map[b, t, y0, x0] == (b * T + t) * HW + y0 * W + x0)

    sp = O.spatial_quadtree(feats, tau_s, root_grid, stats=stats, decide=decide)
    assert (sp.node_map == r.node_map).all(), "node_map differs from the oracle outside the threshold band"
    # levels may differ only for nodes with a single existing child chain (same cells either way)
    assert (sp.node_level == r.node_level).all()
    return sp, worst


def check_temporal(lib, feats, r: GpuResult, sp, tau_t, cands=None, mode: str = "first_passing"):
    B, T, H, W, D = feats.shape
    if cands is None:
        cands, _ = O.temporal_candidates(feats, sp.node_map, sp.node_level)
    HW = H * W
    worst = 0.0
    lvl_flat = sp.node_level.reshape(-1)
    for n, lst in cands.items():
        f = n // HW
        for d, sig in lst:
            # slot = top-left cell of the finer node, in frame f's table
            q = n if lvl_flat[n] <= lvl_flat[d] else d + HW
            got = float(r.pair_sim[q])
            assert (got != got) == (sig != sig), "undefined pair similarity on one side only"
            if sig == sig:
                worst = max(worst, abs(got - sig))
    best = O.best_similarity(cands, sp.node_map, mode)
    for n in cands:
        worst = max(worst, abs(float(r.best_sim[n]) - best[n]))
    assert worst <= SIM_TOL, f"temporal similarity error {worst}"
    gpar = r.parent.reshape(-1)
    tau_b = np.broadcast_to(np.asarray(tau_t, dtype=np.float64), (B,))

    def decide(n, d, sig):
        # inside the band the oracle goes with what the GPU did, as far as its edge tells
        p = int(gpar[n])
        if d == p:
            return True
        if mode == "first_passing":
            if p < 0 or d < p:
                return False
            return None
        if mode == "topleft_only":
            return False if p < 0 else None
        if p < 0:
            return False
        # most similar: a band candidate the GPU did not take may or may not have passed there; it lost either
        # way unless it beats the GPU's choice by more than the band, which the oracle's own ranking settles
        return None

    def choose(n, near_best):
        p = int(gpar[n])
        return p if any(d == p for d, _ in near_best) else None

    tm = O.temporal_merge(feats, sp.node_map, sp.node_level, tau_t, cands=cands, decide=decide, mode=mode,
                          choose=choose)
    nodes = np.unique(sp.node_map)
    assert (tm.parent.reshape(-1)[nodes] == gpar[nodes]).all(), "parent differs outside the threshold band"
    assert (tm.cluster_ids == r.cluster_ids).all(), "cluster_ids differ"
    return tm, worst


def check_positions(r: GpuResult, sp, tm, order: str = "raster"):
    pr = O.positions(tm.cluster_ids, sp.node_level, order)
    assert (r.survived == pr.survived).all() and (r.reassigned == pr.reassigned).all()
    assert (r.root_tyxl == pr.root).all()
    err = float(np.abs(r.merged_pos.astype(np.float64) - pr.merged).max()) if r.K else 0.0
    # fp32 output of an exact integer mean: half an ulp of the largest index
    assert err <= max(1.0, float(pr.merged.max())) * 2.0 ** -23, f"merged position error {err}"
    return err


def check_reduce(feats, r: GpuResult, tm, out_is_bf16: bool, order: str = "raster", out_is_f16: bool = False):
    rd = O.reduce_clusters(feats, tm.cluster_ids, order)
    assert r.K == len(rd.counts)
    assert (r.counts == rd.counts).all() and (r.out_ids == rd.out_ids).all()
    assert (r.offsets == rd.offsets).all()
    assert int(r.counts.sum()) == feats.shape[0] * feats.shape[1] * feats.shape[2] * feats.shape[3]
    if feats.dtype == np.uint16 or out_is_bf16:
        tol, half_ulp = TOL_BF16, 2.0 ** -8
    elif feats.dtype == np.float16 or out_is_f16:
        tol, half_ulp = TOL_F16, 2.0 ** -11
    else:
        tol, half_ulp = TOL_F32, 2.0 ** -23
    if not r.K:
        return rd, 0.0
    # The absolute figures above are half an ulp of the output for values of a few units (what the workloads hold)
    # plus the fp32 sums; the rounding of the output scales with the value, so beyond that range the bound does too.
    diff = np.abs(r.merged.astype(np.float64) - rd.merged)
    bound = np.maximum(tol, half_ulp * np.abs(rd.merged) + TOL_F32)
    err = float(diff.max())
    assert (diff <= bound).all(), f"merged feature error {float((diff - bound).max())} beyond its bound (largest error {err})"
    return rd, err


def budget_tau_acceptable(tau_g: float, vals, wts, base: int, target: int, tau: float, lo: float, hi: float) -> bool:
    """Whether the threshold the GPU found is one the budget rule allows, given that the two sides know every
    similarity only to within BAND of each other. Either it lies in the oracle's own last interval (widened by
    BAND), or -- when values closer together than BAND straddle that interval's edge, e.g. a group of similarities
    that are exactly 1 in fp32 and 1 - 2e-16 for some of them in fp64 -- it is feasible and maximal under the
    band: everything surely below it fits the budget, and taking in the next value above it together with
    everything within BAND of that value would not."""
    if lo - BAND <= tau_g <= hi + BAND or tau_g == tau:
        return True
    v = np.asarray(vals, dtype=np.float64)
    w = np.asarray(wts, dtype=np.float64) if wts is not None else np.ones(len(v))
    if base + w[v <= tau_g - BAND].sum() > target:
        return False
    above = v[v > tau_g + BAND]
    if above.size == 0:
        return tau_g >= 1.0 - BAND or base + w.sum() <= target
    return base + w[v <= above.min() + BAND].sum() > target


def check_parity(lib, feats, r: GpuResult, *, tau_s=None, tau_t=None, keep=None, root_grid=1,
                 out_is_bf16=None, mode: str = "first_passing", order: str = "raster", out_is_f16: bool = False):
    """Full comparison; returns a dict with the error figures and near-threshold counts."""
    B, T, H, W, D = feats.shape
    if out_is_bf16 is None:
        out_is_bf16 = feats.dtype == np.uint16
    stats = O.spatial_stats(feats, root_grid, keep_means=False)
    info = {}
    ts = tau_s
    if tau_s is None:
        ts = r.tau_s.astype(np.float64)
        N1 = T * H * W
        for b, (vals, wts, base) in enumerate(O.spatial_budget_inputs(stats, B, T)):
            keep_b = float(np.broadcast_to(np.asarray(keep, dtype=np.float64), (B,))[b])
            target = int(math.floor(math.sqrt(keep_b) * N1))
            tau, lo, hi, K = O.budget_threshold(vals, wts, base, target)
            assert budget_tau_acceptable(ts[b], vals, wts, base, target, tau, lo, hi), \
                f"tau_s {ts[b]} outside the oracle's interval [{lo}, {hi})"
            assert len(np.unique(r.node_map[b])) <= target or base > target
        info["tau_s"] = ts
    sp, e1 = check_spatial(lib, feats, r, ts, root_grid, stats)
    cands, _ = O.temporal_candidates(feats, sp.node_map, sp.node_level)
    tt = tau_t
    if tau_t is None:
        tt = r.tau_t.astype(np.float64)
        N1 = T * H * W
        for b, (vals, wts, base) in enumerate(O.temporal_budget_inputs(cands, sp.node_map, mode)):
            keep_b = float(np.broadcast_to(np.asarray(keep, dtype=np.float64), (B,))[b])
            target = int(math.floor(keep_b * N1))
            tau, lo, hi, K = O.budget_threshold(vals, wts, base, target)
            assert budget_tau_acceptable(tt[b], vals, wts, base, target, tau, lo, hi), \
                f"tau_t {tt[b]} outside the oracle's interval [{lo}, {hi})"
            assert len(np.unique(r.cluster_ids[b])) <= target or base > target
        info["tau_t"] = tt
    tm, e2 = check_temporal(lib, feats, r, sp, tt, cands, mode)
    rd, e3 = check_reduce(feats, r, tm, out_is_bf16, order, out_is_f16)
    if hasattr(r, "survived"):
        info["merged_pos_err"] = check_positions(r, sp, tm, order)
    info.update(spatial_sim_err=e1, temporal_sim_err=e2, merged_err=e3, near_spatial=sp.near,
                near_temporal=tm.near, K=r.K, N=B * T * H * W, n_spatial=len(np.unique(sp.node_map)))
    return info
