"""The CPU oracle with its per-frame steps spread over processes -- TEST INFRASTRUCTURE ONLY.

Frames are independent in the pyramid / child-similarity steps (O1, O2; Sec. 3.2) and frame pairs in the candidate
step (O5; Sec. 3.3), so those two run in a pool of worker processes over contiguous ranges of frames; everything
that looks at a whole video (budget thresholds, decisions, edges and roots, the per-cluster means) runs serially in
the parent.  Every number comes out of the functions of ``oracle.sttm_oracle`` unchanged: this file only cuts the
frame axis and glues the pieces back together, and ``tests/test_oracle_pins.py`` checks that the result is the
serial one bit for bit.  Used by ``bench.py`` for its all-cores CPU baseline; the product path never imports it.
"""
from __future__ import annotations

import math
import multiprocessing as mp
from typing import List, Tuple

import numpy as np

from oracle import sttm_oracle as O

_FEATS = None      # the video tensor, inherited by forked workers (never pickled)
_MAPS = None       # (node_map, node_level) for the candidate step


def _limit_blas_threads():
    try:
        from threadpoolctl import threadpool_limits
        threadpool_limits(limits=1)
    except Exception:  # pragma: no cover
        pass


def _stats_range(args):
    b, t0, t1, root_grid = args
    grid, frames, ncmp = O.spatial_stats(_FEATS[b:b + 1, t0:t1], root_grid, keep_means=False)
    return b, t0, frames, ncmp


def _cands_range(args):
    """Candidates of the frames t0 <= t < t1 (t >= 1) of video b: the oracle's own routine on the window
    [t0 - 1, t1), with the flat indices of the window moved back to those of the whole tensor."""
    b, t0, t1 = args
    node_map, node_level = _MAPS
    B, T, H, W = node_map.shape
    HW = H * W
    first = (b * T + t0 - 1) * HW
    nm = node_map[b:b + 1, t0 - 1:t1] - first
    cands, ncmp = O.temporal_candidates(_FEATS[b:b + 1, t0 - 1:t1], nm, node_level[b:b + 1, t0 - 1:t1])
    return {n + first: [(d + first, s) for d, s in lst] for n, lst in cands.items()}, ncmp


def _ranges(T: int, parts: int, start: int = 0) -> List[Tuple[int, int]]:
    n = T - start
    parts = max(1, min(parts, n))
    cuts = [start + (n * i) // parts for i in range(parts + 1)]
    return [(cuts[i], cuts[i + 1]) for i in range(parts) if cuts[i + 1] > cuts[i]]


def sttm_parallel(feats: np.ndarray, tau_s=None, tau_t=None, keep=None, root_grid: int = 1,
                  mode: str = "first_passing", order: str = "raster", procs: int = 2):
    """Same arguments and results as ``sttm_oracle.sttm``; ``procs`` worker processes."""
    global _FEATS, _MAPS
    B, T, H, W, D = feats.shape
    _FEATS = feats
    ctx = mp.get_context("fork")
    per_video = max(1, procs // B) * 2          # a few ranges per worker so that the pool stays busy
    with ctx.Pool(procs, initializer=_limit_blas_threads) as pool:
        jobs = [(b, t0, t1, root_grid) for b in range(B) for t0, t1 in _ranges(T, per_video)]
        frames = [None] * (B * T)
        ncmp = 0
        for b, t0, part, c in pool.map(_stats_range, jobs):
            frames[b * T + t0:b * T + t0 + len(part)] = part
            ncmp += c
    stats = (O.Grid(H, W, root_grid), frames, ncmp)
    info = {}
    if tau_s is None:
        keep_b = np.broadcast_to(np.asarray(keep, dtype=np.float64), (B,))
        tau_s = []
        for b, (vals, wts, base) in enumerate(O.spatial_budget_inputs(stats, B, T)):
            target = int(math.floor(math.sqrt(keep_b[b]) * T * H * W))
            tau_s.append(O.budget_threshold(vals, wts, base, target)[0])
        info["tau_s"] = list(tau_s)
    sp = O.spatial_quadtree(feats, tau_s, root_grid, stats=stats)
    _MAPS = (sp.node_map, sp.node_level)
    cands, ncmp_t = {}, 0
    if T > 1:
        with ctx.Pool(procs, initializer=_limit_blas_threads) as pool:   # forked now: the workers see the maps
            jobs = [(b, t0, t1) for b in range(B) for t0, t1 in _ranges(T, per_video, start=1)]
            for part, c in pool.map(_cands_range, jobs):
                cands.update(part)
                ncmp_t += c
    cands = dict(sorted(cands.items()))
    if tau_t is None:
        keep_b = np.broadcast_to(np.asarray(keep, dtype=np.float64), (B,))
        tau_t = []
        for b, (vals, wts, base) in enumerate(O.temporal_budget_inputs(cands, sp.node_map, mode)):
            target = int(math.floor(keep_b[b] * T * H * W))
            tau_t.append(O.budget_threshold(vals, wts, base, target)[0])
        info["tau_t"] = list(tau_t)
    tm = O.temporal_merge(feats, sp.node_map, sp.node_level, tau_t, cands=cands, mode=mode)
    tm.comparisons = ncmp_t
    rd = O.reduce_clusters(feats, tm.cluster_ids, order)
    _FEATS = _MAPS = None
    return sp, tm, rd, info
