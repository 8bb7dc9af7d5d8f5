"""CPU oracle for spatio-temporal token merging -- TEST INFRASTRUCTURE ONLY.

A plain, slow, fp64 statement of what the merge path computes, written from
the paper (Sec. 3.2 spatial quadtree search, Sec. 3.3 directed temporal
merging, Sec. 3.4 output order) and used only by the tests, the smoke check
and the benchmark's ``cpu_baseline`` leg.  It shares no code with the HIP
library and the product path never calls it.

The method is a procedure, not an approximation of some closed form, so the
oracle takes the paper's steps in the paper's order:

  O1  pyramid of block means by repeated 2x2 pooling        (Sec. 3.2, "Building the quadtree", step 2)
  O2  cosine similarity between a node and each child        (Sec. 3.2, granularity decision)
  O3  coarse-to-fine search: keep a node iff all its child
      similarities exceed tau_S, else descend                (Sec. 3.2; Fig. "coarse-to-fine spatial search")
  O5  frame t node -> overlapping frame t-1 nodes, edge iff
      cosine > tau_T; several passing destinations => the
      one towards the top-left                               (Sec. 3.3)
  O6  common root of every chain of edges                    (Sec. 3.3, union-find)
  O8  one token per connected graph: the average             (Sec. 3.1 / 3.3)
  O10 linear order of the merged tokens and their position
      indices under the three strategies                     (Sec. 3.4, "Token Reordering after Merging")
  O9  thresholds from a token budget                         (Sec. 4.1 tunes them by hand; Sec. 5 names the
                                                              automatic search as future work -- the rule
                                                              here is this build's own reading)

Readings taken where the paper is silent (each is also listed in the design
notes of the repository):
  * thresholds are strict (">"), similarities are clamped to <= 1, so a
    threshold >= 1 is the identity;
  * a grid that is not a power of two is embedded top-left in the P x P grid,
    padded cells are excluded from sums, counts and the "all children" test;
  * a node's feature is the mean over its valid cells; zero-norm => sim 0;
  * "towards top-left" = smallest (y0, x0) in raster order;
  * temporal similarities use the spatial node means only (frame pairs are
    independent); the final token is the mean over the original member cells;
  * output rows are ordered by the root's (video, frame, y0, x0); with order="zscan" the spatial key inside a
    frame is the Z-shaped (Morton) rank of (y0, x0) instead of the raster one (Sec. 3.4 names a Z-shaped scan
    and gives earlier frames precedence: read as frame first, then the spatial scan inside the frame);
  * position indices (Sec. 3.4): "survived" = the original index of the root token, "reassigned" = the new
    index in the video's output order, "merged" = the mean of the member tokens' original indices (the
    index-level counterpart of averaging their rotary embeddings);
  * destination choice (Sec. 3.3 and the "Approximated Temporal Matching" ablation): "first_passing" tests
    every overlapping destination and takes the top-left-most passing one (default); "topleft_only" tests
    only the destination under the source's top-left cell; "most_similar" takes the passing destination with
    the highest similarity (ties: top-left-most).

Parity pins live in tests/ (library pooling/cosine on full grids, brute-force
enumeration of quadtree cuts, generic rectangle intersection, connected
components, closed-form invariants).  Against the authors' own implementation
the result is "parity unpinned": the paper prints no worked numerical example.
"""
from __future__ import annotations

import math
from typing import Callable, Dict, List, Optional, Sequence, Tuple

import numpy as np

BAND = 1e-5  # similarities this close to a threshold may be decided either way


# ----------------------------------------------------------------------------
# input handling
# ----------------------------------------------------------------------------
def widen(feats: np.ndarray) -> np.ndarray:
    """Exact widening of the stored input bits to float64 (float32, float16, or uint16 = bfloat16 bits)."""
    if feats.dtype == np.uint16:
        f32 = (feats.astype(np.uint32) << np.uint32(16)).view(np.float32)
        return f32.astype(np.float64)
    if feats.dtype in (np.float16, np.float32, np.float64):
        return feats.astype(np.float64)
    raise TypeError(f"unsupported input dtype {feats.dtype}")


def pow2_ceil(n: int) -> int:
    p = 1
    while p < n:
        p *= 2
    return p


class Grid:
    """Geometry of the dense quadtree over an H x W frame (Sec. 3.2).

    Level 0 is the finest (one cell per node); level ``L`` holds the
    ``root_grid x root_grid`` root nodes.  (The paper numbers levels the other
    way round: its "Lv.1" is the coarsest.)
    """

    def __init__(self, H: int, W: int, root_grid: int = 1):
        self.H, self.W = H, W
        self.P = pow2_ceil(max(H, W))
        if root_grid < 1 or (root_grid & (root_grid - 1)) or root_grid > self.P:
            raise ValueError("root_grid must be a power of two in [1, P]")
        self.R = root_grid
        self.L = int(math.log2(self.P // root_grid))

    def side(self, lvl: int) -> int:       # nodes per side at this level
        return self.P >> lvl

    def cells(self, lvl: int, by: int, bx: int) -> int:
        s = 1 << lvl
        h = max(0, min(self.H, (by + 1) * s) - by * s)
        w = max(0, min(self.W, (bx + 1) * s) - bx * s)
        return h * w

    def exists(self, lvl: int, by: int, bx: int) -> bool:
        return self.cells(lvl, by, bx) > 0


def cosine(a: np.ndarray, b: np.ndarray) -> float:
    """cos(a, b) clamped to <= 1; 0 when either vector has zero norm; NaN when an input holds a NaN or an infinity
    (such a similarity never exceeds a threshold)."""
    with np.errstate(invalid="ignore", over="ignore"):
        na = math.sqrt(float(np.dot(a, a)))
        nb = math.sqrt(float(np.dot(b, b)))
        if na == 0.0 or nb == 0.0:
            return 0.0
        c = float(np.dot(a, b)) / (na * nb)
    if c != c:
        return math.nan
    return min(1.0, c)


# ----------------------------------------------------------------------------
# O1 / O2: pyramid and parent-child similarities (Sec. 3.2)
# ----------------------------------------------------------------------------
def build_pyramid(frame: np.ndarray, grid: Grid):
    """Block means at every level by repeated 2x2 pooling of the level below.

    Returns (mean, cnt): ``mean[l]`` is [side, side, D] (zeros where the node
    does not exist), ``cnt[l]`` is the number of valid cells under each node.
    """
    H, W, D = frame.shape
    P = grid.P
    total = np.zeros((P, P, D), dtype=np.float64)
    total[:H, :W] = frame
    count = np.zeros((P, P), dtype=np.int64)
    count[:H, :W] = 1
    mean, cnt = [], []
    for lvl in range(grid.L + 1):
        if lvl > 0:
            g = grid.side(lvl)
            total = total.reshape(g, 2, g, 2, D).sum(axis=(1, 3))
            count = count.reshape(g, 2, g, 2).sum(axis=(1, 3))
        mu = np.zeros_like(total)
        nz = count > 0
        mu[nz] = total[nz] / count[nz][:, None]
        mean.append(mu)
        cnt.append(count.copy())
    return mean, cnt


def child_similarities(mean, cnt, grid: Grid, counter: Optional[List[int]] = None):
    """sigma(n, c) for every existing node n above the finest level and each existing child c.

    Returns ``sims``: sims[l] is [side, side, 4] (child order (dy,dx) = (0,0),(0,1),(1,0),(1,1);
    NaN for a child that does not exist) and ``m``: m[l][by,bx] = min over existing children.
    ``counter[0]`` is incremented once per comparison (Eq. (1) counts these).
    """
    sims: List[Optional[np.ndarray]] = [None]
    m: List[Optional[np.ndarray]] = [None]
    for lvl in range(1, grid.L + 1):
        g = grid.side(lvl)
        s = np.full((g, g, 4), np.nan)
        mm = np.full((g, g), np.nan)
        for by in range(g):
            for bx in range(g):
                if cnt[lvl][by, bx] == 0:
                    continue
                vals = []
                for k, (dy, dx) in enumerate(((0, 0), (0, 1), (1, 0), (1, 1))):
                    cy, cx = 2 * by + dy, 2 * bx + dx
                    if cnt[lvl - 1][cy, cx] == 0:
                        continue
                    s[by, bx, k] = cosine(mean[lvl][by, bx], mean[lvl - 1][cy, cx])
                    vals.append(s[by, bx, k])
                    if counter is not None:
                        counter[0] += 1
                mm[by, bx] = math.nan if any(v != v for v in vals) else min(vals)   # an undefined similarity splits
        sims.append(s)
        m.append(mm)
    return sims, m


# ----------------------------------------------------------------------------
# O3: coarse-to-fine search (Sec. 3.2)
# ----------------------------------------------------------------------------
def quadtree_search(m, grid: Grid, tau_s: float,
                    decide: Optional[Callable[[int, int, int, float], Optional[bool]]] = None):
    """Top-down granularity decision for one frame.

    A visited node is kept iff it is at the finest level or its smallest child
    similarity exceeds ``tau_s``; otherwise it is pruned and its existing
    children are visited.  Returns (top_left_y, top_left_x, level) maps over the
    H x W cells and the list of kept nodes [(lvl, by, bx)] in visiting order.

    ``decide(lvl, by, bx, m)`` may override a decision, but is consulted only
    when |m - tau_s| <= BAND (near-threshold protocol of the parity tests).
    """
    H, W = grid.H, grid.W
    ty = np.full((H, W), -1, dtype=np.int64)
    tx = np.full((H, W), -1, dtype=np.int64)
    lv = np.full((H, W), -1, dtype=np.int64)
    kept: List[Tuple[int, int, int]] = []
    near = [0]

    def visit(lvl, by, bx):
        if not grid.exists(lvl, by, bx):
            return
        keep = True
        if lvl > 0:
            val = float(m[lvl][by, bx])
            keep = val > tau_s
            if decide is not None and abs(val - tau_s) <= BAND:
                near[0] += 1
                forced = decide(lvl, by, bx, val)
                if forced is not None:
                    keep = bool(forced)
        if keep:
            s = 1 << lvl
            y0, x0 = by * s, bx * s
            ty[y0:min(H, y0 + s), x0:min(W, x0 + s)] = y0
            tx[y0:min(H, y0 + s), x0:min(W, x0 + s)] = x0
            lv[y0:min(H, y0 + s), x0:min(W, x0 + s)] = lvl
            kept.append((lvl, by, bx))
        else:
            for dy in (0, 1):
                for dx in (0, 1):
                    visit(lvl - 1, 2 * by + dy, 2 * bx + dx)

    for ry in range(grid.R):
        for rx in range(grid.R):
            visit(grid.L, ry, rx)
    return ty, tx, lv, kept, near[0]


def split_scores(m, grid: Grid):
    """s_n = max of m over the path from n's root down to n (n above the finest level).

    Node n is split at threshold tau iff s_n <= tau; returns a list of
    (s_n, number_of_existing_children) over all existing non-finest nodes.
    """
    out: List[Tuple[float, int]] = []

    def visit(lvl, by, bx, above):
        if lvl == 0 or not grid.exists(lvl, by, bx):
            return
        mv = float(m[lvl][by, bx])
        s = max(above, -2.0 if mv != mv else mv)          # an undefined m splits at every threshold
        kids = sum(grid.exists(lvl - 1, 2 * by + dy, 2 * bx + dx) for dy in (0, 1) for dx in (0, 1))
        out.append((s, kids))
        for dy in (0, 1):
            for dx in (0, 1):
                visit(lvl - 1, 2 * by + dy, 2 * bx + dx, s)

    for ry in range(grid.R):
        for rx in range(grid.R):
            visit(grid.L, ry, rx, -math.inf)
    return out


# ----------------------------------------------------------------------------
# O9: threshold for a token budget (this build's reading; Sec. 4.1 / Sec. 5)
# ----------------------------------------------------------------------------
def budget_threshold(values: Sequence[float], weights: Sequence[int], base: int, target: int):
    """Largest-interval rule.  K(tau) = base + sum_j weights[j] * [values[j] <= tau].

    Let b_0 < b_1 < ... be the distinct values carrying positive weight, b_-1 = -2.
    K is constant on [b_i, b_{i+1}); tau is the midpoint of the last such interval
    with K <= target; tau = 1 when even K(b_last) <= target, tau = -2 when K(-2) > target.
    Returns (tau, lo, hi, K(tau)) with [lo, hi) the interval tau was taken from.
    """
    vals = np.asarray(values, dtype=np.float64)
    wts = np.asarray(weights, dtype=np.int64)
    vals, wts = vals[wts > 0], wts[wts > 0]
    if base > target:
        return -2.0, -math.inf, (float(vals.min()) if len(vals) else math.inf), int(base)
    order = np.argsort(vals, kind="stable")
    vals, wts = vals[order], wts[order]
    b, start = np.unique(vals, return_index=True)
    w_at = np.add.reduceat(wts, start) if len(vals) else np.zeros(0, dtype=np.int64)
    K_at = base + np.cumsum(w_at)                       # K on [b_i, b_{i+1})
    ok = np.nonzero(K_at <= target)[0]
    i = int(ok[-1]) if len(ok) else -1
    if i == len(b) - 1:
        lo = float(b[-1]) if len(b) else -2.0
        return 1.0, lo, math.inf, int(K_at[-1]) if len(b) else int(base)
    lo = float(b[i]) if i >= 0 else -2.0
    hi = float(b[i + 1])
    return 0.5 * (lo + hi), lo, hi, int(K_at[i]) if i >= 0 else int(base)


# ----------------------------------------------------------------------------
# whole stages over [B, T, H, W, D]
# ----------------------------------------------------------------------------
class SpatialResult:
    def __init__(self):
        self.node_map = None      # int32 [B,T,H,W]: flat index of the kept node's top-left cell
        self.node_level = None    # uint8 [B,T,H,W]
        self.m = None             # list over frames of per-level m tables
        self.sims = None          # list over frames of per-level child similarity tables
        self.means = None         # list over frames of per-level mean tables (optional)
        self.kept = None          # list over frames of [(lvl, by, bx)]
        self.near = 0             # decisions within BAND of the threshold
        self.comparisons = 0


def spatial_stats(feats: np.ndarray, root_grid: int = 1, keep_means: bool = True):
    """O1 + O2 for every frame of every video.  Returns (grid, [per-frame (mean, cnt, sims, m)])."""
    B, T, H, W, D = feats.shape
    grid = Grid(H, W, root_grid)
    frames = []
    counter = [0]
    for b in range(B):
        for t in range(T):
            mean, cnt = build_pyramid(widen(feats[b, t]), grid)
            sims, m = child_similarities(mean, cnt, grid, counter)
            frames.append((mean if keep_means else None, cnt, sims, m))
    return grid, frames, counter[0]


def spatial_quadtree(feats: np.ndarray, tau_s, root_grid: int = 1, stats=None, decide=None) -> SpatialResult:
    """Steps O1-O3 (Sec. 3.2).  ``tau_s`` is a scalar or one value per video.

    ``decide(b, t, lvl, by, bx, m)`` is the optional near-threshold hook (see quadtree_search).
    """
    B, T, H, W, D = feats.shape
    tau = np.broadcast_to(np.asarray(tau_s, dtype=np.float64), (B,))
    grid, frames, ncmp = stats if stats is not None else spatial_stats(feats, root_grid)
    res = SpatialResult()
    res.node_map = np.empty((B, T, H, W), dtype=np.int32)
    res.node_level = np.empty((B, T, H, W), dtype=np.uint8)
    res.m = [f[3] for f in frames]
    res.sims = [f[2] for f in frames]
    res.means = [f[0] for f in frames]
    res.kept = []
    res.comparisons = ncmp
    for b in range(B):
        for t in range(T):
            f = b * T + t
            hook = None
            if decide is not None:
                hook = (lambda lvl, by, bx, val, b=b, t=t: decide(b, t, lvl, by, bx, val))
            ty, tx, lv, kept, near = quadtree_search(frames[f][3], grid, float(tau[b]), hook)
            res.node_map[b, t] = (f * H * W + ty * W + tx).astype(np.int32)
            res.node_level[b, t] = lv.astype(np.uint8)
            res.kept.append(kept)
            res.near += near
    return res


class TemporalResult:
    def __init__(self):
        self.parent = None        # int32 [B,T,H,W]: at a node's top-left cell the flat index of its
                                  # destination node's top-left cell, -1 for roots and non-top-left cells
        self.cluster_ids = None   # int32 [B,T,H,W]: flat index of the root node's top-left cell
        self.cands = None         # {source flat idx: [(dest flat idx, sigma), ...]} in raster order of dest
        self.e = None             # {source flat idx: max sigma over its candidates}
        self.near = 0
        self.comparisons = 0


def node_mean(feats_frame64: np.ndarray, y0: int, x0: int, lvl: int) -> np.ndarray:
    """Mean of the valid cells of the block (the kept node's token, Sec. 3.2 step 2)."""
    s = 1 << lvl
    blk = feats_frame64[y0:y0 + s, x0:x0 + s]
    return blk.reshape(-1, blk.shape[-1]).mean(axis=0)


def temporal_candidates(feats: np.ndarray, node_map: np.ndarray, node_level: np.ndarray):
    """sigma(n, d) for every kept node n of a frame t >= 1 and every kept node d of
    frame t-1 (same video) whose block overlaps n's block (Sec. 3.3).

    Returns {n: [(d, sigma)]} keyed by flat top-left indices, destinations in raster order,
    and the number of comparisons made.
    """
    B, T, H, W, D = feats.shape
    HW = H * W
    cands: Dict[int, List[Tuple[int, float]]] = {}
    ncmp = 0
    for b in range(B):
        prev64 = None
        for t in range(T):
            cur64 = widen(feats[b, t])
            if t > 0:
                f = b * T + t
                nm_t = node_map[b, t].astype(np.int64) - f * HW
                nm_p = node_map[b, t - 1].astype(np.int64) - (f - 1) * HW
                means_p: Dict[int, np.ndarray] = {}
                for n_loc in np.unique(nm_t):
                    y0, x0 = divmod(int(n_loc), W)
                    lvl = int(node_level[b, t, y0, x0])
                    s = 1 << lvl
                    mu_n = node_mean(cur64, y0, x0, lvl)
                    dests = np.unique(nm_p[y0:y0 + s, x0:x0 + s])
                    lst = []
                    for d_loc in dests:
                        d_loc = int(d_loc)
                        if d_loc not in means_p:
                            dy, dx = divmod(d_loc, W)
                            means_p[d_loc] = node_mean(prev64, dy, dx, int(node_level[b, t - 1, dy, dx]))
                        lst.append(((f - 1) * HW + d_loc, cosine(mu_n, means_p[d_loc])))
                        ncmp += 1
                    cands[f * HW + int(n_loc)] = lst
            prev64 = cur64
    return cands, ncmp


MATCH_MODES = ("first_passing", "topleft_only", "most_similar")


def best_similarity(cands, node_map: np.ndarray, mode: str = "first_passing"):
    """e_n: the similarity that decides whether node n merges at all -- the largest one over its candidates,
    or, when only the destination under n's top-left cell is tested, that destination's."""
    B, T, H, W = node_map.shape
    HW = H * W
    flat = node_map.reshape(-1)
    e = {}
    for n, lst in cands.items():
        if mode == "topleft_only":
            d0 = int(flat[n - HW])            # the kept node of frame t-1 covering n's top-left cell
            e[n] = dict(lst)[d0]
            if e[n] != e[n]:
                e[n] = -2.0
        else:
            e[n] = max([s for _, s in lst if s == s], default=-2.0)   # undefined similarities never link
    return e


def temporal_merge(feats: np.ndarray, node_map: np.ndarray, node_level: np.ndarray, tau_t,
                   cands=None, decide=None, mode: str = "first_passing", choose=None) -> TemporalResult:
    """Steps O5-O7 (Sec. 3.3): directed edges to the previous frame, then the common root of every chain.

    ``mode`` picks the destination among several overlapping ones (see MATCH_MODES).
    ``decide(n, d, sigma)`` is the near-threshold hook, consulted only when |sigma - tau_t| <= BAND.
    ``choose(n, passing)`` (most_similar only) is consulted when another passing destination comes within BAND
    of the best one; it returns the destination to take, or None.
    """
    assert mode in MATCH_MODES
    B, T, H, W, D = feats.shape
    HW = H * W
    tau = np.broadcast_to(np.asarray(tau_t, dtype=np.float64), (B,))
    res = TemporalResult()
    if cands is None:
        cands, res.comparisons = temporal_candidates(feats, node_map, node_level)
    res.cands = cands
    res.e = best_similarity(cands, node_map, mode)
    parent = np.full(B * T * HW, -1, dtype=np.int64)
    flat_map = node_map.reshape(-1)

    def passes(n, b, d, sig):
        ok = sig > tau[b]
        if decide is not None and abs(sig - tau[b]) <= BAND:
            res.near += 1
            forced = decide(n, d, sig)
            if forced is not None:
                ok = bool(forced)
        return ok

    for n, lst in cands.items():
        b = n // (T * HW)
        ordered = sorted(lst)                      # raster order = ascending flat index
        if mode == "first_passing":
            for d, sig in ordered:
                if passes(n, b, d, sig):
                    parent[n] = d
                    break
        elif mode == "topleft_only":
            d0 = int(flat_map[n - HW])
            sig = dict(lst)[d0]
            if passes(n, b, d0, sig):
                parent[n] = d0
        else:
            ok = [(d, sig) for d, sig in ordered if passes(n, b, d, sig)]
            if ok:
                top = max(sig for _, sig in ok)
                pick = min(d for d, sig in ok if sig == top)
                if choose is not None and sum(1 for _, sig in ok if sig >= top - BAND) > 1:
                    res.near += 1
                    forced = choose(n, [(d, sig) for d, sig in ok if sig >= top - BAND])
                    if forced is not None:
                        pick = int(forced)
                parent[n] = pick
    res.parent = parent.reshape(B, T, H, W).astype(np.int32)
    flat_nodes = node_map.reshape(-1).astype(np.int64)
    root_of: Dict[int, int] = {}
    for n in np.unique(flat_nodes):                # ascending => parents (earlier frame) come first
        n = int(n)
        r = n
        while parent[r] >= 0:                      # O6: follow the edges to the common root
            r = int(parent[r])
            if r in root_of:
                r = root_of[r]
                break
        root_of[n] = r
    lut = np.zeros(B * T * HW, dtype=np.int64)
    for n, r in root_of.items():
        lut[n] = r
    res.cluster_ids = lut[flat_nodes].reshape(B, T, H, W).astype(np.int32)
    return res


class ReduceResult:
    def __init__(self):
        self.merged = None    # float64 [K, D]
        self.counts = None    # int32 [K]
        self.out_ids = None   # int32 [K] cluster id (= root top-left flat index), ascending
        self.offsets = None   # int64 [B+1]


def zscan_rank(y: int, x: int) -> int:
    """Rank of cell (y, x) in the Z-shaped scan of a power-of-two grid (Sec. 3.4): quadrant by quadrant,
    top-left, top-right, bottom-left, bottom-right, recursively -- the bits of y and x interleaved, x lowest."""
    z = 0
    bit = 0
    while (y >> bit) or (x >> bit):
        z |= ((x >> bit) & 1) << (2 * bit)
        z |= ((y >> bit) & 1) << (2 * bit + 1)
        bit += 1
    return z


def output_order(out_ids, shape, order: str = "raster"):
    """Permutation of the clusters (given by their ids = flat index of the root's top-left cell) into the
    linear order of Sec. 3.4: earlier frames first, inside a frame the spatial scan of the root's top-left."""
    B, T, H, W = shape
    assert order in ("raster", "zscan")

    def key(cid):
        f, c = divmod(int(cid), H * W)
        y, x = divmod(c, W)
        return (f, y * W + x) if order == "raster" else (f, zscan_rank(y, x))

    return sorted(range(len(out_ids)), key=lambda k: key(out_ids[k]))


def reduce_clusters(feats: np.ndarray, cluster_ids: np.ndarray, order: str = "raster") -> ReduceResult:
    """Step O8: one output token per cluster = mean over its member cells, rows in the order of Sec. 3.4
    (video, frame, spatial scan of the root's top-left; raster = ascending cluster id)."""
    B, T, H, W, D = feats.shape
    N = B * T * H * W
    flat = cluster_ids.reshape(-1).astype(np.int64)
    out_ids = np.unique(flat)
    out_ids = out_ids[output_order(out_ids, (B, T, H, W), order)]
    members: Dict[int, List[int]] = {int(k): [] for k in out_ids}
    for i in range(N):
        members[int(flat[i])].append(i)
    rows = feats.reshape(N, D)
    res = ReduceResult()
    res.merged = np.empty((len(out_ids), D), dtype=np.float64)
    res.counts = np.empty(len(out_ids), dtype=np.int32)
    for k, cid in enumerate(out_ids):
        cells = members[int(cid)]
        res.merged[k] = widen(rows[cells]).sum(axis=0) / len(cells)
        res.counts[k] = len(cells)
    res.out_ids = out_ids.astype(np.int32)
    res.offsets = np.array([int((out_ids < b * T * H * W).sum()) for b in range(B + 1)], dtype=np.int64)
    return res


class PositionResult:
    def __init__(self):
        self.survived = None    # int32 [K]: original index (within the video) of the surviving root token
        self.reassigned = None  # int32 [K]: index of the row in the video's output sequence
        self.merged = None      # float64 [K]: mean original index of the member tokens
        self.root = None        # int32 [K, 4]: (t, y0, x0, level) of the root node


def positions(cluster_ids: np.ndarray, node_level: np.ndarray, order: str = "raster") -> PositionResult:
    """Step O10 (Sec. 3.4): position indices of the output rows under the three strategies the paper
    evaluates, plus the root's (t, y, x) for encodings built on those coordinates."""
    B, T, H, W = cluster_ids.shape
    N1 = T * H * W
    flat = cluster_ids.reshape(-1).astype(np.int64)
    out_ids = np.unique(flat)
    out_ids = out_ids[output_order(out_ids, (B, T, H, W), order)]
    res = PositionResult()
    K = len(out_ids)
    res.survived = np.empty(K, dtype=np.int32)
    res.reassigned = np.empty(K, dtype=np.int32)
    res.merged = np.empty(K, dtype=np.float64)
    res.root = np.empty((K, 4), dtype=np.int32)
    seen = [0] * B
    lv = node_level.reshape(-1)
    for k, cid in enumerate(out_ids):
        cid = int(cid)
        b, loc = divmod(cid, N1)
        t, c = divmod(loc, H * W)
        y0, x0 = divmod(c, W)
        res.survived[k] = loc
        res.reassigned[k] = seen[b]
        seen[b] += 1
        cells = np.nonzero(flat == cid)[0]
        res.merged[k] = float((cells - b * N1).sum()) / len(cells)
        res.root[k] = (t, y0, x0, int(lv[cid]))
    return res


# ----------------------------------------------------------------------------
# budget mode (O9) on top of the stages
# ----------------------------------------------------------------------------
def spatial_budget_inputs(stats, B: int, T: int):
    """Per video: (values s_n, weights c_n - 1, base = number of root nodes)."""
    grid, frames, _ = stats
    out = []
    for b in range(B):
        vals, wts, base = [], [], 0
        for t in range(T):
            m = frames[b * T + t][3]
            for s, kids in split_scores(m, grid):
                vals.append(s)
                wts.append(kids - 1)
            base += sum(grid.exists(grid.L, ry, rx) for ry in range(grid.R) for rx in range(grid.R))
        out.append((vals, wts, base))
    return out


def temporal_budget_inputs(cands, node_map: np.ndarray, mode: str = "first_passing"):
    """Per video: (values e_n over nodes of frames >= 1, weights 1, base = nodes of frame 0)."""
    B, T, H, W = node_map.shape
    out = []
    e = best_similarity(cands, node_map, mode)
    for b in range(B):
        n_nodes = len(np.unique(node_map[b]))
        lo, hi = b * T * H * W, (b + 1) * T * H * W
        vals = [e[n] for n in cands if lo <= n < hi]
        out.append((vals, [1] * len(vals), n_nodes - len(vals)))
    return out


def sttm(feats: np.ndarray, tau_s=None, tau_t=None, keep=None, root_grid: int = 1, mode: str = "first_passing",
         order: str = "raster"):
    """The whole path.  Either fixed thresholds, or ``keep`` (fraction of each video's
    T*H*W tokens to retain): sqrt(keep) after the spatial stage, keep after the temporal one."""
    B, T, H, W, D = feats.shape
    stats = spatial_stats(feats, root_grid, keep_means=False)
    info = {}
    if tau_s is None:
        keep_b = np.broadcast_to(np.asarray(keep, dtype=np.float64), (B,))
        tau_s = []
        for b, (vals, wts, base) in enumerate(spatial_budget_inputs(stats, B, T)):
            target = int(math.floor(math.sqrt(keep_b[b]) * T * H * W))
            tau_s.append(budget_threshold(vals, wts, base, target)[0])
        info["tau_s"] = list(tau_s)
    sp = spatial_quadtree(feats, tau_s, root_grid, stats=stats)
    cands, ncmp = temporal_candidates(feats, sp.node_map, sp.node_level)
    if tau_t is None:
        keep_b = np.broadcast_to(np.asarray(keep, dtype=np.float64), (B,))
        tau_t = []
        for b, (vals, wts, base) in enumerate(temporal_budget_inputs(cands, sp.node_map, mode)):
            target = int(math.floor(keep_b[b] * T * H * W))
            tau_t.append(budget_threshold(vals, wts, base, target)[0])
        info["tau_t"] = list(tau_t)
    tm = temporal_merge(feats, sp.node_map, sp.node_level, tau_t, cands=cands, mode=mode)
    tm.comparisons = ncmp
    rd = reduce_clusters(feats, tm.cluster_ids, order)
    return sp, tm, rd, info
