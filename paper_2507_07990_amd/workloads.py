"""Seeded synthetic video-token workloads.

This module only *draws inputs*: block-structured random features whose
shapes follow the paper's workloads (Sec. 4.1: frames sampled at 1 FPS, a
square grid of visual tokens per frame, channels = hidden width of the host
LLM).  It contains none of the merging method's arithmetic, so both the CPU
oracle's tests and the HIP path's tests may import it.

Recipe (per video)
------------------
* Frame 0: a random quadtree over the P x P grid (P = power of two >=
  max(H, W)), grown from one root; every node splits with probability
  ``p_split`` until ``max_depth``.  Every leaf block owns a base vector
  ~ N(0, I_D).  A token is its leaf's base plus ``sigma * N(0, I_D)`` noise
  drawn fresh per token per frame.  Only the H x W valid cells are emitted.
* Frame t: every leaf of frame t-1 persists (same block, same base) with
  probability ``persist``; otherwise its block is regrown as a fresh random
  quadtree with the depth that remains.  If all four siblings were regrown
  in the same frame their parent block is regrown instead (this lets the
  partition coarsen).  A scene cut regrows the whole frame from the root.
* dtype "bf16": values are rounded to bfloat16 (round-to-nearest-even) and
  returned as raw uint16 bit patterns; "f16": numpy float16; "f32": float32.
"""
from __future__ import annotations

import dataclasses
from typing import List, Optional, Tuple

import numpy as np


@dataclasses.dataclass(frozen=True)
class Workload:
    name: str
    seed: int
    B: int
    T: int
    H: int
    W: int
    D: int
    dtype: str                 # "f32" | "bf16" | "f16"
    max_depth: int
    sigma: float               # noise std (per-video range if sigma_hi set)
    persist: float             # leaf persistence prob (range if persist_hi set)
    p_split: float = 0.5
    cut_prob: float = 0.0      # per-frame scene-cut probability
    cut_mean_gap: float = 0.0  # >0: exponential gaps between cuts (mean, frames)
    sigma_hi: Optional[float] = None
    persist_hi: Optional[float] = None
    tau_s: Optional[float] = None     # fixed thresholds, or None => budget mode
    tau_t: Optional[float] = None
    budgets: Tuple[float, ...] = ()   # target keep fractions in budget mode
    root_grid: int = 1                # root nodes per side of the quadtree

    @property
    def n_tokens(self) -> int:
        return self.B * self.T * self.H * self.W


# The configurations this build is measured and parity-tested on: the five the benchmark definition names, then
# two shapes taken from the paper's own set-up (Sec. 4.1 / 4.3): its 14 x 14 grid with 4 x 4 root nodes at up to
# 180 frames, and a wide-channel, non-square grid (a 72B host model's hidden width on a dynamic-resolution encoder).
CONFIGS: List[Workload] = [
    Workload("tiny", 0, 1, 8, 8, 8, 64, "f32", 3, 0.05, 0.7, tau_s=0.8, tau_t=0.8),
    Workload("short_clip", 1, 1, 64, 13, 13, 3584, "bf16", 4, 0.1, 0.8, budgets=(0.5,)),
    Workload("encoder_width", 2, 1, 64, 16, 16, 1152, "bf16", 4, 0.15, 0.6,
             cut_prob=0.1, budgets=(0.3,)),
    Workload("long_video", 3, 1, 512, 13, 13, 3584, "bf16", 4, 0.1, 0.9,
             cut_mean_gap=64.0, budgets=(0.5, 0.3)),
    Workload("batched_unpooled", 4, 32, 32, 27, 27, 1152, "bf16", 5, 0.05, 0.3,
             sigma_hi=0.3, persist_hi=0.95, tau_s=0.9, tau_t=0.85),
    Workload("paper_grid", 5, 1, 180, 14, 14, 3584, "bf16", 4, 0.1, 0.9, cut_mean_gap=64.0,
             budgets=(0.5, 0.3), root_grid=4),
    Workload("wide_nonsquare", 6, 1, 180, 18, 24, 8192, "bf16", 5, 0.1, 0.9, cut_mean_gap=64.0,
             budgets=(0.5, 0.3)),
]


def pow2_ceil(n: int) -> int:
    p = 1
    while p < n:
        p *= 2
    return p


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (nearest, ties to even); returns uint16 bits."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = u + np.uint32(0x7FFF) + lsb
    return (r >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Exact widening of bfloat16 bit patterns to float32."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


class _Leaf:
    __slots__ = ("y0", "x0", "size", "base")

    def __init__(self, y0, x0, size, base):
        self.y0, self.x0, self.size, self.base = y0, x0, size, base


class _Split:
    __slots__ = ("y0", "x0", "size", "kids")

    def __init__(self, y0, x0, size, kids):
        self.y0, self.x0, self.size, self.kids = y0, x0, size, kids


class _VideoState:
    """Evolving block partition of one video; bases are drawn on demand."""

    def __init__(self, rng: np.random.Generator, P: int, max_depth: int, p_split: float, D: int):
        self.rng, self.P, self.max_depth, self.p_split, self.D = rng, P, max_depth, p_split, D
        self.bases = {}          # leaf uid -> base vector (only live leaves are kept)
        self.next_uid = 0

    def _new_base(self) -> int:
        uid = self.next_uid
        self.next_uid += 1
        self.bases[uid] = self.rng.standard_normal(self.D, dtype=np.float32)
        return uid

    def grow(self, y0: int, x0: int, size: int, depth: int):
        if depth < self.max_depth and size > 1 and self.rng.random() < self.p_split:
            h = size // 2
            kids = [self.grow(y0 + dy * h, x0 + dx * h, h, depth + 1) for dy in (0, 1) for dx in (0, 1)]
            return _Split(y0, x0, size, kids)
        return _Leaf(y0, x0, size, self._new_base())

    def evolve(self, node, depth: int, persist: float):
        """Returns (new_node, regrown_flag)."""
        if isinstance(node, _Leaf):
            if self.rng.random() < persist:
                return node, False
            return self.grow(node.y0, node.x0, node.size, depth), True
        out = [self.evolve(k, depth + 1, persist) for k in node.kids]
        if all(flag for _, flag in out):
            return self.grow(node.y0, node.x0, node.size, depth), True
        return _Split(node.y0, node.x0, node.size, [n for n, _ in out]), False

    def leaves(self, node, acc):
        if isinstance(node, _Leaf):
            acc.append(node)
        else:
            for k in node.kids:
                self.leaves(k, acc)
        return acc


def generate(cfg: Workload, *, return_leaf_maps: bool = False):
    """Draw the features of ``cfg``.

    Returns ``feats`` with shape [B, T, H, W, D]: float32 for dtype "f32",
    uint16 bfloat16 bit patterns for "bf16".  With ``return_leaf_maps`` also
    returns an int32 [B, T, H, W] array holding, per cell, a per-video id of
    the generator leaf that produced it (for planted-structure tests).
    """
    rng = np.random.Generator(np.random.Philox(cfg.seed))
    P = pow2_ceil(max(cfg.H, cfg.W))
    out_dtype = {"f32": np.float32, "bf16": np.uint16, "f16": np.float16}[cfg.dtype]
    feats = np.empty((cfg.B, cfg.T, cfg.H, cfg.W, cfg.D), dtype=out_dtype)
    leaf_maps = np.empty((cfg.B, cfg.T, cfg.H, cfg.W), dtype=np.int32) if return_leaf_maps else None
    for b in range(cfg.B):
        sigma = cfg.sigma if cfg.sigma_hi is None else float(rng.uniform(cfg.sigma, cfg.sigma_hi))
        persist = cfg.persist if cfg.persist_hi is None else float(rng.uniform(cfg.persist, cfg.persist_hi))
        st = _VideoState(rng, P, cfg.max_depth, cfg.p_split, cfg.D)
        root = None
        next_cut = None
        if cfg.cut_mean_gap > 0:
            next_cut = int(np.ceil(rng.exponential(cfg.cut_mean_gap)))
        for t in range(cfg.T):
            cut = root is None
            if not cut and cfg.cut_prob > 0 and rng.random() < cfg.cut_prob:
                cut = True
            if not cut and next_cut is not None and t >= next_cut:
                cut = True
                next_cut = t + max(1, int(np.ceil(rng.exponential(cfg.cut_mean_gap))))
            if cut:
                root = st.grow(0, 0, P, 0)
            else:
                root, _ = st.evolve(root, 0, persist)
            ids = np.zeros((P, P), dtype=np.int32)
            live = st.leaves(root, [])
            for lf in live:
                ids[lf.y0:lf.y0 + lf.size, lf.x0:lf.x0 + lf.size] = lf.base
            st.bases = {lf.base: st.bases[lf.base] for lf in live}
            ids = ids[:cfg.H, :cfg.W]
            uniq = np.unique(ids)
            base_rows = np.stack([st.bases[int(i)] for i in uniq])
            remap = np.searchsorted(uniq, ids)
            frame = base_rows[remap]                                   # [H, W, D] float32
            frame = frame + np.float32(sigma) * rng.standard_normal(frame.shape, dtype=np.float32)
            feats[b, t] = f32_to_bf16_bits(frame) if cfg.dtype == "bf16" else frame   # (float16: numpy rounds)
            if leaf_maps is not None:
                leaf_maps[b, t] = ids
    if return_leaf_maps:
        return feats, leaf_maps
    return feats


def generate_alternating(cfg: Workload, sigma_fine: float) -> np.ndarray:
    """The features of ``cfg`` with the noise of every odd frame raised to ``sigma_fine``.

    With a spatial threshold between the two noise levels the even frames merge into coarse nodes and the odd
    frames stay fine, so consecutive frames meet at different granularities in both directions (a coarse node
    over several fine destinations and the reverse) and the similarities of one coarse node to its fine
    destinations spread out: the inputs on which the destination-choice rules of the temporal stage differ."""
    base = generate(dataclasses.replace(cfg, sigma=0.0, sigma_hi=None, dtype="f32"))
    rng = np.random.Generator(np.random.Philox(cfg.seed + 7919))
    out = np.empty_like(base)
    for t in range(cfg.T):
        s = np.float32(sigma_fine if t % 2 else cfg.sigma)
        out[:, t] = base[:, t] + s * rng.standard_normal(base[:, t].shape, dtype=np.float32)
    if cfg.dtype == "bf16":
        return f32_to_bf16_bits(out)
    return out.astype(np.float16) if cfg.dtype == "f16" else out


def small_variant(cfg: Workload, **over) -> Workload:
    """Same recipe at other sizes (used by parity tests for tiles and ragged tails)."""
    return dataclasses.replace(cfg, **over)
