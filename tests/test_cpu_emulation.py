"""The library's kernels compiled for host threads (tests/cpu_emul) against the oracle, on the CPU.

Not a product path: the stand-in runs one OS thread per GPU thread so that the control flow, indexing and
synchronisation of the kernels can be exercised (and debugged with host tools) where there is no GPU."""
import math
import shutil

import numpy as np
import pytest

from paper_2507_07990_amd import workloads as wl
from tests import parity as P

pytestmark = pytest.mark.skipif(shutil.which("g++") is None, reason="needs g++")


class _EmulLib:
    STTM_BF16, STTM_F32, STTM_F16 = 1, 0, 2

    def __init__(self, rc):
        self._lib = rc.load()
        self._lib.sttm_node_index.restype = int

    def sttm_node_index(self, H, W, R, lvl, by, bx):
        return self._lib.sttm_node_index(H, W, R, lvl, by, bx)


@pytest.fixture(scope="module")
def emul():
    from tests.cpu_emul import build_cpu, run_cpu
    build_cpu.build()
    return run_cpu, _EmulLib(run_cpu)


def _variant(seed, B, T, H, W, D, dtype):
    depth = int(math.log2(wl.pow2_ceil(max(H, W))))
    return wl.Workload("v", seed, B, T, H, W, D, dtype, depth, 0.1, 0.7)


@pytest.mark.parametrize("seed,B,T,H,W,D,dtype,kw", [
    (90, 1, 3, 8, 8, 16, "f32", dict(tau_s=0.8, tau_t=0.8)),
    (91, 2, 3, 5, 6, 24, "bf16", dict(keep=0.5)),
    (92, 1, 2, 9, 9, 16, "bf16", dict(tau_s=0.2, tau_t=0.2)),   # nodes that the reduce takes from stored sums
    (93, 1, 3, 8, 8, 24, "f16", dict(tau_s=0.7, tau_t=0.7)),    # half-precision input and output
    (94, 1, 2, 17, 18, 16, "f32", dict(tau_s=0.3, tau_t=0.3)),  # P = 32: two pyramid levels above the 8x8 units
    (97, 2, 3, 14, 14, 24, "bf16", dict(tau_s=0.8, tau_t=0.7, root_grid=4)),  # 4x4 roots: 4x4 join blocks everywhere
    (96, 1, 150, 2, 2, 8, "f32", dict(tau_s=1.0, tau_t=-2.0)),  # four chains of 150 cells: clusters summed item by item
])
def test_emulated_kernels_match_the_oracle(emul, seed, B, T, H, W, D, dtype, kw):
    run_cpu, fake = emul
    feats = wl.generate(_variant(seed, B, T, H, W, D, dtype))
    r = run_cpu.run_cpu(feats, **kw)
    info = P.check_parity(fake, feats, r, **kw)
    assert info["K"] == r.K and int(r.counts.sum()) == feats[..., 0].size


@pytest.mark.parametrize("mode,order", [("topleft_only", "zscan"), ("most_similar", "raster"), ("first_passing", "zscan")])
def test_emulated_destination_rules_orders_and_positions(emul, mode, order):
    """Alternating coarse / fine frames (the rules differ there), rows in either scan, position indices."""
    run_cpu, fake = emul
    cfg = wl.Workload("v", 95, 1, 5, 8, 8, 16, "f32", 2, 0.05, 0.9)
    feats = wl.generate_alternating(cfg, 0.7)
    kw = dict(tau_s=0.9, tau_t=0.8)
    r = run_cpu.run_cpu(feats, match=P.MODES[mode], order=P.ORDERS[order], positions=True, **kw)
    info = P.check_parity(fake, feats, r, mode=mode, order=order, **kw)
    assert "merged_pos_err" in info


def test_emulated_budget_threshold_left_to_the_consumer_kernels(emul):
    """Without a host pointer for the threshold the last digit of the search is resolved by the kernels that use it:
    same partition, same clusters, same rows."""
    run_cpu, fake = emul
    feats = wl.generate(_variant(91, 2, 3, 5, 6, 24, "bf16"))
    a = run_cpu.run_cpu(feats, keep=0.5)
    b = run_cpu.run_cpu(feats, keep=0.5, defer_tau=True)
    assert (a.node_map == b.node_map).all() and (a.cluster_ids == b.cluster_ids).all()
    assert (a.parent == b.parent).all() and a.K == b.K
    np.testing.assert_array_equal(a.merged, b.merged)


@pytest.mark.parametrize("kw", [dict(keep=0.5), dict(tau_s=0.95, tau_t=0.6)])
def test_emulated_temporal_pass_without_the_cell_dot_products(emul, kw):
    """With the option off the temporal pass computes every pair itself: same partition and clusters as with the
    cell-to-cell dot products of the spatial pass, and parity with the oracle either way."""
    run_cpu, fake = emul
    feats = wl.generate(_variant(98, 2, 4, 9, 7, 24, "bf16"))
    a = run_cpu.run_cpu(feats, **kw)
    for level in (0, 2):
        b = run_cpu.run_cpu(feats, cell_dots=level, **kw)
        assert (a.node_map == b.node_map).all() and (a.cluster_ids == b.cluster_ids).all() and a.K == b.K
        P.check_parity(fake, feats, b, **kw)
    P.check_parity(fake, feats, a, **kw)


def _uniform_partition(T, H, W, levels):
    """Node map and levels of a video whose frame t consists of the aligned blocks of level levels[t] only."""
    nm = np.empty((1, T, H, W), np.int32)
    nl = np.empty((1, T, H, W), np.uint8)
    yy, xx = np.meshgrid(np.arange(H), np.arange(W), indexing="ij")
    for t, lv in enumerate(levels):
        nm[0, t] = t * H * W + ((yy >> lv) << lv) * W + ((xx >> lv) << lv)
        nl[0, t] = lv
    return nm, nl


def test_emulated_temporal_work_lists_at_their_largest(emul):
    """The temporal pass lists its work per frame pair by join level and walks every list with a fixed stride and
    a trip count known on entry. On a full 32 x 32 grid, frames of uniform level meet so that every list is as long
    as it can get: 256 regions of 2 x 2 (levels 0|1), 64 blocks of 4 x 4 (1|2 and 2|0), 16 staged sums with 256
    nodes of 2 x 2 under them (3|1), and 1024 single cells under one whole-frame node (5|0) or under sixteen
    8 x 8 nodes (0|3). Every pair similarity, edge, cluster and merged row is compared with the oracle."""
    run_cpu, fake = emul
    levels = [5, 0, 3, 1, 2, 0, 1]
    T, H, W, D = len(levels), 32, 32, 8
    feats = wl.generate(wl.Workload("v", 99, 1, T, H, W, D, "f32", 5, 0.3, 0.8))
    nm, nl = _uniform_partition(T, H, W, levels)
    from oracle import sttm_oracle as O
    sp = O.SpatialResult()
    sp.node_map, sp.node_level = nm, nl
    r = run_cpu.run_cpu(feats, tau_s=0.5, tau_t=0.3, node_map_override=(nm, nl))
    tm, _ = P.check_temporal(fake, feats, r, sp, 0.3)
    P.check_reduce(feats, r, tm, False)


def test_emulated_kernels_run_clean_under_address_and_undefined_behaviour_sanitizers():
    """The host-thread build with -fsanitize=address,undefined (any report aborts): both dtypes, fixed thresholds and
    a budget, every output in a heap block of its exact size, the workspace of exactly sttm_workspace_bytes()."""
    import subprocess
    from tests.cpu_emul import build_cpu
    exe = build_cpu.build_sanitized()
    r = subprocess.run([exe], capture_output=True, text=True, timeout=600)
    assert r.returncode == 0, (r.stdout[-2000:], r.stderr[-4000:])
    assert r.stdout.count("case ") == 2
    assert "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr
