"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on seeded inputs."""
import dataclasses
import math

import numpy as np
import pytest

from paper_2507_07990_amd import workloads as wl
from tests import parity as P
from oracle import sttm_oracle as O

pytestmark = pytest.mark.gpu


def _variant(seed, B, T, H, W, D, dtype, **kw):
    depth = int(math.log2(wl.pow2_ceil(max(H, W))))
    base = dict(sigma=0.1, persist=0.7)
    base.update(kw)
    return wl.Workload("v", seed, B, T, H, W, D, dtype, depth, base.pop("sigma"), base.pop("persist"), **base)


def _run_and_check(lib, cfg, *, tau_s=None, tau_t=None, keep=None, root_grid=1, out_dtype=None, cell_dots=1):
    feats = wl.generate(cfg)
    print(f"case {cfg.name} seed={cfg.seed} shape={feats.shape} dtype={feats.dtype} tau=({tau_s},{tau_t}) "
          f"keep={keep} R={root_grid} cell_dots={cell_dots}", flush=True)
    r = P.run_gpu(lib, feats, tau_s=tau_s, tau_t=tau_t, keep=keep, root_grid=root_grid, out_dtype=out_dtype,
                  cell_dots=cell_dots)
    out_bf16 = (out_dtype == lib.STTM_BF16) if out_dtype is not None else None
    info = P.check_parity(lib, feats, r, tau_s=tau_s, tau_t=tau_t, keep=keep, root_grid=root_grid,
                          out_is_bf16=out_bf16, out_is_f16=out_dtype == lib.STTM_F16)
    print("  ", {k: (float(v) if isinstance(v, (float, np.floating)) else v) for k, v in info.items()
                 if k not in ("tau_s", "tau_t")}, flush=True)
    return feats, r, info


def test_config0_tiny_fixed_thresholds(lib):
    cfg = wl.CONFIGS[0]
    feats, r, info = _run_and_check(lib, cfg, tau_s=cfg.tau_s, tau_t=cfg.tau_t)
    assert info["near_spatial"] == 0 and info["near_temporal"] == 0   # unguided oracle agrees bit for bit
    sp, tm, rd, _ = O.sttm(feats, tau_s=cfg.tau_s, tau_t=cfg.tau_t)
    assert (tm.cluster_ids == r.cluster_ids).all()


@pytest.mark.parametrize("seed,B,T,H,W,D,dtype,tau_s,tau_t,R", [
    (10, 1, 5, 13, 13, 200, "bf16", 0.9, 0.8, 1),     # ragged channel chunk, padded grid
    (11, 2, 4, 16, 16, 520, "bf16", 0.8, 0.9, 1),     # two chunks, second almost empty; two videos
    (12, 1, 3, 27, 27, 72, "f32", 0.85, 0.7, 1),      # P = 32: five levels
    (13, 1, 4, 14, 14, 264, "f32", 0.8, 0.8, 2),      # the paper's 14x14 grid, 2x2 roots
    (14, 1, 4, 14, 14, 64, "bf16", 0.7, 0.8, 4),      # 4x4 roots (the paper's adopted scale)
    (15, 1, 6, 9, 20, 48, "f32", 0.9, 0.6, 1),        # non-square
    (16, 3, 2, 3, 2, 8, "f32", 0.5, 0.5, 1),          # grid smaller than one tile
    (17, 1, 1, 1, 1, 16, "bf16", 0.5, 0.5, 1),        # a single token
    (18, 1, 9, 32, 32, 1032, "bf16", 0.9, 0.9, 1),    # full 32x32, three chunks
    (19, 2, 3, 8, 8, 256, "f32", 0.6, 0.95, 8),       # root_grid == P: nothing to merge spatially
    (20, 1, 5, 13, 13, 200, "f16", 0.9, 0.8, 1),      # half-precision input, ragged chunk
    (21, 2, 3, 14, 14, 1032, "f16", 0.8, 0.85, 4),    # half precision, three chunks, 4x4 roots
    (22, 1, 3, 18, 24, 8192, "bf16", 0.9, 0.8, 1),    # 16 chunks (the widest row one workgroup covers), non-square
    (23, 1, 2, 7, 30, 8200, "f32", 0.8, 0.8, 1),      # fp32, 33 chunks: more chunks than wavefronts per workgroup
    (27, 1, 300, 3, 3, 72, "bf16", 1.0, -2.0, 1),     # nine chains of 300 cells: clusters summed item by item
    (28, 2, 40, 8, 8, 264, "f32", 0.95, 0.2, 1),      # long chains of mixed nodes
])
def test_small_shapes_fixed_thresholds(lib, seed, B, T, H, W, D, dtype, tau_s, tau_t, R):
    cfg = _variant(seed, B, T, H, W, D, dtype)
    _run_and_check(lib, cfg, tau_s=tau_s, tau_t=tau_t, root_grid=R)


@pytest.mark.parametrize("seed,H,W,D,dtype,keep,R", [
    (20, 13, 13, 136, "bf16", 0.5, 1),
    (21, 16, 16, 64, "f32", 0.3, 1),
    (22, 14, 14, 96, "bf16", 0.7, 4),
    (23, 8, 8, 32, "f32", 1.0, 1),
    (24, 8, 8, 32, "f32", 0.001, 1),                  # unreachable budget: thresholds fall to -2
])
def test_small_shapes_budget_mode(lib, seed, H, W, D, dtype, keep, R):
    cfg = _variant(seed, 2, 6, H, W, D, dtype)
    feats, r, info = _run_and_check(lib, cfg, keep=[keep, min(1.0, keep * 1.5)], root_grid=R)
    N1 = 6 * H * W
    for b, k in enumerate([keep, min(1.0, keep * 1.5)]):
        kb = r.offsets[b + 1] - r.offsets[b]
        if r.tau_t[b] > -2:
            assert kb <= math.floor(k * N1)


def test_half_precision_budget_and_output_types(lib):
    cfg = _variant(24, 1, 6, 13, 13, 520, "f16")
    _run_and_check(lib, cfg, keep=0.5)
    _run_and_check(lib, cfg, tau_s=0.9, tau_t=0.8, out_dtype=lib.STTM_F32)
    _run_and_check(lib, _variant(25, 1, 4, 8, 8, 64, "f32"), tau_s=0.9, tau_t=0.8, out_dtype=lib.STTM_F16)
    feats = wl.generate(_variant(26, 1, 2, 8, 8, 64, "bf16"))
    with pytest.raises(lib.SttmError) as e:                       # a 16-bit input is not converted to the other one
        P.run_gpu(lib, feats, tau_s=0.9, tau_t=0.8, out_dtype=lib.STTM_F16)
    assert e.value.code == lib.STTM_ERR_DTYPE


def test_mixed_output_dtypes(lib):
    cfg = _variant(30, 1, 4, 13, 13, 128, "bf16")
    _run_and_check(lib, cfg, tau_s=0.9, tau_t=0.9, out_dtype=lib.STTM_F32)
    cfg = _variant(31, 1, 4, 13, 13, 128, "f32")
    _run_and_check(lib, cfg, tau_s=0.9, tau_t=0.9, out_dtype=lib.STTM_BF16)


def test_degenerate_inputs(lib):
    rng = np.random.default_rng(0)
    v = rng.standard_normal(64).astype(np.float32)
    const = np.broadcast_to(v, (1, 4, 13, 13, 64)).copy()
    r = P.run_gpu(lib, const, tau_s=0.5, tau_t=0.5)
    assert r.K == 1 and r.counts[0] == 4 * 169                        # constant video: one root, one token
    assert (r.node_level == 4).all() and (r.cluster_ids == 0).all()
    np.testing.assert_allclose(r.merged[0], v, atol=1e-4)
    feats = wl.generate(_variant(40, 1, 3, 13, 13, 64, "f32"))
    r = P.run_gpu(lib, feats, tau_s=1.0, tau_t=1.0)                   # threshold >= 1: identity
    assert r.K == 3 * 169 and (r.counts == 1).all()
    np.testing.assert_array_equal(r.merged, feats.reshape(-1, 64))
    r = P.run_gpu(lib, feats, tau_s=-2.0, tau_t=-2.0)                 # everything merges
    assert r.K == 1 and r.counts[0] == 3 * 169
    feats[0, 2] = feats[0, 1]                                         # repeated frame merges into its predecessor
    r = P.run_gpu(lib, feats, tau_s=0.9, tau_t=0.999)
    assert (r.cluster_ids[0, 2] < 2 * 169).all()
    P.check_parity(lib, feats, r, tau_s=0.9, tau_t=0.999)
    zeros = np.zeros((1, 2, 4, 4, 8), dtype=np.float32)               # zero norm: similarity 0
    r = P.run_gpu(lib, zeros, tau_s=0.5, tau_t=0.5)
    assert r.K == 32
    r = P.run_gpu(lib, zeros, tau_s=-0.5, tau_t=-0.5)
    assert r.K == 1
    nan = feats.copy()
    nan[0, 1, 3, 3, 5] = np.nan                                       # NaN never passes a threshold
    r = P.run_gpu(lib, nan, tau_s=-2.0, tau_t=-2.0)
    assert r.node_level[0, 1, 3, 3] == 0 and r.node_level[0, 0].min() == 4
    assert r.cluster_ids[0, 1, 3, 3] == 169 + 3 * 13 + 3


@pytest.mark.parametrize("seed,T,H,W,D,dtype,tau_s,tau_t", [
    (70, 6, 13, 13, 136, "bf16", 0.3, 0.3),      # whole-frame and 8x8 nodes: their stored sums stand for them
    (71, 5, 16, 16, 72, "f32", 0.4, 0.5),
    (72, 7, 9, 9, 64, "bf16", 0.2, 0.2),         # the 8x8 node at (8, 8) holds a single valid cell
    (73, 4, 27, 27, 40, "bf16", 0.5, 0.4),       # five levels
    (74, 40, 8, 8, 16, "f32", 1.0, 0.2),         # long chains of single cells: clusters of more than 64 list slots
])
def test_reduce_with_and_without_node_sums(lib, seed, T, H, W, D, dtype, tau_s, tau_t):
    """The reduce call takes the stage-1 partition as an option; both ways must match the oracle."""
    cfg = _variant(seed, 1, T, H, W, D, dtype)
    feats = wl.generate(cfg)
    print(f"case seed={seed} shape={feats.shape} dtype={feats.dtype}", flush=True)
    a = P.run_gpu(lib, feats, tau_s=tau_s, tau_t=tau_t, use_nodes=True)
    P.check_parity(lib, feats, a, tau_s=tau_s, tau_t=tau_t)
    b = P.run_gpu(lib, feats, tau_s=tau_s, tau_t=tau_t, use_nodes=False, ctx=a.ctx, feats_dev=a.feats_dev)
    P.check_parity(lib, feats, b, tau_s=tau_s, tau_t=tau_t)
    assert (a.counts == b.counts).all() and (a.out_ids == b.out_ids).all() and (a.offsets == b.offsets).all()
    tol = P.TOL_BF16 if dtype == "bf16" else P.TOL_F32
    assert np.abs(a.merged - b.merged).max() <= tol


def test_budget_call_can_be_repeated(lib):
    """One statistics pass serves any number of budget searches (the search state is reset in between)."""
    import torch
    cfg = _variant(80, 2, 6, 13, 13, 72, "bf16")
    feats = wl.generate(cfg)
    B, T, H, W, D = feats.shape
    x = P._to_dev(feats)
    s = lib.Sttm(0)
    s.ensure_workspace(B, T, H, W, D, lib.STTM_BF16, 1)
    s.sttm_spatial_stats(x, lib.STTM_BF16, B, T, H, W, D, 1)
    t50 = s.sttm_budget_threshold(lib.STTM_STAGE_SPATIAL, 0.5)
    t30 = s.sttm_budget_threshold(lib.STTM_STAGE_SPATIAL, [0.3, 0.9])
    again = s.sttm_budget_threshold(lib.STTM_STAGE_SPATIAL, 0.5)
    assert (t50 == again).all() and t30[0] <= t50[0] and t30[1] >= t50[1]
    nm = torch.empty(B * T * H * W, dtype=torch.int32, device="cuda:0")
    lv = torch.empty(B * T * H * W, dtype=torch.uint8, device="cuda:0")
    s.sttm_spatial_quadtree(x, lib.STTM_BF16, B, T, H, W, D, 1, None, nm, lv)
    s.sttm_temporal_stats(x, nm, lv)
    u50 = s.sttm_budget_threshold(lib.STTM_STAGE_TEMPORAL, 0.5)
    u30 = s.sttm_budget_threshold(lib.STTM_STAGE_TEMPORAL, 0.3)
    again = s.sttm_budget_threshold(lib.STTM_STAGE_TEMPORAL, 0.5)
    assert (u50 == again).all() and (u30 <= u50).all()
    r = P.run_gpu(lib, feats, keep=0.5)
    assert (r.tau_s == t50).all() and (r.tau_t == u50).all()


def test_budget_threshold_left_to_the_consumer_kernels(lib):
    """sttm_budget_threshold without a host pointer resolves the last digit of the search inside the decision and
    edge kernels; the outputs must be those of the explicit path, bit for bit."""
    import torch
    cfg = wl.small_variant(wl.CONFIGS[1], T=12, B=2)
    feats = wl.generate(cfg)
    B, T, H, W, D = feats.shape
    N = B * T * H * W
    ref = P.run_gpu(lib, feats, keep=0.5)
    s = lib.Sttm(0)
    s.ensure_workspace(B, T, H, W, D, lib.STTM_BF16, 1)
    x = ref.feats_dev
    nm = torch.empty(N, dtype=torch.int32, device="cuda:0")
    nl = torch.empty(N, dtype=torch.uint8, device="cuda:0")
    cl = torch.empty(N, dtype=torch.int32, device="cuda:0")
    s.sttm_spatial_stats(x, lib.STTM_BF16, B, T, H, W, D, 1)
    s.sttm_budget_threshold(lib.STTM_STAGE_SPATIAL, 0.5, want_tau=False)
    s.sttm_spatial_quadtree(x, lib.STTM_BF16, B, T, H, W, D, 1, None, nm, nl)
    s.sttm_temporal_stats(x, nm, nl)
    s.sttm_budget_threshold(lib.STTM_STAGE_TEMPORAL, 0.5, want_tau=False)
    s.sttm_temporal_merge(x, nm, nl, None, cl)
    assert (nm.cpu().numpy().reshape(ref.node_map.shape) == ref.node_map).all()
    assert (cl.cpu().numpy().reshape(ref.cluster_ids.shape) == ref.cluster_ids).all()
    # the thresholds the kernels worked out are in the workspace: asking for them now gives the explicit path's
    np.testing.assert_array_equal(s.sttm_budget_threshold(lib.STTM_STAGE_TEMPORAL, 0.5), ref.tau_t)
    s.sttm_temporal_merge(x, nm, nl, None, cl)                   # and the stage can be repeated with them
    assert (cl.cpu().numpy().reshape(ref.cluster_ids.shape) == ref.cluster_ids).all()


def test_bitwise_reproducible(lib):
    cfg = _variant(50, 2, 8, 13, 13, 520, "bf16")
    feats = wl.generate(cfg)
    a = P.run_gpu(lib, feats, keep=0.5)
    b = P.run_gpu(lib, feats, keep=0.5, ctx=a.ctx, feats_dev=a.feats_dev)
    for name in ("child_sim", "pair_sim", "node_map", "cluster_ids", "merged", "counts", "out_ids"):
        x, y = getattr(a, name), getattr(b, name)
        if name == "pair_sim":
            continue   # slots that are not pairs are never written
        assert np.array_equal(x, y, equal_nan=True), name
    assert (a.tau_s == b.tau_s).all() and (a.tau_t == b.tau_t).all()


def test_temporal_stage_accepts_any_valid_partition(lib):
    """The temporal call takes the node map as an input: feed it the oracle's own partition."""
    cfg = _variant(60, 1, 5, 13, 13, 64, "f32")
    feats = wl.generate(cfg)
    sp = O.spatial_quadtree(feats, 0.6)
    r = P.run_gpu(lib, feats, tau_s=0.95, tau_t=0.8, node_map_override=(sp.node_map, sp.node_level))
    tm, _ = P.check_temporal(lib, feats, r, sp, 0.8)
    P.check_reduce(feats, r, tm, False)


def test_error_paths(lib):
    import torch
    s = lib.Sttm(0)
    x = torch.zeros(2 * 8 * 8 * 16, device="cuda:0")
    nm = torch.zeros(128, dtype=torch.int32, device="cuda:0")
    with pytest.raises(lib.SttmError) as e:
        s.sttm_spatial_quadtree(x, lib.STTM_F32, 1, 2, 8, 8, 16, 1, [0.5], nm)
    assert e.value.code == lib.STTM_ERR_WORKSPACE
    s.ensure_workspace(1, 2, 8, 8, 16, lib.STTM_F32, 1)
    for bad, code in [((1, 2, 8, 8, 12), lib.STTM_ERR_SHAPE), ((1, 2, 40, 8, 16), lib.STTM_ERR_SHAPE),
                      ((0, 2, 8, 8, 16), lib.STTM_ERR_SHAPE)]:
        with pytest.raises(lib.SttmError) as e:
            s.sttm_spatial_quadtree(x, lib.STTM_F32, *bad, 1, [0.5], nm)
        assert e.value.code == code
    with pytest.raises(lib.SttmError) as e:
        s.sttm_spatial_quadtree(x, lib.STTM_F32, 1, 2, 8, 8, 16, 3, [0.5], nm)
    assert e.value.code == lib.STTM_ERR_SHAPE
    with pytest.raises(lib.SttmError) as e:
        s.sttm_spatial_quadtree(x, 9, 1, 2, 8, 8, 16, 1, [0.5], nm)
    assert e.value.code == lib.STTM_ERR_DTYPE
    with pytest.raises(lib.SttmError) as e:                         # no statistics yet
        s.sttm_spatial_quadtree(x, lib.STTM_F32, 1, 2, 8, 8, 16, 1, None, nm)
    assert e.value.code == lib.STTM_ERR_STATE
    s.sttm_spatial_stats(x, lib.STTM_F32, 1, 2, 8, 8, 16, 1)
    with pytest.raises(lib.SttmError) as e:                         # statistics but no threshold
        s.sttm_spatial_quadtree(x, lib.STTM_F32, 1, 2, 8, 8, 16, 1, None, nm)
    assert e.value.code == lib.STTM_ERR_STATE
    with pytest.raises(lib.SttmError) as e:
        s.sttm_budget_threshold(lib.STTM_STAGE_SPATIAL, [1.5])
    assert e.value.code == lib.STTM_ERR_ARG
    with pytest.raises(lib.SttmError) as e:
        s.sttm_budget_threshold(lib.STTM_STAGE_TEMPORAL, [0.5])
    assert e.value.code == lib.STTM_ERR_STATE
    s.sttm_spatial_quadtree(x, lib.STTM_F32, 1, 2, 8, 8, 16, 1, [0.5], nm)
    cl = torch.zeros(128, dtype=torch.int32, device="cuda:0")
    with pytest.raises(lib.SttmError) as e:
        s.sttm_temporal_merge(x, nm, None, None, cl)
    assert e.value.code == lib.STTM_ERR_STATE
    s.sttm_temporal_merge(x, nm, None, [0.5], cl)                   # node levels derived from the map
    merged = torch.zeros(4, 16, device="cuda:0")
    off = torch.zeros(2, dtype=torch.int64, device="cuda:0")
    x.normal_()
    s.sttm_spatial_quadtree(x, lib.STTM_F32, 1, 2, 8, 8, 16, 1, [1.0], nm)
    s.sttm_temporal_merge(x, nm, None, [1.0], cl)
    with pytest.raises(lib.SttmError) as e:
        s.sttm_reduce(x, cl, None, None, lib.STTM_F32, 4, merged, None, None, off)
    assert e.value.code == lib.STTM_ERR_CAPACITY and int(off[1].item()) == 128
    torch.cuda.synchronize()
    np.testing.assert_array_equal(merged.cpu().numpy(), x.view(128, 16)[:4].cpu().numpy())


@pytest.mark.parametrize("B,T,H,W", [
    (1, 20, 16, 16),        # 5 k tokens: the scatter workgroups add up the histogram rows themselves
    (4, 64, 27, 27),        # 187 k tokens: rows added up in groups first
    (16, 1030, 32, 32),     # 16.9 M tokens: columns turned into running sums in place
])
def test_identity_at_every_size_class_of_the_list_sort(lib, B, T, H, W):
    """Thresholds of 1 merge nothing (the clamp makes every similarity <= 1 and the test is strict): the output
    is the input, row for row, whatever path the element sort takes for its start offsets."""
    import torch
    D, N = 8, B * T * H * W
    gen = torch.Generator(device="cuda:0")
    gen.manual_seed(1234 + N)
    x = torch.randn(N, D, device="cuda:0", generator=gen)
    print(f"case identity B={B} T={T} grid={H}x{W} N={N}", flush=True)
    s = lib.Sttm(0)
    s.ensure_workspace(B, T, H, W, D, lib.STTM_F32, 1)
    nm = torch.empty(N, dtype=torch.int32, device="cuda:0")
    nl = torch.empty(N, dtype=torch.uint8, device="cuda:0")
    cl = torch.empty(N, dtype=torch.int32, device="cuda:0")
    s.sttm_spatial_quadtree(x, lib.STTM_F32, B, T, H, W, D, 1, [1.0] * B, nm, nl)
    s.sttm_temporal_merge(x, nm, nl, [1.0] * B, cl)
    ar = torch.arange(N, dtype=torch.int32, device="cuda:0")
    assert torch.equal(nm, ar) and torch.equal(cl, ar) and int(nl.max().item()) == 0
    merged = torch.zeros(N, D, device="cuda:0")
    counts = torch.zeros(N, dtype=torch.int32, device="cuda:0")
    out_ids = torch.zeros(N, dtype=torch.int32, device="cuda:0")
    off = torch.zeros(B + 1, dtype=torch.int64, device="cuda:0")
    K = s.sttm_reduce(x, cl, nm, nl, lib.STTM_F32, N, merged, counts, out_ids, off)
    assert K == N and torch.equal(out_ids, ar) and int(counts.min().item()) == 1 and int(counts.max().item()) == 1
    assert torch.equal(off, torch.arange(B + 1, dtype=torch.int64, device="cuda:0") * (T * H * W))
    assert torch.equal(merged, x)


def test_longest_video_the_library_accepts_collapses_to_one_token_when_static(lib):
    """65535 frames (the most a context takes) of one constant token: every frame merges into its predecessor, so
    one cluster remains whose root chain is as long as chains get (pointer jumping needs all its rounds)."""
    import torch
    B, T, H, W, D = 1, 65535, 1, 1, 8
    x = torch.full((T, D), 0.75, device="cuda:0")
    s = lib.Sttm(0)
    s.ensure_workspace(B, T, H, W, D, lib.STTM_F32, 1)
    nm = torch.empty(T, dtype=torch.int32, device="cuda:0")
    nl = torch.empty(T, dtype=torch.uint8, device="cuda:0")
    cl = torch.empty(T, dtype=torch.int32, device="cuda:0")
    s.sttm_spatial_quadtree(x, lib.STTM_F32, B, T, H, W, D, 1, [0.5], nm, nl)
    s.sttm_temporal_merge(x, nm, nl, [0.5], cl)
    assert int(cl.max().item()) == 0
    merged = torch.zeros(4, D, device="cuda:0")
    counts = torch.zeros(4, dtype=torch.int32, device="cuda:0")
    off = torch.zeros(2, dtype=torch.int64, device="cuda:0")
    K = s.sttm_reduce(x, cl, nm, nl, lib.STTM_F32, 4, merged, counts, None, off)
    assert K == 1 and int(counts[0].item()) == T
    np.testing.assert_allclose(merged[0].cpu().numpy(), 0.75, rtol=0, atol=1e-4)
    with pytest.raises(lib.SttmError) as e:                         # one frame more is refused
        s.sttm_spatial_stats(x, lib.STTM_F32, 1, 65536, 1, 1, D, 1)
    assert e.value.code == lib.STTM_ERR_SHAPE


def test_positions_without_the_partition(lib):
    cfg = wl.Workload("alt", 95, 2, 5, 8, 8, 16, "f32", 2, 0.05, 0.9)
    feats = wl.generate_alternating(cfg, 0.7)
    r = P.run_gpu(lib, feats, tau_s=0.9, tau_t=0.8, positions=True, use_nodes=False)
    info = P.check_parity(lib, feats, r, tau_s=0.9, tau_t=0.8)
    assert "merged_pos_err" in info


# ---- destination rules (Sec. 3.3 and its ablation), row order and position indices (Sec. 3.4) ------------
@pytest.mark.parametrize("mode", ["first_passing", "topleft_only", "most_similar"])
@pytest.mark.parametrize("order", ["raster", "zscan"])
@pytest.mark.parametrize("seed,T,H,W,D,dtype", [
    (95, 5, 8, 8, 16, "f32"),          # the rules pick different destinations here (oracle pins say so)
    (97, 6, 13, 13, 520, "bf16"),      # padded grid, two chunks
])
def test_destination_rules_orders_and_positions(lib, mode, order, seed, T, H, W, D, dtype):
    cfg = wl.Workload("alt", seed, 1, T, H, W, D, dtype, 2, 0.05, 0.9)
    feats = wl.generate_alternating(cfg, 0.7)
    kw = dict(tau_s=0.9, tau_t=0.8)
    print(f"case alternating seed={seed} shape={feats.shape} mode={mode} order={order}", flush=True)
    r = P.run_gpu(lib, feats, mode=mode, order=order, positions=True, **kw)
    info = P.check_parity(lib, feats, r, mode=mode, order=order, **kw)
    print("  ", {k: v for k, v in info.items() if k in ("K", "near_temporal", "merged_err", "merged_pos_err")}, flush=True)
    if seed == 95:   # the case is not vacuous: the three rules give three different sets of edges
        base = P.run_gpu(lib, feats, mode="first_passing", **kw)
        assert mode == "first_passing" or (base.parent != r.parent).any()


def test_budget_mode_under_the_single_destination_rule(lib):
    """With only the top-left destination tested, e_n and hence the temporal budget threshold change."""
    cfg = wl.Workload("alt", 97, 2, 6, 13, 13, 264, "bf16", 2, 0.05, 0.9)
    feats = wl.generate_alternating(cfg, 0.7)
    print(f"case alternating budget shape={feats.shape}", flush=True)
    r = P.run_gpu(lib, feats, keep=0.4, mode="topleft_only", order="zscan", positions=True)
    info = P.check_parity(lib, feats, r, keep=0.4, mode="topleft_only", order="zscan")
    assert info["K"] <= int(0.4 * 6 * 169) * 2


def test_positions_and_settings_error_paths(lib):
    import torch
    s = lib.Sttm(0)
    with pytest.raises(lib.SttmError) as e:
        s.sttm_set_match_mode(3)
    assert e.value.code == lib.STTM_ERR_ARG
    with pytest.raises(lib.SttmError) as e:
        s.sttm_set_output_order(-1)
    assert e.value.code == lib.STTM_ERR_ARG
    cfg = wl.CONFIGS[0]
    feats = wl.generate(cfg)
    r = P.run_gpu(lib, feats, tau_s=cfg.tau_s, tau_t=cfg.tau_t, ctx=s)
    N = cfg.n_tokens
    cl = torch.from_numpy(r.cluster_ids.reshape(-1)).cuda()       # same ids, another buffer
    off = torch.from_numpy(r.offsets).cuda()
    sv = torch.zeros(N, dtype=torch.int32, device="cuda:0")
    with pytest.raises(lib.SttmError) as e:                        # not the buffer the reduce call saw
        s.sttm_positions(cl, None, None, off, N, sv)
    assert e.value.code == lib.STTM_ERR_STATE
    with pytest.raises(lib.SttmError) as e:
        s.sttm_positions(None, None, None, off, N, sv)
    assert e.value.code == lib.STTM_ERR_NULL
    # the order may not change between the reduce call and its position indices
    x = r.feats_dev
    nm = torch.from_numpy(r.node_map.reshape(-1)).cuda()
    nl = torch.from_numpy(r.node_level.reshape(-1)).cuda()
    merged = torch.zeros(N, feats.shape[-1], device="cuda:0")
    s.sttm_reduce(x, cl, None, None, lib.STTM_F32, N, merged, None, None, off)
    s.sttm_positions(cl, nm, nl, off, N, sv)                     # fine: follows the reduce call on these ids
    s.sttm_set_output_order(lib.STTM_ORDER_ZSCAN)
    with pytest.raises(lib.SttmError) as e:
        s.sttm_positions(cl, nm, nl, off, N, sv)
    assert e.value.code == lib.STTM_ERR_STATE
    s.sttm_set_match_mode(lib.STTM_MATCH_MOST_SIMILAR)             # another rule: the temporal statistics are stale
    with pytest.raises(lib.SttmError) as e:
        s.sttm_budget_threshold(lib.STTM_STAGE_TEMPORAL, [0.5])
    assert e.value.code == lib.STTM_ERR_STATE


@pytest.mark.parametrize("seed,B,T,H,W,D,dtype,kw", [
    (70, 2, 6, 13, 13, 136, "bf16", dict(keep=0.5)),
    (71, 1, 5, 16, 16, 64, "f32", dict(tau_s=0.95, tau_t=0.6)),
    (72, 1, 4, 14, 14, 520, "f16", dict(tau_s=0.7, tau_t=0.7, root_grid=4)),
    (73, 1, 5, 27, 27, 72, "bf16", dict(tau_s=0.6, tau_t=0.5)),       # many 2x2 and 4x4 nodes, ragged edge
])
def test_temporal_pass_without_the_cell_dot_products(lib, seed, B, T, H, W, D, dtype, kw):
    """sttm_set_cell_dots(0): the temporal pass computes the cell-to-cell pairs itself. Parity with the oracle, and
    the same partition and clusters as with the option on."""
    feats = wl.generate(_variant(seed, B, T, H, W, D, dtype))
    print(f"case seed={seed} shape={feats.shape} dtype={feats.dtype} {kw}", flush=True)
    s = lib.Sttm(0)
    off = P.run_gpu(lib, feats, ctx=s, cell_dots=0, **kw)
    P.check_parity(lib, feats, off, **kw)
    for level in (1, 2):                                       # same context: the setting applies to the next pass
        on = P.run_gpu(lib, feats, ctx=s, cell_dots=level, **kw)
        assert (on.node_map == off.node_map).all() and (on.cluster_ids == off.cluster_ids).all() and on.K == off.K
        P.check_parity(lib, feats, on, **kw)


def test_cell_dot_setting_and_feature_pointer_error_paths(lib):
    import torch
    s = lib.Sttm(0)
    with pytest.raises(lib.SttmError) as e:
        s.sttm_set_cell_dots(3)
    assert e.value.code == lib.STTM_ERR_ARG
    cfg = wl.CONFIGS[0]
    feats = wl.generate(cfg)
    r = P.run_gpu(lib, feats, tau_s=cfg.tau_s, tau_t=cfg.tau_t, ctx=s)
    nm = torch.from_numpy(r.node_map.reshape(-1)).cuda()
    cl = torch.zeros(cfg.n_tokens, dtype=torch.int32, device="cuda:0")
    other = r.feats_dev.clone()                                   # same values, another buffer
    with pytest.raises(lib.SttmError) as e:                        # the statistics belong to r.feats_dev
        s.sttm_temporal_merge(other, nm, None, [cfg.tau_t], cl)
    assert e.value.code == lib.STTM_ERR_STATE
    s.sttm_temporal_merge(r.feats_dev, nm, None, [cfg.tau_t], cl)
    assert (cl.cpu().numpy() == r.cluster_ids.reshape(-1)).all()


def test_config3_long_video_most_similar_zscan_positions(lib):
    """The bench workload once more under the alternative rule and scan, with position indices."""
    cfg = wl.CONFIGS[3]
    feats = wl.generate(cfg)
    print(f"case {cfg.name} shape={feats.shape} most_similar zscan", flush=True)
    r = P.run_gpu(lib, feats, keep=0.5, mode="most_similar", order="zscan", positions=True)
    info = P.check_parity(lib, feats, r, keep=0.5, mode="most_similar", order="zscan")
    print("  ", {k: (float(v) if isinstance(v, (float, np.floating)) else v) for k, v in info.items()
                 if k not in ("tau_s", "tau_t")}, flush=True)


# ---- the five configurations at full size, in the launch configuration bench.py times ------------------
def test_config1_short_clip_budget(lib):
    cfg = wl.CONFIGS[1]
    _run_and_check(lib, cfg, keep=cfg.budgets[0])


def test_config2_encoder_width_budget(lib):
    cfg = wl.CONFIGS[2]
    _run_and_check(lib, cfg, keep=cfg.budgets[0])


@pytest.mark.parametrize("keep,cell_dots", [(0.5, 1), (0.3, 1), (0.5, 0), (0.3, 2)])
def test_config3_long_video_budget(lib, keep, cell_dots):
    """The bench workload at both budgets; once more with the spatial and temporal passes kept separate, and once
    with the frame-to-frame dot products of the 2x2 and 4x4 blocks taken in the spatial pass too."""
    cfg = wl.CONFIGS[3]
    _run_and_check(lib, cfg, keep=keep, cell_dots=cell_dots)


@pytest.mark.timeout(900)
@pytest.mark.parametrize("index,keep", [(5, 0.3), (6, 0.5)])
def test_paper_shapes_budget(lib, index, keep):
    """The paper's own grid (14 x 14, 4 x 4 roots, 180 frames) and a wide non-square one (18 x 24 at D = 8192), every
    frame of both compared with the oracle, in budget mode."""
    cfg = wl.CONFIGS[index]
    _run_and_check(lib, cfg, keep=keep, root_grid=cfg.root_grid)


@pytest.fixture(scope="module")
def batched(lib):
    """Config 4 run once on the GPU (all 32 videos in one batch); the tests below compare it video by video."""
    cfg = wl.CONFIGS[4]
    feats = wl.generate(cfg)
    print(f"case {cfg.name} shape={feats.shape}", flush=True)
    r = P.run_gpu(lib, feats, tau_s=cfg.tau_s, tau_t=cfg.tau_t)
    assert int(r.counts.sum()) == cfg.n_tokens and r.offsets[-1] == r.K
    return cfg, feats, r


@pytest.mark.parametrize("b", range(32))
def test_config4_batched_fixed_thresholds_every_video(lib, batched, b):
    """Videos are independent, so a video's slice of every output equals the single-video result shifted by its
    token offset: the oracle runs on each of the 32 videos and is compared element by element."""
    cfg, feats, r = batched
    B, T, H, W, D = feats.shape
    per = T * H * W
    sub = P.GpuResult()
    lo, hi = int(r.offsets[b]), int(r.offsets[b + 1])
    sub.child_sim = r.child_sim[b * T:(b + 1) * T]
    sub.min_sim = r.min_sim[b * T:(b + 1) * T]
    sub.node_map = r.node_map[b:b + 1] - b * per
    sub.node_level = r.node_level[b:b + 1]
    sub.pair_sim = r.pair_sim[b * per:(b + 1) * per]
    sub.best_sim = r.best_sim[b * per:(b + 1) * per]
    par = r.parent[b:b + 1].copy()
    par[par >= 0] -= b * per
    sub.parent = par
    sub.cluster_ids = r.cluster_ids[b:b + 1] - b * per
    sub.K = hi - lo
    sub.merged = r.merged[lo:hi]
    sub.counts = r.counts[lo:hi]
    sub.out_ids = r.out_ids[lo:hi] - b * per
    sub.offsets = np.array([0, hi - lo])
    info = P.check_parity(lib, feats[b:b + 1], sub, tau_s=cfg.tau_s, tau_t=cfg.tau_t)
    print(f"   video {b}:", {k: (float(v) if isinstance(v, (float, np.floating)) else v)
                             for k, v in info.items()}, flush=True)


# ---- state handling, streams, contexts, non-finite inputs -------------------------------------------------------
def test_infinite_and_nan_features_against_the_oracle(lib):
    """An infinity or a NaN makes the similarities it enters undefined; they never pass a threshold, on either side."""
    feats = wl.generate(_variant(41, 1, 4, 13, 13, 72, "f32"))
    feats[0, 1, 5, 6, 3] = np.inf
    feats[0, 2, 12, 12, 70] = -np.inf
    feats[0, 3, 0, 0, 0] = np.nan
    for kw in (dict(tau_s=0.7, tau_t=0.6), dict(tau_s=-2.0, tau_t=-2.0)):
        r = P.run_gpu(lib, feats, **kw)
        sp = O.spatial_quadtree(feats, kw["tau_s"])
        assert (sp.node_map == r.node_map).all() and (sp.node_level == r.node_level).all()
        assert r.node_level[0, 1, 5, 6] == 0 and r.node_level[0, 2, 12, 12] == 0 and r.node_level[0, 3, 0, 0] == 0
        sp2, _ = P.check_spatial(lib, feats, r, kw["tau_s"])
        tm, _ = P.check_temporal(lib, feats, r, sp2, kw["tau_t"])
        assert r.parent[0, 1, 5, 6] == -1 and r.parent[0, 2, 5, 6] == -1      # no edge into or out of the broken token
        assert (r.counts.sum() == feats[..., 0].size) and r.K == len(np.unique(tm.cluster_ids))


def test_new_temporal_statistics_discard_the_pending_threshold(lib):
    """temporal_stats, budget (threshold left to the consumer), temporal_stats again, merge without thresholds:
    the second statistics pass starts the search afresh, so the merge must refuse instead of resolving a
    threshold from an empty search state."""
    import torch
    cfg = _variant(81, 2, 5, 13, 13, 72, "bf16")
    feats = wl.generate(cfg)
    B, T, H, W, D = feats.shape
    N = B * T * H * W
    x = P._to_dev(feats)
    s = lib.Sttm(0)
    s.ensure_workspace(B, T, H, W, D, lib.STTM_BF16, 1)
    nm = torch.empty(N, dtype=torch.int32, device="cuda:0")
    nl = torch.empty(N, dtype=torch.uint8, device="cuda:0")
    cl = torch.empty(N, dtype=torch.int32, device="cuda:0")
    s.sttm_spatial_quadtree(x, lib.STTM_BF16, B, T, H, W, D, 1, [0.9, 0.9], nm, nl)
    s.sttm_temporal_stats(x, nm, nl)
    s.sttm_budget_threshold(lib.STTM_STAGE_TEMPORAL, 0.5, want_tau=False)
    s.sttm_temporal_stats(x, nm, nl)
    with pytest.raises(lib.SttmError) as e:
        s.sttm_temporal_merge(x, nm, nl, None, cl)
    assert e.value.code == lib.STTM_ERR_STATE
    tau = s.sttm_budget_threshold(lib.STTM_STAGE_TEMPORAL, 0.5)
    nm2 = nm.clone()
    with pytest.raises(lib.SttmError) as e:                      # not the node map the statistics were computed for
        s.sttm_temporal_merge(x, nm2, nl, None, cl)
    assert e.value.code == lib.STTM_ERR_STATE
    s.sttm_temporal_merge(x, nm, nl, None, cl)
    ref = P.run_gpu(lib, feats, tau_s=[0.9, 0.9], tau_t=list(tau))
    assert (cl.cpu().numpy().reshape(ref.cluster_ids.shape) == ref.cluster_ids).all()
    # after sttm_invalidate nothing cached is trusted any more
    s.sttm_invalidate()
    for call in (lambda: s.sttm_temporal_merge(x, nm, nl, [0.5, 0.5], cl),
                 lambda: s.sttm_budget_threshold(lib.STTM_STAGE_SPATIAL, 0.5),
                 lambda: s.sttm_spatial_quadtree(x, lib.STTM_BF16, B, T, H, W, D, 1, None, nm, nl)):
        with pytest.raises(lib.SttmError) as e:
            call()
        assert e.value.code == lib.STTM_ERR_STATE
    s.sttm_spatial_quadtree(x, lib.STTM_BF16, B, T, H, W, D, 1, [0.9, 0.9], nm, nl)   # and recomputing works
    s.sttm_temporal_merge(x, nm, nl, list(tau), cl)
    assert (cl.cpu().numpy().reshape(ref.cluster_ids.shape) == ref.cluster_ids).all()


def test_non_default_stream_and_two_contexts_on_one_device(lib):
    """Two contexts with workspaces of their own, one on a stream that is not the default one, interleaved call by
    call on two different videos: each gives what it gives alone."""
    import torch
    fa = wl.generate(_variant(82, 1, 6, 13, 13, 520, "bf16"))
    fb = wl.generate(_variant(83, 2, 4, 16, 16, 136, "f32"))
    ra = P.run_gpu(lib, fa, keep=0.5)
    rb = P.run_gpu(lib, fb, tau_s=0.8, tau_t=0.7)
    side = torch.cuda.Stream(device=0)
    sa = lib.Sttm(0, stream_ptr=side.cuda_stream)
    sb = lib.Sttm(0)
    xa, xb = P._to_dev(fa), P._to_dev(fb)
    torch.cuda.synchronize()
    out = {}
    for name, s, x, f in (("a", sa, xa, fa), ("b", sb, xb, fb)):
        B, T, H, W, D = f.shape
        N = B * T * H * W
        dt = P.lib_dtype(lib, f)
        s.ensure_workspace(B, T, H, W, D, dt, 1)
        out[name] = dict(nm=torch.empty(N, dtype=torch.int32, device="cuda:0"),
                         nl=torch.empty(N, dtype=torch.uint8, device="cuda:0"),
                         cl=torch.empty(N, dtype=torch.int32, device="cuda:0"),
                         mg=torch.zeros(N, D, dtype=x.dtype, device="cuda:0"),
                         ct=torch.zeros(N, dtype=torch.int32, device="cuda:0"),
                         oi=torch.zeros(N, dtype=torch.int32, device="cuda:0"),
                         of=torch.zeros(B + 1, dtype=torch.int64, device="cuda:0"), shape=(B, T, H, W, D), dt=dt, N=N)
    torch.cuda.synchronize()
    a, b = out["a"], out["b"]
    Ba, Ta, Ha, Wa, Da = a["shape"]
    Bb, Tb, Hb, Wb, Db = b["shape"]
    sa.sttm_spatial_stats(xa, a["dt"], Ba, Ta, Ha, Wa, Da, 1)
    sb.sttm_spatial_quadtree(xb, b["dt"], Bb, Tb, Hb, Wb, Db, 1, [0.8] * Bb, b["nm"], b["nl"])
    sa.sttm_budget_threshold(lib.STTM_STAGE_SPATIAL, 0.5, want_tau=False)
    sb.sttm_temporal_merge(xb, b["nm"], b["nl"], [0.7] * Bb, b["cl"])
    sa.sttm_spatial_quadtree(xa, a["dt"], Ba, Ta, Ha, Wa, Da, 1, None, a["nm"], a["nl"])
    sa.sttm_temporal_stats(xa, a["nm"], a["nl"])
    Kb = sb.sttm_reduce(xb, b["cl"], b["nm"], b["nl"], b["dt"], b["N"], b["mg"], b["ct"], b["oi"], b["of"])
    sa.sttm_budget_threshold(lib.STTM_STAGE_TEMPORAL, 0.5, want_tau=False)
    sa.sttm_temporal_merge(xa, a["nm"], a["nl"], None, a["cl"])
    Ka = sa.sttm_reduce(xa, a["cl"], a["nm"], a["nl"], a["dt"], a["N"], a["mg"], a["ct"], a["oi"], a["of"])
    side.synchronize()
    torch.cuda.synchronize()
    for r, o, K in ((ra, a, Ka), (rb, b, Kb)):
        assert K == r.K
        assert (o["cl"].cpu().numpy().reshape(r.cluster_ids.shape) == r.cluster_ids).all()
        assert (o["ct"][:K].cpu().numpy() == r.counts).all() and (o["oi"][:K].cpu().numpy() == r.out_ids).all()
        np.testing.assert_array_equal(o["mg"][:K].float().cpu().numpy(), r.merged)


def test_randomized_shapes_and_settings(lib):
    """Sixty seeded random draws over everything the boundary lets a caller choose -- grid (1x1 to 32x32, any aspect),
    frames, videos, width, element type, root grid, destination rule, row order, which dot products ride along in
    the spatial pass, noise level, fixed thresholds or a budget -- each compared with the oracle like the named
    cases above, position indices included. Every second draw reuses one long-lived context."""
    import random
    rng = random.Random(20250711)
    shared = lib.Sttm(0)   # every second draw runs on one context that is never renewed: shapes and settings change under it
    for case in range(60):
        H = rng.choice([1, 2, 3, 5, 7, 8, 9, 12, 13, 14, 16, 17, 20, 24, 27, 31, 32])
        W = rng.choice([1, 2, 4, 6, 8, 11, 13, 14, 16, 18, 23, 27, 32])
        P2 = wl.pow2_ceil(max(H, W))
        T = rng.choice([1, 2, 3, 4, 5, 7, 9, 12])
        B = rng.choice([1, 1, 2, 3])
        dtype = rng.choice(["bf16", "bf16", "f16", "f32"])
        D = 8 * rng.choice([1, 2, 3, 5, 9, 17, 25, 33, 64, 65, 96, 129, 144])
        while B * T * H * W * D > 3.0e6:
            D = max(8, D // 2 // 8 * 8)
            if B * T * H * W * D > 3.0e6 and T > 2:
                T -= 1
        R = rng.choice([r for r in (1, 1, 1, 2, 4, 8, 16, 32) if r <= P2])
        mode = rng.choice(["first_passing", "first_passing", "topleft_only", "most_similar"])
        order = rng.choice(["raster", "zscan"])
        cell_dots = rng.choice([0, 1, 1, 2])
        sigma = rng.choice([0.02, 0.1, 0.3, 0.8])
        persist = rng.choice([0.3, 0.7, 0.95])
        cfg = wl.Workload("random", 5000 + case, B, T, H, W, D, dtype, int(math.log2(P2)), sigma, persist)
        if rng.random() < 0.5:
            kw = dict(keep=rng.choice([0.1, 0.25, 0.3, 0.5, 0.75, 0.9, 1.0]))
        else:
            kw = dict(tau_s=rng.choice([0.5, 0.7, 0.8, 0.9, 0.95, 1.0, -2.0]),
                      tau_t=rng.choice([0.3, 0.6, 0.8, 0.9, 0.97, 1.0, -2.0]))
        alternating = rng.random() < 0.3
        feats = wl.generate_alternating(cfg, sigma * 4) if alternating else wl.generate(cfg)
        print(f"case {case}: B={B} T={T} {H}x{W} D={D} {dtype} R={R} {mode} {order} cell_dots={cell_dots} "
              f"sigma={sigma} persist={persist} alternating={alternating} {kw}", flush=True)
        r = P.run_gpu(lib, feats, root_grid=R, mode=mode, order=order, positions=True, cell_dots=cell_dots,
                      ctx=shared if case % 2 == 0 else None, **kw)
        info = P.check_parity(lib, feats, r, root_grid=R, mode=mode, order=order, **kw)
        assert info["K"] >= 1
