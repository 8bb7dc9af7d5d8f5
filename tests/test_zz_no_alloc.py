"""sttm_reduce_noalloc (the entry point for callers that cannot allocate) against sttm_reduce, through the C ABI."""
import numpy as np
import pytest

from paper_2507_07990_amd import workloads as wl
from tests import parity as P

pytestmark = pytest.mark.gpu


def _compare(lib, s, feats, r, order):
    """One sttm_reduce call (workspace, no partition) and one sttm_reduce_noalloc call on the same cluster ids."""
    import torch
    B, T, H, W, D = feats.shape
    N = B * T * H * W
    dt = P.lib_dtype(lib, feats)
    x = r.feats_dev
    cl = torch.from_numpy(r.cluster_ids.reshape(-1)).cuda()
    s.sttm_set_output_order(P.ORDERS[order])
    out = []
    for which in ("workspace", "static"):
        gd = P.Guarded()
        merged = gd.alloc("merged", N * D, x.dtype, zero=True).view(N, D)
        counts = gd.alloc("counts", N, torch.int32, zero=True)
        out_ids = gd.alloc("out_ids", N, torch.int32, zero=True)
        offsets = gd.alloc("offsets", B + 1, torch.int64, zero=True)
        if which == "workspace":
            s.ensure_workspace(B, T, H, W, D, dt, 1)
            s.sttm_spatial_stats(x, dt, B, T, H, W, D, 1)      # binds the shape the workspace call works on
            s.sttm_reduce(x, cl, None, None, dt, N, merged, counts, out_ids, offsets)
        else:
            s.sttm_reduce_noalloc(x, dt, B, T, H, W, D, cl, dt, N, merged, counts, out_ids, offsets)
        torch.cuda.synchronize()
        gd.check(f"the {which} reduce call")
        K = int(offsets[B].item())
        out.append((K, merged[:K].float().cpu().numpy(), counts[:K].cpu().numpy(), out_ids[:K].cpu().numpy(),
                    offsets.cpu().numpy()))
    (Ka, ma, ca, ia, oa), (Kb, mb, cb, ib, ob) = out
    assert Ka == Kb == r.K
    assert (ca == cb).all() and (ia == ib).all() and (oa == ob).all()
    np.testing.assert_array_equal(ma, mb)            # same kernels, same summation order: bit for bit
    return mb, cb, ib


def test_noalloc_reduce_matches_the_workspace_call_twice_in_a_row(lib):
    """Two calls in a row on one context, the second on a smaller input (the static array still holds the first
    call's tables), each against sttm_reduce and against the oracle."""
    from oracle import sttm_oracle as O
    s = lib.Sttm(0)
    big = wl.generate(wl.small_variant(wl.CONFIGS[1], T=24, D=520))            # 4056 tokens, clusters of all sizes
    small = wl.generate(wl.small_variant(wl.CONFIGS[0], T=5))                  # 320 tokens, fp32
    chain = wl.generate(wl.Workload("v", 27, 1, 300, 3, 3, 72, "bf16", 2, 0.1, 0.7))   # clusters summed item by item
    cases = [(big, dict(keep=0.4), "raster"), (small, dict(tau_s=0.8, tau_t=0.8), "zscan"),
             (chain, dict(tau_s=1.0, tau_t=-2.0), "raster"), (small, dict(tau_s=0.8, tau_t=0.8), "raster")]
    for feats, kw, order in cases:
        r = P.run_gpu(lib, feats, **kw)
        merged, counts, out_ids = _compare(lib, s, feats, r, order)
        rd = O.reduce_clusters(feats, r.cluster_ids, order)
        assert (counts == rd.counts).all() and (out_ids == rd.out_ids).all()
        tol = P.TOL_BF16 if feats.dtype == np.uint16 else P.TOL_F32
        assert np.abs(merged.astype(np.float64) - rd.merged).max() <= tol


def test_noalloc_reduce_refuses_what_does_not_fit(lib):
    import torch
    s = lib.Sttm(0)
    assert lib.sttm_reduce_noalloc_max_bytes() == 32 << 20
    B, T, H, W, D = 1, 64, 16, 16, 8192                                      # 16384 tokens x 8192 channels
    assert lib.sttm_reduce_noalloc_bytes(B, T, H, W, D, lib.STTM_BF16) > lib.sttm_reduce_noalloc_max_bytes()
    x = torch.zeros(16, dtype=torch.bfloat16, device="cuda:0")               # never read: the call is refused first
    cl = torch.zeros(16, dtype=torch.int32, device="cuda:0")
    off = torch.zeros(2, dtype=torch.int64, device="cuda:0")
    with pytest.raises(lib.SttmError) as e:
        s.sttm_reduce_noalloc(x, lib.STTM_BF16, B, T, H, W, D, cl, lib.STTM_BF16, 16, x, None, None, off)
    assert e.value.code == lib.STTM_ERR_WORKSPACE
    with pytest.raises(lib.SttmError) as e:
        s.sttm_reduce_noalloc(x, lib.STTM_BF16, 1, 1, 40, 2, 8, cl, lib.STTM_BF16, 16, x, None, None, off)
    assert e.value.code == lib.STTM_ERR_SHAPE
    with pytest.raises(lib.SttmError) as e:
        s.sttm_reduce_noalloc(x, lib.STTM_BF16, 1, 1, 2, 2, 8, cl, lib.STTM_F16, 16, x, None, None, off)
    assert e.value.code == lib.STTM_ERR_DTYPE
