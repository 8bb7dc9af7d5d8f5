"""Drives libsttm_cpu.so (the kernels compiled for host threads) through the same C ABI, with numpy
arrays standing in for device memory. Test infrastructure for hunting hangs / out-of-bounds on the CPU."""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
LIB = os.path.join(HERE, "libsttm_cpu.so")

STTM_F32, STTM_BF16, STTM_F16 = 0, 1, 2


class Result:
    pass


def _aligned(nbytes, align=256, garbage=False):
    raw = np.zeros(nbytes + align, dtype=np.uint8)
    if garbage:  # device memory is not zero-initialised: make reads of never-written words visible
        raw[:] = np.random.default_rng(12345).integers(0, 256, size=raw.size, dtype=np.uint8)
    off = (-raw.ctypes.data) % align
    return raw[off:off + nbytes]


def _p(a):
    return C.c_void_p(a.ctypes.data) if a is not None else None


def load():
    lib = C.CDLL(LIB)
    lib.sttm_workspace_bytes.restype = C.c_size_t
    lib.sttm_last_error.restype = C.c_char_p
    lib.sttm_last_error.argtypes = [C.c_void_p]
    return lib


def run_cpu(feats, *, tau_s=None, tau_t=None, keep=None, root_grid=1, out_dtype=None, lib=None, use_nodes=True,
            match=0, order=0, positions=False, defer_tau=False, cell_dots=1, node_map_override=None):
    lib = lib or load()
    B, T, H, W, D = feats.shape
    dt = STTM_BF16 if feats.dtype == np.uint16 else (STTM_F16 if feats.dtype == np.float16 else STTM_F32)
    out_dtype = dt if out_dtype is None else out_dtype
    N = B * T * H * W
    h = C.c_void_p()
    assert lib.sttm_create(C.byref(h), 0, None) == 0

    def chk(rc):
        assert rc == 0, (rc, lib.sttm_last_error(h))

    chk(lib.sttm_set_match_mode(h, match))
    chk(lib.sttm_set_output_order(h, order))
    chk(lib.sttm_set_cell_dots(h, cell_dots))
    need = lib.sttm_workspace_bytes(B, T, H, W, D, dt, root_grid)
    ws = _aligned(need, garbage=True)
    chk(lib.sttm_set_workspace(h, _p(ws), C.c_size_t(need)))
    x = _aligned(feats.nbytes, 16)
    x[:] = np.ascontiguousarray(feats).view(np.uint8).reshape(-1)
    node_map = np.zeros(N, np.int32)
    node_level = np.zeros(N, np.uint8)
    cluster = np.zeros(N, np.int32)
    farr = lambda v: (C.c_float * B)(*[float(t) for t in np.broadcast_to(np.asarray(v, np.float32), (B,))])
    karr = lambda v: (C.c_double * B)(*[float(t) for t in np.broadcast_to(np.asarray(v, np.float64), (B,))])
    r = Result()
    r.tau_s = r.tau_t = None
    if tau_s is None:
        chk(lib.sttm_spatial_stats(h, _p(x), dt, B, T, H, W, D, root_grid))
        out = (C.c_float * B)()
        chk(lib.sttm_budget_threshold(h, 0, karr(keep), None if defer_tau else out))
        r.tau_s = np.array(list(out), np.float32)
        chk(lib.sttm_spatial_quadtree(h, _p(x), dt, B, T, H, W, D, root_grid, None, _p(node_map), _p(node_level)))
    else:
        chk(lib.sttm_spatial_quadtree(h, _p(x), dt, B, T, H, W, D, root_grid, farr(tau_s), _p(node_map),
                                      _p(node_level)))
    lib.sttm_nodes_per_frame.restype = C.c_int
    NN = lib.sttm_nodes_per_frame(H, W, root_grid)
    tbl = np.zeros(B * T * NN, np.float32)
    chk(lib.sttm_export(h, 0, _p(tbl), C.c_size_t(tbl.nbytes)))
    r.child_sim = tbl.reshape(B * T, NN).copy()
    chk(lib.sttm_export(h, 1, _p(tbl), C.c_size_t(tbl.nbytes)))
    r.min_sim = tbl.reshape(B * T, NN).copy()
    r.node_map = node_map.reshape(B, T, H, W).copy()
    r.node_level = node_level.reshape(B, T, H, W).copy()
    if node_map_override is not None:   # any valid quadtree partition per frame may be handed to the temporal stage
        node_map[:] = node_map_override[0].reshape(-1)
        node_level[:] = node_map_override[1].reshape(-1)
    if tau_t is None:
        chk(lib.sttm_temporal_stats(h, _p(x), _p(node_map), _p(node_level)))
        out = (C.c_float * B)()
        chk(lib.sttm_budget_threshold(h, 1, karr(keep), None if defer_tau else out))
        r.tau_t = np.array(list(out), np.float32)
        chk(lib.sttm_temporal_merge(h, _p(x), _p(node_map), _p(node_level), None, _p(cluster)))
    else:
        chk(lib.sttm_temporal_merge(h, _p(x), _p(node_map), _p(node_level), farr(tau_t), _p(cluster)))
    t32 = np.zeros(N, np.float32)
    chk(lib.sttm_export(h, 3, _p(t32), C.c_size_t(t32.nbytes)))
    r.pair_sim = t32.copy()
    chk(lib.sttm_export(h, 4, _p(t32), C.c_size_t(t32.nbytes)))
    r.best_sim = t32.copy()
    ti = np.zeros(N, np.int32)
    chk(lib.sttm_export(h, 5, _p(ti), C.c_size_t(ti.nbytes)))
    r.parent = ti.reshape(B, T, H, W).copy()
    r.cluster_ids = cluster.reshape(B, T, H, W).copy()
    esz = 4 if out_dtype == STTM_F32 else 2
    merged = _aligned(N * D * esz, 16)
    counts = np.zeros(N, np.int32)
    out_ids = np.zeros(N, np.int32)
    offsets = np.zeros(B + 1, np.int64)
    n = C.c_int64(-1)
    chk(lib.sttm_reduce(h, _p(x), _p(cluster), _p(node_map) if use_nodes else None,
                        _p(node_level) if use_nodes else None, out_dtype, C.c_int64(N), _p(merged), _p(counts),
                        _p(out_ids), _p(offsets), C.byref(n)))
    K = int(n.value)
    r.K = K
    if out_dtype == STTM_BF16:
        bits = merged.view(np.uint16)[:K * D].astype(np.uint32) << 16
        r.merged = bits.view(np.float32).reshape(K, D).copy()
    elif out_dtype == STTM_F16:
        r.merged = merged.view(np.float16)[:K * D].astype(np.float32).reshape(K, D).copy()
    else:
        r.merged = merged.view(np.float32)[:K * D].reshape(K, D).copy()
    r.counts = counts[:K].copy()
    r.out_ids = out_ids[:K].copy()
    r.offsets = offsets.copy()
    if positions:
        sv, ra = np.zeros(N, np.int32), np.zeros(N, np.int32)
        mp, rt = np.zeros(N, np.float32), np.zeros(4 * N, np.int32)
        chk(lib.sttm_positions(h, _p(cluster), _p(node_map) if use_nodes else None, _p(node_level), _p(offsets),
                               C.c_int64(N), _p(sv), _p(ra), _p(mp),
                               _p(rt)))
        r.survived, r.reassigned, r.merged_pos = sv[:K].copy(), ra[:K].copy(), mp[:K].copy()
        r.root_tyxl = rt[:4 * K].reshape(K, 4).copy()
    lib.sttm_destroy(h)
    return r
