"""ctypes binding of libsttm.so: same names as include/sttm.h, argument marshalling only.

Device buffers are torch tensors (torch is used for device memory and streams, nothing else); every
step of the path runs inside the library's HIP kernels.  There is no fallback: if the shared library
is missing, importing this module raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

import numpy as np
import torch  # noqa: F401  -- first, so that libsttm.so binds to the HIP runtime torch has already loaded

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libsttm.so")

STTM_OK = 0
STTM_ERR_NULL, STTM_ERR_SHAPE, STTM_ERR_DTYPE, STTM_ERR_ARG = 1, 2, 3, 4
STTM_ERR_WORKSPACE, STTM_ERR_STATE, STTM_ERR_CAPACITY, STTM_ERR_HIP = 5, 6, 7, 8
STTM_F32, STTM_BF16, STTM_F16 = 0, 1, 2
STTM_STAGE_SPATIAL, STTM_STAGE_TEMPORAL = 0, 1
STTM_TBL_CHILD_SIM, STTM_TBL_MIN_SIM, STTM_TBL_NORM2 = 0, 1, 2
STTM_TBL_PAIR_SIM, STTM_TBL_BEST_SIM, STTM_TBL_PARENT = 3, 4, 5

EXPORTS = [
    "sttm_create", "sttm_destroy", "sttm_last_error", "sttm_nodes_per_frame", "sttm_node_index",
    "sttm_workspace_bytes", "sttm_set_workspace", "sttm_spatial_stats", "sttm_spatial_quadtree",
    "sttm_temporal_stats", "sttm_temporal_merge", "sttm_budget_threshold", "sttm_reduce", "sttm_export",
    "sttm_profile_enable", "sttm_profile_read", "sttm_set_match_mode", "sttm_set_output_order", "sttm_positions",
    "sttm_set_cell_dots", "sttm_invalidate", "sttm_reduce_noalloc", "sttm_reduce_noalloc_max_bytes",
    "sttm_reduce_noalloc_bytes",
]
STTM_MATCH_FIRST_PASSING, STTM_MATCH_TOPLEFT_ONLY, STTM_MATCH_MOST_SIMILAR = 0, 1, 2
STTM_ORDER_RASTER, STTM_ORDER_ZSCAN = 0, 1
STTM_KERNEL_PYRAMID_STATS, STTM_KERNEL_TEMPORAL_DOTS, STTM_KERNEL_REDUCE_GATHER = 0, 1, 2


def _load() -> C.CDLL:
    if not os.path.exists(LIB_PATH):
        raise ImportError(
            f"{LIB_PATH} is missing: build it with `python -m paper_2507_07990_amd.build` "
            "(there is no CPU fallback)")
    lib = C.CDLL(LIB_PATH)
    vp, i, i64, sz = C.c_void_p, C.c_int, C.c_int64, C.c_size_t
    lib.sttm_create.argtypes = [C.POINTER(vp), i, vp]
    lib.sttm_destroy.argtypes = [vp]
    lib.sttm_last_error.argtypes = [vp]
    lib.sttm_last_error.restype = C.c_char_p
    lib.sttm_nodes_per_frame.argtypes = [i, i, i]
    lib.sttm_node_index.argtypes = [i, i, i, i, i, i]
    lib.sttm_workspace_bytes.argtypes = [i, i, i, i, i, i, i]
    lib.sttm_workspace_bytes.restype = sz
    lib.sttm_set_workspace.argtypes = [vp, vp, sz]
    lib.sttm_spatial_stats.argtypes = [vp, vp, i, i, i, i, i, i, i]
    lib.sttm_spatial_quadtree.argtypes = [vp, vp, i, i, i, i, i, i, i, C.POINTER(C.c_float), vp, vp]
    lib.sttm_temporal_stats.argtypes = [vp, vp, vp, vp]
    lib.sttm_temporal_merge.argtypes = [vp, vp, vp, vp, C.POINTER(C.c_float), vp]
    lib.sttm_budget_threshold.argtypes = [vp, i, C.POINTER(C.c_double), C.POINTER(C.c_float)]
    lib.sttm_reduce.argtypes = [vp, vp, vp, vp, vp, i, i64, vp, vp, vp, vp, C.POINTER(i64)]
    lib.sttm_export.argtypes = [vp, i, vp, sz]
    lib.sttm_profile_enable.argtypes = [vp, i]
    lib.sttm_profile_read.argtypes = [vp, i, C.POINTER(C.c_double), C.POINTER(i64)]
    lib.sttm_set_match_mode.argtypes = [vp, i]
    lib.sttm_set_output_order.argtypes = [vp, i]
    lib.sttm_set_cell_dots.argtypes = [vp, i]
    lib.sttm_invalidate.argtypes = [vp]
    lib.sttm_reduce_noalloc.argtypes = [vp, vp, i, i, i, i, i, i, vp, i, i64, vp, vp, vp, vp]
    lib.sttm_reduce_noalloc_max_bytes.argtypes = []
    lib.sttm_reduce_noalloc_max_bytes.restype = sz
    lib.sttm_reduce_noalloc_bytes.argtypes = [i, i, i, i, i, i]
    lib.sttm_reduce_noalloc_bytes.restype = sz
    lib.sttm_positions.argtypes = [vp, vp, vp, vp, vp, i64, vp, vp, vp, vp]
    return lib


_lib = _load()


class SttmError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"sttm status {code}: {msg}")
        self.code = code


def sttm_nodes_per_frame(H: int, W: int, root_grid: int = 1) -> int:
    return int(_lib.sttm_nodes_per_frame(H, W, root_grid))


def sttm_node_index(H: int, W: int, root_grid: int, level: int, by: int, bx: int) -> int:
    return int(_lib.sttm_node_index(H, W, root_grid, level, by, bx))


def sttm_workspace_bytes(B, T, H, W, D, dtype, root_grid=1) -> int:
    return int(_lib.sttm_workspace_bytes(B, T, H, W, D, dtype, root_grid))


def sttm_reduce_noalloc_max_bytes() -> int:
    return int(_lib.sttm_reduce_noalloc_max_bytes())


def sttm_reduce_noalloc_bytes(B, T, H, W, D, dtype) -> int:
    return int(_lib.sttm_reduce_noalloc_bytes(B, T, H, W, D, dtype))


def _ptr(t) -> Optional[int]:
    return None if t is None else t.data_ptr()


def _farr(vals: Optional[Sequence[float]], n: int):
    if vals is None:
        return None
    a = np.broadcast_to(np.asarray(vals, dtype=np.float32), (n,))
    return (C.c_float * n)(*[float(v) for v in a])


class Sttm:
    """One library context on one device / stream.  Methods mirror the C entry points."""

    def __init__(self, device: int = 0, stream_ptr: Optional[int] = None):
        import torch
        if stream_ptr is None:
            stream_ptr = torch.cuda.current_stream(device).cuda_stream
        self._h = C.c_void_p()
        rc = _lib.sttm_create(C.byref(self._h), device, C.c_void_p(stream_ptr))
        if rc != STTM_OK:
            raise SttmError(rc, "sttm_create failed")
        self.device = device
        self._ws = None
        self.shape = None

    def close(self):
        if self._h:
            _lib.sttm_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _check(self, rc: int):
        if rc != STTM_OK:
            raise SttmError(rc, _lib.sttm_last_error(self._h).decode())

    # -- workspace ------------------------------------------------------------------------------
    def sttm_set_workspace(self, ws_tensor):
        self._ws = ws_tensor
        self._check(_lib.sttm_set_workspace(self._h, _ptr(ws_tensor), ws_tensor.numel() * ws_tensor.element_size()))

    def ensure_workspace(self, B, T, H, W, D, dtype, root_grid=1):
        import torch
        need = sttm_workspace_bytes(B, T, H, W, D, dtype, root_grid)
        if need == 0:
            raise SttmError(STTM_ERR_SHAPE, "invalid shape")
        if self._ws is None or self._ws.numel() < need:
            self.sttm_set_workspace(torch.empty(need, dtype=torch.uint8, device=f"cuda:{self.device}"))

    # -- stages -----------------------------------------------------------------------------------
    def sttm_spatial_stats(self, feats, dtype, B, T, H, W, D, root_grid=1):
        self._check(_lib.sttm_spatial_stats(self._h, _ptr(feats), dtype, B, T, H, W, D, root_grid))
        self.shape = (B, T, H, W, D, dtype, root_grid)

    def sttm_spatial_quadtree(self, feats, dtype, B, T, H, W, D, root_grid, tau_s, node_map, node_level=None):
        self._check(_lib.sttm_spatial_quadtree(self._h, _ptr(feats), dtype, B, T, H, W, D, root_grid,
                                               _farr(tau_s, B), _ptr(node_map), _ptr(node_level)))
        self.shape = (B, T, H, W, D, dtype, root_grid)

    def sttm_temporal_stats(self, feats, node_map, node_level=None):
        self._check(_lib.sttm_temporal_stats(self._h, _ptr(feats), _ptr(node_map), _ptr(node_level)))

    def sttm_temporal_merge(self, feats, node_map, node_level, tau_t, cluster_ids):
        B = self.shape[0]
        self._check(_lib.sttm_temporal_merge(self._h, _ptr(feats), _ptr(node_map), _ptr(node_level),
                                             _farr(tau_t, B), _ptr(cluster_ids)))

    def sttm_budget_threshold(self, stage, target_keep, want_tau=True):
        B = self.shape[0]
        keep = np.broadcast_to(np.asarray(target_keep, dtype=np.float64), (B,))
        karr = (C.c_double * B)(*[float(v) for v in keep])
        out = (C.c_float * B)() if want_tau else None
        self._check(_lib.sttm_budget_threshold(self._h, stage, karr, out))
        return np.array(list(out), dtype=np.float32) if want_tau else None

    def sttm_reduce(self, feats, cluster_ids, node_map, node_level, out_dtype, capacity, merged, counts, out_ids,
                    offsets, want_n=True):
        n = C.c_int64(-1)
        rc = _lib.sttm_reduce(self._h, _ptr(feats), _ptr(cluster_ids), _ptr(node_map), _ptr(node_level), out_dtype,
                              capacity, _ptr(merged), _ptr(counts), _ptr(out_ids), _ptr(offsets),
                              C.byref(n) if want_n else None)
        self._check(rc)
        return int(n.value) if want_n else None

    def sttm_set_match_mode(self, mode: int):
        self._check(_lib.sttm_set_match_mode(self._h, mode))

    def sttm_set_output_order(self, order: int):
        self._check(_lib.sttm_set_output_order(self._h, order))

    def sttm_reduce_noalloc(self, feats, dtype, B, T, H, W, D, cluster_ids, out_dtype, capacity, merged, counts,
                            out_ids, offsets):
        self._check(_lib.sttm_reduce_noalloc(self._h, _ptr(feats), dtype, B, T, H, W, D, _ptr(cluster_ids), out_dtype,
                                             capacity, _ptr(merged), _ptr(counts), _ptr(out_ids), _ptr(offsets)))

    def sttm_invalidate(self):
        self._check(_lib.sttm_invalidate(self._h))

    def sttm_set_cell_dots(self, on: int):
        self._check(_lib.sttm_set_cell_dots(self._h, on))

    def sttm_positions(self, cluster_ids, node_map, node_level, offsets, capacity, survived=None, reassigned=None,
                       merged_pos=None, root_tyxl=None):
        self._check(_lib.sttm_positions(self._h, _ptr(cluster_ids), _ptr(node_map), _ptr(node_level), _ptr(offsets),
                                        capacity,
                                        _ptr(survived), _ptr(reassigned), _ptr(merged_pos), _ptr(root_tyxl)))

    def sttm_export(self, table, dst):
        self._check(_lib.sttm_export(self._h, table, _ptr(dst), dst.numel() * dst.element_size()))

    def sttm_profile_enable(self, every):
        """every: False / 0 = off, True / 1 = every launch, n = every n-th launch of each feature kernel."""
        self._check(_lib.sttm_profile_enable(self._h, int(every)))

    def sttm_profile_read(self, kernel: int):
        ms, n = C.c_double(0.0), C.c_int64(0)
        self._check(_lib.sttm_profile_read(self._h, kernel, C.byref(ms), C.byref(n)))
        return float(ms.value), int(n.value)
