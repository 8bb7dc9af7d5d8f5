#!/usr/bin/env python3
"""Benchmark of the merge path on one MI355X.

A step = one pass of the whole hot path (pyramid statistics -> spatial threshold from the budget ->
quadtree decision -> temporal similarities -> temporal threshold -> edges + roots -> gather/average)
over one synthetic video batch already resident in HBM.  No host synchronisation happens inside a step.

Prints ONE JSON line: whole-path throughput in input tokens/s, the roofline figure of the dominant
feature kernel (HIP events recorded by the library on its stream during the timed steps), and the CPU
oracle timed on a bounded sample of the same workload.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0


def stored_traffic(config: int, keep):
    """HBM-side bytes per launch of the feature kernels, measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE
    runs of this very script (summaries under profiles/; bench.py itself cannot run a profiler around itself).
    Returns {kernel: read + written bytes} or {} when no summary covers the workload."""
    names = {(3, 0.5): "whole_path_long_video_keep50.txt", (3, 0.3): "whole_path_long_video_keep30.txt",
             (5, 0.5): "whole_path_paper_grid_keep50.txt", (4, None): "whole_path_batched_unpooled.txt"}
    path = os.path.join(ROOT, "profiles", names.get((config, keep), "-"))
    out = {}
    if os.path.exists(path):
        for line in open(path):
            f = line.split()
            if len(f) == 4 and f[0] == "traffic_bytes":
                out[f[1]] = int(f[2]) + int(f[3])
    return out


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=3, help="index into the workload table (default: long video)")
    ap.add_argument("--keep", type=float, default=None, help="token budget (default: the config's first)")
    ap.add_argument("--copies", type=int, default=0,
                    help="distinct device copies of the input the steps rotate over, so that no step finds its input "
                         "in a cache because the step before read the same buffer (default: enough for 512 MB, 2..8)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--event-period", type=int, default=4,
                    help="bracket the feature kernels of every n-th timed step with HIP events (default 4)")
    ap.add_argument("--no-kernel-events", action="store_true",
                    help="do not bracket the feature kernels with HIP events (the roofline block is then empty)")
    ap.add_argument("--cpu-frames", type=int, default=512, help="frames of the workload the oracle is timed on")
    ap.add_argument("--match", choices=["first_passing", "topleft_only", "most_similar"], default="first_passing",
                    help="destination rule of the temporal stage (default: the paper's top-left-most passing one)")
    ap.add_argument("--order", choices=["raster", "zscan"], default="raster", help="row order of the output")
    ap.add_argument("--positions", action="store_true", help="also emit the position indices of the rows each step")
    ap.add_argument("--no-cell-dots", action="store_true",
                    help="keep the spatial and temporal passes separate (sttm_set_cell_dots(0))")
    ap.add_argument("--no-node-sums", action="store_true",
                    help="reduce stage without the stage-1 partition: every cell is read again")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="after the timed steps, run one plain device-to-device copy of the input tensor "
                         "(known size: reads and writes N*D*esz bytes) so that a counter run can scale "
                         "FETCH_SIZE / WRITE_SIZE by what they read for it")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU only (how the path would shard is described in the design notes); "
              "rerun with --gpus 1", file=sys.stderr)
        return 2

    import torch
    from paper_2507_07990_amd import binding as lib
    from paper_2507_07990_amd import workloads as wl

    cfg = wl.CONFIGS[args.config]
    budget_mode = cfg.tau_s is None
    keep = args.keep if args.keep is not None else (cfg.budgets[0] if budget_mode else None)
    t0 = time.time()
    feats = wl.generate(cfg)
    gen_s = time.time() - t0
    B, T, H, W, D = feats.shape
    N = B * T * H * W
    dt = {np.dtype(np.uint16): lib.STTM_BF16, np.dtype(np.float16): lib.STTM_F16}.get(feats.dtype, lib.STTM_F32)
    esz = 4 if dt == lib.STTM_F32 else 2
    R = cfg.root_grid
    dev = "cuda:0"
    torch.cuda.set_device(0)
    if feats.dtype == np.uint16:
        x = torch.from_numpy(feats.view(np.int16)).to(dev).view(torch.bfloat16)
    else:
        x = torch.from_numpy(feats).to(dev)

    # consecutive steps work on different buffers holding the same video
    copies = args.copies if args.copies > 0 else max(2, min(8, -(-(512 << 20) // (N * D * esz))))
    xs = [x] + [x.clone() for _ in range(copies - 1)]
    step_no = [0]

    s = lib.Sttm(0)
    s.sttm_set_match_mode({"first_passing": 0, "topleft_only": 1, "most_similar": 2}[args.match])
    s.sttm_set_output_order({"raster": 0, "zscan": 1}[args.order])
    s.sttm_set_cell_dots(0 if args.no_cell_dots else 1)
    s.ensure_workspace(B, T, H, W, D, dt, R)
    node_map = torch.empty(N, dtype=torch.int32, device=dev)
    node_level = torch.empty(N, dtype=torch.uint8, device=dev)
    cluster = torch.empty(N, dtype=torch.int32, device=dev)
    merged = torch.empty(N, D, dtype=x.dtype, device=dev)
    counts = torch.empty(N, dtype=torch.int32, device=dev)
    out_ids = torch.empty(N, dtype=torch.int32, device=dev)
    offsets = torch.zeros(B + 1, dtype=torch.int64, device=dev)
    if args.positions:
        pos_sv = torch.empty(N, dtype=torch.int32, device=dev)
        pos_ra = torch.empty(N, dtype=torch.int32, device=dev)
        pos_mg = torch.empty(N, dtype=torch.float32, device=dev)
        pos_rt = torch.empty(N, 4, dtype=torch.int32, device=dev)

    def step():
        x = xs[step_no[0] % copies]
        step_no[0] += 1
        if budget_mode:
            s.sttm_spatial_stats(x, dt, B, T, H, W, D, R)
            s.sttm_budget_threshold(lib.STTM_STAGE_SPATIAL, keep, want_tau=False)
            s.sttm_spatial_quadtree(x, dt, B, T, H, W, D, R, None, node_map, node_level)
            s.sttm_temporal_stats(x, node_map, node_level)
            s.sttm_budget_threshold(lib.STTM_STAGE_TEMPORAL, keep, want_tau=False)
            s.sttm_temporal_merge(x, node_map, node_level, None, cluster)
        else:
            s.sttm_spatial_quadtree(x, dt, B, T, H, W, D, R, [cfg.tau_s], node_map, node_level)
            s.sttm_temporal_merge(x, node_map, node_level, [cfg.tau_t], cluster)
        s.sttm_reduce(x, cluster, None if args.no_node_sums else node_map,
                      None if args.no_node_sums else node_level, dt, N, merged, counts, out_ids, offsets, want_n=False)
        if args.positions:
            s.sttm_positions(cluster, node_map, node_level, offsets, N, pos_sv, pos_ra, pos_mg, pos_rt)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    # every 4th step's feature kernels are bracketed by events (a pair costs about 3 us of stream time)
    s.sttm_profile_enable(0 if args.no_kernel_events else args.event_period)
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    prof = {k: s.sttm_profile_read(k) for k in (lib.STTM_KERNEL_PYRAMID_STATS, lib.STTM_KERNEL_TEMPORAL_DOTS,
                                               lib.STTM_KERNEL_REDUCE_GATHER)}
    s.sttm_profile_enable(False)
    ms_per_step = elapsed / args.steps * 1e3
    if args.calibrate_copy:
        merged.view(-1)[:x.numel()].copy_(x.view(-1))
        torch.cuda.synchronize()
    K = int(offsets[B].item())
    assert int(counts[:K].sum().item()) == N, "member counts do not add up to the number of input tokens"
    rho = K / N

    # Algorithmic bytes per launch of each feature kernel: every input element it must see read once,
    # every output element written once (design notes: data layout / kernels). The temporal pass must see the rows
    # of the node pairs it computes: both nodes' cells when the coarser one is at most a 4x4 block, only the finer
    # node's cells above that (the coarser node's sum is stored) -- and nothing for a pair of two single cells when
    # the spatial pass left that dot product. A row needed by two frame pairs counts once.
    lv = node_level.view(B, T, H * W)
    if T > 1:
        a, b = lv[:, 1:].int(), lv[:, :-1].int()
        J = torch.maximum(a, b)
        small = J <= 2
        if not args.no_cell_dots:
            small = small & (J > 0)
        need_t = small | ((J >= 3) & (a < b))   # rows of the later frame of a pair
        need_p = small | ((J >= 3) & (b < a))   # rows of the earlier frame
        need = torch.zeros(B, T, H * W, dtype=torch.bool, device=dev)
        need[:, 1:] |= need_t
        need[:, :-1] |= need_p
        rows_temporal = int(need.sum().item())
    else:
        rows_temporal = 0
    alg = {
        lib.STTM_KERNEL_PYRAMID_STATS: ("k_pyramid_stats", N * D * esz),
        lib.STTM_KERNEL_TEMPORAL_DOTS: ("k_temporal_dots", rows_temporal * D * esz),
        lib.STTM_KERNEL_REDUCE_GATHER: ("k_reduce", N * D * esz + K * D * esz),
    }
    kernels = {}
    for k, (ms, n) in prof.items():
        name, nbytes = alg[k]
        avg_ms = ms / max(n, 1)
        kernels[name] = {"avg_ms": avg_ms, "launches": n, "alg_bytes": nbytes,
                         "GBps": nbytes / (avg_ms * 1e-3) / 1e9 if avg_ms > 0 else None}
    traffic = stored_traffic(args.config, keep)
    for name in kernels:
        kernels[name]["traffic_bytes"] = traffic.get(name)
    dom = max(kernels, key=lambda kk: kernels[kk]["avg_ms"])
    achieved = kernels[dom]["GBps"]
    path_bytes = N * D * esz + K * D * esz + 9 * N + 8 * K
    out = {
        "metric": "input visual tokens merged/sec (Mtok/s) at D=3584 bf16; achieved HBM GB/s vs peak",
        "value": N / (elapsed / args.steps) / 1e6,
        "unit": "Mtok/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": {lib.STTM_BF16: "bf16", lib.STTM_F16: "f16"}.get(dt, "f32"), "data": "synthetic",
        "config": {"workload": f"configs[{args.config}] {cfg.name}: B={B} T={T} grid={H}x{W} D={D} "
                               f"{cfg.dtype}, " + (f"budget keep={keep}" if budget_mode else
                                                   f"tau_s={cfg.tau_s} tau_t={cfg.tau_t}")
                               + (f", root_grid={R}" if R != 1 else "")
                               + (f", match={args.match}" if args.match != "first_passing" else "")
                               + (f", order={args.order}" if args.order != "raster" else "")
                               + (", with position indices" if args.positions else "")
                               + (", separate spatial and temporal passes" if args.no_cell_dots else ""),
                   "tokens": N, "kept_tokens": K, "kept_fraction": rho, "generate_s": gen_s, "input_copies": copies},
        "roofline": {"bound": "hbm", "kernel": dom, "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS if achieved else None, "traffic": traffic.get(dom),
                     "alg_bytes_per_launch": kernels[dom]["alg_bytes"], "kernels": kernels},
        "path": {"alg_bytes_per_step": path_bytes,
                 "whole_path_GBps": path_bytes / (elapsed / args.steps) / 1e9,
                 "whole_path_frac_of_peak": path_bytes / (elapsed / args.steps) / 1e9 / HBM_PEAK_GBS},
        "paper_context": "end-to-end prefill speed-up reported by the paper on 1xA100 80G (LLaVA-Video-7B): "
                         "about 2x at a 50% budget, about 3x at 30%; the merge path alone is not timed there",
    }

    if not args.no_cpu_baseline:
        from oracle import sttm_oracle as O
        try:
            from threadpoolctl import threadpool_limits
            limiter = threadpool_limits(limits=1)
        except Exception:  # pragma: no cover
            limiter = None
        nf = min(T, args.cpu_frames, max(2, int(3.2e8 // (H * W * D))))   # bounds one pass of the oracle
        sample = feats[:1, :nf]
        reps = 0
        t0 = time.perf_counter()
        while True:   # whole passes over the sample until about ten seconds of CPU work have been timed
            if budget_mode:
                O.sttm(sample, keep=keep, root_grid=R, mode=args.match, order=args.order)
            else:
                O.sttm(sample, tau_s=cfg.tau_s, tau_t=cfg.tau_t, root_grid=R, mode=args.match, order=args.order)
            reps += 1
            cpu_s = time.perf_counter() - t0
            if cpu_s >= 10.0 or reps >= 8:
                break
        if limiter is not None:
            limiter.restore_original_limits()
        out["cpu_baseline"] = {"value": reps * nf * H * W / cpu_s / 1e6, "unit": "Mtok/s", "cores": 1, "kind": "oracle",
                               "sample": f"video 0, first {nf} of {T} frames of the same workload "
                                         f"({nf * H * W} tokens), {reps} passes in {cpu_s:.1f} s, fp64 numpy, 1 thread"}
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
