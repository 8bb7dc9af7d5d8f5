#!/usr/bin/env python3
"""Benchmark of the merge path on one MI355X.

A step = one pass of the whole hot path (pyramid statistics -> spatial threshold from the budget ->
quadtree decision -> temporal similarities -> temporal threshold -> edges + roots -> gather/average)
over one synthetic video batch already resident in HBM.  No host synchronisation happens inside a step.

Prints ONE JSON line: whole-path throughput in input tokens/s (from the median of the timed steps, each
bracketed by HIP events on the stream the library launches on), the roofline figure of the dominant
feature kernel (HIP events recorded by the library around that kernel during the timed steps), the same
measurement at the workload's other token budgets, and the CPU oracle timed on a bounded sample of the same
workload (one thread, and with its per-frame steps spread over all cores).
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


def source_digest() -> str:
    """sha256 over the library's kernel sources: a traffic figure is only quoted for the code it was measured on."""
    import hashlib
    h = hashlib.sha256()
    csrc = os.path.join(ROOT, "paper_2507_07990_amd", "csrc")
    for name in sorted(os.listdir(csrc)):
        if name.endswith((".hip", ".h")):
            h.update(name.encode())
            h.update(open(os.path.join(csrc, name), "rb").read())
    return h.hexdigest()


def stored_traffic(config: int, keep):
    """HBM-side bytes per launch of the library's kernels, measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE
    runs of this very script (summaries under profiles/; bench.py itself cannot run a profiler around itself).
    Returns ({kernel: read + written bytes}, {kernel: average microseconds in that run}, note). The figures are
    dropped (with the reason in the note) when the summary was made from other kernel sources than the ones here."""
    names = {(3, 0.5): "whole_path_long_video_keep50.txt", (3, 0.3): "whole_path_long_video_keep30.txt",
             (5, 0.5): "whole_path_paper_grid_keep50.txt", (4, None): "whole_path_batched_unpooled.txt"}
    path = os.path.join(ROOT, "profiles", names.get((config, keep), "-"))
    traffic, avg_us, digest = {}, {}, None
    if not os.path.exists(path):
        return {}, {}, "no counter summary for this workload under profiles/"
    for line in open(path):
        f = line.split()
        if len(f) == 4 and f[0] == "traffic_bytes":
            traffic[f[1]] = int(f[2]) + int(f[3])
        elif len(f) == 3 and f[0] == "kernel_avg_us":
            avg_us[f[1]] = float(f[2])
        elif len(f) == 2 and f[0] == "source_sha256":
            digest = f[1]
    if digest != source_digest():
        return {}, {}, f"{os.path.basename(path)} was measured on other kernel sources: traffic not quoted"
    return traffic, avg_us, os.path.basename(path)


def cpu_baseline_legs(feats, cfg, keep, args):
    """The oracle timed on a bounded sample of the workload: one thread, then its per-frame steps over all the
    cores this process may use. Runs before anything touches the GPU (the second leg forks worker processes)."""
    from oracle import sttm_oracle as O
    from oracle import parallel as OP
    B, T, H, W, D = feats.shape
    R = cfg.root_grid
    nf = min(T, args.cpu_frames, max(2, int(3.2e8 // (H * W * D))))   # bounds one pass of the oracle
    sample = feats[:1, :nf]
    kw = dict(keep=keep) if cfg.tau_s is None else dict(tau_s=cfg.tau_s, tau_t=cfg.tau_t)
    kw.update(root_grid=R, mode=args.match, order=args.order)
    try:
        from threadpoolctl import threadpool_limits
        limiter = threadpool_limits(limits=1)
    except Exception:  # pragma: no cover
        limiter = None

    def timed(fn, budget_s):
        reps, t0 = 0, time.perf_counter()
        while True:   # whole passes over the sample until the time budget is used
            fn()
            reps += 1
            el = time.perf_counter() - t0
            if el >= budget_s or reps >= 8:
                return reps, el

    reps, cpu_s = timed(lambda: O.sttm(sample, **kw), 10.0)
    if limiter is not None:
        limiter.restore_original_limits()
    one = {"value": reps * nf * H * W / cpu_s / 1e6, "unit": "Mtok/s", "cores": 1, "kind": "oracle",
           "sample": f"video 0, first {nf} of {T} frames of the same workload ({nf * H * W} tokens), "
                     f"{reps} passes in {cpu_s:.1f} s, fp64 numpy, 1 thread"}
    try:
        cores = len(os.sched_getaffinity(0))
    except AttributeError:  # pragma: no cover
        cores = os.cpu_count() or 1
    cores = max(1, min(cores, int(os.environ.get("OMP_NUM_THREADS", "16")), 16))
    reps, par_s = timed(lambda: OP.sttm_parallel(sample, procs=cores, **kw), 8.0)
    many = {"value": reps * nf * H * W / par_s / 1e6, "unit": "Mtok/s", "cores": cores, "kind": "oracle",
            "sample": f"the same sample, {reps} passes in {par_s:.1f} s; pyramid / child similarities and the "
                      f"candidate similarities split by frames over {cores} processes, thresholds, decisions, "
                      f"roots and the per-cluster means serial"}
    return one, many


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
    ap.add_argument("--cell-dots-only", action="store_true",
                    help="keep the spatial pass to the cell-against-cell products at every budget (default: the 2x2 and "
                         "4x4 block products ride along too when the budget keeps 35 % of the tokens or less)")
    ap.add_argument("--node-dots", action="store_true",
                    help="frame-to-frame dot products of the 2x2 and 4x4 blocks in the spatial pass too (sttm_set_cell_dots(2))")
    ap.add_argument("--no-node-sums", action="store_true",
                    help="reduce stage without the stage-1 partition: every cell is read again")
    ap.add_argument("--no-two-streams", action="store_true",
                    help="skip the extra leg that runs the timed steps alternately on two contexts and streams")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="after the timed steps, run one plain device-to-device copy of the input tensor "
                         "(known size: reads and writes N*D*esz bytes) so that a counter run can scale "
                         "FETCH_SIZE / WRITE_SIZE by what they read for it")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU only (how the path would shard is described in the design notes); "
              "rerun with --gpus 1", file=sys.stderr)
        return 2

    from paper_2507_07990_amd import workloads as wl

    cfg = wl.CONFIGS[args.config]
    budget_mode = cfg.tau_s is None
    if not budget_mode:
        budgets = [None]
    elif args.keep is not None:
        budgets = [args.keep]
    else:
        budgets = list(cfg.budgets)        # the first one is the headline; the others ride along under "budgets"
    t0 = time.time()
    feats = wl.generate(cfg)
    gen_s = time.time() - t0
    cpu = None
    if not args.no_cpu_baseline:           # before the GPU is touched: the all-cores leg forks worker processes
        cpu = cpu_baseline_legs(feats, cfg, budgets[0], args)

    import torch
    from paper_2507_07990_amd import binding as lib

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

    def dots_level(keep):
        """Which frame-to-frame dot products the spatial pass leaves for the temporal stage (sttm_set_cell_dots):
        measured on the bench workload, the block products (level 2) cost the spatial pass about 6 us and pay
        once many tokens merge spatially, i.e. at budgets of about a third and below."""
        if args.no_cell_dots:
            return 0
        if args.node_dots:
            return 2
        if args.cell_dots_only or keep is None:
            return 1
        return 2 if keep <= 0.35 else 1

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

    def step(keep):
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

    def measure(keep):
        """W warm-up steps, then exactly K timed steps: the wall clock around all of them, and one HIP event
        between consecutive steps on the stream the library launches on, for the median step time."""
        level = dots_level(keep)
        s.sttm_set_cell_dots(level)
        for _ in range(args.warmup):
            step(keep)
        torch.cuda.synchronize()
        # every 4th step's feature kernels are bracketed by events (a pair costs about 3 us of stream time)
        s.sttm_profile_enable(0 if args.no_kernel_events else args.event_period)
        marks = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]
        t0 = time.perf_counter()
        marks[0].record()
        for i in range(args.steps):
            step(keep)
            marks[i + 1].record()
        torch.cuda.synchronize()
        elapsed = time.perf_counter() - t0
        per_step = sorted(marks[i].elapsed_time(marks[i + 1]) for i in range(args.steps))
        median_ms = per_step[len(per_step) // 2] if len(per_step) % 2 else \
            0.5 * (per_step[len(per_step) // 2 - 1] + per_step[len(per_step) // 2])
        prof = {k: s.sttm_profile_read(k) for k in (lib.STTM_KERNEL_PYRAMID_STATS, lib.STTM_KERNEL_TEMPORAL_DOTS,
                                                   lib.STTM_KERNEL_REDUCE_GATHER)}
        s.sttm_profile_enable(False)
        K = int(offsets[B].item())
        assert int(counts[:K].sum().item()) == N, "member counts do not add up to the number of input tokens"

        # Algorithmic bytes per launch of each feature kernel: every input element it must see read once,
        # every output element written once (design notes: data layout / kernels). The temporal pass must see the
        # rows of the node pairs it computes: both nodes' cells when the coarser one is at most a 4x4 block, only the
        # finer node's cells above that (the coarser node's sum is stored) -- and nothing for a pair of two single
        # cells when the spatial pass left that dot product. A row needed by two frame pairs counts once.
        lv = node_level.view(B, T, H * W)
        if T > 1:
            a, b = lv[:, 1:].int(), lv[:, :-1].int()
            J = torch.maximum(a, b)
            small = J <= 2
            if level == 2:
                small = small & (a != b)
            elif level == 1:
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
        traffic, prof_us, traffic_note = stored_traffic(args.config, keep)
        kernels = {}
        for k, (ms, n) in prof.items():
            name, nbytes = alg[k]
            avg_ms = ms / max(n, 1)
            t_bytes = traffic.get(name)
            there_us = prof_us.get(name)
            if name == "k_temporal_dots" and there_us is not None:
                # the bracketed region of the temporal feature pass is its planner plus the pass itself
                there_us += prof_us.get("k_temporal_plan", 0.0)
                if t_bytes is not None:
                    t_bytes += traffic.get("k_temporal_plan", 0)
            # (an event pair around a kernel adds about 3 us to what the trace shows for the kernel alone)
            if t_bytes is not None and there_us is not None and avg_ms > 0 and \
                    abs(there_us - avg_ms * 1e3) > 0.1 * avg_ms * 1e3 + 3.0:
                t_bytes = None      # the counter run's kernel took another time than this one: not the same code path
                traffic_note = f"{traffic_note}: {name} ran {there_us:.1f} us there, {avg_ms * 1e3:.1f} us here"
            kernels[name] = {"avg_ms": avg_ms, "launches": n, "alg_bytes": nbytes, "traffic_bytes": t_bytes,
                             "GBps": nbytes / (avg_ms * 1e-3) / 1e9 if avg_ms > 0 else None}
        dom = max(kernels, key=lambda kk: kernels[kk]["avg_ms"])
        achieved = kernels[dom]["GBps"]
        path_bytes = N * D * esz + K * D * esz + 9 * N + 8 * K
        step_s = median_ms * 1e-3
        path = {"alg_bytes_per_step": path_bytes, "whole_path_GBps": path_bytes / step_s / 1e9,
                "whole_path_frac_of_peak": path_bytes / step_s / 1e9 / HBM_PEAK_GBS}
        if traffic and all(v["traffic_bytes"] is not None for v in kernels.values()):
            tot = sum(traffic.values())      # every kernel of the step that moves more than 2 MB
            path.update(traffic_bytes_per_step=tot, measured_GBps=tot / step_s / 1e9,
                        measured_frac_of_peak=tot / step_s / 1e9 / HBM_PEAK_GBS)
        return {"keep": keep, "cell_dots_level": level, "value": N / step_s / 1e6, "ms_per_step": median_ms,
                "ms_per_step_wall_mean": elapsed / args.steps * 1e3, "ms_per_step_min": per_step[0],
                "ms_per_step_max": per_step[-1], "kept_tokens": K, "kept_fraction": K / N,
                "roofline": {"bound": "hbm", "kernel": dom, "achieved": achieved, "peak": HBM_PEAK_GBS,
                             "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS if achieved else None,
                             "traffic": kernels[dom]["traffic_bytes"], "traffic_source": traffic_note,
                             "alg_bytes_per_launch": kernels[dom]["alg_bytes"], "kernels": kernels},
                "path": path}

    runs = [measure(k) for k in budgets]

    def two_streams(keep):
        """The same K steps, issued alternately on two library contexts with a stream, a workspace and output buffers
        each (default stream priority): the latency-bound integer kernels of one video then run beside the feature
        passes of the other, as they would in a server that merges one video per stream. Whole-job rate by the host
        clock between two device-wide synchronisations; never the headline value."""
        lanes = []
        for _ in range(2):
            st = torch.cuda.Stream(device=dev)
            c = lib.Sttm(0, stream_ptr=st.cuda_stream)
            c.sttm_set_match_mode({"first_passing": 0, "topleft_only": 1, "most_similar": 2}[args.match])
            c.sttm_set_output_order({"raster": 0, "zscan": 1}[args.order])
            c.sttm_set_cell_dots(dots_level(keep))
            c.ensure_workspace(B, T, H, W, D, dt, R)
            bufs = dict(node_map=torch.empty_like(node_map), node_level=torch.empty_like(node_level),
                        cluster=torch.empty_like(cluster), merged=torch.empty_like(merged),
                        counts=torch.empty_like(counts), out_ids=torch.empty_like(out_ids),
                        offsets=torch.zeros_like(offsets))
            lanes.append((c, bufs))
        torch.cuda.synchronize()

        def lane_step(i, c, b):
            xin = xs[i % copies]
            if budget_mode:
                c.sttm_spatial_stats(xin, dt, B, T, H, W, D, R)
                c.sttm_budget_threshold(lib.STTM_STAGE_SPATIAL, keep, want_tau=False)
                c.sttm_spatial_quadtree(xin, dt, B, T, H, W, D, R, None, b["node_map"], b["node_level"])
                c.sttm_temporal_stats(xin, b["node_map"], b["node_level"])
                c.sttm_budget_threshold(lib.STTM_STAGE_TEMPORAL, keep, want_tau=False)
                c.sttm_temporal_merge(xin, b["node_map"], b["node_level"], None, b["cluster"])
            else:
                c.sttm_spatial_quadtree(xin, dt, B, T, H, W, D, R, [cfg.tau_s], b["node_map"], b["node_level"])
                c.sttm_temporal_merge(xin, b["node_map"], b["node_level"], [cfg.tau_t], b["cluster"])
            c.sttm_reduce(xin, b["cluster"], None if args.no_node_sums else b["node_map"],
                          None if args.no_node_sums else b["node_level"], dt, N, b["merged"], b["counts"],
                          b["out_ids"], b["offsets"], want_n=False)

        for i in range(2 * max(1, args.warmup)):
            lane_step(i, *lanes[i % 2])
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(args.steps):
            lane_step(i, *lanes[i % 2])
        torch.cuda.synchronize()
        elapsed = time.perf_counter() - t0
        ks = [int(b["offsets"][B].item()) for _, b in lanes]
        for (c, b), k in zip(lanes, ks):
            assert int(b["counts"][:k].sum().item()) == N, "member counts do not add up to the number of input tokens"
            c.close()
        return {"keep": keep, "streams": 2, "steps": args.steps, "ms_per_step": elapsed / args.steps * 1e3,
                "value": N * args.steps / elapsed / 1e6, "unit": "Mtok/s", "kept_tokens": ks,
                "timing": "host clock around all steps, device-wide synchronisation on both sides"}

    overlapped = None if args.no_two_streams else two_streams(budgets[0])
    if args.calibrate_copy:
        merged.view(-1)[:x.numel()].copy_(x.view(-1))
        torch.cuda.synchronize()
    head = runs[0]
    keep = budgets[0]
    out = {
        "metric": "input visual tokens merged/sec (Mtok/s) at D=3584 bf16; achieved HBM GB/s vs peak",
        "value": head["value"],
        "unit": "Mtok/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": head["ms_per_step"],
        "timing": "median of the timed steps, each bracketed by HIP events on the library's stream; "
                  "ms_per_step_wall_mean is the host clock around all of them",
        "ms_per_step_wall_mean": head["ms_per_step_wall_mean"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": {lib.STTM_BF16: "bf16", lib.STTM_F16: "f16"}.get(dt, "f32"), "data": "synthetic",
        "config": {"workload": f"configs[{args.config}] {cfg.name}: B={B} T={T} grid={H}x{W} D={D} "
                               f"{cfg.dtype}, " + (f"budget keep={keep}" if budget_mode else
                                                   f"tau_s={cfg.tau_s} tau_t={cfg.tau_t}")
                               + (f", root_grid={R}" if R != 1 else "")
                               + (f", match={args.match}" if args.match != "first_passing" else "")
                               + (f", order={args.order}" if args.order != "raster" else "")
                               + (", with position indices" if args.positions else "")
                               + (", separate spatial and temporal passes" if args.no_cell_dots else "")
                               + (", block dot products in the spatial pass" if head["cell_dots_level"] == 2 else ""),
                   "tokens": N, "kept_tokens": head["kept_tokens"], "kept_fraction": head["kept_fraction"],
                   "generate_s": gen_s, "input_copies": copies},
        "roofline": head["roofline"],
        "path": head["path"],
        "paper_context": "end-to-end prefill speed-up reported by the paper on 1xA100 80G (LLaVA-Video-7B): "
                         "about 2x at a 50% budget, about 3x at 30%; the merge path alone is not timed there",
    }
    if len(runs) > 1:   # the workload's other budgets, each measured the same way (warm-up, then the same number of steps)
        out["budgets"] = {f"keep={r['keep']}": r for r in runs[1:]}
    if overlapped is not None:
        out["two_streams"] = overlapped
    if cpu is not None:
        out["cpu_baseline"], out["cpu_baseline_all_cores"] = cpu
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
