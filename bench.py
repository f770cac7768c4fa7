#!/usr/bin/env python3
"""Benchmark of the DSVT hot path on one MI355X.

A step = the whole hot path on one synthetic 30,000-pillar frame (468 x 468 x 1 grid, bf16,
C = 192, 8 heads, tau = 36, windows 12 x 12 x 1): four set partitions (2 window shifts x 2 axes, one call)
and four DSVT blocks (8 layers).  Inputs are resident in HBM before the timed region.  Prints one
JSON line: voxels/s, ms/frame, the roofline of the dominant kernel (per-kernel time from hipEvent
pairs around every launch) and the CPU oracle timed on the host cores on one frame.
"""
import argparse
import json
import sys
import time

import numpy as np


# HBM bytes one launch of the layer kernel moves on this workload, from rocprofv3 FETCH_SIZE and
# WRITE_SIZE (KiB per dispatch, each scaled by its reading for a plain 256 MiB copy); the
# measurement and its commands are in profiles/hbm_traffic_pillar_frame.md.
LAYER_HBM_BYTES_PER_LAUNCH = 33962 * 1024      # 19,253 KiB fetched + 14,709 KiB written


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--no-cpu-baseline", action="store_true", help="skip timing the CPU oracle")
    ap.add_argument("--no-graph", action="store_true", help="time eager launches instead of a captured HIP graph")
    ap.add_argument("--pmc-calibration", action="store_true",
                    help="also run one plain 256 MiB device copy (a kernel of known traffic, to scale rocprofv3's "
                         "FETCH_SIZE / WRITE_SIZE readings)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build is single-GPU by design (frames shard across GPUs with no communication); "
              "run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    import synth
    import paper_2301_06051_amd as dsvt

    torch.cuda.set_device(0)
    cid = 2
    cfg = synth.CONFIGS[cid]
    C, tau, N = cfg["C"], cfg["tau"], cfg["n"]
    coords = synth.make_frame(cid)
    x_np = synth.make_features(33, N, C, cfg["dtype"])
    w_np = [[synth.make_layer_weights(200 + 2 * b + a, C, cfg["heads"], cfg["hidden"], cfg["win"], cfg["dtype"])
             for a in (0, 1)] for b in range(cfg["blocks"])]

    cd = torch.as_tensor(coords).cuda()
    x0 = torch.as_tensor(x_np).cuda().to(torch.bfloat16).contiguous()
    buf = torch.empty_like(x0)
    layers = [[dsvt.LayerWeights(w) for w in pair] for pair in w_np]
    pcfgs = {sh: dsvt.part_cfg(cfg["grid"], cfg["win"], sh, tau, cfg["batch"], 0) for sh in cfg["shifts"]}
    maps = {sh: dsvt.SetMapsXY(pc, N) for sh, pc in pcfgs.items()}       # X- and Y-axis maps of each window shift
    ws = torch.empty((max(dsvt.dsvt_block_workspace_size(layers[0][0], N), 1),), dtype=torch.uint8, device="cuda")

    # The partitions of both window shifts, each in both axes, go through one chain of three launches
    # ahead of the blocks; everything is on one stream.
    shifts = list(cfg["shifts"])

    def step():
        dsvt.dsvt_partition_xy_multi([pcfgs[sh] for sh in shifts], cd, [maps[sh] for sh in shifts])
        src = x0
        for b, pair in enumerate(layers):
            sh = shifts[b % len(shifts)]
            dsvt.dsvt_block(pair, maps[sh], cd, src, x_out=buf, ws=ws)
            src = buf

    if args.pmc_calibration:
        cal_src = torch.zeros(64 * 1024 * 1024, dtype=torch.float32, device="cuda")
        cal_dst = torch.empty_like(cal_src)
        cal_dst.copy_(cal_src)
        torch.cuda.synchronize()
        del cal_src, cal_dst

    step()
    torch.cuda.synchronize()
    eager_out = buf.clone()
    n_sets = {sh: int(maps[sh][0].n_sets.item()) for sh in maps}
    status = max(int(m.status.item()) for ms in maps.values() for m in ms)
    assert status == 0, f"partition status {status}"

    use_graph = not args.no_graph
    run = step
    if use_graph:
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            step()
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            step()
        for _ in range(3):                       # replays must reproduce the eager result bit for bit
            buf.zero_()
            graph.replay()
            torch.cuda.synchronize()
            assert torch.equal(buf, eager_out), "graph replay differs from eager launches"
        run = graph.replay

    for _ in range(args.warmup):
        run()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        run()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt / args.steps * 1e3

    # Per-kernel time: the same steps again, eagerly, with an event pair around every launch.
    launches_per_step = 3 + 4 * 2
    prof_steps = min(args.steps, 50)
    dsvt.prof_enable(launches_per_step * prof_steps)
    for _ in range(prof_steps):
        step()
    torch.cuda.synchronize()
    prof = dsvt.prof_collect()
    per_launch_us = {k: 1e3 * ms / n for k, (ms, n) in prof.items() if n}
    per_step_ms = {k: ms / prof_steps for k, (ms, n) in prof.items() if n}

    # Roofline of the dominant kernel, the fused layer.  Algorithmic flops per voxel per layer
    # (duplicate-row and tile-padding work not counted): 16 C^2 + 4 tau C rho.
    rho = np.mean([n_sets[cfg["shifts"][b % len(cfg["shifts"])]] for b in range(cfg["blocks"])]) * tau / N
    flops = {"layer": N * (16 * C * C + 4 * tau * C * rho)}
    dom = "layer"
    achieved = flops[dom] / (per_launch_us[dom] * 1e-6) / 1e12
    peak = 2500.0
    roofline = {"bound": "mfma", "kernel": dom, "achieved": round(achieved, 2), "peak": peak, "unit": "TFLOP/s",
                "frac": round(achieved / peak, 5), "traffic": LAYER_HBM_BYTES_PER_LAUNCH,
                "avg_launch_us": round(per_launch_us[dom], 2), "flops_per_launch": flops[dom]}

    cpu = None
    if not args.no_cpu_baseline:
        from threadpoolctl import threadpool_info
        from oracle import dsvt_oracle as orc
        t0 = time.perf_counter()
        orc.stack(w_np, coords, x_np, cfg["grid"], cfg["win"], cfg["shifts"], tau)
        cdt = time.perf_counter() - t0
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
        cpu = {"value": round(N / cdt, 1), "unit": "voxels/s", "cores": cores, "kind": "oracle",
               "sample": f"one full frame of the same workload ({N} voxels, 8 layers, 4 partitions), {cdt:.1f} s"}

    line = {
        "metric": "voxels/sec through the 4-block DSVT stack (partition + set attention); ms/frame 4-block",
        "value": round(N / (dt / args.steps), 1), "unit": "voxels/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "configs[1]: 468x468x1 pillar frame, 30000 voxels, C=192, 8 heads, tau=36, "
                               "win 12x12x1, 4 blocks x 2 layers, shift (6,6,0) on odd blocks",
                   "launch": "hip_graph" if use_graph else "eager", "n_sets": {"shift" + "_".join(map(str, k)): v for k, v in n_sets.items()}, "rho": round(float(rho), 4)},
        "ms_per_frame": round(ms_per_step, 4),
        "kernel_ms_per_step": {k: round(v, 4) for k, v in per_step_ms.items()},
        "kernel_us_per_launch": {k: round(v, 2) for k, v in per_launch_us.items()},
        "roofline": roofline, "cpu_baseline": cpu,
    }
    print(json.dumps(line))


if __name__ == "__main__":
    main()
