#!/usr/bin/env python3
"""Benchmark of the DSVT hot path on one MI355X.

A step = the whole hot path on one synthetic 30,000-pillar frame (468 x 468 x 1 grid, bf16,
C = 192, 8 heads, tau = 36, windows 12 x 12 x 1): four set partitions (2 window shifts x 2 axes, one call)
and four DSVT blocks (8 layers).  Inputs are resident in HBM before the timed region.  Prints one
JSON line: voxels/s, ms/frame, the roofline of the dominant kernel (per-kernel time from hipEvent
pairs around every launch) and the CPU oracle timed on the host cores on one frame.

--workload names another of the synthetic workloads instead (the same JSON line, no CPU baseline):
voxel = the 120,000-voxel frame (2 blocks), skewed = the 4-frame batch of 200,000 voxels each
(4 blocks), hybrid = the pillar frame with blocks alternating 12 x 12 and shifted 24 x 24 windows,
dsvtv = the voxel variant's four stages with pooling along z between them, pool = attention-style 3D
pooling of the voxel frame, bev = bird's-eye-view scatter of the pillar frame, vfe = points to pillar rows.
"""
import argparse
import hashlib
import json
import os
import sys
import time

import numpy as np


ROOT = os.path.dirname(os.path.abspath(__file__))
# HBM bytes one launch of the layer kernel moves, per workload: rocprofv3 FETCH_SIZE and WRITE_SIZE readings (KiB
# per dispatch, each scaled by its reading for a plain 256 MiB copy) kept in a small text file beside the
# summaries they come from.  Every line carries the hash of the kernel sources it was measured with: a reading
# taken with other sources is not reported.
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "k_layer_hbm_traffic.txt")
LAYER_SOURCES = ("layer.hip", "mma.h")

STACKS = {"frame": 2, "voxel": 3, "skewed": 5, "nuscenes": 6, "hybrid": 2}  # workload -> synth config id


def layer_source_hash():
    h = hashlib.sha256()
    for f in LAYER_SOURCES:
        with open(os.path.join(ROOT, "paper_2301_06051_amd", "csrc", f), "rb") as fh:
            h.update(fh.read())
    return h.hexdigest()[:16]


def layer_traffic(workload):
    """(bytes per launch of the layer kernel or None, a note saying where the figure is from or why there is none)."""
    try:
        rows = [l.split() for l in open(TRAFFIC_FILE) if l.strip() and not l.startswith("#")]
    except OSError:
        return None, "no traffic file"
    for r in rows:
        kv = dict(f.split("=", 1) for f in r)
        if kv.get("workload") == workload:
            if kv.get("sources") != layer_source_hash():
                return None, f"the reading at commit {kv.get('commit')} was taken with other kernel sources"
            return (int(kv["fetch_kib"]) + int(kv["write_kib"])) * 1024, f"profiles/k_layer_hbm_traffic.txt, commit {kv.get('commit')}"
    return None, "not measured for this workload"


SETTLE_S = 0.2       # untimed steps before the warm-up: the GPU's clocks take some 100 ms of load to settle after the set-up's idle gaps


def timed(run, steps, warmup):
    import torch
    t_end = time.perf_counter() + SETTLE_S
    while time.perf_counter() < t_end:
        for _ in range(10):
            run()
        torch.cuda.synchronize()
    for _ in range(warmup):
        run()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        run()
    torch.cuda.synchronize()
    return time.perf_counter() - t0


def percentiles(run, steps):
    """Per-step time from an event pair around every step (steps still queue back to back): p10 / p50 / p90 in ms."""
    import torch
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
    for a, b in ev:
        a.record()
        run()
        b.record()
    torch.cuda.synchronize()
    ms = np.sort([a.elapsed_time(b) for a, b in ev])
    return {k: round(float(ms[min(int(q * steps), steps - 1)]), 4) for k, q in (("p10", 0.1), ("p50", 0.5), ("p90", 0.9))}


def capture(step, check):
    """step() captured into a HIP graph; three replays must pass check()."""
    import torch
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    for _ in range(3):
        check(graph.replay)
    return graph.replay


def per_kernel(step, launches_per_step, steps):
    """The same steps again, eagerly, with an event pair around every launch."""
    import torch
    import paper_2301_06051_amd as dsvt
    dsvt.prof_enable(launches_per_step * steps)
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    prof = dsvt.prof_collect()
    return ({k: 1e3 * ms / n for k, (ms, n) in prof.items() if n}, {k: ms / steps for k, (ms, n) in prof.items() if n})


def kind_name(kind):
    win, shift = kind
    return "win" + "x".join(map(str, win)) + "_shift" + "_".join(map(str, shift))


def time_one_block(args, use_graph, n_voxels, maps_xy, buf, fns):
    """One DSVT block on its own (the paper's per-block latency): both rotated partitions of one window
    configuration plus the block's two layers, the block alone with the maps reused, the partitions alone."""
    import torch
    one = {}
    for key, fn in fns:
        fn()
        torch.cuda.synchronize()
        watched = maps_xy.y.voxel_slot if key == "partition_xy_only" else buf
        ref = watched.clone()

        def check_one(replay, watched=watched, ref=ref):
            watched.zero_()
            replay()
            torch.cuda.synchronize()
            assert torch.equal(watched, ref), "graph replay differs from eager launches"

        t = timed(capture(fn, check_one) if use_graph else fn, args.steps, args.warmup) / args.steps
        one[key] = {"ms": round(t * 1e3, 4), "voxels_per_s": round(n_voxels / t, 1)}
    return one


def stack_workload(args, name):
    import torch
    import synth
    import paper_2301_06051_amd as dsvt
    cid = STACKS[name]
    cfg = synth.CONFIGS[cid]
    C, tau = cfg["C"], cfg["tau"]
    coords = synth.make_frame(cid)
    N = len(coords)
    x_np = synth.make_features(33, N, C, cfg["dtype"])
    # one (window, shift) per block: the configuration's window with the shift on every other block, or (hybrid)
    # 12 x 12 windows alternating with 24 x 24 windows shifted by half of theirs (Sec. 3.2, hybrid window partition)
    if name == "hybrid":
        kinds = [((12, 12, 1), (0, 0, 0)), ((24, 24, 1), (12, 12, 0))]
    else:
        kinds = [(tuple(cfg["win"]), tuple(sh)) for sh in cfg["shifts"]]
    plan = [kinds[b % len(kinds)] for b in range(cfg["blocks"])]
    w_np = [[synth.make_layer_weights(200 + 2 * b + a, C, cfg["heads"], cfg["hidden"], plan[b][0], cfg["dtype"])
             for a in (0, 1)] for b in range(cfg["blocks"])]

    cd = torch.as_tensor(coords).cuda()
    x0 = torch.as_tensor(x_np).cuda().to(torch.bfloat16).contiguous()
    buf = torch.empty_like(x0)
    layers = [[dsvt.LayerWeights(w) for w in pair] for pair in w_np]
    pcfgs = {k: dsvt.part_cfg(cfg["grid"], k[0], k[1], tau, cfg["batch"], 0) for k in kinds}
    maps = {k: dsvt.SetMapsXY(pc, N) for k, pc in pcfgs.items()}         # X- and Y-axis maps of each window kind
    ws = torch.empty((max(dsvt.dsvt_block_workspace_size(layers[0][0], N), 1),), dtype=torch.uint8, device="cuda")

    # The partitions of both window shifts, each in both axes, go through one chain of launches
    # ahead of the blocks; everything is on one stream.
    def step():
        dsvt.dsvt_partition_xy_multi([pcfgs[k] for k in kinds], cd, [maps[k] for k in kinds])
        src = x0
        for b, pair in enumerate(layers):
            dsvt.dsvt_block(pair, maps[plan[b]], cd, src, x_out=buf, ws=ws)
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
    n_sets = {k: int(maps[k][0].n_sets.item()) for k in maps}
    status = max(int(m.status.item()) for ms in maps.values() for m in ms)
    assert status == 0, f"partition status {status}"

    def check(replay):                           # replays must reproduce the eager result bit for bit
        buf.zero_()
        replay()
        torch.cuda.synchronize()
        assert torch.equal(buf, eager_out), "graph replay differs from eager launches"

    use_graph = not args.no_graph
    run = capture(step, check) if use_graph else step
    dt = timed(run, args.steps, args.warmup)
    step_ms = percentiles(run, min(args.steps, 100))

    # Optional: a serving loop keeps two frames in flight, each with its own maps and feature buffer on a stream of
    # its own, so that one frame's partition and the ramp and tail of its launches are filled by the other's tiles.
    # Every step is still one whole frame; steps that share buffers are on the same stream.  Reported beside the
    # single-stream figures, never instead of them.
    in_flight = None
    if args.frames_in_flight == 2 and use_graph:
        maps_b = {k: dsvt.SetMapsXY(pc, N) for k, pc in pcfgs.items()}
        buf_b = torch.empty_like(x0)

        def step_b():
            dsvt.dsvt_partition_xy_multi([pcfgs[k] for k in kinds], cd, [maps_b[k] for k in kinds])
            src = x0
            for b, pair in enumerate(layers):
                dsvt.dsvt_block(pair, maps_b[plan[b]], cd, src, x_out=buf_b, ws=ws)
                src = buf_b

        def check_b(replay):
            buf_b.zero_()
            replay()
            torch.cuda.synchronize()
            assert torch.equal(buf_b, eager_out), "graph replay differs from eager launches"

        streams = [torch.cuda.Stream(), torch.cuda.Stream()]
        with torch.cuda.stream(streams[1]):
            run_b = capture(step_b, check_b)
        torch.cuda.synchronize()
        runs = (run, run_b)

        def pump(k):
            with torch.cuda.stream(streams[k % 2]):
                runs[k % 2]()

        for k in range(args.warmup):
            pump(k)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for k in range(args.steps):
            pump(k)
        torch.cuda.synchronize()
        t2 = (time.perf_counter() - t0) / args.steps
        buf.zero_(); buf_b.zero_()
        pump(0); pump(1)
        torch.cuda.synchronize()
        assert torch.equal(buf, eager_out) and torch.equal(buf_b, eager_out), "pipelined frames differ from eager launches"
        in_flight = {"frames": 2, "ms_per_frame": round(t2 * 1e3, 4), "voxels_per_s": round(N / t2, 1)}

    # Every window kind of the plan is timed (the shape of the paper's per-block latency table, Sec. 4.4).
    one = {}
    for bi, kind in enumerate(kinds):
        def one_block(kind=kind, bi=bi):
            dsvt.dsvt_partition_xy(pcfgs[kind], cd, out=maps[kind])
            dsvt.dsvt_block(layers[bi], maps[kind], cd, x0, x_out=buf, ws=ws)

        def block_only(kind=kind, bi=bi):
            dsvt.dsvt_block(layers[bi], maps[kind], cd, x0, x_out=buf, ws=ws)

        def partition_only(kind=kind):
            dsvt.dsvt_partition_xy(pcfgs[kind], cd, out=maps[kind])

        one[kind_name(kind)] = time_one_block(args, use_graph, N, maps[kind], buf,
                                   (("partition_and_block", one_block), ("block_maps_reused", block_only),
                                    ("partition_xy_only", partition_only)))
    step()                                                   # (every kind's maps back to the frame's own)
    launches = 6 * len(kinds) + 2 * cfg["blocks"]           # (an upper bound: small frames take 3 partition launches)
    per_launch_us, per_step_ms = per_kernel(step, launches, min(args.steps, 50))

    # The layer kernel's launch duration in the configuration the frame is timed in: the frame's layer launches alone
    # (maps as the partitions left them), replayed from a graph, an event pair around every replay, / launches.  (The
    # event pairs around eager launches above also span the gap to the next eager launch, 2-3 us that a replayed
    # frame does not have; that figure is kept beside it.)
    def layers_only():
        src = x0
        for b, pair in enumerate(layers):
            dsvt.dsvt_block(pair, maps[plan[b]], cd, src, x_out=buf, ws=ws)
            src = buf

    layer_us_eager = per_launch_us["layer"]
    layer_us = layer_us_eager
    if use_graph:
        run_layers = capture(layers_only, check)
        timed(run_layers, 0, args.warmup)
        ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(min(args.steps, 100))]
        for a, b in ev:
            a.record()
            run_layers()
            b.record()
        torch.cuda.synchronize()
        layer_us = 1e3 * float(np.mean([a.elapsed_time(b) for a, b in ev])) / (2 * cfg["blocks"])

    # Roofline of the dominant kernel, the fused layer.  Algorithmic flops per voxel per layer
    # (duplicate-row and tile-padding work not counted): 16 C^2 + 4 tau C rho.
    rho = np.mean([n_sets[k] for k in plan]) * tau / N
    flops = N * (16 * C * C + 4 * tau * C * rho)
    achieved = flops / (layer_us * 1e-6) / 1e12
    traffic, traffic_from = layer_traffic(name)
    roofline = {"bound": "mfma", "kernel": "layer", "achieved": round(achieved, 2), "peak": 2500.0, "unit": "TFLOP/s",
                "frac": round(achieved / 2500.0, 5), "traffic": traffic, "traffic_from": traffic_from,
                "avg_launch_us": round(layer_us, 2), "avg_launch_us_eager": round(layer_us_eager, 2),
                "timing": (f"hipEvent pair around a graph replay of the frame's {2 * cfg['blocks']} layer launches / {2 * cfg['blocks']}"
                           if use_graph else "hipEvent pairs around eager launches"),
                "flops_per_launch": flops}

    # The partition chain against the HBM roofline: algorithmic bytes per voxel and map = 16 B of coordinates read,
    # 4 rho B of set_inds, 4 B of voxel_slot and 8 B of descriptor row written; latency-bound at these sizes.
    n_maps = 2 * len(kinds)
    part_bytes = N * n_maps * (16 + 4 * rho + 4 + 8)
    part_us = sum(v for k, v in per_launch_us.items() if k.startswith("part_"))
    partition_roofline = {"bound": "hbm", "kernel": "partition chain (" + ", ".join(sorted(k for k in per_launch_us if k.startswith("part_"))) + ")",
                          "achieved": round(part_bytes / (part_us * 1e-6) / 1e9, 1), "peak": 8000.0, "unit": "GB/s",
                          "frac": round(part_bytes / (part_us * 1e-6) / 8e12, 5), "traffic": None, "avg_launch_us": round(part_us, 2),
                          "bytes_per_launch": int(part_bytes)}

    cpu = None
    if name == "frame" and not args.no_cpu_baseline:
        from threadpoolctl import threadpool_info, threadpool_limits
        from oracle import dsvt_oracle as orc
        t0 = time.perf_counter()
        orc.stack(w_np, coords, x_np, cfg["grid"], cfg["win"], cfg["shifts"], tau)
        cdt = time.perf_counter() - t0
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
        cpu = {"value": round(N / cdt, 1), "unit": "voxels/s", "cores": cores, "kind": "oracle",
               "sample": f"one full frame of the same workload ({N} voxels, 8 layers, 4 partitions), {cdt:.1f} s"}
        # the oracle on one thread: the tiny pillar frame (configs[0], fp32, one block) and the full frame again
        with threadpool_limits(limits=1):
            for sid in (1, 2):
                c1 = synth.CONFIGS[sid]
                co1 = synth.make_frame(sid)
                x1 = synth.make_features(33, len(co1), c1["C"], c1["dtype"])
                w1 = [[synth.make_layer_weights(200 + 2 * b + a, c1["C"], c1["heads"], c1["hidden"], c1["win"], c1["dtype"])
                       for a in (0, 1)] for b in range(c1["blocks"])]
                t0 = time.perf_counter()
                orc.stack(w1, co1, x1, c1["grid"], c1["win"], c1["shifts"], c1["tau"])
                t1 = time.perf_counter() - t0
                cpu[f"single_thread_configs[{sid - 1}]"] = {"voxels_per_s": round(len(co1) / t1, 1), "seconds": round(t1, 2),
                                                           "voxels": len(co1), "blocks": c1["blocks"]}

    g, nb = cfg["grid"], cfg["blocks"]
    wins = " alternating with ".join(f"win {k[0][0]}x{k[0][1]}x{k[0][2]} shift ({k[1][0]},{k[1][1]},{k[1][2]})" for k in kinds)
    workload = (f"{'configs[' + str(cid - 1) + ']' if cid <= 5 else 'nuScenes shape'}: {g[0]}x{g[1]}x{g[2]} {'pillar' if g[2] == 1 else 'voxel'} frame"
                f"{'s, batch ' + str(cfg['batch']) if cfg['batch'] > 1 else ''}, {N} voxels, C={C}, {cfg['heads']} heads, "
                f"tau={tau}, {nb} blocks x 2 layers, {wins}")
    # `value` is the frame's voxels over the time of the whole stack (every partition and every block of one frame:
    # one step); the figure for a single block with its own partitions is one_block[...]["partition_and_block"].
    return {
        "metric": "voxels/sec through a DSVT block (partition+set attention); ms/frame 4-block" if nb == 4 else
                  f"voxels/sec through a DSVT block (partition+set attention); ms/frame {nb}-block",
        "value": round(N / (dt / args.steps), 1), "unit": "voxels/s", "dtype": "bf16",
        "config": {"workload": workload, "launch": "hip_graph" if use_graph else "eager",
                   "value_is": f"voxels of one frame / time of the whole {nb}-block frame ({n_maps} partitions + {2 * nb} layers)",
                   "n_sets": {kind_name(k): v for k, v in n_sets.items()},
                   "rho_by_window": {kind_name(k): round(v * tau / N, 4) for k, v in n_sets.items()}, "rho": round(float(rho), 4)},
        "ms_per_frame": round(dt / args.steps * 1e3, 4), "step_ms": step_ms, "one_block": one, "two_frames_in_flight": in_flight,
        "kernel_ms_per_step": {k: round(v, 4) for k, v in per_step_ms.items()},
        "kernel_us_per_launch": {k: round(v, 2) for k, v in per_launch_us.items()},
        "roofline": roofline, "partition_roofline": partition_roofline, "cpu_baseline": cpu,
    }, dt


def pool_workload(args):
    """Sec. 3.3: attention-style 3D pooling of the 120,000-voxel frame over 1 x 1 x 4 regions."""
    import torch
    import synth
    import paper_2301_06051_amd as dsvt
    cid = 4
    cfg = synth.CONFIGS[cid]
    C, pool = cfg["C"], cfg["pool"]
    coords = synth.make_frame(cid)
    N = len(coords)
    cd = torch.as_tensor(coords).cuda()
    x = torch.as_tensor(synth.make_features(35, N, C, cfg["dtype"])).cuda().to(torch.bfloat16).contiguous()
    # keys / values = the region's occupied voxels, as the workload is worded (the paper's best variant, which keeps
    # the empty cells as keys, is --pool-keep-empty)
    mask_empty = 0 if args.pool_keep_empty else 1
    pw = dsvt.PoolWeights(synth.make_pool_weights(91, C, cfg["heads"], cfg["dtype"]), cfg["grid"], pool, cfg["batch"], mask_empty)
    ws = torch.empty((max(dsvt.dsvt_attn_pool_workspace_size(pw, N), 1),), dtype=torch.uint8, device="cuda")
    out = (torch.zeros((N, 4), dtype=torch.int32, device="cuda"), torch.zeros_like(x),
           torch.zeros((1,), dtype=torch.int32, device="cuda"), torch.zeros((1,), dtype=torch.int32, device="cuda"))

    dsvt.dsvt_attn_pool(pw, cd, x, out=out, ws=ws)
    torch.cuda.synchronize()
    assert int(out[3].item()) == 0
    M = int(out[2].item())                       # the host sizes the block on the pooled voxels with it (fixed input)
    # the rotated layer pair that follows on the pooled grid
    pgrid = tuple(g // p for g, p in zip(cfg["grid"], pool))
    pc = dsvt.part_cfg(pgrid, cfg["win"], (0, 0, 0), cfg["tau"], cfg["batch"], 0)
    pmaps = dsvt.SetMapsXY(pc, M)
    layers = [dsvt.LayerWeights(synth.make_layer_weights(92 + a, C, cfg["heads"], cfg["hidden"], cfg["win"], cfg["dtype"]))
              for a in (0, 1)]
    y = torch.empty((M, C), dtype=torch.bfloat16, device="cuda")

    def step():
        dsvt.dsvt_attn_pool(pw, cd, x, out=out, ws=ws)
        dsvt.dsvt_partition_xy(pc, out[0][:M], out=pmaps)
        dsvt.dsvt_block(layers, pmaps, out[0][:M], out[1][:M], x_out=y)

    step()
    torch.cuda.synchronize()
    assert int(out[3].item()) == 0 and int(pmaps.x.status.item()) == 0
    ref, ref_y = out[1].clone(), y.clone()

    def check(replay):
        out[1].zero_(); y.zero_()
        replay()
        torch.cuda.synchronize()
        assert torch.equal(out[1], ref) and torch.equal(y, ref_y), "graph replay differs from eager launches"

    use_graph = not args.no_graph
    run = capture(step, check) if use_graph else step
    dt = timed(run, args.steps, args.warmup)
    per_launch_us, per_step_ms = per_kernel(step, 16, min(args.steps, 50))
    # K and V projections of the N occupied cells, Q and output projection of the M regions, 2 C^2 flops each
    flops = 2 * C * C * (2 * N + 2 * M)
    us = per_launch_us["pool_attention"]
    roofline = {"bound": "mfma", "kernel": "pool_attention", "achieved": round(flops / (us * 1e-6) / 1e12, 2), "peak": 2500.0,
                "unit": "TFLOP/s", "frac": round(flops / (us * 1e-6) / 2.5e15, 5), "traffic": None, "avg_launch_us": round(us, 2),
                "flops_per_launch": flops, "hbm_bytes_algorithmic": (N + M) * C * 2,
                "hbm_gbps_algorithmic": round((N + M) * C * 2 / (us * 1e-6) / 1e9, 1)}
    return {
        "metric": "input voxels/sec through attention-style 3D pooling and the rotated layer pair on the pooled grid",
        "value": round(N / (dt / args.steps), 1), "unit": "voxels/s", "dtype": "bf16",
        "config": {"workload": f"configs[3]: 468x468x32 voxel frame, {N} voxels -> {M} regions of {pool[0]}x{pool[1]}x{pool[2]} "
                               f"cells, C={C}, {cfg['heads']} heads, keys = {'all cells (empty ones as bias keys)' if mask_empty == 0 else 'occupied voxels'}; "
                               f"then one block (win 12x12x8, tau={cfg['tau']}) on the {M} pooled voxels",
                   "launch": "hip_graph" if use_graph else "eager"},
        "ms_per_frame": round(dt / args.steps * 1e3, 4),
        "kernel_ms_per_step": {k: round(v, 4) for k, v in per_step_ms.items()},
        "kernel_us_per_launch": {k: round(v, 2) for k, v in per_launch_us.items()},
        "roofline": roofline, "cpu_baseline": None,
    }, dt


def dsvtv_workload(args):
    """Appendix "Network Architecture", the voxel variant: four stages (one block each here) with windows
    12 x 12 x {32, 8, 2, 1}, tau = 48, the shift on every other stage, and attention-style pooling by {4, 4, 2}
    along z between the stages (Sec. 3.3), on the 120,000-voxel frame."""
    import torch
    import synth
    import paper_2301_06051_amd as dsvt
    C, heads, hidden, tau, xy, n = 192, 8, 384, 48, 468, 120000
    zs, strides = [32, 8, 2, 1], [4, 4, 2]
    coords = np.concatenate([np.zeros((n, 1), np.int64), synth.frame_radial(311, (xy, xy, 32), n)], 1).astype(np.int32)
    N = len(coords)
    cd0 = torch.as_tensor(coords).cuda()
    x0 = torch.as_tensor(synth.make_features(312, N, C, "bf16")).cuda().to(torch.bfloat16).contiguous()

    # One eager pass sizes every stage: the pooled voxel counts are fixed by the (fixed) input.
    stages, cd, xd = [], cd0, x0
    for st, z in enumerate(zs):
        grid, win, shift = (xy, xy, z), (12, 12, z), ((0, 0, 0) if st % 2 == 0 else (6, 6, 0))
        m = cd.shape[0]
        pc = dsvt.part_cfg(grid, win, shift, tau, 1, 0)
        maps = dsvt.SetMapsXY(pc, m)
        layers = [dsvt.LayerWeights(synth.make_layer_weights(320 + 2 * st + a, C, heads, hidden, win, "bf16")) for a in (0, 1)]
        y = torch.empty((m, C), dtype=torch.bfloat16, device="cuda")
        ws = torch.empty((max(dsvt.dsvt_block_workspace_size(layers[0], m), 1),), dtype=torch.uint8, device="cuda")
        stage = dict(pc=pc, maps=maps, layers=layers, y=y, ws=ws, cd=cd, x=xd, m=m, grid=grid, win=win)
        dsvt.dsvt_partition_xy(pc, cd, out=maps)
        dsvt.dsvt_block(layers, maps, cd, xd, x_out=y, ws=ws)
        if st < len(strides):
            pw = dsvt.PoolWeights(synth.make_pool_weights(340 + st, C, heads, "bf16"), grid, (1, 1, strides[st]), 1, 1)
            pws = torch.empty((max(dsvt.dsvt_attn_pool_workspace_size(pw, m), 1),), dtype=torch.uint8, device="cuda")
            out = (torch.zeros((m, 4), dtype=torch.int32, device="cuda"), torch.zeros((m, C), dtype=torch.bfloat16, device="cuda"),
                   torch.zeros((1,), dtype=torch.int32, device="cuda"), torch.zeros((1,), dtype=torch.int32, device="cuda"))
            dsvt.dsvt_attn_pool(pw, cd, y, out=out, ws=pws)
            torch.cuda.synchronize()
            assert int(out[3].item()) == 0
            mo = int(out[2].item())
            stage.update(pw=pw, pws=pws, out=out, m_out=mo)
            cd, xd = out[0][:mo], out[1][:mo]
        torch.cuda.synchronize()
        assert int(maps.x.status.item()) == 0
        stage["n_sets"] = int(maps.x.n_sets.item())
        stages.append(stage)

    def step():
        for s in stages:
            dsvt.dsvt_partition_xy(s["pc"], s["cd"], out=s["maps"])
            dsvt.dsvt_block(s["layers"], s["maps"], s["cd"], s["x"], x_out=s["y"], ws=s["ws"])
            if "pw" in s:
                dsvt.dsvt_attn_pool(s["pw"], s["cd"], s["y"], out=s["out"], ws=s["pws"])

    step()
    torch.cuda.synchronize()
    last = stages[-1]["y"]
    ref = last.clone()

    def check(replay):
        last.zero_()
        replay()
        torch.cuda.synchronize()
        assert torch.equal(last, ref), "graph replay differs from eager launches"

    use_graph = not args.no_graph
    run = capture(step, check) if use_graph else step
    dt = timed(run, args.steps, args.warmup)
    step_ms = percentiles(run, min(args.steps, 100))
    per_launch_us, per_step_ms = per_kernel(step, 64, min(args.steps, 50))
    # the layer kernel over the four stages: flops of all eight launches over their summed time
    flops = sum(2 * s["m"] * (16 * C * C + 4 * tau * C * (s["n_sets"] * tau / s["m"])) for s in stages)
    us = per_step_ms["layer"] * 1e3
    roofline = {"bound": "mfma", "kernel": "layer (8 launches, 4 stage sizes)", "achieved": round(flops / (us * 1e-6) / 1e12, 2),
                "peak": 2500.0, "unit": "TFLOP/s", "frac": round(flops / (us * 1e-6) / 2.5e15, 5), "traffic": None,
                "avg_launch_us": round(per_launch_us["layer"], 2), "flops_per_step": flops}
    return {
        "metric": "input voxels/sec through the voxel variant's four stages (partition + block per stage, attention-style "
                  "pooling between stages)",
        "value": round(N / (dt / args.steps), 1), "unit": "voxels/s", "dtype": "bf16",
        "config": {"workload": f"468x468x32 voxel frame, {N} voxels, C={C}, {heads} heads, tau={tau}; stages of one block with windows "
                               "12x12x{32,8,2,1}, shift (6,6,0) on stages 1 and 3, pooling 1x1x{4,4,2} between them",
                   "launch": "hip_graph" if use_graph else "eager",
                   "stages": [{"voxels": s["m"], "grid_z": s["grid"][2], "n_sets": s["n_sets"],
                               "rho": round(s["n_sets"] * tau / s["m"], 4)} for s in stages]},
        "ms_per_frame": round(dt / args.steps * 1e3, 4), "step_ms": step_ms,
        "kernel_ms_per_step": {k: round(v, 4) for k, v in per_step_ms.items()},
        "kernel_us_per_launch": {k: round(v, 2) for k, v in per_launch_us.items()},
        "roofline": roofline, "cpu_baseline": None,
    }, dt


def bev_workload(args):
    """Sec. 3.1: the pillar frame's rows scattered into the dense channels-last bird's-eye-view map."""
    import torch
    import synth
    import paper_2301_06051_amd as dsvt
    cfg = synth.CONFIGS[2]
    C = cfg["C"]
    coords = synth.make_frame(2)
    N = len(coords)
    cd = torch.as_tensor(coords).cuda()
    x = torch.as_tensor(synth.make_features(33, N, C, cfg["dtype"])).cuda().to(torch.bfloat16).contiguous()
    out = torch.empty((cfg["batch"], *cfg["grid"], C), dtype=torch.bfloat16, device="cuda")

    def step():
        dsvt.dsvt_bev_scatter(cd, x, cfg["batch"], cfg["grid"], out=out)

    step()                                       # (eager: the binding allocates the status word per call)
    torch.cuda.synchronize()
    dt = timed(step, args.steps, args.warmup)
    per_launch_us, per_step_ms = per_kernel(step, 2, min(args.steps, 50))
    nbytes = out.numel() * 2 + 2 * N * C * 2 + N * 16      # map zero-filled, rows read and written, coords read
    us = per_launch_us["bev_clear"] + per_launch_us["bev_scatter"]
    roofline = {"bound": "hbm", "kernel": "bev_clear + bev_scatter", "achieved": round(nbytes / (us * 1e-6) / 1e9, 1), "peak": 8000.0,
                "unit": "GB/s", "frac": round(nbytes / (us * 1e-6) / 8e12, 5), "traffic": None, "avg_launch_us": round(us, 2),
                "bytes_per_launch": nbytes}
    return {
        "metric": "voxels/sec scattered into the dense bird's-eye-view map", "value": round(N / (dt / args.steps), 1),
        "unit": "voxels/s", "dtype": "bf16",
        "config": {"workload": f"configs[1]: {N} voxel rows of C={C} into a 468x468x1 channels-last map", "launch": "eager"},
        "ms_per_frame": round(dt / args.steps * 1e3, 4),
        "kernel_ms_per_step": {k: round(v, 4) for k, v in per_step_ms.items()},
        "kernel_us_per_launch": {k: round(v, 2) for k, v in per_launch_us.items()},
        "roofline": roofline, "cpu_baseline": None,
    }, dt


def vfe_workload(args):
    """Sec. 3.1: a LiDAR-shaped point frame encoded into the pillar rows the first DSVT block takes."""
    import torch
    import synth
    import paper_2301_06051_amd as dsvt
    grid, lo, hi, size, C, f_in, P = (468, 468, 1), (-74.88, -74.88, -2.0), (74.88, 74.88, 4.0), (0.32, 0.32, 6.0), 192, 5, 180000
    pts, _ = synth.make_points(24, P, lo, hi, f_in=f_in)
    w, b = synth.make_vfe_weights(25, C, f_in)
    pd, wd, bd = torch.as_tensor(pts).cuda(), torch.as_tensor(w).cuda(), torch.as_tensor(b).cuda()
    vfe = dsvt.Vfe(grid, 1, lo, size, f_in, C, "bf16", P, 65536, wd, bd, True)

    def step():
        dsvt.dsvt_vfe(vfe, pd)

    step()
    torch.cuda.synchronize()
    N = int(vfe.n_voxels.item())
    assert int(vfe.status.item()) == 0
    ref_x, ref_c = vfe.x[:N].clone(), vfe.coords[:N].clone()

    def check(run):                                       # every replay must reproduce the eager result
        vfe.x.zero_(); vfe.coords.zero_(); vfe.n_voxels.zero_()
        run()
        torch.cuda.synchronize()
        assert int(vfe.n_voxels.item()) == N and torch.equal(vfe.x[:N], ref_x) and torch.equal(vfe.coords[:N], ref_c)

    graph = None if args.no_graph else capture(step, check)
    run = step if graph is None else graph
    dt = timed(run, args.steps, args.warmup)
    per_launch_us, per_step_ms = per_kernel(step, 2, min(args.steps, 50))
    nbytes = P * f_in * 4 + N * (C * 2 + 16)               # points read once, rows and coordinates written once
    us = per_launch_us["vfe_group"] + per_launch_us["vfe_reduce"]
    roofline = {"bound": "hbm", "kernel": "vfe_group (7 launches) + vfe_reduce", "achieved": round(nbytes / (us * 1e-6) / 1e9, 1),
                "peak": 8000.0, "unit": "GB/s", "frac": round(nbytes / (us * 1e-6) / 8e12, 5), "traffic": None,
                "avg_launch_us": round(us, 2), "bytes_per_launch": nbytes}
    return {
        "metric": "points/sec encoded into pillar rows", "value": round(P / (dt / args.steps), 1), "unit": "points/s", "dtype": "f32",
        "config": {"workload": f"{P} points ({f_in} floats each) over 468x468x1 pillars of 0.32 m -> {N} rows of C={C} bf16 "
                               "(linear map + ReLU + max)", "launch": "eager" if graph is None else "hip_graph"},
        "ms_per_frame": round(dt / args.steps * 1e3, 4),
        "kernel_ms_per_step": {k: round(v, 4) for k, v in per_step_ms.items()},
        "kernel_us_per_launch": {k: round(v, 2) for k, v in per_launch_us.items()},
        "roofline": roofline, "cpu_baseline": None,
    }, dt


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", choices=["frame", "voxel", "skewed", "nuscenes", "hybrid", "dsvtv", "pool", "bev", "vfe"], default="frame")
    ap.add_argument("--no-cpu-baseline", action="store_true", help="skip timing the CPU oracle")
    ap.add_argument("--no-graph", action="store_true", help="time eager launches instead of a captured HIP graph")
    ap.add_argument("--pool-keep-empty", action="store_true", help="pool workload: empty cells of a region stay keys (zero features)")
    ap.add_argument("--frames-in-flight", type=int, choices=[1, 2], default=1,
                    help="2: also time a loop that keeps two frames in flight on two streams (an extra field of the JSON "
                         "line; `value` and `ms_per_step` are always the single-stream figures)")
    ap.add_argument("--settle-ms", type=float, default=200.0,
                    help="untimed steps for this long before the warm-up steps of every timed loop (clock settling; 0 = none)")
    ap.add_argument("--pmc-calibration", action="store_true",
                    help="also run one plain 256 MiB device copy (a kernel of known traffic, to scale rocprofv3's "
                         "FETCH_SIZE / WRITE_SIZE readings)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build is single-GPU by design (frames shard across GPUs with no communication); "
              "run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    torch.cuda.set_device(0)
    global SETTLE_S
    SETTLE_S = args.settle_ms * 1e-3
    if args.workload in STACKS:
        body, dt = stack_workload(args, args.workload)
    elif args.workload == "dsvtv":
        body, dt = dsvtv_workload(args)
    elif args.workload == "pool":
        body, dt = pool_workload(args)
    elif args.workload == "vfe":
        body, dt = vfe_workload(args)
    else:
        body, dt = bev_workload(args)
    line = {"metric": body.pop("metric"), "value": body.pop("value"), "unit": body.pop("unit"), "n_gpus": 1,
            "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(dt / args.steps * 1e3, 4),
            "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": body.pop("dtype"), "data": "synthetic",
            "settle_ms": args.settle_ms}
    line.update(body)
    print(json.dumps(line))


if __name__ == "__main__":
    main()
