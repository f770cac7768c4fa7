"""Per-phase shader clocks of the layer kernel, from a library built with -DDSVT_PHASE_CLOCKS beside the product
library (csrc/phase_clock.h; the product library carries none of it).

    python -m paper_2301_06051_amd.phase_clocks --build      # here or on the GPU machine: compiles _build/libdsvt_phase.so
    python -m paper_2301_06051_amd.phase_clocks [--config 2]  # on the GPU: one block on the config's frame, a table

Thread 0 of every workgroup notes the clock at the phase boundaries (all behind workgroup barriers); the table gives
the mean over the workgroups of the last layer launch, and the same for the tiles of the first and the second half
of the launch order (tiles are launched longest first)."""
import argparse
import ctypes as C
import os
import sys

from . import build as _build

PHASE_LIB = _build.PHASE_LIB
PHASES = ["descriptor -> rows known", "gather -> rows in LDS", "Q, K, V projection", "attention", "out projection + LN",
          "MLP first matrix + GELU", "MLP second matrix + LN", "scatter"]


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--build", action="store_true")
    ap.add_argument("--config", type=int, default=2, help="synth.CONFIGS id (2: the benchmark's pillar frame)")
    ap.add_argument("--no-position-term", action="store_true", help="layers without the relative position table")
    args = ap.parse_args()
    if args.build:
        _build.build_library()
        _build.build_phase_library()
        return
    if not os.path.exists(PHASE_LIB):
        raise SystemExit(f"{PHASE_LIB} is missing: run with --build first")
    import numpy as np
    import torch
    from . import binding
    binding.LIB_PATH = PHASE_LIB                      # before the first call: this process uses the instrumented library
    import paper_2301_06051_amd as dsvt
    sys.path.insert(0, _build.ROOT)
    import synth
    cfg = synth.CONFIGS[args.config]
    coords = synth.make_frame(args.config)
    x = torch.as_tensor(synth.make_features(31, len(coords), cfg["C"], cfg["dtype"])).cuda()
    x = x.to(torch.bfloat16) if cfg["dtype"] == "bf16" else x
    cd = torch.as_tensor(coords).cuda()
    mk = lambda s: dsvt.LayerWeights(synth.make_layer_weights(s, cfg["C"], cfg["heads"], cfg["hidden"], cfg["win"], cfg["dtype"], not args.no_position_term))
    layers = [mk(61), mk(62)]
    pair = dsvt.dsvt_partition_xy(dsvt.part_cfg(cfg["grid"], cfg["win"], cfg["shifts"][0], cfg["tau"], cfg["batch"], 0), cd)
    out = torch.empty_like(x)
    for _ in range(5):                                # warm: clocks, caches
        dsvt.dsvt_block(layers, pair, cd, x, x_out=out)
    torch.cuda.synchronize()
    L = dsvt.lib()
    blocks, slots = C.c_int32(0), C.c_int32(0)
    buf = (C.c_ulonglong * (2048 * 12))()
    L.dsvt_debug_phase_clocks.argtypes = [C.c_void_p, C.POINTER(C.c_int32), C.POINTER(C.c_int32)]
    assert L.dsvt_debug_phase_clocks(buf, C.byref(blocks), C.byref(slots)) == 0
    t = np.frombuffer(buf, dtype=np.uint64).reshape(blocks.value, slots.value).astype(np.int64)
    nt = min(int(pair[0].n_tiles.item()), blocks.value)
    d = np.diff(t[:nt, :9], axis=1)                   # [tile][phase] clocks
    rows = pair[1].tile_desc.view(-1, 256)[:nt, 0].cpu().numpy()
    print(f"config {args.config}: {len(coords)} voxels, {nt} tiles, {rows.mean():.1f} rows per tile; last layer launch of a block; shader clocks, thread 0 of each workgroup")
    print("| phase | all tiles | first half of the launch order | second half |")
    print("|---|---|---|---|")
    h = nt // 2
    for k, name in enumerate(PHASES):
        print(f"| {name} | {d[:, k].mean():,.0f} | {d[:h, k].mean():,.0f} | {d[h:, k].mean():,.0f} |")
    print(f"| whole tile | {d.sum(1).mean():,.0f} | {d[:h].sum(1).mean():,.0f} | {d[h:].sum(1).mean():,.0f} |")
    print(f"| rows | {rows.mean():.1f} | {rows[:h].mean():.1f} | {rows[h:].mean():.1f} |")


if __name__ == "__main__":
    main()
