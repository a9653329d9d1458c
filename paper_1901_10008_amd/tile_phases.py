"""Where a tile's time goes: phase times per tile class, measured on the device.

A measuring aid, not part of the boundary.  It uses a second build of the library (`build.build_diag()`,
`-DSK_DIAG_CLOCKS`, libsuperkernel_diag.so) in which thread 0 of the first workgroups stamps the device clock at
the phase boundaries of every tile it runs: tile taken up, set-up done, first main-loop step multiplied, main
loop done, outputs stored, next tile's record handed to all waves.  The stamps of one launch are read back and
averaged per tile class:

    python -m paper_1901_10008_amd.tile_phases --config 5
    python -m paper_1901_10008_amd.tile_phases --config 8 --replicate 16
    python -m paper_1901_10008_amd.tile_phases --config 4 --replicate 16 --ends

`--ends` uses a third build that stamps every workgroup of the launch (512 of them, 24 tiles each) and adds
when the workgroups finish: how long they idle, on average, until the last one is done, and on which tiles
the last ones were.

The library to load is chosen before the binding loads anything (environment variable SK_LIBRARY), so the
tool runs in a process of its own.
"""
from __future__ import annotations

import argparse
import ctypes
import os
import sys

PHASES = ("set-up", "first step", "main loop", "outputs", "hand-over", "whole tile")
CLASS_NAMES = {0: "skinny, 16 rows", 3: "skinny, 32 rows", 6: "skinny, 64 rows", 9: "LDS tile 128x128", 10: "LDS tile 128x64"}


def end_summary(stamps) -> str:
    """`stamps` as for phase_table, with every workgroup of the launch in it: when the workgroups finish."""
    import numpy as np

    ends, last = [], []
    begin = None
    for wg in range(stamps.shape[0]):
        t = stamps[wg]
        t = t[(t[:, 0] > 0) & (t[:, 5] > 0)]
        if len(t) == 0:
            continue
        begin = int(t[0, 0]) if begin is None else min(begin, int(t[0, 0]))
        ends.append(int(t[-1, 5]))
        last.append((wg, int(t[-1, 6] - 1) % 100, (int(t[-1, 5]) - int(t[-1, 0])) / 100.0, len(t) == stamps.shape[1]))
    if not ends:
        return "no tiles stamped"
    e = (np.array(ends, dtype=np.float64) - begin) / 100.0
    lines = [f"{len(e)} workgroups; the last finishes {e.max():.1f} us after the first tile was taken up, the mean {e.mean():.1f} us: "
             f"{e.max() - e.mean():.1f} us of idle time per workgroup at the end"]
    if any(x[3] for x in last):
        lines.append("(some workgroups ran more tiles than are stamped: their end is that of the last stamped tile)")
    lines.append("last to finish (workgroup, class and length of its last tile, end): " + "  ".join(
        f"{last[i][0]} {'LDS tile' if last[i][1] >= 9 else 'skinny'} {last[i][2]:.0f} us, {e[i]:.0f}" for i in np.argsort(-e)[:8]))
    return "\n".join(lines)



def phase_table(stamps) -> str:
    """`stamps`: int64 array [WGS, TILES, 8] of 100 MHz clock values; the table as text (microseconds)."""
    import numpy as np

    by = {}
    for wg in range(stamps.shape[0]):
        for t in range(stamps.shape[1]):
            x = stamps[wg, t]
            if x[6] == 0 or x[1] == 0 or x[5] == 0:  # no tile, a tile of the element-wise paths, or not finished
                continue
            key = (int(x[6] - 1) % 100, int(x[6] - 1) // 100 > 1)
            by.setdefault(key, []).append([x[1] - x[0], x[2] - x[1], x[3] - x[2], x[4] - x[3], x[5] - x[4], x[5] - x[0]])
    lines = [f"{'tile class':28s} {'tiles':>6s} " + " ".join(f"{p:>11s}" for p in PHASES) + "   (mean, us)"]
    for key in sorted(by):
        r = np.array(by[key], dtype=np.float64) / 100.0
        name = CLASS_NAMES.get(key[0], f"class {key[0]}") + (", slice" if key[1] else "")
        lines.append(f"{name:28s} {len(r):6d} " + " ".join(f"{r[:, i].mean():11.2f}" for i in range(len(PHASES))))
    return "\n".join(lines)


def main(argv=None) -> int:
    ap = argparse.ArgumentParser(description=__doc__.split("\n")[0])
    ap.add_argument("--config", type=int, default=5)
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--replicate", type=int, default=1, help="copies of the workload in one plan")
    ap.add_argument("--param", action="append", default=[], help="sk_plan_params override name=value")
    ap.add_argument("--rebuild", action="store_true", help="build the diagnostic library even if it exists")
    ap.add_argument("--ends", action="store_true", help="stamp every workgroup of the launch and report when they finish")
    args = ap.parse_args(argv)

    from . import build

    lib_file = build.DIAG_ALL_LIB if args.ends else build.DIAG_LIB
    if args.rebuild or not os.path.exists(lib_file):
        build.build_diag(all_workgroups=args.ends)
    os.environ["SK_LIBRARY"] = lib_file
    import numpy as np
    import torch

    from . import binding as sk
    from .tune import _device_problems

    sys.path.insert(0, build.ROOT)
    import workloads

    specs = workloads.config(args.config, seed=args.seed)
    problems, keep = [], []
    for r in range(args.replicate):
        p, k = _device_problems(specs, args.seed + 1000 * r)
        problems += p
        keep += k
    over = {k: int(v) for k, v in (kv.split("=") for kv in args.param)}
    plan = sk.sk_plan_create(problems, sk.sk_plan_params_default(**over))
    stream = torch.cuda.current_stream().cuda_stream
    L = sk.lib()
    L.sk_diag_read.argtypes = [ctypes.c_void_p, ctypes.c_uint64]
    wgs, tiles = ctypes.c_int(), ctypes.c_int()
    L.sk_diag_shape(ctypes.byref(wgs), ctypes.byref(tiles))
    WGS, TILES = wgs.value, tiles.value
    try:
        for _ in range(3):
            sk.sk_launch(plan, stream)
        torch.cuda.synchronize()
        if L.sk_diag_clear() != 0:
            raise RuntimeError("sk_diag_clear failed")
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        sk.sk_launch(plan, stream)
        e1.record()
        torch.cuda.synchronize()
        buf = np.zeros(WGS * TILES * 8, dtype=np.uint64)
        if L.sk_diag_read(buf.ctypes.data_as(ctypes.c_void_p), ctypes.c_uint64(buf.nbytes)) != 0:
            raise RuntimeError("sk_diag_read failed")
        print(f"workload {args.config} x{args.replicate}: {len(problems)} operators, {sk.sk_plan_num_tiles(plan)} tiles, "
              f"one launch {e0.elapsed_time(e1) * 1e3:.1f} us (diagnostic build); first {WGS} workgroups, up to {TILES} tiles each")
        stamps = buf.reshape(WGS, TILES, 8).astype(np.int64)
        print(phase_table(stamps))
        if args.ends:
            print(end_summary(stamps))
    finally:
        plan.close()
    return 0


if __name__ == "__main__":
    raise SystemExit(main())
