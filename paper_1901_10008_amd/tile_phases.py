"""Where a tile's time goes: phase times per tile class, measured on the device.

A measuring aid, not part of the boundary.  It uses a second build of the library (`build.build_diag()`,
`-DSK_DIAG_CLOCKS`, libsuperkernel_diag.so) in which thread 0 of the first workgroups stamps the device clock at
the phase boundaries of every tile it runs: tile taken up, set-up done, first main-loop step multiplied, main
loop done, outputs stored, next tile's record handed to all waves.  The stamps of one launch are read back and
averaged per tile class:

    python -m paper_1901_10008_amd.tile_phases --config 5
    python -m paper_1901_10008_amd.tile_phases --config 8 --replicate 16

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
WGS, TILES = 16, 64  # SK_DIAG_WGS, SK_DIAG_TILES of kernels.hip.h


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
    args = ap.parse_args(argv)

    from . import build

    if args.rebuild or not os.path.exists(build.DIAG_LIB):
        build.build_diag()
    os.environ["SK_LIBRARY"] = build.DIAG_LIB
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
        print(phase_table(buf.reshape(WGS, TILES, 8).astype(np.int64)))
    finally:
        plan.close()
    return 0


if __name__ == "__main__":
    raise SystemExit(main())
