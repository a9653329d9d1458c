"""Plan-parameter tuner for one batch of operators (Section 5.3 and Table 1 of the paper).

The paper's last experiment tunes the blocking of a kernel twice, once running alone and once
next to other tenants, and finds that the two optima differ (Table 1): a configuration greedily
tuned for isolation is not the one to use under co-tenancy.  The knobs of this library that
play that role are the plan parameters (target bytes per tile, how fast tiles shrink towards
the end of the table, how many workgroups stay resident).  This module sweeps them on the
device for a given operator list and reports the times; `cotenancy()` runs the sweep for one
operator alone and for the same operator inside a mix.

Timing uses HIP events through torch (device memory and streams only); every launch goes
through the C ABI.  Nothing here touches the CPU oracle.

The paper's runtime applies parameters computed ahead of time by the tuning phase (Section
5.3).  `save()` / `load()` / `tuned_params()` keep the best parameter set of a sweep in a plain
text file (one JSON record per line) keyed by a signature of the operator mix, so that a later
process plans the same mix with the tuned values without measuring anything.

    python -m paper_1901_10008_amd.tune --config 5 --save tuned.jsonl
"""
from __future__ import annotations

import argparse
import hashlib
import itertools
import json
import os
import sys
import time
from typing import Dict, Iterable, List, Sequence, Tuple

from . import binding as sk

DEFAULT_GRID: Dict[str, Sequence[int]] = {
    "tile_bytes_max": (512 << 10, 1 << 20, 2 << 20, 4 << 20),
    "tail_div": (0, 256, 384, 768),
    "balance_div": (256, 512, 2048),
    "skinny_max_m": (32, 64),   # which operators stream their weights and which take the LDS tiles
    "xcd_part": (0, 32, 1024),  # LDS tiles by table order, or die by die in parts of 32 output tiles, or whole
                                # operators per die (pays on compute-heavy plans only)
}


def candidates(grid: Dict[str, Sequence[int]] | None = None) -> List[Dict[str, int]]:
    grid = grid or DEFAULT_GRID
    keys = list(grid)
    return [dict(zip(keys, vals)) for vals in itertools.product(*(grid[k] for k in keys))]


def time_plans(problems, param_sets: Iterable[Dict[str, int]], rounds: int = 5, launches: int = 3,
               stream: int | None = None) -> List[Tuple[Dict[str, int], float, int]]:
    """[(params, median microseconds per launch, tiles)] for every parameter set.

    All plans are built first and timed round-robin, so that clock and cache state drift hits
    every candidate alike."""
    import torch

    if stream is None:
        stream = torch.cuda.current_stream().cuda_stream
    sets = list(param_sets)
    plans = [sk.sk_plan_create(problems, sk.sk_plan_params_default(**p)) for p in sets]
    try:
        for pl in plans:
            sk.sk_launch(pl, stream)
        torch.cuda.synchronize()
        samples: List[List[float]] = [[] for _ in plans]
        for _ in range(rounds):
            for i, pl in enumerate(plans):
                e0 = torch.cuda.Event(enable_timing=True)
                e1 = torch.cuda.Event(enable_timing=True)
                e0.record()
                for _ in range(launches):
                    sk.sk_launch(pl, stream)
                e1.record()
                torch.cuda.synchronize()
                samples[i].append(e0.elapsed_time(e1) / launches * 1e3)
        out = []
        for p, pl, s in zip(sets, plans, samples):
            s.sort()
            out.append((p, s[len(s) // 2], sk.sk_plan_num_tiles(pl)))
        return out
    finally:
        for pl in plans:
            pl.close()


def tune(problems, grid: Dict[str, Sequence[int]] | None = None, **kw):
    """(best parameter set, all results sorted by time)."""
    res = sorted(time_plans(problems, candidates(grid), **kw), key=lambda r: r[1])
    return res[0][0], res


# ---- tuned parameters kept between processes ---------------------------------------------------------

def _shape(p) -> tuple:
    """What of an sk_problem decides its tiles: operator, element type and the dimensions, not the addresses."""
    if p.op == sk.SK_GEMM:
        return (int(p.op), int(p.dtype), int(p.M), int(p.N), int(p.K))
    return (int(p.op), int(p.dtype), int(p.Nb), int(p.H), int(p.Wd), int(p.Cin), int(p.Cout), int(p.R), int(p.S),
            int(p.pad_h), int(p.pad_w), int(p.stride))


def signature(problems) -> str:
    """Signature of an operator mix: the multiset of operator shapes (order and addresses do not matter)."""
    shapes = sorted(_shape(p) for p in problems)
    return hashlib.sha256(json.dumps(shapes).encode()).hexdigest()[:24]


def save(path: str, problems, params: Dict[str, int], microseconds: float | None = None, note: str = "") -> str:
    """Appends the tuned parameter set of this operator mix to `path` (a later record of the same mix wins)."""
    sig = signature(problems)
    rec = {"signature": sig, "operators": len(problems), "params": {k: int(v) for k, v in params.items()},
           "us": None if microseconds is None else round(float(microseconds), 2), "note": note,
           "saved_unix": int(time.time())}
    os.makedirs(os.path.dirname(os.path.abspath(path)), exist_ok=True)
    with open(path, "a") as f:
        f.write(json.dumps(rec, sort_keys=True) + "\n")
    return sig


def load(path: str) -> Dict[str, dict]:
    """{signature: record}; a missing file is an empty table, a malformed line is an error."""
    out: Dict[str, dict] = {}
    if not os.path.exists(path):
        return out
    with open(path) as f:
        for n, line in enumerate(f, 1):
            line = line.strip()
            if not line:
                continue
            rec = json.loads(line)
            if not isinstance(rec.get("params"), dict) or "signature" not in rec:
                raise ValueError(f"{path}:{n}: not a tuned-parameter record")
            out[rec["signature"]] = rec
    return out


def tuned_params(problems, path: str):
    """sk_plan_params for this operator mix from the file, or None if the mix has not been tuned.
    Unknown parameter names in the file are an error (AttributeError from the binding)."""
    rec = load(path).get(signature(problems))
    if rec is None:
        return None
    return sk.sk_plan_params_default(**rec["params"])


def cotenancy_table(rep: dict, what: str) -> str:
    """The result of cotenancy() as the text table kept under profiles/."""
    lines = [f"{what}", "", "weight bytes per tile   alone, us   among its co-tenants (whole mix), us"]
    for t, a, m in zip(rep["targets"], rep["solo_us"], rep["mix_us"]):
        mark = ("  <- best alone" if t == rep["solo_best_target"] else "") + ("  <- best for the mix" if t == rep["mix_best_target"] else "")
        lines.append(f"{t:>21d} {a:11.1f} {m:12.1f}{mark}")
    lines += ["", f"the mix's optimum costs the operator alone x{rep['solo_penalty_with_mix_best']}; "
                  f"the operator's own optimum costs the mix x{rep['mix_penalty_with_solo_best']}"]
    return "\n".join(lines) + "\n"


FIXED_TARGETS = tuple(1 << e for e in range(15, 23))  # 32 KiB .. 4 MiB of weights per tile


def cotenancy(problems, index: int, targets: Sequence[int] = FIXED_TARGETS, **kw):
    """The shape of the paper's Table 1 with this library's knob: the weight bytes per tile.

    Every candidate fixes the target (lower clamp = upper clamp, no shrinking tail), once for
    operator `index` launched alone and once for the whole list with the operator among its
    co-tenants.  Reported: the best target in either setting and what it costs to use the one
    setting's optimum in the other."""
    sets = [{"tile_bytes_min": t, "tile_bytes_max": t, "tail_div": 0} for t in targets]
    solo = time_plans([problems[index]], sets, **kw)
    mix = time_plans(problems, sets, **kw)
    i_solo = min(range(len(sets)), key=lambda i: solo[i][1])
    i_mix = min(range(len(sets)), key=lambda i: mix[i][1])
    return {
        "targets": list(targets),
        "solo_us": [round(r[1], 1) for r in solo],
        "mix_us": [round(r[1], 1) for r in mix],
        "solo_best_target": targets[i_solo], "mix_best_target": targets[i_mix],
        "solo_penalty_with_mix_best": round(solo[i_mix][1] / solo[i_solo][1], 3),
        "mix_penalty_with_solo_best": round(mix[i_solo][1] / mix[i_mix][1], 3),
    }


def _device_problems(specs, seed=0):
    import torch
    import workloads

    tdt = {"f32": torch.float32, "bf16": torch.bfloat16, "f16": torch.float16}
    keep, problems = [], []
    for i, s in enumerate(specs):
        a, b = (x.to(tdt[s.dtype]) for x in workloads.draw_device(s, seed, i))
        c = torch.empty(s.c_shape, dtype=tdt[s.dtype], device="cuda")
        keep += [a, b, c]
        problems.append(sk.make_problem(s, a.data_ptr(), b.data_ptr(), c.data_ptr()))
    return problems, keep


def main(argv=None) -> int:
    ap = argparse.ArgumentParser(description=__doc__.split("\n\n")[0])
    ap.add_argument("--config", type=int, default=5)
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--cotenant", type=int, default=None, help="also tune this operator alone and compare")
    ap.add_argument("--top", type=int, default=5)
    ap.add_argument("--save", default=None, help="append the best parameter set to this file, keyed by the mix's signature")
    ap.add_argument("--table", default=None, help="with --cotenant: also write the alone / co-tenant table to this text file")
    args = ap.parse_args(argv)
    import workloads

    specs = workloads.config(args.config, seed=args.seed)
    problems, keep = _device_problems(specs, args.seed)
    best, res = tune(problems)
    out = {"config": args.config, "operators": len(specs), "best": best,
           "top": [{"params": p, "us": round(t, 1), "tiles": n} for p, t, n in res[:args.top]],
           "worst_us": round(res[-1][1], 1)}
    if args.save:
        out["signature"] = save(args.save, problems, best, res[0][1], note=f"config {args.config} seed {args.seed}")
    if args.cotenant is not None:
        out["cotenancy"] = cotenancy(problems, args.cotenant)
        if args.table:
            s = specs[args.cotenant]
            with open(args.table, "w") as f:
                f.write(cotenancy_table(out["cotenancy"], f"operator {args.cotenant} of workload {args.config} ({s.op} "
                                        f"{workloads.canonical_dims(s)}, {s.dtype}) alone and among the other {len(specs) - 1} operators"))
    print(json.dumps(out))
    del keep
    return 0


if __name__ == "__main__":
    sys.exit(main())
