"""Operators that arrive over time: which of them go into the next superkernel (Section 5, items (a)
and (b), and Section 5.2 of the paper).

The paper's runtime not only coalesces what is ready, it also reorders in time: operators with a
tight latency budget go first, and an operator that does not fit well may be held back for the
next launch.  This module replays a seeded arrival trace against the device under three
policies and reports how many latency budgets were met:

  sequential   one launch per operator, in arrival order (time multiplexing, Section 4.1)
  coalesce     whenever the device is free, everything that has arrived goes into one plan
               (earliest deadline first inside it)
  ooo          as coalesce, but a launch is kept short: operators are taken in deadline order
               until the estimated duration reaches `cap_ms`; the rest, those with the most
               slack, wait for the next launch, so that an urgent operator that arrives
               meanwhile never waits behind a long launch (reordering in time)

All arithmetic runs in the library's launches; this file only decides what to put into
`sk_plan_create` and when.  Arrival times are the host's wall clock; an operator's completion
is the time at which the host saw its launch complete, less the device time between the
operator's last tile and the launch's last tile (plans are created with stamps), so an
operator early in a long launch is not charged the whole launch.

    python -m paper_1901_10008_amd.serve --rate 150 --operators 1500
"""
from __future__ import annotations

import argparse
import json
import sys
import time
from dataclasses import dataclass
from typing import List, Sequence

from . import binding as sk

HBM_BYTES_PER_MS = 5.5e9  # what one launch sustains on a large mix (measured); used for estimates only
LAUNCH_FLOOR_MS = 0.02    # a launch is never estimated shorter than this


@dataclass
class Arrival:
    index: int        # position in the operator pool
    t_ms: float       # arrival time
    budget_ms: float  # latency budget from arrival
    bytes: int        # algorithmic bytes (for the duration estimate)


def poisson_trace(pool_bytes: Sequence[int], n: int, rate_per_ms: float, seed: int = 0,
                  budget_ms=(0.5, 5.0)) -> List[Arrival]:
    """n arrivals, exponential gaps with the given rate, operator drawn uniformly from the pool."""
    import numpy as np

    g = np.random.Generator(np.random.PCG64(np.random.SeedSequence([int(seed), 77])))
    t, out = 0.0, []
    for _ in range(n):
        t += float(g.exponential(1.0 / rate_per_ms))
        i = int(g.integers(0, len(pool_bytes)))
        out.append(Arrival(i, t, float(g.uniform(*budget_ms)), int(pool_bytes[i])))
    return out


def estimate_ms(total_bytes: int) -> float:
    return max(LAUNCH_FLOOR_MS, total_bytes / HBM_BYTES_PER_MS)


def run_trace(pool_problems, trace: Sequence[Arrival], policy: str, cap_ms: float = 0.5,
              pipeline: bool = True, timeline: list | None = None) -> dict:
    """Replays `trace` in real time.  pool_problems[i] is the sk_problem of pool operator i, or a list
    of descriptors of it that differ only in the output buffer C.  Arrivals of one pool operator
    that are in flight together each need an output buffer of their own: an arrival for which
    none is free waits for a later launch.

    With `pipeline`, the next plan is made and queued shortly before the running launch is expected
    to end (estimated duration, corrected by what earlier launches took), so that planning and
    the launch itself overlap the device's work; without it, the host waits for every launch
    before it looks at the queue again.  `timeline` collects one record per coalesced launch."""
    import collections

    import torch

    assert policy in ("sequential", "coalesce", "ooo")
    replicas = [list(p) if isinstance(p, (list, tuple)) else [p] for p in pool_problems]
    free = [list(range(len(r))) for r in replicas]  # output buffers not in use, per pool operator
    # A stream of its own, not the legacy default stream: reading the stamps of a finished
    # launch must not wait for the launch queued behind it.
    tstream = torch.cuda.Stream()
    stream = tstream.cuda_stream
    depth = (16 if policy == "sequential" else 2) if pipeline else 1
    pending: List[Arrival] = []
    inflight = collections.deque()  # (plan or None, batch, event, estimated ms)
    nxt = 0
    latencies, met, launches, device_ms = [], 0, 0, 0.0
    corr, prep_ms, t_free = 1.0, 0.1, 0.0
    # time multiplexing needs no planning at run time: one plan per pool operator, built beforehand
    solo = {}
    if policy == "sequential":
        for i in sorted({a.index for a in trace}):
            solo[i] = sk.sk_plan_create([replicas[i][0]])
    t0 = time.perf_counter()
    now = lambda: (time.perf_counter() - t0) * 1e3

    def retire():
        nonlocal met, device_ms, corr, t_free
        plan, batch, ev, est, used = inflight.popleft()
        ev.synchronize()
        t_done = now()
        for a, r in zip(batch, used):
            free[a.index].append(r)
        if plan is None:
            ends = [t_done]
        else:
            done, start, rate = sk.sk_plan_get_stamps(plan)
            plan.close()
            last = max(done)
            # anchored at the end: the host saw the launch complete at t_done
            ends = [t_done - (last - d) / rate for d in done]
            took = (last - start) / rate
            device_ms += took
            if timeline is not None:
                timeline.append({"operators": len(batch), "estimate_ms": est, "kernel_ms": took, "done_ms": t_done})
            corr = 0.8 * corr + 0.2 * min(4.0, max(0.25, took / est))
        for a, e in zip(batch, ends):
            latencies.append(e - a.t_ms)
            met += (e - a.t_ms) <= a.budget_ms
        t_free = max(t_done, t_free) if inflight else t_done

    while nxt < len(trace) or pending or inflight:
        t = now()
        while nxt < len(trace) and trace[nxt].t_ms <= t:
            pending.append(trace[nxt])
            nxt += 1
        if pending and len(inflight) < depth and (policy == "sequential" or not inflight or t >= t_free - prep_ms):
            t_prep = t
            if policy == "sequential":
                batch, used, total = [pending[0]], [], 0  # one stream keeps launches into one buffer ordered
            else:
                order = sorted(pending, key=lambda a: a.t_ms + a.budget_ms)
                batch, used, total = [], [], 0
                for a in order:
                    if not free[a.index]:
                        continue
                    if policy == "ooo" and batch and estimate_ms(total + a.bytes) * corr > cap_ms:
                        break
                    batch.append(a)
                    used.append(free[a.index].pop())
                    total += a.bytes
            if batch:
                if policy == "sequential":
                    pending.pop(0)
                else:
                    chosen = {id(a) for a in batch}
                    pending = [a for a in pending if id(a) not in chosen]
                ev = torch.cuda.Event()
                if policy == "sequential":
                    sk.sk_launch(solo[batch[0].index], stream)
                    ev.record(tstream)
                    inflight.append((None, batch, ev, 0.0, used))
                else:
                    probs = (sk.sk_problem * len(batch))()
                    for j, (a, r) in enumerate(zip(batch, used)):
                        probs[j] = replicas[a.index][r]
                        probs[j].deadline_ms = max(1e-3, a.t_ms + a.budget_ms - t_prep)  # budget left, from now
                    plan = sk.sk_plan_create(probs, sk.sk_plan_params_default(stamps=1))
                    sk.sk_launch(plan, stream)
                    ev.record(tstream)
                    est = estimate_ms(total) * corr
                    inflight.append((plan, batch, ev, estimate_ms(total), used))
                    t_end = now()
                    prep_ms = 0.8 * prep_ms + 0.2 * (t_end - t_prep)
                    t_free = max(t_free, t_end) + est
                launches += 1
                continue
        if inflight and (len(inflight) >= depth or nxt >= len(trace) or not pipeline
                         or (policy != "sequential" and now() >= t_free - prep_ms)
                         or (policy == "sequential" and inflight[0][2].query())):
            retire()
            continue
        if not inflight and not pending and nxt < len(trace):
            time.sleep(max(0.0, (trace[nxt].t_ms - now()) * 1e-3))
    span = now()
    for pl in solo.values():
        pl.close()
    latencies.sort()
    n = len(latencies)
    return {"policy": policy, "operators": n, "launches": launches, "met_fraction": round(met / n, 4),
            "latency_ms_median": round(latencies[n // 2], 3), "latency_ms_p99": round(latencies[int(0.99 * (n - 1))], 3),
            "span_ms": round(span, 2), "kernel_busy_fraction": round(device_ms / span, 3) if device_ms else None}


def main(argv=None) -> int:
    ap = argparse.ArgumentParser(description=__doc__.split("\n\n")[0])
    ap.add_argument("--config", type=int, default=5, help="operator pool")
    ap.add_argument("--operators", type=int, default=1500, help="arrivals in the trace")
    ap.add_argument("--rate", type=float, default=150.0, help="arrivals per millisecond")
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--no-pipeline", action="store_true", help="wait for every launch before planning the next")
    args = ap.parse_args(argv)
    import torch
    import workloads
    from .tune import _device_problems

    def c_bytes(p):
        es = 4 if p.dtype == sk.SK_F32 else 2
        if p.op == sk.SK_GEMM:
            return ((p.M - 1) * (p.ldc or p.N) + p.N) * es
        return p.Nb * (p.H + 2 * p.pad_h - p.R + 1) * (p.Wd + 2 * p.pad_w - p.S + 1) * p.Cout * es

    specs = workloads.config(args.config, seed=args.seed)
    problems, keep = _device_problems(specs, args.seed)
    # eight output buffers per pool operator, so that requests for it can overlap
    pool = []
    for p in problems:
        reps = [p]
        for _ in range(7):
            q = type(p).from_buffer_copy(p)
            c = torch.empty(c_bytes(p), dtype=torch.uint8, device="cuda")
            keep.append(c)
            q.C = c.data_ptr()
            reps.append(q)
        pool.append(reps)
    trace = poisson_trace([workloads.algorithmic_bytes(s) for s in specs], args.operators, args.rate, args.seed)
    out = {"pool": args.config, "rate_per_ms": args.rate,
           "offered_GB_per_s": round(sum(a.bytes for a in trace) / trace[-1].t_ms / 1e6, 1)}
    for policy in ("sequential", "coalesce", "ooo"):
        run_trace(pool, trace[:50], policy, pipeline=not args.no_pipeline)  # warm-up
        out[policy] = run_trace(pool, trace, policy, pipeline=not args.no_pipeline)
    print(json.dumps(out))
    del keep
    return 0


if __name__ == "__main__":
    sys.exit(main())
