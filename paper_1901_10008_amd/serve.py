"""Replay of an arrival trace against the library's arrival queue (Section 5, items (a) and (b), and
Section 5.2 of the paper).

The paper's runtime not only coalesces what is ready, it also reorders in time: operators with a
tight latency budget go first, and an operator that does not fit well may be held back for the
next launch.  The queue that decides this lives behind the C ABI (sk_queue_create / submit / poll /
destroy, policies SK_QUEUE_SEQUENTIAL, SK_QUEUE_COALESCE and SK_QUEUE_OOO); this module only
replays a seeded Poisson arrival trace in real time: it submits every arrival when its time has
come, polls for completions, and reports how many latency budgets were met.

Arrival times are the host's wall clock; an operator's latency runs from its submit call to the
retirement of its last tile (the queue anchors the launch's completion stamps at the host time
at which it saw the launch complete, so an operator early in a long launch is not charged the
whole launch).

    python -m paper_1901_10008_amd.serve --rate 150 --operators 1500
"""
from __future__ import annotations

import argparse
import ctypes as C
import json
import sys
import time
from dataclasses import dataclass
from typing import List, Sequence

from . import binding as sk

HBM_BYTES_PER_MS = 5.5e9  # what one launch sustains on a large mix (measured); the queue's default estimate
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


def run_trace(pool_problems, trace: Sequence[Arrival], policy: str, cap_ms: float = 0.5, depth: int = 0,
              stream: int | None = None) -> dict:
    """Replays `trace` in real time through one sk_queue.  pool_problems[i] is the sk_problem of pool operator
    i, or a list of descriptors of it that differ only in the output buffer C: arrivals of one pool
    operator take its output buffers in turn (the queue never has two operators with one output buffer
    in flight together; a later arrival for a buffer that is still in use waits for a later launch)."""
    import torch

    assert policy in sk.QUEUE_POLICY
    replicas = [list(p) if isinstance(p, (list, tuple)) else [p] for p in pool_problems]
    n = len(trace)
    # everything the replay hands over is laid out beforehand: the loop itself only looks at the clock
    ops = (sk.sk_problem * max(n, 1))()
    budgets = (C.c_double * max(n, 1))()
    tickets = (C.c_uint64 * max(n, 1))()
    turn = [0] * len(replicas)
    for j, a in enumerate(trace):
        r = replicas[a.index]
        ops[j] = r[turn[a.index] % len(r)]
        turn[a.index] += 1
        budgets[j] = a.budget_ms
    times = [a.t_ms for a in trace]
    # A stream of its own, not the legacy default stream: reading the stamps of a finished launch must not
    # wait for the launch queued behind it.
    own = None
    if stream is None:
        own = torch.cuda.Stream()
        stream = own.cuda_stream
    prm = sk.sk_queue_params_default(policy=policy, cap_ms=cap_ms, depth=depth, bytes_per_ms=HBM_BYTES_PER_MS,
                                     launch_floor_ms=LAUNCH_FLOOR_MS)
    done = (sk.sk_completion * 512)()
    latencies, met, failed = [], 0, 0
    by_ticket = {}
    with sk.sk_queue_create(prm, stream) as q:
        t0 = time.perf_counter()
        nxt = 0
        while len(latencies) + failed < n:
            t = (time.perf_counter() - t0) * 1e3
            j = nxt
            while j < n and times[j] <= t:
                j += 1
            if j > nxt:
                sk.sk_queue_submit(q, ops, budgets, nxt, j - nxt, tickets)
                nxt = j
            # all submitted and nothing else to do: sleep inside the library until something completes
            got = sk.sk_queue_poll(q, done, wait=(nxt >= n))
            for i in range(got):
                c = done[i]
                if c.met < 0:
                    failed += 1
                else:
                    latencies.append(c.latency_ms)
                    met += c.met
                by_ticket[c.ticket] = c.launch
            if got == 0 and nxt < n:
                gap = times[nxt] - (time.perf_counter() - t0) * 1e3
                if gap > 0.2:
                    time.sleep((gap - 0.1) * 1e-3)
        stats = sk.sk_queue_get_stats(q)
    if own is not None:
        own.synchronize()
    assert failed == 0, f"{failed} operators could not be planned"
    latencies.sort()
    m = len(latencies)
    return {"policy": policy, "operators": m, "launches": int(stats.launches), "met_fraction": round(met / m, 4),
            "latency_ms_median": round(latencies[m // 2], 3), "latency_ms_p99": round(latencies[int(0.99 * (m - 1))], 3),
            "span_ms": round(stats.span_ms, 2),
            "kernel_busy_fraction": round(stats.device_busy_ms / stats.span_ms, 3) if stats.device_busy_ms else None}


def main(argv=None) -> int:
    ap = argparse.ArgumentParser(description=__doc__.split("\n\n")[0])
    ap.add_argument("--config", type=int, default=5, help="operator pool")
    ap.add_argument("--operators", type=int, default=1500, help="arrivals in the trace")
    ap.add_argument("--rate", type=float, default=150.0, help="arrivals per millisecond")
    ap.add_argument("--seed", type=int, default=0)
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
        run_trace(pool, trace[:50], policy)  # warm-up
        out[policy] = run_trace(pool, trace, policy)
    print(json.dumps(out))
    del keep
    return 0


if __name__ == "__main__":
    sys.exit(main())
