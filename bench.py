#!/usr/bin/env python3
"""Benchmark of the coalesced superkernel on one MI355X.

One step = one sk_launch of the whole operator mix (default: the 256-operator
mixed GEMM/conv mix with deadlines), inputs resident in HBM, the plan built
once before the timed region (its cost is reported beside the result).
Prints ONE JSON line: aggregate TFLOP/s, speedups over one-launch-per-operator
and over multi-stream launches, fraction of the per-operator roofline, the
HBM roofline of the superkernel launch, and the CPU oracle as a baseline.
"""
from __future__ import annotations

import argparse
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_HBM_GBS = 8000.0
PEAK_FLOPS = {"bf16": 2.5e15, "f16": 2.5e15, "f32": 157.3e12}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", type=int, default=5, help="1..10 (default 5: 256 mixed operators, EDF)")
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-baselines", action="store_true", help="skip sequential / multi-stream legs")
    ap.add_argument("--cpu-seconds", type=float, default=15.0, help="target CPU time of the oracle sample")
    ap.add_argument("--param", action="append", default=[], help="sk_plan_params override name=value")
    ap.add_argument("--copies", type=int, default=1,
                    help="independent copies of all buffers, one plan each, launched in rotation (cold-cache timing of "
                         "workloads that fit the 256 MB last-level cache)")
    ap.add_argument("--cold", action="store_true", help="--copies = enough for 512 MB of operands (at most 256)")
    ap.add_argument("--replicate", type=int, default=1,
                    help="put this many independent copies of the workload into ONE plan (steady-state rate of a "
                         "workload too small to outlast a launch)")
    ap.add_argument("--no-ceilings", action="store_true",
                    help="skip the measured ceilings (streaming read, bf16 MFMA loop) the rates are also held against")
    ap.add_argument("--vendor-baseline", action="store_true",
                    help="also time the operators one by one through PyTorch's GEMM and convolution calls "
                         "(rocBLAS/hipBLASLt, MIOpen): context, not part of the metric")
    ap.add_argument("--pmc-calibration", action="store_true",
                    help="also run one plain 1 GiB device copy, so that a rocprofv3 --pmc run of this command "
                         "shows what FETCH_SIZE / WRITE_SIZE read for a kernel of known traffic")
    return ap.parse_args()


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no sharding, no collectives); --gpus must be 1",
              file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import paper_1901_10008_amd as sk
    import workloads

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)

    base_specs = workloads.config(args.config, seed=args.seed)
    specs = base_specs * max(1, args.replicate)
    name = workloads.config_names()[args.config - 1]
    tdt = {"f32": torch.float32, "bf16": torch.bfloat16, "f16": torch.float16}
    copies = max(1, args.copies)
    if args.cold:
        copies = max(copies, min(256, -(-(512 << 20) // sum(workloads.algorithmic_bytes(s) for s in specs))))
    keep, all_problems = [], []
    drawn = {}
    for c in range(copies):
        probs = []
        for i, s in enumerate(specs):
            j = i % len(base_specs)
            if j not in drawn:
                a32, b32 = workloads.draw_device(s, args.seed, j, dev)
                drawn[j] = (a32.to(tdt[s.dtype]).contiguous(), b32.to(tdt[s.dtype]).contiguous())
                del a32, b32
            a, b = drawn[j]
            if c or i >= len(base_specs):  # every copy has operands of its own
                a, b = a.clone(), b.clone()
            cbuf = torch.empty(s.c_shape, dtype=tdt[s.dtype], device=dev)
            keep += [a, b, cbuf]
            probs.append(sk.make_problem(s, a.data_ptr(), b.data_ptr(), cbuf.data_ptr()))
        all_problems.append(probs)
    del drawn
    problems = all_problems[0]
    torch.cuda.synchronize()

    overrides = {}
    for kv in args.param:
        k, v = kv.split("=")
        overrides[k] = int(v)

    flops = sum(workloads.flops(s) for s in specs)
    abytes = sum(workloads.algorithmic_bytes(s) for s in specs)
    t_roof = sum(max(workloads.flops(s) / PEAK_FLOPS[s.dtype], workloads.algorithmic_bytes(s) / (PEAK_HBM_GBS * 1e9))
                 for s in specs)
    t_lb = max(sum(workloads.flops(s) / PEAK_FLOPS[s.dtype] for s in specs), abytes / (PEAK_HBM_GBS * 1e9))

    stream = torch.cuda.current_stream().cuda_stream

    if args.pmc_calibration:
        src = torch.empty(1 << 30, dtype=torch.uint8, device=dev).fill_(1)
        dst = torch.empty_like(src)
        dst.copy_(src)          # the kernel to look for: reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        del src, dst

    # ---- plan cost (host planning + upload), not part of the timed steps ----
    # (create + destroy; the first call of a process also pays for loading the library's code
    # object and is reported separately)
    plan_times = []
    for _ in range(12):
        t0 = time.perf_counter()
        sk.sk_plan_create(problems, sk.sk_plan_params_default(**overrides)).close()
        plan_times.append((time.perf_counter() - t0) * 1e3)
    plan_first_ms = plan_times[0]
    plan_ms = sorted(plan_times[1:])[len(plan_times[1:]) // 2]

    plans = [sk.sk_plan_create(pr, sk.sk_plan_params_default(**overrides)) for pr in all_problems]
    plan = plans[0]
    ntiles = sk.sk_plan_num_tiles(plan)
    turn = [0]

    def next_plan():
        turn[0] += 1
        return plans[turn[0] % copies]

    def timed(fn, steps, warmup):
        for _ in range(warmup):
            fn()
        torch.cuda.synchronize()
        evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
        t0 = time.perf_counter()
        for e0, e1 in evs:
            e0.record()
            fn()
            e1.record()
        torch.cuda.synchronize()
        wall = (time.perf_counter() - t0) / steps
        dev_ms = [e0.elapsed_time(e1) for e0, e1 in evs]
        return wall * 1e3, dev_ms

    wall_ms, dev_ms = timed(lambda: sk.sk_launch(next_plan(), stream), args.steps, args.warmup)
    kern_ms = sum(dev_ms) / len(dev_ms)
    value = flops / (wall_ms * 1e-3) / 1e12

    out = {
        "metric": "aggregate TFLOP/s of the superkernel (one launch for all operators)",
        "value": round(value, 3),
        "unit": "TFLOP/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(wall_ms, 5),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": specs[0].dtype if len({s.dtype for s in specs}) == 1 else "mixed",
        "data": "synthetic",
        "config": {"workload": name, "operators": len(specs), "tiles": ntiles, "grid": sk.sk_plan_grid(plan),
                   "seed": args.seed, "copies_in_rotation": copies, "copies_in_one_plan": max(1, args.replicate),
                   "gflop": round(flops / 1e9, 3), "algorithmic_MB": round(abytes / 1e6, 2),
                   "params": overrides},
        "kernel_ms": {"mean": round(kern_ms, 5), "min": round(min(dev_ms), 5),
                      "median": round(sorted(dev_ms)[len(dev_ms) // 2], 5)},
        "plan_ms": round(plan_ms, 4),
        "plan_first_call_ms": round(plan_first_ms, 4),
        "value_incl_plan": round(flops / ((wall_ms + plan_ms) * 1e-3) / 1e12, 3),
        "per_problem_roofline": {"t_roof_ms": round(t_roof * 1e3, 5), "t_overlap_bound_ms": round(t_lb * 1e3, 5),
                                 "roofline_tflops": round(flops / t_roof / 1e12, 2),
                                 "frac": round(t_roof / (kern_ms * 1e-3), 4)},
        "roofline": roofline(specs, flops, abytes, kern_ms, name, max(1, args.replicate), overrides),
    }

    if not args.no_baselines:
        seq_steps = max(3, args.steps // 3)
        for pl in plans:  # the first sequential launch of a plan builds its tables
            sk.sk_launch_sequential(pl, stream)
        torch.cuda.synchronize()
        seq_wall, seq_dev = timed(lambda: sk.sk_launch_sequential(next_plan(), stream), seq_steps, 1)
        out["sequential"] = {"ms": round(seq_wall, 5), "tflops": round(flops / (seq_wall * 1e-3) / 1e12, 3),
                             "speedup": round(seq_wall / wall_ms, 3)}

        # the same launches replayed from a HIP graph (no per-launch host cost: the strongest form of
        # time multiplexing this library can be given)
        try:
            side = torch.cuda.Stream(device=dev)
            side.wait_stream(torch.cuda.current_stream())
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.stream(side):
                sk.sk_launch_sequential(plan, side.cuda_stream)  # warm the capture stream
                side.synchronize()
                with torch.cuda.graph(graph, stream=side):
                    sk.sk_launch_sequential(plan, side.cuda_stream)
            torch.cuda.synchronize()
            g_wall, _ = timed(graph.replay, seq_steps, 2)
            out["sequential_graph"] = {"ms": round(g_wall, 5), "tflops": round(flops / (g_wall * 1e-3) / 1e12, 3),
                                       "speedup": round(g_wall / wall_ms, 3)}
            del graph
        except Exception as e:  # reported, never fatal: the graph leg is context, not the metric
            out["sequential_graph"] = {"error": str(e)[:200]}

        if args.vendor_baseline:
            # the vendor libraries, one call per operator on one stream (time multiplexing as a framework
            # would do it).  Views only: the calls read the same buffers, outputs go to fresh tensors.
            import torch.nn.functional as F
            calls = []
            for i, sp_ in enumerate(base_specs):
                a, b = keep[3 * i], keep[3 * i + 1]
                if sp_.op == "gemm":
                    calls.append((torch.matmul, (a, b.t()), {}))
                else:
                    calls.append((F.conv2d, (a.permute(0, 3, 1, 2), b.permute(0, 3, 1, 2)),
                                  {"padding": (sp_.pad_h, sp_.pad_w), "stride": sp_.stride}))

            def vendor():
                for fn, a_, kw in calls:
                    fn(*a_, **kw)

            v_wall, _ = timed(vendor, seq_steps, 2)
            out["vendor_sequential"] = {"ms": round(v_wall, 5), "tflops": round(flops / (v_wall * 1e-3) / 1e12, 3),
                                        "speedup": round(v_wall / wall_ms, 3),
                                        "what": "torch.matmul / conv2d (channels_last views) per operator, one stream"}

        # multi-stream baseline: one single-operator plan per operator, round-robin over <= 32 streams
        nstreams = min(32, len(specs))
        streams = [torch.cuda.Stream(device=dev) for _ in range(nstreams)]
        singles = [sk.sk_plan_create([p], sk.sk_plan_params_default(**overrides)) for p in problems]
        cur = torch.cuda.current_stream()

        def multi():
            fork = torch.cuda.Event()
            fork.record(cur)
            for st in streams:
                st.wait_event(fork)
            for i, sp in enumerate(singles):
                sk.sk_launch(sp, streams[i % nstreams].cuda_stream)
            for st in streams:
                ev = torch.cuda.Event()
                ev.record(st)
                cur.wait_event(ev)

        ms_wall, _ = timed(multi, seq_steps, 1)
        out["multistream"] = {"ms": round(ms_wall, 5), "streams": nstreams,
                              "tflops": round(flops / (ms_wall * 1e-3) / 1e12, 3),
                              "speedup": round(ms_wall / wall_ms, 3)}
        for sp in singles:
            sp.close()

        # deadline-met fraction (only meaningful when the mix has deadlines)
        if any(math.isfinite(s.deadline_ms) for s in specs):
            res = {}
            for label, prm, launch in (("superkernel_edf", {"edf": 1}, sk.sk_launch),
                                       ("superkernel_index_order", {"edf": 0}, sk.sk_launch),
                                       ("sequential", {"edf": 1}, sk.sk_launch_sequential)):
                p2 = sk.sk_plan_create(problems, sk.sk_plan_params_default(stamps=1, **{**overrides, **prm}))
                launch(p2, stream)
                torch.cuda.synchronize()
                launch(p2, stream)
                torch.cuda.synchronize()
                done, start, rate = sk.sk_plan_get_stamps(p2)
                lat = [(d - start) / rate for d in done]
                met = sum(1 for l, s in zip(lat, specs) if l <= s.deadline_ms)
                res[label] = {"met_fraction": round(met / len(specs), 4), "max_latency_ms": round(max(lat), 4)}
                p2.close()
            out["deadlines"] = res

    if not args.no_ceilings:
        out["ceilings"] = measured_ceilings(torch, abytes / (kern_ms * 1e-3) / 1e9, out["value"])
        tr = out["roofline"]["traffic"]
        if tr and "achieved_over_stream_read" in out["ceilings"]:
            best = max(out["ceilings"]["stream_read_GBs_rows_of_16384B"], out["ceilings"]["stream_read_GBs_rows_of_2048B"])
            out["ceilings"]["measured_traffic_over_stream_read"] = round(tr / (kern_ms * 1e-3) / 1e9 / best, 4)

    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(specs, args.seed, args.cpu_seconds)

    for pl in plans:
        pl.close()
    print(json.dumps(out))


def measured_ceilings(torch, achieved_gbs, achieved_tflops):
    """What this device attains with kernels that do nothing else (libsk_ceilings.so): a streaming read
    with the superkernel's load map over 2 GiB, for long and for short rows, and a bf16 MFMA loop."""
    import ctypes as C

    path = os.path.join(ROOT, "paper_1901_10008_amd", "libsk_ceilings.so")
    try:
        lib = C.CDLL(path)
        lib.sk_ceiling_stream_read.argtypes = [C.c_void_p, C.c_uint64, C.c_uint64, C.c_int, C.c_void_p,
                                               C.POINTER(C.c_double)]
        lib.sk_ceiling_mfma_bf16.argtypes = [C.c_int, C.c_void_p, C.POINTER(C.c_double)]
        buf = torch.ones(2 << 30, dtype=torch.uint8, device="cuda")
        sink = torch.zeros(1 << 20, dtype=torch.uint8, device="cuda")
        torch.cuda.synchronize()
        res = {}
        for row_bytes in (16384, 2048):
            v = C.c_double()
            st = lib.sk_ceiling_stream_read(buf.data_ptr(), buf.numel(), row_bytes, 5, sink.data_ptr(), C.byref(v))
            if st != 0:
                return {"error": f"sk_ceiling_stream_read status {st}"}
            res[f"stream_read_GBs_rows_of_{row_bytes}B"] = round(v.value, 1)
        v = C.c_double()
        st = lib.sk_ceiling_mfma_bf16(20000, sink.data_ptr(), C.byref(v))
        if st != 0:
            return {"error": f"sk_ceiling_mfma_bf16 status {st}"}
        res["mfma_bf16_TFLOPs"] = round(v.value, 1)
        lib.sk_ceiling_lds_read.argtypes = [C.c_int, C.c_void_p, C.POINTER(C.c_double), C.POINTER(C.c_double)]
        g, bpc = C.c_double(), C.c_double()
        st = lib.sk_ceiling_lds_read(20000, sink.data_ptr(), C.byref(g), C.byref(bpc))
        if st != 0:
            return {"error": f"sk_ceiling_lds_read status {st}"}
        res["lds_fragment_read_GBs"] = round(g.value, 1)
        res["lds_fragment_read_bytes_per_clk_per_cu"] = round(bpc.value, 1)
        # the LDS-tile stage loop by itself on sixteen 2048-cubed products: whole, without operand loads, loads only
        del buf
        lib.sk_ceiling_tile_loop.argtypes = [C.c_int, C.c_void_p, C.c_void_p, C.c_void_p, C.POINTER(C.c_double)]
        ta = (torch.randn(16 * 2048 * 2048, device="cuda") * 0.5).to(torch.bfloat16)
        tb = (torch.randn(16 * 2048 * 2048, device="cuda") * 0.5).to(torch.bfloat16)
        tc = torch.empty(16 * 2048 * 2048, dtype=torch.bfloat16, device="cuda")
        for mode, name in ((0, "lds_tile_loop_TFLOPs"), (1, "lds_tile_loop_without_loads_TFLOPs"),
                           (2, "lds_tile_loop_loads_only_TFLOPs")):
            st = lib.sk_ceiling_tile_loop(mode, ta.data_ptr(), tb.data_ptr(), tc.data_ptr(), C.byref(v))
            if st != 0:
                return {"error": f"sk_ceiling_tile_loop status {st}"}
            res[name] = round(v.value, 1)
        del ta, tb, tc
        buf = None
        best = max(res["stream_read_GBs_rows_of_16384B"], res["stream_read_GBs_rows_of_2048B"])
        res["achieved_over_stream_read"] = round(achieved_gbs / best, 4)
        res["achieved_over_mfma_loop"] = round(achieved_tflops / res["mfma_bf16_TFLOPs"], 4)
        del buf, sink
        return res
    except OSError as e:
        return {"error": str(e)[:200]}


def roofline(specs, flops, abytes, kern_ms, workload, replicate, overrides):
    """The roofline of the superkernel launch: which resource bounds the whole mix (sum of bytes over the
    HBM peak against sum of flops over the matrix-core peak of each operator's type), what the launch
    achieves of it (algorithmic bytes or flops over the HIP-event time of the launch), and the HBM
    traffic the hardware counters saw for this workload and this kernel source, if a profile is committed."""
    import workloads

    t_bytes = abytes / (PEAK_HBM_GBS * 1e9)
    t_flops = sum(workloads.flops(s) / PEAK_FLOPS[s.dtype] for s in specs)
    tr = measured_traffic(workload, replicate, overrides)
    if t_bytes >= t_flops:
        ach = abytes / (kern_ms * 1e-3) / 1e9
        out = {"bound": "hbm", "achieved": round(ach, 1), "peak": PEAK_HBM_GBS, "unit": "GB/s",
               "frac": round(ach / PEAK_HBM_GBS, 4)}
    else:
        dts = {s.dtype for s in specs}
        peak = PEAK_FLOPS[next(iter(dts))] / 1e12 if len(dts) == 1 else flops / t_flops / 1e12
        ach = flops / (kern_ms * 1e-3) / 1e12
        out = {"bound": "mfma", "achieved": round(ach, 1), "peak": round(peak, 1), "unit": "TFLOP/s",
               "frac": round(ach / peak, 4)}
    out["traffic"] = tr["hbm_bytes_per_launch"] if tr else None
    out["traffic_source"] = ({k: tr[k] for k in ("workload", "kernel", "kernel_source_sha256", "profile")} if tr else
                             "no committed counter profile matches this workload, launch configuration and kernel source")
    return out


def kernel_source_hash():
    """SHA-256 over the sources the superkernel is built from: a counter profile is only quoted for the
    kernel it was taken from."""
    import hashlib

    h = hashlib.sha256()
    csrc = os.path.join(ROOT, "paper_1901_10008_amd", "csrc")
    for f in ("kernels.hip.h", "superkernel.hip", "planner.cpp", "sk_internal.h"):
        with open(os.path.join(csrc, f), "rb") as fh:
            h.update(fh.read())
    return h.hexdigest()


def measured_traffic(workload, replicate=1, overrides=None):
    """HBM bytes per superkernel launch from the committed rocprofv3 --pmc summaries (FETCH_SIZE and
    WRITE_SIZE, scaled by what the same counters read for a plain copy of known size): the record for
    this workload, replication and default plan parameters, and only if it was taken from the kernel
    source that is in the tree now.  None otherwise."""
    path = os.path.join(ROOT, "profiles", "superkernel_traffic.json")
    try:
        with open(path) as f:
            recs = json.load(f)
        if overrides:
            return None
        rec = recs[f"{workload} x{replicate}"]
        if rec["kernel_source_sha256"] != kernel_source_hash():
            return None
        return rec
    except (OSError, KeyError, ValueError):
        return None


def cpu_baseline(specs, seed, target_s):
    """The fp64 oracle, as it stands, on the host cores, over a bounded sample of the same mix."""
    import numpy as np

    import workloads
    from oracle import reference as R, rounding as Q

    cores = min(os.cpu_count() or 1, int(os.environ.get("OMP_NUM_THREADS", "0") or 0) or (os.cpu_count() or 1))
    R.set_threads(cores)
    # calibrate on a small GEMM, then take operators in submission order until the budget is used
    a = np.ones((8, 2048), dtype=np.float32)
    b = np.ones((512, 2048), dtype=np.float32)
    R.gemm(a, b)
    t0 = time.perf_counter()
    R.gemm(a, b)
    rate = 2 * 8 * 512 * 2048 / max(time.perf_counter() - t0, 1e-6)
    budget = rate * target_s
    chosen, acc = [], 0
    for i, s in enumerate(specs):
        f = workloads.flops(s)
        if acc + f > budget and chosen:
            continue
        if f > budget:
            continue
        chosen.append(i)
        acc += f
        if acc > 0.9 * budget:
            break
    if not chosen:
        chosen = [min(range(len(specs)), key=lambda i: workloads.flops(specs[i]))]
        acc = workloads.flops(specs[chosen[0]])
    inputs = []
    for i in chosen:
        s = specs[i]
        a32, b32 = workloads.draw_host(s, seed, i)
        inputs.append((s, Q.round_to(s.dtype, a32)[1], Q.round_to(s.dtype, b32)[1]))
    t0 = time.perf_counter()
    for s, av, bv in inputs:
        if s.op == "gemm":
            R.gemm(av, bv)
        else:
            R.conv2d_nhwc(av, bv, s.pad_h, s.pad_w, stride=s.stride)
    dt = time.perf_counter() - t0
    return {"value": round(acc / dt / 1e12, 6), "unit": "TFLOP/s", "cores": cores, "kind": "oracle",
            "sample": f"{len(chosen)} of {len(specs)} operators of the same mix in submission order "
                      f"({acc / 1e9:.2f} GFLOP, {dt:.1f} s, fp64 naive loops, OpenMP over output rows)"}


if __name__ == "__main__":
    main()
