"""GPU parity: the HIP superkernel, called through the C ABI, against the fp64
CPU oracle on the same seeded inputs.  Tolerances: max |c-ref| / max(|ref|,
rms(ref)) <= 1e-5 (fp32), 2e-2 (bf16, fp16), plus the summation-order-free
rounding bound.  Bit-exact: the plan against the reference planner, a relaunch
against the first launch, the index-order plan against the deadline-order plan,
and the coalesced launch against the one-launch-per-operator baseline wherever
their tile tables coincide (plans of one operator); with several operators the
baseline tiles each operator as if it were alone, so its reduction slices can
differ and both are held to the oracle instead."""
import dataclasses
import math
import os

import numpy as np
import pytest
import torch

import paper_1901_10008_amd as sk
import workloads
from workloads import Problem
from oracle import compare, planner as P, reference as R, rounding as Q

import sk_harness as H

pytestmark = pytest.mark.gpu


def _sync():
    torch.cuda.synchronize()


def run_all_modes(specs, seed=0, label="", **batch_kw):
    """Superkernel vs oracle; the one-launch-per-operator baseline (its own tiling, so its own
    summation order) vs oracle; a relaunch and the index-order plan bit-identical to the first launch."""
    b = H.Batch(specs, seed=seed, **batch_kw)
    with b.plan() as plan:
        # plan parity with the reference planner on the real addresses
        table, order, first, count = P.plan(specs)
        assert sk.sk_plan_get_tiles(plan) == table
        assert sk.sk_plan_get_order(plan) == order
        sk.sk_launch(plan, H.stream_handle())
        _sync()
        worst = H.check_against_oracle(b, label + " superkernel")
        coalesced = b.all_output_bits()
        # second launch of the same plan (the queue re-arms itself)
        b.reset_outputs()
        sk.sk_launch(plan, H.stream_handle())
        _sync()
        for x, y in zip(coalesced, b.all_output_bits()):
            assert np.array_equal(x, y), label + ": relaunch differs"
        b.reset_outputs()
        sk.sk_launch_sequential(plan, H.stream_handle())
        _sync()
        H.check_against_oracle(b, label + " sequential")
        # second round of the baseline (its reduction counters re-arm themselves too)
        seq_bits = b.all_output_bits()
        b.reset_outputs()
        sk.sk_launch_sequential(plan, H.stream_handle())
        _sync()
        for i, (x, y) in enumerate(zip(seq_bits, b.all_output_bits())):
            assert np.array_equal(x, y), f"{label}: second sequential round differs on operator {i}"
    with b.plan(edf=0) as plan:
        b.reset_outputs()
        sk.sk_launch(plan, H.stream_handle())
        _sync()
        for i, (x, y) in enumerate(zip(coalesced, b.all_output_bits())):
            assert np.array_equal(x, y), f"{label}: index-order plan differs on operator {i}"
    # LDS tiles handed out through the per-die lists: same table, same bits, whoever runs a tile (twice: the
    # lists' counters re-arm themselves like the queue's)
    for part in (32, 1):
        with b.plan(xcd_part=part) as plan:
            assert sk.sk_plan_get_tiles(plan) == table
            for rnd in range(2):
                b.reset_outputs()
                sk.sk_launch(plan, H.stream_handle())
                _sync()
                for i, (x, y) in enumerate(zip(coalesced, b.all_output_bits())):
                    assert np.array_equal(x, y), f"{label}: xcd_part={part}, launch {rnd}: operator {i} differs"
    return worst


@pytest.mark.parametrize("idx", [1, 2, 3, 4, 6, 7, 8])
def test_config_matches_oracle(idx):
    specs = workloads.config(idx, seed=0)
    worst = run_all_modes(specs, seed=0, label=f"config {idx}")
    print(f"config {idx}: worst gate error {worst}")


@pytest.mark.parametrize("dtype", ["bf16", "f16", "f32"])
def test_configs_in_every_dtype(dtype):
    # the conv mix and a slice of the low-batch GEMM mix, in each operand type
    specs = workloads.config(3, seed=1, dtype=dtype)[4:] + workloads.config(2, seed=1, dtype=dtype)[:4]
    run_all_modes(specs, seed=1, label=f"{dtype}")


def g(m, n, k, dtype="bf16", d=math.inf, a=("normal", 1.0), b=("normal", 0.05)):
    return Problem(op="gemm", dtype=dtype, M=m, N=n, K=k, deadline_ms=d, a_dist=a, b_dist=b)


def c(h, w, cin, cout, r, s, ph, pw, dtype="bf16", nb=1, d=math.inf, st=1):
    return Problem(op="conv", dtype=dtype, Nb=nb, H=h, W=w, Cin=cin, Cout=cout, R=r, S=s, pad_h=ph, pad_w=pw,
                   stride=st, deadline_ms=d, a_dist=("uniform", 0.0, 1.0), b_dist=("normal", 0.1))


RAGGED = [
    g(1, 5, 3, "f32"), g(1, 1, 1), g(17, 33, 129), g(33, 130, 70, "f16"), g(65, 129, 8), g(200, 300, 100, "f32"),
    g(16, 1000, 64), g(32, 40, 4096), g(2, 96, 8192, d=1.5), g(7, 100, 2048, "f32", d=0.25), g(3, 515, 520),
    g(31, 257, 1000, "f16"), g(64, 128, 64), g(128, 128, 128, "f32"), g(129, 130, 136),
    c(5, 5, 3, 7, 3, 3, 1, 1), c(9, 9, 8, 130, 1, 1, 0, 0, d=0.25), c(13, 11, 16, 40, 3, 3, 1, 1, nb=2),
    c(6, 6, 4, 4, 3, 1, 0, 0, "f32"), c(4, 4, 8, 8, 1, 1, 1, 1), c(7, 7, 24, 20, 3, 3, 1, 1, "f16"),
    c(5, 4, 8, 16, 3, 3, 0, 0), c(3, 3, 16, 8, 3, 3, 2, 2), c(10, 10, 5, 6, 3, 3, 1, 1, "f32", nb=3),
    # strides: skinny and LDS-tile classes, 1x1 and 3x3, extents that do not divide, the generic path
    c(9, 8, 16, 40, 3, 3, 1, 1, st=2), c(8, 8, 32, 24, 1, 1, 0, 0, st=2, nb=2), c(30, 29, 8, 130, 3, 3, 1, 1, st=2),
    c(28, 28, 64, 64, 1, 1, 0, 0, "f16", st=2), c(11, 11, 8, 8, 3, 3, 0, 0, "f32", st=3), c(9, 9, 5, 6, 3, 3, 1, 1, st=2),
    # operands that cannot be read in 16-byte pieces, large enough for the matrix-core path: odd reduction
    # lengths in every type, a 3-channel 7x7 stride-2 stem, several 128-blocks per rectangle
    g(300, 200, 77), g(40, 1000, 1001, "f16"), g(130, 260, 37, "f32"), c(40, 40, 3, 64, 7, 7, 3, 3, st=2),
    c(30, 30, 5, 130, 3, 3, 1, 1, "f32"), c(23, 17, 6, 96, 3, 3, 1, 1, "f16", nb=2),
]


def test_ragged_shapes_all_paths():
    run_all_modes(RAGGED, seed=7, label="ragged")


# The direct-load LDS tiles (operands of at least 65 rows that can be read in 16-byte pieces; convolutions with
# whole stages of channels under every tap): reduction lengths with a tail in the last stage, one to many
# stages, rows and columns that end inside a tile, every type (a stage is 64 halves or 32 floats), filters
# from 1x1 to 5x5 and 1x7 (25 and 7 taps), padding on one side, strides 2 and 3, several images per tile,
# the narrow class (at most 64 columns) with its three-stage ring and the wide one with two, single-stage
# tiles, and one convolution with more than 31 taps, which keeps the register-ring path.
DIRECT = [
    g(65, 129, 64), g(200, 64, 72), g(130, 300, 520), g(129, 65, 8), g(256, 128, 4096), g(300, 40, 1096, "f16"),
    g(131, 130, 32, "f32"), g(140, 70, 104, "f32"), g(128, 128, 136, "f32"),
    c(12, 12, 64, 64, 3, 3, 1, 1), c(12, 12, 128, 130, 3, 3, 1, 1, nb=3), c(20, 9, 64, 40, 5, 5, 2, 2),
    c(16, 16, 64, 200, 1, 7, 0, 3), c(17, 15, 64, 64, 3, 3, 1, 0, st=2), c(31, 31, 192, 96, 3, 3, 0, 0, "f16", st=3),
    c(10, 10, 32, 48, 3, 3, 1, 1, "f32", nb=2), c(9, 9, 64, 8, 1, 1, 0, 0, nb=3), c(14, 14, 64, 64, 7, 7, 3, 3),
]


def test_direct_load_tiles():
    run_all_modes(DIRECT, seed=31, label="direct-load tiles")
    # small targets cut the long reductions into slices (hand-over through the workspace)
    b = H.Batch([s for s in DIRECT if H.kg_of(s) >= 1024], seed=32)
    with b.plan(tile_bytes_min=16384, tile_bytes_max=16384) as plan:
        assert max(t["S"] for t in P.decode(sk.sk_plan_get_tiles(plan))) > 1
        sk.sk_launch(plan, H.stream_handle())
        _sync()
        H.check_against_oracle(b, "direct-load tiles, split reductions")
    # the same tiles in the kernel instantiation for mixed types and operands of any alignment (one operator with
    # an odd reduction length brings it in): the build with the most registers in use, where the compiler keeps
    # scalars in spill lanes and fetches them right in front of the direct loads
    b = H.Batch(DIRECT + [g(7, 33, 77, "f32"), g(70, 40, 1001)], seed=33)
    for prm in ({}, {"xcd_part": 2, "grid_limit": 37}, {"tile_bytes_min": 16384, "tile_bytes_max": 16384}):
        with b.plan(**prm) as plan:
            b.reset_outputs()
            sk.sk_launch(plan, H.stream_handle())
            _sync()
            H.check_against_oracle(b, f"direct-load tiles among operands of any alignment {prm}")


def nchw(h, w, cin, cout, r, s, ph, pw, dtype="bf16", nb=1, d=math.inf, st=1):
    return Problem(op="conv_nchw", dtype=dtype, Nb=nb, H=h, W=w, Cin=cin, Cout=cout, R=r, S=s, pad_h=ph, pad_w=pw,
                   stride=st, deadline_ms=d, a_dist=("uniform", 0.0, 1.0), b_dist=("normal", 0.1))


# channel-major convolutions: outputs of one thread each and matrix-core blocks, every type, 1x1 up to 7x7,
# strides, padding on one side only, several images, more than one 128-block in both directions
NCHW = [
    nchw(5, 5, 3, 7, 3, 3, 1, 1), nchw(9, 9, 8, 130, 1, 1, 0, 0, d=0.25), nchw(13, 11, 16, 40, 3, 3, 1, 1, nb=2),
    nchw(6, 6, 4, 4, 3, 1, 0, 0, "f32"), nchw(7, 7, 24, 20, 3, 3, 1, 1, "f16"), nchw(3, 3, 16, 8, 3, 3, 2, 2),
    nchw(10, 10, 5, 6, 3, 3, 1, 1, "f32", nb=3), nchw(30, 29, 8, 130, 3, 3, 1, 1, st=2),
    nchw(40, 40, 3, 64, 7, 7, 3, 3, st=2), nchw(23, 17, 6, 96, 3, 3, 1, 0, "f16", nb=2),
    nchw(28, 28, 64, 64, 1, 1, 0, 0, "f16", st=2), nchw(20, 20, 32, 200, 3, 3, 1, 1, "f32"), nchw(1, 1, 64, 10, 1, 1, 0, 0),
    nchw(14, 14, 256, 256, 3, 3, 1, 1, d=0.5),
]


def test_channel_major_convolutions():
    # among NHWC convolutions and GEMMs of the fast paths, in one plan
    run_all_modes(NCHW + [c(13, 11, 16, 40, 3, 3, 1, 1, nb=2), g(16, 1000, 64), g(129, 130, 136)], seed=21, label="nchw")
    run_all_modes(NCHW[:8], seed=22, label="misaligned nchw", a_off=4, b_off=4, c_off=4)


def test_misaligned_and_strided_operands():
    specs = [s for s in RAGGED if s.op == "gemm"]
    # 2/4-byte offsets break 16-byte alignment (element-wise load/store paths); padded row strides
    run_all_modes(specs, seed=8, label="misaligned", a_off=4, b_off=4, c_off=4)
    run_all_modes(specs, seed=9, label="strided", pad_lda=8, pad_ldb=16, pad_ldc=4)
    run_all_modes(specs, seed=10, label="odd strides", pad_lda=3, pad_ldb=1, pad_ldc=1)
    convs = [s for s in RAGGED if s.op == "conv"]
    run_all_modes(convs, seed=11, label="misaligned conv", a_off=4, b_off=4, c_off=4)


@pytest.mark.parametrize("seed", [int(x) for x in os.environ.get("SK_RANDOM_MIX_SEEDS", "0,1,2,3,4,5,6,7,8,9,10,11").split(",")])
def test_random_mixes_under_random_plan_parameters(seed):
    """Seeded random operator lists under random plan parameters (small tile targets force split reductions in
    every class, including the LDS tiles; tiny group caps force many passes): outputs against the oracle."""
    rng = np.random.default_rng(500 + seed)
    dts = ["bf16", "f16", "f32"]
    specs = []
    for _ in range(14):
        dt = dts[int(rng.integers(0, 3))]
        d = float(rng.choice([np.inf, 0.5, 0.5, 2.0]))
        if rng.random() < 0.6:
            m = int(rng.choice([1, 7, 16, 17, 33, 64, 65, 130, 260]))
            n = int(rng.choice([5, 33, 128, 129, 500, 1024]))
            k = int(rng.choice([8, 64, 72, 77, 256, 1000, 1001, 2048, 4096]))   # 77, 1001: not readable in 16-byte pieces
            specs.append(g(m, n, k, dt, d=d))
        else:
            hw = int(rng.choice([4, 7, 9, 14, 20]))
            r = int(rng.choice([1, 3]))
            make = nchw if seed >= 2 and rng.random() < 0.3 else c   # (seeds 0 and 1 keep their earlier draws)
            specs.append(make(hw, hw, int(rng.choice([3, 8, 16, 64, 128, 256])), int(rng.choice([8, 40, 64, 128, 136])),
                              r, r, r // 2, r // 2, dt, nb=int(rng.integers(1, 3)), d=d, st=int(rng.choice([1, 1, 2]))))
    tmin = int(rng.choice([4096, 32768, 1 << 17]))
    prm = {"skinny_max_m": int(rng.choice([16, 32, 64])), "tile_bytes_min": tmin,
           "tile_bytes_max": tmin * int(rng.choice([1, 4, 16])), "balance_div": int(rng.choice([16, 2048])),
           "max_groups": int(rng.choice([4, 8, 256])), "tail_div": int(rng.choice([0, 8, 384])),
           "grid_limit": int(rng.choice([0, 7, 100]))}
    prm["xcd_part"] = [0, 2, 32, 1][seed % 4]   # seeds 1 to 3: LDS tiles handed out through the per-die lists
    b = H.Batch(specs, seed=seed)
    with b.plan(**prm) as plan:
        ref = {k: v for k, v in prm.items() if k not in ("grid_limit", "xcd_part")}
        assert sk.sk_plan_get_tiles(plan) == P.plan(specs, P.Params(**ref))[0]
        for launch in (sk.sk_launch, sk.sk_launch_sequential, sk.sk_launch):
            b.reset_outputs()
            launch(plan, H.stream_handle())
            _sync()
            H.check_against_oracle(b, f"random mix {seed} {prm}")


@pytest.mark.parametrize("grid", [3, 9, 40, 0])
def test_die_lists_under_every_hand_over(grid):
    """LDS tiles taken from the per-die lists with few workgroups (so that each runs many tiles and every way
    from one tile to the next occurs: an entry drawn in advance and used, drawn and kept over skinny tiles,
    drawn on the spot, taken from another die's list, run after the tickets are used up, tickets that stand
    for nothing), with split reductions and completion stamps: bit for bit what the plain queue gives."""
    specs = (workloads.config(3, seed=0) + workloads.config(2, seed=2)[:6] + workloads.config(4, seed=0)[:5]
             + workloads.config(3, seed=1, dtype="f16")[3:6] + [g(200, 300, 72, "f32"), g(130, 129, 1001, "bf16")])
    # interleave skinny and LDS-tile operators in the execution order
    specs = [dataclasses.replace(s, deadline_ms=1.0 + (7 * i) % len(specs)) for i, s in enumerate(specs)]
    b = H.Batch(specs, seed=5)
    prm = {"grid_limit": grid, "tile_bytes_min": 16384, "tile_bytes_max": 262144}
    with b.plan(**prm) as plan:
        sk.sk_launch(plan, H.stream_handle())
        _sync()
        H.check_against_oracle(b, f"die lists, grid {grid}: plain queue")
        want = b.all_output_bits()
        n_lds = sum(t["cls"] >= P.CLS_TILE_128x128 for t in P.decode(sk.sk_plan_get_tiles(plan)))
        n_all = sk.sk_plan_num_tiles(plan)
    assert 0 < n_lds < n_all
    for part in (1, 4, 32):
        with b.plan(xcd_part=part, stamps=1, **prm) as plan:
            assert sum(len(l) for l in sk.sk_plan_get_xcd_lists(plan)) == n_lds
            for rnd in range(3):
                b.reset_outputs()
                sk.sk_launch(plan, H.stream_handle())
                _sync()
                for i, (x, y) in enumerate(zip(want, b.all_output_bits())):
                    assert np.array_equal(x, y), f"grid {grid}, xcd_part {part}, launch {rnd}: operator {i} differs"
                done, start, rate = sk.sk_plan_get_stamps(plan)
                assert all(d >= start for d in done), "an operator without a completion stamp"


def test_tuner_sweeps_plan_parameters():
    from paper_1901_10008_amd import tune
    specs = workloads.config(2, seed=0)
    b = H.Batch(specs, seed=0)
    grid = {"tile_bytes_max": (256 << 10, 2 << 20), "tail_div": (0, 384)}
    best, res = tune.tune(b.problems, grid, rounds=2, launches=2, stream=H.stream_handle())
    assert len(res) == 4 and all(t > 0 and n > 0 for _, t, n in res)
    assert res[0][0] == best and res[0][1] == min(t for _, t, _ in res)
    assert set(best) == {"tile_bytes_max", "tail_div"}
    # the tuner only times launches: outputs are whatever the last plan wrote, and still right
    H.check_against_oracle(b, "after tuning")
    rep = tune.cotenancy(b.problems, 0, (1 << 15, 1 << 18, 1 << 21), rounds=2, launches=2, stream=H.stream_handle())
    assert len(rep["solo_us"]) == 3 and len(rep["mix_us"]) == 3
    assert rep["solo_penalty_with_mix_best"] >= 1.0 and rep["mix_penalty_with_solo_best"] >= 1.0


def test_tuned_parameters_are_picked_up_by_a_second_process(tmp_path):
    """The tuning phase leaves its result in a file (Section 5.3: the runtime applies pre-computed parameters); a
    second process that only knows the operator shapes finds the record and plans with it; launched with the
    loaded parameters the outputs are still the oracle's."""
    import json
    import subprocess
    import sys
    from paper_1901_10008_amd import tune
    specs = workloads.config(2, seed=0)[:8] + workloads.config(4, seed=0)[:6]
    b = H.Batch(specs, seed=0)
    path = str(tmp_path / "tuned.jsonl")
    grid = {"tile_bytes_max": (256 << 10, 2 << 20), "skinny_max_m": (32, 64)}
    best, res = tune.tune(b.problems, grid, rounds=2, launches=2, stream=H.stream_handle())
    tune.save(path, b.problems, best, res[0][1], note="test")
    # the other process: shapes only (made-up addresses), no GPU work
    child = (
        "import json, sys, workloads, paper_1901_10008_amd as sk\n"
        "from paper_1901_10008_amd import tune\n"
        "specs = workloads.config(2, seed=0)[:8] + workloads.config(4, seed=0)[:6]\n"
        "probs = [sk.make_problem(s, 4096 * (3 * i + 1), 4096 * (3 * i + 2), (1 << 40) + (i << 32)) for i, s in enumerate(specs)]\n"
        "p = tune.tuned_params(probs, sys.argv[1])\n"
        "p.host_only = 1\n"
        "plan = sk.sk_plan_create(probs, p)\n"
        "print(json.dumps({'tile_bytes_max': p.tile_bytes_max, 'skinny_max_m': p.skinny_max_m, 'tiles': sk.sk_plan_num_tiles(plan)}))\n")
    out = subprocess.run([sys.executable, "-c", child, path], capture_output=True, text=True, cwd=os.path.dirname(H.__file__) + "/..")
    assert out.returncode == 0, out.stderr
    seen = json.loads(out.stdout.strip().splitlines()[-1])
    assert seen["tile_bytes_max"] == best["tile_bytes_max"] and seen["skinny_max_m"] == best["skinny_max_m"]
    loaded = tune.tuned_params(b.problems, path)
    with sk.sk_plan_create(b.problems, loaded, keepalive=b) as plan:
        assert sk.sk_plan_num_tiles(plan) == seen["tiles"]
        b.reset_outputs()
        sk.sk_launch(plan, H.stream_handle())
        _sync()
        H.check_against_oracle(b, "tuned parameters from the file")


def test_arrival_trace_policies():
    """Operators arriving over time under the three batching policies: every arrival is served, and whatever
    the batching, the outputs are the oracle's."""
    from paper_1901_10008_amd import serve
    specs = workloads.config(2, seed=0)
    b = H.Batch(specs, seed=0)
    trace = serve.poisson_trace([workloads.algorithmic_bytes(s) for s in specs], 60, rate_per_ms=40.0, seed=1)
    assert len(trace) == 60 and all(x.t_ms < y.t_ms for x, y in zip(trace, trace[1:]))
    for policy, depth, cap in (("sequential", 0, 0.5), ("coalesce", 0, 0.5), ("ooo", 0, 0.5), ("coalesce", 1, 0.5),
                               ("ooo", 3, 0.03)):
        b.reset_outputs()
        rep = serve.run_trace(b.problems, trace, policy, cap_ms=cap, depth=depth)
        _sync()
        assert rep["operators"] == 60 and 0.0 <= rep["met_fraction"] <= 1.0
        assert rep["launches"] == 60 if policy == "sequential" else rep["launches"] <= 60
        served = {a.index for a in trace}
        H.check_against_oracle(b, "trace " + policy, only=served)


def test_arrival_queue_calls():
    """The queue through its C calls: tickets, completions in full, operators that share an output buffer go
    into different launches, a batch the planner rejects completes as failed, an empty queue polls empty."""
    import ctypes as C
    specs = workloads.config(2, seed=3)[:6]
    b = H.Batch(specs, seed=3)
    n = len(specs)
    ops = (sk.sk_problem * (2 * n))(*b.problems, *b.problems)     # every operator twice: same output buffers
    budgets = (C.c_double * (2 * n))(*([1.0] * n + [0.0] * n))      # the second half without a budget
    tickets = (C.c_uint64 * (2 * n))()
    done = (sk.sk_completion * 64)()
    side = torch.cuda.Stream()
    with sk.sk_queue_create(sk.sk_queue_params_default(policy="coalesce"), side.cuda_stream) as q:
        assert sk.sk_queue_poll(q, done, wait=True) == 0             # nothing submitted: returns at once
        sk.sk_queue_submit(q, ops, budgets, 0, 2 * n, tickets)
        assert list(tickets) == list(range(1, 2 * n + 1))
        seen = {}
        while len(seen) < 2 * n:
            for i in range(sk.sk_queue_poll(q, done, wait=True)):
                seen[done[i].ticket] = (done[i].launch, done[i].met, done[i].latency_ms, done[i].budget_ms)
        st = sk.sk_queue_get_stats(q)
        assert (st.submitted, st.completed, st.launches) == (2 * n, 2 * n, 2) and st.device_busy_ms > 0
        for i in range(n):
            first, second = seen[tickets[i]], seen[tickets[n + i]]
            assert first[0] != second[0], "two operators with one output buffer shared a launch"
            assert first[1] in (0, 1) and second[1] == 1 and second[3] == math.inf and 0 < first[2] < 1000
        side.synchronize()
        H.check_against_oracle(b, "queue")
        # a batch the planner rejects (a dimension of zero): its operator completes as failed, the call says why
        bad = (sk.sk_problem * 1)(b.problems[0])
        bad[0].M = 0
        with pytest.raises(sk.SkError) as e:
            sk.sk_queue_submit(q, bad, None, 0, 1, None)
        assert e.value.status == sk.SK_ERR_INVALID_ARG
        assert sk.sk_queue_poll(q, done, wait=True) == 1 and done[0].met == -1
    with pytest.raises(sk.SkError):
        sk.sk_queue_create(sk.sk_queue_params_default(cap_ms=0.0))


def test_recycled_plan_tables():
    """Destroyed plans hand their device tables to the next plan.  A recycled block holds the last plan's
    queue counters, split-K arrival counts and partial sums; results must not depend on them.  A plan may
    be destroyed while its launch still runs."""
    big = workloads.config(2, seed=3)[:10] + workloads.config(3, seed=1)[:4]
    small = workloads.config(2, seed=4)[:7]
    bb, bs = H.Batch(big, seed=3), H.Batch(small, seed=4)
    split = {"tile_bytes_min": 4096, "tile_bytes_max": 4096}  # many reduction slices: arrival counters in use
    for rnd in range(3):
        for b, prm in ((bb, split), (bs, split), (bb, {}), (bs, {"stamps": 1}), (bb, split)):
            b.reset_outputs()
            plan = b.plan(**prm)
            sk.sk_launch(plan, H.stream_handle())
            plan.close()           # no synchronisation by the caller
            _sync()
            H.check_against_oracle(b, f"recycled round {rnd} {prm}")
        if rnd == 1:
            sk.sk_release_cached_memory()
    sk.sk_release_cached_memory()
    sk.sk_release_cached_memory()  # empty pool


def test_launches_replayed_from_a_graph():
    """Both launch calls captured into HIP graphs and replayed several times, with eager launches and
    synchronisations between the replays: every replay gives the oracle's result (the kernels re-arm
    their own counters; nothing in the captured work is a memset)."""
    specs = workloads.config(2, seed=1)[:8] + workloads.config(3, seed=0)[3:6]
    b = H.Batch(specs, seed=1)
    side = torch.cuda.Stream()
    with b.plan(tile_bytes_min=8192, tile_bytes_max=8192) as plan:   # small tiles: split reductions in the graph
        graphs = []
        for launch in (sk.sk_launch, sk.sk_launch_sequential):
            with torch.cuda.stream(side):
                launch(plan, side.cuda_stream)
                side.synchronize()
                gr = torch.cuda.CUDAGraph()
                with torch.cuda.graph(gr, stream=side):
                    launch(plan, side.cuda_stream)
            graphs.append(gr)
        _sync()
        for rep in range(3):
            for gi, gr in enumerate(graphs):
                b.reset_outputs()
                _sync()
                gr.replay()
                _sync()
                H.check_against_oracle(b, f"graph {gi} replay {rep}")
                b.reset_outputs()
                sk.sk_launch(plan, H.stream_handle())   # eager work between the replays
                _sync()
                H.check_against_oracle(b, f"eager after graph {gi} replay {rep}")
        del graphs


def test_plans_running_concurrently_on_several_streams():
    """The spatial-multiplexing baseline (Section 4.2): one plan per operator over several streams at once, and a
    coalesced plan of other operators beside them.  Plans share nothing but read-only state, so every output is
    the oracle's; plans are destroyed while later launches still run."""
    specs = workloads.config(2, seed=7)[:10] + workloads.config(3, seed=0)[1:5] + workloads.config(4, seed=1)[:4]
    b = H.Batch(specs, seed=12)
    streams = [torch.cuda.Stream() for _ in range(4)]
    for rep in range(3):
        b.reset_outputs()
        _sync()
        singles = [sk.sk_plan_create([p], sk.sk_plan_params_default(stamps=rep % 2)) for p in b.problems[:12]]
        rest = sk.sk_plan_create(b.problems[12:], sk.sk_plan_params_default(tile_bytes_min=8192, tile_bytes_max=8192))
        for i, pl in enumerate(singles):
            sk.sk_launch(pl, streams[i % 4].cuda_stream)
        sk.sk_launch(rest, H.stream_handle())
        for i, pl in enumerate(singles):
            if i % 3 == 0:     # a second launch of the same plan: behind the first one, on its stream
                sk.sk_launch_sequential(pl, streams[i % 4].cuda_stream)
        for pl in singles[::2]:
            pl.close()          # waits for that plan's own launches only
        _sync()
        for pl in singles[1::2] + [rest]:
            pl.close()
        H.check_against_oracle(b, f"concurrent streams round {rep}")


def test_host_threads_plan_and_launch_side_by_side():
    """Serving threads each plan, launch and destroy their own plans (own stream, own operators) at the
    same time: the table pool is shared, the upload staging and the error string are per thread."""
    import threading

    nthreads, rounds = 4, 6
    batches = [H.Batch(workloads.config(2, seed=20 + t)[:6] + workloads.config(3, seed=0)[t: t + 2], seed=30 + t)
               for t in range(nthreads)]
    reference_tables = []
    for b in batches:
        with b.plan(host_only=1) as plan:
            reference_tables.append(sk.sk_plan_get_tiles(plan))
    errors = []

    def serve(t):
        try:
            torch.cuda.set_device(0)
            stream = torch.cuda.Stream()
            b = batches[t]
            for r in range(rounds):
                with sk.sk_plan_create(b.problems, sk.sk_plan_params_default(stamps=r % 2)) as plan:
                    assert sk.sk_plan_get_tiles(plan) == reference_tables[t]
                    if r % 3 == 2:
                        sk.sk_launch_sequential(plan, stream.cuda_stream)
                    else:
                        sk.sk_launch(plan, stream.cuda_stream)
                    if r % 2:
                        stream.synchronize()
                with pytest.raises(sk.SkError) as bad:   # an error in one thread: its own detail string
                    sk.sk_plan_create([sk.make_problem(Problem(op="gemm", dtype="bf16", M=t + 1, N=8, K=8), 0, 0, 0)])
                assert "null" in bad.value.detail
            stream.synchronize()
        except BaseException as e:  # noqa: BLE001 -- reported by the main thread
            errors.append((t, repr(e)))

    threads = [threading.Thread(target=serve, args=(t,)) for t in range(nthreads)]
    for th in threads:
        th.start()
    for th in threads:
        th.join()
    assert not errors, errors
    _sync()
    for t, b in enumerate(batches):
        H.check_against_oracle(b, f"thread {t}")


def test_thousands_of_tiny_operators():
    """Far more operators than workgroups: 3000 GEMMs and convolutions of a few hundred outputs each, every
    fourth with a deadline, in one plan; coalesced, one launch per operator, and with completion stamps."""
    rng = np.random.default_rng(77)
    specs = []
    for i in range(3000):
        d = float(rng.choice([0.2, 0.5, 1.0])) if i % 4 == 0 else math.inf
        if i % 5 == 4:
            specs.append(c(int(rng.integers(2, 6)), int(rng.integers(2, 6)), 8, 8, 3, 3, 1, 1, d=d))
        else:
            specs.append(g(int(rng.integers(1, 9)), int(rng.choice([8, 16, 40, 64])), int(rng.choice([8, 24, 64])), d=d))
    b = H.Batch(specs, seed=31)
    with b.plan(stamps=1) as plan:
        table, order, first, count = P.plan(specs)
        assert sk.sk_plan_get_tiles(plan) == table and sk.sk_plan_get_order(plan) == order
        sk.sk_launch(plan, H.stream_handle())
        _sync()
        H.check_against_oracle(b, "tiny operators")
        done, start, rate = sk.sk_plan_get_stamps(plan)
        # the start stamp is the earliest first clock of any workgroup: no operator can complete before it
        assert len(done) == len(specs) and min(done) >= start and max(done) <= start + 50.0 * rate, \
            (start, min(done), max(done), rate)
        print(f"earliest completion {(min(done) - start) / rate * 1e3:.2f} us after the launch started, latest {(max(done) - start) / rate * 1e3:.1f} us")
        b.reset_outputs()
        sk.sk_launch_sequential(plan, H.stream_handle())
        _sync()
        H.check_against_oracle(b, "tiny operators, sequential")


@pytest.mark.parametrize("idx", [1, 2, 3, 4])
def test_one_operator_plans_coalesced_equals_sequential_bit_for_bit(idx):
    """Packing must not change a result (Section 1, item (b): the streams' operators are independent).
    For a plan of one operator the coalesced table and the baseline's table are the same table, so the
    two launch calls must produce identical bits: same tiles, same reduction slices, same order of
    summation, whichever workgroup takes which tile."""
    specs = workloads.config(idx, seed=0)
    b = H.Batch(specs, seed=0)
    for i, p in enumerate(b.problems):
        for prm in ({}, {"tile_bytes_min": 8192, "tile_bytes_max": 8192}):   # the second: split reductions
            with sk.sk_plan_create([p], sk.sk_plan_params_default(**prm)) as plan:
                b.reset_outputs()
                sk.sk_launch(plan, H.stream_handle())
                _sync()
                one = b.output_bits(i)
                b.reset_outputs()
                sk.sk_launch_sequential(plan, H.stream_handle())
                _sync()
                assert np.array_equal(one, b.output_bits(i)), f"config {idx} operator {i} {prm}"
    H.check_against_oracle(b, f"config {idx}, last operator only", only={len(specs) - 1})


def test_operator_order_does_not_change_any_result():
    """The same operators submitted in another order (and so packed in another order) give the same bits per
    operator, as long as the tile sizes do not depend on the position (tail rule off)."""
    specs = workloads.config(2, seed=2)[:8] + workloads.config(3, seed=0)[2:6] + workloads.config(4, seed=2)[:6]
    b = H.Batch(specs, seed=2)
    perm = np.random.default_rng(4).permutation(len(specs))
    with b.plan(tail_div=0) as plan:
        sk.sk_launch(plan, H.stream_handle())
        _sync()
        H.check_against_oracle(b, "submission order")
        first = b.all_output_bits()
    b.reset_outputs()
    shuffled = [b.problems[j] for j in perm]
    with sk.sk_plan_create(shuffled, sk.sk_plan_params_default(tail_div=0)) as plan:
        sk.sk_launch(plan, H.stream_handle())
        _sync()
    for i, (x, y) in enumerate(zip(first, b.all_output_bits())):
        assert np.array_equal(x, y), f"operator {i} changed with the submission order"


def test_second_stream_is_refused_while_the_plan_still_runs():
    """A plan has one tile queue: a launch on another stream while the previous one still runs is refused
    with SK_ERR_BUSY (nothing is launched), and admitted once that launch has completed."""
    specs = workloads.config(2, seed=0) * 8   # 128 launches' worth of work for the sequential call: milliseconds
    b = H.Batch(specs, seed=0)
    other = torch.cuda.Stream()
    with b.plan() as plan:
        sk.sk_launch_sequential(plan, H.stream_handle())   # (builds the baseline tables)
        _sync()
        for _ in range(3):
            sk.sk_launch_sequential(plan, H.stream_handle())
        with pytest.raises(sk.SkError) as e:
            sk.sk_launch(plan, other.cuda_stream)
        assert e.value.status == sk.SK_ERR_BUSY
        with pytest.raises(sk.SkError) as e:
            sk.sk_launch_sequential(plan, other.cuda_stream)
        assert e.value.status == sk.SK_ERR_BUSY
        sk.sk_launch(plan, H.stream_handle())               # the same stream is always fine
        _sync()
        b.reset_outputs()
        sk.sk_launch(plan, other.cuda_stream)               # the previous launch has completed
        other.synchronize()
        H.check_against_oracle(b, "after the refusals")
        sk.sk_launch(plan, H.stream_handle())               # and back
        _sync()


def test_single_and_empty_plans():
    run_all_modes([g(1, 64, 64)], seed=3, label="single")
    with sk.sk_plan_create([], None) as plan:
        assert sk.sk_plan_grid(plan) == 0
        sk.sk_launch(plan, H.stream_handle())
        sk.sk_launch_sequential(plan, H.stream_handle())
        _sync()


def test_small_grid_and_split_modes():
    # few persistent workgroups: every workgroup walks many tiles through the atomic queue
    specs = workloads.config(2, seed=5)[:6] + workloads.config(3, seed=0)[2:5]
    b = H.Batch(specs, seed=5)
    ref_bits = None
    for prm in ({"grid_limit": 3}, {"grid_limit": 64}, {}):
        with b.plan(**prm) as plan:
            b.reset_outputs()
            sk.sk_launch(plan, H.stream_handle())
            _sync()
            H.check_against_oracle(b, f"grid {prm}")
            bits = b.all_output_bits()
            if ref_bits is not None:
                for x, y in zip(ref_bits, bits):
                    assert np.array_equal(x, y)
            ref_bits = bits
    # tile-size parameters change the reduction split (wk = 1, 2, 4): all within tolerance
    for prm in ({"tile_bytes_min": 4096, "tile_bytes_max": 4096}, {"tile_bytes_min": 1 << 20, "tile_bytes_max": 1 << 20},
                {"skinny_max_m": 0}, {"skinny_max_m": 16}):
        with b.plan(**prm) as plan:
            assert sk.sk_plan_get_tiles(plan) == P.plan(specs, P.Params(**prm))[0]
            b.reset_outputs()
            sk.sk_launch(plan, H.stream_handle())
            _sync()
            H.check_against_oracle(b, f"params {prm}")


def test_exact_integer_products():
    # small integers: every product and partial sum is exact in fp32 and bf16, so the result is exact
    M, N, K = 9, 70, 96
    A = (np.arange(M * K).reshape(M, K) % 5 - 2).astype(np.float32)
    B = (np.arange(N * K).reshape(N, K) % 7 - 3).astype(np.float32)
    want = R.gemm(A, B)
    for dtype in ("bf16", "f16", "f32"):
        spec = g(M, N, K, dtype)
        b = H.Batch([spec], seed=0)
        bitsA, _ = Q.round_to(dtype, A)
        bitsB, _ = Q.round_to(dtype, B)
        b.bufs[0].zero_()
        b.bufs[0][:M * K] = torch.from_numpy(bitsA.view(np.int32 if dtype == "f32" else np.int16).ravel()).to("cuda")
        b.bufs[1][:N * K] = torch.from_numpy(bitsB.view(np.int32 if dtype == "f32" else np.int16).ravel()).to("cuda")
        with b.plan() as plan:
            sk.sk_launch(plan, H.stream_handle())
            _sync()
        assert np.array_equal(b.output(0), want), dtype


@pytest.mark.parametrize("dtype,keep,extra", [("bf16", 8, 8), ("f16", 11, 10)])
def test_outputs_round_to_nearest_even(dtype, keep, extra):
    """Accumulators with more bits than the output type, exact in fp32: the stored pattern must be the
    round-to-nearest-even one, bit for bit (ties both ways, carries into the exponent, overflow to inf)."""
    rng = np.random.default_rng(7)
    n = 4096
    # x = sign * 1.f * 2^e with `keep + extra` significant bits
    mant = rng.integers(1 << (keep + extra - 1), 1 << (keep + extra), size=n).astype(np.int64)
    half = 1 << (extra - 1)
    mant[:512] = (mant[:512] >> extra << extra) | half                       # exact ties, upper part even or odd
    mant[512:640] = (1 << (keep + extra)) - 1 - rng.integers(0, half, size=128)  # round up into the next binade
    e = rng.integers(0, 6, size=n)
    x = (mant.astype(np.float64) * np.exp2(e - (keep + extra - 1))).astype(np.float32)
    x *= np.where(rng.integers(0, 2, size=n) == 1, -1.0, 1.0).astype(np.float32)
    if dtype == "bf16":
        x[640:648] = np.array([0x7F7FFF00, 0x7F7F8000, 0x7F7F7F00, 0x7F7F0000, 0xFF7FFF00, 0x00800000,
                               0x7F800000, 0xFF800000], dtype=np.uint32).view(np.float32)
    trunc_mask = np.uint32(0xFFFF0000) if dtype == "bf16" else None
    if dtype == "bf16":
        hi = (x.view(np.uint32) & trunc_mask).view(np.float32)
    else:
        hi = (mant >> extra << extra).astype(np.float64) * np.exp2(e - (keep + extra - 1))
        hi = (np.sign(x) * hi).astype(np.float32)
    with np.errstate(invalid="ignore"):
        rem = np.where(np.isfinite(x), x - hi, 0.0).astype(np.float32)
    hb, hv = Q.round_to(dtype, hi)
    rb, rv = Q.round_to(dtype, rem)
    assert np.array_equal(hv, hi) and np.array_equal(rv, rem), "test values must be exact in the input type"
    want_bits, _ = Q.round_to(dtype, x)
    K = 16
    for M in (1, 40, 70):                      # one, four row blocks; LDS tile
        A = np.zeros((M, K), dtype=np.float32)
        A[:, 0] = 1.0
        A[:, 1] = 1.0
        B = np.zeros((n, K), dtype=np.float32)
        B[:, 0] = hi
        B[:, 1] = rem
        spec = g(M, n, K, dtype)
        b = H.Batch([spec], seed=0)
        bitsA, _ = Q.round_to(dtype, A)
        bitsB, _ = Q.round_to(dtype, B)
        b.bufs[0].zero_()
        b.bufs[1].zero_()
        b.bufs[0][:M * K] = torch.from_numpy(bitsA.view(np.int16).ravel()).to("cuda")
        b.bufs[1][:n * K] = torch.from_numpy(bitsB.view(np.int16).ravel()).to("cuda")
        with b.plan() as plan:
            sk.sk_launch(plan, H.stream_handle())
            _sync()
        got = b.output_bits(0)
        for m in range(M):
            bad = np.nonzero(got[m] != want_bits.view(got.dtype))[0]
            assert bad.size == 0, (dtype, M, m, bad[:5], x[bad[:5]], got[m][bad[:5]], want_bits[bad[:5]])


def test_completion_stamps():
    specs = workloads.config(5, seed=0)[:24]
    b = H.Batch(specs, seed=0)
    with b.plan(stamps=1) as plan:
        for launch in (sk.sk_launch, sk.sk_launch_sequential, sk.sk_launch):
            b.reset_outputs()
            launch(plan, H.stream_handle())
            _sync()
            done, start, rate = sk.sk_plan_get_stamps(plan)
            assert rate > 0 and len(done) == len(specs)
            lat_ms = [(d - start) / rate for d in done]
            assert all(0 <= x < 1000 for x in lat_ms), lat_ms
            H.check_against_oracle(b, "stamps")
    with b.plan() as plan:
        with pytest.raises(sk.SkError):
            sk.sk_plan_get_stamps(plan)
