"""Host-side logic that needs no GPU: arrival traces, duration estimates, tuner candidate grids."""
import math

from paper_1901_10008_amd import serve, tune


def test_poisson_trace_is_seeded_sorted_and_in_range():
    sizes = [1000, 2000, 3000, 4000]
    a = serve.poisson_trace(sizes, 500, rate_per_ms=20.0, seed=3)
    b = serve.poisson_trace(sizes, 500, rate_per_ms=20.0, seed=3)
    c = serve.poisson_trace(sizes, 500, rate_per_ms=20.0, seed=4)
    assert [(x.index, x.t_ms, x.budget_ms) for x in a] == [(x.index, x.t_ms, x.budget_ms) for x in b]
    assert [(x.index, x.t_ms) for x in a] != [(x.index, x.t_ms) for x in c]
    assert all(x.t_ms < y.t_ms for x, y in zip(a, a[1:]))
    assert all(0 <= x.index < 4 and x.bytes == sizes[x.index] and 0.5 <= x.budget_ms <= 5.0 for x in a)
    # mean gap of an exponential with rate 20 per ms is 0.05 ms (500 samples: within 20 %)
    assert abs(a[-1].t_ms / 500 - 0.05) < 0.01
    assert {x.index for x in a} == {0, 1, 2, 3}


def test_duration_estimate_has_a_floor_and_scales_with_bytes():
    assert serve.estimate_ms(0) == serve.LAUNCH_FLOOR_MS
    assert serve.estimate_ms(10 ** 9) == 10 ** 9 / serve.HBM_BYTES_PER_MS
    assert math.isclose(serve.estimate_ms(4 * 10 ** 9), 4 * serve.estimate_ms(10 ** 9))


def test_tuner_candidates_span_the_grid():
    cands = tune.candidates({"tile_bytes_max": (1, 2), "tail_div": (0, 384, 768)})
    assert len(cands) == 6 and {"tile_bytes_max": 2, "tail_div": 768} in cands
    assert len(tune.candidates()) == math.prod(len(v) for v in tune.DEFAULT_GRID.values())
    assert len({tuple(sorted(c.items())) for c in tune.candidates()}) == len(tune.candidates())


def test_ceilings_library_exports_its_two_calls():
    import ctypes
    import os
    import paper_1901_10008_amd
    path = os.path.join(os.path.dirname(paper_1901_10008_amd.__file__), "libsk_ceilings.so")
    lib = ctypes.CDLL(path)   # built by paper_1901_10008_amd.build; loading needs no GPU
    assert lib.sk_ceiling_stream_read and lib.sk_ceiling_mfma_bf16 and lib.sk_ceiling_lds_read


def test_tuned_parameters_round_trip_through_a_file(tmp_path):
    import ctypes
    import paper_1901_10008_amd as sk
    from workloads import Problem
    specs = [Problem(op="gemm", dtype="bf16", M=4, N=512, K=1024), Problem(op="gemm", dtype="f16", M=70, N=256, K=128),
             Problem(op="conv", dtype="bf16", Nb=1, H=14, W=14, Cin=64, Cout=64, R=3, S=3, pad_h=1, pad_w=1)]
    probs = [sk.make_problem(s, 0x1000 * (i + 1), 0x100000 * (i + 1), 0x10000000 * (i + 1)) for i, s in enumerate(specs)]
    path = str(tmp_path / "sub" / "tuned.jsonl")
    assert tune.load(path) == {} and tune.tuned_params(probs, path) is None
    sig = tune.save(path, probs, {"tile_bytes_max": 1 << 20, "tail_div": 0, "skinny_max_m": 32}, 12.5, note="first")
    # the signature ignores order and addresses, not shapes
    moved = [sk.make_problem(s, 0x77000, 0x88000, 0x99000 + 0x100000 * i) for i, s in enumerate(reversed(specs))]
    assert tune.signature(moved) == sig == tune.signature(probs)
    assert tune.signature(probs[:2]) != sig
    got = tune.tuned_params(moved, path)
    assert (got.tile_bytes_max, got.tail_div, got.skinny_max_m) == (1 << 20, 0, 32)
    assert got.balance_div == sk.sk_plan_params_default().balance_div           # untouched fields keep their defaults
    tune.save(path, probs, {"tile_bytes_max": 2 << 20}, 11.0, note="second")    # a later record of the same mix wins
    assert tune.tuned_params(probs, path).tile_bytes_max == 2 << 20 and len(tune.load(path)) == 1
    assert tune.tuned_params(probs[:1], path) is None
    # a plan made with the loaded parameters is the plan made with the same values given by hand (host-only: no GPU)
    loaded = tune.tuned_params(probs, path)
    loaded.host_only = 1
    with sk.sk_plan_create(probs, loaded) as a, \
            sk.sk_plan_create(probs, sk.sk_plan_params_default(host_only=1, tile_bytes_max=2 << 20)) as b:
        assert sk.sk_plan_get_tiles(a) == sk.sk_plan_get_tiles(b)


def test_cotenancy_table_marks_both_optima():
    rep = {"targets": [1024, 2048], "solo_us": [10.0, 12.0], "mix_us": [90.0, 80.0], "solo_best_target": 1024,
           "mix_best_target": 2048, "solo_penalty_with_mix_best": 1.2, "mix_penalty_with_solo_best": 1.125}
    txt = tune.cotenancy_table(rep, "operator 0")
    assert "best alone" in txt.splitlines()[3] and "best for the mix" in txt.splitlines()[4] and "x1.2;" in txt


def test_tile_phase_table_from_stamps():
    """tile_phases: the table is built from the stamps alone (no device): tiles without stamps are skipped,
    classes and reduction slices are told apart, times are differences of the 100 MHz stamps in microseconds."""
    import numpy as np
    from paper_1901_10008_amd import tile_phases as tp

    st = np.zeros((16, 64, 8), dtype=np.int64)
    # one skinny 16-row tile: taken up at 1000, set-up 100 ticks, first step 300, loop 10000, outputs 50, hand-over 150
    st[0, 0] = [1000, 1100, 1400, 11400, 11450, 11600, 1 + 0 + 100 * 1, 0]
    # two 128x128 slices of a split reduction (3 slices) with different loop times
    st[1, 0] = [0, 200, 400, 2400, 2600, 2700, 1 + 9 + 100 * 3, 0]
    st[1, 1] = [5000, 5200, 5400, 9400, 9600, 9700, 1 + 9 + 100 * 3, 0]
    st[2, 5] = [7, 0, 0, 0, 0, 0, 1 + 6 + 100, 0]   # a tile that left no further stamps: skipped
    txt = tp.phase_table(st).splitlines()
    assert len(txt) == 3
    sk16 = txt[1].split()
    assert txt[1].startswith("skinny, 16 rows") and sk16[-6:] == ["1.00", "3.00", "100.00", "0.50", "1.50", "106.00"] and sk16[-7] == "1"
    sl = txt[2].split()
    assert txt[2].startswith("LDS tile 128x128, slice") and sl[-7] == "2"
    assert sl[-6:] == ["2.00", "2.00", "30.00", "2.00", "1.00", "37.00"]


def test_tile_phase_end_summary_from_stamps():
    """When the workgroups of a launch finish, from hand-made stamps (100 ticks per microsecond)."""
    import numpy as np
    from paper_1901_10008_amd import tile_phases
    st = np.zeros((3, 4, 8), dtype=np.int64)
    # workgroup 0: two tiles, ends at tick 21000; workgroup 1: one LDS tile, ends at 30000; workgroup 2: nothing
    st[0, 0] = [1000, 1100, 1400, 9000, 9100, 9200, 1 + 0 + 100, 0]
    st[0, 1] = [9200, 9300, 9600, 20000, 20500, 21000, 1 + 6 + 100, 0]
    st[1, 0] = [2000, 2100, 2400, 29000, 29500, 30000, 1 + 9 + 100, 0]
    text = tile_phases.end_summary(st)
    # begin = 1000; ends 200 and 290 us after it; mean 245, idle 45
    assert "2 workgroups" in text and "290.0 us" in text and "245.0 us" in text and "45.0 us of idle" in text
    assert "1 LDS tile 280 us, 290" in text and "0 skinny 118 us, 200" in text
    assert tile_phases.end_summary(np.zeros((2, 2, 8), dtype=np.int64)) == "no tiles stamped"
