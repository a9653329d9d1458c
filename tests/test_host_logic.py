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
    assert lib.sk_ceiling_stream_read and lib.sk_ceiling_mfma_bf16
