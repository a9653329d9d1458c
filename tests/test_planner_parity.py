"""Host logic behind the C ABI, checked without a GPU: the C++ planner's tile
table, operator order and ranges equal the reference planner's byte for byte;
argument validation returns error codes; the library exports every declared
symbol."""
import math
import os
import re
from types import SimpleNamespace as NS

import pytest

import paper_1901_10008_amd as sk
import workloads
from oracle import planner as P

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
ES = {"f32": 4, "bf16": 2, "f16": 2}


def fake_problems(specs, misalign=None):
    """sk_problem list with made-up, disjoint, 256-byte aligned device addresses (never dereferenced)."""
    out = []
    addr = 0x10000000
    for i, s in enumerate(specs):
        es = ES[s.dtype]
        if s.op == "gemm":
            na, nb, nc = s.M * s.K, s.N * s.K, s.M * s.N
        else:
            st = getattr(s, "stride", 1)
            ho = (s.H + 2 * s.pad_h - s.R) // st + 1
            wo = (s.W + 2 * s.pad_w - s.S) // st + 1
            na, nb, nc = s.Nb * s.H * s.W * s.Cin, s.Cout * s.R * s.S * s.Cin, s.Nb * ho * wo * s.Cout
        ptrs = []
        for cnt in (na, nb, nc):
            ptrs.append(addr)
            addr += (cnt * es + 255) // 256 * 256 + 256
        out.append(sk.make_problem(s, *ptrs))
    return out


def host_plan(specs, **prm):
    params = sk.sk_plan_params_default(host_only=1, **prm)
    return sk.sk_plan_create(fake_problems(specs), params)


def ref_params(**kw):
    return P.Params(**kw)


@pytest.mark.parametrize("idx", [1, 2, 3, 4, 5, 6, 7, 8])
@pytest.mark.parametrize("seed", [0, 1])
def test_plan_bytes_match_reference_on_configs(idx, seed):
    specs = workloads.config(idx, seed=seed)
    with host_plan(specs) as plan:
        table, order, first, count = P.plan(specs)
        assert sk.sk_plan_num_problems(plan) == len(specs)
        assert sk.sk_plan_num_tiles(plan) == len(table) // 32
        assert sk.sk_plan_get_tiles(plan) == table
        assert sk.sk_plan_get_order(plan) == order
        assert sk.sk_plan_get_ranges(plan) == (first, count)
        P.check_coverage(specs, sk.sk_plan_get_tiles(plan))


def _g(m, n, k, dtype="bf16", d=math.inf):
    return NS(op="gemm", dtype=dtype, M=m, N=n, K=k, deadline_ms=d)


def _c(h, w, cin, cout, r, s, ph, pw, dtype="bf16", nb=1, d=math.inf, st=1):
    return NS(op="conv", dtype=dtype, Nb=nb, H=h, W=w, Cin=cin, Cout=cout, R=r, S=s, pad_h=ph, pad_w=pw,
              stride=st, deadline_ms=d)


RAGGED = [_g(1, 5, 3, "f32"), _g(17, 33, 129), _g(33, 130, 70, "f16"), _g(65, 129, 8), _g(200, 300, 100, "f32"),
          _g(16, 9000, 64), _g(32, 40, 8192), _g(2, 8192, 8192, d=1.5), _g(7, 100, 2048, "f32", d=0.25),
          _c(5, 5, 3, 7, 3, 3, 1, 1), _c(9, 9, 8, 130, 1, 1, 0, 0, d=0.25), _c(13, 11, 16, 40, 3, 3, 1, 1, nb=2),
          _c(6, 6, 4, 4, 3, 1, 0, 0, "f32"), _c(4, 4, 8, 8, 1, 1, 1, 1),
          _c(56, 56, 64, 128, 1, 1, 0, 0, st=2), _c(15, 14, 8, 24, 3, 3, 1, 1, st=2), _c(9, 9, 8, 8, 3, 3, 0, 0, "f32", st=3)]


@pytest.mark.parametrize("prm", [
    {},
    {"edf": 0},
    {"skinny_max_m": 16},
    {"skinny_max_m": 32},
    {"skinny_max_m": 0},
    {"tile_bytes_min": 4096, "tile_bytes_max": 8192, "balance_div": 7},
    {"tile_bytes_min": 1 << 20, "tile_bytes_max": 1 << 22, "max_groups": 3},
])
def test_plan_bytes_match_reference_ragged_and_params(prm):
    with host_plan(RAGGED, **prm) as plan:
        table, order, first, count = P.plan(RAGGED, ref_params(**prm))
        assert sk.sk_plan_get_tiles(plan) == table
        assert sk.sk_plan_get_order(plan) == order
        assert sk.sk_plan_get_ranges(plan) == (first, count)
        P.check_coverage(RAGGED, table)


@pytest.mark.parametrize("seed", range(24))
def test_plan_bytes_match_reference_on_random_mixes(seed):
    """Seeded random operator lists (odd sizes, all element types, tied / missing / non-finite deadlines) under
    random plan parameters: the two planners must agree byte for byte, and the table must cover every output
    exactly once."""
    import numpy as np
    rng = np.random.default_rng(1000 + seed)
    dts = ["bf16", "f16", "f32"]
    deadlines = [math.inf, 0.0, -1.0, float("nan"), 0.5, 0.5, 1.25, 3.0]
    specs = []
    for _ in range(int(rng.integers(1, 24))):
        d = deadlines[int(rng.integers(0, len(deadlines)))]
        dt = dts[int(rng.integers(0, 3))]
        if rng.random() < 0.6:
            m = int(rng.choice([1, 2, 7, 16, 17, 31, 32, 33, 63, 64, 65, 100, 129, 300]))
            n = int(rng.choice([1, 5, 31, 32, 33, 127, 128, 129, 500, 1024, 4097]))
            k = int(rng.choice([1, 3, 8, 63, 64, 65, 256, 1000, 1024, 4096, 9000]))
            specs.append(_g(m, n, k, dt, d))
        else:
            h, w = int(rng.integers(1, 30)), int(rng.integers(1, 30))
            r, sq = int(rng.choice([1, 3, 5])), int(rng.choice([1, 3]))
            ph, pw = int(rng.integers(0, 3)), int(rng.integers(0, 2))
            if h + 2 * ph - r + 1 < 1 or w + 2 * pw - sq + 1 < 1:
                r, sq, ph, pw = 1, 1, 0, 0
            cin, cout = int(rng.choice([1, 3, 8, 64, 200, 512])), int(rng.choice([1, 7, 64, 130, 256]))
            specs.append(_c(h, w, cin, cout, r, sq, ph, pw, dt, nb=int(rng.integers(1, 3)), d=d,
                            st=int(rng.choice([1, 1, 2, 3]))))
            if seed % 3 == 2 and len(specs) % 2:   # the storage order of a convolution does not enter the table
                specs[-1].op = "conv_nchw"
    tmin = int(rng.choice([1024, 4096, 32768, 1 << 18]))
    prm = {"edf": int(rng.integers(0, 2)), "skinny_max_m": int(rng.choice([0, 8, 16, 32, 64])),
           "tile_bytes_min": tmin, "tile_bytes_max": tmin * int(rng.choice([1, 2, 16, 64])),
           "balance_div": int(rng.choice([1, 7, 64, 2048])), "max_groups": int(rng.choice([1, 3, 4, 64, 256])),
           "tail_div": int(rng.choice([0, 1, 16, 384, 5000]))}
    part = int(rng.choice([-1, 0, 1, 3, 32, 1000]))
    with host_plan(specs, xcd_part=part, **prm) as plan:
        table, order, first, count = P.plan(specs, ref_params(**prm))
        assert sk.sk_plan_get_tiles(plan) == table, prm
        assert sk.sk_plan_get_order(plan) == order
        assert sk.sk_plan_get_ranges(plan) == (first, count)
        P.check_coverage(specs, table)
        if part < 0:
            part = P.auto_die_part(specs, table, first)
        assert sk.sk_plan_get_xcd_lists(plan) == P.die_lists(specs, table, order, first, part), (prm, part)


def test_die_lists_by_default_only_for_compute_bound_plans_of_lds_tiles():
    """xcd_part = -1 (the default): lists for the sixteen 2048-cubed GEMMs (512 rectangles per part: two whole
    operators per die) and the 28x28x128 convolution tenants, none for the memory-bound conv2_2 tenants, for a
    plan with skinny operators, or for an empty plan; a single large GEMM is cut into eighths."""
    for idx, want in ((9, [512] * 8), (10, None), (8, [0] * 8), (5, [0] * 8), (3, [0] * 8)):
        specs = workloads.config(idx, seed=0)
        with host_plan(specs) as plan:
            table, order, first, count = P.plan(specs)
            got = sk.sk_plan_get_xcd_lists(plan)
            part = P.auto_die_part(specs, table, first)
            assert got == P.die_lists(specs, table, order, first, part)
            if want is not None:
                assert [len(l) for l in got] == want, idx
            else:
                assert part > 0 and sum(len(l) for l in got) == len(table) // 32
    one = [_g(4096, 4096, 4096)]
    with host_plan(one) as plan:
        assert [len(l) for l in sk.sk_plan_get_xcd_lists(plan)] == [128] * 8
    with host_plan([]) as plan:
        assert sk.sk_plan_get_xcd_lists(plan) == [[]] * 8
    # 2 * 2048^3 flops * 2 * 1573 against 3 * 2048^2 * 2 bytes * 983125: compute-bound; the same GEMM in fp32
    # (weight 25000, 4-byte elements) even more so; with 128 rows per operator the bytes win
    spec = [_g(2048, 2048, 2048)]
    table, order, first, count = P.plan(spec)
    assert P.auto_die_part(spec, table, first) == 32
    thin = [_g(128, 2048, 2048)]
    table, order, first, count = P.plan(thin)
    assert 2 * 128 * 2048 * 2048 * 2 * 1573 < (128 * 2048 * 2 + 2048 * 2048) * 2 * 983125 and P.auto_die_part(thin, table, first) == 0


@pytest.mark.parametrize("idx,rep,part", [(3, 16, 32), (5, 1, 32), (8, 2, 32), (9, 1, 32), (9, 1, 7), (4, 16, 1), (7, 3, 0)])
def test_die_lists_match_reference_on_configs(idx, rep, part):
    specs = [s for _ in range(rep) for s in workloads.config(idx, seed=0)]
    with host_plan(specs, xcd_part=part) as plan:
        table, order, first, count = P.plan(specs)
        got = sk.sk_plan_get_xcd_lists(plan)
        assert got == P.die_lists(specs, table, order, first, part)
        lds = [i for i, t in enumerate(P.decode(table)) if t["cls"] >= P.CLS_TILE_128x128]
        assert sorted(x for l in got for x in l) == (lds if part else [])


def test_permuting_operators_permutes_the_plan_consistently():
    import dataclasses
    specs = workloads.config(4, seed=3)
    perm = list(range(len(specs)))[::-1]
    strip = lambda t, idx: sorted((idx(x["problem"]), x["cls"], x["m0"], x["n0"], x["m_len"], x["n_len"],
                                   x["k0"], x["k_len"]) for x in t)
    # An operator's tiles depend on its place in the execution order only through the tail rule.
    # Without that rule any permutation of the submission order permutes the plan ...
    with host_plan(specs, tail_div=0) as a, host_plan([specs[i] for i in perm], tail_div=0) as b:
        ta, tb = P.decode(sk.sk_plan_get_tiles(a)), P.decode(sk.sk_plan_get_tiles(b))
        assert strip(ta, lambda i: i) == strip(tb, lambda i: perm[i])
    # ... and with it, so does one that leaves the execution order alone (all deadlines distinct).
    dl = [dataclasses.replace(s, deadline_ms=1.0 + 0.37 * ((7 * i) % len(specs))) for i, s in enumerate(specs)]
    with host_plan(dl) as a, host_plan([dl[i] for i in perm]) as b:
        ta, tb = P.decode(sk.sk_plan_get_tiles(a)), P.decode(sk.sk_plan_get_tiles(b))
        assert strip(ta, lambda i: i) == strip(tb, lambda i: perm[i])
        assert [perm[i] for i in sk.sk_plan_get_order(b)] == sk.sk_plan_get_order(a)


def test_channel_major_convolution_plans_like_the_nhwc_form():
    """Same canonical GEMM, same tiles, whatever the storage order; the dense output range is checked for
    overlap in the same way."""
    convs = [_c(14, 14, 256, 256, 3, 3, 1, 1), _c(56, 56, 64, 64, 3, 3, 1, 1, st=2, nb=2), _c(7, 9, 3, 5, 5, 3, 2, 1, "f32")]
    nchw = [NS(**{**vars(s), "op": "conv_nchw"}) for s in convs]
    with host_plan(convs) as a, host_plan(nchw) as b:
        assert sk.sk_plan_get_tiles(a) == sk.sk_plan_get_tiles(b) == P.plan(nchw)[0]
        P.check_coverage(nchw, sk.sk_plan_get_tiles(b))
    bad = fake_problems(nchw[:2])
    bad[1].C = bad[0].C + 2 * (14 * 14 * 256 - 1)     # last element of the first output
    _expect(-3, bad)
    bad[1].C = bad[0].C + 2 * (14 * 14 * 256)         # right behind it
    sk.sk_plan_create(bad, sk.sk_plan_params_default(host_only=1)).close()


def test_empty_plan():
    with sk.sk_plan_create([], sk.sk_plan_params_default(host_only=1)) as plan:
        assert sk.sk_plan_num_tiles(plan) == 0 and sk.sk_plan_num_problems(plan) == 0
        assert sk.sk_plan_get_tiles(plan) == b"" and sk.sk_plan_get_order(plan) == []
        assert sk.sk_plan_grid(plan) == 0


def _expect(status, problems, **prm):
    with pytest.raises(sk.SkError) as e:
        sk.sk_plan_create(problems, sk.sk_plan_params_default(host_only=1, **prm))
    assert e.value.status == status, e.value
    assert e.value.detail


def test_validation_errors():
    ok = fake_problems([_g(4, 64, 64), _g(4, 64, 64)])
    # dimension < 1
    bad = fake_problems([_g(4, 64, 64)])
    bad[0].M = 0
    _expect(-1, bad)
    # null pointer
    bad = fake_problems([_g(4, 64, 64)])
    bad[0].B = None
    _expect(-1, bad)
    # stride shorter than a row
    bad = fake_problems([_g(4, 64, 64)])
    bad[0].lda = 32
    _expect(-1, bad)
    # unknown dtype / op
    bad = fake_problems([_g(4, 64, 64)])
    bad[0].dtype = 9
    _expect(-2, bad)
    bad = fake_problems([_g(4, 64, 64)])
    bad[0].op = 5
    _expect(-2, bad)
    # filter larger than the image
    _expect(-1, fake_problems([_c(2, 2, 4, 4, 3, 3, 0, 0)]))
    # negative stride; stride 0 means 1
    bad = fake_problems([_c(8, 8, 8, 8, 3, 3, 1, 1)])
    bad[0].stride = -2
    _expect(-1, bad)
    zero = fake_problems([_c(8, 8, 8, 8, 3, 3, 1, 1)])
    zero[0].stride = 0
    with sk.sk_plan_create(zero, sk.sk_plan_params_default(host_only=1)) as plan:
        assert sk.sk_plan_get_tiles(plan) == P.plan([_c(8, 8, 8, 8, 3, 3, 1, 1)])[0]
    # overlapping outputs (same C) -> overlap; sharing A and B is fine
    bad = fake_problems([_g(4, 64, 64), _g(4, 64, 64)])
    bad[1].C = bad[0].C + 64
    _expect(-3, bad)
    shared = fake_problems([_g(4, 64, 64), _g(4, 64, 64)])
    shared[1].A, shared[1].B = shared[0].A, shared[0].B
    sk.sk_plan_create(shared, sk.sk_plan_params_default(host_only=1)).close()
    # adjacent but disjoint outputs are fine; strided outputs interleaving in address but overlapping in range are not
    adj = fake_problems([_g(4, 64, 64), _g(4, 64, 64)])
    adj[1].C = adj[0].C + 4 * 64 * 2
    sk.sk_plan_create(adj, sk.sk_plan_params_default(host_only=1)).close()
    # parameter out of range
    _expect(-1, ok, skinny_max_m=65)
    _expect(-1, ok, balance_div=0)
    # launching a host-only plan is a state error
    with sk.sk_plan_create(ok, sk.sk_plan_params_default(host_only=1)) as plan:
        with pytest.raises(sk.SkError) as e:
            sk.sk_launch(plan)
        assert e.value.status == sk.SK_ERR_STATE
        with pytest.raises(sk.SkError) as e:
            sk.sk_plan_get_stamps(plan)
        assert e.value.status == sk.SK_ERR_STATE


def test_library_exports_every_declared_symbol():
    with open(os.path.join(ROOT, "include", "superkernel.h")) as f:
        text = f.read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    declared = set(re.findall(r"\b(sk_[a-z_]+)\s*\(", text))
    assert declared == set(sk.EXPORTED_SYMBOLS)
    L = sk.lib()
    for name in declared:
        assert getattr(L, name) is not None
    assert sk.sk_strerror(0) == "success" and "overlap" in sk.sk_strerror(-3)
    assert (sk.SK_ERR_BUSY, sk.SK_ERR_STATE) == (-6, -7)
    assert "another stream" in sk.sk_strerror(sk.SK_ERR_BUSY) and "state" in sk.sk_strerror(sk.SK_ERR_STATE)


def test_struct_layout_matches_header():
    import ctypes
    from paper_1901_10008_amd import binding
    assert ctypes.sizeof(binding.sk_problem) == 120
    assert ctypes.sizeof(binding.PlanParams) == 56
