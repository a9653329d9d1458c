"""Pins for the reference tile planner and its coverage checker (CPU only)."""
import math
import struct
from types import SimpleNamespace as NS

import pytest

import workloads
from oracle import planner as P


def gemm(m, n, k, dtype="bf16", deadline=math.inf):
    return NS(op="gemm", dtype=dtype, M=m, N=n, K=k, deadline_ms=deadline)


def conv(hw, cin, cout, r, dtype="bf16", deadline=math.inf):
    return NS(op="conv", dtype=dtype, Nb=1, H=hw, W=hw, Cin=cin, Cout=cout, R=r, S=r,
              pad_h=(r - 1) // 2, pad_w=(r - 1) // 2, deadline_ms=deadline)


def test_canonical_view_of_conv_and_gemm():
    assert P.canonical(gemm(3, 5, 7)) == (3, 5, 7)
    assert P.canonical(conv(56, 64, 256, 1)) == (3136, 256, 64)
    assert P.canonical(conv(7, 512, 512, 3)) == (49, 512, 4608)
    c = NS(op="conv", dtype="bf16", Nb=2, H=8, W=6, Cin=4, Cout=3, R=3, S=3, pad_h=0, pad_w=1, deadline_ms=0)
    assert P.canonical(c) == (2 * 6 * 6, 3, 36)
    # stride: the residual networks' down-sampling layers (56x56 -> 28x28), and extents that do not divide
    c = NS(op="conv", dtype="bf16", Nb=1, H=56, W=56, Cin=64, Cout=128, R=3, S=3, pad_h=1, pad_w=1, stride=2,
           deadline_ms=0)
    assert P.canonical(c) == (28 * 28, 128, 576)
    c = NS(op="conv", dtype="bf16", Nb=1, H=56, W=56, Cin=256, Cout=512, R=1, S=1, pad_h=0, pad_w=0, stride=2,
           deadline_ms=0)
    assert P.canonical(c) == (28 * 28, 512, 256)
    c = NS(op="conv", dtype="bf16", Nb=3, H=7, W=10, Cin=2, Cout=5, R=3, S=3, pad_h=0, pad_w=0, stride=3,
           deadline_ms=0)
    assert P.canonical(c) == (3 * 2 * 3, 5, 18)   # rows 0,3 and columns 0,3,6 fit


def test_hand_enumerated_skinny_plan():
    # M=1, N=70, K=3, fp32: one 32-row weight group is 32*3*4 = 384 B, far below the 32 KiB
    # floor => wk=1, G = 4*(32768 // (4*384)) = 84 groups, capped by nothing: BN = 2688 >= N.
    # One tile covering all 70 columns.
    table, order, first, count = P.plan([gemm(1, 70, 3, "f32")])
    t = P.decode(table)
    assert len(t) == 1 and order == [0] and first == [0] and count == [1]
    assert t[0] == dict(problem=0, cls=0, ks_idx=0, S=1, m0=0, n0=0, m_len=1, n_len=70, k0=0, k_len=3,
                        out_tile_id=0)
    # bytes, field by field, little endian
    assert table == struct.pack("<IHBBIIHHIII", 0, 0, 0, 1, 0, 0, 1, 70, 0, 3, 0)


def test_hand_enumerated_reduction_slices():
    prm = P.Params(tile_bytes_min=32768, tile_bytes_max=32768)   # T fixed at 32 KiB
    # K=1024 bf16: one 32-row group is 64 KiB, four groups (256 KiB) exceed T => 128-row tiles whose
    # reduction is cut into whole 512-element chunks: 2 chunks, wanted 8 slices, so 2 slices of 512
    t = P.decode(P.plan([gemm(4, 100, 1024)], prm)[0])
    assert [(x["cls"], x["n0"], x["n_len"], x["ks_idx"], x["S"], x["k0"], x["k_len"], x["out_tile_id"]) for x in t] == \
        [(0, 0, 100, 0, 2, 0, 512, 0), (0, 0, 100, 1, 2, 512, 512, 0)]
    # K=2304 bf16, Mg=20 (two row blocks, chunk = 256 elements): 9 chunks, four groups = 576 KiB -> wanted 18,
    # capped at 9 slices of one chunk; two column blocks
    t = P.decode(P.plan([gemm(20, 200, 2304)], prm)[0])
    assert len(t) == 18 and {x["cls"] for x in t} == {3}
    assert [(x["n0"], x["n_len"]) for x in t[::9]] == [(0, 128), (128, 72)]
    assert [(x["ks_idx"], x["k0"], x["k_len"]) for x in t[:9]] == [(i, 256 * i, 256) for i in range(9)]
    assert [x["out_tile_id"] for x in t] == [0] * 9 + [1] * 9
    # K=1280 bf16, Mg=8: chunks of 512 -> 3 chunks (512, 512, 256); four groups = 320 KiB -> wanted 10 -> 3 slices
    t = P.decode(P.plan([gemm(8, 64, 1280)], prm)[0])
    assert [(x["ks_idx"], x["S"], x["k0"], x["k_len"]) for x in t] == [(0, 3, 0, 512), (1, 3, 512, 512), (2, 3, 1024, 256)]
    # K=256 bf16, Mg=20: one chunk only => no split even though four groups exceed T
    t = P.decode(P.plan([gemm(20, 100, 256)], prm)[0])
    assert [(x["cls"], x["n0"], x["n_len"], x["m_len"], x["S"], x["k_len"]) for x in t] == [(3, 0, 100, 20, 1, 256)]
    # K=64 bf16: group = 4 KiB, four groups fit twice into T => 8 groups = 256 rows per tile, no split
    t = P.decode(P.plan([gemm(16, 600, 64)], prm)[0])
    assert [x["cls"] for x in t] == [0, 0, 0] and all(x["S"] == 1 for x in t)
    assert [(x["n0"], x["n_len"]) for x in t] == [(0, 256), (256, 256), (512, 88)]
    # slices of unequal count: 5 chunks wanted in 2 slices -> 3 + 2 chunks
    prm2 = P.Params(tile_bytes_min=3 * 65536, tile_bytes_max=3 * 65536)
    t = P.decode(P.plan([gemm(4, 32, 2560)], prm2)[0])   # four groups = 640 KiB, T = 192 KiB -> wanted 4 -> per 2 -> 3 slices
    assert [(x["k0"], x["k_len"]) for x in t] == [(0, 1024), (1024, 1024), (2048, 512)]


def test_hand_enumerated_tail_rule():
    # three operators of 2 MiB of weights each; T_all = 6 MiB / 16 = 384 KiB.  With tail_div = 16 the operator
    # at position 0 may use min(384, 6 MiB/16 = 384) KiB, the next min(384, 4 MiB/16 = 256) KiB and the last
    # min(384, 2 MiB/16 = 128) KiB.  One 32-row group is 64 KiB, four groups 256 KiB: the first two operators
    # get 128-row tiles over the whole reduction, the last one has to cut its reduction in two
    # (two chunks of 512 elements, wanted ceil(256/128) = 2 slices).
    prm = P.Params(tile_bytes_min=4096, tile_bytes_max=1 << 20, balance_div=16, tail_div=16)
    ops = [gemm(1, 1024, 1024) for _ in range(3)]
    table, order, first, count = P.plan(ops, prm)
    assert order == [0, 1, 2] and count == [8, 8, 16] and first == [0, 8, 16]
    t = P.decode(table)
    assert all(x["S"] == 1 and x["k_len"] == 1024 and x["n_len"] == 128 for x in t[:16])
    assert [(x["n0"], x["ks_idx"], x["S"], x["k0"], x["k_len"]) for x in t[16:20]] == \
        [(0, 0, 2, 0, 512), (0, 1, 2, 512, 512), (128, 0, 2, 0, 512), (128, 1, 2, 512, 512)]
    # the rule follows the execution order, not the submission order: with deadlines 3, 2, 1 ms the operator
    # submitted first runs last and is the one that is cut
    rev = [gemm(1, 1024, 1024, deadline=3.0 - i) for i in range(3)]
    table, order, first, count = P.plan(rev, prm)
    assert order == [2, 1, 0] and count == [16, 8, 8] and first == [16, 8, 0]
    # tail_div = 0 switches the rule off
    table, order, first, count = P.plan(ops, P.Params(tile_bytes_min=4096, tile_bytes_max=1 << 20, balance_div=16, tail_div=0))
    assert count == [8, 8, 8]
    # never below eight times the lower clamp: T_all = 1 MiB, the tail would ask for ~0, the floor is 8 * 64 KiB
    prm3 = P.Params(tile_bytes_min=1 << 16, tile_bytes_max=1 << 20, balance_div=1, tail_div=1 << 20)
    assert P.plan(ops, prm3)[3] == [4, 4, 4]   # T = 512 KiB everywhere: G = 4 * (512 // 256) = 8 groups = 256 rows
    # a table whose own target is below that floor does not shrink at all: T_all = 256 KiB -> 128-row tiles
    prm4 = P.Params(tile_bytes_min=1 << 16, tile_bytes_max=1 << 18, balance_div=1, tail_div=1 << 20)
    assert P.plan(ops, prm4)[3] == [8, 8, 8]
    # with the defaults the floor is 256 KiB: the last operators of a large table are tiled for 256 KiB, not 32
    many = [gemm(1, 2048, 4096) for _ in range(64)]   # 16 MiB each, 1 GiB in all: T_all = 2 MiB
    t = P.decode(P.plan(many)[0])
    last = [x for x in t if x["problem"] == 63]
    # group = 32 * 4096 * 2 = 256 KiB; four groups exceed 256 KiB: reduction in 1 MiB / 256 KiB = 4 slices of 1024
    assert len(last) == (2048 // 128) * 4 and {(x["n_len"], x["S"], x["k_len"]) for x in last} == {(128, 4, 1024)}


def test_hand_enumerated_four_row_block_class():
    prm = P.Params(tile_bytes_min=32768, tile_bytes_max=32768)
    # Mg = 49 (7x7 image) => four row blocks (cls 6), chunk = 128 elements.
    # Kg = 9*64 = 576 bf16: group = 36 KiB; four groups = 144 KiB -> wanted 5 slices; 5 chunks -> 5 slices
    t = P.decode(P.plan([conv(7, 64, 256, 3)], prm)[0])
    assert len(t) == 10 and {x["cls"] for x in t} == {6}
    assert [(x["n0"], x["n_len"], x["ks_idx"], x["k0"], x["k_len"]) for x in t[:5]] == \
        [(0, 128, 0, 0, 128), (0, 128, 1, 128, 128), (0, 128, 2, 256, 128), (0, 128, 3, 384, 128), (0, 128, 4, 512, 64)]
    assert [x["n0"] for x in t[5:]] == [128] * 5
    # Kg = 64: group = 4 KiB => 8 groups, no split
    t = P.decode(P.plan([conv(7, 64, 300, 1)], prm)[0])
    assert [(x["cls"], x["n0"], x["n_len"], x["S"]) for x in t] == [(6, 0, 256, 1), (6, 256, 44, 1)]
    # M = 64 is the last skinny size, 65 goes to LDS tiles
    assert P.decode(P.plan([gemm(64, 32, 64)], prm)[0])[0]["cls"] == 6
    assert P.decode(P.plan([gemm(65, 32, 64)], prm)[0])[0]["cls"] == 10      # at most 64 columns: the narrow tile
    assert P.decode(P.plan([gemm(64, 32, 64)], P.Params(skinny_max_m=32))[0])[0]["cls"] == 10
    assert P.decode(P.plan([gemm(65, 65, 64)], prm)[0])[0]["cls"] == 9


def test_hand_enumerated_lds_tiles():
    # Mg = 196 -> 128x128 tiles, rows outer, columns inner (target of 1 MiB: reduction not cut)
    whole = P.Params(tile_bytes_min=1 << 20, tile_bytes_max=1 << 20)
    t = P.decode(P.plan([conv(14, 64, 192 + 8, 3)], whole)[0])
    assert [(x["cls"], x["m0"], x["n0"], x["m_len"], x["n_len"], x["k_len"]) for x in t] == \
        [(9, 0, 0, 128, 128, 576), (9, 0, 128, 128, 72, 576),
         (9, 128, 0, 68, 128, 576), (9, 128, 128, 68, 72, 576)]
    assert [x["out_tile_id"] for x in t] == list(range(4))
    assert all(x["S"] == 1 and x["k0"] == 0 for x in t)
    # a short reduction is never cut, however small the target (a slice hands over 64 KB of partial sums
    # and is at least 1024 elements long): Kg = 576
    prm = P.Params(tile_bytes_min=32 << 10, tile_bytes_max=32 << 10)
    assert all(x["S"] == 1 for x in P.decode(P.plan([conv(14, 64, 192 + 8, 3)], prm)[0]))
    # Kg = 2304 (3x3x256): operands 1152 KiB, target 32 KiB: 9 chunks of 256, wanted min(9, 36, 2304 // 1024 = 2)
    # = 2 slices: five and four chunks
    t = P.decode(P.plan([conv(14, 256, 128, 3)], prm)[0])
    assert [(x["m0"], x["ks_idx"], x["S"], x["k0"], x["k_len"], x["out_tile_id"]) for x in t] == \
        [(0, 0, 2, 0, 1280, 0), (0, 1, 2, 1280, 1024, 0), (128, 0, 2, 0, 1280, 1), (128, 1, 2, 1280, 1024, 1)]
    # not cut while the operands stay within twice the target: 1152 KiB <= 2 * 576 KiB
    prm = P.Params(tile_bytes_min=576 << 10, tile_bytes_max=576 << 10)
    assert all(x["S"] == 1 for x in P.decode(P.plan([conv(14, 256, 128, 3)], prm)[0]))
    # Kg = 4608 (3x3x512), target 1 MiB: operands 2304 KiB > 2 MiB; 18 chunks, wanted ceil(2304/1024) = 3,
    # six chunks per slice
    t = P.decode(P.plan([conv(14, 512, 128, 3)], whole)[0])
    assert [(x["m0"], x["ks_idx"], x["S"], x["k0"], x["k_len"]) for x in t] == \
        [(0, 0, 3, 0, 1536), (0, 1, 3, 1536, 1536), (0, 2, 3, 3072, 1536),
         (128, 0, 3, 0, 1536), (128, 1, 3, 1536, 1536), (128, 2, 3, 3072, 1536)]


def test_hand_enumerated_narrow_lds_tiles():
    # at most 64 output columns: 128 x 64 tiles (cls 10).  Mg = 196, Ng = 64, Kg = 576: two row blocks
    whole = P.Params(tile_bytes_min=1 << 20, tile_bytes_max=1 << 20)
    t = P.decode(P.plan([conv(14, 64, 64, 3)], whole)[0])
    assert [(x["cls"], x["m0"], x["n0"], x["m_len"], x["n_len"], x["k_len"], x["S"]) for x in t] == \
        [(10, 0, 0, 128, 64, 576, 1), (10, 128, 0, 68, 64, 576, 1)]
    # 40 columns: one ragged column block; 65 columns: back to 128-wide tiles, the second one ragged
    t = P.decode(P.plan([gemm(130, 40, 64)], whole)[0])
    assert [(x["cls"], x["m0"], x["n_len"]) for x in t] == [(10, 0, 40), (10, 128, 40)]
    t = P.decode(P.plan([gemm(130, 65, 64)], whole)[0])
    assert [(x["cls"], x["m0"], x["n0"], x["n_len"]) for x in t] == [(9, 0, 0, 65), (9, 128, 0, 65)]
    # the reduction of a narrow tile is cut by the bytes of ITS operands: (128 + 64) * 4608 * 2 = 1728 KiB is
    # within twice the 1 MiB target, where the 128-wide tile's 2304 KiB are not
    assert all(x["S"] == 1 for x in P.decode(P.plan([conv(14, 512, 64, 3)], whole)[0]))
    assert all(x["S"] == 3 for x in P.decode(P.plan([conv(14, 512, 128, 3)], whole)[0]))
    # ... and is cut below that: target 512 KiB, 18 chunks, wanted min(18, ceil(1728/512) = 4, 4608 // 1024 = 4) = 4,
    # five chunks per slice -> slices of 1280, 1280, 1280, 768
    half = P.Params(tile_bytes_min=512 << 10, tile_bytes_max=512 << 10)
    t = P.decode(P.plan([conv(14, 512, 64, 3)], half)[0])
    assert [(x["ks_idx"], x["S"], x["k0"], x["k_len"]) for x in t[:4]] == \
        [(0, 4, 0, 1280), (1, 4, 1280, 1280), (2, 4, 2560, 1280), (3, 4, 3840, 768)]
    P.check_coverage([conv(14, 512, 64, 3)], P.plan([conv(14, 512, 64, 3)], half)[0])


def test_edf_order_is_stable_sort_by_deadline_then_index():
    ds = [3.0, math.inf, 1.0, 3.0, 0.0, -2.0, 1.0, float("nan"), 0.75]
    probs = [gemm(1, 32, 64, deadline=d) for d in ds]
    want = [8, 2, 6, 0, 3, 1, 4, 5, 7]      # by hand: 0.75, 1.0(2), 1.0(6), 3.0(0), 3.0(3), then no-deadline by index
    assert P.order(probs, 1) == want
    assert P.order(probs, 0) == list(range(len(ds)))
    table, order, first, count = P.plan(probs)
    assert order == want
    assert [x["problem"] for x in P.decode(table)] == want
    assert [first[i] for i in want] == list(range(len(ds)))
    # no deadlines at all => submission order
    probs = [gemm(1, 32, 64) for _ in range(5)]
    assert P.order(probs, 1) == [0, 1, 2, 3, 4]


def test_target_bytes_rule():
    prm = P.Params()
    small = [gemm(1, 256, 256, "f32")]
    assert P.target_tile_bytes(small, prm) == prm.tile_bytes_min
    assert prm.balance_div == 512
    big = [gemm(1, 8192, 8192)] * 2      # 2 x 128 MiB of weights / 512 = 512 KiB
    assert P.target_tile_bytes(big, prm) == 512 * 1024
    huge = [gemm(1, 8192, 8192)] * 16    # 2 GiB / 512 = 4 MiB -> clamped to 2 MiB
    assert P.target_tile_bytes(huge, prm) == prm.tile_bytes_max == 2048 * 1024
    mid = [gemm(1, 4096, 4096)]          # 32 MiB / 512 = 64 KiB
    assert P.target_tile_bytes(mid, prm) == 65536
    assert P.target_tile_bytes(mid * 4, P.Params(balance_div=2048)) == 65536


@pytest.mark.parametrize("idx", [1, 2, 3, 4, 5, 6, 7, 8])
def test_coverage_on_every_config(idx):
    probs = workloads.config(idx, seed=0)
    table, order, first, count = P.plan(probs)
    assert len(table) == 32 * sum(count)
    P.check_coverage(probs, table)
    tiles = P.decode(table)
    # tiles of one operator are contiguous and in EDF order
    seen = []
    for t in tiles:
        if not seen or seen[-1] != t["problem"]:
            seen.append(t["problem"])
    assert seen == order == sorted(range(len(probs)), key=lambda i: (probs[i].deadline_ms, i))
    for i in range(len(probs)):
        assert all(t["problem"] == i for t in tiles[first[i]:first[i] + count[i]])


def test_coverage_on_ragged_shapes():
    probs = [gemm(1, 5, 3, "f32"), gemm(17, 33, 129), gemm(33, 130, 70, "f16"), gemm(65, 129, 8),
             gemm(200, 300, 100, "f32"), conv(5, 3, 7, 3), conv(9, 8, 130, 1), conv(13, 16, 40, 3)]
    table = P.plan(probs)[0]
    P.check_coverage(probs, table)


def _mutate(table, idx, **kw):
    tiles = P.decode(table)
    tiles[idx].update(kw)
    names = ("problem", "cls", "ks_idx", "S", "m0", "n0", "m_len", "n_len", "k0", "k_len", "out_tile_id")
    return b"".join(P.RECORD.pack(*[t[n] for n in names]) for t in tiles)


def test_coverage_checker_catches_planted_mistakes():
    probs = [gemm(100, 300, 128), gemm(4, 256, 4096)]
    table = P.plan(probs)[0]
    P.check_coverage(probs, table)
    n = len(table) // 32
    assert n >= 4 and P.decode(table)[1]["n0"] == 128
    with pytest.raises(AssertionError):
        P.check_coverage(probs, table[:-32])                       # a tile dropped
    with pytest.raises(AssertionError):
        P.check_coverage(probs, table + table[-32:])               # a tile doubled (same id)
    with pytest.raises(AssertionError):
        P.check_coverage(probs, _mutate(table, 1, n0=64))          # overlapping rectangle
    with pytest.raises(AssertionError):
        P.check_coverage(probs, _mutate(table, 0, k_len=64))       # reduction cut short
    with pytest.raises(AssertionError):
        P.check_coverage(probs, _mutate(table, 0, n_len=129))      # rectangle too wide
    with pytest.raises(AssertionError):
        P.check_coverage(probs, _mutate(table, 2, out_tile_id=0))  # id collision


def test_targets_count_the_bytes_the_tiles_load():
    # Hand-worked.  Defaults: balance_div 512, clamps 32 KiB .. 2 MiB, tail_div 384, floor of the tail rule 256 KiB.
    prm = P.Params()
    # a skinny operator loads its weights once; an LDS-tile operator loads 128 + BN operand rows per output tile
    assert P.stream_bytes(gemm(8, 4096, 1024), prm) == 4096 * 1024 * 2
    assert P.stream_bytes(gemm(2048, 2048, 2048), prm) == 16 * 16 * 256 * 2048 * 2          # 256 MiB, weights: 8 MiB
    assert P.stream_bytes(gemm(65, 64, 1024), prm) == 1 * 1 * 192 * 1024 * 2                # one 128x64 tile
    assert P.stream_bytes(conv(56, 64, 64, 3), prm) == 25 * 1 * 192 * 576 * 2               # 3136 rows: 25 row blocks
    assert P.stream_bytes(gemm(200, 300, 512, "f32"), prm) == 2 * 3 * 256 * 512 * 4
    # Two 2048-cubed GEMMs.  A tile's operands over the whole reduction are 256 * 2048 * 2 = 1 MiB.
    # Whole-table target: 2 * 256 MiB / 512 = 1 MiB; tail rule: first operator 512 MiB / 384 > 1 MiB, second
    # 256 MiB / 384 = 699050 B, so 1 MiB <= 2 T for both: no reduction slices, 2 * 256 tiles.
    # (Measured in weight bytes the target would be the 32 KiB floor resp. 256 KiB under the tail rule, and every
    # tile would be cut in two.)
    t = P.decode(P.plan([gemm(2048, 2048, 2048), gemm(2048, 2048, 2048)], prm)[0])
    assert len(t) == 512 and all(x["S"] == 1 and x["k_len"] == 2048 and x["cls"] == 9 for x in t)
    # One 256 x 256 x 4096 GEMM alone: 4 tiles of 256 * 4096 * 2 = 2 MiB each; stream bytes 8 MiB -> 16 KiB, clamped
    # to 32 KiB; tail rule: max(256 KiB, 8 MiB / 384) = 256 KiB, capped by the 32 KiB table target.  2 MiB > 64 KiB:
    # wanted min(16 chunks, 64, 255, 4096 / 1024) = 4 slices of 1024.
    t = P.decode(P.plan([gemm(256, 256, 4096)], prm)[0])
    assert len(t) == 16 and [(x["ks_idx"], x["S"], x["k0"], x["k_len"]) for x in t[:4]] == \
        [(0, 4, 0, 1024), (1, 4, 1024, 1024), (2, 4, 2048, 1024), (3, 4, 3072, 1024)]
    # A skinny operator behind a large LDS-tile operator: the table target is the upper clamp (2 MiB) because of the
    # large one, and the skinny operator, last in order, falls under the tail rule with its own weights only:
    # 4096 * 4096 * 2 = 32 MiB / 384 = 87381 -> floor 256 KiB; one group is 32 * 4096 * 2 = 256 KiB, four exceed it:
    # 4 groups per tile, reduction cut: chunk 512, 8 chunks, wanted min(8, 4, 255) = 4 slices of 1024.
    t = P.decode(P.plan([gemm(4096, 4096, 4096, deadline=1.0), gemm(4, 4096, 4096, deadline=2.0)], prm)[0])
    sk = [x for x in t if x["problem"] == 1]
    assert len(sk) == 32 * 4 and {(x["n_len"], x["S"], x["k_len"]) for x in sk} == {(128, 4, 1024)}
    assert all(x["S"] == 1 for x in t if x["problem"] == 0)   # 256 * 4096 * 2 = 2 MiB <= 2 * 2 MiB


def test_die_lists_hand_worked():
    """Which die takes which LDS tile, on cases small enough to enumerate by hand."""
    # 300 x 520 GEMM: MB = 3 row blocks, NB = 5 column blocks of 128 (the last 8 wide), 15 rectangles, one slice
    # each: table index = 5 * row block + column block.
    big = NS(op="gemm", dtype="bf16", M=300, N=520, K=256, deadline_ms=math.inf)
    small = NS(op="gemm", dtype="bf16", M=8, N=64, K=256, deadline_ms=math.inf)       # skinny: in no list
    ops = [small, big]
    table, order, first, count = P.plan(ops, P.Params(tile_bytes_min=1 << 20, tile_bytes_max=1 << 20))
    assert first[1] == count[0] and count[1] == 15
    f = first[1]
    # part = 16: one part, one die (die 0: all lists are empty); Z-order inside the 8 x 8 block: (0,0) (0,1) (1,0)
    # (1,1) (0,2) (0,3) (1,2) (1,3) (2,0) (2,1) then row 3 does not exist, (2,2) (2,3), then columns 4..7 of
    # rows 0..3: (0,4) (1,4) (2,4)
    lists = P.die_lists(ops, table, order, first, 16)
    rc = lambda r, c: f + 5 * r + c
    assert lists[0] == [rc(0, 0), rc(0, 1), rc(1, 0), rc(1, 1), rc(0, 2), rc(0, 3), rc(1, 2), rc(1, 3),
                        rc(2, 0), rc(2, 1), rc(2, 2), rc(2, 3), rc(0, 4), rc(1, 4), rc(2, 4)]
    assert lists[1:] == [[]] * 7
    # part = 8: 15 > 8 -> two parts.  Grids: 2 x 1 (pm = 2, pn = 1) fetches 1 * 3 * 128 + 2 * 5 * 128 = 1664 rows,
    # 1 x 2 fetches 2 * 3 * 128 + 1 * 5 * 128 = 1408: the columns are cut, [0, 2) and [2, 5); dies 0 and 1.
    lists = P.die_lists(ops, table, order, first, 8)
    assert lists[0] == [rc(0, 0), rc(0, 1), rc(1, 0), rc(1, 1), rc(2, 0), rc(2, 1)]
    assert lists[1] == [rc(0, 2), rc(0, 3), rc(1, 2), rc(1, 3), rc(0, 4), rc(1, 4), rc(2, 2), rc(2, 3), rc(2, 4)]
    assert lists[2:] == [[]] * 6
    # part = 1: eight parts at most.  Grids with pm <= 3, pn <= 5: only 2 x 4 (rows cut in [0,1) [1,3), columns in
    # [0,1) [1,2) [2,3) [3,5)); parts row-major onto dies 0..7
    lists = P.die_lists(ops, table, order, first, 1)
    assert lists == [[rc(0, 0)], [rc(0, 1)], [rc(0, 2)], [rc(0, 3), rc(0, 4)],
                     [rc(1, 0), rc(2, 0)], [rc(1, 1), rc(2, 1)], [rc(1, 2), rc(2, 2)], [rc(1, 3), rc(1, 4), rc(2, 3), rc(2, 4)]]
    # a second operator goes to the dies with the shortest lists: after part = 8 above, dies 2 and 3
    two = [big, big]
    table, order, first, count = P.plan(two, P.Params(tile_bytes_min=1 << 20, tile_bytes_max=1 << 20))
    lists = P.die_lists(two, table, order, first, 8)
    assert [len(l) for l in lists] == [6, 9, 6, 9, 0, 0, 0, 0]
    assert lists[2][0] == first[1] and lists[3][0] == first[1] + 2
    # reduction slices of a rectangle stay together; part = 0 switches the lists off
    deep = NS(op="gemm", dtype="bf16", M=128, N=256, K=8192, deadline_ms=math.inf)
    table, order, first, count = P.plan([deep], P.Params(tile_bytes_min=4096, tile_bytes_max=4096, balance_div=1))
    S = P.decode(table)[0]["S"]
    assert S > 1 and count[0] == 2 * S
    assert P.die_lists([deep], table, order, first, 32)[0] == list(range(2 * S))
    assert P.die_lists([deep], table, order, first, 0) == [[]] * 8
