"""Reference tile planner and coverage checker -- TEST INFRASTRUCTURE ONLY.

The paper's runtime packs many small kernels into one large launch (Section
5.3) and serves the streams with the least latency slack first (Section 5,
item (a)); it gives no packing algorithm, table layout or policy.
This module fixes this build's reading as a pure integer function of the
operator list and a few parameters, in plain Python, so that the C++ planner
behind the C ABI can be compared with it byte for byte:

  1. canonical GEMM view of every operator (a convolution is the GEMM that
     backs it: rows = output pixels, columns = output channels, reduction =
     filter taps x input channels);
  2. tile class and tile extents per operator;
  3. operator order: earliest deadline first, ties (and "no deadline") by
     submission index;
  4. the flat table: operators in that order, row blocks outer, column blocks
     inner, reduction slices innermost; one fixed-size record per tile;
  5. optionally (Section 1, item (c): the shape of the execution blocks is the
     runtime's choice) which of the GPU's eight dies runs which LDS tile
     (`die_lists`): tiles that share operand rows meet behind one L2.

It shares no code with the product's planner.

Pins (tests/test_oracle_planner.py): tiny cases enumerated by hand, brute-force
coverage (every output element owned by exactly one rectangle, reduction slices
partition [0,Kg)), table length == sum of tile counts, order == Python's sorted.
"""
from __future__ import annotations

import math
import struct
from dataclasses import dataclass
from typing import List, Sequence

import numpy as np

ELEM_SIZE = {"f32": 4, "bf16": 2, "f16": 2}

RECORD = struct.Struct("<IHBBIIHHIII")  # 32 bytes
assert RECORD.size == 32

# tile classes
#   0, 3, 6  "skinny": all rows of a small-M operator (rm = 1, 2 or 4 blocks of 16 rows)
#         against a block of 32*G weight rows; long reductions are cut into S slices
#         that different workgroups take.   id = 3*log2(rm)
#   9     128 x 128 output tile staged through LDS
#   10    128 x 64 output tile, for operators with at most 64 output columns
CLS_TILE_128x128 = 9
CLS_TILE_128x64 = 10


@dataclass
class Params:
    edf: int = 1
    skinny_max_m: int = 64          # <= 64
    tile_bytes_max: int = 2048 * 1024
    tile_bytes_min: int = 32 * 1024
    balance_div: int = 512
    max_groups: int = 256
    tail_div: int = 384             # 0: tiles do not shrink towards the end of the table


def canonical(p):
    """(Mg, Ng, Kg) of an operator description with .op/.M/.N/.K or conv fields."""
    if p.op == "gemm":
        return p.M, p.N, p.K
    st = getattr(p, "stride", 1) or 1
    ho = (p.H + 2 * p.pad_h - p.R) // st + 1
    wo = (p.W + 2 * p.pad_w - p.S) // st + 1
    return p.Nb * ho * wo, p.Cout, p.R * p.S * p.Cin


def _deadline_key(d):
    if d is None or not (d > 0.0) or math.isinf(d):   # <=0, NaN, inf: no deadline
        return math.inf
    return float(d)


def order(problems: Sequence, edf: int = 1) -> List[int]:
    n = len(problems)
    if not edf:
        return list(range(n))
    return sorted(range(n), key=lambda i: (_deadline_key(problems[i].deadline_ms), i))


def weight_bytes(p) -> int:
    _, ng, kg = canonical(p)
    return ng * kg * ELEM_SIZE[p.dtype]


def stream_bytes(p, prm: Params) -> int:
    """Operand bytes the operator's tiles load, the unit of the tile targets: the weights, once, for a skinny
    operator; for an LDS-tile operator the 128 + BN operand rows of every 128 x BN output tile over the whole
    reduction."""
    mg, ng, kg = canonical(p)
    if mg <= prm.skinny_max_m:
        return weight_bytes(p)
    bn = 64 if ng <= 64 else 128
    return -(-mg // 128) * -(-ng // bn) * (128 + bn) * kg * ELEM_SIZE[p.dtype]


def target_tile_bytes(problems: Sequence, prm: Params) -> int:
    total = sum(stream_bytes(p, prm) for p in problems)
    return max(prm.tile_bytes_min, min(prm.tile_bytes_max, total // prm.balance_div))


def tiling(p, T: int, prm: Params):
    """(cls, BM, BN, S, slice_len) for one operator given the target bytes per skinny tile."""
    mg, ng, kg = canonical(p)
    es = ELEM_SIZE[p.dtype]
    if mg <= prm.skinny_max_m:
        rm_code = 0 if mg <= 16 else (1 if mg <= 32 else 2)
        gb = 32 * kg * es
        if 4 * gb <= T:
            G = min(prm.max_groups, 4 * max(1, T // (4 * gb)))
            S, slice_len = 1, kg
        else:
            # four groups already exceed the target: cut the reduction into slices of whole chunks
            G = 4
            chunk = (16384 // (16 << rm_code)) // es
            nchunks = -(-kg // chunk)
            want = min(nchunks, -(-4 * gb // T), 255)
            per = -(-nchunks // want)
            S = -(-nchunks // per)
            slice_len = per * chunk
        return 3 * rm_code, mg, 32 * G, S, slice_len
    # LDS tile: cut the reduction when the operand bytes of one tile are far beyond the target
    S, slice_len = 1, kg
    bn = 64 if ng <= 64 else 128
    tb = (128 + bn) * kg * es
    if tb > 2 * T:
        chunk = 256
        nchunks = -(-kg // chunk)
        want = min(nchunks, -(-tb // T), 255, max(1, kg // 1024))   # slices of at least 1024 elements
        per = -(-nchunks // want)
        S = -(-nchunks // per)
        slice_len = per * chunk
    return (CLS_TILE_128x64 if bn == 64 else CLS_TILE_128x128), 128, bn, S, slice_len


def plan(problems: Sequence, prm: Params | None = None):
    """Returns (table_bytes, order, first_tile[n], tile_count[n]) -- first/count by submission index."""
    prm = prm or Params()
    n = len(problems)
    T_all = target_tile_bytes(problems, prm) if n else prm.tile_bytes_min
    ordr = order(problems, prm.edf)
    first = [0] * n
    count = [0] * n
    recs = []
    out_id = 0
    for pos, i in enumerate(ordr):
        p = problems[i]
        mg, ng, kg = canonical(p)
        T = T_all
        if prm.tail_div > 0:
            # stream bytes of this operator and of all that execute after it
            remaining = sum(stream_bytes(problems[j], prm) for j in ordr[pos:])
            # never below eight times the lower clamp (unless the whole table's target is)
            T = min(T_all, max(8 * prm.tile_bytes_min, remaining // prm.tail_div))
        cls, BM, BN, S, slice_len = tiling(p, T, prm)
        first[i] = len(recs)
        for m0 in range(0, mg, BM):
            for n0 in range(0, ng, BN):
                for ks in range(S):
                    k0 = ks * slice_len
                    recs.append(RECORD.pack(i, cls, ks, S, m0, n0, min(BM, mg - m0), min(BN, ng - n0),
                                            k0, min(slice_len, kg - k0), out_id))
                out_id += 1
        count[i] = len(recs) - first[i]
    return b"".join(recs), ordr, first, count


def _z_order_8x8():
    """(row offset, column offset) of the 64 cells of an 8 x 8 block along a Z-order curve that
    starts with a step along the columns."""
    cells = []
    for code in range(64):
        dn = sum(((code >> (2 * b)) & 1) << b for b in range(3))
        dm = sum(((code >> (2 * b + 1)) & 1) << b for b in range(3))
        cells.append((dm, dn))
    return cells


def auto_die_part(problems: Sequence, table: bytes, first: Sequence[int]) -> int:
    """The `part` the planner takes when none is given (xcd_part = -1): 0 (no lists) if the plan has an operator
    in the skinny classes, or if memory rather than the matrix cores bounds it: sum of flops / peak against sum of
    operand bytes / bandwidth over the operators, datasheet figures (2500 TFLOP/s for bf16 and fp16, 157.3 for
    fp32, 8 TB/s), in whole numbers: flops * 2 * (1573 | 25000) against bytes * 983125.  Otherwise an eighth of all
    output rectangles of the plan, rounded up."""
    tiles = decode(table)
    t_flops = t_bytes = rects = 0
    for i, p in enumerate(problems):
        t0 = tiles[first[i]]
        if t0["cls"] not in (CLS_TILE_128x128, CLS_TILE_128x64):
            return 0
        mg, ng, kg = canonical(p)
        bn = 64 if t0["cls"] == CLS_TILE_128x64 else 128
        rects += -(-mg // 128) * -(-ng // bn)
        es = ELEM_SIZE[p.dtype]
        if p.op == "gemm":
            nbytes = es * (p.M * p.K + p.N * p.K + p.M * p.N)
        else:
            nbytes = es * (p.Nb * p.H * p.W * p.Cin + p.Cout * p.R * p.S * p.Cin + mg * p.Cout)
        t_flops += 2 * mg * ng * kg * 2 * (25000 if p.dtype == "f32" else 1573)
        t_bytes += nbytes * 983125
    if rects == 0 or t_flops <= t_bytes:
        return 0
    return -(-rects // 8)


def die_lists(problems: Sequence, table: bytes, ordr: Sequence[int], first: Sequence[int], part: int):
    """Eight lists of table indices: the LDS tiles of the table, die by die, in the order a die takes them.

    Operators in execution order.  The MB x NB output rectangles of an LDS-tile operator are cut into
    p = 1, 2, 4 or 8 parts (the fewest with at most `part` rectangles each), as a pm x pn grid with
    pm * pn = p, pm <= MB, pn <= NB that fetches the fewest operand rows in all (every row block is read by pn
    dies, every column block by pm: pn * MB * 128 + pm * NB * BN; ties go to fewer parts along the columns; if no
    such grid exists, min(p, MB) parts along the rows only);
    part (a, b) covers row blocks [a MB / pm, (a+1) MB / pm) and column blocks [b NB / pn, (b+1) NB / pn).
    Parts go, a outer and b inner, to the die with the shortest list so far that this operator has not used yet
    (lowest index on ties).  Inside a part: blocks of 8 x 8 rectangles row by row, a Z-order curve inside
    each block, the reduction slices of a rectangle together."""
    lists = [[] for _ in range(8)]
    if part <= 0:
        return lists
    tiles = decode(table)
    zcells = _z_order_8x8()
    for i in ordr:
        t0 = tiles[first[i]]
        if t0["cls"] not in (CLS_TILE_128x128, CLS_TILE_128x64):
            continue
        mg, ng, _ = canonical(problems[i])
        bn = 64 if t0["cls"] == CLS_TILE_128x64 else 128
        MB, NB, S = -(-mg // 128), -(-ng // bn), t0["S"]
        p = 1
        while p < 8 and MB * NB > p * part:
            p *= 2
        grids = [(p // cn, cn) for cn in (1, 2, 4, 8) if cn <= p and p // cn <= MB and cn <= NB]
        pm, pn = min(grids, key=lambda g: (g[1] * MB * 128 + g[0] * NB * bn, g[1])) if grids else (min(p, MB), 1)
        used = set()
        for a in range(pm):
            for b in range(pn):
                die = min((x for x in range(8) if x not in used), key=lambda x: (len(lists[x]), x))
                used.add(die)
                m_lo, m_hi = a * MB // pm, (a + 1) * MB // pm
                n_lo, n_hi = b * NB // pn, (b + 1) * NB // pn
                for bm in range(m_lo, m_hi, 8):
                    for bc in range(n_lo, n_hi, 8):
                        for dm, dn in zcells:
                            if bm + dm < m_hi and bc + dn < n_hi:
                                rect = (bm + dm) * NB + (bc + dn)
                                lists[die].extend(first[i] + rect * S + ks for ks in range(S))
    return lists


def decode(table: bytes):
    names = ("problem", "cls", "ks_idx", "S", "m0", "n0", "m_len", "n_len", "k0", "k_len", "out_tile_id")
    return [dict(zip(names, RECORD.unpack_from(table, off))) for off in range(0, len(table), RECORD.size)]


def check_coverage(problems: Sequence, table: bytes) -> None:
    """Brute force: every output element of every operator is owned by exactly one
    output rectangle, and the reduction slices of a rectangle partition [0, Kg).
    Raises AssertionError with the first violation."""
    tiles = decode(table)
    dims = [canonical(p) for p in problems]
    own = [np.zeros((mg, ng), dtype=np.int32) for (mg, ng, _) in dims]
    slices = {}
    for t in tiles:
        i = t["problem"]
        assert 0 <= i < len(problems), f"tile names operator {i}"
        mg, ng, kg = dims[i]
        assert t["m_len"] >= 1 and t["n_len"] >= 1 and t["k_len"] >= 1
        assert t["m0"] + t["m_len"] <= mg and t["n0"] + t["n_len"] <= ng, f"tile leaves operator {i}"
        assert t["k0"] + t["k_len"] <= kg
        key = (i, t["m0"], t["n0"], t["m_len"], t["n_len"], t["out_tile_id"])
        if key not in slices:
            own[i][t["m0"]:t["m0"] + t["m_len"], t["n0"]:t["n0"] + t["n_len"]] += 1
            slices[key] = []
        slices[key].append((t["ks_idx"], t["S"], t["k0"], t["k_len"]))
    for i, o in enumerate(own):
        assert o.size == 0 or (o.min() == 1 and o.max() == 1), \
            f"operator {i}: some output element is owned {o.min()}..{o.max()} times"
    ids = set()
    for key, sl in slices.items():
        assert key[5] not in ids, "two output rectangles share an out_tile_id"
        ids.add(key[5])
        kg = dims[key[0]][2]
        sl.sort()
        S = sl[0][1]
        assert len(sl) == S and [s[0] for s in sl] == list(range(S)), f"slice indices of {key}"
        pos = 0
        for (_, s, k0, kl) in sl:
            assert s == S and k0 == pos, f"reduction slices of {key} do not tile [0,{kg})"
            pos += kl
        assert pos == kg, f"reduction slices of {key} stop at {pos} of {kg}"
    assert ids == set(range(len(ids))), "out_tile_id is not a running index"
