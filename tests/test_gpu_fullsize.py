"""Full-size parity: the 256-operator mixed plan (about 5 GB of weights), in the launch
configuration bench.py times (2 MiB tile target, tiles of up to 256 weight groups, shrinking
tail), checked on EVERY output element of every operator.

Inputs are drawn on the GPU (seeded); operator by operator the operands are copied back and
the oracle's plain C loops compute the whole result with its sum of magnitudes, so no expected
value comes from the HIP path.  The plan must equal the reference planner's.  The
one-launch-per-operator baseline tiles every operator as if it were alone (other reduction
slices, another order of summation): it is held to the oracle in the same way, not to the bits
of the coalesced launch.  A second test covers operands beyond 4 GiB on sampled outputs.
"""
import numpy as np
import pytest
import torch

import paper_1901_10008_amd as sk
import workloads
from oracle import compare, planner as P, reference as R

import sk_harness as H

pytestmark = pytest.mark.gpu


def _whole_operator_check(b, specs, outs, label):
    """Every element of every operator against the oracle: written, within the gate (the operator's
    own rms) and under the summation-order-free rounding bound."""
    worst = 0.0
    for i, s in enumerate(specs):
        rows, cols, ldc, off = b.c_meta[i]
        out = outs[i][off: off + rows * ldc].view(torch.bfloat16).view(rows, ldc)[:, :cols]
        got = out.float().cpu().numpy().astype(np.float64)
        assert not np.isnan(got).any(), f"{label} operator {i}: output not fully written"
        A = b.dA[i].float().cpu().numpy()
        W = b.dB[i].float().cpu().numpy()
        if s.op == "gemm":
            ref, mag = R.gemm(A, W, want_mag=True)
        else:
            Y, Sm = R.conv2d_nhwc(A, W, s.pad_h, s.pad_w, want_mag=True, stride=s.stride)
            ref, mag = Y.reshape(rows, cols), Sm.reshape(rows, cols)
        del A, W
        e = compare.errors(got, ref, mag)
        assert e["gate"] <= compare.TOL[s.dtype], (label, i, s, e)
        over = np.abs(got - ref) > compare.order_free_bound(ref, mag, H.kg_of(s), s.dtype)
        assert not over.any(), (label, i, s, int(over.sum()), e)
        worst = max(worst, e["gate"])
    return worst


def test_config5_full_size_every_element():
    seed = 0
    specs = workloads.config(5, seed=seed)
    b = H.Batch(specs, seed=seed, host_draw=False)
    R.set_threads(16)
    with b.plan() as plan:
        table, order, first, count = P.plan(specs)
        assert sk.sk_plan_get_tiles(plan) == table and sk.sk_plan_get_order(plan) == order
        sk.sk_launch(plan, H.stream_handle())
        torch.cuda.synchronize()
        outs = [c.clone() for c in b.c_bufs]
        b.reset_outputs()
        sk.sk_launch_sequential(plan, H.stream_handle())
        torch.cuda.synchronize()
        seq = [c.clone() for c in b.c_bufs]
        # a relaunch of the coalesced plan gives the same bits (fixed order of the split reductions)
        b.reset_outputs()
        sk.sk_launch(plan, H.stream_handle())
        torch.cuda.synchronize()
        for i, (x, y) in enumerate(zip(outs, b.c_bufs)):
            assert torch.equal(x, y), f"operator {i}: relaunch differs"
    print("config 5 full size, every element: worst gate error",
          _whole_operator_check(b, specs, outs, "coalesced"), "coalesced,",
          _whole_operator_check(b, specs, seq, "sequential"), "sequential")


def _rows_around(limit_row, last):
    """Row indices next to the first row whose byte offset passes 4 GiB, plus both ends."""
    near = [limit_row - 1, limit_row, limit_row + 1]
    return [r for r in [0, 1, *near, last - 1, last] if 0 <= r <= last]


def test_operands_larger_than_4_gib():
    """Activations, weights and outputs of more than 4 GiB each: element offsets do not fit 32
    bits.  One tall GEMM (LDS-tiled), one wide weight-streaming GEMM and one batched 3x3
    convolution share a plan with two small operators; outputs are sampled on both sides of the
    4 GiB line of every large buffer and at both ends."""
    from workloads import Problem

    four_gib = 1 << 32
    specs = [
        Problem(op="gemm", dtype="bf16", M=5_000_011, N=512, K=520, a_dist=("normal", 1.0), b_dist=("normal", 0.04)),
        Problem(op="gemm", dtype="bf16", M=4, N=5_000_008, K=520, a_dist=("normal", 1.0), b_dist=("normal", 0.04)),
        Problem(op="conv", dtype="bf16", Nb=40, H=1024, W=1024, Cin=64, Cout=64, R=3, S=3, pad_h=1, pad_w=1,
                a_dist=("uniform", 0.0, 1.0), b_dist=("normal", 0.06)),
        Problem(op="gemm", dtype="bf16", M=8, N=1000, K=2048, a_dist=("normal", 1.0), b_dist=("normal", 0.02)),
        Problem(op="gemm", dtype="f32", M=3, N=77, K=129, a_dist=("normal", 1.0), b_dist=("normal", 0.1)),
        # rows of an odd length cannot be read in 16-byte pieces: the element-wise paths
        Problem(op="gemm", dtype="bf16", M=4_200_003, N=40, K=521, a_dist=("normal", 1.0), b_dist=("normal", 0.04)),
        Problem(op="gemm", dtype="bf16", M=3, N=4_200_001, K=521, a_dist=("normal", 1.0), b_dist=("normal", 0.04)),
    ]
    b = H.Batch(specs, seed=11, host_draw=False)
    g = np.random.default_rng(7)
    with b.plan() as plan:
        sk.sk_launch(plan, H.stream_handle())
        torch.cuda.synchronize()
    dev = lambda idx: torch.as_tensor(np.asarray(idx), device="cuda")
    views = []
    for i, s in enumerate(specs):
        rows, cols, ldc, off = b.c_meta[i]
        real = torch.float32 if s.dtype == "f32" else torch.bfloat16
        out = b.c_bufs[i][off: off + rows * ldc].view(real).view(rows, ldc)[:, :cols]
        assert not torch.isnan(out).any(), f"operator {i}: output not fully written"
        views.append(out)

    def check(i, got, ref, mag, what):
        s = specs[i]
        got = got.float().cpu().numpy().astype(np.float64).reshape(ref.shape)
        e = compare.errors(got, ref, mag)
        assert e["gate"] <= compare.TOL[s.dtype], (what, e)
        assert not (np.abs(got - ref) > compare.order_free_bound(ref, mag, H.kg_of(s), s.dtype)).any(), (what, e)
        print(f"{what}: {got.size} outputs sampled, gate error {e['gate']:.2e}")

    # tall GEMM: rows of A pass 4 GiB at 2^32 / (K * 2), rows of C at 2^32 / (N * 2)
    s = specs[0]
    ms = np.unique(np.concatenate([_rows_around(four_gib // (s.K * 2), s.M - 1), _rows_around(four_gib // (s.N * 2), s.M - 1),
                                   g.integers(0, s.M, size=24)]))
    ref, mag = R.gemm(b.dA[0][dev(ms)].float().cpu().numpy(), b.dB[0].float().cpu().numpy(), want_mag=True)
    check(0, views[0][dev(ms)], ref, mag, "tall GEMM")
    # wide GEMM: rows of the weights pass 4 GiB at 2^32 / (K * 2)
    s = specs[1]
    ns = np.unique(np.concatenate([_rows_around(four_gib // (s.K * 2), s.N - 1), g.integers(0, s.N, size=120)]))
    ref, mag = R.gemm(b.dA[1].float().cpu().numpy(), b.dB[1][dev(ns)].float().cpu().numpy(), want_mag=True)
    check(1, views[1][:, dev(ns)], ref, mag, "wide GEMM")
    # convolution: bands of four output rows; the image rows they read are copied with a zero row
    # where the band touches the padding, so the oracle runs with no padding in that direction
    s = specs[2]
    Wt = b.dB[2].float().cpu().numpy()
    X = b.dA[2]
    image_bytes = s.H * s.W * s.Cin * 2
    out4 = views[2].view(s.Nb, s.H, s.W, s.Cout)  # same size output: 3x3, padding 1, stride 1
    for img, h0 in [(0, 0), (four_gib // image_bytes, 0), (four_gib // image_bytes - 1, s.H - 4),
                    (int(g.integers(0, s.Nb)), int(g.integers(1, s.H - 5))), (s.Nb - 1, s.H - 4)]:
        lo, hi = h0 - 1, h0 + 5  # input rows [lo, hi) feed output rows h0 .. h0+3
        band = torch.zeros((1, hi - lo, s.W, s.Cin), dtype=torch.float32, device="cuda")
        a, z = max(lo, 0), min(hi, s.H)
        band[0, a - lo: z - lo] = X[img, a:z].float()
        Y, Sm = R.conv2d_nhwc(band.cpu().numpy(), Wt, 0, s.pad_w, want_mag=True)
        assert Y.shape == (1, 4, s.W, s.Cout)
        check(2, out4[img, h0: h0 + 4], Y[0], Sm[0], f"convolution image {img} rows {h0}..{h0 + 3}")
    s = specs[5]
    ms = np.unique(np.concatenate([_rows_around(four_gib // (s.K * 2), s.M - 1), g.integers(0, s.M, size=24)]))
    ref, mag = R.gemm(b.dA[5][dev(ms)].float().cpu().numpy(), b.dB[5].float().cpu().numpy(), want_mag=True)
    check(5, views[5][dev(ms)], ref, mag, "tall GEMM, odd row length")
    s = specs[6]
    ns = np.unique(np.concatenate([_rows_around(four_gib // (s.K * 2), s.N - 1), g.integers(0, s.N, size=120)]))
    ref, mag = R.gemm(b.dA[6].float().cpu().numpy(), b.dB[6][dev(ns)].float().cpu().numpy(), want_mag=True)
    check(6, views[6][:, dev(ns)], ref, mag, "wide GEMM, odd row length")
    # the two small operators, in full
    for i in (3, 4):
        ref, mag = R.gemm(b.dA[i].float().cpu().numpy(), b.dB[i].float().cpu().numpy(), want_mag=True)
        check(i, views[i], ref, mag, f"small operator {i}")
