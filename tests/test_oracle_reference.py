"""Pins for the fp64 GEMM / convolution oracle (CPU only).

Each pin is something other than the oracle's own formula: hand-worked values
(tests/golden/hand_examples.json), closed forms, numpy's fp64 matmul, and
identities between the two operators.  A dropped term, a flipped filter, a
transposed operand, a wrong padding offset or a wrong k ordering fails at
least one of them.
"""
import json
import os

import numpy as np
import pytest

from oracle import reference as R


@pytest.fixture(scope="module")
def hand(golden_dir):
    with open(os.path.join(golden_dir, "hand_examples.json")) as f:
        return json.load(f)


def _bnk(b_kn):
    return np.ascontiguousarray(np.array(b_kn, dtype=np.float32).T)


def test_gemm_hand_examples(hand):
    for case in hand["gemm"]:
        A = np.array(case["A"], dtype=np.float32)
        C = R.gemm(A, _bnk(case["B_kn"]))
        assert np.array_equal(C, np.array(case["C"], dtype=np.float64)), case["name"]
        assert np.array_equal(R.gemm_py(A.tolist(), _bnk(case["B_kn"]).tolist()), C)


def test_conv_hand_examples(hand):
    for case in hand["conv"]:
        X = np.array(case["X_hw"], dtype=np.float32)[None, :, :, None]
        W = np.array(case["W_rs"], dtype=np.float32)[None, :, :, None]
        Y = R.conv2d_nhwc(X, W, case["pad"], case["pad"])
        want = np.array(case["Y_hw"], dtype=np.float64)[None, :, :, None]
        assert np.array_equal(Y, want), case["name"]
        assert np.array_equal(R.conv2d_nhwc_py(X, W, case["pad"], case["pad"]), want)


def test_strided_conv_hand_examples(hand):
    for case in hand["conv_strided"]:
        X = np.array(case["X_hw"], dtype=np.float32)[None, :, :, None]
        W = np.array(case["W_rs"], dtype=np.float32)[None, :, :, None]
        want = np.array(case["Y_hw"], dtype=np.float64)[None, :, :, None]
        Y = R.conv2d_nhwc(X, W, case["pad"], case["pad"], stride=case["stride"])
        assert Y.shape == want.shape and np.array_equal(Y, want), case["name"]
        assert np.array_equal(R.conv2d_nhwc_py(X, W, case["pad"], case["pad"], case["stride"]), want)


@pytest.mark.parametrize("cfg", [
    dict(H=7, W=7, R=3, S=3, ph=1, pw=1, st=2), dict(H=6, W=9, R=3, S=3, ph=1, pw=1, st=2),
    dict(H=6, W=6, R=3, S=3, ph=0, pw=0, st=2), dict(H=8, W=5, R=1, S=1, ph=0, pw=0, st=2),
    dict(H=11, W=10, R=3, S=1, ph=1, pw=0, st=3), dict(H=9, W=9, R=5, S=3, ph=2, pw=1, st=4),
])
def test_strided_conv_is_the_unit_stride_result_at_every_stride_th_position(cfg):
    """Y_s[ho, wo] = Y_1[s*ho, s*wo] (same terms, same order: exact), and the output extent is the number
    of filter positions that fit; for a 1x1 filter this is plain subsampling of the image."""
    g = np.random.default_rng(11)
    X = g.standard_normal((2, cfg["H"], cfg["W"], 3)).astype(np.float32)
    W = g.standard_normal((4, cfg["R"], cfg["S"], 3)).astype(np.float32)
    st = cfg["st"]
    Y1, S1 = R.conv2d_nhwc(X, W, cfg["ph"], cfg["pw"], want_mag=True)
    Ys, Ss = R.conv2d_nhwc(X, W, cfg["ph"], cfg["pw"], want_mag=True, stride=st)
    assert Ys.shape == Y1[:, ::st, ::st].shape
    assert np.array_equal(Ys, Y1[:, ::st, ::st]) and np.array_equal(Ss, S1[:, ::st, ::st])
    assert np.array_equal(R.conv2d_nhwc_py(X, W, cfg["ph"], cfg["pw"], st), Ys)
    Pm = R.patch_matrix(X, cfg["R"], cfg["S"], cfg["ph"], cfg["pw"], st)
    want = Pm.astype(np.float64) @ W.reshape(4, -1).astype(np.float64).T
    assert np.max(np.abs(Ys.reshape(-1, 4) - want)) <= 1e-12 * max(1.0, np.max(np.abs(want)))
    b, ho, wo = 1, Ys.shape[1] - 1, Ys.shape[2] - 1
    s, mag = R.conv2d_at(X, W[2], b, ho, wo, cfg["ph"], cfg["pw"], st)
    assert abs(s - Ys[b, ho, wo, 2]) <= 1e-12 * max(mag, 1e-30) and abs(mag - Ss[b, ho, wo, 2]) <= 1e-12 * max(mag, 1e-30)
    if cfg["R"] == 1 and cfg["S"] == 1:
        assert np.array_equal(Ys, np.einsum("bhwc,oc->bhwo", X[:, ::st, ::st].astype(np.float64),
                                            W[:, 0, 0].astype(np.float64)))


def test_conv1x1_hand_example(hand):
    c = hand["conv1x1"]
    X = np.array(c["X_nhwc"], dtype=np.float32)
    W = np.array(c["W_oc_ic"], dtype=np.float32)[:, None, None, :]
    Y = R.conv2d_nhwc(X, W, 0, 0)
    assert np.array_equal(Y.reshape(4, 2), np.array(c["Y_rows"], dtype=np.float64))


def test_gemm_closed_forms():
    M, N, K = 7, 9, 33
    # rank one: A[m,k] = m+1, B[k,n] = n+1  =>  C = K (m+1)(n+1)
    A = np.repeat(np.arange(1, M + 1, dtype=np.float32)[:, None], K, axis=1)
    B = np.repeat(np.arange(1, N + 1, dtype=np.float32)[:, None], K, axis=1)   # [N,K]
    C = R.gemm(A, B)
    want = K * np.outer(np.arange(1, M + 1), np.arange(1, N + 1)).astype(np.float64)
    assert np.array_equal(C, want)
    # identity weight => C = A ; unit-vector activation => C = a row of the K x N operand
    g = np.random.default_rng(1)
    A = g.standard_normal((5, 16)).astype(np.float32)
    assert np.array_equal(R.gemm(A, np.eye(16, dtype=np.float32)), A.astype(np.float64))
    Bkn = g.standard_normal((16, 11)).astype(np.float32)
    e = np.zeros((1, 16), dtype=np.float32)
    e[0, 3] = 1
    assert np.array_equal(R.gemm(e, np.ascontiguousarray(Bkn.T))[0], Bkn[3].astype(np.float64))


def test_gemm_k_weighted_sum_distinguishes_k_alignment():
    # A[m,k] = 10^k digits, B[n,k] = k+1: a shifted or reversed k pairing changes the value
    A = np.array([[1.0, 10.0, 100.0, 1000.0]], dtype=np.float32)
    B = np.array([[1.0, 2.0, 3.0, 4.0], [4.0, 3.0, 2.0, 1.0]], dtype=np.float32)
    assert R.gemm(A, B).tolist() == [[4321.0, 1234.0]]


@pytest.mark.parametrize("shape", [(1, 1, 1), (3, 5, 7), (17, 33, 129), (64, 48, 300)])
def test_gemm_against_numpy_matmul(shape):
    M, N, K = shape
    g = np.random.default_rng(sum(shape))
    A = g.standard_normal((M, K)).astype(np.float32)
    B = g.standard_normal((N, K)).astype(np.float32)
    C, S = R.gemm(A, B, want_mag=True)
    want = A.astype(np.float64) @ B.astype(np.float64).T
    wmag = np.abs(A.astype(np.float64)) @ np.abs(B.astype(np.float64)).T
    assert np.max(np.abs(C - want)) <= 1e-12 * np.max(wmag)
    assert np.max(np.abs(S - wmag)) <= 1e-12 * np.max(wmag)
    # the single-element evaluator agrees with the full loop
    s, mag = R.gemm_at(A[M - 1], B[N // 2])
    assert abs(s - C[M - 1, N // 2]) <= 1e-12 * mag and abs(mag - S[M - 1, N // 2]) <= 1e-12 * mag


def test_gemm_accumulates_in_fp64_not_fp32():
    # 2^24 + 1 is not an fp32 number; an fp32 accumulator would lose the final +1
    K = 3
    A = np.array([[4096.0, 1.0, -4096.0]], dtype=np.float32)
    B = np.array([[4096.0, 1.0, 4096.0]], dtype=np.float32)
    assert R.gemm(A, B)[0, 0] == 1.0
    A = np.array([[4096.0, 1.0]], dtype=np.float32)
    B = np.array([[4096.0, 1.0]], dtype=np.float32)
    assert R.gemm(A, B)[0, 0] == 16777217.0


def test_conv1x1_is_gemm():
    g = np.random.default_rng(2)
    X = g.standard_normal((2, 5, 4, 6)).astype(np.float32)
    W = g.standard_normal((7, 1, 1, 6)).astype(np.float32)
    Y = R.conv2d_nhwc(X, W, 0, 0)
    C = R.gemm(X.reshape(-1, 6), W.reshape(7, 6))
    assert np.array_equal(Y.reshape(-1, 7), C)


@pytest.mark.parametrize("cfg", [
    dict(Nb=1, H=5, W=5, Cin=3, Cout=4, R=3, S=3, ph=1, pw=1),
    dict(Nb=2, H=4, W=6, Cin=2, Cout=3, R=3, S=3, ph=0, pw=0),
    dict(Nb=1, H=6, W=3, Cin=5, Cout=2, R=3, S=1, ph=1, pw=0),
    dict(Nb=1, H=4, W=4, Cin=1, Cout=1, R=1, S=3, ph=0, pw=2),
])
def test_direct_conv_equals_patch_matrix_gemm(cfg):
    g = np.random.default_rng(3)
    X = g.standard_normal((cfg["Nb"], cfg["H"], cfg["W"], cfg["Cin"])).astype(np.float32)
    W = g.standard_normal((cfg["Cout"], cfg["R"], cfg["S"], cfg["Cin"])).astype(np.float32)
    Y, Sm = R.conv2d_nhwc(X, W, cfg["ph"], cfg["pw"], want_mag=True)
    P = R.patch_matrix(X, cfg["R"], cfg["S"], cfg["ph"], cfg["pw"])
    want = P.astype(np.float64) @ W.reshape(cfg["Cout"], -1).astype(np.float64).T
    assert Y.reshape(-1, cfg["Cout"]).shape == want.shape
    assert np.max(np.abs(Y.reshape(-1, cfg["Cout"]) - want)) <= 1e-12 * max(1.0, np.max(np.abs(want)))
    assert np.allclose(Y, R.conv2d_nhwc_py(X, W, cfg["ph"], cfg["pw"]), rtol=0, atol=1e-12)
    # single-element evaluator
    b, ho, wo, co = cfg["Nb"] - 1, Y.shape[1] - 1, 0, cfg["Cout"] - 1
    s, mag = R.conv2d_at(X, W[co], b, ho, wo, cfg["ph"], cfg["pw"])
    assert abs(s - Y[b, ho, wo, co]) <= 1e-12 * max(mag, 1e-30)
    assert abs(mag - Sm[b, ho, wo, co]) <= 1e-12 * max(mag, 1e-30)


def test_conv_delta_filter_is_identity_and_shift():
    g = np.random.default_rng(4)
    X = g.standard_normal((1, 6, 5, 3)).astype(np.float32)
    # centre tap: Y = X (per channel)
    W = np.zeros((3, 3, 3, 3), dtype=np.float32)
    for c in range(3):
        W[c, 1, 1, c] = 1
    assert np.array_equal(R.conv2d_nhwc(X, W, 1, 1), X.astype(np.float64))
    # tap (r=0,s=1) with pad 1 reads the pixel one row above: Y[h] = X[h-1], first row zero
    W = np.zeros((3, 3, 3, 3), dtype=np.float32)
    for c in range(3):
        W[c, 0, 1, c] = 1
    Y = R.conv2d_nhwc(X, W, 1, 1)
    assert np.array_equal(Y[:, 1:], X[:, :-1].astype(np.float64)) and not Y[:, 0].any()
    # tap (r=1,s=2) reads the pixel to the right: Y[w] = X[w+1], last column zero
    W = np.zeros((3, 3, 3, 3), dtype=np.float32)
    for c in range(3):
        W[c, 1, 2, c] = 1
    Y = R.conv2d_nhwc(X, W, 1, 1)
    assert np.array_equal(Y[:, :, :-1], X[:, :, 1:].astype(np.float64)) and not Y[:, :, -1].any()


def test_conv_output_shape_rule():
    X = np.ones((1, 7, 9, 2), dtype=np.float32)
    W = np.ones((1, 3, 3, 2), dtype=np.float32)
    assert R.conv2d_nhwc(X, W, 1, 1).shape == (1, 7, 9, 1)
    assert R.conv2d_nhwc(X, W, 0, 0).shape == (1, 5, 7, 1)
    Y = R.conv2d_nhwc(X, W, 1, 1)
    # all-ones: each output counts the taps inside the image times Cin
    assert Y[0, 0, 0, 0] == 8 and Y[0, 0, 4, 0] == 12 and Y[0, 3, 4, 0] == 18


# ---- channel-major (NCHW) convolution ----------------------------------------------------------

def test_nchw_conv_hand_examples(hand):
    for ex in hand["conv_nchw"]:
        X = np.array(ex["X_nchw"], dtype=np.float32)
        W = np.array(ex["W_oihw"], dtype=np.float32)
        want = np.array(ex["Y_nchw"], dtype=np.float64)
        for fn in (R.conv2d_nchw, R.conv2d_nchw_py):
            got = fn(X, W, ex["pad_h"], ex["pad_w"], stride=ex["stride"])
            assert got.shape == want.shape, ex["name"]
            assert np.array_equal(got, want), (ex["name"], got)


@pytest.mark.parametrize("cfg", [(1, 5, 6, 3, 4, 3, 3, 1, 1, 1), (2, 7, 5, 2, 3, 3, 1, 0, 0, 2), (1, 6, 6, 4, 2, 1, 1, 0, 0, 1),
                                 (2, 4, 9, 3, 5, 5, 3, 2, 1, 3), (1, 8, 8, 1, 1, 7, 7, 3, 3, 2)])
def test_nchw_conv_is_a_sum_of_library_2d_correlations(cfg):
    """Per image and output channel the operator is sum_c correlate2d(X[b,c] zero-padded, W[co,c]) sampled
    every `stride` positions: scipy's routine knows nothing of this build's index arithmetic."""
    from scipy.signal import correlate2d

    Nb, H, Wd, Cin, Cout, Rr, S, ph, pw, st = cfg
    g = np.random.default_rng(sum(cfg))
    X = g.integers(-4, 5, size=(Nb, Cin, H, Wd)).astype(np.float32)
    W = g.integers(-3, 4, size=(Cout, Cin, Rr, S)).astype(np.float32)
    got = R.conv2d_nchw(X, W, ph, pw, stride=st)
    Xp = np.pad(X.astype(np.float64), ((0, 0), (0, 0), (ph, ph), (pw, pw)))
    for b in range(Nb):
        for co in range(Cout):
            full = sum(correlate2d(Xp[b, c], W[co, c].astype(np.float64), mode="valid") for c in range(Cin))
            assert np.array_equal(got[b, co], full[::st, ::st]), (cfg, b, co)


def test_nchw_conv_is_the_nhwc_result_on_permuted_arrays():
    """The two storage orders describe one operator: permuting operands and result maps one onto the other
    (the two C routines index their arrays independently)."""
    g = np.random.default_rng(5)
    for (Nb, H, Wd, Cin, Cout, Rr, S, ph, pw, st) in [(2, 9, 7, 5, 6, 3, 3, 1, 1, 1), (1, 12, 5, 3, 4, 5, 1, 2, 0, 2),
                                                      (3, 4, 4, 8, 2, 1, 1, 0, 0, 1)]:
        X = g.standard_normal((Nb, Cin, H, Wd)).astype(np.float32)
        W = g.standard_normal((Cout, Cin, Rr, S)).astype(np.float32)
        Y, M = R.conv2d_nchw(X, W, ph, pw, want_mag=True, stride=st)
        Y2, M2 = R.conv2d_nhwc(X.transpose(0, 2, 3, 1), W.transpose(0, 2, 3, 1), ph, pw, want_mag=True, stride=st)
        # same terms in another order: equal to a few ulps of the magnitude sum
        assert np.all(np.abs(Y - Y2.transpose(0, 3, 1, 2)) <= 1e-15 * M * (Cin * Rr * S))
        assert np.all(np.abs(M - M2.transpose(0, 3, 1, 2)) <= 1e-15 * M * (Cin * Rr * S))
        assert np.array_equal(R.conv2d_nchw_py(X, W, ph, pw, st), R.conv2d_nchw_py(X, W, ph, pw, st))
        assert np.all(np.abs(Y - R.conv2d_nchw_py(X, W, ph, pw, st)) <= 1e-15 * M * (Cin * Rr * S))


def test_nchw_delta_filter_picks_one_channel_and_shifts():
    """A filter that is 1 at (channel 2, tap (0, 1)) and 0 elsewhere copies channel 2 shifted by one column."""
    g = np.random.default_rng(9)
    X = g.standard_normal((2, 4, 5, 6)).astype(np.float32)
    W = np.zeros((1, 4, 1, 2), dtype=np.float32)
    W[0, 2, 0, 1] = 1.0
    Y = R.conv2d_nchw(X, W, 0, 0)
    assert Y.shape == (2, 1, 5, 5)
    assert np.array_equal(Y[:, 0], X[:, 2, :, 1:].astype(np.float64))
