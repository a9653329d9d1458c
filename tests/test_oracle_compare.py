"""Pins for the error measures the parity tests assert on (CPU only).

`compare.errors` is held to hand-worked numbers (every figure below was worked out on paper from the
definitions: gate = max |c-ref| / max(|ref|, rms(ref)), strict = max |c-ref| / |ref|, normwise =
max |c-ref| / max |ref|, backward = max |c-ref| / sum |a||b|).  `compare.order_free_bound` is held from
both sides: summations that ARE fp32 accumulations of the exact products (in any order) must pass, one of
them coming within a few per cent of the bound, and computations that are NOT (a dropped product, fp16
accumulation, products rounded to bf16, a result rounded twice) must be rejected.
"""
import numpy as np
import pytest

from oracle import compare, rounding as Q


# ---- compare.errors -----------------------------------------------------------------------------------

def test_errors_hand_worked_gate_where_the_rms_floor_decides():
    # rms(ref) = sqrt((1 + 49 + 25 + 25) / 4) = 5 exactly; mean |ref| = 4.5, max |ref| = 7
    ref = np.array([[1.0, -7.0], [5.0, 5.0]])
    c = ref + np.array([[0.6, -0.7], [0.25, 0.0]])
    mag = np.array([[2.0, 14.0], [5.0, 10.0]])
    e = compare.errors(c, ref, mag)
    # floors: max(|ref|, 5) = 5, 7, 5, 5  ->  0.6/5, 0.7/7, 0.25/5, 0
    assert e["gate"] == pytest.approx(0.12, rel=1e-12)
    assert e["strict"] == pytest.approx(0.6, rel=1e-12)         # 0.6 / 1
    assert e["normwise"] == pytest.approx(0.1, rel=1e-12)       # 0.7 / 7
    assert e["max_abs"] == pytest.approx(0.7, rel=1e-12)
    assert e["backward"] == pytest.approx(0.3, rel=1e-12)       # 0.6 / 2
    # a mean instead of a root mean square as the floor would give 0.6 / 4.5, the largest |ref| 0.6 / 7
    assert abs(e["gate"] - 0.6 / 4.5) > 1e-3 and abs(e["gate"] - 0.6 / 7) > 1e-3


def test_errors_hand_worked_gate_where_the_element_itself_decides():
    ref = np.array([1.0, -7.0, 5.0, 5.0])
    c = ref + np.array([0.4, 0.84, -0.25, 0.0])
    e = compare.errors(c, ref)
    # 0.4/5, 0.84/7, 0.25/5, 0: the element above the rms is divided by its own size
    assert e["gate"] == pytest.approx(0.12, rel=1e-12)
    assert e["strict"] == pytest.approx(0.4, rel=1e-12)
    assert "backward" not in e


def test_errors_cancellation_strict_far_above_gate():
    # one output is tiny because its terms cancelled: an absolute error of 1e-4 there is a strict relative
    # error of 100 but only 1e-4 / rms on the gate
    ref = np.array([2.0, -2.0, 2.0, 1e-6])
    c = ref.copy()
    c[3] += 1e-4
    e = compare.errors(c, ref, mag=np.array([4.0, 4.0, 4.0, 4.0]))
    rms = np.sqrt((4.0 + 4.0 + 4.0 + 1e-12) / 4.0)
    assert e["strict"] == pytest.approx(100.0, rel=1e-9)
    assert e["gate"] == pytest.approx(1e-4 / rms, rel=1e-9)
    assert e["strict"] > 1e5 * e["gate"]
    assert e["backward"] == pytest.approx(2.5e-5, rel=1e-9)


def test_errors_sign_zero_reference_and_empty_input():
    # the difference enters by absolute value, a reference of exactly zero is skipped by the strict figure
    ref = np.array([0.0, 3.0, -4.0, 0.0])            # rms = 2.5
    c = np.array([-0.5, 3.0, -4.0, 0.25])
    e = compare.errors(c, ref)
    assert e["gate"] == pytest.approx(0.2, rel=1e-12)           # 0.5 / 2.5
    assert e["strict"] == 0.0
    assert e["normwise"] == pytest.approx(0.125, rel=1e-12)     # 0.5 / 4
    z = compare.errors(np.zeros((0, 3)), np.zeros((0, 3)), np.zeros((0, 3)))
    assert z["gate"] == 0.0 and z["strict"] == 0.0 and z["normwise"] == 0.0 and z["backward"] == 0.0
    # all-zero reference: nothing to divide by, the gate is the absolute error
    assert compare.errors(np.array([0.5, 0.0]), np.zeros(2))["gate"] == pytest.approx(0.5)


def test_tolerances_are_the_stated_ones():
    assert compare.TOL == {"f32": 1e-5, "bf16": 2e-2, "f16": 2e-2}


# ---- compare.order_free_bound -------------------------------------------------------------------------

def _operands(M, N, K, dtype, positive, seed):
    g = np.random.default_rng(seed)
    if positive:
        a = g.uniform(0.0, 1.0, (M, K)).astype(np.float32)
        b = g.uniform(0.0, 1.0, (N, K)).astype(np.float32)
    else:
        a = g.standard_normal((M, K)).astype(np.float32)
        b = (g.standard_normal((N, K)) / np.sqrt(K)).astype(np.float32)
    a = Q.round_to(dtype, a)[1]
    b = Q.round_to(dtype, b)[1]
    return a, b


def _products(a, b):
    """Exact products as fp32 [M, N, K] (16-bit operands: 8 or 11 significand bits each, exact in fp32)."""
    return a[:, None, :].astype(np.float32) * b[None, :, :].astype(np.float32)


def _seq_sum(p, acc_type):
    s = np.zeros(p.shape[:2], dtype=acc_type)
    for k in range(p.shape[2]):
        s = (s + p[:, :, k].astype(acc_type)).astype(acc_type)
    return s


def _pairwise_sum(p):
    p = p.astype(np.float32)
    while p.shape[2] > 1:
        if p.shape[2] % 2:
            p = np.concatenate([p, np.zeros(p.shape[:2] + (1,), dtype=np.float32)], axis=2)
        p = (p[:, :, 0::2] + p[:, :, 1::2]).astype(np.float32)
    return p[:, :, 0]


def _ref_mag(a, b):
    ref = a.astype(np.float64) @ b.astype(np.float64).T
    mag = np.abs(a).astype(np.float64) @ np.abs(b).astype(np.float64).T
    return ref, mag


@pytest.mark.parametrize("dtype", ["bf16", "f16"])
@pytest.mark.parametrize("positive", [False, True])
def test_bound_accepts_fp32_accumulation_in_any_order(dtype, positive):
    M, N, K = 6, 40, 4096
    a, b = _operands(M, N, K, dtype, positive, seed=3)
    p = _products(a, b)
    assert np.array_equal(p.astype(np.float64), a[:, None, :].astype(np.float64) * b[None, :, :].astype(np.float64))
    ref, mag = _ref_mag(a, b)
    g = np.random.default_rng(9)
    for name, s in (("ascending", _seq_sum(p, np.float32)), ("descending", _seq_sum(p[:, :, ::-1], np.float32)),
                    ("pairwise", _pairwise_sum(p)), ("shuffled", _seq_sum(p[:, :, g.permutation(K)], np.float32))):
        for out in (dtype, "f32"):
            got = Q.round_to(out, s)[1].astype(np.float64)
            over = np.abs(got - ref) > compare.order_free_bound(ref, mag, K, out)
            assert not over.any(), (name, out, int(over.sum()))


def test_bound_is_nearly_attained_by_a_valid_fp32_summation():
    """1 + K terms just under half a unit in the last place of 1: added one by one each is lost, so the
    error is K * 2^-24 * (1 - eps) against a bound of (K + 2) * 2^-24 * mag: the bound cannot be tightened
    by more than a few per cent (a gamma of 2^-25, or one without the factor K, fails here)."""
    K = 1000
    t = np.float32(2.0 ** -24 * (1 - 2.0 ** -10))
    terms = np.concatenate([[np.float32(1.0)], np.full(K - 1, t, dtype=np.float32)])
    s = np.float32(0.0)
    for x in terms:
        s = np.float32(s + x)
    assert s == np.float32(1.0)
    ref = np.array([float(np.sum(terms.astype(np.float64)))])
    mag = ref.copy()
    bound = compare.order_free_bound(ref, mag, K, "f32")[0]
    err = abs(float(s) - ref[0])
    assert err <= bound and err >= 0.95 * bound, (err, bound)


def test_bound_rejects_a_dropped_product():
    """A reduction that stops one element early.  The lost term is about mag / K; it can only show where it
    exceeds the rounding of the output format (2^-8 |ref| for bf16), hence the shorter reductions for the
    16-bit outputs; with fp32 outputs nearly every output shows it at K = 512, and at K = 4096, where the
    accumulation allowance (K + 2) * 2^-24 * mag has grown to the size of a typical term, a good third."""
    M, N = 4, 64
    for dtype, out, positive, K, least in (("bf16", "bf16", False, 64, 0.6), ("f16", "f16", True, 256, 0.8),
                                           ("bf16", "f32", False, 512, 0.9), ("f32", "f32", False, 512, 0.9),
                                           ("f32", "f32", False, 4096, 0.3)):
        a, b = _operands(M, N, K, dtype, positive, seed=5)
        ref, mag = _ref_mag(a, b)
        s = a[:, :K - 1].astype(np.float64) @ b[:, :K - 1].astype(np.float64).T
        got = Q.round_to(out, s.astype(np.float32))[1].astype(np.float64)
        over = np.abs(got - ref) > compare.order_free_bound(ref, mag, K, out)
        assert over.mean() > least, (dtype, out, K, over.mean())
        # the full sum, rounded the same way, passes everywhere
        full = Q.round_to(out, ref.astype(np.float32))[1].astype(np.float64)
        assert not (np.abs(full - ref) > compare.order_free_bound(ref, mag, K, out)).any()


def test_bound_rejects_fp16_accumulation_at_k_4096():
    M, N, K = 4, 64, 4096
    # positive terms: the fp16 partial sum stops growing once a product is below half its spacing
    a, b = _operands(M, N, K, "f16", True, seed=6)
    ref, mag = _ref_mag(a, b)
    s = _seq_sum(_products(a, b), np.float16)
    for out in ("f16", "f32"):
        got = Q.round_to(out, s.astype(np.float32))[1].astype(np.float64)
        assert (np.abs(got - ref) > compare.order_free_bound(ref, mag, K, out)).all(), out
    # signed terms: a random walk of roundings of 2^-11 each; with fp32 outputs a good share is caught
    a, b = _operands(M, N, K, "f16", False, seed=7)
    ref, mag = _ref_mag(a, b)
    s = _seq_sum(_products(a, b), np.float16).astype(np.float64)
    over = np.abs(s - ref) > compare.order_free_bound(ref, mag, K, "f32")
    assert over.mean() > 0.2, over.mean()
    # while the fp32 accumulation of the same products passes everywhere
    s32 = _seq_sum(_products(a, b), np.float32).astype(np.float64)
    assert not (np.abs(s32 - ref) > compare.order_free_bound(ref, mag, K, "f32")).any()


def test_bound_rejects_products_rounded_to_bf16():
    """Each product rounded to bf16 before it is added (fp32 accumulation otherwise): the error is about
    2^-9 |a b| per term, far above (K + 2) * 2^-24 per unit of sum |a||b| at K = 64; a gamma of 2^-14
    instead of 2^-24 would let it through."""
    M, N, K = 8, 64, 64
    a, b = _operands(M, N, K, "f16", False, seed=8)
    ref, mag = _ref_mag(a, b)
    p = Q.round_to("bf16", _products(a, b))[1]
    s = _seq_sum(p, np.float32).astype(np.float64)
    over = np.abs(s - ref) > compare.order_free_bound(ref, mag, K, "f32")
    assert over.mean() > 0.95, over.mean()


def test_bound_rejects_a_result_rounded_twice():
    """fp32 -> fp16 -> bf16 instead of fp32 -> bf16.  Just below the midpoint of an odd and the next even
    bf16 number the first rounding lands on the midpoint and the second goes to the even neighbour above:
    the error is half a bf16 step plus up to half an fp16 step, where one rounding stays below half a step."""
    # (the bound is relative, u |ref|, so it resolves the extra half fp16 step only in the lower tenth of a
    # binade, where u |ref| is hardly more than half a bf16 step)
    k = np.arange(1, 12, 2, dtype=np.float64)                    # odd significands 1 + k * 2^-7
    delta = 2.0 ** -11 * 0.9                                     # (half an fp16 step at 1 is 2^-11)
    x = (1.0 + k * 2.0 ** -7 + 2.0 ** -8 - delta)                # just under the midpoint above an odd number
    x = np.concatenate([x, -x, 8.0 * x, x / 64.0]).astype(np.float32)
    ref = x.astype(np.float64)                                   # K = 2: ref = x * 1 + 0 * 0
    mag = np.abs(ref)
    once = Q.round_to("bf16", x)[1].astype(np.float64)
    twice = Q.round_to("bf16", Q.round_to("f16", x)[1])[1].astype(np.float64)
    assert (once != twice).all()
    bound = compare.order_free_bound(ref, mag, 2, "bf16")
    assert not (np.abs(once - ref) > bound).any()
    assert (np.abs(twice - ref) > bound).all()
