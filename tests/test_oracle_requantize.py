"""Pins for the oracle's requantize and encode_multiplier.

The operator is named in Sec. 6.1 (Quantized Model Realization) and Sec. 6.2
(QNN requantize); its Q31-multiplier / rounding-shift form is this build's
convention.  The pins are the exact rational definition evaluated with Python
big integers and fractions, hand-worked vectors, and invariants.
"""
from fractions import Fraction
import math

import numpy as np
import pytest

from conftest import read_golden

I32_MIN, I32_MAX = -(2 ** 31), 2 ** 31 - 1


def exact_nearest(acc, M, sh):
    """Nearest integer to acc*M/2^(31+sh), ties toward +infinity."""
    return math.floor(Fraction(acc * M, 2 ** (31 + sh)) + Fraction(1, 2))


def clip(v, lo, hi):
    return max(lo, min(hi, v))


def test_golden_vectors_are_exact_and_oracle_matches(ref):
    rows = read_golden("requantize_vectors.txt")
    assert len(rows) >= 20
    for acc, M, sh, z, lo, hi, want in (map(int, r) for r in rows):
        assert clip(exact_nearest(acc, M, sh) + z, lo, hi) == want, (acc, M, sh)
        assert ref.requantize_one(acc, M, sh, z, lo, hi) == want, (acc, M, sh)


@pytest.mark.parametrize("M,sh", [(2 ** 30, 0), (2 ** 30, 3), (1717986918, 3),
                                  (1395864371, 7), (2 ** 31 - 1, 0), (1288490189, 15),
                                  (2 ** 31 - 1, 31), (2 ** 30, 31)])
def test_brute_force_against_integer_floor_division(ref, M, sh):
    # floor((2*acc*M + 2^t) / 2^(t+1)) with unbounded integers: the same real
    # number floor(acc*M/2^t + 1/2), written without any shift.
    t = 31 + sh
    accs = np.arange(-70000, 70001, dtype=np.int64)
    mult = np.full(1, M, np.int32)
    shift = np.full(1, sh, np.int32)
    rq = ref.Requant(mult, shift, out_dtype=ref.I8, clip_lo=-128, clip_hi=127)
    got_clipped = ref.requantize(accs.astype(np.int32).reshape(1, 1, -1), rq).reshape(-1)
    for i in range(0, accs.size, 7):  # every 7th value one by one, unclipped
        a = int(accs[i])
        want = (2 * a * M + 2 ** t) // 2 ** (t + 1)
        assert ref.requantize_one(a, M, sh) == want
    want_all = np.array([clip((2 * int(a) * M + 2 ** t) // 2 ** (t + 1), -128, 127) for a in accs])
    assert np.array_equal(got_clipped.astype(np.int64), want_all)


def test_fraction_definition_on_random_and_extreme_inputs(ref):
    rng = np.random.default_rng(1)
    accs = list(rng.integers(I32_MIN, I32_MAX, 3000, endpoint=True)) + [I32_MIN, I32_MAX, 0, 1, -1]
    for a in accs:
        M = int(rng.integers(2 ** 30, 2 ** 31))
        sh = int(rng.integers(0, 32))
        got = ref.requantize_one(int(a), M, sh)
        want = exact_nearest(int(a), M, sh)
        assert got == want
        assert abs(Fraction(got) - Fraction(int(a) * M, 2 ** (31 + sh))) <= Fraction(1, 2)


def test_invariants(ref):
    rng = np.random.default_rng(2)
    for _ in range(50):
        M = int(rng.integers(2 ** 30, 2 ** 31))
        sh = int(rng.integers(0, 16))
        assert ref.requantize_one(0, M, sh) == 0
        accs = np.sort(rng.integers(-10 ** 6, 10 ** 6, 400))
        r = [ref.requantize_one(int(a), M, sh) for a in accs]
        assert all(x <= y for x, y in zip(r, r[1:]))  # monotone


def test_power_of_two_threshold_reduces_to_a_rounding_shift(ref):
    # Sec. 5.1: power-of-two thresholds let requantize be a pure shift.
    # With M = 2^30 the multiplier is 1/2: r = floor(acc / 2^(sh+1) + 1/2).
    rng = np.random.default_rng(3)
    for a in list(rng.integers(I32_MIN, I32_MAX, 2000)) + [I32_MIN, I32_MAX]:
        for sh in (0, 1, 5, 13, 31):
            want = math.floor(Fraction(int(a), 2 ** (sh + 1)) + Fraction(1, 2))
            assert ref.requantize_one(int(a), 2 ** 30, sh) == want


def test_zero_point_and_clip(ref):
    rng = np.random.default_rng(4)
    for _ in range(2000):
        a = int(rng.integers(-10 ** 6, 10 ** 6))
        M = int(rng.integers(2 ** 30, 2 ** 31))
        sh = int(rng.integers(4, 16))
        z = int(rng.integers(-128, 256))
        base = ref.requantize_one(a, M, sh)
        got = ref.requantize_one(a, M, sh, z, -128, 127)
        assert -128 <= got <= 127
        assert got == clip(base + z, -128, 127)


def test_per_channel_indexing_and_int16_input(ref):
    rng = np.random.default_rng(5)
    outer, ch, inner = 3, 5, 7
    mult = rng.integers(2 ** 30, 2 ** 31, ch).astype(np.int32)
    shift = rng.integers(0, 12, ch).astype(np.int32)
    for dt, lo, hi in ((np.int32, -10 ** 5, 10 ** 5), (np.int16, -32768, 32767)):
        acc = rng.integers(lo, hi, (outer, ch, inner)).astype(dt)
        for out_dtype, z, clo, chi in ((ref.I8, 3, -128, 127), (ref.U8, 128, 0, 255), (ref.I8, 0, -7, 7)):
            rq = ref.Requant(mult, shift, out_dtype=out_dtype, out_zero_point=z, clip_lo=clo, clip_hi=chi)
            got = ref.requantize(acc, rq)
            assert got.dtype == (np.int8 if out_dtype == ref.I8 else np.uint8)
            for o in range(outer):
                for c in range(ch):
                    for i in range(inner):
                        want = clip(exact_nearest(int(acc[o, c, i]), int(mult[c]), int(shift[c])) + z, clo, chi)
                        assert int(got[o, c, i]) == want
    # per-tensor: only entry 0 is used
    rq = ref.Requant(mult[:1], shift[:1], out_dtype=ref.I8)
    acc = rng.integers(-10 ** 5, 10 ** 5, (2, 4, 3)).astype(np.int32)
    got = ref.requantize(acc, rq)
    want = np.vectorize(lambda a: clip(exact_nearest(int(a), int(mult[0]), int(shift[0])), -128, 127))(acc)
    assert np.array_equal(got.astype(np.int64), want)


def test_encode_multiplier_golden_and_accuracy(ref):
    for m, M, sh in read_golden("encode_multiplier.txt"):
        m, M, sh = float(m), int(M), int(sh)
        if M < 0:
            with pytest.raises(ref.RefError):
                ref.encode_multiplier(m)
        else:
            assert ref.encode_multiplier(m) == (M, sh)
    rng = np.random.default_rng(6)
    for _ in range(2000):
        m = float(np.exp(rng.uniform(np.log(2.0 ** -31), np.log(0.999))))
        M, sh = ref.encode_multiplier(m)
        assert 2 ** 30 <= M < 2 ** 31 and 0 <= sh <= 31
        # nearest Q31 value: relative error at most 2^-31
        assert abs(Fraction(M, 2 ** (31 + sh)) - Fraction(m)) <= Fraction(m) / 2 ** 31


def test_bad_arguments_are_rejected(ref):
    acc = np.zeros((1, 2, 3), np.int32)
    with pytest.raises(ref.RefError):
        ref.requantize(acc, ref.Requant([2 ** 30, 2 ** 30], [0, 32]))
    with pytest.raises(ref.RefError):
        ref.requantize(acc, ref.Requant([2 ** 30, 2 ** 30], [0, 1], clip_lo=5, clip_hi=4))


# ---- the second tie rule: nearest integer, halves away from zero

def exact_half_away(acc, M, sh):
    """Nearest integer to acc*M/2^(31+sh), ties away from zero, in exact rationals."""
    q = Fraction(acc * M, 2 ** (31 + sh))
    mag = math.floor(abs(q) + Fraction(1, 2))
    return mag if q >= 0 else -mag


def test_half_away_hand_worked_ties(ref):
    """M = 2^30 is the real multiplier 1/2: acc/2^(1+sh).  Ties: 0.5 -> 1, -0.5 -> -1, 1.5 -> 2,
    -1.5 -> -2, -2.5 -> -3 (toward +infinity they would be 1, 0, 2, -1, -2)."""
    A = ref.ROUND_HALF_AWAY
    for acc, want_away, want_up in ((1, 1, 1), (-1, -1, 0), (3, 2, 2), (-3, -2, -1), (-5, -3, -2), (5, 3, 3),
                                    (2, 1, 1), (-2, -1, -1), (0, 0, 0), (-4, -2, -2)):
        assert ref.requantize_one(acc, 2 ** 30, 0, rounding=A) == want_away
        assert ref.requantize_one(acc, 2 ** 30, 0) == want_up
    # sh = 2: acc / 8; -12 / 8 = -1.5 -> -2 (away), -1 (upward); -11 / 8 = -1.375 -> -1 under both
    assert ref.requantize_one(-12, 2 ** 30, 2, rounding=A) == -2 and ref.requantize_one(-12, 2 ** 30, 2) == -1
    assert ref.requantize_one(-11, 2 ** 30, 2, rounding=A) == -1 and ref.requantize_one(-11, 2 ** 30, 2) == -1
    # zero point and clip act after the rounding
    assert ref.requantize_one(-3, 2 ** 30, 0, 10, -128, 127, A) == 8
    assert ref.requantize_one(-3000, 2 ** 30, 0, 0, -128, 127, A) == -128


def test_half_away_fraction_definition_and_where_the_rules_differ(ref):
    rng = np.random.default_rng(2)
    A = ref.ROUND_HALF_AWAY
    diff = 0
    for M, sh in ((2 ** 30, 0), (2 ** 30, 4), (1717986918, 3), (2 ** 31 - 1, 0), (1288490189, 15), (3 << 29, 1),
                  (2 ** 31 - 1, 31), (2 ** 30, 31)):
        accs = np.concatenate([rng.integers(I32_MIN, I32_MAX, 300), rng.integers(-2000, 2000, 300),
                               [I32_MIN, I32_MAX, 0, -1, 1]])
        for acc in map(int, accs):
            want = exact_half_away(acc, M, sh)
            got = ref.requantize_one(acc, M, sh, rounding=A)
            assert got == want, (acc, M, sh, got, want)
            up = ref.requantize_one(acc, M, sh)
            # the two rules differ exactly on negative ties, and there by one
            tie = (acc * M) % (2 ** (31 + sh)) == 2 ** (30 + sh)
            assert (got != up) == (tie and acc * M < 0), (acc, M, sh)
            if got != up:
                assert got == up - 1
                diff += 1
    assert diff > 20


def test_half_away_is_an_odd_function(ref):
    """round-half-away(-x) = -round-half-away(x): with no zero point and a symmetric clip the
    operator is odd, which ties toward +infinity are not."""
    rng = np.random.default_rng(4)
    A = ref.ROUND_HALF_AWAY
    for M, sh in ((2 ** 30, 3), (1395864371, 7), (2 ** 31 - 1, 0)):
        for acc in map(int, rng.integers(-10 ** 6, 10 ** 6, 400)):
            assert ref.requantize_one(-acc, M, sh, 0, -127, 127, A) == -ref.requantize_one(acc, M, sh, 0, -127, 127, A)
    assert ref.requantize_one(-1, 2 ** 30, 0) != -ref.requantize_one(1, 2 ** 30, 0)


def test_half_away_through_the_tensor_entry_points(ref):
    """requantize, qdense and qconv2d apply the struct's tie rule: products of small integers with
    M = 2^30 are full of ties."""
    rng = np.random.default_rng(8)
    acc = rng.integers(-40, 40, (2, 3, 50)).astype(np.int32)
    mult = np.full(3, 2 ** 30, np.int32)
    shift = np.array([0, 1, 2], np.int32)
    rq = ref.Requant(mult, shift, rounding=ref.ROUND_HALF_AWAY)
    got = ref.requantize(acc, rq)
    want = np.array([[[exact_half_away(int(v), 2 ** 30, int(shift[c])) for v in acc[o, c]] for c in range(3)]
                     for o in range(2)])
    assert np.array_equal(got.astype(np.int64), np.clip(want, -128, 127))
    assert not np.array_equal(got, ref.requantize(acc, ref.Requant(mult, shift)))
    a = rng.integers(-3, 4, (5, 8)).astype(np.int8)
    w = rng.integers(-3, 4, (3, 8)).astype(np.int8)
    raw = ref.qdense(a, 0, w)
    got = ref.qdense(a, 0, w, None, ref.I32, rq)
    want = np.array([[exact_half_away(int(raw[m, n]), 2 ** 30, int(shift[n])) for n in range(3)] for m in range(5)])
    assert np.array_equal(got.astype(np.int64), want)
    with pytest.raises(Exception):
        ref.requantize(acc, ref.Requant(mult, shift, rounding=2))
