"""Pins for the oracle's variant operators: shift-only requantize for power-of-two scales (Sec. 5.1),
int16 x int16 -> int32 operands (Sec. 1, Sec. 4.1), 24-bit accumulation (Sec. 4.1) and
simulated_quantize with the overflow of the simulated integer type (Sec. 5.2).  Each is pinned to
hand-worked vectors, exact big-integer / rational arithmetic, and the special cases in which it
reduces to an operator that is already pinned."""
import math
from fractions import Fraction

import numpy as np
import pytest

from conftest import read_golden


# ---------------------------------------------------------------- shift-only requantize
def _exact_round(v, rounding):
    if rounding == 0:
        return math.floor(v + Fraction(1, 2))
    m = math.floor(abs(v) + Fraction(1, 2))
    return -m if v < 0 else m


def test_requantize_shift_hand_worked_vectors(ref):
    for acc, sh, rd, want in read_golden("requantize_shift_vectors.txt"):
        assert ref.requantize_shift_one(int(acc), int(sh), rounding=int(rd)) == int(want), (acc, sh, rd)


def test_requantize_shift_is_the_exact_rounded_quotient(ref):
    rng = np.random.default_rng(5)
    accs = list(range(-300, 301)) + [int(v) for v in rng.integers(-2 ** 31, 2 ** 31, 3000)] + \
        [2 ** 31 - 1, -2 ** 31, 2 ** 30, -2 ** 30, 2 ** 30 - 1, -2 ** 30 + 1]
    for sh in (0, 1, 2, 3, 7, 15, 16, 30, 31):
        for rd in (0, 1):
            for acc in accs:
                want = _exact_round(Fraction(acc, 2 ** sh), rd)
                assert ref.requantize_shift_one(acc, sh, rounding=rd) == want, (acc, sh, rd)


def test_requantize_shift_equals_the_general_operator_with_multiplier_one_half(ref):
    """acc * 2^30 / 2^(31 + sh) = acc / 2^(sh + 1): for shifts >= 1 the shift-only form is the general
    requantize (pinned elsewhere) with multiplier 2^30 and shift one less."""
    rng = np.random.default_rng(6)
    for acc in [int(v) for v in rng.integers(-2 ** 31, 2 ** 31, 2000)] + [2 ** 31 - 1, -2 ** 31]:
        for sh in (1, 2, 9, 31):
            for rd in (0, 1):
                assert ref.requantize_shift_one(acc, sh, rounding=rd) == ref.requantize_one(acc, 2 ** 30, sh - 1, rounding=rd)


def test_requantize_shift_zero_point_and_clip(ref):
    assert ref.requantize_shift_one(1000, 3, z_out=10, lo=-128, hi=127) == 127      # 125 + 10 saturates
    assert ref.requantize_shift_one(800, 3, z_out=10, lo=-128, hi=127) == 110
    assert ref.requantize_shift_one(-5000, 3, z_out=-3, lo=-128, hi=127) == -128
    assert ref.requantize_shift_one(-40, 3, z_out=128, lo=0, hi=255) == 123          # -5 + 128
    # through the array entry points: multiplier None selects the shift-only form per channel
    acc = np.array([[[5, -5, 96], [-96, 7, 1000]]], np.int32)
    rq = ref.Requant(None, np.array([1, 6], np.int32), clip_lo=-128, clip_hi=127)
    assert ref.requantize(acc, rq).tolist() == [[[3, -2, 48], [-1, 0, 16]]]
    rq = ref.Requant(None, np.array([1, 6], np.int32), clip_lo=-128, clip_hi=127, rounding=ref.ROUND_HALF_AWAY)
    assert ref.requantize(acc, rq).tolist() == [[[3, -3, 48], [-2, 0, 16]]]
    a = np.array([[3, 4], [5, 6]], np.int8)
    w = np.array([[1, 1], [2, -1]], np.int8)
    rq = ref.Requant(None, np.array([1, 0], np.int32))
    assert ref.qdense(a, 0, w, None, ref.I32, rq).tolist() == [[4, 2], [6, 4]]       # (7, 2) -> 3.5 -> 4 | 2; (11, 4) -> 5.5 -> 6 | 4


# ---------------------------------------------------------------- 24-bit accumulation
def _wrap(v, bits):
    v %= 1 << bits
    return v - (1 << bits) if v >= 1 << (bits - 1) else v


def test_acc24_hand_worked_wraps(ref):
    for K, A, Wt, exact, want in read_golden("acc24_wraps.txt"):
        K, A, Wt, exact, want = int(K), int(A), int(Wt), int(exact), int(want)
        a = np.full((1, K), A, np.int8)
        w = np.full((1, K), Wt, np.int8)
        got = ref.qdense(a, 0, w, None, ref.I24)
        assert got.dtype == np.int32 and int(got[0, 0]) == want, (K, A, Wt, got)


def test_acc24_is_the_low_24_bits_of_the_int32_sum(ref):
    rng = np.random.default_rng(24)
    a = rng.integers(-128, 128, (9, 2500)).astype(np.int8)
    w = np.where(rng.random((7, 2500)) < 0.8, 127, rng.integers(-127, 128, (7, 2500))).astype(np.int8)
    a[:3] = np.where(rng.random((3, 2500)) < 0.9, 127, a[:3])       # rows that do wrap
    bias = rng.integers(-2 ** 23, 2 ** 23, 7).astype(np.int32)
    acc32 = ref.qdense(a, 3, w, bias, ref.I32).astype(np.int64)
    acc24 = ref.qdense(a, 3, w, bias, ref.I24)
    want = np.vectorize(lambda v: _wrap(int(v), 24))(acc32)
    assert np.array_equal(acc24, want) and (np.abs(acc32) >= 2 ** 23).any() and (np.abs(acc32) < 2 ** 23).any()
    # conv too, and the requantize that follows takes the wrapped value
    x = rng.integers(0, 256, (1, 64, 6, 6)).astype(np.uint8)
    k = np.full((3, 64, 3, 3), 127, np.int8)
    c32 = ref.qconv2d(x, 0, k, None, ref.NCHW, (1, 1), (1, 1), 1, ref.I32).astype(np.int64)
    c24 = ref.qconv2d(x, 0, k, None, ref.NCHW, (1, 1), (1, 1), 1, ref.I24)
    assert np.array_equal(c24, np.vectorize(lambda v: _wrap(int(v), 24))(c32)) and (c32 >= 2 ** 23).any()
    rq = ref.Requant(np.full(3, 2 ** 30, np.int32), np.full(3, 15, np.int32))
    got = ref.qconv2d(x, 0, k, None, ref.NCHW, (1, 1), (1, 1), 1, ref.I24, rq)
    assert np.array_equal(got, ref.requantize(c24.reshape(1, 3, 36), rq).reshape(got.shape))


def test_acc_safe_bound_against_enumeration(ref):
    for bits, amax, wmax in ((24, 127, 127), (24, 128, 128), (16, 15, 7), (16, 8, 8), (32, 128, 128), (24, 32767, 32767)):
        limit = 2 ** (bits - 1) - 1
        kmax = limit // (amax * wmax)
        assert ref.acc_safe(kmax, amax, wmax, bits) or kmax == 0
        assert not ref.acc_safe(kmax + 1, amax, wmax, bits)
    assert ref.acc_safe(520, 127, 127, 24) and not ref.acc_safe(521, 127, 127, 24)
    assert ref.acc_safe(312, 15, 7, 16) == ref.acc16_safe(312, 15, 7) and not ref.acc_safe(313, 15, 7, 16)
    assert ref.acc_safe(0, 10 ** 6, 10 ** 6, 16) and not ref.acc_safe(5, 3, 3, 20)    # unknown width


# ---------------------------------------------------------------- int16 x int16 -> int32
def _py_dense(a, za, w, bias, bits=32):
    M, K = a.shape
    out = np.empty((M, w.shape[0]), np.int64)
    for m in range(M):
        for n in range(w.shape[0]):
            s = int(bias[n]) if bias is not None else 0
            for k in range(K):
                s += (int(a[m, k]) - za) * int(w[n, k])
            out[m, n] = _wrap(s, bits)
    return out


def test_int16_operands_brute_force_with_python_integers(ref):
    rng = np.random.default_rng(16)
    a = rng.integers(-32768, 32768, (5, 23)).astype(np.int16)
    w = rng.integers(-32768, 32768, (4, 23)).astype(np.int16)
    a[0], w[0] = -32768, -32768            # 23 * 2^30 wraps an int32
    a[1], w[1] = 32767, -32768
    bias = np.array([2 ** 31 - 1, -2 ** 31, 5, -7], np.int32)
    for za in (0, -11, 300):
        got = ref.qdense(a, za, w, bias, ref.I32)
        assert got.dtype == np.int32 and np.array_equal(got, _py_dense(a, za, w, bias))
    assert np.array_equal(ref.qdense(a, 0, w, bias, ref.I24), _py_dense(a, 0, w, bias, 24))
    with pytest.raises(ref.RefError):       # the paper's triples: int16 operands accumulate in 32 bits
        ref.qdense(a, 0, w, bias, ref.I16)
    with pytest.raises(ref.RefError):       # both operands int16, or neither
        ref.qdense(a.astype(np.int8), 0, w, bias, ref.I32)


def test_int16_operands_against_float64_and_the_int8_path(ref):
    rng = np.random.default_rng(17)
    a = rng.integers(-2000, 2000, (12, 300)).astype(np.int16)
    w = rng.integers(-2000, 2000, (10, 300)).astype(np.int16)
    want = (a.astype(np.float64) - 5.0) @ w.astype(np.float64).T          # |sum| < 2^31: exact, no wrap
    assert np.array_equal(ref.qdense(a, 5, w).astype(np.float64), want)
    # values that fit int8 give the int8 operator's result, dense and conv, requantized or not
    a8 = rng.integers(-128, 128, (2, 6, 7, 5)).astype(np.int8)
    w8 = rng.integers(-127, 128, (4, 6, 3, 3)).astype(np.int8)
    mult = rng.integers(2 ** 30, 2 ** 31, 4).astype(np.int32)
    rq = ref.Requant(mult, np.full(4, 9, np.int32))
    for layout, tr in ((ref.NCHW, (0, 1, 2, 3)), (ref.NHWC, (0, 2, 3, 1))):
        x, k = np.ascontiguousarray(a8.transpose(tr)), np.ascontiguousarray(w8.transpose(tr))
        for r in (None, rq):
            assert np.array_equal(ref.qconv2d(x.astype(np.int16), -3, k.astype(np.int16), None, layout, (2, 1), (1, 1), 1, ref.I32, r),
                                  ref.qconv2d(x, -3, k, None, layout, (2, 1), (1, 1), 1, ref.I32, r))
    # conv == im2col + dense for int16 operands too
    x = rng.integers(-32768, 32768, (1, 3, 5, 6)).astype(np.int16)
    k = rng.integers(-32768, 32768, (2, 3, 3, 3)).astype(np.int16)
    conv = ref.qconv2d(x, 0, k, None, ref.NCHW, (1, 1), (0, 0), 1)
    cols = np.stack([x[0, :, y:y + 3, c:c + 3].reshape(-1) for y in range(3) for c in range(4)])
    assert np.array_equal(conv[0].reshape(2, -1).T, ref.qdense(cols, 0, k.reshape(2, -1)))


# ---------------------------------------------------------------- overflow-simulating simulated_quantize
def test_simquant_wrap_hand_worked_vectors(ref):
    for s, z, bits, signed, lo, hi, x, y in read_golden("simquant_wrap_vectors.txt"):
        got = ref.simquant_wrap(np.array([[[float(x)]]], np.float32), [float(s)], [int(z)], int(bits), int(signed),
                                int(lo), int(hi))[0, 0, 0]
        if y == "nan":
            assert np.isnan(got), (x, got)
        else:
            assert got == np.float32(float(y)) and not (got == 0 and np.signbit(got)), (s, z, bits, signed, x, got, y)


def test_simquant_wrap_without_overflow_is_simulated_quantize(ref):
    """Codes inside the simulated type's range are untouched: bit-for-bit the plain operator."""
    rng = np.random.default_rng(52)
    x = (rng.standard_normal((2, 3, 500)) * 40).astype(np.float32)
    x[0, 0, :6] = [np.nan, 0.0, -0.0, 0.5, -0.5, 1e-30]
    s = np.array([0.25, 0.5, 1.0], np.float32)
    z = np.array([0, 3, -7], np.int32)
    for bits, lo, hi in ((16, -128, 127), (16, -32768, 32767), (24, -8, 7), (32, -128, 127)):
        a = ref.simquant_wrap(x, s, z, bits, True, lo, hi)
        b = ref.simquant(x, s, z, lo, hi)
        assert a.tobytes() == b.tobytes() or np.array_equal(a.view(np.uint32)[~np.isnan(b)], b.view(np.uint32)[~np.isnan(b)])
        assert np.isnan(a[0, 0, 0])


def test_simquant_wrap_against_exact_integers(ref):
    rng = np.random.default_rng(53)
    x = rng.integers(-400000, 400000, 4000).astype(np.float32).reshape(1, 2, -1)   # integers: x / 1 is exact
    z = np.array([0, 100], np.int32)
    for bits, signed in ((16, True), (8, True), (8, False), (12, False), (20, True)):
        lo, hi = (-(1 << (bits - 1)), (1 << (bits - 1)) - 1) if signed else (0, (1 << bits) - 1)
        got = ref.simquant_wrap(x, [1.0, 1.0], z, bits, signed, lo, hi)
        for c in range(2):
            for xv, gv in zip(x[0, c], got[0, c]):
                code = (int(xv) + int(z[c])) % (1 << bits)
                if signed and code >= 1 << (bits - 1):
                    code -= 1 << bits
                assert int(gv) == code - int(z[c]), (bits, signed, xv, gv)
    # periodic in the real value with period 2^bits * s
    base = rng.integers(-1000, 1000, 200).astype(np.float32).reshape(1, 1, -1)
    y0 = ref.simquant_wrap(base * 0.5, [0.5], [0], 10, True, -512, 511)
    y1 = ref.simquant_wrap(base * 0.5 + 512.0 * 3, [0.5], [0], 10, True, -512, 511)
    assert np.array_equal(y0, y1)
