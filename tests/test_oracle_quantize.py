"""Pins for the oracle's quantize and dequantize (the two operators with which the realized
graph of Sec. 6.1 enters and leaves the integer domain; Eq. 3 split in its two halves).

Pins: hand-worked codes, exact rational arithmetic, numpy's own binary32 division and rounding,
the correctly rounded product for dequantize, and the identity that ties both to the separately
pinned simulated_quantize: dequantize(quantize(x)) == simulated_quantize(x) bit for bit.
"""
from fractions import Fraction

import numpy as np

from conftest import read_golden


def test_golden_codes(ref):
    rows = read_golden("quantize_codes.txt")
    assert len(rows) >= 19
    for x, s, z, lo, hi, want in rows:
        got = ref.quantize(np.float32(x).reshape(1, 1, 1), [np.float32(s)], [int(z)], int(lo), int(hi))
        assert int(got.reshape(-1)[0]) == int(want), (x, s, z, got, want)


def test_codes_against_exact_rationals_and_numpy(ref):
    rng = np.random.default_rng(5)
    for s, z, lo, hi in ((0.0123, 0, -128, 127), (0.031, 128, 0, 255), (0.11, 0, -8, 7),
                         (1e-3, 3, -32, 31), (3.3e-5, -7, -128, 127), (0.5, 1000, -32768, 32767)):
        s32 = np.float32(s)
        x = (rng.standard_normal(2000) * 1.5).astype(np.float32)
        got = ref.quantize(x.reshape(1, 1, -1), [s32], [z], lo, hi).reshape(-1)
        # numpy: IEEE binary32 division, rint = round half to even
        t = x / s32
        assert t.dtype == np.float32
        want = np.clip(np.rint(t).astype(np.int64) + z, lo, hi)
        assert np.array_equal(got, want)
        # exact rationals wherever the quotient is not within one binary32 rounding of a tie
        for xi, gi in zip(x[:300], got[:300]):
            q = Fraction(float(xi)) / Fraction(float(s32))
            frac = abs(q - round(q))
            if abs(frac - Fraction(1, 2)) > Fraction(1, 10 ** 4):
                assert gi == min(max(round(q) + z, lo), hi)


def test_special_values(ref):
    x = np.array([np.nan, np.inf, -np.inf, -0.0, 0.0, 3e38, -3e38], np.float32).reshape(1, 1, -1)
    got = ref.quantize(x, [np.float32(0.1)], [5], -20, 100).reshape(-1)
    assert got.tolist() == [5, 100, -20, 5, 5, 100, -20]   # NaN -> the code of real zero
    got = ref.quantize(x, [np.float32(0.1)], [500], -20, 100).reshape(-1)
    assert got[0] == 100                                    # ... clipped like any other code


def test_dequantize_is_the_correctly_rounded_product(ref):
    rng = np.random.default_rng(6)
    for s, z in ((0.0123, 0), (0.031, 128), (3.3e-5, -7), (0.25, 0), (7.5, 12345)):
        s32 = np.float32(s)
        q = rng.integers(-40000, 40000, 3000).astype(np.int32)
        got = ref.dequantize(q.reshape(1, 1, -1), [s32], [z]).reshape(-1)
        # (q - z) is an exact small integer; its product with a binary32 number is exact in
        # binary64 (24 + 24 bits), so one rounding to binary32 gives the correctly rounded product
        want = ((q.astype(np.int64) - z).astype(np.float64) * np.float64(s32)).astype(np.float32)
        assert got.tobytes() == want.tobytes()
    assert ref.dequantize(np.array([[[7]]], np.int32), [np.float32(0.5)], [7]).tobytes() == np.float32(0.0).tobytes()


def test_dequantize_of_quantize_is_simulated_quantize(ref):
    rng = np.random.default_rng(7)
    x = (rng.standard_normal((3, 5, 400)) * rng.uniform(0.1, 30, (1, 5, 1))).astype(np.float32)
    x.reshape(-1)[:6] = [np.inf, -np.inf, 0.0, -0.0, 1e30, -1e30]
    scale = rng.uniform(0.01, 0.3, 5).astype(np.float32)
    for z, lo, hi in ((np.zeros(5, np.int32), -128, 127), (np.full(5, 128, np.int32), 0, 255),
                      (rng.integers(-5, 6, 5).astype(np.int32), -8, 7)):
        q = ref.quantize(x, scale, z, lo, hi)
        assert q.min() >= lo and q.max() <= hi
        y = ref.dequantize(q, scale, z)
        assert y.tobytes() == ref.simquant(x, scale, z, lo, hi).tobytes()
    # per-tensor parameters
    q = ref.quantize(x, scale[:1], [3], -128, 127)
    assert ref.dequantize(q, scale[:1], [3]).tobytes() == ref.simquant(x, scale[:1], [3], -128, 127).tobytes()


def test_monotone_and_idempotent_codes(ref):
    x = np.sort(np.random.default_rng(8).standard_normal(5000).astype(np.float32)).reshape(1, 1, -1)
    q = ref.quantize(x, [np.float32(0.02)], [3], -128, 127).reshape(-1)
    assert np.all(np.diff(q) >= 0)
    y = ref.dequantize(q.reshape(1, 1, -1), [np.float32(0.02)], [3])
    assert np.array_equal(ref.quantize(y, [np.float32(0.02)], [3], -128, 127).reshape(-1), q)


def test_simquant_codes_pair(ref):
    """The variant of simulated_quantize that also emits its codes: on the hand-worked vectors the
    codes are the golden ones, and y is q * s recomputed here in exact arithmetic (NaN aside)."""
    rows = read_golden("quantize_codes.txt")
    for x, s, z, lo, hi, want in rows:
        y, q = ref.simquant_codes(np.float32(x).reshape(1, 1, 1), [np.float32(s)], [int(z)], int(lo), int(hi))
        assert int(q.reshape(-1)[0]) == int(want)
        exact = np.float32(float(Fraction(int(want) - int(z)) * Fraction(float(np.float32(s)))))
        assert y.reshape(-1)[0].tobytes() == exact.tobytes(), (x, s, z, y, exact)
    x = np.array([np.nan, 1.0, -np.inf], np.float32).reshape(1, 1, -1)
    y, q = ref.simquant_codes(x, [np.float32(0.5)], [3], -8, 7)
    assert np.isnan(y.reshape(-1)[0]) and q.reshape(-1).tolist() == [3, 5, -8]
    assert y.reshape(-1)[1:].tolist() == [1.0, -5.5]
