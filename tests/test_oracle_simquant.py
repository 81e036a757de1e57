"""Pins for the oracle's simulated_quantize, scale (Eq. 1) and absmax (Eq. 2).

simulated_quantize is the operator of Sec. 4.2 built on Eq. 3; the pins are
hand-worked binary32 vectors, exact rational arithmetic with a single
rounding per operation, and invariants (idempotence, error bound, monotone).
"""
from fractions import Fraction

import numpy as np
import pytest

from conftest import read_golden


def f32(fr):
    """Correctly rounded binary32 of an exact rational (|fr| within range).

    float(Fraction) is correctly rounded to binary64; for the quotient or the
    product of two binary32 numbers a second rounding to binary32 is
    innocuous (53 >= 2*24 + 2)."""
    return np.float32(float(fr))


def exact_simquant(x, s, z, lo, hi):
    x, s = np.float32(x), np.float32(s)
    if np.isnan(x):
        return np.float32(np.nan)
    if np.isinf(x):
        v = hi if x > 0 else lo
        return f32(Fraction(v - z) * Fraction(float(s)))
    t = f32(Fraction(float(x)) / Fraction(float(s)))
    if np.isinf(t):
        v = hi if t > 0 else lo
        return f32(Fraction(v - z) * Fraction(float(s)))
    u = round(Fraction(float(t)))  # Python rounds exact halves to even
    v = f32(Fraction(u) + z)       # the code, as binary32
    v = Fraction(float(v))
    v = min(max(v, lo), hi)
    return f32((v - z) * Fraction(float(s)))


def run(ref, x, s, z, lo, hi):
    x = np.asarray(x, np.float32).reshape(1, 1, -1)
    return ref.simquant(x, [s], [z], lo, hi).reshape(-1)


def test_golden_vectors(ref):
    rows = read_golden("simquant_vectors.txt")
    assert len(rows) >= 19
    for x, s, z, lo, hi, want in rows:
        x, s, want = np.float32(x), np.float32(s), np.float32(want)
        z, lo, hi = int(z), int(lo), int(hi)
        got = run(ref, [x], s, z, lo, hi)[0]
        assert got.tobytes() == want.tobytes(), (x, s, z, got, want)
        assert exact_simquant(x, s, z, lo, hi).tobytes() == want.tobytes()


def test_exact_rationals_on_random_inputs(ref):
    rng = np.random.default_rng(11)
    for s, z, lo, hi in ((0.0123, 0, -128, 127), (0.031, 128, 0, 255), (0.11, 0, -8, 7),
                         (1e-3, 3, -32, 31), (3.3e-5, -7, -128, 127)):
        x = (rng.standard_normal(1500) * 1.5).astype(np.float32)
        x[:6] = [0.0, -0.0, s * 0.5, -s * 0.5, s * 2.5, 1e30]
        got = run(ref, x, s, z, lo, hi)
        for xi, gi in zip(x, got):
            want = exact_simquant(xi, s, z, lo, hi)
            assert gi.tobytes() == want.tobytes(), (xi, s, z, gi, want)


def test_division_not_reciprocal(ref):
    # Eq. 3 divides.  Find an input where x * (1/s) rounds differently before
    # the integer rounding and check the oracle follows the division.
    s = np.float32(0.0123)
    rng = np.random.default_rng(12)
    x = (rng.standard_normal(200000)).astype(np.float32)
    div = np.rint(x / s)
    rcp = np.rint(x * (np.float32(1) / s))
    idx = np.nonzero(div != rcp)[0]
    if idx.size:  # the two differ on a few ties-adjacent values
        sel = x[idx]
        got = run(ref, sel, s, 0, -2 ** 24, 2 ** 24)
        for xi, gi in zip(sel, got):
            assert gi.tobytes() == exact_simquant(xi, s, 0, -2 ** 24, 2 ** 24).tobytes()


def test_invariants(ref):
    rng = np.random.default_rng(13)
    x = rng.standard_normal(200000).astype(np.float32)
    for s, z, lo, hi in ((np.float32(4.0 / 128), 0, -128, 127), (np.float32(0.02), 120, 0, 255)):
        y = run(ref, x, s, z, lo, hi)
        yy = run(ref, y, s, z, lo, hi)
        assert y.tobytes() == yy.tobytes()                      # idempotent
        assert len(np.unique(y)) <= hi - lo + 1                 # at most one value per code
        inside = (x > (lo - z) * float(s)) & (x < (hi - z) * float(s))
        err = np.abs(y[inside].astype(np.float64) - x[inside].astype(np.float64))
        assert err.max() <= float(s) / 2 * (1 + 1e-6)           # rounding error bound
        order = np.argsort(x, kind="stable")
        assert np.all(np.diff(y[order]) >= 0)                   # monotone
        assert run(ref, [0.0], s, z, lo, hi)[0] == 0.0
        # saturation: far outside the range every value maps to an end code
        assert run(ref, [1e9], s, z, lo, hi)[0] == np.float32((hi - z) * s)
        assert run(ref, [-1e9], s, z, lo, hi)[0] == np.float32((lo - z) * s)


def test_nan_inf_and_signed_zero(ref):
    s = np.float32(0.25)
    y = run(ref, [np.nan, np.inf, -np.inf, -0.0, -0.1], s, 0, -128, 127)
    assert np.isnan(y[0])
    assert y[1] == np.float32(31.75) and y[2] == np.float32(-32.0)
    assert y[3].tobytes() == np.float32(0.0).tobytes()  # +0, never -0
    assert y[4].tobytes() == np.float32(0.0).tobytes()


def test_per_channel_indexing(ref):
    rng = np.random.default_rng(14)
    outer, ch, inner = 3, 4, 5
    x = rng.standard_normal((outer, ch, inner)).astype(np.float32)
    s = np.array([0.01, 0.02, 0.04, 0.08], np.float32)
    z = np.array([0, 5, -3, 100], np.int32)
    y = ref.simquant(x, s, z, -128, 127)
    for c in range(ch):
        want = ref.simquant(np.ascontiguousarray(x[:, c:c + 1, :]), s[c:c + 1], z[c:c + 1], -128, 127)
        assert y[:, c:c + 1, :].tobytes() == want.tobytes()
        for o in range(outer):
            for i in range(inner):
                assert y[o, c, i].tobytes() == exact_simquant(x[o, c, i], s[c], int(z[c]), -128, 127).tobytes()
    # per-tensor
    y = ref.simquant(x, s[:1], z[:1], -128, 127)
    assert y.tobytes() == ref.simquant(x.reshape(1, 1, -1), s[:1], z[:1], -128, 127).tobytes()


def test_scale_eq1_and_absmax_eq2(ref):
    # Eq. 1: s = threshold / 2^(bit - sign)
    assert ref.scale(4.0, 8, 1) == 4.0 / 128
    assert ref.scale(1.0, 4, 1) == 0.125
    assert ref.scale(6.0, 8, 0) == 6.0 / 256
    assert ref.scale(3.0, 6, 1) == 3.0 / 32
    # Eq. 2 against numpy's own reduction
    rng = np.random.default_rng(15)
    x = rng.standard_normal((4, 6, 50)).astype(np.float32)
    assert np.array_equal(ref.absmax(x, True), np.abs(x).max(axis=(0, 2)))
    assert ref.absmax(x, False)[0] == np.abs(x).max()
    assert ref.bit_range(8, True) == (-128, 127)
    assert ref.bit_range(4, True) == (-8, 7)
    assert ref.bit_range(4, False) == (0, 15)
    assert ref.bit_range(8, False) == (0, 255)
    with pytest.raises(ref.RefError):
        ref.bit_range(0, True)


def test_batched_candidates_on_the_worked_vectors(ref):
    # Sec. 6.3: several candidate parameter sets over one tensor.  The golden rows with s = 0.25
    # give two candidates (signed with z = 0, unsigned with z = 128) whose expected outputs are
    # the hand-worked ones; this pins the [candidate][...] layout and the parameter indexing.
    rows = read_golden("simquant_vectors.txt")
    cand = {(0, -128, 127): {}, (128, 0, 255): {}}
    for x, s, z, lo, hi, want in rows:
        if float(s) == 0.25 and (int(z), int(lo), int(hi)) in cand:
            cand[(int(z), int(lo), int(hi))][np.float32(x).tobytes()] = np.float32(want)
    xs = sorted(set(cand[(0, -128, 127)]) | set(cand[(128, 0, 255)]))
    x = np.frombuffer(b"".join(xs), np.float32).reshape(1, 1, -1)
    y = ref.simquant_batched(x, [[0.25], [0.25]], [[0], [128]], [-128, 0], [127, 255], per_channel=False)
    assert y.shape == (2, 1, 1, len(xs))
    for b, key in enumerate(((0, -128, 127), (128, 0, 255))):
        for i, xb in enumerate(xs):
            if xb in cand[key]:
                assert y[b, 0, 0, i].tobytes() == cand[key][xb].tobytes()
    # per-channel candidates: channel c of candidate b uses scales[b][c]
    x = np.array([[[0.375], [0.375]]], np.float32)          # [1, 2, 1]
    y = ref.simquant_batched(x, [[0.25, 0.125], [0.5, 0.25]], [[0, 0], [0, 0]], [-128, -128], [127, 127])
    assert y[:, 0, :, 0].tolist() == [[0.5, 0.375], [0.5, 0.5]]   # 1.5->2, 3->3 | 0.75->1, 1.5->2


def test_absmax_ignores_nan_and_handles_infinities(ref):
    """Reading taken where Eq. 2 is silent: a NaN element never wins the comparison `|v| > t`, so
    the threshold is the maximum over the other elements (numpy's nanmax); an infinity wins; the
    result is never -0; an all-NaN or empty reduction gives 0."""
    x = np.array([[[1.5, np.nan, -3.25, 0.0], [np.nan, np.nan, np.nan, np.nan], [-0.0, 0.0, -0.0, 0.0],
                   [2.0, -np.inf, 7.0, np.nan]]], np.float32)
    thr = ref.absmax(x, True)
    assert thr.tolist() == [3.25, 0.0, 0.0, np.inf]
    assert not np.signbit(thr).any()
    want = np.abs(np.where(np.isnan(x), np.float32(0), x)).max(axis=(0, 2))   # the maximum over the non-NaN elements
    assert np.array_equal(thr, want.astype(np.float32))
    assert ref.absmax(x, False).tolist() == [np.inf]
    assert ref.absmax(x[:, :3], False).tolist() == [3.25]
    assert ref.absmax(np.zeros((0, 3, 4), np.float32), True).tolist() == [0.0, 0.0, 0.0]
