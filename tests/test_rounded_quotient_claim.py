"""The claim behind the row kernels' rounded quotient (csrc/elementwise.hip, rounded_quotient):
with rc = RN(1 / s), qt = RN(x * rc), n = rint(qt), d = qt - n, the value n equals rint(RN(x / s))
whenever |d| < RN(0.5 - |qt| * 2^-21), for every binary32 x and every s with 2^-100 <= |s| <= 2^100.
Checked here in numpy's IEEE binary32 arithmetic (no GPU, no oracle): random and adversarial x
(exact ties of the quotient and their neighbours, a few ulps either way) for many scales."""
import numpy as np


def _fast_path(x, s):
    """(n, taken): the fast path's value and where the kernel would take it."""
    with np.errstate(all="ignore"):
        rc = (np.float32(1.0) / s).astype(np.float32)
        qt = (x * rc).astype(np.float32)
        n = np.rint(qt).astype(np.float32)
        d = (qt - n).astype(np.float32)
        thr = (0.5 - np.abs(qt).astype(np.float64) * 2.0 ** -21).astype(np.float32)  # one rounding, as fmaf
        taken = np.abs(d) < thr
    return n, taken


def _check(x, s, what):
    x = x.astype(np.float32)
    s = np.broadcast_to(s.astype(np.float32), x.shape)
    with np.errstate(all="ignore"):
        want = np.rint((x / s).astype(np.float32))
    n, taken = _fast_path(x, s)
    bad = taken & ~((n == want) & (np.signbit(n) == np.signbit(want)))
    assert not bad.any(), (what, x[bad][:5], s[bad][:5], n[bad][:5], want[bad][:5])
    return float(taken.mean())


def _neighbours(v, k):
    """v moved by k ulps (k may be negative)."""
    out = v.astype(np.float32).copy()
    step = np.float32(np.inf) if k > 0 else np.float32(-np.inf)
    for _ in range(abs(k)):
        out = np.nextafter(out, step)
    return out


def test_fast_value_equals_rounded_division_wherever_the_test_passes():
    rng = np.random.default_rng(20260)
    scales = np.concatenate([
        rng.uniform(0.001, 0.1, 40), 2.0 ** rng.uniform(-20, 20, 40), 2.0 ** rng.integers(-30, 30, 10).astype(np.float64),
        [1.0 / 3.0, 0.1, 3.0, 7.0, 1.0, 255.0 / 256.0, 1.9999999, 1.0000001, 2.0 ** -100, 2.0 ** 100,
         1.5 * 2.0 ** -100, 0.75 * 2.0 ** 100, -0.037, -5.0],
    ]).astype(np.float32)
    taken_total = []
    for s in scales:
        # random magnitudes over many binades
        x = (rng.standard_normal(200_000) * 2.0 ** rng.uniform(-12, 22, 200_000)).astype(np.float32) * s
        taken_total.append(_check(x, np.array(s), f"random, s={s}"))
        # exact ties (k + 1/2) * s as nearly as binary32 allows, and their neighbours
        k = rng.integers(-(1 << 21), 1 << 21, 100_000).astype(np.float64)
        k[:2000] = np.arange(-1000, 1000)
        tie = ((k + 0.5) * np.float64(s)).astype(np.float32)
        for ulps in range(-4, 5):
            _check(_neighbours(tie, ulps), np.array(s), f"ties {ulps:+d} ulp, s={s}")
        # whole multiples and tiny / huge / special values
        whole = (k * np.float64(s)).astype(np.float32)
        _check(whole, np.array(s), f"multiples, s={s}")
        special = np.array([0.0, -0.0, 1e-45, -1e-45, 1e-40, 1e-38, -1e-38, 3e38, -3e38, np.inf, -np.inf, np.nan,
                            2.0 ** 20, 2.0 ** 23, 2.0 ** 24, 2.0 ** 25, 0.49999997, 0.5, 0.50000006], np.float32)
        _check(special, np.array(s), f"special, s={s}")
        with np.errstate(all="ignore"):
            scaled = special * s
        _check(scaled, np.array(s), f"special * s, s={s}")
    # the fast path is the common one on ordinary data
    assert np.mean(taken_total) > 0.9


def test_scales_outside_the_range_never_take_the_fast_path():
    """quotient_reciprocal hands out NaN for them; with NaN every comparison of the test is false."""
    x = np.array([0.0, 1.0, -3.5, 1e-40, 3e38, np.inf], np.float32)
    with np.errstate(all="ignore"):
        qt = x * np.float32(np.nan)
        n = np.rint(qt)
        d = qt - n
        thr = (0.5 - np.abs(qt).astype(np.float64) * 2.0 ** -21).astype(np.float32)
        assert not (np.abs(d) < thr).any()


def test_reciprocal_division_of_job_indices():
    """The row kernels divide 32-bit job indices by the segment and channel counts with the host's
    floor(2^32 / d) (0xffffffff for d = 1), a multiply-high and two conditional corrections
    (csrc/elementwise.hip, div32): exact for every 32-bit n and d >= 1."""
    rng = np.random.default_rng(5)
    d = np.concatenate([np.array([1, 2, 3, 5, 7, 144, 255, 256, 257, 65535, 65536, 65537, 1000003, 2 ** 31 - 1, 2 ** 31,
                                  2 ** 32 - 2, 2 ** 32 - 1], np.uint64),
                        (rng.integers(1, 2 ** 32, 3000, dtype=np.uint64) >> rng.integers(0, 31, 3000).astype(np.uint64)) | np.uint64(1)])
    for dd in d:
        dd = int(dd)
        inv = 0xffffffff if dd <= 1 else (1 << 32) // dd
        n = np.concatenate([rng.integers(0, 2 ** 32, 2000, dtype=np.uint64),
                            np.uint64(2 ** 32 - 1) - rng.integers(0, 1000, 200, dtype=np.uint64),
                            (rng.integers(0, 2 ** 32 // dd + 1, 500, dtype=np.uint64) * np.uint64(dd)
                             + np.uint64(dd - 1)) % np.uint64(2 ** 32)])
        q = (n * np.uint64(inv)) >> np.uint64(32)
        r = n - q * np.uint64(dd)
        for _ in range(2):
            fix = r >= np.uint64(dd)
            q = q + fix.astype(np.uint64)
            r = r - fix.astype(np.uint64) * np.uint64(dd)
        assert np.array_equal(q, n // np.uint64(dd)) and np.array_equal(r, n % np.uint64(dd)), dd
