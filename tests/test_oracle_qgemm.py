"""Pins for the oracle's quantized dense / conv2d / depthwise and the int16
accumulation mode (Introduction: u8 x i8 -> i32 and i8 x i8 -> i16 operand
triples; Sec. 6.2: conv2d and dense on the integer fast path).

Pins: brute force in float64 / Python integers on tiny shapes, a library
cross-check (torch conv2d / matmul in float64, exact below 2^53), closed forms
for constant tensors and delta kernels, and equivalences between operators.
"""
import itertools

import numpy as np
import pytest
import torch

from conftest import read_golden


def rnd_act(rng, shape, dtype):
    if dtype == np.uint8:
        return rng.integers(0, 256, shape).astype(np.uint8)
    return rng.integers(-128, 128, shape).astype(np.int8)


def rnd_w(rng, shape):
    return rng.integers(-127, 128, shape).astype(np.int8)


def brute_dense(a, za, w, bias):
    M, K = a.shape
    N = w.shape[0]
    out = np.zeros((M, N), dtype=object)
    for m in range(M):
        for n in range(N):
            s = int(bias[n]) if bias is not None else 0
            for k in range(K):
                s += (int(a[m, k]) - za) * int(w[n, k])
            out[m, n] = s
    return out.astype(np.int64)


def brute_conv_nchw(a, za, w, bias, stride, pad, groups):
    B, C, H, W = a.shape
    O, Cg, KH, KW = w.shape
    OH = (H + 2 * pad[0] - KH) // stride[0] + 1
    OW = (W + 2 * pad[1] - KW) // stride[1] + 1
    Og = O // groups
    # pad with the zero point so that padded taps contribute (z - z) * w = 0
    ap = np.full((B, C, H + 2 * pad[0], W + 2 * pad[1]), za, dtype=np.int64)
    ap[:, :, pad[0]:pad[0] + H, pad[1]:pad[1] + W] = a
    out = np.zeros((B, O, OH, OW), dtype=np.int64)
    for b, o, y, x in itertools.product(range(B), range(O), range(OH), range(OW)):
        g = o // Og
        patch = ap[b, g * Cg:(g + 1) * Cg, y * stride[0]:y * stride[0] + KH, x * stride[1]:x * stride[1] + KW]
        out[b, o, y, x] = int(((patch - za) * w[o].astype(np.int64)).sum()) + (int(bias[o]) if bias is not None else 0)
    return out


@pytest.mark.parametrize("adt", [np.uint8, np.int8])
def test_dense_brute_force(ref, adt):
    rng = np.random.default_rng(21)
    for (M, N, K), za in (((3, 4, 5), 0), ((5, 2, 17), 128 if adt == np.uint8 else -3), ((1, 1, 1), 7), ((2, 3, 0), 1)):
        a, w = rnd_act(rng, (M, K), adt), rnd_w(rng, (N, K))
        bias = rng.integers(-1000, 1000, N).astype(np.int32)
        got = ref.qdense(a, za, w, bias)
        assert np.array_equal(got.astype(np.int64), brute_dense(a, za, w, bias))
        got = ref.qdense(a, za, w, None)
        assert np.array_equal(got.astype(np.int64), brute_dense(a, za, w, None))


def test_dense_vs_float64_matmul_and_zero_point_identity(ref):
    rng = np.random.default_rng(22)
    a, w = rnd_act(rng, (33, 300), np.uint8), rnd_w(rng, (19, 300))
    za = 117
    got = ref.qdense(a, za, w).astype(np.int64)
    want = torch.from_numpy(a.astype(np.float64) - za) @ torch.from_numpy(w.astype(np.float64)).T
    assert np.array_equal(got, want.numpy().astype(np.int64))
    # sum (a - z) w = sum a w - z sum w
    raw = ref.qdense(a, 0, w).astype(np.int64)
    assert np.array_equal(got, raw - za * w.astype(np.int64).sum(axis=1)[None, :])
    # transposed-operand mistake would show: N != M and w indexed [n, k]
    assert got.shape == (33, 19)


CONV_CASES = [
    # B C H W O KH KW stride pad groups
    (1, 3, 5, 6, 4, 3, 3, (1, 1), (1, 1), 1),
    (2, 4, 7, 5, 6, 3, 3, (2, 2), (1, 1), 1),
    (1, 2, 6, 6, 3, 1, 1, (1, 1), (0, 0), 1),
    (1, 3, 8, 7, 2, 3, 2, (1, 2), (0, 1), 1),
    (2, 5, 6, 7, 5, 3, 3, (1, 1), (1, 1), 5),   # depthwise
    (1, 4, 9, 9, 4, 3, 3, (2, 2), (0, 0), 4),   # depthwise, stride 2, no pad
    (1, 4, 5, 5, 6, 3, 3, (1, 1), (1, 1), 2),   # grouped
    (1, 2, 4, 4, 2, 5, 5, (1, 1), (2, 2), 1),   # kernel larger than the image
]


@pytest.mark.parametrize("case", CONV_CASES)
@pytest.mark.parametrize("adt,za", [(np.uint8, 128), (np.uint8, 0), (np.int8, 0), (np.int8, -5)])
def test_conv_brute_force_and_torch(ref, case, adt, za):
    B, C, H, W, O, KH, KW, stride, pad, groups = case
    rng = np.random.default_rng(hash(case) % 2 ** 31)
    a = rnd_act(rng, (B, C, H, W), adt)
    w = rnd_w(rng, (O, C // groups, KH, KW))
    bias = rng.integers(-5000, 5000, O).astype(np.int32)
    got = ref.qconv2d(a, za, w, bias, ref.NCHW, stride, pad, groups).astype(np.int64)
    assert np.array_equal(got, brute_conv_nchw(a, za, w, bias, stride, pad, groups))
    # library cross-check: float64 conv on (a - z) with zero padding
    t = torch.nn.functional.conv2d(torch.from_numpy(a.astype(np.float64) - za),
                                   torch.from_numpy(w.astype(np.float64)),
                                   torch.from_numpy(bias.astype(np.float64)),
                                   stride=stride, padding=pad, groups=groups)
    assert np.array_equal(got, t.numpy().astype(np.int64))
    # NHWC / OHWI computes the same numbers
    got_nhwc = ref.qconv2d(np.ascontiguousarray(a.transpose(0, 2, 3, 1)), za,
                           np.ascontiguousarray(w.transpose(0, 2, 3, 1)), bias, ref.NHWC, stride, pad, groups)
    assert np.array_equal(got_nhwc.transpose(0, 3, 1, 2).astype(np.int64), got)


def test_conv_closed_forms(ref):
    # constant tensors: acc = (#in-bounds taps) * C * (a - z) * w
    C, H, W = 3, 6, 7
    a = np.full((1, C, H, W), 200, np.uint8)
    w = np.full((2, C, 3, 3), -5, np.int8)
    got = ref.qconv2d(a, 128, w, None, ref.NCHW, (1, 1), (1, 1), 1)
    per_tap = (200 - 128) * -5 * C
    assert got[0, 0, 0, 0] == 4 * per_tap and got[0, 1, H - 1, W - 1] == 4 * per_tap   # corners
    assert got[0, 0, 0, 3] == 6 * per_tap and got[0, 0, 2, 0] == 6 * per_tap           # edges
    assert got[0, 0, 2, 3] == 9 * per_tap                                              # interior
    # delta kernel: output = input - z
    rng = np.random.default_rng(23)
    a = rnd_act(rng, (2, 1, 5, 5), np.uint8)
    w = np.zeros((1, 1, 3, 3), np.int8)
    w[0, 0, 1, 1] = 1
    got = ref.qconv2d(a, 77, w, None, ref.NCHW, (1, 1), (1, 1), 1)
    assert np.array_equal(got[:, 0], a[:, 0].astype(np.int32) - 77)
    # off-centre delta shifts (cross-correlation, no kernel flip)
    w[:] = 0
    w[0, 0, 0, 2] = 1   # tap (ky=0, kx=2) reads input[y-1, x+1]
    got = ref.qconv2d(a, 0, w, None, ref.NCHW, (1, 1), (1, 1), 1)
    assert got[0, 0, 2, 2] == a[0, 0, 1, 3]
    # a == z everywhere: acc = bias
    a = np.full((1, 2, 4, 4), 9, np.int8)
    bias = np.array([5, -6, 7], np.int32)
    got = ref.qconv2d(a, 9, rnd_w(rng, (3, 2, 3, 3)), bias, ref.NCHW, (1, 1), (1, 1), 1)
    assert np.array_equal(got, np.broadcast_to(bias[None, :, None, None], got.shape))


def test_conv_equivalences(ref):
    rng = np.random.default_rng(24)
    B, C, H, W, O = 2, 6, 5, 7, 4
    a = rnd_act(rng, (B, C, H, W), np.uint8)
    za = 131
    # 1x1 conv == dense over [B*H*W, C]
    w1 = rnd_w(rng, (O, C, 1, 1))
    conv = ref.qconv2d(a, za, w1, None, ref.NCHW, (1, 1), (0, 0), 1)
    dense = ref.qdense(np.ascontiguousarray(a.transpose(0, 2, 3, 1)).reshape(-1, C), za, w1.reshape(O, C))
    assert np.array_equal(conv.transpose(0, 2, 3, 1).reshape(-1, O), dense)
    # 3x3 conv == explicit im2col (padded with z) + dense
    w3 = rnd_w(rng, (O, C, 3, 3))
    conv = ref.qconv2d(a, za, w3, None, ref.NCHW, (1, 1), (1, 1), 1)
    ap = np.full((B, C, H + 2, W + 2), za, np.uint8)
    ap[:, :, 1:-1, 1:-1] = a
    cols = np.empty((B, H, W, C, 3, 3), np.uint8)
    for ky in range(3):
        for kx in range(3):
            cols[:, :, :, :, ky, kx] = ap[:, :, ky:ky + H, kx:kx + W].transpose(0, 2, 3, 1)
    dense = ref.qdense(cols.reshape(B * H * W, C * 9), za, w3.reshape(O, C * 9))
    assert np.array_equal(conv.transpose(0, 2, 3, 1).reshape(-1, O), dense)
    # depthwise == C independent single-channel convs
    wd = rnd_w(rng, (C, 1, 3, 3))
    dw = ref.qconv2d(a, za, wd, None, ref.NCHW, (1, 1), (1, 1), C)
    for c in range(C):
        one = ref.qconv2d(np.ascontiguousarray(a[:, c:c + 1]), za, wd[c:c + 1], None, ref.NCHW, (1, 1), (1, 1), 1)
        assert np.array_equal(dw[:, c:c + 1], one)


def test_acc16_wraps_golden_and_low_bits(ref):
    for K, A, Wt, exact, want in (map(int, r) for r in read_golden("acc16_wraps.txt")):
        assert K * A * Wt == exact
        assert ((exact + 2 ** 15) % 2 ** 16) - 2 ** 15 == want       # two's complement reduction
        a = np.full((1, K), A, np.int8)
        w = np.full((1, K), Wt, np.int8)
        assert int(ref.qdense(a, 0, w, None, ref.I16)[0, 0]) == want
        assert int(ref.qdense(a, 0, w, None, ref.I32)[0, 0]) == exact
    # conv form of the config-3 adversarial case: 128 channels x 3x3 = 1152 taps
    a = np.full((1, 128, 4, 4), 15, np.int8)
    w = np.full((2, 128, 3, 3), 7, np.int8)
    got = ref.qconv2d(a, 0, w, None, ref.NCHW, (1, 1), (1, 1), 1, ref.I16)
    assert got.dtype == np.int16 and got[0, 0, 1, 1] == -10112
    assert got[0, 0, 0, 0] == 4 * 128 * 105 - 65536  # corner: 53760 wraps too
    # acc16 is the low 16 bits of acc32 on arbitrary data, bias included
    rng = np.random.default_rng(25)
    a, w = rnd_act(rng, (7, 900), np.int8), rnd_w(rng, (5, 900))
    bias = rng.integers(-2 ** 31, 2 ** 31 - 1, 5).astype(np.int32)
    a32 = ref.qdense(a, 3, w, bias, ref.I32)
    a16 = ref.qdense(a, 3, w, bias, ref.I16)
    assert np.array_equal(a16, a32.astype(np.int16))  # numpy's cast keeps the low 16 bits
    assert np.array_equal(a16.astype(np.int64), ((a32.astype(np.int64) + 2 ** 15) % 2 ** 16) - 2 ** 15)


def test_acc16_bound_against_enumeration(ref):
    # the closed-form bound K * Amax * Wmax <= 32767 (Sec. 5.3 motivates
    # effective bits by this overflow) against the largest safe K found by search
    for amax, wmax, kmax in ((8, 8, 511), (7, 7, 668), (15, 7, 312), (32, 32, 31), (128, 128, 1), (255, 127, 1)):
        ks = [k for k in range(0, 1200) if ref.acc16_safe(k, amax, wmax)]
        assert max(ks) == kmax
        # on inputs that satisfy the bound, acc16 == acc32 even for the worst case
        a = np.full((1, kmax), min(amax, 127), np.int8)
        w = np.full((1, kmax), -min(wmax, 127), np.int8)
        assert int(ref.qdense(a, 0, w, None, ref.I16)[0, 0]) == int(ref.qdense(a, 0, w, None, ref.I32)[0, 0])
    assert not ref.acc16_safe(1152, 8, 8)       # 73728 does not fit
    assert not ref.acc16_safe(1152, 15, 7)


def test_int32_wraparound_is_two_complement(ref):
    a = np.full((1, 4), 127, np.int8)
    w = np.full((1, 4), 127, np.int8)
    bias = np.array([2 ** 31 - 1], np.int32)
    got = int(ref.qdense(a, 0, w, bias)[0, 0])
    assert got == ((2 ** 31 - 1 + 4 * 127 * 127 + 2 ** 31) % 2 ** 32) - 2 ** 31


def test_fused_requantize_matches_standalone(ref):
    rng = np.random.default_rng(26)
    a, w = rnd_act(rng, (9, 64), np.uint8), rnd_w(rng, (6, 64))
    mult = rng.integers(2 ** 30, 2 ** 31, 6).astype(np.int32)
    shift = rng.integers(6, 10, 6).astype(np.int32)
    rq = ref.Requant(mult, shift, out_dtype=ref.U8, out_zero_point=10, clip_lo=10, clip_hi=255)
    fused = ref.qdense(a, 128, w, None, ref.I32, rq)
    raw = ref.qdense(a, 128, w)
    assert np.array_equal(fused, ref.requantize(raw.reshape(9, 6, 1), rq).reshape(9, 6))
    assert fused.min() >= 10
    # conv: channel axis is O in NCHW and the last axis in NHWC
    a4 = rnd_act(rng, (2, 3, 5, 5), np.int8)
    w4 = rnd_w(rng, (6, 3, 3, 3))
    rq = ref.Requant(mult, shift, out_dtype=ref.I8)
    fused = ref.qconv2d(a4, 0, w4, None, ref.NCHW, (1, 1), (1, 1), 1, ref.I32, rq)
    raw = ref.qconv2d(a4, 0, w4, None, ref.NCHW, (1, 1), (1, 1), 1)
    assert np.array_equal(fused, ref.requantize(raw.reshape(2, 6, 25), rq).reshape(fused.shape))
    # int16 accumulator then requantize: sign-extended 16-bit value goes in
    fused16 = ref.qconv2d(a4, 0, w4, None, ref.NCHW, (1, 1), (1, 1), 1, ref.I16, rq)
    raw16 = ref.qconv2d(a4, 0, w4, None, ref.NCHW, (1, 1), (1, 1), 1, ref.I16)
    assert np.array_equal(fused16, ref.requantize(raw16.reshape(2, 6, 25), rq).reshape(fused.shape))


def test_bad_arguments(ref):
    a = np.zeros((1, 4, 4, 4), np.int8)
    w = np.zeros((4, 2, 3, 3), np.int8)
    with pytest.raises(ref.RefError):
        ref.qconv2d(a, 0, w, None, ref.NCHW, (1, 1), (1, 1), 3)     # groups does not divide
    with pytest.raises(ref.RefError):
        ref.qconv2d(a, 0, np.zeros((4, 4, 7, 7), np.int8), None, ref.NCHW, (1, 1), (0, 0), 1)  # kernel > image


def test_threaded_helper_equals_the_plain_oracle(ref):
    """qdense_threaded (the timing helper of the benchmark's CPU baseline and of the full-size parity
    test) only slices rows: its result is the plain oracle's, for every thread count, ragged splits
    included."""
    rng = np.random.default_rng(31)
    a = rng.integers(0, 256, (37, 50)).astype(np.uint8)
    w = rng.integers(-127, 128, (19, 50)).astype(np.int8)
    bias = rng.integers(-1000, 1000, 19).astype(np.int32)
    mult = rng.integers(2 ** 30, 2 ** 31, 19).astype(np.int32)
    shift = rng.integers(5, 12, 19).astype(np.int32)
    for rq in (None, ref.Requant(mult, shift)):
        for acc in (ref.I32, ref.I16):
            want = ref.qdense(a, 128, w, bias, acc, rq)
            for threads in (1, 2, 5, 16, 64):
                got = ref.qdense_threaded(a, 128, w, bias, acc, rq, threads=threads)
                assert got.dtype == want.dtype and np.array_equal(got, want), (threads, acc)
