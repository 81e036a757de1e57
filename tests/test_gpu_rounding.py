"""The second tie rule of requantize (nearest, halves away from zero) through every operator that
requantizes.  Multipliers of 2^30 and 3 * 2^29 with small shifts make a large share of the results
exact ties, so the two rules really differ on the data; every case also checks that they do."""
import numpy as np
import pytest
import torch

from gpu_util import *  # noqa: F401,F403

pytestmark = pytest.mark.gpu

AWAY = hago.ROUND_HALF_AWAY


def tie_params(rng, n):
    mult = rng.choice(np.array([2 ** 30, 3 * 2 ** 29], np.int64), n).astype(np.int32)
    shift = rng.integers(0, 5, n).astype(np.int32)
    return mult, shift


@pytest.mark.parametrize("shape", [(2, 5, 7), (3, 4, 1024), (2, 24, 3136), (1, 1, 70000), (64, 128, 1)])
@pytest.mark.parametrize("acc_dt", [np.int32, np.int16])
def test_requantize_half_away(shape, acc_dt):
    rng = np.random.default_rng(abs(hash((shape, acc_dt.__name__))) % 2 ** 31)
    acc = rng.integers(-3000, 3000, shape).astype(acc_dt)
    mult, shift = tie_params(rng, shape[1])
    want = ref.requantize(acc, ref_requant(mult, shift, False, 3, rounding=AWAY))
    got = hago.requantize(dev(acc), gpu_requant(mult, shift, False, 3, rounding=AWAY))
    assert_same(host(got), want, f"requantize half away {shape}")
    up = ref.requantize(acc, ref_requant(mult, shift, False, 3))
    assert np.any(up != want) or acc.size < 100
    assert_same(host(hago.requantize(dev(acc), gpu_requant(mult, shift, False, 3))), up, "requantize upward")


@pytest.mark.parametrize("M,N,K", [(64, 128, 256), (600, 528, 448), (300, 70, 37), (4096, 768, 64)])
def test_qdense_half_away(M, N, K):
    rng = np.random.default_rng(M + N + K)
    a = rng.integers(0, 256, (M, K)).astype(np.uint8)
    w = rng.integers(-127, 128, (N, K)).astype(np.int8)
    bias = rng.integers(-5000, 5000, N).astype(np.int32)
    mult, shift = tie_params(rng, N)
    shift += 8
    a_t, w_t = hago.QType(hago.U8, zero_point=121), hago.QType(hago.I8)
    want = ref.qdense(a, 121, w, bias, ref.I32, ref_requant(mult, shift, rounding=AWAY))
    got = hago.qdense(dev(a), a_t, dev(w), w_t, dev(bias), hago.I32, gpu_requant(mult, shift, rounding=AWAY))
    assert_same(host(got), want, "qdense half away")
    up = ref.qdense(a, 121, w, bias, ref.I32, ref_requant(mult, shift))
    assert np.any(up != want)
    assert_same(host(hago.qdense(dev(a), a_t, dev(w), w_t, dev(bias), hago.I32, gpu_requant(mult, shift))), up,
                "qdense upward")
    # int16 accumulation, requantized
    want = ref.qdense(a, 121, w, bias, ref.I16, ref_requant(mult, shift - 6, rounding=AWAY))
    got = hago.qdense(dev(a), a_t, dev(w), w_t, dev(bias), hago.I16, gpu_requant(mult, shift - 6, rounding=AWAY))
    assert_same(host(got), want, "qdense acc16 half away")


CONV = [
    # B C H W O KH KW stride pad groups layout
    (2, 16, 12, 12, 40, 3, 3, (1, 1), (1, 1), 1, "nchw"),
    (2, 16, 12, 12, 40, 3, 3, (1, 1), (1, 1), 1, "nhwc"),
    (1, 3, 9, 7, 5, 3, 3, (2, 2), (1, 1), 1, "nchw"),
    (2, 48, 8, 8, 24, 1, 1, (1, 1), (0, 0), 1, "nchw"),       # the pointwise geometry
    (2, 144, 28, 28, 24, 1, 1, (1, 1), (0, 0), 1, "nchw"),
    (2, 24, 28, 28, 144, 1, 1, (1, 1), (0, 0), 1, "nchw"),    # few input, many output channels
    (2, 24, 56, 56, 24, 3, 3, (1, 1), (1, 1), 24, "nchw"),    # depthwise: the register kernel's geometry
    (1, 5, 17, 31, 5, 3, 3, (1, 1), (1, 1), 5, "nchw"),       # depthwise, width not a multiple of 4
    (1, 4, 9, 9, 4, 3, 3, (2, 2), (0, 0), 4, "nchw"),         # depthwise, strided
    (1, 6, 150, 20, 6, 3, 3, (1, 1), (1, 1), 6, "nhwc"),
    (2, 40, 14, 14, 40, 3, 3, (1, 1), (1, 1), 40, "nchw"),    # depthwise, small planes
    (2, 40, 14, 14, 40, 3, 3, (1, 1), (1, 1), 40, "nhwc"),    # depthwise, channel-last kernel
]


@pytest.mark.parametrize("case", CONV)
def test_qconv2d_half_away(case):
    B, C, H, W, O, KH, KW, stride, pad, groups, layout = case
    rng = np.random.default_rng(abs(hash(case)) % 2 ** 31)
    a = rng.integers(-128, 128, (B, C, H, W)).astype(np.int8)
    w = rng.integers(-127, 128, (O, C // groups, KH, KW)).astype(np.int8)
    bias = rng.integers(-500, 500, O).astype(np.int32)
    mult, shift = tie_params(rng, O)
    shift += 6
    if layout == "nhwc":
        a, w = a.transpose(0, 2, 3, 1), w.transpose(0, 2, 3, 1)
    lay_g, lay_r = (hago.NHWC, ref.NHWC) if layout == "nhwc" else (hago.NCHW, ref.NCHW)
    a_t, w_t = hago.QType(hago.I8, zero_point=-2), hago.QType(hago.I8)
    want = ref.qconv2d(a, -2, w, bias, lay_r, stride, pad, groups, ref.I32, ref_requant(mult, shift, rounding=AWAY))
    got = hago.qconv2d(dev(a), a_t, dev(w), w_t, dev(bias), lay_g, stride, pad, groups, hago.I32,
                       gpu_requant(mult, shift, rounding=AWAY))
    assert_same(host(got), want, f"qconv2d half away {case}")
    up = ref.qconv2d(a, -2, w, bias, lay_r, stride, pad, groups, ref.I32, ref_requant(mult, shift))
    assert np.any(up != want) or want.size < 5000
    got = hago.qconv2d(dev(a), a_t, dev(w), w_t, dev(bias), lay_g, stride, pad, groups, hago.I32,
                       gpu_requant(mult, shift))
    assert_same(host(got), up, f"qconv2d upward {case}")
