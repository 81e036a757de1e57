"""GPU parity (bit-exact) of the operand / accumulator / requantize variants against the oracle:
shift-only requantize for power-of-two scales (Sec. 5.1), int16 x int16 operands (Sec. 1, 4.1),
24-bit accumulation (Sec. 4.1), simulated quantize with overflow (Sec. 5.2)."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

from gpu_util import *  # noqa: E402,F401,F403
from paper_2103_14949_amd import datagen


def _shift_rq_gpu(shift, out_u8=False, z_out=0, clip=None, rounding=0):
    q = hago.QType(hago.U8 if out_u8 else hago.I8, 8, not out_u8, z_out)
    lo, hi = clip if clip is not None else (None, None)
    return hago.Requant(None, dev(np.asarray(shift, np.int32)), q, lo, hi, rounding=rounding)


def _shift_rq_ref(shift, out_u8=False, z_out=0, clip=None, rounding=0):
    lo, hi = clip if clip is not None else ((0, 255) if out_u8 else (-128, 127))
    return ref.Requant(None, shift, out_dtype=ref.U8 if out_u8 else ref.I8, out_zero_point=z_out, clip_lo=lo,
                       clip_hi=hi, rounding=rounding)


# ---------------------------------------------------------------- shift-only requantize
@pytest.mark.parametrize("shape", [(2, 5, 1024), (3, 7, 77), (64, 16, 1), (1, 1, 5000), (2, 12, 1)])
@pytest.mark.parametrize("rounding", [0, 1])
def test_requantize_shift_only(shape, rounding):
    rng = np.random.default_rng(sum(shape) + rounding)
    C = shape[1]
    shift = rng.integers(0, 32, C).astype(np.int32)
    shift[0] = 0
    acc = rng.integers(-2 ** 31, 2 ** 31, shape).astype(np.int32)
    small = rng.integers(-2000, 2000, shape).astype(np.int32)       # ties and unsaturated results
    acc = np.where(rng.random(shape) < 0.5, acc, small << np.minimum(shift, 20)[None, :, None]).astype(np.int32)
    acc.reshape(-1)[:4] = [2 ** 31 - 1, -2 ** 31, 2 ** 30, -2 ** 30]
    for out_u8, z_out in ((False, 0), (True, 131), (False, -7)):
        want = ref.requantize(acc, _shift_rq_ref(shift, out_u8, z_out, rounding=rounding))
        got = hago.requantize(dev(acc), _shift_rq_gpu(shift, out_u8, z_out, rounding=rounding))
        assert_same(host(got), want, f"shift-only requantize {shape} u8={out_u8}")
    a16 = rng.integers(-2 ** 15, 2 ** 15, shape).astype(np.int16)
    s16 = np.minimum(shift, 12)
    want = ref.requantize(a16, _shift_rq_ref(s16, rounding=rounding))
    assert_same(host(hago.requantize(dev(a16), _shift_rq_gpu(s16, rounding=rounding))), want, "int16 input")
    assert len(np.unique(want)) > 10
    # one shift for the whole tensor
    want = ref.requantize(acc, _shift_rq_ref(np.array([9], np.int32), rounding=rounding))
    assert_same(host(hago.requantize(dev(acc), _shift_rq_gpu(np.array([9], np.int32), rounding=rounding))), want, "per tensor")


@pytest.mark.parametrize("tile", [-1, 0, 2, 4])
def test_fused_shift_only_dense_and_conv(tile, stream_tile, conv_entry):
    """The fused epilogues with no multiplier array: every shift from 0 (the identity, which the folded
    arithmetic cannot express) upward, dense (streaming tiles and the general kernel), 3x3 conv,
    pointwise and depthwise."""
    stream_tile(tile)
    rng = np.random.default_rng(700 + tile)
    M, N, K = 300, 144, 192
    a, w = rng.integers(0, 256, (M, K)).astype(np.uint8), rng.integers(-127, 128, (N, K)).astype(np.int8)
    bias = rng.integers(-10 ** 4, 10 ** 4, N).astype(np.int32)
    shift = rng.integers(9, 15, N).astype(np.int32)
    shift[[0, 33, 70]] = 0
    shift[[1, 34, 71]] = 1
    shift[[2, 100]] = 31
    for rounding in (0, 1):
        want = ref.qdense(a, 128, w, bias, ref.I32, _shift_rq_ref(shift, rounding=rounding))
        got = hago.qdense(dev(a), act_qtype(a, 128), dev(w), hago.QType(hago.I8), dev(bias), hago.I32,
                          _shift_rq_gpu(shift, rounding=rounding))
        assert_same(host(got), want, f"dense shift-only tile {tile} rounding {rounding}")
    assert len(np.unique(want)) > 100
    if tile != -1:
        return
    # convolutions: 3x3, pointwise (1x1 NCHW, few output channels) and depthwise
    x = rng.integers(-128, 128, (2, 16, 12, 16)).astype(np.int8)
    for O, k, groups in ((24, 3, 1), (24, 1, 1), (16, 3, 16)):
        wt = rng.integers(-127, 128, (O, 16 // groups, k, k)).astype(np.int8)
        sh = rng.integers(5, 12, O).astype(np.int32)
        sh[:3] = [0, 1, 31]
        b = rng.integers(-1000, 1000, O).astype(np.int32)
        pad = (k // 2, k // 2)
        want = ref.qconv2d(x, -3, wt, b, ref.NCHW, (1, 1), pad, groups, ref.I32, _shift_rq_ref(sh))
        got = qconv2d(dev(x), act_qtype(x, -3), dev(wt), hago.QType(hago.I8), dev(b), hago.NCHW, (1, 1), pad, groups,
                      hago.I32, _shift_rq_gpu(sh))
        assert_same(host(got), want, f"conv shift-only O={O} k={k} groups={groups}")
        xn, wn = np.ascontiguousarray(x.transpose(0, 2, 3, 1)), np.ascontiguousarray(wt.transpose(0, 2, 3, 1))
        want = ref.qconv2d(xn, -3, wn, b, ref.NHWC, (1, 1), pad, groups, ref.I32, _shift_rq_ref(sh))
        got = qconv2d(dev(xn), act_qtype(xn, -3), dev(wn), hago.QType(hago.I8), dev(b), hago.NHWC, (1, 1), pad, groups,
                      hago.I32, _shift_rq_gpu(sh))
        assert_same(host(got), want, f"conv shift-only nhwc O={O} k={k} groups={groups}")


def test_depthwise_config4_shape_shift_only():
    """The register depthwise kernel (56 x 56 planes) with power-of-two scales."""
    rng = np.random.default_rng(44)
    x = rng.integers(-128, 128, (2, 8, 56, 56)).astype(np.int8)
    wt = rng.integers(-127, 128, (8, 1, 3, 3)).astype(np.int8)
    sh = np.array([0, 1, 6, 7, 8, 9, 20, 31], np.int32)
    for stride in ((1, 1), (2, 2)):
        want = ref.qconv2d(x, 0, wt, None, ref.NCHW, stride, (1, 1), 8, ref.I32, _shift_rq_ref(sh))
        got = hago.qconv2d(dev(x), act_qtype(x, 0), dev(wt), hago.QType(hago.I8), None, hago.NCHW, stride, (1, 1), 8,
                           hago.I32, _shift_rq_gpu(sh))
        assert_same(host(got), want, f"depthwise shift-only stride {stride}")


# ---------------------------------------------------------------- 24-bit accumulation
@pytest.mark.parametrize("tile", [-1, 0, 2, 4])
def test_acc24_dense(tile, stream_tile):
    stream_tile(tile)
    rng = np.random.default_rng(2400 + tile)
    M, N, K = 200, 80, 1024
    a = np.where(rng.random((M, K)) < 0.7, 127, rng.integers(-128, 128, (M, K))).astype(np.int8)
    w = np.where(rng.random((N, K)) < 0.7, 127, rng.integers(-127, 128, (N, K))).astype(np.int8)
    a[100:] = rng.integers(-128, 128, (100, K))                      # rows that do not wrap
    bias = rng.integers(-2 ** 22, 2 ** 22, N).astype(np.int32)
    want = ref.qdense(a, 2, w, bias, ref.I24)
    got = hago.qdense(dev(a), act_qtype(a, 2), dev(w), hago.QType(hago.I8), dev(bias), hago.I24)
    assert got.dtype == torch.int32
    assert_same(host(got), want, f"acc24 raw tile {tile}")
    acc32 = ref.qdense(a, 2, w, bias, ref.I32)
    assert (acc32 != want).any() and (acc32 == want).any()           # some sums wrapped, some did not
    mult, shift = datagen.requant_params(rng, np.full(N, 2.0 ** 21), 40.0)
    want = ref.qdense(a, 2, w, bias, ref.I24, ref_requant(mult, shift))
    got = hago.qdense(dev(a), act_qtype(a, 2), dev(w), hago.QType(hago.I8), dev(bias), hago.I24, gpu_requant(mult, shift))
    assert_same(host(got), want, f"acc24 requantized tile {tile}")
    with pytest.raises(hago.HagoError) as e:
        hago.qdense(dev(a), act_qtype(a, 2), dev(w), hago.QType(hago.I8), dev(bias), hago.I24, flags=hago.STRICT_ACC16)
    assert e.value.code == 6


@pytest.mark.parametrize("layout", ["nchw", "nhwc"])
def test_acc24_conv_pointwise_depthwise(layout, conv_entry):
    rng = np.random.default_rng(2450)
    x = rng.integers(0, 256, (2, 64, 10, 12)).astype(np.uint8)
    lay_g, lay_r = (hago.NCHW, ref.NCHW) if layout == "nchw" else (hago.NHWC, ref.NHWC)
    tr = (0, 1, 2, 3) if layout == "nchw" else (0, 2, 3, 1)
    xh = np.ascontiguousarray(x.transpose(tr))
    for O, k, groups in ((40, 3, 1), (24, 1, 1), (64, 3, 64)):
        wt = np.where(rng.random((O, 64 // groups, k, k)) < 0.8, 127, rng.integers(-127, 128, (O, 64 // groups, k, k))).astype(np.int8)
        if groups > 1:
            bias = rng.integers(2 ** 23 - 200000, 2 ** 23 - 1000, O).astype(np.int32)   # depthwise sums are small: start near the edge
        else:
            bias = rng.integers(2 ** 22, 2 ** 23 - 1000, O).astype(np.int32)
        wh = np.ascontiguousarray(wt.transpose(tr))
        pad = (k // 2, k // 2)
        want = ref.qconv2d(xh, 0, wh, bias, lay_r, (1, 1), pad, groups, ref.I24)
        got = qconv2d(dev(xh), act_qtype(xh, 0), dev(wh), hago.QType(hago.I8), dev(bias), lay_g, (1, 1), pad, groups, hago.I24)
        assert_same(host(got), want, f"acc24 conv O={O} k={k} groups={groups} {layout}")
        assert (ref.qconv2d(xh, 0, wh, bias, lay_r, (1, 1), pad, groups, ref.I32) != want).any()
        mult, shift = datagen.requant_params(rng, np.full(O, 2.0 ** 21), 40.0)
        want = ref.qconv2d(xh, 0, wh, bias, lay_r, (1, 1), pad, groups, ref.I24, ref_requant(mult, shift))
        got = qconv2d(dev(xh), act_qtype(xh, 0), dev(wh), hago.QType(hago.I8), dev(bias), lay_g, (1, 1), pad, groups,
                      hago.I24, gpu_requant(mult, shift))
        assert_same(host(got), want, f"acc24 conv requantized O={O} k={k} groups={groups} {layout}")


# ---------------------------------------------------------------- int16 x int16 operands
I16T = None


def _i16(z=0, bits=16):
    return hago.QType(hago.I16, bits, True, z)


@pytest.mark.parametrize("M,N,K", [(1, 1, 1), (5, 7, 3), (64, 64, 32), (130, 70, 100), (77, 200, 264), (300, 65, 31), (9, 9, 0)])
@pytest.mark.parametrize("za", [0, -11, 300])
def test_qdense_int16_operands(M, N, K, za):
    rng = np.random.default_rng(M * 31 + N + K + za)
    a = rng.integers(-32768, 32768, (M, K)).astype(np.int16)
    w = rng.integers(-32768, 32768, (N, K)).astype(np.int16)
    if M > 4 and K > 0:
        a[0], w[0] = -32768, -32768                       # K * 2^30: wraps an int32
        a[1] = 32767
    bias = rng.integers(-2 ** 31, 2 ** 31, N).astype(np.int32)
    want = ref.qdense(a, za, w, bias, ref.I32)
    got = hago.qdense(dev(a), _i16(za), dev(w), _i16(), dev(bias), hago.I32)
    assert_same(host(got), want, f"int16 dense {M}x{N}x{K}")
    assert_same(host(hago.qdense(dev(a), _i16(za), dev(w), _i16(), None, hago.I24)), ref.qdense(a, za, w, None, ref.I24), "int16, 24 bits")
    # realistic magnitudes, requantized: 12-bit operands
    a12 = rng.integers(-2048, 2048, (M, K)).astype(np.int16)
    w12 = rng.integers(-2047, 2048, (N, K)).astype(np.int16)
    mult, shift = datagen.requant_params(rng, np.full(N, 1182.0 * 1182.0 * np.sqrt(max(K, 1))), 40.0)
    for rq_r, rq_g in ((ref_requant(mult, shift), gpu_requant(mult, shift)),
                       (ref_requant(mult, shift, True, 10, rounding=1), gpu_requant(mult, shift, True, 10, rounding=1)),
                       (_shift_rq_ref(shift + 12), _shift_rq_gpu(shift + 12))):
        want = ref.qdense(a12, za, w12, bias // 4096, ref.I32, rq_r)
        got = hago.qdense(dev(a12), _i16(za, 12), dev(w12), _i16(0, 12), dev(bias // 4096), hago.I32, rq_g)
        assert_same(host(got), want, f"int16 dense requantized {M}x{N}x{K}")
    with pytest.raises(hago.HagoError) as e:
        hago.qdense(dev(a), _i16(za), dev(w), _i16(), None, hago.I16)
    assert e.value.code == 3


CONV16 = [
    # B C H W O KH KW stride pad
    (1, 3, 5, 6, 4, 3, 3, (1, 1), (1, 1)),
    (2, 4, 7, 5, 6, 3, 3, (2, 2), (1, 1)),
    (1, 16, 9, 8, 70, 1, 1, (1, 1), (0, 0)),
    (1, 3, 8, 7, 2, 3, 2, (1, 2), (0, 1)),
    (2, 8, 12, 12, 40, 3, 3, (1, 1), (1, 1)),
    (1, 2, 4, 4, 2, 5, 5, (1, 1), (2, 2)),
]


@pytest.mark.parametrize("case", CONV16)
@pytest.mark.parametrize("layout", ["nchw", "nhwc"])
def test_qconv2d_int16_operands(case, layout, conv_entry):
    B, C, H, W, O, KH, KW, stride, pad = case
    rng = np.random.default_rng(abs(hash(case)) % 2 ** 31)
    x = rng.integers(-32768, 32768, (B, C, H, W)).astype(np.int16)
    wt = rng.integers(-32768, 32768, (O, C, KH, KW)).astype(np.int16)
    bias = rng.integers(-10 ** 6, 10 ** 6, O).astype(np.int32)
    lay_g, lay_r = (hago.NCHW, ref.NCHW) if layout == "nchw" else (hago.NHWC, ref.NHWC)
    tr = (0, 1, 2, 3) if layout == "nchw" else (0, 2, 3, 1)
    xh, wh = np.ascontiguousarray(x.transpose(tr)), np.ascontiguousarray(wt.transpose(tr))
    for za in (0, 777):
        want = ref.qconv2d(xh, za, wh, bias, lay_r, stride, pad, 1, ref.I32)
        got = qconv2d(dev(xh), _i16(za), dev(wh), _i16(), dev(bias), lay_g, stride, pad, 1, hago.I32)
        assert_same(host(got), want, f"int16 conv {case} {layout} za={za}")
    x12, w12 = (xh // 16).astype(np.int16), (wh // 16).astype(np.int16)
    mult, shift = datagen.requant_params(rng, np.full(O, 1182.0 * 1182.0 * np.sqrt(C * KH * KW)), 40.0)
    want = ref.qconv2d(x12, -5, w12, bias, lay_r, stride, pad, 1, ref.I32, ref_requant(mult, shift))
    got = qconv2d(dev(x12), _i16(-5, 12), dev(w12), _i16(0, 12), dev(bias), lay_g, stride, pad, 1, hago.I32, gpu_requant(mult, shift))
    assert_same(host(got), want, f"int16 conv requantized {case} {layout}")
    assert len(np.unique(want)) > 10 or want.size < 100


def test_int16_depthwise_is_refused():
    x = torch.zeros((1, 4, 5, 5), dtype=torch.int16, device=DEV)
    w = torch.zeros((4, 1, 3, 3), dtype=torch.int16, device=DEV)
    with pytest.raises(hago.HagoError) as e:
        hago.qconv2d(x, _i16(), w, _i16(), None, hago.NCHW, (1, 1), (1, 1), 4, hago.I32)
    assert e.value.code == 3


# ---------------------------------------------------------------- overflow-simulating simulated quantize
@pytest.mark.parametrize("shape", [(2, 3, 1024), (1, 5, 77), (4, 1, 4096)])
@pytest.mark.parametrize("dt,bits,signed", [(hago.I16, 16, True), (hago.I8, 8, True), (hago.U8, 8, False), (hago.I24, 24, True),
                                           (hago.I32, 25, True), (hago.I16, 6, True)])
def test_simquant_wrap(shape, dt, bits, signed):
    rng = np.random.default_rng(sum(shape) + bits)
    C = shape[1]
    wrap_bits = {hago.I16: 16, hago.I8: 8, hago.U8: 8, hago.I24: 24, hago.I32: 32}[dt]
    s = rng.uniform(0.01, 0.05, C).astype(np.float32)
    z = rng.integers(-3, 4, C).astype(np.int32) if signed else rng.integers(100, 140, C).astype(np.int32)
    # codes spread over several multiples of the type's range, plus the awkward reals
    x = (rng.standard_normal(shape) * (2.0 ** wrap_bits) * 1.5 * s.reshape(1, C, 1)).astype(np.float32)
    x[..., ::3] = (rng.standard_normal(x[..., ::3].shape) * 40 * s.reshape(1, C, 1)).astype(np.float32)   # no overflow
    x.reshape(-1)[:12] = [np.nan, np.inf, -np.inf, 1e30, -1e30, 0.0, -0.0, 3.0e38, 5e18 * float(s[0]), 1e-40, 2.0 ** 31, -2.0 ** 31]
    lo, hi = hago.bit_range(min(bits, 25), signed)
    want = ref.simquant_wrap(x, s, z, wrap_bits, dt != hago.U8, lo, hi)
    got = hago.simquant_wrap(dev(x), dev(s), dev(z), hago.QType(dt, bits, signed), lo, hi)
    assert_same_bits(host(got), want, f"simquant_wrap {shape} bits {wrap_bits}")
    plain = ref.simquant(x, s, z, lo, hi)
    ok = ~np.isnan(want)
    assert (want[ok] != plain[ok]).any()            # the overflow changed something
    # per tensor, in place
    want = ref.simquant_wrap(x, s[:1], z[:1], wrap_bits, dt != hago.U8, lo, hi)
    xd = dev(x)
    assert_same_bits(host(hago.simquant_wrap(xd, dev(s[:1]), dev(z[:1]), hago.QType(dt, bits, signed), lo, hi, out=xd)), want, "in place")
