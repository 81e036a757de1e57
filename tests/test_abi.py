"""Host-only checks of the C-ABI library: it loads, exports every declared
symbol, and rejects bad arguments before touching the device."""
import ctypes as C
import os
import re

import pytest

from conftest import ROOT

import paper_2103_14949_amd as hago
from paper_2103_14949_amd import binding


@pytest.fixture(scope="module")
def L():
    if not os.path.exists(hago.library_path()):
        from paper_2103_14949_amd import build
        build.build()
    return hago.lib()


def test_every_declared_symbol_is_exported(L):
    header = open(os.path.join(ROOT, "include", "hago.h")).read()
    declared = set(re.findall(r"\b(hago_[a-z0-9_]+)\s*\(", header))
    assert {"hago_simquant", "hago_qdense", "hago_qconv2d", "hago_requantize", "hago_absmax",
            "hago_quantize", "hago_dequantize", "hago_simquant_codes", "hago_simquant_batched",
            "hago_status_string"} <= declared
    for name in declared:
        assert hasattr(L, name), name
    assert set(binding.EXPORTS) == declared


def test_status_strings(L):
    seen = {L.hago_status_string(i) for i in range(9)}
    assert len(seen) == 9 and all(seen)


BAD = 0x1000  # a non-null pointer that is never dereferenced: validation fails first


def _rq(out_dtype=hago.I8, bits=8, signed=1, z=0, lo=-128, hi=127, mult=BAD, shift=BAD, pc=1, rounding=0):
    return binding._Requant(mult, shift, pc, binding._QType(out_dtype, bits, signed, z), lo, hi, rounding)


def _qt(dt, bits=8, signed=None, z=0):
    return binding._QType(dt, bits, int(dt != hago.U8) if signed is None else signed, z)


def test_qdense_argument_errors(L):
    u8, i8 = _qt(hago.U8, z=128), _qt(hago.I8)
    call = lambda *a: L.hago_qdense(*a)  # noqa: E731
    ok_tail = (hago.I32, None, BAD, 0, None)
    assert call(None, u8, BAD, i8, None, 4, 4, 4, *ok_tail) == 1
    assert call(BAD, u8, None, i8, None, 4, 4, 4, *ok_tail) == 1
    assert call(BAD, u8, BAD, i8, None, 4, 4, 4, hago.I32, None, None, 0, None) == 1
    assert call(BAD, u8, BAD, i8, None, -1, 4, 4, *ok_tail) == 2
    assert call(BAD, u8, BAD, i8, None, 4, 2 ** 31, 4, *ok_tail) == 2
    assert call(BAD, _qt(hago.I16), BAD, i8, None, 4, 4, 4, *ok_tail) == 3
    assert call(BAD, u8, BAD, _qt(hago.U8), None, 4, 4, 4, *ok_tail) == 3
    assert call(BAD, u8, BAD, _qt(hago.I8, z=1), None, 4, 4, 4, *ok_tail) == 3     # asymmetric weights
    assert call(BAD, u8, BAD, i8, None, 4, 4, 4, hago.F32, None, BAD, 0, None) == 3
    assert call(BAD, _qt(hago.U8, bits=9), BAD, i8, None, 4, 4, 4, *ok_tail) == 4
    assert call(BAD, _qt(hago.U8, bits=0), BAD, i8, None, 4, 4, 4, *ok_tail) == 4
    assert call(BAD, _qt(hago.U8, z=256), BAD, i8, None, 4, 4, 4, *ok_tail) == 4
    assert call(BAD, _qt(hago.I8, bits=8, signed=0), BAD, i8, None, 4, 4, 4, *ok_tail) == 4   # 0..255 in an int8
    assert call(BAD, u8, BAD, i8, None, 4, 4, 4, hago.I32, None, BAD, 2, None) == 5
    # requantize struct errors
    for rq, code in ((_rq(shift=None), 1), (_rq(out_dtype=hago.I16, bits=16), 3), (_rq(lo=5, hi=4), 4),
                     (_rq(lo=-129), 4), (_rq(out_dtype=hago.U8, signed=0, lo=0, hi=256), 4),
                     (_rq(bits=4, lo=-8, hi=8), 4), (_rq(pc=2), 5), (_rq(z=200), 4),
                     (_rq(rounding=2), 5), (_rq(rounding=-1), 5)):
        assert call(BAD, u8, BAD, i8, None, 4, 4, 4, hago.I32, C.byref(rq), BAD, 0, None) == code
    # operand triples: int16 operands come in pairs and do not accumulate in 16 bits
    i16 = _qt(hago.I16, 16)
    assert call(BAD, i16, BAD, i8, None, 4, 4, 4, *ok_tail) == 3
    assert call(BAD, u8, BAD, i16, None, 4, 4, 4, *ok_tail) == 3
    assert call(BAD, i16, BAD, i16, None, 4, 4, 4, hago.I16, None, BAD, 0, None) == 3
    assert call(BAD, i16, BAD, _qt(hago.I16, 16, z=3), None, 4, 4, 4, *ok_tail) == 3
    # strict 24-bit accumulation bound: K * Amax * Wmax <= 2^23 - 1
    strict24 = (hago.I24, None, BAD, hago.STRICT_ACC16, None)
    assert call(BAD, _qt(hago.I8, 8, 1), BAD, i8, None, 4, 4, 512, *strict24) == 6     # 512 * 128 * 128 = 2^23
    assert call(BAD, i16, BAD, i16, None, 4, 4, 1, *strict24) == 6                     # 2^15 * 2^15
    # strict int16 accumulation bound: K * Amax * Wmax <= 32767
    a4, w4 = _qt(hago.I8, 4, 0), _qt(hago.I8, 4, 1)        # 0..15 x -8..7 -> 120 per term
    strict = (hago.I16, None, BAD, hago.STRICT_ACC16, None)
    assert call(BAD, a4, BAD, w4, None, 4, 4, 274, *strict) == 6
    assert call(BAD, _qt(hago.I8, 8, 1), BAD, i8, None, 4, 4, 2, *strict) == 6       # 2 * 128 * 128 = 32768


def test_qconv2d_argument_errors(L):
    u8, i8 = _qt(hago.U8, z=128), _qt(hago.I8)

    def call(B=1, Cc=4, H=8, W=8, O=4, KH=3, KW=3, sh=1, sw=1, ph=1, pw=1, groups=1, layout=0, a=BAD, out=BAD):
        return L.hago_qconv2d(a, u8, BAD, i8, None, layout, B, Cc, H, W, O, KH, KW, sh, sw, ph, pw, groups,
                              hago.I32, None, out, 0, None)

    assert call(a=None) == 1 and call(out=None) == 1
    assert call(groups=2) == 2 and call(groups=4, O=8) == 2 and call(groups=0) == 2
    assert call(KH=11, ph=0) == 2          # kernel larger than the image
    assert call(sh=0) == 2 and call(ph=-1) == 2 and call(layout=2) == 2 and call(Cc=0) == 2
    assert call(B=2 ** 20, Cc=2 ** 10, H=64, W=64) == 2   # beyond the 31-bit index range


def test_qconv2d_workspace_queries_and_errors(L):
    """hago_qconv2d_workspace_bytes is host-only arithmetic; hago_qconv2d_ws refuses a workspace that
    is missing, too small or misaligned before anything is launched."""
    wsb = lambda **k: L.hago_qconv2d_workspace_bytes(*[k.get(n, d) for n, d in (  # noqa: E731
        ("layout", 0), ("B", 1), ("C", 64), ("H", 56), ("W", 56), ("O", 64), ("KH", 3), ("KW", 3),
        ("sh", 1), ("sw", 1), ("ph", 1), ("pw", 1), ("groups", 1))])
    r256 = lambda v: (v + 255) // 256 * 256  # noqa: E731
    # config 2: weights [64][9][64], activations [1][58][58][64]
    assert wsb() == r256(64 * 9 * 64) + r256(58 * 58 * 64)
    # the weight part does not depend on the batch; channels are rounded up to 16
    assert wsb(B=8) - wsb(B=7) == 58 * 58 * 64     # a multiple of 256
    assert wsb(C=3, O=4, H=5, W=6) == r256(4 * 9 * 16) + r256(7 * 8 * 16)
    assert wsb(groups=64) == 0                      # depthwise needs none
    assert wsb(B=0) == 0
    assert wsb(groups=3) == -1 and wsb(KH=70, ph=0) == -1 and wsb(layout=5) == -1
    # 32-bit limits of the rewritten copies: the general kernel serves those shapes without scratch
    assert wsb(B=640, C=1024, H=56, W=56, O=8) == 0
    u8, i8 = _qt(hago.U8, z=128), _qt(hago.I8)

    def call(ws, nbytes, flags=0, groups=1, O=64):
        return L.hago_qconv2d_ws(BAD, u8, BAD, i8, None, 0, 1, 64, 56, 56, O, 3, 3, 1, 1, 1, 1, groups,
                                 hago.I32, None, BAD, ws, nbytes, flags, None)

    need = wsb()
    assert call(None, need) == 1                    # needed but NULL
    assert call(0x100000, need - 1) == 5            # too small
    assert call(0x100010, need) == 5                # not 256-byte aligned
    assert call(0x100000, -1) == 5
    assert call(0x100000, need, flags=8) == 5       # unknown flag
    assert L.hago_qconv2d(BAD, u8, BAD, i8, None, 0, 1, 64, 56, 56, 64, 3, 3, 1, 1, 1, 1, 1, hago.I32, None, BAD,
                          hago.WS_WEIGHTS_READY, None) == 5   # a workspace flag without a workspace


def test_bit_range(L):
    assert hago.bit_range(8, True) == (-128, 127) and hago.bit_range(8, False) == (0, 255)
    assert hago.bit_range(4, True) == (-8, 7) and hago.bit_range(1, False) == (0, 1)
    assert hago.bit_range(32, True) == (-2 ** 31, 2 ** 31 - 1)
    lo, hi = C.c_int32(), C.c_int32()
    assert L.hago_bit_range(0, 1, C.byref(lo), C.byref(hi)) == 4
    assert L.hago_bit_range(32, 0, C.byref(lo), C.byref(hi)) == 4
    assert L.hago_bit_range(8, 1, None, C.byref(hi)) == 1


def test_simquant_and_requantize_argument_errors(L):
    q = _qt(hago.I8)
    sq = lambda *a: L.hago_simquant(*a)  # noqa: E731
    assert sq(None, BAD, 1, 1, 1, BAD, BAD, 0, q, -128, 127, None) == 1
    assert sq(BAD, BAD, 1, 1, 1, None, BAD, 0, q, -128, 127, None) == 1
    assert sq(BAD, BAD, -1, 1, 1, BAD, BAD, 0, q, -128, 127, None) == 2
    assert sq(BAD, BAD, 1, 1, 1, BAD, BAD, 0, _qt(hago.F32), -128, 127, None) == 3
    assert sq(BAD, BAD, 1, 1, 1, BAD, BAD, 0, q, -129, 127, None) == 4
    assert sq(BAD, BAD, 1, 1, 1, BAD, BAD, 0, q, 3, 2, None) == 4
    assert sq(BAD, BAD, 1, 1, 1, BAD, BAD, 0, _qt(hago.I8, 4), -8, 8, None) == 4
    assert sq(BAD, BAD, 1, 1, 1, BAD, BAD, 2, q, -128, 127, None) == 5
    assert sq(BAD, BAD, 1, 1, 1, BAD, BAD, 0, _qt(hago.I32, 32), -2 ** 31, 2 ** 31 - 1, None) == 4  # not exact in fp32
    rq = _rq()
    req = lambda *a: L.hago_requantize(*a)  # noqa: E731
    assert req(None, hago.I32, 1, 1, 1, C.byref(rq), BAD, None) == 1
    assert req(BAD, hago.I32, 1, 1, 1, None, BAD, None) == 1
    assert req(BAD, hago.I8, 1, 1, 1, C.byref(rq), BAD, None) == 3
    assert req(BAD, hago.I32, 1, -1, 1, C.byref(rq), BAD, None) == 2


def test_quantize_and_dequantize_argument_errors(L):
    q = _qt(hago.I8)
    qz = lambda *a: L.hago_quantize(*a)  # noqa: E731
    assert qz(None, BAD, 1, 1, 1, BAD, BAD, 0, q, -128, 127, None) == 1
    assert qz(BAD, BAD, 1, 1, 1, BAD, None, 0, q, -128, 127, None) == 1
    assert qz(BAD, BAD, 1, -1, 1, BAD, BAD, 0, q, -128, 127, None) == 2
    assert qz(BAD, BAD, 1, 1, 1, BAD, BAD, 0, _qt(hago.F32), -128, 127, None) == 3
    assert qz(BAD, BAD, 1, 1, 1, BAD, BAD, 0, q, -129, 127, None) == 4
    assert qz(BAD, BAD, 1, 1, 1, BAD, BAD, 0, _qt(hago.I32, 32), -2 ** 31, 2 ** 31 - 1, None) == 4
    assert qz(BAD, BAD, 1, 1, 1, BAD, BAD, 3, q, -128, 127, None) == 5
    sc = lambda *a: L.hago_simquant_codes(*a)  # noqa: E731
    assert sc(BAD, None, BAD, 1, 1, 1, BAD, BAD, 0, q, -128, 127, None) == 1
    assert sc(BAD, BAD, None, 1, 1, 1, BAD, BAD, 0, q, -128, 127, None) == 1
    assert sc(BAD, BAD, BAD, -1, 1, 1, BAD, BAD, 0, q, -128, 127, None) == 2
    assert sc(BAD, BAD, BAD, 1, 1, 1, BAD, BAD, 0, _qt(hago.F32), -128, 127, None) == 3
    assert sc(BAD, BAD, BAD, 1, 1, 1, BAD, BAD, 0, q, -128, 128, None) == 4
    assert sc(BAD, BAD, BAD, 1, 1, 1, BAD, BAD, 2, q, -128, 127, None) == 5
    assert sc(None, None, None, 0, 4, 4, BAD, BAD, 0, q, -128, 127, None) == 0   # empty: a no-op
    dq = lambda *a: L.hago_dequantize(*a)  # noqa: E731
    assert dq(None, q, BAD, 1, 1, 1, BAD, BAD, 0, None) == 1
    assert dq(BAD, q, None, 1, 1, 1, BAD, BAD, 0, None) == 1
    assert dq(BAD, q, BAD, 1, 1, -1, BAD, BAD, 0, None) == 2
    assert dq(BAD, _qt(hago.F32), BAD, 1, 1, 1, BAD, BAD, 0, None) == 3
    assert dq(BAD, q, BAD, 1, 1, 1, BAD, BAD, 2, None) == 5


def test_simquant_batched_argument_errors(L):
    q = _qt(hago.I8)
    lo = (C.c_int32 * 2)(-128, -8)
    hi = (C.c_int32 * 2)(127, 7)
    sb = lambda *a: L.hago_simquant_batched(*a)  # noqa: E731
    assert sb(None, BAD, 1, 1, 1, 2, BAD, BAD, 1, q, lo, hi, None) == 1
    assert sb(BAD, BAD, 1, 1, 1, 2, BAD, BAD, 1, q, None, hi, None) == 1
    assert sb(BAD, BAD, 1, 1, -1, 2, BAD, BAD, 1, q, lo, hi, None) == 2
    assert sb(BAD, BAD, 1, 1, 1, 17, BAD, BAD, 1, q, lo, hi, None) == 5
    assert sb(BAD, BAD, 1, 1, 1, 2, BAD, BAD, 1, _qt(hago.F32), lo, hi, None) == 3
    bad_hi = (C.c_int32 * 2)(127, 200)
    assert sb(BAD, BAD, 1, 1, 1, 2, BAD, BAD, 1, q, lo, bad_hi, None) == 4


def test_absmax_argument_errors(L):
    am = lambda *a: L.hago_absmax(*a)  # noqa: E731
    assert am(None, 1, 1, 1, 1, BAD, None) == 1
    assert am(BAD, 1, 1, 1, 1, None, None) == 1
    assert am(BAD, 1, -1, 1, 1, BAD, None) == 2
    assert am(BAD, 2 ** 40, 2 ** 40, 2, 1, BAD, None) == 2
    assert am(BAD, 1, 1, 1, 2, BAD, None) == 5


def test_binding_fails_loudly_without_the_library(monkeypatch, tmp_path):
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "_LIB_PATH", str(tmp_path / "missing.so"))
    with pytest.raises(FileNotFoundError):
        binding.lib()
