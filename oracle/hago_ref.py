"""ctypes front end of the CPU oracle (TEST INFRASTRUCTURE ONLY).

Loads ``libhago_ref.so`` (built from ``hago_ref.cpp`` with g++) and exposes
numpy-in / numpy-out wrappers.  Nothing here or in the C++ file is shared with
the GPU library; only tests, the smoke check and the benchmark's cpu_baseline
leg import this module.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
import threading

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "hago_ref.cpp")
_LIB = os.path.join(_HERE, "libhago_ref.so")

U8, I8, I16, I32, F32, I24 = 0, 1, 2, 3, 4, 5   # I24: accumulator only, stored sign-extended in int32
NCHW, NHWC = 0, 1

_NP_OF = {U8: np.uint8, I8: np.int8, I16: np.int16, I32: np.int32, I24: np.int32}
_CODE_OF = {np.dtype(np.uint8): U8, np.dtype(np.int8): I8,
            np.dtype(np.int16): I16, np.dtype(np.int32): I32}

CXXFLAGS = ["-O2", "-std=c++17", "-ffp-contract=off", "-fno-fast-math",
            "-shared", "-fPIC"]


def build(force: bool = False, extra_flags=(), out: str | None = None) -> str:
    """Compile the oracle with g++; returns the path of the shared library."""
    out = out or _LIB
    if (not force and os.path.exists(out)
            and os.path.getmtime(out) >= max(os.path.getmtime(_SRC),
                                             os.path.getmtime(os.path.join(_HERE, "hago_ref.h")))):
        return out
    cmd = ["g++", *CXXFLAGS, *extra_flags, _SRC, "-o", out]
    subprocess.run(cmd, check=True)
    return out


class _Requant(C.Structure):
    _fields_ = [("multiplier", C.c_void_p), ("shift", C.c_void_p),
                ("per_channel", C.c_int32), ("out_dtype", C.c_int32),
                ("out_zero_point", C.c_int32), ("clip_lo", C.c_int32),
                ("clip_hi", C.c_int32), ("rounding", C.c_int32)]


_lib = None
_lock = threading.Lock()


def lib(path: str | None = None):
    global _lib
    with _lock:
        if _lib is None or path is not None:
            L = C.CDLL(path or build())
            i32, i64, vp, dbl = C.c_int32, C.c_int64, C.c_void_p, C.c_double
            L.hago_ref_scale.restype = dbl
            L.hago_ref_scale.argtypes = [dbl, i32, i32]
            L.hago_ref_absmax.argtypes = [vp, i64, i64, i64, i32, vp]
            L.hago_ref_quantize.argtypes = [vp, vp, i64, i64, i64, vp, vp, i32, i32, i32]
            L.hago_ref_dequantize.argtypes = [vp, vp, i64, i64, i64, vp, vp, i32]
            L.hago_ref_bit_range.argtypes = [i32, i32, vp, vp]
            L.hago_ref_simquant.argtypes = [vp, vp, i64, i64, i64, vp, vp, i32, i32, i32]
            L.hago_ref_encode_multiplier.argtypes = [dbl, vp, vp]
            L.hago_ref_requantize_one.restype = i64
            L.hago_ref_requantize_one.argtypes = [i32] * 6
            L.hago_ref_requantize_one_mode.restype = i64
            L.hago_ref_requantize_one_mode.argtypes = [i32] * 7
            L.hago_ref_requantize.argtypes = [vp, i32, i64, i64, i64, vp, vp]
            L.hago_ref_acc16_safe.argtypes = [i64, i64, i64]
            L.hago_ref_acc_safe.argtypes = [i64, i64, i64, i32]
            L.hago_ref_requantize_shift_one.restype = i64
            L.hago_ref_requantize_shift_one.argtypes = [i32] * 6
            L.hago_ref_simquant_wrap.argtypes = [vp, vp, i64, i64, i64, vp, vp, i32, i32, i32, i32, i32]
            L.hago_ref_qdense_x.argtypes = [vp, i32, i32, vp, i32, vp, i64, i64, i64, i32, vp, vp]
            L.hago_ref_qconv2d_x.argtypes = [vp, i32, i32, vp, i32, vp, i32] + [i64] * 5 + [i32] * 7 + [i32, vp, vp]
            L.hago_ref_qdense.argtypes = [vp, i32, i32, vp, vp, i64, i64, i64, i32, vp, vp]
            L.hago_ref_qconv2d.argtypes = [vp, i32, i32, vp, vp, i32] + [i64] * 5 + [i32] * 7 + [i32, vp, vp]
            if path is not None:
                return L
            _lib = L
        return _lib


class RefError(RuntimeError):
    def __init__(self, code):
        super().__init__(f"oracle returned status {code}")
        self.code = code


def _chk(rc):
    if rc != 0:
        raise RefError(rc)


def _p(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


class Requant:
    """Requantize parameters (host arrays).  multiplier=None: power-of-two scales, the rounding
    right shift alone (Sec. 5.1)."""

    def __init__(self, multiplier, shift, out_dtype=I8, out_zero_point=0,
                 clip_lo=-128, clip_hi=127, per_channel=None, rounding=0):
        self.multiplier = (None if multiplier is None
                           else np.ascontiguousarray(multiplier, dtype=np.int32).reshape(-1))
        self.shift = np.ascontiguousarray(shift, dtype=np.int32).reshape(-1)
        self.per_channel = int(self.shift.size > 1) if per_channel is None else int(per_channel)
        self.out_dtype = out_dtype
        self.out_zero_point = int(out_zero_point)
        self.clip_lo = int(clip_lo)
        self.clip_hi = int(clip_hi)
        self.rounding = int(rounding)   # ROUND_UPWARD or ROUND_HALF_AWAY

    def c_struct(self):
        return _Requant(None if self.multiplier is None else self.multiplier.ctypes.data, self.shift.ctypes.data,
                        self.per_channel, self.out_dtype, self.out_zero_point,
                        self.clip_lo, self.clip_hi, self.rounding)


def scale(threshold, bits, sign):
    return lib().hago_ref_scale(float(threshold), int(bits), int(sign))


def bit_range(bits, is_signed):
    lo, hi = C.c_int32(), C.c_int32()
    _chk(lib().hago_ref_bit_range(bits, int(is_signed), C.addressof(lo), C.addressof(hi)))
    return lo.value, hi.value


def absmax(x, per_channel=True):
    """x: float32 [outer, channels, inner]."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    o, c, i = x.shape
    thr = np.empty(c if per_channel else 1, np.float32)
    _chk(lib().hago_ref_absmax(_p(x), o, c, i, int(per_channel), _p(thr)))
    return thr


def simquant(x, scale, zero_point, clip_lo, clip_hi, per_channel=None):
    """x: float32 [outer, channels, inner] -> same shape."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    o, c, i = x.shape
    s = np.ascontiguousarray(scale, dtype=np.float32).reshape(-1)
    z = np.ascontiguousarray(zero_point, dtype=np.int32).reshape(-1)
    pc = int(s.size > 1) if per_channel is None else int(per_channel)
    y = np.empty_like(x)
    _chk(lib().hago_ref_simquant(_p(x), _p(y), o, c, i, _p(s), _p(z), pc,
                                 int(clip_lo), int(clip_hi)))
    return y


def simquant_wrap(x, scale, zero_point, wrap_bits, wrap_signed, clip_lo, clip_hi, per_channel=None):
    """simulated_quantize with the overflow of a wrap_bits-wide (un)signed integer type (Sec. 5.2)."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    o, c, i = x.shape
    s = np.ascontiguousarray(scale, dtype=np.float32).reshape(-1)
    z = np.ascontiguousarray(zero_point, dtype=np.int32).reshape(-1)
    pc = int(s.size > 1) if per_channel is None else int(per_channel)
    y = np.empty_like(x)
    _chk(lib().hago_ref_simquant_wrap(_p(x), _p(y), o, c, i, _p(s), _p(z), pc, int(wrap_bits),
                                      int(bool(wrap_signed)), int(clip_lo), int(clip_hi)))
    return y


def simquant_batched(x, scales, zero_points, clip_lo, clip_hi, per_channel=True):
    """Batched search evaluation (Sec. 6.3): candidate b applies simulated_quantize with its own
    scales[b], zero_points[b] ([channels] each, or one entry) and clip range to the SAME tensor x.
    Returns y[b, outer, channels, inner].  By definition: one simquant per candidate."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    nb = len(clip_lo)
    s = np.ascontiguousarray(scales, dtype=np.float32).reshape(nb, -1)
    z = np.ascontiguousarray(zero_points, dtype=np.int32).reshape(nb, -1)
    y = np.empty((nb,) + x.shape, np.float32)
    for b in range(nb):
        y[b] = simquant(x, s[b], z[b], int(clip_lo[b]), int(clip_hi[b]), per_channel)
    return y


def quantize(x, scale, zero_point, clip_lo, clip_hi, per_channel=None):
    """x: float32 [outer, channels, inner] -> int32 codes of the same shape."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    o, c, i = x.shape
    s = np.ascontiguousarray(scale, dtype=np.float32).reshape(-1)
    z = np.ascontiguousarray(zero_point, dtype=np.int32).reshape(-1)
    pc = int(s.size > 1) if per_channel is None else int(per_channel)
    q = np.empty(x.shape, np.int32)
    _chk(lib().hago_ref_quantize(_p(x), _p(q), o, c, i, _p(s), _p(z), pc, int(clip_lo), int(clip_hi)))
    return q


def simquant_codes(x, scale, zero_point, clip_lo, clip_hi, per_channel=None):
    """simulated_quantize that also hands out the integer codes it passes through (Sec. 6.1: the
    realized graph keeps q, the simulated graph keeps q * s; Eq. 3).  By definition the pair
    (simquant(x), quantize(x)): a NaN stays NaN in y and takes the code of real zero in q."""
    return (simquant(x, scale, zero_point, clip_lo, clip_hi, per_channel),
            quantize(x, scale, zero_point, clip_lo, clip_hi, per_channel))


def dequantize(q, scale, zero_point, per_channel=None):
    """q: integer codes [outer, channels, inner] -> float32."""
    q = np.ascontiguousarray(q, dtype=np.int32)
    o, c, i = q.shape
    s = np.ascontiguousarray(scale, dtype=np.float32).reshape(-1)
    z = np.ascontiguousarray(zero_point, dtype=np.int32).reshape(-1)
    pc = int(s.size > 1) if per_channel is None else int(per_channel)
    y = np.empty(q.shape, np.float32)
    _chk(lib().hago_ref_dequantize(_p(q), _p(y), o, c, i, _p(s), _p(z), pc))
    return y


def encode_multiplier(m):
    q, s = C.c_int32(), C.c_int32()
    _chk(lib().hago_ref_encode_multiplier(float(m), C.addressof(q), C.addressof(s)))
    return q.value, s.value


ROUND_UPWARD, ROUND_HALF_AWAY = 0, 1


def requantize_one(acc, multiplier, shift, z_out=0, lo=-(2 ** 31), hi=2 ** 31 - 1, rounding=ROUND_UPWARD):
    return lib().hago_ref_requantize_one_mode(int(acc), int(multiplier), int(shift),
                                              int(z_out), int(lo), int(hi), int(rounding))


def requantize_shift_one(acc, shift, z_out=0, lo=-(2 ** 31), hi=2 ** 31 - 1, rounding=ROUND_UPWARD):
    return lib().hago_ref_requantize_shift_one(int(acc), int(shift), int(z_out), int(lo), int(hi), int(rounding))


def requantize(acc, rq: Requant):
    """acc: int32 or int16 [outer, channels, inner]."""
    acc = np.ascontiguousarray(acc)
    code = _CODE_OF[acc.dtype]
    o, c, i = acc.shape
    out = np.empty(acc.shape, _NP_OF[rq.out_dtype])
    st = rq.c_struct()
    _chk(lib().hago_ref_requantize(_p(acc), code, o, c, i, C.addressof(st), _p(out)))
    return out


def acc16_safe(K, a_absmax, w_absmax):
    return bool(lib().hago_ref_acc16_safe(int(K), int(a_absmax), int(w_absmax)))


def acc_safe(K, a_absmax, w_absmax, acc_bits):
    return bool(lib().hago_ref_acc_safe(int(K), int(a_absmax), int(w_absmax), int(acc_bits)))


def _weights(w):
    """int8 weights, or int16 ones for the int16 x int16 operand triple."""
    w = np.ascontiguousarray(w)
    return w if w.dtype == np.int16 else np.ascontiguousarray(w, dtype=np.int8)


def _out_dtype(acc_dtype, rq):
    return _NP_OF[rq.out_dtype] if rq is not None else _NP_OF[acc_dtype]


def qdense(a, a_zero_point, w, bias=None, acc_dtype=I32, rq: Requant | None = None, out=None):
    a = np.ascontiguousarray(a)
    w = _weights(w)
    M, K = a.shape
    N = w.shape[0]
    assert w.shape[1] == K
    if bias is not None:
        bias = np.ascontiguousarray(bias, dtype=np.int32)
    if out is None:
        out = np.empty((M, N), _out_dtype(acc_dtype, rq))
    st = rq.c_struct() if rq is not None else None
    _chk(lib().hago_ref_qdense_x(_p(a), _CODE_OF[a.dtype], int(a_zero_point), _p(w), _CODE_OF[w.dtype], _p(bias),
                                 M, N, K, acc_dtype,
                                 C.addressof(st) if st is not None else None, _p(out)))
    return out


def conv_out_hw(H, W, KH, KW, stride, pad):
    return ((H + 2 * pad[0] - KH) // stride[0] + 1,
            (W + 2 * pad[1] - KW) // stride[1] + 1)


def qconv2d(a, a_zero_point, w, bias=None, layout=NCHW, stride=(1, 1), pad=(0, 0),
            groups=1, acc_dtype=I32, rq: Requant | None = None):
    a = np.ascontiguousarray(a)
    w = _weights(w)
    if layout == NCHW:
        B, Cc, H, W = a.shape
        O, _, KH, KW = w.shape
    else:
        B, H, W, Cc = a.shape
        O, KH, KW, _ = w.shape
    OH, OW = conv_out_hw(H, W, KH, KW, stride, pad)
    if bias is not None:
        bias = np.ascontiguousarray(bias, dtype=np.int32)
    OHa, OWa = max(OH, 0), max(OW, 0)  # a bad shape is for the C side to reject
    shape = (B, O, OHa, OWa) if layout == NCHW else (B, OHa, OWa, O)
    out = np.empty(shape, _out_dtype(acc_dtype, rq))
    st = rq.c_struct() if rq is not None else None
    _chk(lib().hago_ref_qconv2d_x(_p(a), _CODE_OF[a.dtype], int(a_zero_point), _p(w), _CODE_OF[w.dtype], _p(bias),
                                  layout, B, Cc, H, W, O, KH, KW, stride[0], stride[1],
                                  pad[0], pad[1], groups, acc_dtype,
                                  C.addressof(st) if st is not None else None, _p(out)))
    return out


def qdense_threaded(a, a_zero_point, w, bias=None, acc_dtype=I32, rq=None, threads=1):
    """The unchanged oracle called on disjoint row slices from `threads` threads."""
    a = np.ascontiguousarray(a)
    M = a.shape[0]
    out = np.empty((M, w.shape[0]), _out_dtype(acc_dtype, rq))
    bounds = np.linspace(0, M, threads + 1).astype(np.int64)
    ts = []
    for t in range(threads):
        lo, hi = int(bounds[t]), int(bounds[t + 1])
        if hi > lo:
            th = threading.Thread(target=qdense, args=(a[lo:hi], a_zero_point, w, bias, acc_dtype, rq, out[lo:hi]))
            th.start()
            ts.append(th)
    for th in ts:
        th.join()
    return out
