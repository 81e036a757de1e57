"""ctypes binding of libhago.so: same names as the C ABI, argument marshalling only.

Tensors are torch tensors on the GPU; the binding passes their device pointers
and the current torch stream to the library and allocates the output tensor.
There is no CPU fallback: if the library is missing, loading fails.
"""
from __future__ import annotations

import ctypes as C
import os

U8, I8, I16, I32, F32, I24 = 0, 1, 2, 3, 4, 5   # I24: accumulator / simulated type only
NCHW, NHWC = 0, 1
STRICT_ACC16 = 1
WS_WEIGHTS_READY = 2
STATIC_SCRATCH_BYTES = 64 << 20   # HAGO_STATIC_SCRATCH_BYTES
HOOK_GEMM_PATH, HOOK_STREAM_TILE, HOOK_GENERAL_TILE = 0, 1, 2   # hago_set_test_hook keys
ROUND_UPWARD, ROUND_HALF_AWAY = 0, 1   # hago_rounding

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libhago.so")

EXPORTS = ("hago_simquant", "hago_simquant_batched", "hago_absmax", "hago_simquant_wrap", "hago_quantize", "hago_dequantize", "hago_simquant_codes", "hago_qdense", "hago_qconv2d", "hago_qconv2d_ws", "hago_qconv2d_workspace_bytes", "hago_qconv2d_static", "hago_requantize",
           "hago_status_string", "hago_bit_range", "hago_set_test_hook", "hago_probe_mfma_i8", "hago_probe_copy")


class _QType(C.Structure):
    _fields_ = [("dtype", C.c_int32), ("bits", C.c_int32), ("is_signed", C.c_int32),
                ("zero_point", C.c_int32)]


class _Requant(C.Structure):
    _fields_ = [("multiplier", C.c_void_p), ("shift", C.c_void_p), ("per_channel", C.c_int32),
                ("out", _QType), ("clip_lo", C.c_int32), ("clip_hi", C.c_int32), ("rounding", C.c_int32)]


class HagoError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__(f"libhago: {msg} (status {code})")
        self.code = code


def library_path() -> str:
    return _LIB_PATH


_lib = None


def lib():
    """Load libhago.so (built by paper_2103_14949_amd/build.py); raises if absent."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise FileNotFoundError(
                f"{_LIB_PATH} is missing: build it with `python -m paper_2103_14949_amd.build` "
                "(there is no fallback path)")
        L = C.CDLL(_LIB_PATH)
        i32, i64, u32, vp = C.c_int32, C.c_int64, C.c_uint32, C.c_void_p
        L.hago_status_string.restype = C.c_char_p
        L.hago_status_string.argtypes = [i32]
        L.hago_simquant.restype = i32
        L.hago_simquant.argtypes = [vp, vp, i64, i64, i64, vp, vp, i32, _QType, i32, i32, vp]
        L.hago_simquant_wrap.restype = i32
        L.hago_simquant_wrap.argtypes = L.hago_simquant.argtypes
        L.hago_simquant_batched.restype = i32
        L.hago_simquant_batched.argtypes = [vp, vp, i64, i64, i64, i32, vp, vp, i32, _QType, vp, vp, vp]
        L.hago_quantize.restype = i32
        L.hago_quantize.argtypes = [vp, vp, i64, i64, i64, vp, vp, i32, _QType, i32, i32, vp]
        L.hago_simquant_codes.restype = i32
        L.hago_simquant_codes.argtypes = [vp, vp, vp, i64, i64, i64, vp, vp, i32, _QType, i32, i32, vp]
        L.hago_dequantize.restype = i32
        L.hago_dequantize.argtypes = [vp, _QType, vp, i64, i64, i64, vp, vp, i32, vp]
        L.hago_absmax.restype = i32
        L.hago_absmax.argtypes = [vp, i64, i64, i64, i32, vp, vp]
        L.hago_requantize.restype = i32
        L.hago_requantize.argtypes = [vp, i32, i64, i64, i64, C.POINTER(_Requant), vp, vp]
        L.hago_qdense.restype = i32
        L.hago_qdense.argtypes = [vp, _QType, vp, _QType, vp, i64, i64, i64, i32,
                                  C.POINTER(_Requant), vp, u32, vp]
        L.hago_qconv2d.restype = i32
        L.hago_qconv2d.argtypes = [vp, _QType, vp, _QType, vp, i32, i64, i64, i64, i64, i64,
                                   i32, i32, i32, i32, i32, i32, i32, i32,
                                   C.POINTER(_Requant), vp, u32, vp]
        L.hago_qconv2d_static.restype = i32
        L.hago_qconv2d_static.argtypes = L.hago_qconv2d.argtypes
        L.hago_qconv2d_ws.restype = i32
        L.hago_qconv2d_ws.argtypes = [vp, _QType, vp, _QType, vp, i32, i64, i64, i64, i64, i64,
                                      i32, i32, i32, i32, i32, i32, i32, i32,
                                      C.POINTER(_Requant), vp, vp, i64, u32, vp]
        L.hago_qconv2d_workspace_bytes.restype = i64
        L.hago_qconv2d_workspace_bytes.argtypes = [i32, i64, i64, i64, i64, i64, i32, i32, i32, i32, i32, i32, i32]
        L.hago_bit_range.restype = i32
        L.hago_bit_range.argtypes = [i32, i32, C.POINTER(i32), C.POINTER(i32)]
        L.hago_probe_mfma_i8.restype = i32
        L.hago_probe_mfma_i8.argtypes = [vp, vp, i32, i32, vp]
        L.hago_probe_copy.restype = i32
        L.hago_probe_copy.argtypes = [vp, vp, i64, vp]
        L.hago_set_test_hook.restype = None
        L.hago_set_test_hook.argtypes = [i32, i32]
        _lib = L
    return _lib


def bit_range(bits, is_signed):
    """hago_bit_range: the inclusive code range of `bits` effective bits."""
    lo, hi = C.c_int32(), C.c_int32()
    _check(lib().hago_bit_range(int(bits), int(bool(is_signed)), C.byref(lo), C.byref(hi)))
    return lo.value, hi.value


def probe_mfma_i8(operands, sink, workgroups, iters):
    """hago_probe_mfma_i8: operands 8192 bytes, sink 4 bytes (device tensors)."""
    assert operands.numel() * operands.element_size() >= 8192 and sink.numel() * sink.element_size() >= 4
    _check(lib().hago_probe_mfma_i8(_ptr(operands), _ptr(sink), int(workgroups), int(iters), _stream()))


def probe_copy(src, dst):
    """hago_probe_copy between two device tensors of the same byte size."""
    n = src.numel() * src.element_size()
    assert n == dst.numel() * dst.element_size()
    _check(lib().hago_probe_copy(_ptr(src), _ptr(dst), n, _stream()))


def set_test_hook(key, value):
    """hago_set_test_hook: force a GEMM kernel family / tile for the following calls (tests)."""
    lib().hago_set_test_hook(int(key), int(value))


def _check(code):
    if code != 0:
        raise HagoError(code, lib().hago_status_string(code).decode())


class QType:
    """Container dtype, effective bits, signedness of the effective range, zero point."""

    def __init__(self, dtype, bits=None, is_signed=None, zero_point=0):
        self.dtype = dtype
        self.bits = {U8: 8, I8: 8, I16: 16, I32: 32, I24: 24}.get(dtype, 0) if bits is None else bits
        self.is_signed = (dtype != U8) if is_signed is None else bool(is_signed)
        self.zero_point = int(zero_point)

    def c(self):
        return _QType(self.dtype, self.bits, int(self.is_signed), self.zero_point)


class Requant:
    """Requantize parameters; multiplier/shift are int32 device tensors (multiplier None: the
    shift-only form for power-of-two scales)."""

    def __init__(self, multiplier, shift, out: QType, clip_lo=None, clip_hi=None, per_channel=None,
                 rounding=0):
        self.multiplier = multiplier
        self.shift = shift
        self.out = out
        lo, hi = bit_range(out.bits, out.is_signed)
        self.clip_lo = lo if clip_lo is None else int(clip_lo)
        self.clip_hi = hi if clip_hi is None else int(clip_hi)
        self.per_channel = int(shift.numel() > 1) if per_channel is None else int(per_channel)
        self.rounding = int(rounding)   # ROUND_UPWARD or ROUND_HALF_AWAY

    def c(self):
        return _Requant(None if self.multiplier is None else self.multiplier.data_ptr(), self.shift.data_ptr(), self.per_channel,
                        self.out.c(), self.clip_lo, self.clip_hi, self.rounding)


def _torch():
    import torch
    return torch


def _stream():
    return _torch().cuda.current_stream().cuda_stream


def _tdtype(code):
    t = _torch()
    return {U8: t.uint8, I8: t.int8, I16: t.int16, I32: t.int32, F32: t.float32, I24: t.int32}[code]


def _code(tensor):
    t = _torch()
    return {t.uint8: U8, t.int8: I8, t.int16: I16, t.int32: I32, t.float32: F32}[tensor.dtype]


def _ptr(t):
    return None if t is None else t.data_ptr()


class Prepared:
    """A library call with its arguments already marshalled; calling it re-issues the same
    launch (same buffers, same stream) with one foreign-function call."""

    __slots__ = ("_fn", "_args", "_keep", "out")

    def __init__(self, fn, args, keep, out):
        self._fn, self._args, self._keep, self.out = fn, args, keep, out

    def __call__(self):
        code = self._fn(*self._args)
        if code != 0:
            _check(code)
        return self.out


def simquant(x, scale, zero_point, q: QType, clip_lo=None, clip_hi=None, per_channel=None, out=None,
             prepare=False):
    """hago_simquant over x[outer, channels, inner] (fp32, contiguous)."""
    assert x.dim() == 3 and x.is_contiguous()
    outer, channels, inner = x.shape
    lo, hi = bit_range(q.bits, q.is_signed)
    clip_lo = lo if clip_lo is None else clip_lo
    clip_hi = hi if clip_hi is None else clip_hi
    pc = int(scale.numel() > 1) if per_channel is None else int(per_channel)
    y = _torch().empty_like(x) if out is None else out
    args = (_ptr(x), _ptr(y), outer, channels, inner, _ptr(scale), _ptr(zero_point), pc, q.c(),
            int(clip_lo), int(clip_hi), _stream())
    if prepare:
        return Prepared(lib().hago_simquant, args, (x, y, scale, zero_point), y)
    _check(lib().hago_simquant(*args))
    return y


def simquant_wrap(x, scale, zero_point, q: QType, clip_lo=None, clip_hi=None, per_channel=None, out=None,
                  prepare=False):
    """hago_simquant_wrap over x[outer, channels, inner]: simulated quantize with the overflow of q's container."""
    assert x.dim() == 3 and x.is_contiguous()
    outer, channels, inner = x.shape
    lo, hi = bit_range(min(q.bits, 25), q.is_signed)
    clip_lo = lo if clip_lo is None else clip_lo
    clip_hi = hi if clip_hi is None else clip_hi
    pc = int(scale.numel() > 1) if per_channel is None else int(per_channel)
    y = _torch().empty_like(x) if out is None else out
    args = (_ptr(x), _ptr(y), outer, channels, inner, _ptr(scale), _ptr(zero_point), pc, q.c(),
            int(clip_lo), int(clip_hi), _stream())
    if prepare:
        return Prepared(lib().hago_simquant_wrap, args, (x, y, scale, zero_point), y)
    _check(lib().hago_simquant_wrap(*args))
    return y


def simquant_batched(x, scales, zero_points, q: QType, clip_lo, clip_hi, per_channel=True, out=None,
                     prepare=False):
    """hago_simquant_batched: candidates b over x[outer, channels, inner]; scales / zero_points are
    device tensors [nbatch, channels] (or [nbatch, 1]); clip_lo / clip_hi are host sequences."""
    assert x.dim() == 3 and x.is_contiguous() and scales.is_contiguous() and zero_points.is_contiguous()
    outer, channels, inner = x.shape
    nb = len(clip_lo)
    assert len(clip_hi) == nb and scales.shape[0] == nb and zero_points.shape[0] == nb
    t = _torch()
    y = t.empty((nb,) + tuple(x.shape), dtype=t.float32, device=x.device) if out is None else out
    lo = (C.c_int32 * max(nb, 1))(*[int(v) for v in clip_lo])
    hi = (C.c_int32 * max(nb, 1))(*[int(v) for v in clip_hi])
    args = (_ptr(x), _ptr(y), outer, channels, inner, nb, _ptr(scales), _ptr(zero_points),
            int(bool(per_channel)), q.c(), C.cast(lo, C.c_void_p), C.cast(hi, C.c_void_p), _stream())
    if prepare:
        return Prepared(lib().hago_simquant_batched, args, (x, y, scales, zero_points, lo, hi), y)
    _check(lib().hago_simquant_batched(*args))
    return y


_TORCH_OF = {U8: "uint8", I8: "int8", I16: "int16", I32: "int32"}


def quantize(x, scale, zero_point, q: QType, clip_lo=None, clip_hi=None, per_channel=None, out=None,
             prepare=False):
    """hago_quantize over x[outer, channels, inner] (fp32): integer codes in q's container."""
    assert x.dim() == 3 and x.is_contiguous()
    outer, channels, inner = x.shape
    lo, hi = bit_range(q.bits, q.is_signed)
    clip_lo = lo if clip_lo is None else clip_lo
    clip_hi = hi if clip_hi is None else clip_hi
    pc = int(scale.numel() > 1) if per_channel is None else int(per_channel)
    t = _torch()
    codes = t.empty(x.shape, dtype=getattr(t, _TORCH_OF[q.dtype]), device=x.device) if out is None else out
    args = (_ptr(x), _ptr(codes), outer, channels, inner, _ptr(scale), _ptr(zero_point), pc, q.c(),
            int(clip_lo), int(clip_hi), _stream())
    if prepare:
        return Prepared(lib().hago_quantize, args, (x, codes, scale, zero_point), codes)
    _check(lib().hago_quantize(*args))
    return codes


def simquant_codes(x, scale, zero_point, q: QType, clip_lo=None, clip_hi=None, per_channel=None, out=None,
                   out_codes=None, prepare=False):
    """hago_simquant_codes over x[outer, channels, inner] (fp32): (simulated-quantized fp32, integer codes)."""
    assert x.dim() == 3 and x.is_contiguous()
    outer, channels, inner = x.shape
    lo, hi = bit_range(q.bits, q.is_signed)
    clip_lo = lo if clip_lo is None else clip_lo
    clip_hi = hi if clip_hi is None else clip_hi
    pc = int(scale.numel() > 1) if per_channel is None else int(per_channel)
    t = _torch()
    y = t.empty_like(x) if out is None else out
    codes = (t.empty(x.shape, dtype=getattr(t, _TORCH_OF[q.dtype]), device=x.device)
             if out_codes is None else out_codes)
    args = (_ptr(x), _ptr(y), _ptr(codes), outer, channels, inner, _ptr(scale), _ptr(zero_point), pc, q.c(),
            int(clip_lo), int(clip_hi), _stream())
    if prepare:
        return Prepared(lib().hago_simquant_codes, args, (x, y, codes, scale, zero_point), (y, codes))
    _check(lib().hago_simquant_codes(*args))
    return y, codes


def dequantize(codes, q: QType, scale, zero_point, per_channel=None, out=None, prepare=False):
    """hago_dequantize over codes[outer, channels, inner] in q's container: fp32."""
    assert codes.dim() == 3 and codes.is_contiguous()
    outer, channels, inner = codes.shape
    pc = int(scale.numel() > 1) if per_channel is None else int(per_channel)
    t = _torch()
    y = t.empty(codes.shape, dtype=t.float32, device=codes.device) if out is None else out
    args = (_ptr(codes), q.c(), _ptr(y), outer, channels, inner, _ptr(scale), _ptr(zero_point), pc,
            _stream())
    if prepare:
        return Prepared(lib().hago_dequantize, args, (codes, y, scale, zero_point), y)
    _check(lib().hago_dequantize(*args))
    return y


def absmax(x, per_channel=True, out=None, prepare=False):
    """hago_absmax over x[outer, channels, inner] (fp32, contiguous): thresholds [channels] or [1]."""
    assert x.dim() == 3 and x.is_contiguous()
    outer, channels, inner = x.shape
    n = channels if per_channel else 1
    thr = _torch().empty(n, dtype=_torch().float32, device=x.device) if out is None else out
    args = (_ptr(x), outer, channels, inner, int(bool(per_channel)), _ptr(thr), _stream())
    if prepare:
        return Prepared(lib().hago_absmax, args, (x, thr), thr)
    _check(lib().hago_absmax(*args))
    return thr


def requantize(acc, rq: Requant, out=None, prepare=False):
    """hago_requantize over acc[outer, channels, inner] (int32 / int16)."""
    assert acc.dim() == 3 and acc.is_contiguous()
    outer, channels, inner = acc.shape
    if out is None:
        out = _torch().empty(acc.shape, dtype=_tdtype(rq.out.dtype), device=acc.device)
    st = rq.c()
    args = (_ptr(acc), _code(acc), outer, channels, inner, C.byref(st), _ptr(out), _stream())
    if prepare:
        return Prepared(lib().hago_requantize, args, (acc, rq, st, out), out)
    _check(lib().hago_requantize(*args))
    return out


def qdense(a, a_t: QType, w, w_t: QType, bias=None, acc_dtype=I32, rq: Requant | None = None,
           flags=0, out=None, prepare=False):
    """hago_qdense: a [M,K] (uint8/int8), w [N,K] int8 -> [M,N].

    prepare=True returns a Prepared call instead of launching."""
    assert a.dim() == 2 and w.dim() == 2 and a.is_contiguous() and w.is_contiguous()
    M, K = a.shape
    N = w.shape[0]
    assert w.shape[1] == K
    if out is None:
        dt = _tdtype(rq.out.dtype) if rq is not None else _tdtype(acc_dtype)
        out = _torch().empty((M, N), dtype=dt, device=a.device)
    st = rq.c() if rq is not None else None
    args = (_ptr(a), a_t.c(), _ptr(w), w_t.c(), _ptr(bias), M, N, K, acc_dtype,
            C.byref(st) if st is not None else None, _ptr(out), flags, _stream())
    if prepare:
        return Prepared(lib().hago_qdense, args, (a, w, bias, rq, st, out), out)
    _check(lib().hago_qdense(*args))
    return out


def _conv_dims(a, w, layout):
    if layout == NCHW:
        B, Cc, H, W = a.shape
        O, _, KH, KW = w.shape
    else:
        B, H, W, Cc = a.shape
        O, KH, KW, _ = w.shape
    return B, Cc, H, W, O, KH, KW


def qconv2d_workspace_bytes(a_shape, w_shape, layout=NCHW, stride=(1, 1), pad=(0, 0), groups=1):
    """hago_qconv2d_workspace_bytes for tensors of these shapes."""
    class _S:
        def __init__(self, shape):
            self.shape = tuple(shape)
    B, Cc, H, W, O, KH, KW = _conv_dims(_S(a_shape), _S(w_shape), layout)
    return int(lib().hago_qconv2d_workspace_bytes(layout, B, Cc, H, W, O, KH, KW, stride[0], stride[1],
                                                  pad[0], pad[1], groups))


def qconv2d(a, a_t: QType, w, w_t: QType, bias=None, layout=NCHW, stride=(1, 1), pad=(0, 0),
            groups=1, acc_dtype=I32, rq: Requant | None = None, flags=0, out=None, prepare=False,
            workspace=None, static_scratch=False):
    """hago_qconv2d: NCHW a [B,C,H,W], w [O,C/g,KH,KW]; NHWC a [B,H,W,C], w [O,KH,KW,C/g].

    With `workspace` (a uint8 device tensor of at least qconv2d_workspace_bytes(...) bytes, or an
    empty one when that is 0) the call goes to hago_qconv2d_ws; with static_scratch=True to
    hago_qconv2d_static."""
    assert a.dim() == 4 and w.dim() == 4 and a.is_contiguous() and w.is_contiguous()
    B, Cc, H, W, O, KH, KW = _conv_dims(a, w, layout)
    OH = (H + 2 * pad[0] - KH) // stride[0] + 1
    OW = (W + 2 * pad[1] - KW) // stride[1] + 1
    if out is None:
        dt = _tdtype(rq.out.dtype) if rq is not None else _tdtype(acc_dtype)
        shape = (B, O, max(OH, 0), max(OW, 0)) if layout == NCHW else (B, max(OH, 0), max(OW, 0), O)
        out = _torch().empty(shape, dtype=dt, device=a.device)
    st = rq.c() if rq is not None else None
    args = (_ptr(a), a_t.c(), _ptr(w), w_t.c(), _ptr(bias), layout, B, Cc, H, W, O,
            KH, KW, stride[0], stride[1], pad[0], pad[1], groups, acc_dtype,
            C.byref(st) if st is not None else None, _ptr(out))
    if workspace is not None:
        fn = lib().hago_qconv2d_ws
        args += (_ptr(workspace) if workspace.numel() else None, workspace.numel() * workspace.element_size(),
                 flags, _stream())
    else:
        fn = lib().hago_qconv2d_static if static_scratch else lib().hago_qconv2d
        args += (flags, _stream())
    if prepare:
        return Prepared(fn, args, (a, w, bias, rq, st, out, workspace), out)
    _check(fn(*args))
    return out
