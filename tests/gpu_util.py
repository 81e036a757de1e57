"""Helpers shared by the GPU parity tests: move seeded host arrays to the GPU,
call libhago through its binding, run the CPU oracle on the same arrays."""
import numpy as np
import torch

import paper_2103_14949_amd as hago
from oracle import hago_ref as ref

DEV = "cuda:0"


def dev(x):
    return None if x is None else torch.from_numpy(np.ascontiguousarray(x)).to(DEV)


def host(t):
    torch.cuda.synchronize()
    return t.cpu().numpy()


def act_qtype(a, z, bits=8, is_signed=None):
    dt = hago.U8 if a.dtype == np.uint8 else hago.I8
    return hago.QType(dt, bits, (dt == hago.I8) if is_signed is None else is_signed, z)


def gpu_requant(mult, shift, out_u8=False, z_out=0, clip=None, bits=8, rounding=0):
    q = hago.QType(hago.U8 if out_u8 else hago.I8, bits, not out_u8, z_out)
    lo, hi = clip if clip is not None else (None, None)
    return hago.Requant(dev(np.asarray(mult, np.int32)), dev(np.asarray(shift, np.int32)), q, lo, hi,
                        rounding=rounding)


def ref_requant(mult, shift, out_u8=False, z_out=0, clip=None, rounding=0):
    lo, hi = clip if clip is not None else ((0, 255) if out_u8 else (-128, 127))
    return ref.Requant(mult, shift, out_dtype=ref.U8 if out_u8 else ref.I8, out_zero_point=z_out,
                       clip_lo=lo, clip_hi=hi, rounding=rounding)


def assert_same(got, want, what=""):
    got = np.asarray(got)
    want = np.asarray(want)
    assert got.shape == want.shape and got.dtype == want.dtype, (what, got.shape, want.shape, got.dtype, want.dtype)
    if not np.array_equal(got, want):
        bad = np.argwhere(got != want)
        i = tuple(bad[0])
        raise AssertionError(f"{what}: {len(bad)} of {got.size} differ; first at {i}: got {got[i]} want {want[i]}")


def assert_same_bits(got, want, what=""):
    """Bitwise equality of float arrays, except that any NaN matches any NaN."""
    g = got.view(np.uint32).copy()
    w = want.view(np.uint32).copy()
    both_nan = np.isnan(got) & np.isnan(want)
    g[both_nan] = 0
    w[both_nan] = 0
    assert_same(g, w, what)


# Which convolution entry point the parity tests call (set by the `conv_entry` fixture):
#   "plain"  hago_qconv2d (no scratch memory)
#   "ws"     hago_qconv2d_ws with a workspace of exactly the queried size, filled with garbage
CONV_ENTRY = {"name": "plain"}


def qconv2d(a, a_t, w, w_t, bias=None, layout=None, stride=(1, 1), pad=(0, 0), groups=1, acc_dtype=None,
            rq=None, flags=0):
    """hago.qconv2d through the entry point under test."""
    layout = hago.NCHW if layout is None else layout
    acc_dtype = hago.I32 if acc_dtype is None else acc_dtype
    if CONV_ENTRY["name"] == "plain":
        return hago.qconv2d(a, a_t, w, w_t, bias, layout, stride, pad, groups, acc_dtype, rq, flags)
    need = hago.qconv2d_workspace_bytes(a.shape, w.shape, layout, stride, pad, groups)
    assert need >= 0
    ws = torch.full((need,), 0xA5, dtype=torch.uint8, device=DEV)
    assert need == 0 or ws.data_ptr() % 256 == 0
    return hago.qconv2d(a, a_t, w, w_t, bias, layout, stride, pad, groups, acc_dtype, rq, flags, workspace=ws)
