"""hago_qconv2d_static, the convolution entry point that allocates nothing (its scratch is a fixed
array of static device memory): called through the C ABI, its output must equal
hago_qconv2d_ws's (caller-owned workspace) bit for bit, and the oracle's, on two calls in a row,
the second on a smaller input, so that whatever the first call left in the shared array is seen
not to matter."""
import ctypes as C

import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

from gpu_util import *  # noqa: E402,F401,F403
from paper_2103_14949_amd import binding, datagen


def _call_static(L, a, a_t, w, w_t, bias, layout, stride, pad, acc_dtype, rq, out):
    """One hago_qconv2d_static call with hand-marshalled arguments (no binding helper in between)."""
    if layout == hago.NCHW:
        B, Cc, H, W = a.shape
        O, _, KH, KW = w.shape
    else:
        B, H, W, Cc = a.shape
        O, KH, KW, _ = w.shape
    st = rq.c() if rq is not None else None
    code = L.hago_qconv2d_static(a.data_ptr(), a_t.c(), w.data_ptr(), w_t.c(),
                                 None if bias is None else bias.data_ptr(), layout, B, Cc, H, W, O, KH, KW,
                                 stride[0], stride[1], pad[0], pad[1], 1, acc_dtype,
                                 C.byref(st) if st is not None else None, out.data_ptr(), 0,
                                 torch.cuda.current_stream().cuda_stream)
    assert code == 0, L.hago_status_string(code)


def _case(rng, B, Cc, H, W, O, k, adt, za, acc16):
    a = (rng.integers(0, 256, (B, Cc, H, W)).astype(np.uint8) if adt == np.uint8
         else rng.integers(-128, 128, (B, Cc, H, W)).astype(np.int8))
    w = rng.integers(-127, 128, (O, Cc, k, k)).astype(np.int8)
    bias = rng.integers(-10 ** 5, 10 ** 5, O).astype(np.int32)
    mult, shift = datagen.requant_params(rng, np.full(O, 74.0 * 73.0 * np.sqrt(Cc * k * k)), 40.0)
    return dict(a=a, w=w, bias=bias, mult=mult, shift=shift, za=za, pad=(k // 2, k // 2), acc16=acc16)


@pytest.mark.parametrize("layout", ["nchw", "nhwc"])
def test_static_scratch_matches_workspace_entry_point_twice(layout):
    L = hago.lib()
    rng = np.random.default_rng(20260 + (layout == "nhwc"))
    # first a larger input (several tiles, ragged in pixels and channels), then a smaller one whose
    # rewritten operands cover only the start of the array the first call filled
    cases = [_case(rng, 3, 72, 20, 28, 80, 3, np.uint8, 131, False),
             _case(rng, 1, 24, 9, 12, 40, 3, np.int8, -3, True)]
    for i, c in enumerate(cases):
        lay_g, lay_r = (hago.NCHW, ref.NCHW) if layout == "nchw" else (hago.NHWC, ref.NHWC)
        a = c["a"] if layout == "nchw" else np.ascontiguousarray(c["a"].transpose(0, 2, 3, 1))
        w = c["w"] if layout == "nchw" else np.ascontiguousarray(c["w"].transpose(0, 2, 3, 1))
        a_t, w_t = act_qtype(a, c["za"]), hago.QType(hago.I8)
        acc_g, acc_r = (hago.I16, ref.I16) if c["acc16"] else (hago.I32, ref.I32)
        for with_rq in (True, False):
            rq_g = gpu_requant(c["mult"], c["shift"]) if with_rq else None
            rq_r = ref_requant(c["mult"], c["shift"]) if with_rq else None
            da, dw, db = dev(a), dev(w), dev(c["bias"])
            need = hago.qconv2d_workspace_bytes(a.shape, w.shape, lay_g, (1, 1), c["pad"], 1)
            assert 0 < need <= hago.STATIC_SCRATCH_BYTES
            ws = torch.full((need,), 0x5A, dtype=torch.uint8, device=DEV)
            want_ws = hago.qconv2d(da, a_t, dw, w_t, db, lay_g, (1, 1), c["pad"], 1, acc_g, rq_g, workspace=ws)
            out = torch.full_like(want_ws, 77)
            _call_static(L, da, a_t, dw, w_t, db, lay_g, (1, 1), c["pad"], acc_g, rq_g, out)
            got, want_ws = host(out), host(want_ws)
            assert_same(got, want_ws, f"static vs workspace, call {i}, {layout}, requant={with_rq}")
            want = ref.qconv2d(a, c["za"], w, c["bias"], lay_r, (1, 1), c["pad"], 1, acc_r, rq_r)
            assert_same(got, want, f"static vs oracle, call {i}, {layout}, requant={with_rq}")


def test_static_scratch_config2_and_config3_as_specified():
    """The two benchmark convolutions at their specified sizes, back to back through the fixed array."""
    L = hago.lib()
    c = datagen.config2()
    rq = ref_requant(c["mult"], c["shift"], True, 0, (0, 255))
    want = ref.qconv2d(c["a"], 0, c["w"], None, ref.NCHW, (1, 1), (1, 1), 1, ref.I32, rq)
    out = torch.empty(want.shape, dtype=torch.uint8, device=DEV)
    _call_static(L, dev(c["a"]), act_qtype(c["a"], 0), dev(c["w"]), hago.QType(hago.I8), None, hago.NCHW, (1, 1),
                 (1, 1), hago.I32, gpu_requant(c["mult"], c["shift"], True, 0, (0, 255)), out)
    assert_same(host(out), want, "config 2 through the fixed array")
    c = datagen.config3()
    want = ref.qconv2d(c["a"], 0, c["w"], None, ref.NCHW, (1, 1), (1, 1), 1, ref.I16)
    out = torch.empty(want.shape, dtype=torch.int16, device=DEV)
    _call_static(L, dev(c["a"]), hago.QType(hago.I8, 4, False, 0), dev(c["w"]), hago.QType(hago.I8, 4, True, 0), None,
                 hago.NCHW, (1, 1), (1, 1), hago.I16, None, out)
    assert_same(host(out), want, "config 3 through the fixed array")


def test_static_scratch_refuses_what_does_not_fit():
    """Beyond the array's size the call is refused on the host (status 8) and nothing is written."""
    L = hago.lib()
    B = 400   # 400 x 58 x 58 x 64 bytes of rewritten activations: more than 64 MiB
    assert hago.qconv2d_workspace_bytes((B, 64, 56, 56), (64, 64, 3, 3), hago.NCHW, (1, 1), (1, 1)) > hago.STATIC_SCRATCH_BYTES
    out = torch.full((16,), 9, dtype=torch.uint8, device=DEV)
    a_t, w_t = binding._QType(hago.U8, 8, 0, 0), binding._QType(hago.I8, 8, 1, 0)
    code = L.hago_qconv2d_static(out.data_ptr(), a_t, out.data_ptr(), w_t, None, hago.NCHW, B, 64, 56, 56, 64, 3, 3,
                                 1, 1, 1, 1, 1, hago.I32, None, out.data_ptr(), 0, None)
    assert code == 8 and b"scratch" in L.hago_status_string(code)
    assert (host(out) == 9).all()
