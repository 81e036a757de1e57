"""The entry points launch kernels only (no allocation, no memset, no synchronisation), so a caller can
record them into a HIP graph.  A graph of several operators is replayed three times with eager work and
synchronisations in between, and every replay must reproduce the eager results bit for bit."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

from gpu_util import *  # noqa: E402,F401,F403
from paper_2103_14949_amd import datagen


def rnd_act(rng, shape, dt):
    return rng.integers(0, 256, shape).astype(np.uint8) if dt == np.uint8 else rng.integers(-128, 128, shape).astype(np.int8)


def rnd_w(rng, shape):
    return rng.integers(-127, 128, shape).astype(np.int8)


def test_operators_replay_identically_from_a_captured_graph():
    rng = np.random.default_rng(11)
    # dense (streaming MFMA kernel), 3x3 convolution (one launch), depthwise, requantize, simquant, absmax
    c5 = datagen.config5_layer(1, M=512)
    a5, w5, b5 = dev(c5["a"]), dev(c5["w"]), dev(c5["bias"])
    rq5 = gpu_requant(c5["mult"], c5["shift"])
    a_t5 = act_qtype(c5["a"], c5["z_a"])
    xa = rnd_act(rng, (2, 64, 12, 16), np.uint8)
    xw = rnd_w(rng, (48, 64, 3, 3))
    mult, shift = datagen.requant_params(rng, np.full(48, 74.0 * 73.0 * 24.0), 40.0)
    da, dw_ = dev(xa), dev(xw)
    rqc = gpu_requant(mult, shift)
    dwt = dev(rnd_w(rng, (64, 1, 3, 3)))
    acc = dev(rng.integers(-2 ** 20, 2 ** 20, (2, 48, 640)).astype(np.int32))
    x = dev(rng.standard_normal((2, 48, 1024)).astype(np.float32))
    sc = dev(rng.uniform(0.02, 0.04, 48).astype(np.float32))
    zp = dev(np.zeros(48, np.int32))
    need = hago.qconv2d_workspace_bytes((2, 60, 12, 16), (48, 60, 3, 3), hago.NCHW, (1, 1), (1, 1))
    ws = torch.empty(need, dtype=torch.uint8, device=DEV)
    xa60, xw60 = dev(rnd_act(rng, (2, 60, 12, 16), np.uint8)), dev(rnd_w(rng, (48, 60, 3, 3)))

    outs = {
        "dense": torch.empty((512, c5["w"].shape[0]), dtype=torch.int8, device=DEV),
        "conv": torch.empty((2, 48, 12, 16), dtype=torch.int8, device=DEV),
        "conv_ws": torch.empty((2, 48, 12, 16), dtype=torch.int8, device=DEV),
        "dw": torch.empty((2, 64, 12, 16), dtype=torch.int32, device=DEV),
        "rq": torch.empty((2, 48, 640), dtype=torch.int8, device=DEV),
        "sq": torch.empty((2, 48, 1024), dtype=torch.float32, device=DEV),
        "am": torch.empty(48, dtype=torch.float32, device=DEV),
    }

    def run():
        hago.qdense(a5, a_t5, w5, hago.QType(hago.I8), b5, hago.I32, rq5, out=outs["dense"])
        hago.qconv2d(da, act_qtype(xa, 128), dw_, hago.QType(hago.I8), None, hago.NCHW, (1, 1), (1, 1), 1, hago.I32,
                     rqc, out=outs["conv"])
        hago.qconv2d(xa60, act_qtype(xa, 128), xw60, hago.QType(hago.I8), None, hago.NCHW, (1, 1), (1, 1), 1,
                     hago.I32, rqc, out=outs["conv_ws"], workspace=ws)
        hago.qconv2d(da, act_qtype(xa, 128), dwt, hago.QType(hago.I8), None, hago.NCHW, (1, 1), (1, 1), 64,
                     hago.I32, None, out=outs["dw"])
        hago.requantize(acc, rqc, out=outs["rq"])
        hago.simquant(x, sc, zp, hago.QType(hago.I8), out=outs["sq"])
        hago.absmax(x, True, out=outs["am"])

    run()   # eager: also raises the kernels' LDS limits, which must not happen inside a capture
    torch.cuda.synchronize()
    eager = {k: v.clone() for k, v in outs.items()}

    side = torch.cuda.Stream()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(g, stream=side):
            run()
    for replay in range(3):
        for v in outs.values():
            v.zero_()
        ws.fill_(0x3C + replay)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        for k in outs:
            assert torch.equal(outs[k].view(torch.uint8), eager[k].view(torch.uint8)), f"{k}, replay {replay}"
        # the program's own eager work between replays
        hago.simquant(x, sc, zp, hago.QType(hago.I8))
        torch.cuda.synchronize()
