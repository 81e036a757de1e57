"""Seeded synthetic inputs for the five benchmark configurations.

This module only DRAWS inputs (numpy, on the host).  It contains none of the
quantization arithmetic: integer tensors are drawn directly from the
distributions that quantized activations / weights have, and requantize
parameters are random Q31 multipliers with a shift picked from the
accumulator's expected magnitude.  The same arrays feed the CPU oracle (in the
tests) and the GPU library.

The tensors stand in for the paper's workloads (ImageNet CNN layers, a
MobileNet block, BERT-base dense layers): same shapes, plausible value
distributions, no dataset and no trained weights.
"""
from __future__ import annotations

import numpy as np

SEED0 = 0x4841474F  # "HAGO"


def rng_for(config: int, stream: int = 0) -> np.random.Generator:
    return np.random.default_rng([SEED0 + config, stream])


def uniform_int(rng, lo, hi, shape, dtype):
    return rng.integers(lo, hi + 1, size=shape).astype(dtype)


def rounded_normal_int8(rng, shape, sigma, limit=127):
    """int8 values ~ round(N(0, sigma)) clipped to +-limit (sigma scalar or per-row array)."""
    x = rng.standard_normal(size=shape, dtype=np.float32)
    x = np.rint(x * np.asarray(sigma, dtype=np.float32))
    return np.clip(x, -limit, limit).astype(np.int8)


def rounded_normal_uint8(rng, shape, mean, sigma):
    x = rng.standard_normal(size=shape, dtype=np.float32)
    return np.clip(np.rint(x * np.float32(sigma) + np.float32(mean)), 0, 255).astype(np.uint8)


def requant_params(rng, acc_sigma, target_sigma):
    """Random Q31 multipliers in [2^30, 2^31) and, per channel, the shift that brings
    an accumulator of standard deviation acc_sigma[c] to about target_sigma."""
    acc_sigma = np.maximum(np.asarray(acc_sigma, dtype=np.float64).reshape(-1), 1e-9)
    mult = rng.integers(2 ** 30, 2 ** 31, size=acc_sigma.size).astype(np.int64)
    shift = np.rint(np.log2(mult / 2.0 ** 31 * acc_sigma / target_sigma))
    shift = np.clip(shift, 0, 31).astype(np.int32)
    return mult.astype(np.int32), shift


def _acc_sigma(a_centered_sq_mean, w):
    """sqrt(E[(a - z)^2] * sum_k w[n,k]^2) per output channel."""
    w2 = (w.astype(np.float64).reshape(w.shape[0], -1) ** 2).sum(axis=1)
    return np.sqrt(a_centered_sq_mean * w2)


def config1(M=64, variant="as_specified"):
    """Single dense layer: u8 [M,256] x i8 [128,256] -> i8, per-channel requantize."""
    r = rng_for(1)
    a = uniform_int(r, 0, 255, (M, 256), np.uint8)
    w = uniform_int(r, -127, 127, (128, 256), np.int8)
    mult = r.integers(2 ** 30, 2 ** 31, size=128).astype(np.int32)
    if variant == "as_specified":
        shift = r.integers(0, 16, size=128).astype(np.int32)      # mostly saturating
    else:
        shift = r.integers(10, 14, size=128).astype(np.int32)     # discriminating
    return dict(a=a, z_a=128, w=w, mult=mult, shift=shift, out_u8=False, z_out=0,
                clip=(-128, 127))


def config2(B=1, z_a=0):
    """ResNet-style 3x3 conv, NCHW 64x56x56 -> 64, u8 in, fused requantize + ReLU to u8."""
    r = rng_for(2)
    a = uniform_int(r, 0, 255, (B, 64, 56, 56), np.uint8)
    w = rounded_normal_int8(r, (64, 64, 3, 3), 40.0)
    e2 = float(((a[:1].astype(np.float64) - z_a) ** 2).mean())
    mult, shift = requant_params(r, _acc_sigma(e2, w), 255.0 / 3.0)
    return dict(a=a, z_a=z_a, w=w, mult=mult, shift=shift, out_u8=True, z_out=0, clip=(0, 255),
                stride=(1, 1), pad=(1, 1))


def config3(B=8, adversarial=False):
    """int16 accumulation: 3x3 conv 128x28x28 -> 128, 4-bit operands in int8 containers."""
    r = rng_for(3)
    if adversarial:
        a = np.full((B, 128, 28, 28), 15, np.int8)
        w = np.full((128, 128, 3, 3), 7, np.int8)
    else:
        a = uniform_int(r, 0, 15, (B, 128, 28, 28), np.int8)
        w = uniform_int(r, -7, 7, (128, 128, 3, 3), np.int8)
    return dict(a=a, z_a=0, w=w, a_bits=4, w_bits=4, stride=(1, 1), pad=(1, 1))


def config4(B=32):
    """MobileNet block: depthwise 3x3 on 144x56x56 int8, pointwise 144 -> 24, simquant input."""
    r = rng_for(4)
    a = rounded_normal_int8(r, (B, 144, 56, 56), 40.0)
    w_dw = uniform_int(r, -127, 127, (144, 1, 3, 3), np.int8)
    e2 = float((a[:1].astype(np.float64) ** 2).mean())
    m_dw, s_dw = requant_params(r, _acc_sigma(e2, w_dw), 127.0 / 3.0)
    w_pw = uniform_int(r, -127, 127, (24, 144, 1, 1), np.int8)
    # the pointwise input is the depthwise output, which has about the target spread
    m_pw, s_pw = requant_params(r, _acc_sigma((127.0 / 3.0) ** 2, w_pw), 127.0 / 3.0)
    return dict(a=a, z_a=0, w_dw=w_dw, mult_dw=m_dw, shift_dw=s_dw, w_pw=w_pw, mult_pw=m_pw,
                shift_pw=s_pw, clip=(-128, 127), z_out=0)


def config4_simquant(B=32):
    """fp32 [B,144,56,56] ~ N(0,1) with per-channel scales of the size max-abs calibration
    gives for such data (max |x| of ~1e5 normal samples is 4.2 .. 5.2; 8 signed bits)."""
    r = rng_for(4, 1)
    x = r.standard_normal(size=(B, 144, 56, 56), dtype=np.float32)
    scale = (r.uniform(4.2, 5.2, size=144) / 128.0).astype(np.float32)
    zp = np.zeros(144, np.int32)
    return dict(x=x, scale=scale, zp=zp, clip=(-128, 127))


BERT_LAYERS = ((768, 2304), (768, 768), (768, 3072), (3072, 768))  # (K, N)


def config5_layer(idx, M=4096):
    """BERT-base dense layer idx: u8 activations (asymmetric), per-channel symmetric int8
    weights, int32 accumulate, per-channel requantize to int8."""
    K, N = BERT_LAYERS[idx]
    r = rng_for(5, idx)
    z_a = int(r.integers(118, 139))
    a = rounded_normal_uint8(r, (M, K), z_a, 255.0 / 9.4)
    sigma_rows = 128.0 / r.uniform(3.0, 4.0, size=(N, 1))
    w = rounded_normal_int8(r, (N, K), sigma_rows)
    e2 = float(((a[:256].astype(np.float64) - z_a) ** 2).mean())
    mult, shift = requant_params(r, _acc_sigma(e2, w), 127.0 / 3.0)
    bias = np.zeros(N, np.int32)
    return dict(a=a, z_a=z_a, w=w, bias=bias, mult=mult, shift=shift, out_u8=False, z_out=0,
                clip=(-128, 127))
