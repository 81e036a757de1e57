"""MI355X-native quantized operators of HAGO (arXiv 2103.14949).

The package is a thin ctypes binding over ``libhago.so`` (hand-written HIP
kernels behind a C ABI, see ``include/hago.h``).  Every operator runs in those
kernels; Python only marshals arguments.  PyTorch supplies device memory and
streams.
"""
from .binding import (  # noqa: F401
    HagoError, QType, Requant, Prepared, lib, library_path,
    simquant, simquant_batched, simquant_wrap, requantize, qdense, qconv2d, qconv2d_workspace_bytes, absmax, quantize,
    dequantize, simquant_codes, bit_range, set_test_hook, probe_mfma_i8, probe_copy,
    U8, I8, I16, I32, F32, I24, NCHW, NHWC, STRICT_ACC16, WS_WEIGHTS_READY, STATIC_SCRATCH_BYTES, ROUND_UPWARD, ROUND_HALF_AWAY,
    HOOK_GEMM_PATH, HOOK_STREAM_TILE, HOOK_GENERAL_TILE,
)
