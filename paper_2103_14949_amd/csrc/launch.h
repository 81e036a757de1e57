// Host-side launch entry points of the kernel families; called only from the
// C ABI layer after all arguments have been validated.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>

namespace hago {

// The dynamic-LDS limit of a kernel is a per-device attribute.  `done` holds one bit per device
// (ids modulo 64) on which it has been raised; concurrent first calls may both set it, which is
// harmless.
inline hipError_t raise_lds_limit(const void* kern, int lds_bytes, std::atomic<uint64_t>& done) {
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  const uint64_t bit = 1ull << (dev & 63);
  if (done.load(std::memory_order_acquire) & bit) return hipSuccess;
  e = hipFuncSetAttribute(kern, hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes);
  if (e == hipSuccess) done.fetch_or(bit, std::memory_order_release);
  return e;
}


struct RequantArgs {
  const int32_t* multiplier;  // device
  const int32_t* shift;       // device
  int32_t per_channel;
  int32_t out_unsigned;  // 1: uint8 container, 0: int8
  int32_t z_out, clip_lo, clip_hi;
  int32_t half_away;  // 1: nearest with halves away from zero; 0: ties toward +infinity
};

// fp32 simulated quantize over [outer, channels, inner].
hipError_t launch_simquant(const float* x, float* y, int64_t outer, int64_t channels, int64_t inner,
                           const float* scale, const int32_t* zp, int per_channel, int32_t clip_lo,
                           int32_t clip_hi, hipStream_t st);

// simulated quantize with the overflow of a wrap_bits-wide integer type (signed: two's complement).
hipError_t launch_simquant_wrap(const float* x, float* y, int64_t outer, int64_t channels, int64_t inner,
                                const float* scale, const int32_t* zp, int per_channel, int32_t wrap_bits,
                                int32_t wrap_signed, int32_t clip_lo, int32_t clip_hi, hipStream_t st);

// nbatch (<= 16) candidate parameter sets over one tensor: y[nbatch][outer][channels][inner];
// scale / zp: [nbatch][channels] (or [nbatch]); clip_lo / clip_hi: host arrays [nbatch].
hipError_t launch_simquant_batched(const float* x, float* y, int64_t outer, int64_t channels,
                                   int64_t inner, int32_t nbatch, const float* scale,
                                   const int32_t* zp, int per_channel, const int32_t* clip_lo,
                                   const int32_t* clip_hi, hipStream_t st);

// op 0: quantize (fp32 -> codes), 1: dequantize (codes -> fp32), 2: quantize plus the
// simulated_quantize value into out2, over [outer, channels, inner].
// container: 0 int8, 1 uint8, 2 int16, 3 int32.
hipError_t launch_quant(const void* in, void* out, float* out2, int container, int op, int64_t outer,
                        int64_t channels, int64_t inner, const float* scale, const int32_t* zp,
                        int per_channel, int32_t clip_lo, int32_t clip_hi, hipStream_t st);

// max-abs calibration over [outer, channels, inner]: thr[channels] (or [1]).
hipError_t launch_absmax(const float* x, int64_t outer, int64_t channels, int64_t inner,
                         int per_channel, float* thr, hipStream_t st);

// standalone requantize over [outer, channels, inner]; acc16 != 0: int16 input.
hipError_t launch_requantize(const void* acc, int acc16, int64_t outer, int64_t channels,
                             int64_t inner, const RequantArgs& rq, void* out, hipStream_t st);

struct ConvGeom {
  int32_t B, C, H, W, O, OH, OW, KH, KW, stride_h, stride_w, pad_h, pad_w;
  int32_t nhwc;
};

struct GemmArgs {
  const void* act;    // activations, uint8 or int8 container
  const int8_t* wgt;  // weights [N, K] (conv: [O, C*KH*KW] in the layout's own order)
  const int32_t* bias;
  void* out;
  int32_t M, N, K;
  int32_t operand16;     // 1: both operands are int16 (act and wgt point to int16 data)
  int32_t act_unsigned;  // 1: uint8 container
  int32_t act_zero_point;
  int32_t acc16;           // reduce accumulator modulo 2^16 (raw results are int16)
  int32_t acc_wrap_shift;  // 32 - accumulator bits: 0 (int32), 16 (int16) or 8 (24 bits, kept in an int32)
  int32_t has_rq;          // 0: store raw accumulators
  RequantArgs rq;
};

// int16 x int16 operands (dense, or a groups == 1 convolution when cg != nullptr) on the vector ALUs.
hipError_t launch_qgemm16(const GemmArgs& g, const ConvGeom* cg, hipStream_t st);
// C[M,N] = act[M,K] x wgt[N,K]^T on int8 MFMA; out row-major [M,N].
hipError_t launch_qdense(const GemmArgs& g, hipStream_t st);

// Scratch of the fast implicit-GEMM convolution (groups == 1): the operand rewrite writes
// [weights as [O][KH*KW][Cp], rounded up to 256 bytes][padded NHWC activations, same rounding]
// into it and the GEMM streams both from there.  Returns the byte count for a geometry, or -1
// when the geometry is outside what that path indexes with 32 bits (the generic kernel, which
// needs no scratch, serves it).
int64_t qconv_workspace_bytes(const ConvGeom& cg);
// Implicit-GEMM convolution, groups == 1.  ws: device scratch of at least
// qconv_workspace_bytes(cg) bytes, 256-byte aligned, or nullptr (then, unless one of the
// scratch-free special kernels takes the geometry, the generic register-staged kernel runs).
// weights_ready: the weight part of ws already holds this call's weights (same tensor, same
// geometry), so only the activations are rewritten.
hipError_t launch_qconv_gemm(const GemmArgs& g, const ConvGeom& cg, void* ws, bool weights_ready,
                             hipStream_t st);
// The library's fixed scratch array on the current device (static device memory: nothing is
// allocated or freed, the address never changes) and its capacity in bytes.
hipError_t static_scratch(void** ptr, int64_t* capacity);
hipError_t launch_conv_prepack(const GemmArgs& g, const ConvGeom& cg, int32_t Cp, uint8_t* act_out,
                               int8_t* wgt_out, bool skip_weights, hipStream_t st);
// Test hooks (see hago_set_test_hook): which GEMM kernel family and tile serve the next calls.
enum { kHookGemmPath = 0, kHookDmaTile = 1, kHookGenericTile = 2, kNumHooks = 3 };
void set_test_hook(int key, int value);
// 3x3 stride-1 pad-1 NCHW convolution in one launch, no scratch; false when the geometry is not
// that kernel's (nothing is launched then).
bool try_qconv3x3_nchw(const GemmArgs& g, const ConvGeom& cg, hipStream_t st, hipError_t* err);
// 1x1 stride-1 unpadded NCHW convolution straight from the caller's buffers; false when the
// geometry is not that kernel's (nothing is launched then).
bool try_qconv_pointwise_nchw(const GemmArgs& g, const ConvGeom& cg, hipStream_t st, hipError_t* err);
// depthwise convolution (groups == C == O), no MFMA.
hipError_t launch_qconv_depthwise(const GemmArgs& g, const ConvGeom& cg, hipStream_t st);

}  // namespace hago
