/*
 * hago.h -- C ABI of libhago: the quantized-operator hot path of HAGO
 * (arXiv 2103.14949, "Automated Backend-Aware Post-Training Quantization")
 * as hand-written HIP kernels for AMD MI355X (gfx950).
 *
 * The library exports the operators the paper's realization pass produces and
 * its search loop executes:
 *   hago_simquant   -- simulated_quantize (Sec. 4.2; Eq. 3; Sec. 5.2)
 *   hago_qdense     -- integer dense, integer accumulate, fused requantize
 *   hago_qconv2d    -- integer conv2d (groups == 1 or depthwise), same epilogue
 *   hago_requantize -- the standalone requantize operator (Sec. 6.1, 6.2)
 *   hago_simquant_batched -- several candidate settings over one tensor (Sec. 6.3)
 *   hago_absmax     -- max-abs calibration thresholds (Eq. 2)
 *   hago_quantize, hago_dequantize -- fp32 <-> integer codes (Sec. 6.1; Eq. 3)
 *   hago_simquant_codes -- simulated_quantize plus its integer codes, one pass
 *   hago_simquant_wrap  -- simulated_quantize with the overflow of the simulated
 *                          integer type (Sec. 5.2)
 * and the operand / accumulator variants the paper names: int16 x int16
 * operands, 24-bit accumulators (Sec. 4.1), shift-only requantize for
 * power-of-two scales (Sec. 5.1).
 *
 * Conventions common to every call
 *   - Pointers marked "device" are GPU addresses valid on the current HIP
 *     device; "host" are ordinary pointers.  The caller owns every buffer it
 *     passes: the library never frees or keeps such a pointer after returning.
 *   - No entry point allocates, frees or keeps device memory, and none waits
 *     for the device.  The one operator that wants scratch memory, the
 *     groups == 1 convolution (it rewrites its operands before the matrix
 *     cores read them), takes it from the caller: hago_qconv2d_ws.
 *   - A call is kernel launches on `stream` and nothing else, so it may be
 *     recorded into a HIP graph.  The first call that reaches a kernel with a
 *     large LDS footprint raises that kernel's limit on the current device
 *     (hipFuncSetAttribute): make one ordinary call of the same operator and
 *     geometry before capturing.
 *   - Tensors are dense and contiguous in the stated order.  `out` must not
 *     overlap any input.  A tensor with zero elements may be passed as NULL.
 *   - `stream` is the caller's hipStream_t (NULL = the default stream).  Calls
 *     enqueue work on it and return without synchronizing.
 *   - Every argument error is detected on the host BEFORE anything is
 *     launched and reported as a status code; nothing is written in that
 *     case.  The CONTENTS of device arrays (multiplier, shift, scale) cannot
 *     be inspected without a synchronizing copy and are the caller's
 *     contract: multiplier in [0, 2^31), shift in [0, 31], scale finite and
 *     non-zero.
 *   - Quantization parameters that the search varies (scales, zero points,
 *     multipliers, shifts, clip limits, effective bits) are runtime arguments,
 *     never compile-time constants (Sec. 6.3, batched search).
 */
#ifndef HAGO_H_
#define HAGO_H_

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  HAGO_OK = 0,
  HAGO_ERR_NULL = 1,      /* a required pointer is NULL                          */
  HAGO_ERR_SHAPE = 2,     /* negative/zero/inconsistent dimension, bad groups,
                             bad layout, a size beyond the 32-bit index range   */
  HAGO_ERR_DTYPE = 3,     /* operand / accumulator / output dtype combination
                             that the operator does not define                  */
  HAGO_ERR_BITS = 4,      /* effective bits < 1 or > container width, zero point
                             or clip range outside the container / bit range    */
  HAGO_ERR_PARAM = 5,     /* other invalid scalar parameter (flags, per_channel) */
  HAGO_ERR_ACC_BOUND = 6, /* HAGO_STRICT_ACC16 set and K*Amax*Wmax > 32767       */
  HAGO_ERR_DEVICE = 7,    /* the HIP runtime refused the launch                  */
  HAGO_ERR_SCRATCH = 8    /* hago_qconv2d_static: the rewritten operands exceed
                             HAGO_STATIC_SCRATCH_BYTES                          */
} hago_status;

/* Container data types.  "Effective bits" (Sec. 2, Sec. 5.3) may be fewer
 * than the container's width: a 6-bit value is still stored in an int8. */
typedef enum {
  HAGO_U8 = 0,
  HAGO_I8 = 1,
  HAGO_I16 = 2,
  HAGO_I32 = 3,
  HAGO_F32 = 4,
  HAGO_I24 = 5  /* accumulator type only (Sec. 4.1: accelerators with 24-bit
                   accumulation): 24-bit two's complement, held sign-extended
                   in an int32; also a simulated type of hago_simquant_wrap */
} hago_dtype;

typedef enum {
  HAGO_NCHW = 0, /* activations [B,C,H,W], weights [O,C/g,KH,KW], out [B,O,OH,OW] */
  HAGO_NHWC = 1  /* activations [B,H,W,C], weights [O,KH,KW,C/g], out [B,OH,OW,O] */
} hago_layout;

/* flags */
#define HAGO_STRICT_ACC16 1u /* refuse 16-bit (and 24-bit) accumulation unless
                                the declared operand ranges prove that it
                                cannot overflow */
#define HAGO_WS_WEIGHTS_READY 2u /* hago_qconv2d_ws only: the workspace still
                                holds this layer's rewritten weights from an
                                earlier call with the same w, geometry and
                                workspace; only the activations are rewritten */

/* A quantized tensor type: container, effective bit count, signedness of the
 * effective range, zero point.  `bits` is a CONTRACT on the value range
 * (signed b bits: [-2^(b-1), 2^(b-1)-1]; unsigned: [0, 2^b-1]); kernels never
 * mask operands to it.  It bounds the zero point and clip limits and feeds the
 * int16-accumulation overflow check. */
typedef struct {
  hago_dtype dtype;
  int32_t bits;
  int32_t is_signed;
  int32_t zero_point;
} hago_qtype;

/* Requantize epilogue (Sec. 6.1 realization; Sec. 6.2 "integer-only
 * computations"): for an accumulator acc of output channel c
 *     r   = floor(acc * multiplier[c] / 2^(31 + shift[c]) + 1/2)
 *     out = clip(r + out.zero_point, clip_lo, clip_hi)  cast to out.dtype
 * evaluated exactly in 64-bit integers (single rounding, ties toward
 * +infinity).  With rounding == HAGO_ROUND_HALF_AWAY, r is instead the nearest
 * integer to acc * multiplier[c] / 2^(31 + shift[c]) with halves away from
 * zero (the two tie rules of the compiler stack the paper generates code
 * with; the results differ, by one, exactly on negative ties).  The fastest
 * kernel variants implement the first rule; the second takes each operator's
 * more general variant.  ReLU / ReLU6 are expressed through clip_lo /
 * clip_hi in the output's quantized domain (Sec. 6.1).
 * multiplier == NULL selects the form for power-of-two scales (Sec. 5.1:
 * thresholds rounded to powers of two "make it possible to use shifting to
 * replace multiplication"): r is acc / 2^shift[c] rounded by the same tie
 * rule, shift 0..31 (0: r = acc).  The standalone operator then runs a kernel
 * without a multiplication; the fused epilogues use the identity
 * acc / 2^s = acc * 2^30 / 2^(31 + s - 1). */
typedef enum { HAGO_ROUND_UPWARD = 0, HAGO_ROUND_HALF_AWAY = 1 } hago_rounding;

typedef struct {
  const int32_t* multiplier; /* device, [channels] or [1]; Q31; NULL: shift only */
  const int32_t* shift;      /* device, [channels] or [1]; 0..31                */
  int32_t per_channel;       /* 0: entry 0 serves every channel; 1: one each    */
  hago_qtype out;            /* dtype HAGO_I8 or HAGO_U8; bits; zero_point      */
  int32_t clip_lo, clip_hi;  /* inclusive; within out's effective-bit range     */
  int32_t rounding;          /* HAGO_ROUND_UPWARD or HAGO_ROUND_HALF_AWAY       */
} hago_requant;

/*
 * simulated_quantize (Sec. 4.2 "Simulated Quantize Operator"; Eq. 3;
 * rounding and saturation errors of Sec. 5.2).  Elementwise over
 * x[outer, channels, inner] (device, fp32):
 *     y = (clip(rint(x / s) + z, clip_lo, clip_hi) - z) * s
 * in IEEE binary32 with true division, round-half-to-even and a
 * compare-select clip (NaN stays NaN, +-inf saturates, no -0 results).
 * s = scale[c], z = zero_point[c] (device, [channels]) when per_channel != 0,
 * else entry 0.  q names the simulated container / effective bits and bounds
 * clip_lo/clip_hi and nothing else.  y (device) may equal x (in place).
 * Errors: NULL, SHAPE (negative dim), DTYPE (q.dtype not U8/I8/I16/I32),
 * BITS (clip range outside q), DEVICE.  Empty tensors are a no-op.
 */
hago_status hago_simquant(const float* x, float* y, int64_t outer,
                          int64_t channels, int64_t inner, const float* scale,
                          const int32_t* zero_point, int32_t per_channel,
                          hago_qtype q, int32_t clip_lo, int32_t clip_hi,
                          void* stream);

/*
 * Quantized dense (Introduction: u8 x i8 -> i32, i8 x i8 -> i16 and
 * i16 x i16 -> i32 operand triples; Sec. 6.2: dense on the fast integer
 * instruction):
 *     acc[m,n] = bias[n] + sum_k (a[m,k] - a_t.zero_point) * w[n,k]
 * reduced modulo 2^32 (acc_dtype HAGO_I32), modulo 2^16 and sign-extended
 * (HAGO_I16, the int16-accumulation mode of Sec. 8.4) or modulo 2^24 and
 * sign-extended (HAGO_I24, Sec. 4.1; raw results are int32).  With rq != NULL (host
 * pointer to the struct) each accumulator is requantized with channel = n and
 * out is [M,N] of rq->out.dtype; with rq == NULL the raw accumulators are
 * stored as [M,N] int32 / int16.
 * a: device [M,K], HAGO_U8 or HAGO_I8.  w: device [N,K] HAGO_I8, symmetric
 * (w_t.zero_point must be 0).  bias: device [N] int32 or NULL.
 * Or both operands HAGO_I16 (int16 data, acc_dtype HAGO_I32 or HAGO_I24): there
 * is no 16-bit matrix instruction, so this triple runs on the vector ALUs.
 * Errors: NULL, SHAPE (negative dims, > 2^31-1), DTYPE, BITS, PARAM,
 * ACC_BOUND (flags & HAGO_STRICT_ACC16 and acc_dtype I16 / I24 and
 * K * max|a - z_a| * max|w| over the declared bit ranges > 2^15 - 1 /
 * 2^23 - 1), DEVICE.
 * M == 0 or N == 0 is a no-op; K == 0 yields the bias.
 */
hago_status hago_qdense(const void* a, hago_qtype a_t, const void* w,
                        hago_qtype w_t, const int32_t* bias, int64_t M,
                        int64_t N, int64_t K, hago_dtype acc_dtype,
                        const hago_requant* rq, void* out, uint32_t flags,
                        void* stream);

/*
 * Quantized conv2d (same operand triples; Sec. 6.2 conv2d; depthwise is the
 * memory-bound MobileNet case of Sec. 8.3).  Cross-correlation, dilation 1:
 *     acc[b,o,y,x] = bias[o] + sum_{c,ky,kx} (a[b,c,y*sh+ky-ph,x*sw+kx-pw] - z_a)
 *                                            * w[o,c,ky,kx]
 * where taps outside the image contribute exactly 0 (the input is padded with
 * its zero point).  OH = (H + 2*pad_h - KH) / stride_h + 1 (floor), same for
 * OW.  groups must be 1, or equal C and O (depthwise).  Accumulator width,
 * requantize (channel = o) and raw output as for hago_qdense.
 * Errors as for hago_qdense; additionally SHAPE for any other `groups`, a
 * kernel larger than the padded image, stride < 1, pad < 0; DTYPE for int16
 * operands with groups != 1.
 * This entry point uses no scratch memory.  Depthwise, 1x1 (either layout) and
 * NCHW 3x3 stride-1 pad-1 convolutions with C a multiple of 32 up to 128 and
 * W a multiple of 4 up to 128 (configs 2 and 3) run one kernel that reads
 * the caller's tensors directly, as fast as or faster than hago_qconv2d_ws;
 * every other groups == 1 geometry runs a general kernel that gathers its
 * operands from the caller's layout and is several times slower than
 * hago_qconv2d_ws.
 */
hago_status hago_qconv2d(const void* a, hago_qtype a_t, const void* w,
                         hago_qtype w_t, const int32_t* bias,
                         hago_layout layout, int64_t B, int64_t C, int64_t H,
                         int64_t W, int64_t O, int32_t KH, int32_t KW,
                         int32_t stride_h, int32_t stride_w, int32_t pad_h,
                         int32_t pad_w, int32_t groups, hago_dtype acc_dtype,
                         const hago_requant* rq, void* out, uint32_t flags,
                         void* stream);

/*
 * The same operator with caller-owned scratch memory (Sec. 6.2: conv2d on the
 * fast integer instruction).  The matrix cores read 16 consecutive reduction
 * elements per lane, so a groups == 1 convolution first rewrites, in one
 * launch, the activations into a padded channel-last int8 copy and the
 * weights into [O][KH*KW][C rounded up to 16] inside `workspace`, then runs
 * the implicit GEMM over the copies.  (Geometries for which hago_qconv2d has
 * a kernel of its own that is at least as fast run that kernel here too and
 * leave the workspace untouched.)
 *   hago_qconv2d_workspace_bytes  (host only, launches nothing): bytes this
 *     geometry wants; 0 when it runs without scratch (depthwise, or shapes
 *     only the general kernel indexes); -1 for arguments hago_qconv2d would
 *     refuse with SHAPE.  The weight copy comes first and its size does not
 *     depend on B.
 *   hago_qconv2d_ws: `workspace` is device memory, 256-byte aligned, of
 *     `workspace_bytes` >= that count (NULL / 0 allowed when the count is 0).
 *     Its contents need not be initialised and are overwritten; the library
 *     keeps no pointer to it after the call's work has run.  Calls that share
 *     one workspace must be ordered on one stream; calls with distinct
 *     workspaces may overlap freely.  With HAGO_WS_WEIGHTS_READY the weight
 *     part is taken as written by an earlier call (weights are constants of a
 *     layer) and only the activations are rewritten.
 * Results are identical to hago_qconv2d's.  Errors as for hago_qconv2d;
 * additionally NULL (workspace needed but NULL) and PARAM (workspace too
 * small, misaligned, or negative size).
 */
int64_t hago_qconv2d_workspace_bytes(hago_layout layout, int64_t B, int64_t C,
                                     int64_t H, int64_t W, int64_t O,
                                     int32_t KH, int32_t KW, int32_t stride_h,
                                     int32_t stride_w, int32_t pad_h,
                                     int32_t pad_w, int32_t groups);
hago_status hago_qconv2d_ws(const void* a, hago_qtype a_t, const void* w,
                            hago_qtype w_t, const int32_t* bias,
                            hago_layout layout, int64_t B, int64_t C, int64_t H,
                            int64_t W, int64_t O, int32_t KH, int32_t KW,
                            int32_t stride_h, int32_t stride_w, int32_t pad_h,
                            int32_t pad_w, int32_t groups, hago_dtype acc_dtype,
                            const hago_requant* rq, void* out, void* workspace,
                            int64_t workspace_bytes, uint32_t flags,
                            void* stream);

/*
 * hago_qconv2d for callers that cannot allocate device memory and have no
 * workspace to hand over: code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  Same arguments and results as
 * hago_qconv2d_ws, but the scratch is a fixed array of
 * HAGO_STATIC_SCRATCH_BYTES of static device memory inside the library (each
 * GPU the library runs on holds its own copy until the process ends).  The
 * call allocates and frees nothing and does not wait for the device.
 * A geometry whose hago_qconv2d_workspace_bytes exceeds the array is refused
 * with HAGO_ERR_SCRATCH before anything is launched (use hago_qconv2d_ws).
 * Every call on a GPU uses that GPU's one array, which is overwritten by each
 * call: calls that may run at the same time on one GPU (different streams,
 * different host threads) race and must be ordered by the caller; calls on
 * one stream are safe.
 */
#define HAGO_STATIC_SCRATCH_BYTES (64ll << 20)
hago_status hago_qconv2d_static(const void* a, hago_qtype a_t, const void* w,
                                hago_qtype w_t, const int32_t* bias,
                                hago_layout layout, int64_t B, int64_t C,
                                int64_t H, int64_t W, int64_t O, int32_t KH,
                                int32_t KW, int32_t stride_h, int32_t stride_w,
                                int32_t pad_h, int32_t pad_w, int32_t groups,
                                hago_dtype acc_dtype, const hago_requant* rq,
                                void* out, uint32_t flags, void* stream);

/*
 * simulated_quantize with the overflow of the simulated integer type (Sec. 5.2
 * "Model Simulation": besides the rounding and the saturation error there is
 * "the overflow error, possible when the output of quantized operator is beyond
 * the limit of output data type can represent").  As hago_simquant, but the
 * code rint(x / s) + z is first reduced modulo 2^w into the range of q.dtype's
 * container: w = 8 (HAGO_I8 two's complement, HAGO_U8 0..255), 16 (HAGO_I16),
 * 24 (HAGO_I24) or 32 (HAGO_I32); then clipped to clip_lo..clip_hi (within
 * q's effective bits and +-2^24) and dequantized.  With q the accumulator
 * type of a quantized operator this reproduces, in the simulated graph, what
 * hago_qdense / hago_qconv2d with that acc_dtype do to a sum that does not fit.
 * A code of magnitude >= 4e18 or an infinite one reduces to 0; NaN stays NaN.
 * Errors as for hago_simquant.
 */
hago_status hago_simquant_wrap(const float* x, float* y, int64_t outer,
                               int64_t channels, int64_t inner,
                               const float* scale, const int32_t* zero_point,
                               int32_t per_channel, hago_qtype q,
                               int32_t clip_lo, int32_t clip_hi, void* stream);

/*
 * Batched candidate evaluation of simulated_quantize (Sec. 6.3 "Batched GPU
 * Search": quantization parameters are runtime arguments, and a batch of
 * candidate settings is evaluated in one go).  The tensor x[outer, channels,
 * inner] (device, fp32) is read once; candidate b = 0..nbatch-1 (at most 16)
 * writes y[b, outer, channels, inner] (device, fp32) = hago_simquant(x) with
 * scale[b*P + c], zero_point[b*P + c] (device; P = channels if per_channel
 * else 1) and the clip range clip_lo[b]..clip_hi[b] (HOST arrays, read before
 * the call returns).  q bounds every clip range as in hago_simquant (use the
 * widest candidate's bits).  y must not overlap x.
 * Errors: NULL, SHAPE, DTYPE, BITS (some clip range outside q or +-2^24),
 * PARAM (per_channel not 0/1, nbatch > 16), DEVICE.  Empty is a no-op.
 */
hago_status hago_simquant_batched(const float* x, float* y, int64_t outer,
                                  int64_t channels, int64_t inner,
                                  int32_t nbatch, const float* scale,
                                  const int32_t* zero_point,
                                  int32_t per_channel, hago_qtype q,
                                  const int32_t* clip_lo,
                                  const int32_t* clip_hi, void* stream);

/*
 * quantize and dequantize (Sec. 6.1: the operators with which the realized
 * graph enters and leaves the integer domain; the two halves of Eq. 3).
 *     q = clip(rint(x / s) + z, clip_lo, clip_hi)      stored as qt.dtype
 *     y = ((float)q - (float)z) * s
 * x, y: device fp32 [outer, channels, inner]; q: device, container qt.dtype
 * (HAGO_I8, HAGO_U8, HAGO_I16 or HAGO_I32), same shape.  s, z as for
 * hago_simquant.  The code is formed exactly as in hago_simquant (binary32
 * division, round half to even, compare-select clip), so
 * hago_dequantize(hago_quantize(x)) equals hago_simquant(x) bit for bit; a NaN
 * input takes the code of real zero, clip(z).  clip_lo/clip_hi must lie within
 * qt's effective-bit range and within +-2^24.  hago_dequantize converts q to
 * binary32 first (exact for |q| <= 2^24).
 * Errors: NULL, SHAPE, DTYPE (qt.dtype HAGO_F32 or unknown), BITS, PARAM
 * (per_channel not 0/1), DEVICE.  Empty tensors are a no-op.
 */
hago_status hago_quantize(const float* x, void* q, int64_t outer,
                          int64_t channels, int64_t inner, const float* scale,
                          const int32_t* zero_point, int32_t per_channel,
                          hago_qtype qt, int32_t clip_lo, int32_t clip_hi,
                          void* stream);
hago_status hago_dequantize(const void* q, hago_qtype qt, float* y,
                            int64_t outer, int64_t channels, int64_t inner,
                            const float* scale, const int32_t* zero_point,
                            int32_t per_channel, void* stream);

/*
 * simulated_quantize that also emits the integer codes it passes through
 * (Sec. 6.1: realization replaces simulated_quantize by operators on q, so the
 * codes are what the realized graph carries where the simulated graph carries
 * q * s; Eq. 3).  One pass over x: y = hago_simquant(x) and q = hago_quantize(x)
 * with the same arguments, bit for bit (a NaN stays NaN in y and takes the
 * code of real zero in q).  x, y: device fp32 [outer, channels, inner]; q:
 * device, container qt.dtype, same shape; none of them may overlap.
 * Errors as for hago_quantize.  Empty tensors are a no-op.
 */
hago_status hago_simquant_codes(const float* x, float* y, void* q,
                                int64_t outer, int64_t channels, int64_t inner,
                                const float* scale, const int32_t* zero_point,
                                int32_t per_channel, hago_qtype qt,
                                int32_t clip_lo, int32_t clip_hi, void* stream);

/*
 * Max-abs calibration (Sec. 2, Eq. 2: threshold = max |x|; Sec. 5.1 statistics
 * collection): the thresholds that Eq. 1 turns into the scales of
 * simulated_quantize.  x[outer, channels, inner] (device, fp32);
 *     threshold[c] = max over o, i of |x[o, c, i]|      (per_channel != 0)
 *     threshold[0] = max over the whole tensor           (per_channel == 0)
 * threshold (device) has `channels` entries, or one.  NaN elements are ignored
 * (they never win a comparison); an empty reduction gives 0; the result is
 * never -0.  The result is exact (a maximum does not depend on the order).
 * Errors: NULL, SHAPE (negative dim or overflowing element count), PARAM
 * (per_channel not 0/1), DEVICE.
 */
hago_status hago_absmax(const float* x, int64_t outer, int64_t channels,
                        int64_t inner, int32_t per_channel, float* threshold,
                        void* stream);

/*
 * Standalone requantize (Sec. 6.1, 6.2): acc[outer, channels, inner] (device,
 * HAGO_I32 or HAGO_I16; int16 is sign-extended) -> out of rq->out.dtype with
 * the same shape, channel = axis 1.  rq must be non-NULL.
 */
hago_status hago_requantize(const void* acc, hago_dtype acc_dtype,
                            int64_t outer, int64_t channels, int64_t inner,
                            const hago_requant* rq, void* out, void* stream);

/* Static, NUL-terminated description of a status code. */
const char* hago_status_string(hago_status s);

/*
 * The inclusive range of integer codes that `bits` effective bits hold
 * (Sec. 2: a b-bit data type has 2^b bins; Sec. 5.3: fewer effective bits than
 * the container): signed [-2^(bits-1), 2^(bits-1)-1], unsigned [0, 2^bits-1].
 * These are the widest clip limits a call accepts for that bit count and the
 * defaults a binding should pass.  lo, hi: host pointers.  Errors: NULL, BITS
 * (bits < 1, > 32, or 32 unsigned, which int32 cannot hold).
 */
hago_status hago_bit_range(int32_t bits, int32_t is_signed, int32_t* lo,
                           int32_t* hi);

/*
 * Measurement probes, not part of the operator set: what this chip delivers
 * when a kernel does nothing but the bounding operation, printed by the
 * benchmark beside the published peaks.
 *   hago_probe_mfma_i8: `workgroups` workgroups of four wavefronts each issue
 *     16 * iters int8 matrix instructions (32x32x32) back to back on the operands
 *     at `operands` (device, 8192 bytes, read once; real data matters, the clock
 *     under matrix-core load depends on it); 2 * 32*32*32 * 16 * iters *
 *     workgroups operations in all.  sink: device, 4 bytes, practically never
 *     written.
 *   hago_probe_copy: streaming copy of `bytes` (a multiple of 16, 16-byte aligned
 *     device pointers) with the elementwise kernels' access pattern.
 * Errors: NULL, SHAPE, PARAM (alignment), DEVICE.
 */
hago_status hago_probe_mfma_i8(const void* operands, void* sink,
                               int32_t workgroups, int32_t iters, void* stream);
hago_status hago_probe_copy(const void* src, void* dst, int64_t bytes,
                            void* stream);

/*
 * Test hook, not part of the operator set: forces which GEMM kernel family
 * and tile shape serve the following hago_qdense / hago_qconv2d* calls of
 * this process, so that tests can compare every variant with the oracle on
 * one shape.  Results never depend on it.  Keys:
 *   HAGO_HOOK_GEMM_PATH     0 automatic; 1 the general register-staged kernel;
 *                           2 the streaming kernel, skipping the kernels
 *                           specialised for 1x1 and 3x3 convolutions
 *   HAGO_HOOK_STREAM_TILE   -1 automatic; 0..4 a tile of the streaming dense kernel
 *   HAGO_HOOK_GENERAL_TILE  -1 automatic; 0..6 a tile of the general kernel
 * Unknown keys are ignored.
 */
#define HAGO_HOOK_GEMM_PATH 0
#define HAGO_HOOK_STREAM_TILE 1
#define HAGO_HOOK_GENERAL_TILE 2
void hago_set_test_hook(int32_t key, int32_t value);

#ifdef __cplusplus
}
#endif
#endif /* HAGO_H_ */
