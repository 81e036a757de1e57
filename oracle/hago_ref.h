/*
 * hago_ref.h -- CPU oracle for the quantized-operator hot path of HAGO
 * (arXiv 2103.14949).  TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow, scalar C++17 implementation of what the path computes, used
 * to check the GPU library and as the timed CPU baseline.  It is independent
 * of the GPU library: it includes none of its headers and shares no code,
 * tables or helpers with it.  Only tests, the smoke check and the benchmark's
 * cpu_baseline leg may call it; no product code path may.
 *
 * All pointers are HOST pointers.  Tensors are dense and contiguous.  Every
 * function returns 0 on success and a non-zero code on an argument it cannot
 * give a meaning to (it never aborts).
 *
 * Pinned by tests/test_oracle_*.py against exact big-integer / rational
 * arithmetic, closed forms, invariants and brute force (see each function).
 * The tie rule of requantize (ties toward +infinity) is a convention the
 * paper does not fix; it is pinned only by the exact-rational definition.
 */
#ifndef HAGO_REF_H_
#define HAGO_REF_H_

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* container dtypes (values chosen by this file alone) */
enum { REF_U8 = 0, REF_I8 = 1, REF_I16 = 2, REF_I32 = 3, REF_F32 = 4,
       REF_I24 = 5 /* accumulator only: 24-bit two's complement, stored
                      sign-extended in an int32 (Sec. 4.1: accelerators with
                      24-bit accumulation) */ };
enum { REF_NCHW = 0, REF_NHWC = 1 }; /* weights OIHW / OHWI respectively */

enum {
  REF_OK = 0,
  REF_ERR_NULL = 1,
  REF_ERR_SHAPE = 2,
  REF_ERR_DTYPE = 3,
  REF_ERR_BITS = 4,
  REF_ERR_PARAM = 5
};

/* Requantize parameters.  multiplier/shift have `channels` entries when
 * per_channel != 0, else one entry.  out_dtype is REF_I8 or REF_U8. */
typedef struct {
  const int32_t* multiplier; /* Q31 fixed point, value = multiplier / 2^31;
                                NULL: power-of-two scales (Sec. 5.1), the
                                requantize is the rounding right shift alone,
                                r = round(acc / 2^shift) */
  const int32_t* shift;      /* extra right shift, 0..31 */
  int32_t per_channel;
  int32_t out_dtype;
  int32_t out_zero_point;
  int32_t clip_lo, clip_hi; /* inclusive, in the output's quantized domain */
  int32_t rounding;         /* REF_ROUND_UPWARD or REF_ROUND_HALF_AWAY */
} ref_requant;

/* Tie rule of the requantize rounding.  The paper names the operator only;
 * the two rules are the ones of the compiler stack it generates code with:
 * ties toward +infinity, and ties away from zero. */
enum { REF_ROUND_UPWARD = 0, REF_ROUND_HALF_AWAY = 1 };

/* Sec. 2 (Background), Eq. 1: s = threshold / 2^(bit - sign). */
double hago_ref_scale(double threshold, int32_t bits, int32_t sign);

/* Sec. 2, Eq. 2: per-channel (axis 1 of [outer, channels, inner]) or
 * per-tensor max |x|.  thr has `channels` entries (or 1). */
int hago_ref_absmax(const float* x, int64_t outer, int64_t channels,
                    int64_t inner, int32_t per_channel, float* thr);

/* Default integer range of `bits` effective bits: signed
 * [-2^(b-1), 2^(b-1)-1], unsigned [0, 2^b-1]. */
int hago_ref_bit_range(int32_t bits, int32_t is_signed, int32_t* lo,
                       int32_t* hi);

/* simulated_quantize (Sec. 4.2; Eq. 3; error sources of Sec. 5.2):
 * y = (clip(rint(x / s) + z, lo, hi) - z) * s in IEEE binary32, round half
 * to even, true division, no contraction.  Clip is compare-select, so NaN
 * stays NaN and +-inf saturates. */
int hago_ref_simquant(const float* x, float* y, int64_t outer,
                      int64_t channels, int64_t inner, const float* scale,
                      const int32_t* zero_point, int32_t per_channel,
                      int32_t clip_lo, int32_t clip_hi);

/* quantize (Sec. 6.1: the operator that enters the integer domain; the inner
 * part of Eq. 3): code = clip(rint(x / s) + z, lo, hi), with x / s and the
 * rounding in IEEE binary32 as in simulated_quantize.  NaN quantizes to the
 * code of real zero, clip(z).  q receives the codes as int32. */
int hago_ref_quantize(const float* x, int32_t* q, int64_t outer,
                      int64_t channels, int64_t inner, const float* scale,
                      const int32_t* zero_point, int32_t per_channel,
                      int32_t clip_lo, int32_t clip_hi);

/* dequantize (Sec. 6.1: back to real values; Eq. 3's r ~= q * s):
 * y = ((float)q - (float)z) * s in IEEE binary32. */
int hago_ref_dequantize(const int32_t* q, float* y, int64_t outer,
                        int64_t channels, int64_t inner, const float* scale,
                        const int32_t* zero_point, int32_t per_channel);

/* Real multiplier m in (2^-32, 1) -> (Q31 multiplier in [2^30, 2^31), shift
 * in [0, 31]) with m ~= multiplier * 2^-(31+shift). */
int hago_ref_encode_multiplier(double m, int32_t* multiplier, int32_t* shift);

/* One requantize (Sec. 6.1 names the operator; the fixed-point form is the
 * build's convention): r = floor(acc*M / 2^(31+sh) + 1/2); out =
 * clip(r + z_out, lo, hi).  Exposed so tests can probe single values. */
int64_t hago_ref_requantize_one(int32_t acc, int32_t multiplier, int32_t shift,
                                int32_t z_out, int32_t lo, int32_t hi);
/* The same with the tie rule chosen: REF_ROUND_HALF_AWAY rounds
 * acc*M / 2^(31+sh) to the nearest integer, halves away from zero. */
int64_t hago_ref_requantize_one_mode(int32_t acc, int32_t multiplier,
                                     int32_t shift, int32_t z_out, int32_t lo,
                                     int32_t hi, int32_t rounding);

/* Requantize for power-of-two scales (Sec. 5.1: thresholds rounded to powers
 * of two so that shifting replaces the multiplication): r = round(acc / 2^sh),
 * sh in 0..31, same tie rules as above (sh == 0: r = acc);
 * out = clip(r + z_out, lo, hi).  No multiplication anywhere. */
int64_t hago_ref_requantize_shift_one(int32_t acc, int32_t shift, int32_t z_out,
                                      int32_t lo, int32_t hi, int32_t rounding);

/* Standalone requantize over acc[outer, channels, inner] (REF_I32 or REF_I16;
 * int16 is sign-extended) -> out (REF_I8 / REF_U8). */
int hago_ref_requantize(const void* acc, int32_t acc_dtype, int64_t outer,
                        int64_t channels, int64_t inner, const ref_requant* rq,
                        void* out);

/* Largest |sum| the declared operand ranges allow: K * Amax * Wmax, and
 * whether it fits int16 (<= 32767).  Returns 1 if safe, 0 if not. */
int hago_ref_acc16_safe(int64_t K, int64_t a_absmax, int64_t w_absmax);

/* The same bound for an accumulator of acc_bits bits (16, 24 or 32):
 * K * Amax * Wmax <= 2^(acc_bits-1) - 1. */
int hago_ref_acc_safe(int64_t K, int64_t a_absmax, int64_t w_absmax,
                      int32_t acc_bits);

/* simulated_quantize with the overflow of the simulated integer type (Sec. 5.2
 * names three error sources: rounding, saturation, and overflow "when the
 * output of quantized operator is beyond the limit of output data type").
 * The code u = rint(x / s) + z is first reduced modulo 2^wrap_bits into
 * [-2^(wrap_bits-1), 2^(wrap_bits-1)) (wrap_signed != 0, two's complement) or
 * [0, 2^wrap_bits) (unsigned), wrap_bits in 2..32 being the width of the
 * simulated accumulator / container, then clipped and dequantized as in
 * simulated_quantize.  Codes of magnitude >= 2^62 and
 * infinities reduce to 0 (every float that large is a multiple of 2^32); NaN
 * stays NaN.  The wrapped code is converted back to binary32 (exact for
 * wrap_bits <= 25). */
int hago_ref_simquant_wrap(const float* x, float* y, int64_t outer,
                           int64_t channels, int64_t inner, const float* scale,
                           const int32_t* zero_point, int32_t per_channel,
                           int32_t wrap_bits, int32_t wrap_signed,
                           int32_t clip_lo, int32_t clip_hi);

/* Quantized dense (Sec. 1 / Sec. 6.2: low-precision operands, integer
 * accumulation): acc[m,n] = bias[n] + sum_k (a[m,k] - z_a) * w[n,k], reduced
 * mod 2^32 (acc_dtype REF_I32) or mod 2^16 (REF_I16), then requantized per
 * output channel n when rq != NULL, else stored raw.
 * a: [M,K] REF_U8|REF_I8; w: [N,K] REF_I8; bias: [N] int32 or NULL. */
int hago_ref_qdense(const void* a, int32_t a_dtype, int32_t a_zero_point,
                    const int8_t* w, const int32_t* bias, int64_t M, int64_t N,
                    int64_t K, int32_t acc_dtype, const ref_requant* rq,
                    void* out);

/* Quantized conv2d, cross-correlation, dilation 1, groups == 1 or depthwise
 * (groups == C == O).  Out-of-bounds taps contribute exactly 0 (i.e. the
 * input is padded with z_a).  Layout REF_NCHW: a [B,C,H,W], w [O,C/g,KH,KW],
 * out [B,O,OH,OW]; REF_NHWC: a [B,H,W,C], w [O,KH,KW,C/g], out [B,OH,OW,O].
 * OH = (H + 2*pad_h - KH) / stride_h + 1 (floor), likewise OW. */
int hago_ref_qconv2d(const void* a, int32_t a_dtype, int32_t a_zero_point,
                     const int8_t* w, const int32_t* bias, int32_t layout,
                     int64_t B, int64_t C, int64_t H, int64_t W, int64_t O,
                     int32_t KH, int32_t KW, int32_t stride_h, int32_t stride_w,
                     int32_t pad_h, int32_t pad_w, int32_t groups,
                     int32_t acc_dtype, const ref_requant* rq, void* out);

/* The same two operators with the weight container named: REF_I8 as above, or
 * the second operand triple of Sec. 1 / Sec. 4.1, int16 x int16 with int32
 * accumulation (a_dtype == w_dtype == REF_I16, acc_dtype REF_I32 or REF_I24).
 * Products are formed exactly and the sum wraps modulo 2^32 as before. */
int hago_ref_qdense_x(const void* a, int32_t a_dtype, int32_t a_zero_point,
                      const void* w, int32_t w_dtype, const int32_t* bias,
                      int64_t M, int64_t N, int64_t K, int32_t acc_dtype,
                      const ref_requant* rq, void* out);
int hago_ref_qconv2d_x(const void* a, int32_t a_dtype, int32_t a_zero_point,
                       const void* w, int32_t w_dtype, const int32_t* bias,
                       int32_t layout, int64_t B, int64_t C, int64_t H, int64_t W,
                       int64_t O, int32_t KH, int32_t KW, int32_t stride_h,
                       int32_t stride_w, int32_t pad_h, int32_t pad_w,
                       int32_t groups, int32_t acc_dtype, const ref_requant* rq,
                       void* out);

#ifdef __cplusplus
}
#endif
#endif /* HAGO_REF_H_ */
