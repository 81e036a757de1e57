// C ABI of libhago: argument validation (host only, before any launch) and
// dispatch to the kernel families.  See include/hago.h for the contract.
#include "../../include/hago.h"

#include "launch.h"

namespace {

using hago::ConvGeom;
using hago::GemmArgs;
using hago::RequantArgs;

constexpr int64_t kI32Max = 2147483647ll;

int container_bits(hago_dtype d) {
  switch (d) {
    case HAGO_U8: case HAGO_I8: return 8;
    case HAGO_I16: return 16;
    case HAGO_I32: return 32;
    default: return 0;
  }
}

// Inclusive value range of `bits` effective bits (Sec. 2: 2^bit bins).
void bit_range(int bits, int is_signed, int64_t* lo, int64_t* hi) {
  if (is_signed) {
    *lo = -((int64_t)1 << (bits - 1));
    *hi = ((int64_t)1 << (bits - 1)) - 1;
  } else {
    *lo = 0;
    *hi = ((int64_t)1 << bits) - 1;
  }
}

void container_range(hago_dtype d, int64_t* lo, int64_t* hi) {
  switch (d) {
    case HAGO_U8: *lo = 0; *hi = 255; break;
    case HAGO_I8: *lo = -128; *hi = 127; break;
    case HAGO_I16: *lo = -32768; *hi = 32767; break;
    default: *lo = -2147483648ll; *hi = 2147483647ll; break;
  }
}

// bits within the container, effective range inside the container's range.
hago_status check_qtype(const hago_qtype& q, bool zero_point_in_container) {
  const int cb = container_bits(q.dtype);
  if (cb == 0) return HAGO_ERR_DTYPE;
  if (q.bits < 1 || q.bits > cb) return HAGO_ERR_BITS;
  int64_t blo, bhi, clo, chi;
  bit_range(q.bits, q.is_signed != 0, &blo, &bhi);
  container_range(q.dtype, &clo, &chi);
  if (blo < clo || bhi > chi) return HAGO_ERR_BITS;  // e.g. 8 unsigned bits in an int8
  if (zero_point_in_container && (q.zero_point < clo || q.zero_point > chi)) return HAGO_ERR_BITS;
  return HAGO_OK;
}

hago_status check_requant(const hago_requant* rq, RequantArgs* out) {
  if (!rq->shift) return HAGO_ERR_NULL;  // (no multiplier array: power-of-two scales, shift only)
  if (rq->out.dtype != HAGO_I8 && rq->out.dtype != HAGO_U8) return HAGO_ERR_DTYPE;
  if (rq->per_channel != 0 && rq->per_channel != 1) return HAGO_ERR_PARAM;
  if (rq->rounding != HAGO_ROUND_UPWARD && rq->rounding != HAGO_ROUND_HALF_AWAY) return HAGO_ERR_PARAM;
  hago_status s = check_qtype(rq->out, true);
  if (s != HAGO_OK) return s;
  int64_t blo, bhi;
  bit_range(rq->out.bits, rq->out.is_signed != 0, &blo, &bhi);
  if (rq->clip_lo > rq->clip_hi || rq->clip_lo < blo || rq->clip_hi > bhi) return HAGO_ERR_BITS;
  out->multiplier = rq->multiplier;
  out->shift = rq->shift;
  out->per_channel = rq->per_channel;
  out->out_unsigned = rq->out.dtype == HAGO_U8;
  out->z_out = rq->out.zero_point;
  out->clip_lo = rq->clip_lo;
  out->clip_hi = rq->clip_hi;
  out->half_away = rq->rounding == HAGO_ROUND_HALF_AWAY;
  return HAGO_OK;
}

// Shared operand checks of qdense / qconv2d.
hago_status check_operands(const void* a, const hago_qtype& a_t, const void* w,
                           const hago_qtype& w_t, hago_dtype acc_dtype, const hago_requant* rq,
                           const void* out, uint32_t flags, int64_t K, bool a_empty,
                           bool w_empty, bool out_empty, GemmArgs* g) {
  // an empty tensor may come with a NULL pointer
  if ((!a && !a_empty) || (!w && !w_empty) || (!out && !out_empty)) return HAGO_ERR_NULL;
  // operand triples (Introduction; Sec. 4.1): (u8 | i8) x i8 with 32-, 24- or 16-bit accumulation,
  // or i16 x i16 with 32- or 24-bit accumulation
  const bool op16 = a_t.dtype == HAGO_I16 && w_t.dtype == HAGO_I16;
  if (!op16 && ((a_t.dtype != HAGO_U8 && a_t.dtype != HAGO_I8) || w_t.dtype != HAGO_I8)) return HAGO_ERR_DTYPE;
  if (op16 && acc_dtype == HAGO_I16) return HAGO_ERR_DTYPE;
  if (w_t.zero_point != 0) return HAGO_ERR_DTYPE;  // weights are symmetric
  if (acc_dtype != HAGO_I32 && acc_dtype != HAGO_I16 && acc_dtype != HAGO_I24) return HAGO_ERR_DTYPE;
  if (flags & ~HAGO_STRICT_ACC16) return HAGO_ERR_PARAM;
  hago_status s = check_qtype(a_t, true);
  if (s != HAGO_OK) return s;
  s = check_qtype(w_t, false);
  if (s != HAGO_OK) return s;
  g->has_rq = 0;
  g->rq = RequantArgs{};
  if (rq) {
    s = check_requant(rq, &g->rq);
    if (s != HAGO_OK) return s;
    g->has_rq = 1;
  }
  if ((flags & HAGO_STRICT_ACC16) && acc_dtype != HAGO_I32) {
    const int64_t acc_max = acc_dtype == HAGO_I16 ? 32767 : 8388607;  // 2^15 - 1, 2^23 - 1
    // Worst case of |sum_k (a - z_a) w| over the declared ranges (Sec. 5.3:
    // effective bits are what keeps a 16-bit accumulator from overflowing).
    int64_t alo, ahi, wlo, whi;
    bit_range(a_t.bits, a_t.is_signed != 0, &alo, &ahi);
    bit_range(w_t.bits, w_t.is_signed != 0, &wlo, &whi);
    const int64_t amax = (ahi - a_t.zero_point > a_t.zero_point - alo) ? ahi - a_t.zero_point
                                                                       : a_t.zero_point - alo;
    const int64_t wmax = (whi > -wlo) ? whi : -wlo;
    if (amax > 0 && wmax > 0 && K > 0) {
      if (amax > acc_max || wmax > acc_max || K > acc_max || amax * wmax > acc_max ||
          K > acc_max / (amax * wmax))
        return HAGO_ERR_ACC_BOUND;
    }
  }
  g->act = a;
  g->wgt = static_cast<const int8_t*>(w);
  g->out = const_cast<void*>(out);
  g->operand16 = op16;
  g->act_unsigned = a_t.dtype == HAGO_U8;
  g->act_zero_point = a_t.zero_point;
  g->acc16 = acc_dtype == HAGO_I16;
  g->acc_wrap_shift = acc_dtype == HAGO_I16 ? 16 : (acc_dtype == HAGO_I24 ? 8 : 0);
  return HAGO_OK;
}

hago_status from_hip(hipError_t e) { return e == hipSuccess ? HAGO_OK : HAGO_ERR_DEVICE; }

}  // namespace

extern "C" {

const char* hago_status_string(hago_status s) {
  switch (s) {
    case HAGO_OK: return "ok";
    case HAGO_ERR_NULL: return "a required pointer is NULL";
    case HAGO_ERR_SHAPE: return "invalid or unsupported shape";
    case HAGO_ERR_DTYPE: return "unsupported dtype combination";
    case HAGO_ERR_BITS: return "effective bits, zero point or clip range outside the container";
    case HAGO_ERR_PARAM: return "invalid parameter";
    case HAGO_ERR_ACC_BOUND: return "int16 accumulation may overflow for the declared bit widths";
    case HAGO_ERR_DEVICE: return "HIP runtime error";
    case HAGO_ERR_SCRATCH: return "the operands do not fit the library's fixed scratch array";
  }
  return "unknown status";
}

hago_status hago_simquant(const float* x, float* y, int64_t outer, int64_t channels, int64_t inner,
                          const float* scale, const int32_t* zero_point, int32_t per_channel,
                          hago_qtype q, int32_t clip_lo, int32_t clip_hi, void* stream) {
  if (outer < 0 || channels < 0 || inner < 0) return HAGO_ERR_SHAPE;
  const bool sq_empty = outer == 0 || channels == 0 || inner == 0;
  if (((!x || !y) && !sq_empty) || !scale || !zero_point) return HAGO_ERR_NULL;
  if (per_channel != 0 && per_channel != 1) return HAGO_ERR_PARAM;
  if (q.dtype == HAGO_F32) return HAGO_ERR_DTYPE;
  hago_status s = check_qtype(q, false);
  if (s != HAGO_OK) return s;
  int64_t blo, bhi;
  bit_range(q.bits, q.is_signed != 0, &blo, &bhi);
  if (clip_lo > clip_hi || clip_lo < blo || clip_hi > bhi) return HAGO_ERR_BITS;
  // codes must be exactly representable in binary32
  if (clip_lo < -(1 << 24) || clip_hi > (1 << 24)) return HAGO_ERR_BITS;
  if (outer && channels && inner) {
    if (outer > INT64_MAX / channels || outer * channels > INT64_MAX / inner) return HAGO_ERR_SHAPE;
  }
  return from_hip(hago::launch_simquant(x, y, outer, channels, inner, scale, zero_point,
                                        per_channel, clip_lo, clip_hi,
                                        static_cast<hipStream_t>(stream)));
}

hago_status hago_simquant_wrap(const float* x, float* y, int64_t outer, int64_t channels, int64_t inner,
                               const float* scale, const int32_t* zero_point, int32_t per_channel,
                               hago_qtype q, int32_t clip_lo, int32_t clip_hi, void* stream) {
  if (outer < 0 || channels < 0 || inner < 0) return HAGO_ERR_SHAPE;
  const bool empty = outer == 0 || channels == 0 || inner == 0;
  if (((!x || !y) && !empty) || !scale || !zero_point) return HAGO_ERR_NULL;
  if (per_channel != 0 && per_channel != 1) return HAGO_ERR_PARAM;
  // the simulated type: its container decides the width and signedness of the overflow
  int wrap_bits = 0;
  switch (q.dtype) {
    case HAGO_U8: case HAGO_I8: wrap_bits = 8; break;
    case HAGO_I16: wrap_bits = 16; break;
    case HAGO_I24: wrap_bits = 24; break;
    case HAGO_I32: wrap_bits = 32; break;
    default: return HAGO_ERR_DTYPE;
  }
  if (q.bits < 1 || q.bits > wrap_bits) return HAGO_ERR_BITS;
  if (q.dtype == HAGO_U8 && q.is_signed) return HAGO_ERR_BITS;
  int64_t blo, bhi;
  bit_range(q.bits, q.is_signed != 0, &blo, &bhi);
  if (q.dtype != HAGO_U8 && !q.is_signed && bhi >= ((int64_t)1 << (wrap_bits - 1))) return HAGO_ERR_BITS;
  if (clip_lo > clip_hi || clip_lo < blo || clip_hi > bhi) return HAGO_ERR_BITS;
  if (clip_lo < -(1 << 24) || clip_hi > (1 << 24)) return HAGO_ERR_BITS;
  if (!empty) {
    if (outer > INT64_MAX / channels || outer * channels > INT64_MAX / inner) return HAGO_ERR_SHAPE;
  }
  return from_hip(hago::launch_simquant_wrap(x, y, outer, channels, inner, scale, zero_point, per_channel,
                                             wrap_bits, q.dtype != HAGO_U8, clip_lo, clip_hi,
                                             static_cast<hipStream_t>(stream)));
}

hago_status hago_simquant_batched(const float* x, float* y, int64_t outer, int64_t channels,
                                  int64_t inner, int32_t nbatch, const float* scale,
                                  const int32_t* zero_point, int32_t per_channel, hago_qtype q,
                                  const int32_t* clip_lo, const int32_t* clip_hi, void* stream) {
  if (outer < 0 || channels < 0 || inner < 0 || nbatch < 0) return HAGO_ERR_SHAPE;
  if (nbatch > 16) return HAGO_ERR_PARAM;
  const bool empty = outer == 0 || channels == 0 || inner == 0 || nbatch == 0;
  if (((!x || !y) && !empty) || !scale || !zero_point || ((!clip_lo || !clip_hi) && nbatch > 0))
    return HAGO_ERR_NULL;
  if (per_channel != 0 && per_channel != 1) return HAGO_ERR_PARAM;
  if (q.dtype == HAGO_F32) return HAGO_ERR_DTYPE;
  hago_status s = check_qtype(q, false);
  if (s != HAGO_OK) return s;
  int64_t blo, bhi;
  bit_range(q.bits, q.is_signed != 0, &blo, &bhi);
  for (int b = 0; b < nbatch; ++b) {
    if (clip_lo[b] > clip_hi[b] || clip_lo[b] < blo || clip_hi[b] > bhi) return HAGO_ERR_BITS;
    if (clip_lo[b] < -(1 << 24) || clip_hi[b] > (1 << 24)) return HAGO_ERR_BITS;
  }
  if (!empty) {
    if (outer > INT64_MAX / channels || outer * channels > INT64_MAX / inner ||
        outer * channels * inner > INT64_MAX / nbatch)
      return HAGO_ERR_SHAPE;
  }
  return from_hip(hago::launch_simquant_batched(x, y, outer, channels, inner, nbatch, scale,
                                                zero_point, per_channel, clip_lo, clip_hi,
                                                static_cast<hipStream_t>(stream)));
}

namespace {
// Shared checks of quantize / dequantize; container id for launch_quant.
hago_status check_quant(hago_qtype q, int32_t per_channel, int64_t outer, int64_t channels,
                        int64_t inner, const void* scale, const void* zero_point, int* container) {
  if (outer < 0 || channels < 0 || inner < 0) return HAGO_ERR_SHAPE;
  if (!scale || !zero_point) return HAGO_ERR_NULL;
  if (per_channel != 0 && per_channel != 1) return HAGO_ERR_PARAM;
  if (q.dtype == HAGO_F32) return HAGO_ERR_DTYPE;
  hago_status s = check_qtype(q, false);
  if (s != HAGO_OK) return s;
  if (outer && channels && inner) {
    if (outer > INT64_MAX / channels || outer * channels > INT64_MAX / inner) return HAGO_ERR_SHAPE;
  }
  *container = q.dtype == HAGO_I8 ? 0 : (q.dtype == HAGO_U8 ? 1 : (q.dtype == HAGO_I16 ? 2 : 3));
  return HAGO_OK;
}
}  // namespace

hago_status hago_quantize(const float* x, void* q, int64_t outer, int64_t channels, int64_t inner,
                          const float* scale, const int32_t* zero_point, int32_t per_channel,
                          hago_qtype qt, int32_t clip_lo, int32_t clip_hi, void* stream) {
  int container = 0;
  hago_status s = check_quant(qt, per_channel, outer, channels, inner, scale, zero_point, &container);
  if (s != HAGO_OK) return s;
  const bool empty = outer == 0 || channels == 0 || inner == 0;
  if ((!x || !q) && !empty) return HAGO_ERR_NULL;
  int64_t blo, bhi;
  bit_range(qt.bits, qt.is_signed != 0, &blo, &bhi);
  if (clip_lo > clip_hi || clip_lo < blo || clip_hi > bhi) return HAGO_ERR_BITS;
  // codes are formed in binary32
  if (clip_lo < -(1 << 24) || clip_hi > (1 << 24)) return HAGO_ERR_BITS;
  return from_hip(hago::launch_quant(x, q, nullptr, container, 0, outer, channels, inner, scale, zero_point,
                                     per_channel, clip_lo, clip_hi, static_cast<hipStream_t>(stream)));
}

hago_status hago_simquant_codes(const float* x, float* y, void* q, int64_t outer, int64_t channels,
                                int64_t inner, const float* scale, const int32_t* zero_point,
                                int32_t per_channel, hago_qtype qt, int32_t clip_lo, int32_t clip_hi,
                                void* stream) {
  int container = 0;
  hago_status s = check_quant(qt, per_channel, outer, channels, inner, scale, zero_point, &container);
  if (s != HAGO_OK) return s;
  const bool empty = outer == 0 || channels == 0 || inner == 0;
  if ((!x || !y || !q) && !empty) return HAGO_ERR_NULL;
  int64_t blo, bhi;
  bit_range(qt.bits, qt.is_signed != 0, &blo, &bhi);
  if (clip_lo > clip_hi || clip_lo < blo || clip_hi > bhi) return HAGO_ERR_BITS;
  if (clip_lo < -(1 << 24) || clip_hi > (1 << 24)) return HAGO_ERR_BITS;
  return from_hip(hago::launch_quant(x, q, y, container, 2, outer, channels, inner, scale, zero_point,
                                     per_channel, clip_lo, clip_hi, static_cast<hipStream_t>(stream)));
}

hago_status hago_dequantize(const void* q, hago_qtype qt, float* y, int64_t outer, int64_t channels,
                            int64_t inner, const float* scale, const int32_t* zero_point,
                            int32_t per_channel, void* stream) {
  int container = 0;
  hago_status s = check_quant(qt, per_channel, outer, channels, inner, scale, zero_point, &container);
  if (s != HAGO_OK) return s;
  const bool empty = outer == 0 || channels == 0 || inner == 0;
  if ((!q || !y) && !empty) return HAGO_ERR_NULL;
  return from_hip(hago::launch_quant(q, y, nullptr, container, 1, outer, channels, inner, scale, zero_point,
                                     per_channel, 0, 0, static_cast<hipStream_t>(stream)));
}

hago_status hago_absmax(const float* x, int64_t outer, int64_t channels, int64_t inner,
                        int32_t per_channel, float* threshold, void* stream) {
  if (outer < 0 || channels < 0 || inner < 0) return HAGO_ERR_SHAPE;
  if (per_channel != 0 && per_channel != 1) return HAGO_ERR_PARAM;
  const bool empty = outer == 0 || channels == 0 || inner == 0;
  const int64_t nthr = per_channel ? channels : 1;
  if ((!x && !empty) || (!threshold && nthr > 0)) return HAGO_ERR_NULL;
  if (!empty) {
    if (outer > INT64_MAX / channels || outer * channels > INT64_MAX / inner) return HAGO_ERR_SHAPE;
  }
  return from_hip(hago::launch_absmax(x, outer, channels, inner, per_channel, threshold,
                                      static_cast<hipStream_t>(stream)));
}

hago_status hago_requantize(const void* acc, hago_dtype acc_dtype, int64_t outer, int64_t channels,
                            int64_t inner, const hago_requant* rq, void* out, void* stream) {
  if (outer < 0 || channels < 0 || inner < 0) return HAGO_ERR_SHAPE;
  const bool rq_empty = outer == 0 || channels == 0 || inner == 0;
  if (((!acc || !out) && !rq_empty) || !rq) return HAGO_ERR_NULL;
  if (acc_dtype != HAGO_I32 && acc_dtype != HAGO_I16) return HAGO_ERR_DTYPE;
  RequantArgs ra{};
  hago_status s = check_requant(rq, &ra);
  if (s != HAGO_OK) return s;
  if (outer && channels && inner) {
    if (outer > INT64_MAX / channels || outer * channels > INT64_MAX / inner) return HAGO_ERR_SHAPE;
  }
  return from_hip(hago::launch_requantize(acc, acc_dtype == HAGO_I16, outer, channels, inner, ra,
                                          out, static_cast<hipStream_t>(stream)));
}

hago_status hago_qdense(const void* a, hago_qtype a_t, const void* w, hago_qtype w_t,
                        const int32_t* bias, int64_t M, int64_t N, int64_t K, hago_dtype acc_dtype,
                        const hago_requant* rq, void* out, uint32_t flags, void* stream) {
  GemmArgs g{};
  if (M < 0 || N < 0 || K < 0) return HAGO_ERR_SHAPE;
  hago_status s = check_operands(a, a_t, w, w_t, acc_dtype, rq, out, flags, K, M == 0 || K == 0,
                                 N == 0 || K == 0, M == 0 || N == 0, &g);
  if (s != HAGO_OK) return s;
  // tile counts, row offsets inside a tile and K + 64 use 32-bit arithmetic
  if (M > kI32Max - 512 || N > kI32Max - 512 || K > kI32Max - 512) return HAGO_ERR_SHAPE;
  g.bias = bias;
  g.M = (int32_t)M;
  g.N = (int32_t)N;
  g.K = (int32_t)K;
  return from_hip(hago::launch_qdense(g, static_cast<hipStream_t>(stream)));
}

}  // extern "C"

namespace {

// Geometry checks shared by the convolution entry points, in two steps (the operand checks come
// between them): the scalars, then the 32-bit index limits; the second fills cg.
hago_status check_conv_scalars(hago_layout layout, int64_t B, int64_t C, int64_t H, int64_t W, int64_t O,
                               int32_t KH, int32_t KW, int32_t stride_h, int32_t stride_w, int32_t pad_h,
                               int32_t pad_w, int32_t groups, int64_t* kred, bool* depthwise) {
  if (B < 0 || C < 1 || H < 1 || W < 1 || O < 1 || KH < 1 || KW < 1 || stride_h < 1 ||
      stride_w < 1 || pad_h < 0 || pad_w < 0)
    return HAGO_ERR_SHAPE;
  if (layout != HAGO_NCHW && layout != HAGO_NHWC) return HAGO_ERR_SHAPE;
  *depthwise = (groups != 1) && (groups == C) && (groups == O);
  if (groups != 1 && !*depthwise) return HAGO_ERR_SHAPE;
  if (H + 2 * (int64_t)pad_h < KH || W + 2 * (int64_t)pad_w < KW) return HAGO_ERR_SHAPE;
  *kred = *depthwise ? (int64_t)KH * KW : C * (int64_t)KH * KW;
  return HAGO_OK;
}

hago_status check_conv_limits(hago_layout layout, int64_t B, int64_t C, int64_t H, int64_t W, int64_t O,
                              int32_t KH, int32_t KW, int32_t stride_h, int32_t stride_w, int32_t pad_h,
                              int32_t pad_w, int64_t kred, ConvGeom* cg) {
  const int64_t OH = (H + 2 * (int64_t)pad_h - KH) / stride_h + 1;
  const int64_t OW = (W + 2 * (int64_t)pad_w - KW) / stride_w + 1;
  // every flat offset into the input, weights and (per image) output fits 31 bits
  const int64_t lim = kI32Max - 512;
  if (KH > 4096 || KW > 4096 || pad_h > 4096 || pad_w > 4096 || stride_h > 4096 ||
      stride_w > 4096)
    return HAGO_ERR_SHAPE;
  if (C > lim || H > lim || W > lim || O > lim || B > lim) return HAGO_ERR_SHAPE;
  if ((B ? B : 1) * C > lim / H / W) return HAGO_ERR_SHAPE;         // input elements
  if ((B ? B : 1) * OH * OW > lim) return HAGO_ERR_SHAPE;            // GEMM rows
  if ((B ? B : 1) * O > lim / OH / OW) return HAGO_ERR_SHAPE;        // output elements
  if (O * kred > lim) return HAGO_ERR_SHAPE;                          // weight elements
  cg->B = (int32_t)B; cg->C = (int32_t)C; cg->H = (int32_t)H; cg->W = (int32_t)W; cg->O = (int32_t)O;
  cg->OH = (int32_t)OH; cg->OW = (int32_t)OW; cg->KH = KH; cg->KW = KW;
  cg->stride_h = stride_h; cg->stride_w = stride_w; cg->pad_h = pad_h; cg->pad_w = pad_w;
  cg->nhwc = layout == HAGO_NHWC;
  return HAGO_OK;
}

// Scratch the convolution asks for: 0 for depthwise and for geometries only the generic kernel serves.
int64_t conv_scratch_need(const ConvGeom& cg, bool depthwise) {
  if (depthwise || cg.B == 0) return 0;
  const int64_t n = hago::qconv_workspace_bytes(cg);
  return n < 0 ? 0 : n;
}

enum class Scratch { kNone, kCaller, kStatic };

hago_status qconv2d_impl(const void* a, hago_qtype a_t, const void* w, hago_qtype w_t,
                         const int32_t* bias, hago_layout layout, int64_t B, int64_t C, int64_t H,
                         int64_t W, int64_t O, int32_t KH, int32_t KW, int32_t stride_h,
                         int32_t stride_w, int32_t pad_h, int32_t pad_w, int32_t groups,
                         hago_dtype acc_dtype, const hago_requant* rq, void* out, uint32_t flags,
                         void* stream, Scratch mode, void* workspace, int64_t workspace_bytes) {
  GemmArgs g{};
  ConvGeom cg{};
  int64_t Kred = 0;
  bool depthwise = false;
  hago_status s = check_conv_scalars(layout, B, C, H, W, O, KH, KW, stride_h, stride_w, pad_h, pad_w,
                                     groups, &Kred, &depthwise);
  if (s != HAGO_OK) return s;
  const uint32_t ws_flags = mode == Scratch::kCaller ? HAGO_WS_WEIGHTS_READY : 0u;
  s = check_operands(a, a_t, w, w_t, acc_dtype, rq, out, flags & ~ws_flags, Kred, B == 0, false,
                     B == 0, &g);
  if (s != HAGO_OK) return s;
  s = check_conv_limits(layout, B, C, H, W, O, KH, KW, stride_h, stride_w, pad_h, pad_w, Kred, &cg);
  if (s != HAGO_OK) return s;
  g.bias = bias;
  g.M = (int32_t)(B * cg.OH * cg.OW);
  g.N = (int32_t)O;
  g.K = (int32_t)Kred;
  hipStream_t st = static_cast<hipStream_t>(stream);
  if (depthwise && g.operand16) return HAGO_ERR_DTYPE;  // int16 operands: groups == 1 only
  if (depthwise) return from_hip(hago::launch_qconv_depthwise(g, cg, st));
  void* ws = nullptr;
  if (mode == Scratch::kCaller) {
    const int64_t need = conv_scratch_need(cg, false);
    if (need > 0) {
      if (!workspace) return HAGO_ERR_NULL;
      if (workspace_bytes < need || (reinterpret_cast<uintptr_t>(workspace) & 255u) != 0) return HAGO_ERR_PARAM;
      ws = workspace;
    }
  } else if (mode == Scratch::kStatic) {
    const int64_t need = conv_scratch_need(cg, false);
    if (need > (int64_t)HAGO_STATIC_SCRATCH_BYTES) return HAGO_ERR_SCRATCH;
    if (need > 0) {
      int64_t cap = 0;
      if (hago::static_scratch(&ws, &cap) != hipSuccess) return HAGO_ERR_DEVICE;
    }
  }
  return from_hip(hago::launch_qconv_gemm(g, cg, ws, (flags & HAGO_WS_WEIGHTS_READY) != 0, st));
}

}  // namespace

extern "C" {

hago_status hago_qconv2d(const void* a, hago_qtype a_t, const void* w, hago_qtype w_t,
                         const int32_t* bias, hago_layout layout, int64_t B, int64_t C, int64_t H,
                         int64_t W, int64_t O, int32_t KH, int32_t KW, int32_t stride_h,
                         int32_t stride_w, int32_t pad_h, int32_t pad_w, int32_t groups,
                         hago_dtype acc_dtype, const hago_requant* rq, void* out, uint32_t flags,
                         void* stream) {
  return qconv2d_impl(a, a_t, w, w_t, bias, layout, B, C, H, W, O, KH, KW, stride_h, stride_w, pad_h,
                      pad_w, groups, acc_dtype, rq, out, flags, stream, Scratch::kNone, nullptr, 0);
}

int64_t hago_qconv2d_workspace_bytes(hago_layout layout, int64_t B, int64_t C, int64_t H, int64_t W,
                                     int64_t O, int32_t KH, int32_t KW, int32_t stride_h,
                                     int32_t stride_w, int32_t pad_h, int32_t pad_w, int32_t groups) {
  ConvGeom cg{};
  int64_t Kred = 0;
  bool depthwise = false;
  if (check_conv_scalars(layout, B, C, H, W, O, KH, KW, stride_h, stride_w, pad_h, pad_w, groups, &Kred,
                         &depthwise) != HAGO_OK ||
      check_conv_limits(layout, B, C, H, W, O, KH, KW, stride_h, stride_w, pad_h, pad_w, Kred, &cg) != HAGO_OK)
    return -1;
  return conv_scratch_need(cg, depthwise);
}

hago_status hago_qconv2d_ws(const void* a, hago_qtype a_t, const void* w, hago_qtype w_t,
                            const int32_t* bias, hago_layout layout, int64_t B, int64_t C, int64_t H,
                            int64_t W, int64_t O, int32_t KH, int32_t KW, int32_t stride_h,
                            int32_t stride_w, int32_t pad_h, int32_t pad_w, int32_t groups,
                            hago_dtype acc_dtype, const hago_requant* rq, void* out,
                            void* workspace, int64_t workspace_bytes, uint32_t flags, void* stream) {
  if (workspace_bytes < 0) return HAGO_ERR_PARAM;
  return qconv2d_impl(a, a_t, w, w_t, bias, layout, B, C, H, W, O, KH, KW, stride_h, stride_w, pad_h,
                      pad_w, groups, acc_dtype, rq, out, flags, stream, Scratch::kCaller, workspace,
                      workspace_bytes);
}

hago_status hago_qconv2d_static(const void* a, hago_qtype a_t, const void* w, hago_qtype w_t,
                                const int32_t* bias, hago_layout layout, int64_t B, int64_t C,
                                int64_t H, int64_t W, int64_t O, int32_t KH, int32_t KW,
                                int32_t stride_h, int32_t stride_w, int32_t pad_h, int32_t pad_w,
                                int32_t groups, hago_dtype acc_dtype, const hago_requant* rq,
                                void* out, uint32_t flags, void* stream) {
  return qconv2d_impl(a, a_t, w, w_t, bias, layout, B, C, H, W, O, KH, KW, stride_h, stride_w, pad_h,
                      pad_w, groups, acc_dtype, rq, out, flags, stream, Scratch::kStatic, nullptr, 0);
}

void hago_set_test_hook(int32_t key, int32_t value) { hago::set_test_hook(key, value); }

hago_status hago_bit_range(int32_t bits, int32_t is_signed, int32_t* lo, int32_t* hi) {
  if (!lo || !hi) return HAGO_ERR_NULL;
  if (bits < 1 || bits > 32 || (bits == 32 && !is_signed)) return HAGO_ERR_BITS;
  int64_t l, h;
  bit_range(bits, is_signed != 0, &l, &h);
  *lo = (int32_t)l;
  *hi = (int32_t)h;
  return HAGO_OK;
}

}  // extern "C"
