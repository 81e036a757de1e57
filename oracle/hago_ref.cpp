/*
 * hago_ref.cpp -- CPU oracle (TEST INFRASTRUCTURE ONLY; see hago_ref.h).
 *
 * Plain scalar C++17.  Every operator is the written-out definition: no
 * blocking, no fusion, no reordering, no intrinsics.  Build with
 *   g++ -O2 -std=c++17 -ffp-contract=off -fno-fast-math -shared -fPIC
 * Integer sums are carried in uint32_t so that two's-complement wrap-around
 * is defined behaviour.
 */
#include "hago_ref.h"

#include <cmath>
#include <cstddef>
#include <cstdint>

namespace {

inline int32_t load_operand(const void* p, int32_t dtype, int64_t i) {
  if (dtype == REF_U8) return (int32_t) static_cast<const uint8_t*>(p)[i];
  if (dtype == REF_I16) return (int32_t) static_cast<const int16_t*>(p)[i];
  return (int32_t) static_cast<const int8_t*>(p)[i];
}

/* Operand triples: (u8 | i8) x i8, or i16 x i16 (Sec. 1, Sec. 4.1). */
inline bool operand_pair_ok(int32_t a_dtype, int32_t w_dtype, int32_t acc_dtype) {
  if (w_dtype == REF_I8) return a_dtype == REF_U8 || a_dtype == REF_I8;
  if (w_dtype == REF_I16) return a_dtype == REF_I16 && acc_dtype != REF_I16;
  return false;
}

inline bool acc_dtype_ok(int32_t dtype) {
  return dtype == REF_I32 || dtype == REF_I16 || dtype == REF_I24;
}

/* Reduce a 32-bit wrapped sum to the accumulator type and sign-extend. */
inline int32_t finish_acc(uint32_t sum, int32_t acc_dtype) {
  if (acc_dtype == REF_I16) return (int32_t)(int16_t)(uint16_t)(sum & 0xFFFFu);
  if (acc_dtype == REF_I24) {
    const uint32_t low = sum & 0xFFFFFFu;
    return (low & 0x800000u) ? (int32_t)low - (int32_t)0x1000000 : (int32_t)low;
  }
  return (int32_t)sum;
}

bool requant_ok(const ref_requant* rq, int64_t channels) {
  if (!rq->shift) return false;
  if (rq->out_dtype != REF_I8 && rq->out_dtype != REF_U8) return false;
  if (rq->clip_lo > rq->clip_hi) return false;
  if (rq->rounding != REF_ROUND_UPWARD && rq->rounding != REF_ROUND_HALF_AWAY) return false;
  const int64_t n = rq->per_channel ? channels : 1;
  for (int64_t c = 0; c < n; ++c)
    if (rq->shift[c] < 0 || rq->shift[c] > 31) return false;
  return true;
}

/* Store one accumulator at flat index i of `out`, channel c. */
inline void emit(void* out, int64_t i, int64_t c, int32_t acc,
                 int32_t acc_dtype, const ref_requant* rq) {
  if (!rq) {
    if (acc_dtype == REF_I16)
      static_cast<int16_t*>(out)[i] = (int16_t)acc;
    else /* int32, and 24 bits sign-extended into an int32 */
      static_cast<int32_t*>(out)[i] = acc;
    return;
  }
  const int64_t pc = rq->per_channel ? c : 0;
  const int64_t v =
      rq->multiplier
          ? hago_ref_requantize_one_mode(acc, rq->multiplier[pc], rq->shift[pc],
                                         rq->out_zero_point, rq->clip_lo,
                                         rq->clip_hi, rq->rounding)
          : hago_ref_requantize_shift_one(acc, rq->shift[pc], rq->out_zero_point,
                                          rq->clip_lo, rq->clip_hi, rq->rounding);
  if (rq->out_dtype == REF_U8)
    static_cast<uint8_t*>(out)[i] = (uint8_t)v;
  else
    static_cast<int8_t*>(out)[i] = (int8_t)v;
}

}  // namespace

extern "C" {

double hago_ref_scale(double threshold, int32_t bits, int32_t sign) {
  return threshold / std::ldexp(1.0, bits - sign);
}

int hago_ref_absmax(const float* x, int64_t outer, int64_t channels,
                    int64_t inner, int32_t per_channel, float* thr) {
  if (!x || !thr) return REF_ERR_NULL;
  if (outer < 0 || channels < 0 || inner < 0) return REF_ERR_SHAPE;
  const int64_t n = per_channel ? channels : 1;
  for (int64_t c = 0; c < n; ++c) thr[c] = 0.0f;
  for (int64_t o = 0; o < outer; ++o)
    for (int64_t c = 0; c < channels; ++c)
      for (int64_t i = 0; i < inner; ++i) {
        const float v = std::fabs(x[(o * channels + c) * inner + i]);
        float& t = thr[per_channel ? c : 0];
        if (v > t) t = v;
      }
  return REF_OK;
}

int hago_ref_bit_range(int32_t bits, int32_t is_signed, int32_t* lo,
                       int32_t* hi) {
  if (!lo || !hi) return REF_ERR_NULL;
  if (bits < 1 || bits > 31) return REF_ERR_BITS;
  if (is_signed) {
    *lo = -(int32_t)(1u << (bits - 1));
    *hi = (int32_t)(1u << (bits - 1)) - 1;
  } else {
    *lo = 0;
    *hi = (int32_t)((1u << bits) - 1u);
  }
  return REF_OK;
}

int hago_ref_simquant(const float* x, float* y, int64_t outer,
                      int64_t channels, int64_t inner, const float* scale,
                      const int32_t* zero_point, int32_t per_channel,
                      int32_t clip_lo, int32_t clip_hi) {
  if (!x || !y || !scale || !zero_point) return REF_ERR_NULL;
  if (outer < 0 || channels < 0 || inner < 0) return REF_ERR_SHAPE;
  if (clip_lo > clip_hi) return REF_ERR_BITS;
  const float lo = (float)clip_lo;
  const float hi = (float)clip_hi;
  for (int64_t o = 0; o < outer; ++o)
    for (int64_t c = 0; c < channels; ++c) {
      const float s = scale[per_channel ? c : 0];
      const float zf = (float)zero_point[per_channel ? c : 0];
      for (int64_t i = 0; i < inner; ++i) {
        const int64_t idx = (o * channels + c) * inner + i;
        const float t = x[idx] / s;          /* Eq. 3: r / s        */
        const float u = std::nearbyintf(t);  /* round, ties to even */
        float v = u + zf;                    /* integer code        */
        v = (v < lo) ? lo : ((v > hi) ? hi : v); /* saturation      */
        y[idx] = (v - zf) * s;               /* r ~= q * s          */
      }
    }
  return REF_OK;
}

int hago_ref_quantize(const float* x, int32_t* q, int64_t outer,
                      int64_t channels, int64_t inner, const float* scale,
                      const int32_t* zero_point, int32_t per_channel,
                      int32_t clip_lo, int32_t clip_hi) {
  if (!x || !q || !scale || !zero_point) return REF_ERR_NULL;
  if (outer < 0 || channels < 0 || inner < 0) return REF_ERR_SHAPE;
  if (clip_lo > clip_hi) return REF_ERR_BITS;
  for (int64_t o = 0; o < outer; ++o)
    for (int64_t c = 0; c < channels; ++c) {
      const float s = scale[per_channel ? c : 0];
      const int64_t z = zero_point[per_channel ? c : 0];
      for (int64_t i = 0; i < inner; ++i) {
        const int64_t idx = (o * channels + c) * inner + i;
        const float u = std::nearbyintf(x[idx] / s); /* round(r / s) */
        int64_t code;
        if (u != u) code = z;                        /* NaN: real zero */
        else if (u >= 4.0e18f) code = INT64_MAX / 2; /* saturates below */
        else if (u <= -4.0e18f) code = -(INT64_MAX / 2);
        else code = (int64_t)u + z;                  /* u is an integer */
        if (code < clip_lo) code = clip_lo;
        if (code > clip_hi) code = clip_hi;
        q[idx] = (int32_t)code;
      }
    }
  return REF_OK;
}

int hago_ref_dequantize(const int32_t* q, float* y, int64_t outer,
                        int64_t channels, int64_t inner, const float* scale,
                        const int32_t* zero_point, int32_t per_channel) {
  if (!q || !y || !scale || !zero_point) return REF_ERR_NULL;
  if (outer < 0 || channels < 0 || inner < 0) return REF_ERR_SHAPE;
  for (int64_t o = 0; o < outer; ++o)
    for (int64_t c = 0; c < channels; ++c) {
      const float s = scale[per_channel ? c : 0];
      const float zf = (float)zero_point[per_channel ? c : 0];
      for (int64_t i = 0; i < inner; ++i) {
        const int64_t idx = (o * channels + c) * inner + i;
        y[idx] = ((float)q[idx] - zf) * s; /* r ~= q * s */
      }
    }
  return REF_OK;
}

int hago_ref_encode_multiplier(double m, int32_t* multiplier, int32_t* shift) {
  if (!multiplier || !shift) return REF_ERR_NULL;
  if (!(m > 0.0) || !std::isfinite(m)) return REF_ERR_PARAM;
  int e = 0;
  const double f = std::frexp(m, &e); /* m = f * 2^e, f in [0.5, 1) */
  long long q = std::llround(std::ldexp(f, 31));
  if (q == (1LL << 31)) { /* f rounded up to 1.0 */
    q = 1LL << 30;
    e += 1;
  }
  const int sh = -e;
  if (sh < 0 || sh > 31) return REF_ERR_PARAM;
  *multiplier = (int32_t)q;
  *shift = (int32_t)sh;
  return REF_OK;
}

int64_t hago_ref_requantize_one(int32_t acc, int32_t multiplier, int32_t shift,
                                int32_t z_out, int32_t lo, int32_t hi) {
  const int64_t p = (int64_t)acc * (int64_t)multiplier; /* |p| < 2^62 */
  const int t = 31 + shift;
  /* add one half in units of 2^-t, then floor: arithmetic right shift */
  const int64_t r = (p + ((int64_t)1 << (t - 1))) >> t;
  int64_t o = r + (int64_t)z_out;
  if (o < (int64_t)lo) o = lo;
  if (o > (int64_t)hi) o = hi;
  return o;
}

int64_t hago_ref_requantize_one_mode(int32_t acc, int32_t multiplier,
                                     int32_t shift, int32_t z_out, int32_t lo,
                                     int32_t hi, int32_t rounding) {
  if (rounding == REF_ROUND_UPWARD)
    return hago_ref_requantize_one(acc, multiplier, shift, z_out, lo, hi);
  /* nearest integer to p / 2^t, halves away from zero: round the magnitude
   * half up and give it the sign back */
  const int64_t p = (int64_t)acc * (int64_t)multiplier; /* |p| < 2^62 */
  const int t = 31 + shift;
  const int64_t half = (int64_t)1 << (t - 1);
  const int64_t mag = ((p < 0 ? -p : p) + half) >> t;
  int64_t o = (p < 0 ? -mag : mag) + (int64_t)z_out;
  if (o < (int64_t)lo) o = lo;
  if (o > (int64_t)hi) o = hi;
  return o;
}

int64_t hago_ref_requantize_shift_one(int32_t acc, int32_t shift, int32_t z_out,
                                      int32_t lo, int32_t hi, int32_t rounding) {
  const int64_t p = (int64_t)acc;
  int64_t r;
  if (shift <= 0) {
    r = p; /* scale 1: nothing to round */
  } else {
    const int64_t half = (int64_t)1 << (shift - 1);
    if (rounding == REF_ROUND_HALF_AWAY) {
      const int64_t mag = ((p < 0 ? -p : p) + half) >> shift;
      r = p < 0 ? -mag : mag;
    } else {
      r = (p + half) >> shift; /* floor(acc / 2^sh + 1/2) */
    }
  }
  int64_t o = r + (int64_t)z_out;
  if (o < (int64_t)lo) o = lo;
  if (o > (int64_t)hi) o = hi;
  return o;
}

int hago_ref_requantize(const void* acc, int32_t acc_dtype, int64_t outer,
                        int64_t channels, int64_t inner, const ref_requant* rq,
                        void* out) {
  if (!acc || !rq || !out) return REF_ERR_NULL;
  if (outer < 0 || channels < 0 || inner < 0) return REF_ERR_SHAPE;
  if (acc_dtype != REF_I32 && acc_dtype != REF_I16) return REF_ERR_DTYPE;
  if (!requant_ok(rq, channels)) return REF_ERR_PARAM;
  for (int64_t o = 0; o < outer; ++o)
    for (int64_t c = 0; c < channels; ++c)
      for (int64_t i = 0; i < inner; ++i) {
        const int64_t idx = (o * channels + c) * inner + i;
        const int32_t v = (acc_dtype == REF_I16)
                              ? (int32_t) static_cast<const int16_t*>(acc)[idx]
                              : static_cast<const int32_t*>(acc)[idx];
        emit(out, idx, c, v, REF_I32, rq);
      }
  return REF_OK;
}

int hago_ref_acc16_safe(int64_t K, int64_t a_absmax, int64_t w_absmax) {
  /* sizes here are tiny; guard the product anyway */
  if (K < 0 || a_absmax < 0 || w_absmax < 0) return 0;
  if (K == 0 || a_absmax == 0 || w_absmax == 0) return 1;
  if (a_absmax > 32767 || w_absmax > 32767 || K > 32767) return 0;
  return (K * a_absmax * w_absmax <= 32767) ? 1 : 0;
}

int hago_ref_acc_safe(int64_t K, int64_t a_absmax, int64_t w_absmax,
                      int32_t acc_bits) {
  if (acc_bits != 16 && acc_bits != 24 && acc_bits != 32) return 0;
  const int64_t limit = ((int64_t)1 << (acc_bits - 1)) - 1;
  if (K < 0 || a_absmax < 0 || w_absmax < 0) return 0;
  if (K == 0 || a_absmax == 0 || w_absmax == 0) return 1;
  if (a_absmax > limit || w_absmax > limit || K > limit) return 0;
  if (a_absmax > limit / w_absmax) return 0; /* the product alone is too large */
  if (K > limit / (a_absmax * w_absmax)) return 0;
  return 1;
}

int hago_ref_simquant_wrap(const float* x, float* y, int64_t outer,
                           int64_t channels, int64_t inner, const float* scale,
                           const int32_t* zero_point, int32_t per_channel,
                           int32_t wrap_bits, int32_t wrap_signed,
                           int32_t clip_lo, int32_t clip_hi) {
  if (!x || !y || !scale || !zero_point) return REF_ERR_NULL;
  if (outer < 0 || channels < 0 || inner < 0) return REF_ERR_SHAPE;
  if (clip_lo > clip_hi || wrap_bits < 2 || wrap_bits > 32) return REF_ERR_BITS;
  const float lo = (float)clip_lo;
  const float hi = (float)clip_hi;
  const int64_t modulus = (int64_t)1 << wrap_bits;
  const int64_t top = (int64_t)1 << (wrap_bits - 1);
  for (int64_t o = 0; o < outer; ++o)
    for (int64_t c = 0; c < channels; ++c) {
      const float s = scale[per_channel ? c : 0];
      const float zf = (float)zero_point[per_channel ? c : 0];
      for (int64_t i = 0; i < inner; ++i) {
        const int64_t idx = (o * channels + c) * inner + i;
        const float t = x[idx] / s;          /* Eq. 3: r / s        */
        const float u = std::nearbyintf(t);  /* round, ties to even */
        float v = u + zf;                    /* integer code        */
        if (v == v) {                        /* not NaN: overflow   */
          int64_t code = 0;                  /* huge and infinite codes: 0 */
          if (v > -4.0e18f && v < 4.0e18f) {
            code = (int64_t)v;               /* v holds an integer  */
            code = ((code % modulus) + modulus) % modulus; /* 0 .. 2^b - 1 */
            if (wrap_signed && code >= top) code -= modulus; /* two's complement */
          }
          v = (float)code;
        }
        v = (v < lo) ? lo : ((v > hi) ? hi : v); /* saturation      */
        y[idx] = (v - zf) * s;               /* r ~= q * s          */
      }
    }
  return REF_OK;
}

int hago_ref_qdense(const void* a, int32_t a_dtype, int32_t a_zero_point,
                    const int8_t* w, const int32_t* bias, int64_t M, int64_t N,
                    int64_t K, int32_t acc_dtype, const ref_requant* rq,
                    void* out) {
  return hago_ref_qdense_x(a, a_dtype, a_zero_point, w, REF_I8, bias, M, N, K,
                           acc_dtype, rq, out);
}

int hago_ref_qdense_x(const void* a, int32_t a_dtype, int32_t a_zero_point,
                      const void* w, int32_t w_dtype, const int32_t* bias,
                      int64_t M, int64_t N, int64_t K, int32_t acc_dtype,
                      const ref_requant* rq, void* out) {
  if (!a || !w || !out) return REF_ERR_NULL;
  if (M < 0 || N < 0 || K < 0) return REF_ERR_SHAPE;
  if (!acc_dtype_ok(acc_dtype) || !operand_pair_ok(a_dtype, w_dtype, acc_dtype))
    return REF_ERR_DTYPE;
  if (rq && !requant_ok(rq, N)) return REF_ERR_PARAM;
  for (int64_t m = 0; m < M; ++m)
    for (int64_t n = 0; n < N; ++n) {
      uint32_t sum = bias ? (uint32_t)bias[n] : 0u;
      for (int64_t k = 0; k < K; ++k) {
        const int64_t av = load_operand(a, a_dtype, m * K + k) - a_zero_point;
        const int64_t wv = load_operand(w, w_dtype, n * K + k);
        sum += (uint32_t)(uint64_t)(av * wv); /* exact product, sum mod 2^32 */
      }
      emit(out, m * N + n, n, finish_acc(sum, acc_dtype), acc_dtype, rq);
    }
  return REF_OK;
}

int hago_ref_qconv2d(const void* a, int32_t a_dtype, int32_t a_zero_point,
                     const int8_t* w, const int32_t* bias, int32_t layout,
                     int64_t B, int64_t C, int64_t H, int64_t W, int64_t O,
                     int32_t KH, int32_t KW, int32_t stride_h, int32_t stride_w,
                     int32_t pad_h, int32_t pad_w, int32_t groups,
                     int32_t acc_dtype, const ref_requant* rq, void* out) {
  return hago_ref_qconv2d_x(a, a_dtype, a_zero_point, w, REF_I8, bias, layout, B,
                            C, H, W, O, KH, KW, stride_h, stride_w, pad_h, pad_w,
                            groups, acc_dtype, rq, out);
}

int hago_ref_qconv2d_x(const void* a, int32_t a_dtype, int32_t a_zero_point,
                       const void* w, int32_t w_dtype, const int32_t* bias,
                       int32_t layout, int64_t B, int64_t C, int64_t H, int64_t W,
                       int64_t O, int32_t KH, int32_t KW, int32_t stride_h,
                       int32_t stride_w, int32_t pad_h, int32_t pad_w,
                       int32_t groups, int32_t acc_dtype, const ref_requant* rq,
                       void* out) {
  if (!a || !w || !out) return REF_ERR_NULL;
  if (B < 0 || C < 1 || H < 1 || W < 1 || O < 1 || KH < 1 || KW < 1 ||
      stride_h < 1 || stride_w < 1 || pad_h < 0 || pad_w < 0)
    return REF_ERR_SHAPE;
  if (groups < 1 || C % groups != 0 || O % groups != 0) return REF_ERR_SHAPE;
  if (layout != REF_NCHW && layout != REF_NHWC) return REF_ERR_SHAPE;
  if (H + 2 * (int64_t)pad_h < KH || W + 2 * (int64_t)pad_w < KW)
    return REF_ERR_SHAPE;
  if (!acc_dtype_ok(acc_dtype) || !operand_pair_ok(a_dtype, w_dtype, acc_dtype))
    return REF_ERR_DTYPE;
  if (rq && !requant_ok(rq, O)) return REF_ERR_PARAM;

  const int64_t OH = (H + 2 * pad_h - KH) / stride_h + 1;
  const int64_t OW = (W + 2 * pad_w - KW) / stride_w + 1;
  const int64_t Cg = C / groups; /* input channels per group  */
  const int64_t Og = O / groups; /* output channels per group */
  const bool nchw = (layout == REF_NCHW);

  for (int64_t b = 0; b < B; ++b)
    for (int64_t o = 0; o < O; ++o) {
      const int64_t g = o / Og;
      for (int64_t oy = 0; oy < OH; ++oy)
        for (int64_t ox = 0; ox < OW; ++ox) {
          uint32_t sum = bias ? (uint32_t)bias[o] : 0u;
          for (int64_t ci = 0; ci < Cg; ++ci) {
            const int64_t c = g * Cg + ci;
            for (int64_t ky = 0; ky < KH; ++ky) {
              const int64_t iy = oy * stride_h + ky - pad_h;
              if (iy < 0 || iy >= H) continue; /* tap outside: adds 0 */
              for (int64_t kx = 0; kx < KW; ++kx) {
                const int64_t ix = ox * stride_w + kx - pad_w;
                if (ix < 0 || ix >= W) continue;
                const int64_t ai = nchw ? ((b * C + c) * H + iy) * W + ix
                                        : ((b * H + iy) * W + ix) * C + c;
                const int64_t wi = nchw ? ((o * Cg + ci) * KH + ky) * KW + kx
                                        : ((o * KH + ky) * KW + kx) * Cg + ci;
                const int64_t av = load_operand(a, a_dtype, ai) - a_zero_point;
                const int64_t wv = load_operand(w, w_dtype, wi);
                sum += (uint32_t)(uint64_t)(av * wv); /* exact product, sum mod 2^32 */
              }
            }
          }
          const int64_t oi = nchw ? ((b * O + o) * OH + oy) * OW + ox
                                  : ((b * OH + oy) * OW + ox) * O + o;
          emit(out, oi, o, finish_acc(sum, acc_dtype), acc_dtype, rq);
        }
    }
  return REF_OK;
}

} /* extern "C" */
