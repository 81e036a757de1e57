// Bandwidth-bound elementwise kernels: fp32 simulated_quantize, the standalone
// integer requantize and the max-abs calibration reduction.  The first two stream
// [outer, channels, inner] tensors once (read) and once (write); the only reuse is
// the per-channel parameter, which is block-uniform in the row kernels and so lives
// in scalar registers.  The reduction reads the tensor once.
//
// Two launch shapes per operator:
//   rows : one workgroup per (row = outer*channels index, segment of inner);
//          128-bit loads/stores; parameters fetched once per workgroup.
//   flat : one element per lane with the channel recovered by division; used
//          for short or unaligned rows (e.g. channel-last tensors).
#include "hago_device.h"
#include "launch.h"

#include <type_traits>

namespace hago {

namespace {

constexpr int kThreads = 256;
constexpr int kVecPerLane = 4;  // 128-bit vectors per lane and job of the row kernels

typedef float v4f __attribute__((ext_vector_type(4)));
typedef int32_t v4i32 __attribute__((ext_vector_type(4)));
typedef int16_t v4i16 __attribute__((ext_vector_type(4)));

// A row of inner_vec vectors is cut into nseg jobs of seg_len vectors, as even as possible.
inline void split_row(int64_t inner_vec, int u, int32_t* nseg, int32_t* seg_len) {
  const int64_t per_job = (int64_t)kThreads * u;
  const int64_t n = (inner_vec + per_job - 1) / per_job;
  *nseg = (int32_t)n;
  *seg_len = (int32_t)((inner_vec + n - 1) / n);
}

// Row and channel of a row kernel's job (job = row * nseg + segment).  A job streams a dozen
// kilobytes, so its bookkeeping counts: jobs below 2^32, the usual case, are divided with the
// host's reciprocals floor(2^32 / d) (a multiply-high and at most two corrections, all on
// wavefront-uniform values, i.e. scalar instructions) instead of the 25 vector instructions of an
// integer division each.
struct JobDiv {
  uint32_t inv_nseg, inv_channels;
};
inline uint32_t reciprocal32(int64_t d) { return d <= 1 ? 0xffffffffu : (uint32_t)((1ull << 32) / (uint64_t)d); }

__device__ __forceinline__ uint32_t div32(uint32_t n, uint32_t d, uint32_t inv, uint32_t& rem) {
  uint32_t q = __umulhi(n, inv);   // q - 2 <= this <= q
  uint32_t r = n - q * d;
  if (r >= d) { ++q; r -= d; }
  if (r >= d) { ++q; r -= d; }
  rem = r;
  return q;
}

__device__ __forceinline__ void job_row_channel(int64_t job, int32_t nseg, int32_t channels, int per_channel,
                                                JobDiv jd, int64_t& row, int32_t& c) {
  if (job <= 0xffffffffll) {
    uint32_t seg, cc;
    const uint32_t r32 = div32((uint32_t)job, (uint32_t)nseg, jd.inv_nseg, seg);
    row = r32;
    div32(r32, (uint32_t)channels, jd.inv_channels, cc);
    c = per_channel ? (int32_t)cc : 0;
  } else {
    row = job / nseg;
    c = per_channel ? (int32_t)(row % channels) : 0;
  }
}

// u = rintf(x / s), the rounded quotient of Eq. 3 (correctly rounded binary32 division, then
// round half to even), for a divisor that many elements share.  The division expands to about
// fifteen vector instructions, which made the row kernels issue-bound; this takes five on
// almost every element and gives the SAME value on every element:
//   rc = RN(1 / s), computed once per row with |s| in [2^-100, 2^100] (so rc is normal and within
//   2^-24 of 1 / s, relatively); qt = RN(x * rc) is within |x / s| * (2^-23 + 2^-48) of the
//   exact quotient, and so is RN(x / s) within |x / s| * 2^-24: the two differ by less than
//   |qt| * 2^-22.  With n = rintf(qt) and d = qt - n (exact: |qt| < 2^23 here), both lie strictly
//   inside (n - 1/2, n + 1/2) whenever |d| + |qt| * 2^-22 < 1/2, and then rintf of either is n
//   (an underflowing qt has n = 0, as the quotient has).  The test below asks for twice that margin,
//   which also covers the rounding of the threshold itself.
//   Anything else takes the division: quotients within about 2^-21 |qt| of a tie (one element in
//   2^14 for |qt| near 32), |qt| >= 2^20, infinities and NaN (every comparison false), and, through
//   rc = NaN, scales outside the range above.
__device__ __forceinline__ float quotient_reciprocal(float s) {
  const float a = fabsf(s);
  return (a >= 0x1p-100f && a <= 0x1p100f) ? 1.0f / s : __builtin_nanf("");
}

// Four elements at once, so that a kernel branches once per 128-bit vector: true when all four
// pass the test, and then n[e] = rintf(x[e] / s), all finite; otherwise the caller redoes the four
// with the division.
__device__ __forceinline__ bool fast_quotient4(v4f x, float rc, v4f& n) {
  bool ok = true;
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    const float qt = x[e] * rc;
    n[e] = rintf(qt);
    const float d = qt - n[e];
    const float thr = __builtin_fmaf(fabsf(qt), -0x1p-21f, 0.5f);
    ok = ok && (fabsf(d) < thr);
  }
  return ok;
}

// Eq. 3 with zero point and saturation, in binary32, from the rounded quotient u.  The scalar
// definition clips with two compare-selects, (v < lo) ? lo : ((v > hi) ? hi : v), under which NaN
// stays NaN; for every other v (lo <= hi, both finite) that is the median of the three, one
// instruction, and v is never -0 here (a sum that is zero is +0), so no zero changes sign.
__device__ __forceinline__ float simquant_of(float u, float s, float zf, float lo, float hi) {
  const float v = u + zf;
  const float c = (v != v) ? v : __builtin_amdgcn_fmed3f(v, lo, hi);
  return (c - zf) * s;
}

// The same for a finite u (what fast_quotient4 hands out): no NaN to keep.
__device__ __forceinline__ float simquant_of_finite(float u, float s, float zf, float lo, float hi) {
  return (__builtin_amdgcn_fmed3f(u + zf, lo, hi) - zf) * s;
}

__device__ __forceinline__ float simquant_one(float x, float s, float zf, float lo, float hi) {
  return simquant_of(rintf(x / s), s, zf, lo, hi);
}


// The same with the overflow of the simulated integer type (Sec. 5.2 of the paper: the third error
// source): the code is reduced modulo 2^wrap_bits before the clip, into the two's-complement range
// (wrap_signed) or into 0 .. 2^wrap_bits - 1.  A code of magnitude 4e18 or more, or an infinite one,
// reduces to 0 (every binary32 number that large is a multiple of 2^32); NaN stays NaN.
__device__ __forceinline__ float simquant_wrap_of(float u, float s, float zf, float lo, float hi,
                                                  int wrap_bits, int wrap_signed) {
  float v = u + zf;
  if (v == v) {
    long long code = 0;
    if (v > -4.0e18f && v < 4.0e18f) {
      code = (long long)v;  // v holds an integer below 2^62
      const int sh = 64 - wrap_bits;
      const unsigned long long low = (unsigned long long)code << sh;
      code = wrap_signed ? ((long long)low >> sh) : (long long)(low >> sh);
    }
    v = (float)code;  // exact up to 25 bits, round to nearest beyond
  }
  v = (v < lo) ? lo : ((v > hi) ? hi : v);
  return (v - zf) * s;
}

// U: 128-bit vectors per lane and job; all of a job's loads are issued before the first
// result is computed.  Loads and stores carry the nontemporal hint: the tensors are streamed
// once, and without the hint the copy rate of this chip is about 10 % lower.
// WRAP: the overflow-simulating form (wrap_bits, wrap_signed).
template <int U, bool WRAP = false>
__global__ __launch_bounds__(kThreads) void simquant_rows_kernel(
    const v4f* __restrict__ x, v4f* __restrict__ y, int64_t rows, int32_t channels,
    int64_t inner_vec, int32_t nseg, int32_t seg_len, const float* __restrict__ scale,
    const int32_t* __restrict__ zp, int per_channel, JobDiv jd, float lo, float hi, int wrap_bits = 0,
    int wrap_signed = 0) {
  for (int64_t job = blockIdx.x; job < rows * nseg; job += gridDim.x) {
    int64_t row;
    int32_t c;
    job_row_channel(job, nseg, channels, per_channel, jd, row, c);
    const int32_t seg = (int32_t)(job - row * nseg);
    const float s = scale[c];
    const float zf = (float)zp[c];
    const float rc = quotient_reciprocal(s);
    auto of = [&](float u, float s, float zf) {
      if constexpr (WRAP) return simquant_wrap_of(u, s, zf, lo, hi, wrap_bits, wrap_signed);
      else return simquant_of(u, s, zf, lo, hi);
    };
    const int64_t v0 = (int64_t)seg * seg_len;
    const int64_t v1 = (v0 + seg_len < inner_vec) ? v0 + seg_len : inner_vec;
    const v4f* xr = x + row * inner_vec;
    v4f* yr = y + row * inner_vec;
    for (int64_t vb = v0 + threadIdx.x; vb < v1; vb += (int64_t)kThreads * U) {
      v4f a[U];
#pragma unroll
      for (int u = 0; u < U; ++u)
        if (vb + u * kThreads < v1) a[u] = __builtin_nontemporal_load(xr + vb + u * kThreads);
#pragma unroll
      for (int u = 0; u < U; ++u) {
        if (vb + u * kThreads < v1) {
          v4f n, r;
          if (__builtin_expect(fast_quotient4(a[u], rc, n), 1)) {
            if constexpr (WRAP) r = v4f{of(n.x, s, zf), of(n.y, s, zf), of(n.z, s, zf), of(n.w, s, zf)};
            else r = v4f{simquant_of_finite(n.x, s, zf, lo, hi), simquant_of_finite(n.y, s, zf, lo, hi),
                         simquant_of_finite(n.z, s, zf, lo, hi), simquant_of_finite(n.w, s, zf, lo, hi)};
          } else {  // IEEE division (correctly rounded)
            r = v4f{of(rintf(a[u].x / s), s, zf), of(rintf(a[u].y / s), s, zf), of(rintf(a[u].z / s), s, zf),
                    of(rintf(a[u].w / s), s, zf)};
          }
          __builtin_nontemporal_store(r, yr + vb + u * kThreads);
        }
      }
    }
  }
}

// Batched candidates (Sec. 6.3): x is read ONCE and every candidate b writes its own
// y[b][...] with scale[b][c], zero_point[b][c] and clip range b.  4 + 4 B bytes per element
// instead of 8 B for B separate launches.
constexpr int kMaxCandidates = 16;
struct CandidateClips {
  float lo[kMaxCandidates], hi[kMaxCandidates];
};

template <int U>
__global__ __launch_bounds__(kThreads) void simquant_batched_rows_kernel(
    const v4f* __restrict__ x, v4f* __restrict__ y, int64_t rows, int32_t channels,
    int64_t inner_vec, int32_t nseg, int32_t seg_len, int32_t nbatch, int32_t nparam,
    const float* __restrict__ scale, const int32_t* __restrict__ zp, int per_channel, JobDiv jd,
    CandidateClips clips) {
  const int64_t batch_stride = rows * inner_vec;  // vectors per candidate output
  for (int64_t job = blockIdx.x; job < rows * nseg; job += gridDim.x) {
    int64_t row;
    int32_t c;
    job_row_channel(job, nseg, channels, per_channel, jd, row, c);
    const int32_t seg = (int32_t)(job - row * nseg);
    const int64_t v0 = (int64_t)seg * seg_len;
    const int64_t v1 = (v0 + seg_len < inner_vec) ? v0 + seg_len : inner_vec;
    const v4f* xr = x + row * inner_vec;
    v4f* yr = y + row * inner_vec;
    for (int64_t vb = v0 + threadIdx.x; vb < v1; vb += (int64_t)kThreads * U) {
      v4f a[U];
#pragma unroll
      for (int u = 0; u < U; ++u)
        if (vb + u * kThreads < v1) a[u] = __builtin_nontemporal_load(xr + vb + u * kThreads);
      for (int b = 0; b < nbatch; ++b) {
        const float s = scale[(int64_t)b * nparam + c];
        const float zf = (float)zp[(int64_t)b * nparam + c];
        const float lo = clips.lo[b], hi = clips.hi[b];
        const float rc = quotient_reciprocal(s);
#pragma unroll
        for (int u = 0; u < U; ++u) {
          if (vb + u * kThreads < v1) {
            v4f n, r;
            if (__builtin_expect(fast_quotient4(a[u], rc, n), 1)) {
              r = v4f{simquant_of_finite(n.x, s, zf, lo, hi), simquant_of_finite(n.y, s, zf, lo, hi),
                      simquant_of_finite(n.z, s, zf, lo, hi), simquant_of_finite(n.w, s, zf, lo, hi)};
            } else {
              r = v4f{simquant_one(a[u].x, s, zf, lo, hi), simquant_one(a[u].y, s, zf, lo, hi),
                      simquant_one(a[u].z, s, zf, lo, hi), simquant_one(a[u].w, s, zf, lo, hi)};
            }
            __builtin_nontemporal_store(r, yr + b * batch_stride + vb + u * kThreads);
          }
        }
      }
    }
  }
}

__global__ __launch_bounds__(kThreads) void simquant_batched_flat_kernel(
    const float* __restrict__ x, float* __restrict__ y, int64_t total, int64_t inner,
    int64_t channels, int32_t nbatch, int32_t nparam, const float* __restrict__ scale,
    const int32_t* __restrict__ zp, int per_channel, CandidateClips clips) {
  const int64_t stride = (int64_t)gridDim.x * kThreads;
  for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < total; i += stride) {
    const int64_t c = per_channel ? (i / inner) % channels : 0;
    const float v = x[i];
    for (int b = 0; b < nbatch; ++b)
      y[(int64_t)b * total + i] = simquant_one(v, scale[(int64_t)b * nparam + c],
                                               (float)zp[(int64_t)b * nparam + c], clips.lo[b],
                                               clips.hi[b]);
  }
}

template <bool WRAP = false>
__global__ __launch_bounds__(kThreads) void simquant_flat_kernel(
    const float* __restrict__ x, float* __restrict__ y, int64_t total, int64_t inner,
    int64_t channels, const float* __restrict__ scale, const int32_t* __restrict__ zp,
    int per_channel, float lo, float hi, int wrap_bits = 0, int wrap_signed = 0) {
  const int64_t stride = (int64_t)gridDim.x * kThreads;
  for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < total; i += stride) {
    const int64_t c = per_channel ? (i / inner) % channels : 0;
    if constexpr (WRAP) y[i] = simquant_wrap_of(rintf(x[i] / scale[c]), scale[c], (float)zp[c], lo, hi, wrap_bits, wrap_signed);
    else y[i] = simquant_one(x[i], scale[c], (float)zp[c], lo, hi);
  }
}

// AWAY: the launch's tie rule is halves away from zero (the general form); else the plain one.
template <bool AWAY>
__device__ __forceinline__ int32_t requant_pick(int32_t acc, int32_t mult, int32_t sh, const RequantScalars& rs) {
  if constexpr (AWAY) return requant_half_away(acc, mult, sh, rs);
  else return requant_one(acc, mult, sh, rs);
}

template <typename AccT>
__device__ __forceinline__ int32_t load_acc(const AccT* p, int64_t i) {
  return (int32_t)p[i];
}

// rows: 4 accumulators -> 4 output bytes per step, 128-bit loads for int32; U steps per lane
// and job with all loads issued first, nontemporal as above.
// POW2: no multiplier array (power-of-two scales): the rounding shift alone, no multiplication.
template <typename AccT, int U, bool AWAY, bool POW2 = false>
__global__ __launch_bounds__(kThreads) void requant_rows_kernel(
    const AccT* __restrict__ acc, uint32_t* __restrict__ out, int64_t rows, int32_t channels,
    int64_t inner_vec, int32_t nseg, int32_t seg_len, const int32_t* __restrict__ mult,
    const int32_t* __restrict__ shift, int per_channel, JobDiv jd, RequantScalars rs) {
  using VecT = typename std::conditional<sizeof(AccT) == 4, v4i32, v4i16>::type;
  for (int64_t job = blockIdx.x; job < rows * nseg; job += gridDim.x) {
    int64_t row;
    int32_t c;
    job_row_channel(job, nseg, channels, per_channel, jd, row, c);
    const int32_t seg = (int32_t)(job - row * nseg);
    const int32_t m = POW2 ? 0 : rq_mult(mult, c);
    const int32_t sh = POW2 ? shift[c] : rq_shift(mult, shift, c);
    auto one = [&](int32_t a) {
      if constexpr (POW2) return med3(shift_round(a, sh), rs.lo_rel, rs.hi_rel) + rs.z_out;
      else return requant_pick<AWAY>(a, m, sh, rs);
    };
    const int64_t v0 = (int64_t)seg * seg_len;
    const int64_t v1 = (v0 + seg_len < inner_vec) ? v0 + seg_len : inner_vec;
    const VecT* ar = reinterpret_cast<const VecT*>(acc) + row * inner_vec;
    uint32_t* orow = out + row * inner_vec;
    for (int64_t vb = v0 + threadIdx.x; vb < v1; vb += (int64_t)kThreads * U) {
      VecT q[U];
#pragma unroll
      for (int u = 0; u < U; ++u)
        if (vb + u * kThreads < v1) q[u] = __builtin_nontemporal_load(ar + vb + u * kThreads);
#pragma unroll
      for (int u = 0; u < U; ++u) {
        if (vb + u * kThreads < v1) {
          const uint32_t r = pack4(one((int32_t)q[u].x), one((int32_t)q[u].y), one((int32_t)q[u].z), one((int32_t)q[u].w));
          __builtin_nontemporal_store(r, orow + vb + u * kThreads);
        }
      }
    }
  }
}

// channel-last (inner == 1) with channels % 4 == 0: 4 consecutive channels.
template <typename AccT, bool AWAY>
__global__ __launch_bounds__(kThreads) void requant_lastaxis_kernel(
    const AccT* __restrict__ acc, uint32_t* __restrict__ out, int64_t total_vec,
    int32_t channels_vec, const int4* __restrict__ mult, const int4* __restrict__ shift,
    RequantScalars rs) {
  const int64_t stride = (int64_t)gridDim.x * kThreads;
  for (int64_t v = (int64_t)blockIdx.x * kThreads + threadIdx.x; v < total_vec; v += stride) {
    const int32_t cv = (int32_t)(v % channels_vec);
    const int4 m = mult[cv];
    const int4 sh = shift[cv];
    int32_t a0, a1, a2, a3;
    if constexpr (sizeof(AccT) == 4) {
      const int4 q = reinterpret_cast<const int4*>(acc)[v];
      a0 = q.x; a1 = q.y; a2 = q.z; a3 = q.w;
    } else {
      const short4 q = reinterpret_cast<const short4*>(acc)[v];
      a0 = q.x; a1 = q.y; a2 = q.z; a3 = q.w;
    }
    out[v] = pack4(requant_pick<AWAY>(a0, m.x, sh.x, rs), requant_pick<AWAY>(a1, m.y, sh.y, rs),
                   requant_pick<AWAY>(a2, m.z, sh.z, rs), requant_pick<AWAY>(a3, m.w, sh.w, rs));
  }
}

template <typename AccT, bool AWAY>
__global__ __launch_bounds__(kThreads) void requant_flat_kernel(
    const AccT* __restrict__ acc, uint8_t* __restrict__ out, int64_t total, int64_t inner,
    int64_t channels, const int32_t* __restrict__ mult, const int32_t* __restrict__ shift,
    int per_channel, RequantScalars rs) {
  const int64_t stride = (int64_t)gridDim.x * kThreads;
  for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < total; i += stride) {
    const int64_t c = per_channel ? (i / inner) % channels : 0;
    out[i] = (uint8_t)requant_pick<AWAY>(load_acc(acc, i), rq_mult(mult, c), rq_shift(mult, shift, c), rs);
  }
}

// ---- quantize / dequantize (the two halves of Eq. 3; Sec. 6.1): the code is formed exactly as in
// simulated_quantize (binary32 division, round half to even, zero point added as a float,
// compare-select clip), then stored in the integer container; NaN takes the code of real zero.
__device__ __forceinline__ int32_t quantize_of(float u, float zf, float lo, float hi) {
  const float v = (u != u) ? zf : u + zf;                  // never NaN from here on
  return (int32_t)__builtin_amdgcn_fmed3f(v, lo, hi);      // the clip; integral and within +-2^24
}

__device__ __forceinline__ int32_t quantize_of_finite(float u, float zf, float lo, float hi) {
  return (int32_t)__builtin_amdgcn_fmed3f(u + zf, lo, hi);
}

__device__ __forceinline__ int32_t quantize_one(float x, float s, float zf, float lo, float hi) {
  return quantize_of(rintf(x / s), zf, lo, hi);
}

__device__ __forceinline__ float dequantize_one(int32_t q, float s, float zf) {
  return ((float)q - zf) * s;
}

template <typename Q> struct QVec;  // four codes of a container as one store / load
template <> struct QVec<int8_t> { typedef uint32_t T; };
template <> struct QVec<uint8_t> { typedef uint32_t T; };
template <> struct QVec<int16_t> { typedef v4i16 T; };
template <> struct QVec<int32_t> { typedef v4i32 T; };

template <typename Q>
__device__ __forceinline__ typename QVec<Q>::T pack_codes(int32_t a, int32_t b, int32_t c, int32_t d) {
  if constexpr (sizeof(Q) == 1) return pack4(a, b, c, d);
  else if constexpr (sizeof(Q) == 2) return v4i16{(int16_t)a, (int16_t)b, (int16_t)c, (int16_t)d};
  else return v4i32{a, b, c, d};
}

template <typename Q>
__device__ __forceinline__ void unpack_codes(typename QVec<Q>::T v, int32_t (&q)[4]) {
  if constexpr (sizeof(Q) == 1) {
#pragma unroll
    for (int e = 0; e < 4; ++e) q[e] = (int32_t)(Q)((v >> (8 * e)) & 0xffu);
  } else {
    q[0] = (int32_t)v.x; q[1] = (int32_t)v.y; q[2] = (int32_t)v.z; q[3] = (int32_t)v.w;
  }
}

// Row kernels as for simulated_quantize.  OP 0: fp32 -> codes; 1: codes -> fp32; 2: fp32 -> codes
// (out) and the simulated_quantize value (out2) in one pass over x.
template <typename Q, int OP, int U>
__global__ __launch_bounds__(kThreads) void quant_rows_kernel(
    const void* __restrict__ in, void* __restrict__ out, float* __restrict__ out2, int64_t rows, int32_t channels,
    int64_t inner_vec, int32_t nseg, int32_t seg_len, const float* __restrict__ scale,
    const int32_t* __restrict__ zp, int per_channel, JobDiv jd, float lo, float hi) {
  using VQ = typename QVec<Q>::T;
  for (int64_t job = blockIdx.x; job < rows * nseg; job += gridDim.x) {
    int64_t row;
    int32_t c;
    job_row_channel(job, nseg, channels, per_channel, jd, row, c);
    const int32_t seg = (int32_t)(job - row * nseg);
    const float s = scale[c];
    const float zf = (float)zp[c];
    const float rc = OP == 1 ? 0.0f : quotient_reciprocal(s);
    const int64_t v0 = (int64_t)seg * seg_len;
    const int64_t v1 = (v0 + seg_len < inner_vec) ? v0 + seg_len : inner_vec;
    for (int64_t vb = v0 + threadIdx.x; vb < v1; vb += (int64_t)kThreads * U) {
      if constexpr (OP == 1) {
        const VQ* qr = static_cast<const VQ*>(in) + row * inner_vec;
        v4f* yr = static_cast<v4f*>(out) + row * inner_vec;
        VQ a[U];
#pragma unroll
        for (int u = 0; u < U; ++u)
          if (vb + u * kThreads < v1) a[u] = __builtin_nontemporal_load(qr + vb + u * kThreads);
#pragma unroll
        for (int u = 0; u < U; ++u) {
          if (vb + u * kThreads < v1) {
            int32_t q[4];
            unpack_codes<Q>(a[u], q);
            const v4f r = {dequantize_one(q[0], s, zf), dequantize_one(q[1], s, zf),
                           dequantize_one(q[2], s, zf), dequantize_one(q[3], s, zf)};
            __builtin_nontemporal_store(r, yr + vb + u * kThreads);
          }
        }
      } else {
        const v4f* xr = static_cast<const v4f*>(in) + row * inner_vec;
        VQ* qr = static_cast<VQ*>(out) + row * inner_vec;
        v4f a[U];
#pragma unroll
        for (int u = 0; u < U; ++u)
          if (vb + u * kThreads < v1) a[u] = __builtin_nontemporal_load(xr + vb + u * kThreads);
#pragma unroll
        for (int u = 0; u < U; ++u) {
          if (vb + u * kThreads < v1) {
            v4f n, y;
            VQ r;
            if (__builtin_expect(fast_quotient4(a[u], rc, n), 1)) {   // four finite quotients
              r = pack_codes<Q>(quantize_of_finite(n.x, zf, lo, hi), quantize_of_finite(n.y, zf, lo, hi),
                                quantize_of_finite(n.z, zf, lo, hi), quantize_of_finite(n.w, zf, lo, hi));
              if constexpr (OP == 2)
                y = v4f{simquant_of_finite(n.x, s, zf, lo, hi), simquant_of_finite(n.y, s, zf, lo, hi),
                        simquant_of_finite(n.z, s, zf, lo, hi), simquant_of_finite(n.w, s, zf, lo, hi)};
            } else {
              r = pack_codes<Q>(quantize_one(a[u].x, s, zf, lo, hi), quantize_one(a[u].y, s, zf, lo, hi),
                                quantize_one(a[u].z, s, zf, lo, hi), quantize_one(a[u].w, s, zf, lo, hi));
              if constexpr (OP == 2)
                y = v4f{simquant_one(a[u].x, s, zf, lo, hi), simquant_one(a[u].y, s, zf, lo, hi),
                        simquant_one(a[u].z, s, zf, lo, hi), simquant_one(a[u].w, s, zf, lo, hi)};
            }
            __builtin_nontemporal_store(r, qr + vb + u * kThreads);
            if constexpr (OP == 2) {
              __builtin_nontemporal_store(y, reinterpret_cast<v4f*>(out2) + row * inner_vec + vb + u * kThreads);
            }
          }
        }
      }
    }
  }
}

template <typename Q, int OP>
__global__ __launch_bounds__(kThreads) void quant_flat_kernel(
    const void* __restrict__ in, void* __restrict__ out, float* __restrict__ out2, int64_t total, int64_t inner,
    int64_t channels, const float* __restrict__ scale, const int32_t* __restrict__ zp,
    int per_channel, float lo, float hi) {
  const int64_t stride = (int64_t)gridDim.x * kThreads;
  for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < total; i += stride) {
    const int64_t c = per_channel ? (i / inner) % channels : 0;
    if constexpr (OP == 1) {
      static_cast<float*>(out)[i] = dequantize_one((int32_t)static_cast<const Q*>(in)[i], scale[c], (float)zp[c]);
    } else {
      const float x = static_cast<const float*>(in)[i];
      static_cast<Q*>(out)[i] = (Q)quantize_one(x, scale[c], (float)zp[c], lo, hi);
      if constexpr (OP == 2) out2[i] = simquant_one(x, scale[c], (float)zp[c], lo, hi);
    }
  }
}

// ---- max-abs calibration (Eq. 2): thr[c] = max |x[o, c, i]| over o, i.  NaN never wins a
// comparison and is therefore ignored; the result is never negative zero.  |x| of a non-NaN
// float orders like its bit pattern as an unsigned integer, so partial results are merged with
// one integer atomic max per workgroup (order-independent: the result is exact).
__device__ __forceinline__ float absmax_step(float m, float v) {
  const float a = fabsf(v);
  return a > m ? a : m;
}

__device__ __forceinline__ float wave_max(float m) {
#pragma unroll
  for (int d = 32; d >= 1; d >>= 1) {
    const float o = __shfl_xor(m, d);
    m = o > m ? o : m;
  }
  return m;
}

// thr must hold zeros on entry.
__device__ __forceinline__ void block_merge_max(float m, uint32_t* thr_c) {
  __shared__ float s_m[kThreads / 64];
  m = wave_max(m);
  if ((threadIdx.x & 63) == 0) s_m[threadIdx.x >> 6] = m;
  __syncthreads();
  if (threadIdx.x == 0) {
#pragma unroll
    for (int w = 1; w < kThreads / 64; ++w) m = s_m[w] > m ? s_m[w] : m;
    if (m > 0.0f) atomicMax(thr_c, __float_as_uint(m));
  }
  __syncthreads();
}

__global__ __launch_bounds__(kThreads) void fill_zero_kernel(uint32_t* p, int64_t n) {
  const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
  if (i < n) p[i] = 0u;
}

// rows: as the other row kernels (row = outer * channels index, 128-bit nontemporal loads, U
// vectors per lane in flight).  A job is (channel, row segment, group of outer indices): the
// workgroup walks the rows o = og, og + ogroups, ... of its channel and merges once, so the
// barriers and the atomic are paid once per several rows.
template <int U>
__global__ __launch_bounds__(kThreads) void absmax_rows_kernel(
    const v4f* __restrict__ x, int64_t outer, int32_t channels, int64_t inner_vec, int32_t nseg,
    int32_t seg_len, int32_t ogroups, int per_channel, uint32_t* __restrict__ thr) {
  // per tensor the "row" is the whole tensor: outer == 1, channels == 1
  const int64_t jobs = (int64_t)channels * nseg * ogroups;
  for (int64_t job = blockIdx.x; job < jobs; job += gridDim.x) {
    // job = og * (channels * nseg) + c * nseg + seg: neighbouring workgroups, neighbouring rows
    int32_t og, seg, c;
    const int64_t per_group = (int64_t)channels * nseg;
    if (jobs <= 0xffffffffll) {  // the usual case: 32-bit divisions
      og = (int32_t)((uint32_t)job / (uint32_t)per_group);
      const uint32_t cs = (uint32_t)job - (uint32_t)og * (uint32_t)per_group;
      c = (int32_t)(cs / (uint32_t)nseg);
      seg = (int32_t)(cs - (uint32_t)c * (uint32_t)nseg);
    } else {
      og = (int32_t)(job / per_group);
      const int64_t cs = job - og * per_group;
      c = (int32_t)(cs / nseg);
      seg = (int32_t)(cs - (int64_t)c * nseg);
    }
    const int64_t v0 = (int64_t)seg * seg_len;
    const int64_t v1 = (v0 + seg_len < inner_vec) ? v0 + seg_len : inner_vec;
    float m = 0.0f;
    for (int64_t o = og; o < outer; o += ogroups) {
      const v4f* xr = x + (o * channels + c) * inner_vec;
      for (int64_t vb = v0 + threadIdx.x; vb < v1; vb += (int64_t)kThreads * U) {
        v4f a[U];
#pragma unroll
        for (int u = 0; u < U; ++u)
          a[u] = vb + u * kThreads < v1 ? __builtin_nontemporal_load(xr + vb + u * kThreads)
                                        : v4f{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int u = 0; u < U; ++u) {
          m = absmax_step(m, a[u].x); m = absmax_step(m, a[u].y);
          m = absmax_step(m, a[u].z); m = absmax_step(m, a[u].w);
        }
      }
    }
    block_merge_max(m, thr + (per_channel ? c : 0));
  }
}

// columns: the tensor as [outer][channels * inner]; a lane owns one column j (channel j / inner)
// and walks a chunk of `orows` outer rows, so neighbouring lanes read neighbouring addresses.
// Used for short, unaligned or channel-last rows.  One atomic per lane and chunk.
__global__ __launch_bounds__(kThreads) void absmax_cols_kernel(
    const float* __restrict__ x, int64_t outer, int64_t cols, int64_t inner, int64_t orows,
    int per_channel, uint32_t* __restrict__ thr) {
  const int64_t j = (int64_t)blockIdx.x * kThreads + threadIdx.x;
  if (j >= cols) return;
  const int64_t o0 = (int64_t)blockIdx.y * orows;
  const int64_t o1 = (o0 + orows < outer) ? o0 + orows : outer;
  float m = 0.0f;
  for (int64_t o = o0; o < o1; ++o) m = absmax_step(m, x[o * cols + j]);
  if (m > 0.0f) atomicMax(thr + (per_channel ? j / inner : 0), __float_as_uint(m));
}

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

inline int grid_for(int64_t jobs) {
  const int64_t cap = 1ll << 30;  // one job per workgroup; the kernels loop beyond this
  return (int)(jobs < cap ? (jobs > 0 ? jobs : 1) : cap);
}

}  // namespace

hipError_t launch_simquant(const float* x, float* y, int64_t outer, int64_t channels, int64_t inner,
                           const float* scale, const int32_t* zp, int per_channel, int32_t clip_lo,
                           int32_t clip_hi, hipStream_t st) {
  const int64_t total = outer * channels * inner;
  if (total == 0) return hipSuccess;
  const float lo = (float)clip_lo, hi = (float)clip_hi;
  // Per-tensor parameters: the whole tensor is one row.
  int64_t rows = per_channel ? outer * channels : 1;
  int64_t row_len = per_channel ? inner : total;
  if (row_len % 4 == 0 && row_len >= 512 && aligned16(x) && aligned16(y)) {
    const int64_t inner_vec = row_len / 4;
    int32_t nseg, seg_len;
    split_row(inner_vec, kVecPerLane, &nseg, &seg_len);
    hipLaunchKernelGGL((simquant_rows_kernel<kVecPerLane, false>), dim3(grid_for(rows * nseg)), dim3(kThreads), 0, st,
                       reinterpret_cast<const v4f*>(x), reinterpret_cast<v4f*>(y), rows,
                       (int32_t)(per_channel ? channels : 1), inner_vec, nseg, seg_len, scale, zp,
                       per_channel, JobDiv{reciprocal32(nseg), reciprocal32(per_channel ? channels : 1)}, lo, hi, 0, 0);
  } else {
    hipLaunchKernelGGL(simquant_flat_kernel<false>, dim3(grid_for((total + kThreads - 1) / kThreads)),
                       dim3(kThreads), 0, st, x, y, total, inner, channels, scale, zp, per_channel,
                       lo, hi, 0, 0);
  }
  return hipGetLastError();
}

hipError_t launch_simquant_wrap(const float* x, float* y, int64_t outer, int64_t channels, int64_t inner,
                                const float* scale, const int32_t* zp, int per_channel, int32_t wrap_bits,
                                int32_t wrap_signed, int32_t clip_lo, int32_t clip_hi, hipStream_t st) {
  const int64_t total = outer * channels * inner;
  if (total == 0) return hipSuccess;
  const float lo = (float)clip_lo, hi = (float)clip_hi;
  int64_t rows = per_channel ? outer * channels : 1;
  int64_t row_len = per_channel ? inner : total;
  if (row_len % 4 == 0 && row_len >= 512 && aligned16(x) && aligned16(y)) {
    const int64_t inner_vec = row_len / 4;
    int32_t nseg, seg_len;
    split_row(inner_vec, kVecPerLane, &nseg, &seg_len);
    hipLaunchKernelGGL((simquant_rows_kernel<kVecPerLane, true>), dim3(grid_for(rows * nseg)), dim3(kThreads), 0, st,
                       reinterpret_cast<const v4f*>(x), reinterpret_cast<v4f*>(y), rows,
                       (int32_t)(per_channel ? channels : 1), inner_vec, nseg, seg_len, scale, zp,
                       per_channel, JobDiv{reciprocal32(nseg), reciprocal32(per_channel ? channels : 1)}, lo, hi,
                       wrap_bits, wrap_signed);
  } else {
    hipLaunchKernelGGL(simquant_flat_kernel<true>, dim3(grid_for((total + kThreads - 1) / kThreads)),
                       dim3(kThreads), 0, st, x, y, total, inner, channels, scale, zp, per_channel,
                       lo, hi, wrap_bits, wrap_signed);
  }
  return hipGetLastError();
}

hipError_t launch_simquant_batched(const float* x, float* y, int64_t outer, int64_t channels,
                                   int64_t inner, int32_t nbatch, const float* scale,
                                   const int32_t* zp, int per_channel, const int32_t* clip_lo,
                                   const int32_t* clip_hi, hipStream_t st) {
  const int64_t total = outer * channels * inner;
  if (total == 0 || nbatch == 0) return hipSuccess;
  if (nbatch > kMaxCandidates) return hipErrorInvalidValue;
  CandidateClips clips{};
  for (int b = 0; b < nbatch; ++b) {
    clips.lo[b] = (float)clip_lo[b];
    clips.hi[b] = (float)clip_hi[b];
  }
  const int32_t nparam = (int32_t)(per_channel ? channels : 1);
  const int64_t rows = per_channel ? outer * channels : 1;
  const int64_t row_len = per_channel ? inner : total;
  if (row_len % 4 == 0 && row_len >= 512 && aligned16(x) && aligned16(y)) {
    const int64_t inner_vec = row_len / 4;
    constexpr int kU = 2;  // fewer vectors in flight per lane: every one is stored nbatch times
    int32_t nseg, seg_len;
    split_row(inner_vec, kU, &nseg, &seg_len);
    hipLaunchKernelGGL(simquant_batched_rows_kernel<kU>, dim3(grid_for(rows * nseg)), dim3(kThreads),
                       0, st, reinterpret_cast<const v4f*>(x), reinterpret_cast<v4f*>(y), rows,
                       nparam, inner_vec, nseg, seg_len, nbatch, nparam, scale, zp, per_channel,
                       JobDiv{reciprocal32(nseg), reciprocal32(nparam)}, clips);
  } else {
    hipLaunchKernelGGL(simquant_batched_flat_kernel, dim3(grid_for((total + kThreads - 1) / kThreads)),
                       dim3(kThreads), 0, st, x, y, total, inner, channels, nbatch, nparam, scale, zp,
                       per_channel, clips);
  }
  return hipGetLastError();
}

template <typename Q, int OP>
static hipError_t launch_quant_t(const void* in, void* out, float* out2, int64_t outer, int64_t channels,
                                 int64_t inner, const float* scale, const int32_t* zp,
                                 int per_channel, int32_t clip_lo, int32_t clip_hi, hipStream_t st) {
  const int64_t total = outer * channels * inner;
  if (total == 0) return hipSuccess;
  const float lo = (float)clip_lo, hi = (float)clip_hi;
  const int64_t rows = per_channel ? outer * channels : 1;
  const int64_t row_len = per_channel ? inner : total;
  if (row_len % 4 == 0 && row_len >= 512 && aligned16(in) && aligned16(out) && aligned16(out2)) {
    const int64_t inner_vec = row_len / 4;
    int32_t nseg, seg_len;
    split_row(inner_vec, kVecPerLane, &nseg, &seg_len);
    hipLaunchKernelGGL((quant_rows_kernel<Q, OP, kVecPerLane>), dim3(grid_for(rows * nseg)),
                       dim3(kThreads), 0, st, in, out, out2, rows, (int32_t)(per_channel ? channels : 1),
                       inner_vec, nseg, seg_len, scale, zp, per_channel,
                       JobDiv{reciprocal32(nseg), reciprocal32(per_channel ? channels : 1)}, lo, hi);
  } else {
    hipLaunchKernelGGL((quant_flat_kernel<Q, OP>), dim3(grid_for((total + kThreads - 1) / kThreads)),
                       dim3(kThreads), 0, st, in, out, out2, total, inner, channels, scale, zp, per_channel,
                       lo, hi);
  }
  return hipGetLastError();
}

// container: 0 int8, 1 uint8, 2 int16, 3 int32.  op 0: fp32 -> codes; 1: codes -> fp32;
// 2: fp32 -> codes and the simulated_quantize value (out2).
hipError_t launch_quant(const void* in, void* out, float* out2, int container, int op, int64_t outer,
                        int64_t channels, int64_t inner, const float* scale, const int32_t* zp,
                        int per_channel, int32_t clip_lo, int32_t clip_hi, hipStream_t st) {
#define HAGO_QUANT_CASE(ID, T)                                                                       \
  case ID:                                                                                           \
    return op == 1 ? launch_quant_t<T, 1>(in, out, nullptr, outer, channels, inner, scale, zp,       \
                                          per_channel, clip_lo, clip_hi, st)                         \
         : op == 2 ? launch_quant_t<T, 2>(in, out, out2, outer, channels, inner, scale, zp,          \
                                          per_channel, clip_lo, clip_hi, st)                         \
                   : launch_quant_t<T, 0>(in, out, nullptr, outer, channels, inner, scale, zp,       \
                                          per_channel, clip_lo, clip_hi, st);
  switch (container) {
    HAGO_QUANT_CASE(0, int8_t)
    HAGO_QUANT_CASE(1, uint8_t)
    HAGO_QUANT_CASE(2, int16_t)
    HAGO_QUANT_CASE(3, int32_t)
    default: return hipErrorInvalidValue;
  }
#undef HAGO_QUANT_CASE
}

hipError_t launch_absmax(const float* x, int64_t outer, int64_t channels, int64_t inner,
                         int per_channel, float* thr, hipStream_t st) {
  const int64_t nthr = per_channel ? channels : 1;
  if (nthr == 0) return hipSuccess;
  uint32_t* t = reinterpret_cast<uint32_t*>(thr);
  // (a fill kernel, not hipMemsetAsync: the call may be captured into a graph)
  hipLaunchKernelGGL(fill_zero_kernel, dim3((unsigned)((nthr + kThreads - 1) / kThreads)),
                     dim3(kThreads), 0, st, t, nthr);
  const int64_t total = outer * channels * inner;
  if (total == 0) return hipGetLastError();
  const int64_t row_len = per_channel ? inner : total;
  if (row_len % 4 == 0 && row_len >= 512 && aligned16(x)) {
    const int64_t inner_vec = row_len / 4;
    int32_t nseg, seg_len;
    split_row(inner_vec, kVecPerLane, &nseg, &seg_len);
    // about four workgroups per CU: rows of one channel beyond that share a workgroup (config 4
    // tensor: 12.8 us with 8 rows per workgroup, 15.8 us with one)
    const int64_t nchan = per_channel ? channels : 1, nouter = per_channel ? outer : 1;
    int64_t rows_per_wg = nouter * nchan * nseg / (256 * 4);
    if (rows_per_wg < 1) rows_per_wg = 1;
    const int64_t ogroups = (nouter + rows_per_wg - 1) / rows_per_wg;
    const int64_t jobs = nchan * nseg * ogroups;
    const int64_t cap = 256 * 32;
    hipLaunchKernelGGL(absmax_rows_kernel<kVecPerLane>, dim3((unsigned)(jobs < cap ? jobs : cap)),
                       dim3(kThreads), 0, st, reinterpret_cast<const v4f*>(x), nouter, (int32_t)nchan,
                       inner_vec, nseg, seg_len, (int32_t)ogroups, per_channel, t);
  } else {
    const int64_t cols = per_channel ? channels * inner : inner * channels;
    const int64_t col_inner = per_channel ? inner : cols;
    const int64_t xblocks = (cols + kThreads - 1) / kThreads;
    if (xblocks >= (1ll << 31)) return hipErrorInvalidValue;
    // enough row chunks to fill the chip, at most 65535
    int64_t chunks = (256 * 8 + xblocks - 1) / xblocks;
    if (chunks > outer) chunks = outer;
    if (chunks > 65535) chunks = 65535;
    if (chunks < 1) chunks = 1;
    const int64_t orows = (outer + chunks - 1) / chunks;
    chunks = (outer + orows - 1) / orows;
    hipLaunchKernelGGL(absmax_cols_kernel, dim3((unsigned)xblocks, (unsigned)chunks), dim3(kThreads),
                       0, st, x, outer, cols, col_inner, orows, per_channel, t);
  }
  return hipGetLastError();
}

template <typename AccT>
static hipError_t launch_requantize_t(const AccT* acc, int64_t outer, int64_t channels,
                                      int64_t inner, const RequantArgs& rq, void* out,
                                      hipStream_t st) {
  const int64_t total = outer * channels * inner;
  if (total == 0) return hipSuccess;
  const RequantScalars rs{rq.z_out, rq.clip_lo - rq.z_out, rq.clip_hi - rq.z_out, rq.half_away};
  const int pc = rq.per_channel;
  int64_t rows = pc ? outer * channels : 1;
  int64_t row_len = pc ? inner : total;
  const bool io_aligned = aligned16(acc) && aligned16(out);
  if (row_len % 4 == 0 && row_len >= 512 && io_aligned) {
    const int64_t inner_vec = row_len / 4;
    int32_t nseg, seg_len;
    split_row(inner_vec, kVecPerLane, &nseg, &seg_len);
    auto kern = rq.half_away ? requant_rows_kernel<AccT, kVecPerLane, true>
                : (rq.multiplier ? requant_rows_kernel<AccT, kVecPerLane, false>
                                 : requant_rows_kernel<AccT, kVecPerLane, false, true>);
    hipLaunchKernelGGL(kern, dim3(grid_for(rows * nseg)), dim3(kThreads), 0, st,
                       acc, reinterpret_cast<uint32_t*>(out), rows, (int32_t)(pc ? channels : 1),
                       inner_vec, nseg, seg_len, rq.multiplier, rq.shift, pc,
                       JobDiv{reciprocal32(nseg), reciprocal32(pc ? channels : 1)}, rs);
  } else if (pc && inner == 1 && channels % 4 == 0 && io_aligned && rq.multiplier && aligned16(rq.multiplier) &&
             aligned16(rq.shift)) {
    const int64_t total_vec = total / 4;
    auto kern = rq.half_away ? requant_lastaxis_kernel<AccT, true> : requant_lastaxis_kernel<AccT, false>;
    hipLaunchKernelGGL(kern,
                       dim3(grid_for((total_vec + kThreads - 1) / kThreads)), dim3(kThreads), 0, st,
                       acc, reinterpret_cast<uint32_t*>(out), total_vec, (int32_t)(channels / 4),
                       reinterpret_cast<const int4*>(rq.multiplier),
                       reinterpret_cast<const int4*>(rq.shift), rs);
  } else {
    auto kern = rq.half_away ? requant_flat_kernel<AccT, true> : requant_flat_kernel<AccT, false>;
    hipLaunchKernelGGL(kern, dim3(grid_for((total + kThreads - 1) / kThreads)),
                       dim3(kThreads), 0, st, acc, reinterpret_cast<uint8_t*>(out), total, inner,
                       channels, rq.multiplier, rq.shift, pc, rs);
  }
  return hipGetLastError();
}

hipError_t launch_requantize(const void* acc, int acc16, int64_t outer, int64_t channels,
                             int64_t inner, const RequantArgs& rq, void* out, hipStream_t st) {
  if (acc16)
    return launch_requantize_t(static_cast<const int16_t*>(acc), outer, channels, inner, rq, out, st);
  return launch_requantize_t(static_cast<const int32_t*>(acc), outer, channels, inner, rq, out, st);
}

}  // namespace hago
