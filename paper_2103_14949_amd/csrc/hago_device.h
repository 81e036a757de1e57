// Device-side helpers shared by the libhago kernels (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace hago {

// Requantize epilogue parameters that are uniform over a launch.  The clip
// limits are stored relative to the output zero point:
//   clip(r + z, lo, hi) == clip(r, lo - z, hi - z) + z
// so the sum r + z is only formed once r is already small.
struct RequantScalars {
  int32_t z_out;
  int32_t lo_rel;  // clip_lo - z_out
  int32_t hi_rel;  // clip_hi - z_out
  int32_t half_away;  // tie rule: 0 toward +infinity, 1 away from zero (general code paths only)
};

// r = floor(acc * mult / 2^(31 + sh) + 1/2), exact in 64-bit integers
// (|acc * mult| < 2^62, rounding term <= 2^61).  The result always fits in
// int32 for mult < 2^31.
__device__ __forceinline__ int32_t rounding_mul_shift(int32_t acc, int32_t mult, int32_t sh) {
  const int64_t p = (int64_t)acc * (int64_t)mult + ((int64_t)1 << (30 + sh));
  return (int32_t)(p >> (31 + sh));
}

// Power-of-two scales (Sec. 5.1 of the paper: shifting replaces the multiplication): the
// multiplier array is absent and the requantize is round(acc / 2^s).  That is the general form
// with multiplier 2^30 (one half) and shift s - 1; the 64-bit forms below accept the resulting
// shift of -1 for s == 0 (rounding term 2^29, shift distance 30), the folded fast paths of the
// kernels exclude it like they exclude shift 0.
__device__ __forceinline__ int32_t rq_mult(const int32_t* mult, int64_t i) {
  return mult ? mult[i] : (1 << 30);
}
__device__ __forceinline__ int32_t rq_shift(const int32_t* mult, const int32_t* shift, int64_t i) {
  return shift[i] - (mult ? 0 : 1);
}
// The shift-only form itself, without a multiplication: floor(acc / 2^s + 1/2) is the floored
// quotient plus the first bit shifted out (no rounding term is added, so nothing can wrap).
__device__ __forceinline__ int32_t shift_round(int32_t acc, int32_t s) {
  return s > 0 ? (acc >> s) + ((acc >> (s - 1)) & 1) : acc;
}

// Accumulators narrower than 32 bits (int16 accumulation; 24-bit accumulators): the 32-bit sum
// reduced modulo 2^bits and sign-extended, which equals accumulating in that width all along
// (the reduction is a ring homomorphism).  wrap_shift = 32 - bits, 0 for a full int32.
__device__ __forceinline__ int32_t wrap_acc_bits(int32_t acc, int32_t wrap_shift) {
  return (int32_t)((uint32_t)acc << wrap_shift) >> wrap_shift;
}

// median of three = clamp when lo <= hi; one instruction instead of two compare/select pairs
__device__ __forceinline__ int32_t med3(int32_t x, int32_t lo, int32_t hi) {
  int32_t r;
  asm("v_med3_i32 %0, %1, %2, %3" : "=v"(r) : "v"(x), "v"(lo), "v"(hi));
  return r;
}

__device__ __forceinline__ int32_t requant_one(int32_t acc, int32_t mult, int32_t sh,
                                               const RequantScalars& rs) {
  const int32_t r = rounding_mul_shift(acc, mult, sh);
  return med3(r, rs.lo_rel, rs.hi_rel) + rs.z_out;
}

// Nearest with halves away from zero: round the magnitude half up and give the sign back,
// which for a negative product is floor((product + rounding term - 1) / 2^(31 + sh)).  The
// product has the sign of acc (mult >= 0; a zero product rounds to 0 either way), so the
// correction is acc's sign bit added to the 64-bit sum.  It differs from ties toward +infinity
// exactly on negative ties, and there by one.
__device__ __forceinline__ int32_t requant_half_away(int32_t acc, int32_t mult, int32_t sh,
                                                     const RequantScalars& rs) {
  const int64_t p = (int64_t)acc * (int64_t)mult + ((int64_t)1 << (30 + sh)) + (int64_t)(acc >> 31);
  return med3((int32_t)(p >> (31 + sh)), rs.lo_rel, rs.hi_rel) + rs.z_out;
}

// The general form, with the launch's tie rule.
__device__ __forceinline__ int32_t requant_general(int32_t acc, int32_t mult, int32_t sh,
                                                   const RequantScalars& rs) {
  return rs.half_away ? requant_half_away(acc, mult, sh, rs) : requant_one(acc, mult, sh, rs);
}

// Byte B of dst <- low byte of (src >> sh) (arithmetic); B == 0 clears the other bytes, the
// later ones keep them: four of these in a row shift and pack four results with no separate
// pack instructions (the destination-byte select of the sub-dword addressing forms).
template <int B>
__device__ __forceinline__ void ashr_into_byte(uint32_t& dst, int32_t src, int32_t sh) {
  static_assert(B >= 0 && B < 4, "byte index");
  if constexpr (B == 0)
    asm("v_ashrrev_i32_sdwa %0, %1, %2 dst_sel:BYTE_0 dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:DWORD"
        : "=v"(dst) : "v"(sh), "v"(src));
  else if constexpr (B == 1)
    asm("v_ashrrev_i32_sdwa %0, %1, %2 dst_sel:BYTE_1 dst_unused:UNUSED_PRESERVE src0_sel:DWORD src1_sel:DWORD"
        : "+v"(dst) : "v"(sh), "v"(src));
  else if constexpr (B == 2)
    asm("v_ashrrev_i32_sdwa %0, %1, %2 dst_sel:BYTE_2 dst_unused:UNUSED_PRESERVE src0_sel:DWORD src1_sel:DWORD"
        : "+v"(dst) : "v"(sh), "v"(src));
  else
    asm("v_ashrrev_i32_sdwa %0, %1, %2 dst_sel:BYTE_3 dst_unused:UNUSED_PRESERVE src0_sel:DWORD src1_sel:DWORD"
        : "+v"(dst) : "v"(sh), "v"(src));
}

// Clip limits moved in front of a right shift by s: clip(y >> s, lo, hi) == clip(y, lo * 2^s,
// (hi + 1) * 2^s - 1) >> s for the flooring shift; a limit that leaves int32 saturates there
// (no y lies beyond it, so it is inactive, as it should be).
__device__ __forceinline__ int32_t clip_lo_before_shift(int32_t lo, int32_t s) {
  const int64_t v = (int64_t)lo * ((int64_t)1 << s);
  return v < INT32_MIN ? INT32_MIN : (v > INT32_MAX ? INT32_MAX : (int32_t)v);
}
__device__ __forceinline__ int32_t clip_hi_before_shift(int32_t hi, int32_t s) {
  const int64_t v = ((int64_t)hi + 1) * ((int64_t)1 << s) - 1;
  return v > INT32_MAX ? INT32_MAX : (v < INT32_MIN ? INT32_MIN : (int32_t)v);
}

// Four results -> one little-endian dword of their low bytes.
__device__ __forceinline__ uint32_t pack4_perm(int32_t b0, int32_t b1, int32_t b2, int32_t b3) {
  const uint32_t lo = __builtin_amdgcn_perm((uint32_t)b1, (uint32_t)b0, 0x0c0c0400u);
  const uint32_t hi = __builtin_amdgcn_perm((uint32_t)b3, (uint32_t)b2, 0x04000c0cu);
  return lo | hi;
}

__device__ __forceinline__ uint32_t pack4(int32_t b0, int32_t b1, int32_t b2, int32_t b3) {
  return (uint32_t)(b0 & 0xff) | ((uint32_t)(b1 & 0xff) << 8) | ((uint32_t)(b2 & 0xff) << 16) |
         ((uint32_t)b3 << 24);
}

}  // namespace hago
