// Pieces shared by the two int8-MFMA GEMM kernels (register-staged generic
// kernel and the LDS-DMA dense kernel): launch parameters, the per-tile
// channel terms and the requantize/store epilogue.
#pragma once

#include "hago_device.h"
#include "launch.h"

#include <cstdlib>

namespace hago {

#ifdef HAGO_PHASE_TIMING
#ifdef HAGO_STAMP_CYCLES
#define HAGO_STAMP_CLOCK clock64       // shader clock cycles
#else
#define HAGO_STAMP_CLOCK wall_clock64  // 100 MHz
#endif
#define HAGO_STAMP(p, i) do { if (threadIdx.x == 0 && (p).dbg) (p).dbg[blockIdx.x * 8 + (i)] = HAGO_STAMP_CLOCK(); } while (0)
#else
#define HAGO_STAMP(p, i) do { } while (0)
#endif

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

#ifdef HAGO_PHASE_TIMING
// development builds only: where the kernels write their phase timestamps (set by the timing driver)
inline long long* g_stamp_buffer = nullptr;
inline int g_stamp_skip = 0;
#endif

struct QgemmParams {
  const uint8_t* act;
  const int8_t* wgt;
  const int32_t* bias;
  void* out;
  const int32_t* mult;
  const int32_t* shift;
  int32_t M, N, K;
  int32_t per_channel, has_rq, acc16;
  int32_t acc_wrap_shift;  // 32 - accumulator bits (0, 16 or 8)
  int32_t out_mode;    // 0: requantized 8-bit, 1: raw int32, 2: raw int16
  uint32_t act_xor4;   // 0x80808080 for uint8 activations, else 0
  int32_t corr_coef;   // off - z_a
  uint32_t pad_byte;   // staged value of a padded tap: (z_a XOR act_xor) & 0xff
  int32_t vec_k;       // rows of both operands can be read as aligned 16-byte chunks
  int32_t vec_out;     // four consecutive results along the packed axis form one aligned store
  int32_t vec16_out;   // dense: output rows can be written as aligned 16-byte pieces
  RequantScalars rs;
  ConvGeom g;
  // implicit GEMM over a prepacked copy: its byte size and ceil(2^32 / C), ceil(2^32 / KW)
  uint32_t act_bytes, inv_c, inv_kw;
#ifdef HAGO_PHASE_TIMING
  long long* dbg;  // per-workgroup phase timestamps (development builds only)
  int dbg_skip;    // bit mask of main-loop parts to leave out in timing experiments
#endif
};

inline QgemmParams make_qgemm_params(const GemmArgs& a, const ConvGeom* cg) {
  QgemmParams p{};
  p.act = static_cast<const uint8_t*>(a.act);
  p.wgt = a.wgt;
  p.bias = a.bias;
  p.out = a.out;
  p.mult = a.rq.multiplier;
  p.shift = a.rq.shift;
  p.M = a.M; p.N = a.N; p.K = a.K;
  p.per_channel = a.rq.per_channel;
  p.has_rq = a.has_rq;
  p.acc16 = a.acc16;
  p.acc_wrap_shift = a.acc_wrap_shift;
  p.out_mode = a.has_rq ? 0 : (a.acc16 ? 2 : 1);
  p.act_xor4 = a.act_unsigned ? 0x80808080u : 0u;
  p.corr_coef = (a.act_unsigned ? 128 : 0) - a.act_zero_point;
  p.pad_byte = ((uint32_t)a.act_zero_point ^ (a.act_unsigned ? 0x80u : 0u)) & 0xffu;
  p.rs = RequantScalars{a.rq.z_out, a.rq.clip_lo - a.rq.z_out, a.rq.clip_hi - a.rq.z_out, a.rq.half_away};
  if (cg) p.g = *cg;
#ifdef HAGO_PHASE_TIMING
  p.dbg = g_stamp_buffer;
  p.dbg_skip = g_stamp_skip;
#endif
  return p;
}

inline bool ptr_aligned(const void* ptr, size_t n) {
  return (reinterpret_cast<uintptr_t>(ptr) & (n - 1)) == 0;
}
inline size_t qgemm_out_elem_size(const GemmArgs& a) { return a.has_rq ? 1 : (a.acc16 ? 2 : 4); }

// Workgroups are handed to the 8 XCDs round-robin; remap so that the tiles an
// XCD works on are consecutive (they then share operand panels in its L2).
__device__ __forceinline__ int xcd_remap(int bid, int ntiles) {
  const int x = bid & 7, slot = bid >> 3;
  const int q = ntiles >> 3, r = ntiles & 7;
  return x * q + (x < r ? x : r) + slot;
}

// Turn the weight row sums that sit in s_corr[0..CH) into the per-channel
// terms of the tile: corr = bias + (off - z_a) * sum_k w, multiplier, shift.
// Channels beyond N get zeros.  Ends with a barrier.
template <int NT, int CH>
__device__ __forceinline__ void stage_channel_terms(const QgemmParams& p, int w0, int32_t* s_corr,
                                                    int32_t* s_mult, int32_t* s_shift) {
  const int t = threadIdx.x;
  for (int ci = t; ci < CH; ci += NT) {
    const int n = w0 + ci;
    int32_t corr = 0, mu = 0, sh = 0;
    if (n < p.N) {
      corr = (p.bias ? p.bias[n] : 0) + p.corr_coef * s_corr[ci];
      if (p.has_rq) {
        mu = rq_mult(p.mult, p.per_channel ? n : 0);
        sh = rq_shift(p.mult, p.shift, p.per_channel ? n : 0);
      }
    }
    s_corr[ci] = corr;
    s_mult[ci] = mu;
    s_shift[ci] = sh;
  }
  __syncthreads();
}

// Per-channel epilogue inputs fetched at kernel start (so that their latency hides
// behind the main loop); one slot per channel this lane is responsible for.
template <int NT, int CH>
struct ChannelRegs {
  static constexpr int kSlots = (CH + NT - 1) / NT;
  int32_t bias[kSlots], mult[kSlots], shift[kSlots];
};

template <int NT, int CH>
__device__ __forceinline__ void load_channel_regs(const QgemmParams& p, int w0, ChannelRegs<NT, CH>& r) {
#pragma unroll
  for (int s = 0; s < ChannelRegs<NT, CH>::kSlots; ++s) {
    const int ci = (int)threadIdx.x + NT * s;
    const int n = w0 + ci;
    r.bias[s] = 0; r.mult[s] = 0; r.shift[s] = 1;
    if (ci < CH && n < p.N) {
      if (p.bias) r.bias[s] = p.bias[n];
      if (p.has_rq) {
        r.mult[s] = rq_mult(p.mult, p.per_channel ? n : 0);
        r.shift[s] = rq_shift(p.mult, p.shift, p.per_channel ? n : 0);
      }
    }
  }
}

// s_corr holds the weight row sums on entry (s_sum2, if given, a second part to add; it may be
// s_mult); on exit s_corr/s_mult/s_shift hold the
// per-channel terms and s_c64 the folded addend corr * mult + 2^(30+shift), with which
// (acc + corr) * mult + rounding term is one 64-bit multiply-add per element.
// Returns (block-uniform) whether the tile needs the general arithmetic: some channel has
// shift 0 (the result is then not the high dword shifted right), or a correction so large
// that acc + corr could leave int32 (whose wrap-around the folded form would not reproduce;
// |acc| <= K * 2^14 < 2^30 for K <= 2^16).
template <int NT, int CH>
__device__ __forceinline__ bool finish_channel_terms(const QgemmParams& p, const ChannelRegs<NT, CH>& r,
                                                     int32_t* s_corr, int32_t* s_mult,
                                                     int32_t* s_shift, int64_t* s_c64,
                                                     const int32_t* s_sum2 = nullptr,
                                                     int32_t* s_shm1 = nullptr) {
  int general = p.K > 65536;
#pragma unroll
  for (int s = 0; s < ChannelRegs<NT, CH>::kSlots; ++s) {
    const int ci = (int)threadIdx.x + NT * s;
    if (ci < CH) {
      const int32_t wsum = s_corr[ci] + (s_sum2 ? s_sum2[ci] : 0);
      const int32_t corr = r.bias[s] + p.corr_coef * wsum;
      s_corr[ci] = corr;
      s_mult[ci] = r.mult[s];
      s_shift[ci] = r.shift[s];
      if (s_shm1) s_shm1[ci] = r.shift[s] - 1;  // the folded form shifts the high dword by this
      s_c64[ci] = (int64_t)corr * (int64_t)r.mult[s] + ((int64_t)1 << (30 + (r.shift[s] & 31)));
      general |= (r.shift[s] <= 0) | (corr >= (1 << 30)) | (corr <= -(1 << 30));
    }
  }
  return __syncthreads_or(general) != 0;
}

// r = floor((a * m + 2^(30+sh)) / 2^(31+sh)).  With SH_GE1 (sh >= 1) the shift
// distance is at least 32, so the result is the high dword shifted by sh - 1:
// one 32-bit shift instead of a 64-bit one.
template <bool SH_GE1>
__device__ __forceinline__ int32_t mul_shift_fast(int32_t a, int32_t m, int64_t rnd, int32_t sh) {
  const int64_t pr = (int64_t)a * (int64_t)m + rnd;
  if constexpr (SH_GE1) return (int32_t)(pr >> 32) >> (sh - 1);
  return (int32_t)(pr >> (31 + sh));
}

// Dense epilogue of a tile (interior or ragged, N % 16 == 0) through LDS: requantize, pack four channels
// per dword, write the tile to LDS in output order [row m][channel n], then copy
// it out with 16-byte stores that cover whole output rows.  LDS rows are BP + 16 bytes
// apart, so the 32 rows a wavefront writes at once spread over the banks.
// s_out: BQ * (BP + 16) bytes.  FOLDED: the tile qualifies for the folded arithmetic
// (see finish_channel_terms); otherwise the general form is used.
template <int WP, int WQ, int TP, int TQ, bool FOLDED>
__device__ __forceinline__ void qgemm_epilogue_dense_staged(const QgemmParams& p,
                                                            v16i (&acc)[TP][TQ], int p0, int q0,
                                                            const int32_t* s_corr,
                                                            const int32_t* s_mult,
                                                            const int32_t* s_shift,
                                                            const int64_t* s_c64,
                                                            const int32_t* s_shm1,
                                                            uint8_t* s_out) {
  constexpr int NT = 64 * WP * WQ;
  constexpr int BP = WP * TP * 32, BQ = WQ * TQ * 32;
  constexpr int CPR = BP / 16;   // 16-byte chunks per tile row
  constexpr int RS = BP + 16;    // LDS row stride
  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const int wp = wave % WP, wq = wave / WP;
  const int frow = lane & 31, fhalf = lane >> 5;
  int32_t lo = p.rs.lo_rel, hi = p.rs.hi_rel;
  const int32_t z = p.rs.z_out;
  // v_med3 takes one scalar operand at most: keep the bounds in vector registers once
  asm volatile("" : "+v"(lo), "+v"(hi));
  uint8_t* my_row = s_out + ((wq * TQ) * 32 + frow) * RS + wp * TP * 32 + fhalf * 4;
  // Per-channel terms of group g = (ti, g4): four consecutive channels.  The terms of the next
  // group are fetched while the current one is computed, and no further ahead (fetching all
  // groups up front would cost more registers than the accumulators leave).
  struct Terms { int4 m4, s4, c4; longlong2 ca, cb; };
  auto load_terms = [&](int g) {
    const int i_loc = (wp * TP + g / 4) * 32 + (g % 4) * 8 + fhalf * 4;
    Terms t;
    t.m4 = *reinterpret_cast<const int4*>(s_mult + i_loc);
    t.s4 = *reinterpret_cast<const int4*>((FOLDED ? s_shm1 : s_shift) + i_loc);
    if constexpr (FOLDED) {
      t.ca = *reinterpret_cast<const longlong2*>(s_c64 + i_loc);
      t.cb = *reinterpret_cast<const longlong2*>(s_c64 + i_loc + 2);
    } else {
      t.c4 = *reinterpret_cast<const int4*>(s_corr + i_loc);
    }
    return t;
  };
  Terms cur = load_terms(0);
#pragma unroll
  for (int g = 0; g < TP * 4; ++g) {
    const int ti = g / 4, g4 = g % 4;
    Terms nxt = cur;
    if (g + 1 < TP * 4) nxt = load_terms(g + 1);
    __builtin_amdgcn_sched_barrier(0);
    const int32_t mm[4] = {cur.m4.x, cur.m4.y, cur.m4.z, cur.m4.w};
    const int32_t ss[4] = {cur.s4.x, cur.s4.y, cur.s4.z, cur.s4.w};
    int32_t r[TQ][4];
    if constexpr (FOLDED) {
      const int64_t c64[4] = {cur.ca.x, cur.ca.y, cur.cb.x, cur.cb.y};
#pragma unroll
      for (int tj = 0; tj < TQ; ++tj)
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const int64_t pr = (int64_t)acc[ti][tj][g4 * 4 + e] * (int64_t)mm[e] + c64[e];
          r[tj][e] = (int32_t)(pr >> 32) >> ss[e];  // ss = shift - 1 here
        }
    } else {
      const int32_t cc[4] = {cur.c4.x, cur.c4.y, cur.c4.z, cur.c4.w};
#pragma unroll
      for (int tj = 0; tj < TQ; ++tj)
#pragma unroll
        for (int e = 0; e < 4; ++e)
          r[tj][e] = mul_shift_fast<false>(acc[ti][tj][g4 * 4 + e] + cc[e], mm[e],
                                           (int64_t)1 << (30 + ss[e]), ss[e]);
    }
#pragma unroll
    for (int tj = 0; tj < TQ; ++tj) {
      int32_t r0 = med3(r[tj][0], lo, hi), r1 = med3(r[tj][1], lo, hi);
      int32_t r2 = med3(r[tj][2], lo, hi), r3 = med3(r[tj][3], lo, hi);
      if (z != 0) { r0 += z; r1 += z; r2 += z; r3 += z; }
      *reinterpret_cast<uint32_t*>(my_row + tj * 32 * RS + ti * 32 + g4 * 8) =
          pack4_perm(r0, r1, r2, r3);
    }
    __builtin_amdgcn_sched_barrier(0);
    cur = nxt;
  }
  __syncthreads();
  HAGO_STAMP(p, 5);
  uint8_t* out8 = static_cast<uint8_t*>(p.out);
  const bool ragged = q0 + BQ > p.M || p0 + BP > p.N;  // block-uniform
#pragma unroll
  for (int s = 0; s < (BQ * CPR) / NT; ++s) {
    const int q = (int)threadIdx.x + NT * s;
    const int row = q / CPR, c = q % CPR;
    const v4i v = *reinterpret_cast<const v4i*>(s_out + row * RS + c * 16);
    // ragged tiles: rows beyond M and 16-channel chunks beyond N (N % 16 == 0) stay in LDS
    if (!ragged || (q0 + row < p.M && p0 + c * 16 < p.N))
      // streaming store: the tile is complete and nothing in this launch reads it again, so it
      // need not stay in L2 until the end-of-kernel write-back (large outputs: 1 us per launch)
      __builtin_nontemporal_store(v, reinterpret_cast<v4i*>(out8 + (size_t)(q0 + row) * p.N + p0 + c * 16));
  }
  HAGO_STAMP(p, 6);
}

// Straight-line epilogue of a tile (interior or ragged) whose packed stores are aligned.
// OM: 0 requantized 8-bit, 1 raw int32, 2 raw int16.
template <int OM>
__device__ __forceinline__ void store_group(void* out, size_t off, int32_t v0, int32_t v1,
                                            int32_t v2, int32_t v3) {
  if constexpr (OM == 0)
    *reinterpret_cast<uint32_t*>(static_cast<uint8_t*>(out) + off) = pack4(v0, v1, v2, v3);
  else if constexpr (OM == 1)
    *reinterpret_cast<int4*>(static_cast<int32_t*>(out) + off) = make_int4(v0, v1, v2, v3);
  else
    *reinterpret_cast<short4*>(static_cast<int16_t*>(out) + off) =
        make_short4((short)v0, (short)v1, (short)v2, (short)v3);
}

template <int OM, bool AWAY>
__device__ __forceinline__ int32_t finish_one(int32_t a, int32_t m, int32_t sh, int32_t acc16,
                                              const RequantScalars& rs) {
  if (acc16) a = wrap_acc_bits(a, acc16);  // (the wrap shift of a narrow accumulator, 0 for int32)
  if constexpr (OM == 0) a = AWAY ? requant_half_away(a, m, sh, rs) : requant_one(a, m, sh, rs);
  return a;
}

// Row r of a 32-row block holds pixel pix_perm(r) of the block when the loader placed the pixels
// that way (PIXPERM): registers 4g + e of lane half h are then the 16 consecutive pixels
// 16h + 4g + e, which go out as one 16-byte store per channel instead of four scattered dwords.
__device__ __forceinline__ constexpr int pix_perm(int r) {
  return 16 * ((r >> 2) & 1) + 4 * (r >> 3) + (r & 3);
}

template <int WP, int WQ, int TP, int TQ, bool ACT_ON_P, int OM, bool PIXPERM, bool RAGGED, bool AWAY>
__device__ __forceinline__ void qgemm_epilogue_fast(const QgemmParams& p, v16i (&acc)[TP][TQ],
                                                    int p0, int q0, const int32_t* s_corr,
                                                    const int32_t* s_mult,
                                                    const int32_t* s_shift) {
  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const int wp = wave % WP, wq = wave / WP;
  const int frow = lane & 31, fhalf = lane >> 5;
  const RequantScalars rs = p.rs;
  const int32_t acc16 = p.acc_wrap_shift;
  // ragged tiles: a group of four results along the packed axis is inside the tensor or outside
  // (the packed extent is a multiple of 4, of 16 where 16-byte stores are used)
  const int P_ext = ACT_ON_P ? p.M : p.N;
  const int Q_ext = ACT_ON_P ? p.N : p.M;
  if constexpr (!ACT_ON_P) {
#pragma unroll
    for (int ti = 0; ti < TP; ++ti) {
#pragma unroll
      for (int g4 = 0; g4 < 4; ++g4) {
        const int i_loc = (wp * TP + ti) * 32 + g4 * 8 + fhalf * 4;
        const int4 c4 = *reinterpret_cast<const int4*>(s_corr + i_loc);
        const int4 m4 = *reinterpret_cast<const int4*>(s_mult + i_loc);
        const int4 s4 = *reinterpret_cast<const int4*>(s_shift + i_loc);
#pragma unroll
        for (int tj = 0; tj < TQ; ++tj) {
          const int j = q0 + (wq * TQ + tj) * 32 + frow;
          const int32_t r0 = finish_one<OM, AWAY>(acc[ti][tj][g4 * 4 + 0] + c4.x, m4.x, s4.x, acc16, rs);
          const int32_t r1 = finish_one<OM, AWAY>(acc[ti][tj][g4 * 4 + 1] + c4.y, m4.y, s4.y, acc16, rs);
          const int32_t r2 = finish_one<OM, AWAY>(acc[ti][tj][g4 * 4 + 2] + c4.z, m4.z, s4.z, acc16, rs);
          const int32_t r3 = finish_one<OM, AWAY>(acc[ti][tj][g4 * 4 + 3] + c4.w, m4.w, s4.w, acc16, rs);
          if (!RAGGED || (j < Q_ext && p0 + i_loc < P_ext))
            store_group<OM>(p.out, (size_t)j * p.N + (p0 + i_loc), r0, r1, r2, r3);
        }
      }
    }
  } else {
    const int ohw = p.g.OH * p.g.OW;
    // 16 consecutive pixels of a lane lie in one image and form one aligned store
    const bool vec16 = PIXPERM && OM == 0 && (ohw & 15) == 0 && (reinterpret_cast<uintptr_t>(p.out) & 15u) == 0;
#pragma unroll
    for (int tj = 0; tj < TQ; ++tj) {
      const int j_loc = (wq * TQ + tj) * 32 + frow;
      const int j = q0 + j_loc;
      const int32_t c = s_corr[j_loc], m = s_mult[j_loc], sh = s_shift[j_loc];
#pragma unroll
      for (int ti = 0; ti < TP; ++ti) {
        if constexpr (PIXPERM && OM == 0) {
          if (vec16) {
            const int i = p0 + (wp * TP + ti) * 32 + fhalf * 16;
            const int b = i / ohw;
            const int pix = i - b * ohw;
            uint32_t dw[4];
#pragma unroll
            for (int g4 = 0; g4 < 4; ++g4)
              dw[g4] = pack4(finish_one<OM, AWAY>(acc[ti][tj][g4 * 4 + 0] + c, m, sh, acc16, rs),
                             finish_one<OM, AWAY>(acc[ti][tj][g4 * 4 + 1] + c, m, sh, acc16, rs),
                             finish_one<OM, AWAY>(acc[ti][tj][g4 * 4 + 2] + c, m, sh, acc16, rs),
                             finish_one<OM, AWAY>(acc[ti][tj][g4 * 4 + 3] + c, m, sh, acc16, rs));
            if (!RAGGED || (j < Q_ext && i < P_ext))
              *reinterpret_cast<uint4*>(static_cast<uint8_t*>(p.out) + ((size_t)b * p.N + j) * ohw + pix) =
                  make_uint4(dw[0], dw[1], dw[2], dw[3]);
            continue;
          }
        }
        if constexpr (PIXPERM && OM == 2) {
          // raw int16: the lane's 16 pixels are 32 contiguous bytes, two aligned 16-byte stores
          if ((ohw & 7) == 0 && (reinterpret_cast<uintptr_t>(p.out) & 15u) == 0) {
#pragma unroll
            for (int g2 = 0; g2 < 2; ++g2) {
              const int i = p0 + (wp * TP + ti) * 32 + fhalf * 16 + g2 * 8;
              const int b = i / ohw;
              const int pix = i - b * ohw;
              uint32_t dw[4];
#pragma unroll
              for (int x = 0; x < 4; ++x) {
                const int32_t lo16 = finish_one<OM, AWAY>(acc[ti][tj][g2 * 8 + 2 * x] + c, m, sh, acc16, rs);
                const int32_t hi16 = finish_one<OM, AWAY>(acc[ti][tj][g2 * 8 + 2 * x + 1] + c, m, sh, acc16, rs);
                dw[x] = ((uint32_t)lo16 & 0xffffu) | ((uint32_t)hi16 << 16);
              }
              if (!RAGGED || (j < Q_ext && i < P_ext))
                *reinterpret_cast<uint4*>(static_cast<int16_t*>(p.out) + ((size_t)b * p.N + j) * ohw + pix) =
                    make_uint4(dw[0], dw[1], dw[2], dw[3]);
            }
            continue;
          }
        }
#pragma unroll
        for (int g4 = 0; g4 < 4; ++g4) {
          const int i = p0 + (wp * TP + ti) * 32 + (PIXPERM ? fhalf * 16 + g4 * 4 : g4 * 8 + fhalf * 4);
          const int b = i / ohw;
          const int pix = i - b * ohw;
          const int32_t r0 = finish_one<OM, AWAY>(acc[ti][tj][g4 * 4 + 0] + c, m, sh, acc16, rs);
          const int32_t r1 = finish_one<OM, AWAY>(acc[ti][tj][g4 * 4 + 1] + c, m, sh, acc16, rs);
          const int32_t r2 = finish_one<OM, AWAY>(acc[ti][tj][g4 * 4 + 2] + c, m, sh, acc16, rs);
          const int32_t r3 = finish_one<OM, AWAY>(acc[ti][tj][g4 * 4 + 3] + c, m, sh, acc16, rs);
          if (!RAGGED || (j < Q_ext && i < P_ext))
            store_group<OM>(p.out, ((size_t)b * p.N + j) * ohw + pix, r0, r1, r2, r3);
        }
      }
    }
  }
}

// Epilogue of one workgroup tile.  acc[ti][tj] is the 32x32 MFMA result of
// sub-tile (ti, tj) of this wavefront: lane l owns column j = l % 32 and, in
// registers 4g .. 4g+3, rows 8g + 4*(l / 32) + 0..3.
//   ACT_ON_P == false (dense, NHWC): i = output channel n, j = row m, out[m*N + n]
//   ACT_ON_P == true  (NCHW)       : i = pixel m, j = channel n, out[(b*N + n)*OHW + pix]
// Tensors whose groups of four results along the packed axis are aligned stores
// take a straight-line path (ragged tiles included: a group is inside or outside);
// everything else goes through the element-wise generic path.
template <int WP, int WQ, int TP, int TQ, bool ACT_ON_P, bool PIXPERM = false>
__device__ __forceinline__ void qgemm_epilogue(const QgemmParams& p, v16i (&acc)[TP][TQ], int p0,
                                               int q0, const int32_t* s_corr,
                                               const int32_t* s_mult, const int32_t* s_shift) {
  constexpr int BP = WP * TP * 32, BQ = WQ * TQ * 32;
  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const int wp = wave % WP, wq = wave / WP;
  const int frow = lane & 31, fhalf = lane >> 5;
  const int P_ext = ACT_ON_P ? p.M : p.N;
  const int Q_ext = ACT_ON_P ? p.N : p.M;
  const int ohw = p.g.OH * p.g.OW;
  const bool fast = p.vec_out;  // groups of four along the packed axis are aligned stores

  if (fast) {
    // interior tiles (block-uniform) run without the per-store bounds checks
    const bool ragged = p0 + BP > P_ext || q0 + BQ > Q_ext;
#define HAGO_FAST_EPILOGUE_R(OM, AWAY)                                                                  \
  (ragged ? qgemm_epilogue_fast<WP, WQ, TP, TQ, ACT_ON_P, OM, PIXPERM, true, AWAY>(p, acc, p0, q0,      \
                                                                                   s_corr, s_mult,      \
                                                                                   s_shift)             \
          : qgemm_epilogue_fast<WP, WQ, TP, TQ, ACT_ON_P, OM, PIXPERM, false, AWAY>(p, acc, p0, q0,     \
                                                                                    s_corr, s_mult,     \
                                                                                    s_shift))
    // (the tie rule only matters for requantized output)
#define HAGO_FAST_EPILOGUE(OM) HAGO_FAST_EPILOGUE_R(OM, false)
    if (p.out_mode == 0) {
      if (p.rs.half_away)
        HAGO_FAST_EPILOGUE_R(0, true);
      else
        HAGO_FAST_EPILOGUE(0);
    } else if (p.out_mode == 1) {
      HAGO_FAST_EPILOGUE(1);
    } else {
      HAGO_FAST_EPILOGUE(2);
    }
#undef HAGO_FAST_EPILOGUE_R
#undef HAGO_FAST_EPILOGUE
    return;
  }

  // ---- NCHW output whose image size is not a multiple of 4 (7 x 7 feature maps): a lane's 16
  // consecutive pixels are stored one by one, walking (image, pixel) without a division per element
  if constexpr (ACT_ON_P && PIXPERM) {
    const int32_t acc16 = p.acc_wrap_shift;
#pragma unroll 1
    for (int tj = 0; tj < TQ; ++tj) {
      const int j_loc = (wq * TQ + tj) * 32 + frow;
      const int j = q0 + j_loc;
      const int32_t c = s_corr[j_loc], m = s_mult[j_loc], sh = s_shift[j_loc];
#pragma unroll
      for (int ti = 0; ti < TP; ++ti) {
        const int i0 = p0 + (wp * TP + ti) * 32 + fhalf * 16;
        int b = i0 / ohw;
        int pix = i0 - b * ohw;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          // acc[..][tj] with a runtime tj would need dynamic register indexing; select instead
          int32_t raw = 0;
#pragma unroll
          for (int x = 0; x < TQ; ++x) raw = (x == tj) ? acc[ti][x][r] : raw;
          int32_t a = raw + c;
          if (acc16) a = wrap_acc_bits(a, acc16);
          if (p.has_rq) a = requant_general(a, m, sh, p.rs);
          if (j < Q_ext && i0 + r < P_ext) {
            const int64_t o = ((int64_t)b * p.N + j) * ohw + pix;
            if (p.out_mode == 0)
              static_cast<uint8_t*>(p.out)[o] = (uint8_t)a;
            else if (p.out_mode == 1)
              static_cast<int32_t*>(p.out)[o] = a;
            else
              static_cast<int16_t*>(p.out)[o] = (int16_t)a;
          }
          if (++pix == ohw) { pix = 0; ++b; }
        }
      }
    }
    return;
  }

  // ---- generic path: any output mode, partial tiles, unaligned outputs
#pragma unroll 1
  for (int tj = 0; tj < TQ; ++tj) {
    const int j_loc = (wq * TQ + tj) * 32 + frow;
    const int j = q0 + j_loc;
#pragma unroll
    for (int ti = 0; ti < TP; ++ti) {
#pragma unroll
      for (int g4 = 0; g4 < 4; ++g4) {
        const int i_loc = (wp * TP + ti) * 32 + (PIXPERM ? fhalf * 16 + g4 * 4 : g4 * 8 + fhalf * 4);
        const int i = p0 + i_loc;
        int32_t v[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const int ci = ACT_ON_P ? j_loc : i_loc + r;
          // acc[..][tj] with a runtime tj would need dynamic register indexing; select instead
          int32_t raw = 0;
#pragma unroll
          for (int x = 0; x < TQ; ++x) raw = (x == tj) ? acc[ti][x][g4 * 4 + r] : raw;
          int32_t a = raw + s_corr[ci];
          if (p.acc_wrap_shift) a = wrap_acc_bits(a, p.acc_wrap_shift);
          if (p.has_rq) a = requant_general(a, s_mult[ci], s_shift[ci], p.rs);
          v[r] = a;
        }
        if (j >= Q_ext || i >= P_ext) continue;
        // flat offset of (i, j) in the output tensor
        int64_t off;
        int b = 0, pix = 0;
        if constexpr (ACT_ON_P) {
          b = i / ohw;
          pix = i - b * ohw;
          off = ((int64_t)b * p.N + j) * ohw + pix;
        } else {
          off = (int64_t)j * p.N + i;
        }
        if (p.vec_out && i + 3 < P_ext) {
          if (p.out_mode == 0)
            *reinterpret_cast<uint32_t*>(static_cast<uint8_t*>(p.out) + off) =
                pack4(v[0], v[1], v[2], v[3]);
          else if (p.out_mode == 1)
            *reinterpret_cast<int4*>(static_cast<int32_t*>(p.out) + off) =
                make_int4(v[0], v[1], v[2], v[3]);
          else
            *reinterpret_cast<short4*>(static_cast<int16_t*>(p.out) + off) =
                make_short4((short)v[0], (short)v[1], (short)v[2], (short)v[3]);
        } else {
#pragma unroll
          for (int r = 0; r < 4; ++r) {
            if (i + r >= P_ext) break;
            int64_t o = off + r;
            if constexpr (ACT_ON_P) {
              int pr = pix + r, br = b;
              while (pr >= ohw) { pr -= ohw; ++br; }
              o = ((int64_t)br * p.N + j) * ohw + pr;
            }
            if (p.out_mode == 0)
              static_cast<uint8_t*>(p.out)[o] = (uint8_t)v[r];
            else if (p.out_mode == 1)
              static_cast<int32_t*>(p.out)[o] = v[r];
            else
              static_cast<int16_t*>(p.out)[o] = (int16_t)v[r];
          }
        }
      }
    }
  }
}

}  // namespace hago
