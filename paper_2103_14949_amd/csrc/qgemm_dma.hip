// Dense int8 GEMM, fast path: operands stream from global memory straight
// into LDS (buffer_load ... lds, 16 bytes per lane) through a ring of 64-byte
// k-stages, so no vector registers and no LDS-write instructions are spent on
// staging and two stages of loads are in flight behind the one being read.
//
// Layout.  D[i][j] = sum_k P[i][k] Q[j][k] with P = weights [N,K] (i = output
// channel, contiguous in the output) and Q = activations [M,K].  A stage holds
// BP + BQ rows of 64 bytes.  One DMA instruction of a wavefront fills 1024
// contiguous LDS bytes = 16 rows x four 16-byte slots; the lane that owns slot
// (row, s) fetches the logical chunk s ^ f(row) of that row from memory, which
// realises the bank swizzle on the global side because the LDS side of the DMA
// is fixed (lane l -> byte l * 16).
//
// Out-of-range data.  Every load goes through a buffer descriptor whose size
// is the tensor's exact byte count, and lanes whose row or k lies outside the
// matrix are given an offset beyond it: the hardware then writes zeros to LDS.
// Zero weights make the padded k contribute nothing; padded rows are never
// stored.
//
// uint8 activations and the zero point are handled on the fragments: the
// activation fragment is XORed with 0x80 per byte after it is read from LDS,
// and the weight row sums needed for the zero-point term are accumulated from
// the weight fragments (see qgemm.hip for the identity) with v_sad_u8 on the
// sign-flipped bytes: v_dot4 competes with the MFMAs for the matrix pipe,
// plain vector instructions run in their shadow.
//
// Schedule.  The ring is unrolled in the main loop, so LDS addresses are
// constants.  At the top of iteration kt both fragment sets (one per 32-k half)
// hold stage kt.  One s_waitcnt vmcnt + s_barrier per stage says that stage
// kt+1 has landed for every wavefront and that every wavefront has its
// fragments of stage kt-1, whose ring slot this iteration's DMA instructions
// refill with stage kt+kStages-1.  Each fragment register is re-read from stage
// kt+1 right after the last MFMA that uses it, i.e. a whole stage of MFMAs
// before it is needed, and the flips are applied to the set that is not being
// multiplied.  DMA instructions, flips, sums and fragment reads are dealt out
// behind individual MFMAs.  The k offset of a full stage travels in the DMA
// instruction's scalar offset, so the steady state computes no addresses.
#include "qgemm_common.h"

#include <cstdlib>
#include <type_traits>
#include <utility>

namespace hago {

namespace {

constexpr int kBK = 64;       // k-bytes per stage
constexpr uint32_t kOob = 0x80000000u;  // offset beyond any tensor (sizes are < 2^31 bytes)

__device__ __forceinline__ int swz4(int row) { return ((row >> 1) ^ (row >> 3)) & 3; }

__device__ __forceinline__ void dma16(v4i rsrc, uint32_t lds_addr, uint32_t voff) {
  // m0 = LDS byte address of the wavefront's 1 KB window; lane l lands at m0 + 16 * l
  asm volatile("s_mov_b32 m0, %0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds"
               :
               : "s"(lds_addr), "v"(voff), "s"(rsrc)
               : "memory");
}

// Same with a scalar byte offset added to every lane's address (not range checked).
__device__ __forceinline__ void dma16s(v4i rsrc, uint32_t lds_addr, uint32_t voff, uint32_t soff) {
  asm volatile("s_mov_b32 m0, %0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds"
               :
               : "s"(lds_addr), "v"(voff), "s"(rsrc), "s"(soff)
               : "memory");
}

__device__ __forceinline__ v4i make_rsrc(const void* base, uint32_t bytes) {
  const uint64_t a = reinterpret_cast<uint64_t>(base);
  v4i r;
  r.x = __builtin_amdgcn_readfirstlane((int)(uint32_t)a);
  r.y = __builtin_amdgcn_readfirstlane((int)(uint32_t)(a >> 32));  // stride 0, no swizzle
  r.z = __builtin_amdgcn_readfirstlane((int)bytes);
  r.w = 0x00020000;  // raw buffer, 32-bit data format
  return r;
}

// kStages: depth of the LDS ring; OCC: wavefronts per SIMD the register budget must allow
// (two 4-wavefront workgroups per CU keep the matrix pipe busy across each other's barriers).
// CONV: the activation operand is an implicit im2col view of a padded NHWC copy of the input
// (see conv_prepack.hip); ACT_ON_P: activations are the P operand (NCHW output).
template <int WP, int WQ, int TP, int TQ, int kStages, int OCC, bool CONV, bool ACT_ON_P>
__global__ __launch_bounds__(64 * WP * WQ, OCC) void qgemm_dma_kernel(QgemmParams p) {
  HAGO_STAMP(p, 7);
  constexpr int NW = WP * WQ;          // wavefronts
  constexpr int NT = 64 * NW;
  constexpr int BP = WP * TP * 32;
  constexpr int BQ = WQ * TQ * 32;
  constexpr int STAGE = (BP + BQ) * kBK;
  constexpr int GP = BP / 16, GQ = BQ / 16;  // 16-row groups (one DMA instruction each)
  constexpr int G = GP + GQ;
  // Groups are dealt round-robin: wavefront w issues groups w, w + NW, ...  Every wavefront
  // issues exactly L instructions per stage (the wait counts rely on it); a slot without a
  // group fetches out-of-range data into a spare 1 KB of LDS.
  constexpr int L = (G + NW - 1) / NW;
  constexpr int CH = ACT_ON_P ? BQ : BP;  // output channels covered by the tile

  extern __shared__ __attribute__((aligned(16))) uint8_t smem[];
  int32_t* s_corr = reinterpret_cast<int32_t*>(smem + kStages * STAGE + 1024);  // after the spare
  int32_t* s_mult = s_corr + CH;
  int32_t* s_shift = s_mult + CH;
  int64_t* s_c64 = reinterpret_cast<int64_t*>(s_shift + CH);

  const int t = threadIdx.x;
  const int lane = t & 63;
  const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
  const int wp = wave % WP;
  const int wq = wave / WP;

  const int P_ext = ACT_ON_P ? p.M : p.N;
  const int Q_ext = ACT_ON_P ? p.N : p.M;
  const int tiles_p = (P_ext + BP - 1) / BP;
  const int tile = xcd_remap(blockIdx.x, gridDim.x);
  const int tile_p = tile % tiles_p;
  const int tile_q = tile / tiles_p;
  const int p0 = tile_p * BP;  // first P row of the tile
  const int q0 = tile_q * BQ;  // first Q row of the tile
  const int w0 = ACT_ON_P ? q0 : p0;  // first output channel

  const v4i rs_w = make_rsrc(p.wgt, (uint32_t)p.N * (uint32_t)p.K);
  const v4i rs_a = make_rsrc(p.act, CONV ? p.act_bytes : (uint32_t)p.M * (uint32_t)p.K);
  const v4i rs_p = ACT_ON_P ? rs_a : rs_w;
  const v4i rs_q = ACT_ON_P ? rs_w : rs_a;
  const uint32_t lds0 =
      (uint32_t)(size_t)(__attribute__((address_space(3))) uint8_t*)smem;

  // Per-lane global offset of the row this lane fetches in DMA slot d (without the k part), and
  // the logical chunk (in bytes) it fetches inside a stage.
  // weights: row * K.  activations: dense row * K; conv: offset of the output pixel's window
  // origin in the padded NHWC copy.
  auto row_offset = [&](int row, bool is_act) -> uint32_t {
    if (!is_act) return row < p.N ? (uint32_t)row * (uint32_t)p.K : kOob;
    if (row >= p.M) return kOob;
    if constexpr (!CONV) {
      return (uint32_t)row * (uint32_t)p.K;
    } else {
      const ConvGeom& g = p.g;  // H, W, C are the padded copy's dimensions
      const int ohw = g.OH * g.OW;
      const int b = row / ohw;
      const int pix = row - b * ohw;
      const int oy = pix / g.OW;
      const int ox = pix - oy * g.OW;
      return (uint32_t)(((b * g.H + oy * g.stride_h) * g.W + ox * g.stride_w) * g.C);
    }
  };
  uint32_t voff[L];  // row offset + chunk: the per-lane part of a full stage's address
  uint32_t m0s[L];   // LDS address of the slot's 1 KB window in ring slot 0 (wavefront-uniform)
  bool slot_real[L]; // false: the slot has no group, it fetches zeros into the spare window
  bool slot_q[L], slot_act[L];
  const int lrow = lane >> 2;  // row inside a 16-row group
  const int lslot = lane & 3;  // physical 16-byte slot
  const uint32_t spare = lds0 + (uint32_t)kStages * STAGE;
  // The swizzle depends on the row inside a 32-row block only, and a wavefront's groups all
  // have the parity of its index, so the logical chunk is the same in every slot.
  static_assert(NW % 2 == 0 && GP % 2 == 0, "group parity must not depend on the slot");
  const int lck = (lslot ^ swz4((wave & 1) * 16 + lrow)) * 16;  // chunk (bytes) inside a stage
#pragma unroll
  for (int d = 0; d < L; ++d) {
    const int grp = wave + NW * d;
    const bool isq = grp >= GP;
    const int rt = (isq ? grp - GP : grp) * 16 + lrow;  // row inside its tile
    slot_q[d] = isq;
    slot_act[d] = isq ? !ACT_ON_P : ACT_ON_P;
    slot_real[d] = grp < G;
    uint32_t off = kOob;
    m0s[d] = spare;
    if (grp < G) {
      off = row_offset((isq ? q0 : p0) + rt, slot_act[d]);
      m0s[d] = (uint32_t)__builtin_amdgcn_readfirstlane(
          (int)(lds0 + (uint32_t)(isq ? BP * kBK + (grp - GP) * 1024 : grp * 1024)));
    }
    voff[d] = off == kOob ? kOob : off + (uint32_t)lck;
  }
  // k (position along the reduction) -> byte offset relative to the row offset
  auto k_offset = [&](int kk, bool is_act) -> uint32_t {
    if constexpr (CONV) {
      if (is_act) {
        const ConvGeom& g = p.g;
        const int t = (int)__umulhi((uint32_t)kk, p.inv_c);      // kk / C   (tap index)
        const int c = kk - t * g.C;
        const int ky = g.KW == 1 ? t : (int)__umulhi((uint32_t)t, p.inv_kw);  // t / KW
        const int kx = t - ky * g.KW;
        return (uint32_t)((ky * g.W + kx) * g.C + c);
      }
    }
    return (uint32_t)kk;
  };
  // A stage whose 64 k lie inside K and (conv) inside one filter tap has the same k offset in
  // every lane: it travels in the instruction's scalar offset, which is not range checked, and
  // the per-lane offsets never change.  Other stages (the K tail, the zero fills beyond K,
  // conv stages that straddle taps) compute per-lane offsets.
  const int KF = p.K / kBK;  // stages that lie fully inside K
  const bool uniform_k = !CONV || (p.g.C % kBK == 0);

  // DMA slot d (0 .. L-1) of stage stage_idx into ring slot RS.  d and RS are compile-time
  // constants at every call site.
  auto issue_one = [&](int stage_idx, auto rsconst, auto dconst) {
    constexpr int d = decltype(dconst)::value;
    constexpr int RS = decltype(rsconst)::value;
    const int k0 = stage_idx * kBK;
    const v4i rs = slot_q[d] ? rs_q : rs_p;
    const uint32_t dst = slot_real[d] ? m0s[d] + (uint32_t)(RS * STAGE) : spare;
    if (uniform_k && stage_idx < KF) {
      dma16s(rs, dst, voff[d], k_offset(k0, slot_act[d]));
    } else {
      uint32_t o = voff[d] - (uint32_t)lck + k_offset(k0 + lck, slot_act[d]);
      if (voff[d] == kOob || k0 + lck >= p.K) o = kOob;
      dma16(rs, dst, o);
    }
  };
  auto issue_range = [&](int stage_idx, auto rsconst, auto lo, auto hi) {
    constexpr int kLo = decltype(lo)::value, kHi = decltype(hi)::value;
    [&]<int... I>(std::integer_sequence<int, I...>) {
      (issue_one(stage_idx, rsconst, std::integral_constant<int, kLo + I>{}), ...);
    }(std::make_integer_sequence<int, kHi - kLo>{});
  };
  constexpr int LH = (L + 1) / 2;  // a stage is issued in two parts (LH and L - LH instructions),
                                  // spread over two MFMA groups
  using IC0 = std::integral_constant<int, 0>;
  using ICL = std::integral_constant<int, L>;

  HAGO_STAMP(p, 0);
  ChannelRegs<NT, CH> chregs;
  load_channel_regs<NT, CH>(p, w0, chregs);

  v16i acc[TP][TQ];
#pragma unroll
  for (int i = 0; i < TP; ++i)
#pragma unroll
    for (int j = 0; j < TQ; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0;
  constexpr int TW = ACT_ON_P ? TQ : TP;  // weight fragments per wavefront
  uint32_t wsum[TW];  // biased: every byte counts as w + 128
#pragma unroll
  for (int i = 0; i < TW; ++i) wsum[i] = 0;

  const int KT = (p.K + kBK - 1) / kBK;
  // prologue: stages 0 .. kStages-2 (stages beyond K are all-zero fills, which keeps the
  // number of outstanding loads uniform)
  [&]<int... S>(std::integer_sequence<int, S...>) {
    (issue_range(S, std::integral_constant<int, S>{}, IC0{}, ICL{}), ...);
  }(std::make_integer_sequence<int, kStages - 1>{});
  HAGO_STAMP(p, 1);

  const int frow = lane & 31;
  const int fhalf = lane >> 5;
  // every wavefront sums its weight fragments (no branch); one per fragment row stores them
  const bool sums_here = ACT_ON_P ? (wp == 0) : (wq == 0);
  const bool need_wsum = (p.corr_coef != 0);
  // Fragment addresses inside a stage (bytes).  Fragment i of a wavefront lies i * 32 rows
  // after fragment 0 and has the same swizzle (it depends on the row inside a 32-row block
  // only), so one register per operand and k-half serves every fragment, ring slot and
  // operand region through constant offsets.
  int pa[2], qa[2];
#pragma unroll
  for (int ks = 0; ks < 2; ++ks) {
    const int chunk = ((ks * 2 + fhalf) ^ swz4(frow)) * 16;
    pa[ks] = (wp * TP * 32 + frow) * kBK + chunk;
    qa[ks] = (wq * TQ * 32 + frow) * kBK + chunk;
  }
  constexpr int kFrag = 32 * kBK;     // bytes between consecutive fragments of a wavefront
  constexpr int kQBase = BP * kBK;    // the Q rows follow the P rows inside a stage

  // Fragment sets for the two 32-k halves of a stage.  A fragment register is refilled with the
  // NEXT stage's data right after the last MFMA that reads it, a whole stage of MFMAs before it
  // is needed again, so LDS latency (and the burst of reads after a barrier) stays hidden.
  v4i pf0[TP], qf0[TQ], pf1[TP], qf1[TQ];
  auto read_frags = [&](const uint8_t* base, int ks, v4i (&pf)[TP], v4i (&qf)[TQ]) {
#pragma unroll
    for (int i = 0; i < TP; ++i) pf[i] = *reinterpret_cast<const v4i*>(base + pa[ks] + i * kFrag);
#pragma unroll
    for (int j = 0; j < TQ; ++j)
      qf[j] = *reinterpret_cast<const v4i*>(base + qa[ks] + kQBase + j * kFrag);
  };
  // Flipping the sign bit of uint8 activation fragments and summing the weight fragments are
  // vector instructions that a wavefront can issue in the shadow of its own MFMAs, a few per
  // MFMA, as long as the next MFMA does not wait for them: the flips are applied to the OTHER
  // fragment set (read during the previous half), the sums to the current one before its refill.
  // FLIP / WSUM are compile-time, so that the steady state has no branches.
  constexpr int NM = TP * TQ;  // MFMAs per half
  auto flip = [&](v4i& f) {
    const int x4 = (int)p.act_xor4;
    f = v4i{f.x ^ x4, f.y ^ x4, f.z ^ x4, f.w ^ x4};
  };
  auto sum4 = [&](uint32_t& a, const v4i& f) {
    // sum of the bytes, each + 128 (v_dot4 would stall the matrix pipe, v_sad_u8 does not)
#pragma unroll
    for (int u = 0; u < 4; ++u) a = __builtin_amdgcn_sad_u8((uint32_t)f[u] ^ 0x80808080u, 0u, a);
  };
  // One 32-k half KS of a stage: multiply the current set (pf, qf); behind the MFMAs go the
  // weight sums, the flips of the other set's activation fragments (pn, qn), the refills of the
  // current set from the next stage (at `next`), and this half's share of a stage's DMA
  // instructions (so the memory pipe is fed a few instructions at a time).
  auto multiply = [&](v4i (&pf)[TP], v4i (&qf)[TQ], v4i (&pn)[TP], v4i (&qn)[TQ], const uint8_t* next,
                      auto kshalf, int dma_stage, auto dma_slot, auto flipc, auto wsumc) {
    constexpr int KS = decltype(kshalf)::value;
    constexpr bool FLIP = decltype(flipc)::value;
    constexpr bool WSUM = decltype(wsumc)::value;
    [&]<int... Mi>(std::integer_sequence<int, Mi...>) {
      ([&] {
        constexpr int m = Mi;
        constexpr int j = m / TP, i = m % TP;
        acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(pf[i], qf[j], acc[i][j], 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
        if constexpr (WSUM) {  // at the first use of a weight fragment
          if constexpr (!ACT_ON_P && j == 0) sum4(wsum[i], pf[i]);
          if constexpr (ACT_ON_P && i == 0) sum4(wsum[j], qf[j]);
        }
        if constexpr (FLIP && i == TP - 1) {
          if constexpr (!ACT_ON_P) flip(qn[j]);
          else if constexpr (j < TP) flip(pn[j]);
        }
        if constexpr (FLIP && ACT_ON_P && TP > TQ && m == NM - 1) {
#pragma unroll
          for (int r = TQ; r < TP; ++r) flip(pn[r]);
        }
        // refills: qf[j] after the last MFMA of column j, the pf after the last column
        if constexpr (i == TP - 1)
          qf[j] = *reinterpret_cast<const v4i*>(next + qa[KS] + kQBase + j * kFrag);
        if constexpr (m == NM - 1) {
#pragma unroll
          for (int r = 0; r < TP; ++r)
            pf[r] = *reinterpret_cast<const v4i*>(next + pa[KS] + r * kFrag);
        }
        // DMA instructions [first, last) of this half go behind MFMA m
        constexpr int cnt = KS == 0 ? LH : L - LH;   // instructions of this half
        constexpr int org = KS == 0 ? 0 : LH;
        constexpr int first = (m * cnt) / NM, last = ((m + 1) * cnt) / NM;
        if constexpr (last > first)
          issue_range(dma_stage, dma_slot, std::integral_constant<int, org + first>{},
                      std::integral_constant<int, org + last>{});
        __builtin_amdgcn_sched_barrier(0);
      }(), ...);
    }(std::make_integer_sequence<int, NM>{});
  };

  // The main loop is unrolled over the ring, so every LDS address in it is the sum of a
  // loop-invariant register and a constant.  R: ring slot of stage kt.
  // At the top of iteration kt both fragment sets hold stage kt.  The barrier there says: stage
  // kt+1 has landed for everybody (only the youngest stages may still be in flight), and
  // everybody has received its fragments of stage kt-1, whose slot is refilled by this
  // iteration's DMA instructions with stage kt + kStages - 1.
  static_assert(kStages >= 3, "ring: one stage being read, one landing, one in flight");
  auto stage_body = [&](int kt, auto ring, auto flipc, auto wsumc) {
    constexpr int R = decltype(ring)::value;
    constexpr int RN = (R + 1) % kStages;             // slot of stage kt + 1
    constexpr int RD = (R + kStages - 1) % kStages;   // slot of stage kt - 1 and kt + kStages - 1
    // A bare s_barrier: fragment reads still in flight here belong to stage kt, whose slot
    // stays untouched until the next barrier, so they need not be waited for.
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"((kStages - 3) * L) : "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    multiply(pf0, qf0, pf1, qf1, smem + RN * STAGE, std::integral_constant<int, 0>{},
             kt + kStages - 1, std::integral_constant<int, RD>{}, flipc, wsumc);
    multiply(pf1, qf1, pf0, qf0, smem + RN * STAGE, std::integral_constant<int, 1>{},
             kt + kStages - 1, std::integral_constant<int, RD>{}, flipc, wsumc);
  };
  auto main_loop = [&](auto flipc, auto wsumc) {
    read_frags(smem, 0, pf0, qf0);
    read_frags(smem, 1, pf1, qf1);
    if constexpr (decltype(flipc)::value) {  // the first half's fragments
      if constexpr (ACT_ON_P) { for (int i = 0; i < TP; ++i) flip(pf0[i]); }
      else { for (int j = 0; j < TQ; ++j) flip(qf0[j]); }
    }
    for (int kt0 = 0; kt0 < KT; kt0 += kStages) {
      bool done = false;
      [&]<int... R>(std::integer_sequence<int, R...>) {
        ([&] {
          if (!done) {
            if (kt0 + R < KT) stage_body(kt0 + R, std::integral_constant<int, R>{}, flipc, wsumc);
            else done = true;
          }
        }(), ...);
      }(std::make_integer_sequence<int, kStages>{});
    }
  };

  // stage 0 has landed once only the younger stages are outstanding
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"((kStages - 2) * L) : "memory");
  __syncthreads();
  HAGO_STAMP(p, 2);
  if (!CONV && p.act_xor4 != 0) main_loop(std::true_type{}, std::true_type{});
  else if (need_wsum) main_loop(std::false_type{}, std::true_type{});
  else main_loop(std::false_type{}, std::false_type{});
  HAGO_STAMP(p, 3);
  // drain the zero-fill stages before LDS is reused and before the workgroup may exit
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();

  // weight row sums: the two 32-lane halves hold the two k-halves of each row
#pragma unroll
  for (int i = 0; i < TW; ++i) {
    // remove the bias: each lane has summed 32 bytes per stage, zero fills included
    int32_t v = (int32_t)(wsum[i] - (uint32_t)KT * (32u * 128u));
    v += __shfl_xor(v, 32);
    const int ci = ACT_ON_P ? (wq * TQ + i) * 32 + frow : (wp * TP + i) * 32 + frow;
    if (sums_here && fhalf == 0) s_corr[ci] = v;
  }
  __syncthreads();
  const bool general = finish_channel_terms<NT, CH>(p, chregs, s_corr, s_mult, s_shift, s_c64);
  HAGO_STAMP(p, 4);
  if constexpr (!ACT_ON_P) {
    constexpr bool kCanStage = BQ * (BP + 16) <= kStages * STAGE && (BQ * BP / 16) % NT == 0;
    if constexpr (kCanStage) {
      if (p.out_mode == 0 && !p.acc16 && p.vec16_out && p0 + BP <= p.N && q0 + BQ <= p.M) {
        if (general)
          qgemm_epilogue_dense_staged<WP, WQ, TP, TQ, false>(p, acc, p0, q0, s_corr, s_mult, s_shift,
                                                             s_c64, smem);
        else
          qgemm_epilogue_dense_staged<WP, WQ, TP, TQ, true>(p, acc, p0, q0, s_corr, s_mult, s_shift,
                                                            s_c64, smem);
        return;
      }
    }
  }
  qgemm_epilogue<WP, WQ, TP, TQ, ACT_ON_P>(p, acc, p0, q0, s_corr, s_mult, s_shift);
}

template <int WP, int WQ, int TP, int TQ, int kStages, int OCC, bool CONV, bool ACT_ON_P>
hipError_t launch_dma_cfg(const QgemmParams& p, hipStream_t st) {
  constexpr int BP = WP * TP * 32, BQ = WQ * TQ * 32;
  constexpr int CH = ACT_ON_P ? BQ : BP;
  constexpr size_t lds = (size_t)kStages * (BP + BQ) * kBK + 1024 + 5 * CH * sizeof(int32_t);
  const int P_ext = ACT_ON_P ? p.M : p.N;
  const int Q_ext = ACT_ON_P ? p.N : p.M;
  const int64_t tiles = (int64_t)((P_ext + BP - 1) / BP) * ((Q_ext + BQ - 1) / BQ);
  auto kern = qgemm_dma_kernel<WP, WQ, TP, TQ, kStages, OCC, CONV, ACT_ON_P>;
  static bool attr_set = false;  // raising the dynamic-LDS limit is needed once per kernel
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  hipLaunchKernelGGL(kern, dim3((unsigned)tiles), dim3(64 * WP * WQ), lds, st, p);
  return hipGetLastError();
}

}  // namespace

// Requires: K % 16 == 0, K >= 16, 16-byte aligned operands, N*K and M*K below 2^31.
hipError_t launch_qdense_dma(const QgemmParams& p, int shape, hipStream_t st) {
  switch (shape) {
    case 1: return launch_dma_cfg<2, 4, 3, 2, 4, 1, false, false>(p, st);   // 192 x 256
    case 2: return launch_dma_cfg<4, 2, 1, 2, 4, 1, false, false>(p, st);   // 128 x 128
    default: return launch_dma_cfg<4, 2, 2, 4, 4, 1, false, false>(p, st);  // 256 x 256
  }
}

// Implicit-GEMM convolution over the prepacked operands (p.act: padded NHWC copy, p.wgt:
// [O][KH*KW*C] copy, p.g: geometry of the padded copy, p.K = KH*KW*C with C % 16 == 0).
// nchw_out: output [B,O,OH,OW] (activations are the P operand) else [B,OH,OW,O].
hipError_t launch_qconv_dma(const QgemmParams& p, bool nchw_out, hipStream_t st) {
  const int64_t small_m = p.M <= 256 * 128;  // fewer than ~half the CUs with 256-pixel tiles
  if (nchw_out) {  // P = pixels, Q = channels
    if (p.N <= 32) return small_m ? launch_dma_cfg<4, 1, 1, 1, 4, 2, true, true>(p, st)    // 128 x 32
                                  : launch_dma_cfg<4, 1, 2, 1, 4, 2, true, true>(p, st);   // 256 x 32
    if (p.N <= 64) return small_m ? launch_dma_cfg<4, 1, 1, 2, 4, 2, true, true>(p, st)    // 128 x 64
                                  : launch_dma_cfg<4, 1, 2, 2, 4, 2, true, true>(p, st);   // 256 x 64
    if (p.N <= 128) return small_m ? launch_dma_cfg<2, 2, 2, 2, 4, 2, true, true>(p, st)   // 128 x 128
                                   : launch_dma_cfg<4, 1, 2, 4, 4, 1, true, true>(p, st);  // 256 x 128
    return small_m ? launch_dma_cfg<2, 2, 2, 2, 4, 2, true, true>(p, st)
                   : launch_dma_cfg<4, 2, 2, 4, 4, 1, true, true>(p, st);                  // 256 x 256
  }
  // P = channels, Q = pixels
  if (p.N <= 32) return launch_dma_cfg<1, 4, 1, 2, 4, 2, true, false>(p, st);     // 32 x 256
  if (p.N <= 64) return launch_dma_cfg<1, 4, 2, 2, 4, 2, true, false>(p, st);     // 64 x 256
  if (p.N <= 128 || small_m) return launch_dma_cfg<2, 2, 2, 2, 4, 2, true, false>(p, st);  // 128 x 128
  return launch_dma_cfg<4, 2, 2, 4, 4, 1, true, false>(p, st);                    // 256 x 256
}

}  // namespace hago
