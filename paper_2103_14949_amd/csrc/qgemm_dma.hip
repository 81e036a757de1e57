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
// instruction's scalar offset, so the steady state computes no addresses and has no branches:
// stages whose refill is such a full stage run a straight-line body, the last few stages of a
// tile (K tail, zero fills) a general one.
//
// Weight row sums.  Each 32-row block of the weight tile is summed by one wavefront, which reads
// it from LDS a second time (two 16-byte reads per lane and stage), independent of the
// fragments it multiplies; summing the fragments themselves would repeat the work in every
// wavefront that holds the same weights.
#include "qgemm_common.h"

#include <type_traits>
#include <utility>

namespace hago {

namespace {

constexpr int kBK = 64;       // k-bytes per stage (default; small tiles use 128)
constexpr uint32_t kOob = 0x80000000u;  // offset beyond any tensor (sizes are < 2^31 bytes)

// Chunk permutation of an LDS row of BK bytes.  With these a fragment read (lane -> row lane % 32,
// chunk 2 h + lane / 32 for 32-k group h) runs at the full LDS rate (measured; other XOR patterns
// of the row bits run at half rate or less).  It depends on the row inside a 16-row block only.
template <int BK>
__device__ __forceinline__ int swz(int row) {
  return BK == 64 ? (row >> 2) & 3 : (row >> 1) & 7;
}

// The L DMA instructions of a stage are dealt over its nh 32-k groups: group h issues
// [dma_first(h), dma_first(h + 1)).
constexpr int dma_first(int h, int l, int nh) { return (h * l + nh - 1) / nh; }

__device__ __forceinline__ void dma16(v4i rsrc, uint32_t lds_addr, uint32_t voff) {
  // m0 = LDS byte address of the wavefront's 1 KB window; lane l lands at m0 + 16 * l
  asm volatile("s_mov_b32 m0, %0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds"
               :
               : "s"(lds_addr), "v"(voff), "s"(rsrc)
               : "memory", "m0");
}

// Same with a scalar byte offset added to every lane's address (not range checked).
__device__ __forceinline__ void dma16s(v4i rsrc, uint32_t lds_addr, uint32_t voff, uint32_t soff) {
  asm volatile("s_mov_b32 m0, %0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds"
               :
               : "s"(lds_addr), "v"(voff), "s"(rsrc), "s"(soff)
               : "memory", "m0");
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
// FLIP: uint8 activations (dense only; the convolution's copy is already flipped).
// UNIFORM: K (and the channel count of a convolution) is a multiple of 64, so every stage has one
// k offset for all lanes, which travels in the DMA instruction's scalar offset: the main loop
// then computes no addresses and has no branches.  Otherwise every DMA instruction gets per-lane
// offsets (K tail, stages that straddle filter taps).
// BK: k-bytes per stage, 64 or 128.  With 128 a DMA instruction fetches whole 128-byte lines (8 rows)
// and a stage has four 32-k groups instead of two, i.e. half as many barriers per k.
template <int WP, int WQ, int TP, int TQ, int kStages, int OCC, bool CONV, bool ACT_ON_P, bool FLIP,
          bool UNIFORM, int BK = kBK>
__global__ __launch_bounds__(64 * WP * WQ, OCC) void qgemm_dma_kernel(QgemmParams p) {
  static_assert(!FLIP || (!CONV && !ACT_ON_P), "only dense layers flip, and keep activations on Q");
  constexpr bool kPixPerm = CONV && ACT_ON_P;
  static_assert(BK == 64 || BK == 128, "stage width");
  constexpr int NH = BK / 32;       // 32-k groups per stage
  constexpr int RPI = 1024 / BK;    // rows per DMA instruction
  constexpr int CPR = BK / 16;      // 16-byte chunks per row
  HAGO_STAMP(p, 7);
  constexpr int NW = WP * WQ;          // wavefronts
  constexpr int NT = 64 * NW;
  constexpr int BP = WP * TP * 32;
  constexpr int BQ = WQ * TQ * 32;
  constexpr int STAGE = (BP + BQ) * BK;
  constexpr int GP = BP / RPI, GQ = BQ / RPI;  // row groups (one DMA instruction each)
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
  int32_t* s_shm1 = reinterpret_cast<int32_t*>(s_c64 + CH);  // shift - 1

  const int t = threadIdx.x;
  const int lane = t & 63;
  const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
  const int wp = wave % WP;
  const int wq = wave / WP;

  const int P_ext = ACT_ON_P ? p.M : p.N;
  const int Q_ext = ACT_ON_P ? p.N : p.M;
  const int tiles_p = (P_ext + BP - 1) / BP;
  const int tile = xcd_remap(blockIdx.x, gridDim.x);
  // Tiles are numbered panel by panel (kPanel tiles wide along P, all of Q), row by row inside
  // a panel: the tiles that run on an XCD at the same time then form a compact block and share
  // both operands' rows in its L2.
  constexpr int kPanel = 8;
  int tile_p, tile_q;
  {
    const int tiles_q = (Q_ext + BQ - 1) / BQ;
    const int full = tiles_p / kPanel;
    const int per_panel = kPanel * tiles_q;
    int r = tile, w = kPanel, base = 0;
    if (tile >= full * per_panel) {
      r = tile - full * per_panel;
      w = tiles_p - full * kPanel;
      base = full * kPanel;
    } else {
      const int pn = tile / per_panel;
      r = tile - pn * per_panel;
      base = pn * kPanel;
    }
    tile_q = r / w;
    tile_p = base + (r - tile_q * w);
  }
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
  // DMA slot d of wavefront w is group w + NW * d of the stage (P groups first, then Q groups),
  // whose 1 KB window lies (w + NW * d) * 1024 bytes into the stage.  When the wavefront count
  // divides both group counts (kEven) the operand of a slot is the same in every wavefront and
  // every slot has a group; otherwise both are per-wavefront values.
  constexpr bool kEven = (GP % NW == 0) && (G % NW == 0);
  uint32_t voff[L];  // row offset + chunk: the per-lane part of a full stage's address
  bool slot_real[L]; // false: the slot has no group, it fetches zeros into the spare window
  bool slot_q[L];
  const int lrow = lane / CPR;  // row inside a group
  const int lslot = lane % CPR;  // physical 16-byte slot
  const uint32_t spare = lds0 + (uint32_t)kStages * STAGE;
  const uint32_t wave_lds = lds0 + (uint32_t)wave * 1024u;
  // The swizzle depends on the row inside a 16-row block only; an 8-row group is the half of
  // such a block that its parity says, and every group of a wavefront has the wavefront's
  // parity, so the logical chunk is the same in every slot.
  static_assert(RPI == 16 || NW % 2 == 0, "group parity must not depend on the slot");
  const int lck = (lslot ^ swz<BK>((RPI == 16 ? 0 : (wave & 1) * 8) + lrow)) * 16;  // chunk (bytes) inside a stage
#pragma unroll
  for (int d = 0; d < L; ++d) {
    const int grp = wave + NW * d;
    const bool isq = kEven ? (d >= GP / NW) : (grp >= GP);
    int rt = (isq ? grp - GP : grp) * RPI + lrow;  // row inside its tile
    // NCHW convolution: the pixels of a 32-row block are placed so that a lane's accumulator
    // registers are 16 consecutive pixels (one 16-byte store per channel in the epilogue)
    if constexpr (kPixPerm) {
      if (!isq) rt = (rt & ~31) | pix_perm(rt & 31);
    }
    slot_q[d] = isq;
    slot_real[d] = kEven || grp < G;
    uint32_t off = kOob;
    if (slot_real[d]) off = row_offset((isq ? q0 : p0) + rt, isq ? !ACT_ON_P : ACT_ON_P);
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
  const int KT = (p.K + BK - 1) / BK;
  const v4i rs_null = {rs_w.x, rs_w.y, 0, rs_w.w};  // zero records: every access reads zeros

  // DMA slot d (0 .. L-1) of stage stage_idx into ring slot RS; d and RS are compile-time
  // constants at every call site.  UNIFORM: dp / dq are the stage's descriptors (the null
  // descriptor for stages beyond K, which only keep the count of outstanding loads uniform),
  // soff_w / soff_a its scalar k offsets for weight and activation slots.
  auto issue_one = [&](int stage_idx, const v4i& dp, const v4i& dq, uint32_t soff_w, uint32_t soff_a,
                       auto rsconst, auto dconst) {
    constexpr int d = decltype(dconst)::value;
    constexpr int RS = decltype(rsconst)::value;
    const bool isq = kEven ? (d >= GP / NW) : slot_q[d];
    const bool is_act = isq ? !ACT_ON_P : ACT_ON_P;
    const uint32_t dst =
        slot_real[d] ? wave_lds + (uint32_t)(NW * d * 1024 + RS * STAGE) : spare;
    if constexpr (UNIFORM) {
      dma16s(isq ? dq : dp, dst, voff[d], is_act ? soff_a : soff_w);
    } else {
      const int k0 = stage_idx * BK;
      uint32_t o = voff[d] - (uint32_t)lck + k_offset(k0 + lck, is_act);
      if (voff[d] == kOob || k0 + lck >= p.K) o = kOob;
      dma16(isq ? rs_q : rs_p, dst, o);
    }
  };
  auto issue_range = [&](int stage_idx, const v4i& dp, const v4i& dq, uint32_t soff_w,
                         uint32_t soff_a, auto rsconst, auto lo, auto hi) {
    constexpr int kLo = decltype(lo)::value, kHi = decltype(hi)::value;
    [&]<int... I>(std::integer_sequence<int, I...>) {
      (issue_one(stage_idx, dp, dq, soff_w, soff_a, rsconst, std::integral_constant<int, kLo + I>{}),
       ...);
    }(std::make_integer_sequence<int, kHi - kLo>{});
  };
  // descriptors and scalar offsets of a stage (UNIFORM)
  struct StageArgs { v4i dp, dq; uint32_t soff_w, soff_a; };
  auto stage_args = [&](int stage_idx) {
    StageArgs a{rs_p, rs_q, 0u, 0u};
    if constexpr (UNIFORM) {
      const bool valid = stage_idx < KT;
      a.dp = valid ? rs_p : rs_null;
      a.dq = valid ? rs_q : rs_null;
      a.soff_w = (uint32_t)__builtin_amdgcn_readfirstlane((int)k_offset(stage_idx * BK, false));
      a.soff_a = (uint32_t)__builtin_amdgcn_readfirstlane((int)k_offset(stage_idx * BK, true));
    }
    return a;
  };
  using IC0 = std::integral_constant<int, 0>;
  using ICL = std::integral_constant<int, L>;

  HAGO_STAMP(p, 0);
  // prologue: stages 0 .. kStages-2 go out before anything else is set up (stages beyond K are
  // all-zero fills, which keeps the number of outstanding loads uniform)
  [&]<int... S>(std::integer_sequence<int, S...>) {
    ([&] {
      const StageArgs a = stage_args(S);
      issue_range(S, a.dp, a.dq, a.soff_w, a.soff_a, std::integral_constant<int, S>{}, IC0{}, ICL{});
    }(), ...);
  }(std::make_integer_sequence<int, kStages - 1>{});
  HAGO_STAMP(p, 1);
  __builtin_amdgcn_sched_barrier(0);
  ChannelRegs<NT, CH> chregs;
  load_channel_regs<NT, CH>(p, w0, chregs);

  v16i acc[TP][TQ];
#pragma unroll
  for (int i = 0; i < TP; ++i)
#pragma unroll
    for (int j = 0; j < TQ; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0;
  // Weight tile rows are summed in 32-row blocks, block w + NW * n by wavefront w, one 32-k group
  // (one 16-byte read per lane) at a time.  With at least two wavefronts per block a block is
  // shared by two, which take the even and the odd 32-k groups.
  constexpr int WBLK = (ACT_ON_P ? BQ : BP) / 32;
  constexpr bool kSplitSum = NW >= 2 * WBLK;
  constexpr int NSB = (WBLK + NW - 1) / NW;
  constexpr int NSG = kSplitSum ? NH / 2 : NH;  // 32-k groups a wavefront sums per stage and block
  uint32_t wsum[NSB];  // biased: every byte counts as w + 128
#pragma unroll
  for (int i = 0; i < NSB; ++i) wsum[i] = 0;


  const int frow = lane & 31;
  const int fhalf = lane >> 5;
  // Fragment addresses inside a stage (bytes).  Fragment i of a wavefront lies i * 32 rows
  // after fragment 0 and has the same swizzle (it depends on the row inside a 16-row block
  // only), so one register per operand and 32-k group serves every fragment, ring slot and
  // operand region through constant offsets.
  int pa[NH], qa[NH];
#pragma unroll
  for (int h = 0; h < NH; ++h) {
    const int chunk = ((h * 2 + fhalf) ^ swz<BK>(frow & 15)) * 16;
    pa[h] = (wp * TP * 32 + frow) * BK + chunk;
    qa[h] = (wq * TQ * 32 + frow) * BK + chunk;
  }
  constexpr int kFrag = 32 * BK;     // bytes between consecutive fragments of a wavefront
  constexpr int kQBase = BP * BK;    // the Q rows follow the P rows inside a stage
  // weight row block wave + NW * n, read like a fragment; wavefronts without such a block read
  // the last one again (and do not store their sums).  Entry g is the g-th 32-k group this
  // wavefront sums.
  int sa[NSB][NSG];
#pragma unroll
  for (int n = 0; n < NSB; ++n) {
    int blk = wave + NW * n < WBLK ? wave + NW * n : WBLK - 1;
    if constexpr (kSplitSum) blk = wave % WBLK;
#pragma unroll
    for (int g = 0; g < NSG; ++g) {
      const int h = kSplitSum ? 2 * g + ((wave / WBLK) & 1) : g;
      sa[n][g] = (ACT_ON_P ? kQBase : 0) + (blk * 32 + frow) * BK +
                 ((h * 2 + fhalf) ^ swz<BK>(frow & 15)) * 16;
    }
  }

  // One fragment set per 32-k group of a stage.  A fragment register is refilled with the NEXT
  // stage's data right after the last MFMA that reads it, a whole stage of MFMAs before it is
  // needed again, so LDS latency (and the burst of reads after a barrier) stays hidden.
  v4i pf[NH][TP], qf[NH][TQ];
  // Flipping the sign bit of uint8 activation fragments and summing weight rows are vector
  // instructions dealt out one or two per MFMA: the flips are applied to the NEXT group's
  // fragment set (read a stage earlier); the rows to sum (of the next stage, like the refills)
  // are read early in a group and summed later in it (split sums: read in an even group, summed
  // in the odd one after it).
  constexpr int NM = TP * TQ;  // MFMAs per 32-k group
  constexpr int NFL = TQ * 4;  // dwords to flip per group (dense: the activations are on Q)
  auto flip1 = [&](v4i& f, int u) {
    // in place, so that no copy of the fragment is made
    int x = f[u];
    asm volatile("v_xor_b32 %0, %1, %0" : "+v"(x) : "s"(p.act_xor4));
    f[u] = x;
  };
  auto sum1 = [&](uint32_t& a, int f) {
    // bytes + 128 each (v_dot4 would stall the matrix pipe, v_sad_u8 does not)
    a = __builtin_amdgcn_sad_u8((uint32_t)f ^ 0x80808080u, 0u, a);
  };
  v4i sd[NSB];  // rows being summed
  // One 32-k group H of a stage: multiply its set; behind the MFMAs go the weight sums, the flips
  // of the next group's activation fragments, the refills of this set from the next stage (at
  // `next`), and this group's share of a stage's DMA instructions (so the memory pipe is fed a few
  // instructions at a time).
  auto multiply = [&](const uint8_t* next, auto hconst, int dma_stage, const StageArgs& sa_,
                      auto dma_slot) {
    constexpr int H = decltype(hconst)::value;
    constexpr int HN = (H + 1) % NH;  // the set multiplied next
    [&]<int... Mi>(std::integer_sequence<int, Mi...>) {
      ([&] {
        constexpr int m = Mi;
        constexpr int j = m / TP, i = m % TP;
        acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(pf[H][i], qf[H][j], acc[i][j], 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
        {
          constexpr bool kRead = !kSplitSum || H % 2 == 0;
          constexpr bool kSum = !kSplitSum || H % 2 == 1;
          constexpr int g = kSplitSum ? H / 2 : H;
          if constexpr (kRead && m < NSB) sd[m] = *reinterpret_cast<const v4i*>(next + sa[m][g]);
          constexpr int lo = NM > NSB * 4 ? NM - NSB * 4 : (NM > 1 ? 1 : 0);
          if constexpr (kSum) {
#pragma unroll
            for (int e = 0; e < NSB * 4; ++e) {
              const int at = lo + (e * (NM - lo)) / (NSB * 4);
              if (at == m) sum1(wsum[e / 4], sd[e / 4][e % 4]);
            }
          }
        }
        if constexpr (FLIP) {
          // dealt over the later MFMAs of the group
          constexpr int lo = NM / 4;
#pragma unroll
          for (int e = 0; e < NFL; ++e) {
            const int at = lo + (e * (NM - lo)) / NFL;
            if (at == m) flip1(qf[HN][e / 4], e % 4);
          }
        }
        // refills: qf[j] after the last MFMA of column j, pf[i] after its MFMA of the last column
        if constexpr (i == TP - 1)
          qf[H][j] = *reinterpret_cast<const v4i*>(next + qa[H] + kQBase + j * kFrag);
        if constexpr (j == TQ - 1)
          pf[H][i] = *reinterpret_cast<const v4i*>(next + pa[H] + i * kFrag);
        // DMA instructions [first, last) of this group go behind MFMA m
        constexpr int org = dma_first(H, L, NH);
        constexpr int cnt = dma_first(H + 1, L, NH) - org;
        constexpr int first = (m * cnt) / NM, last = ((m + 1) * cnt) / NM;
        if constexpr (last > first)
          issue_range(dma_stage, sa_.dp, sa_.dq, sa_.soff_w, sa_.soff_a, dma_slot,
                      std::integral_constant<int, org + first>{},
                      std::integral_constant<int, org + last>{});
        __builtin_amdgcn_sched_barrier(0);
      }(), ...);
    }(std::make_integer_sequence<int, NM>{});
  };

  // The main loop is unrolled over the ring, so every LDS address in it is the sum of a
  // loop-invariant register and a constant.  R: ring slot of stage kt.
  // At the top of iteration kt every fragment set holds stage kt.  The barrier there says: stage
  // kt+1 has landed for everybody (only the youngest stages may still be in flight), and
  // everybody has received its fragments of stage kt-1, whose slot is refilled by this
  // iteration's DMA instructions with stage kt + kStages - 1.
  static_assert(kStages >= 3, "ring: one stage being read, one landing, one in flight");
  auto stage_body = [&](int kt, auto ring) {
    constexpr int R = decltype(ring)::value;
    constexpr int RN = (R + 1) % kStages;             // slot of stage kt + 1
    constexpr int RD = (R + kStages - 1) % kStages;   // slot of stage kt - 1 and kt + kStages - 1
    const int ds = kt + kStages - 1;
    const StageArgs a = stage_args(ds);
    // A bare s_barrier: fragment reads still in flight here belong to stage kt, whose slot
    // stays untouched until the next barrier, so they need not be waited for.
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"((kStages - 3) * L) : "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    [&]<int... Hi>(std::integer_sequence<int, Hi...>) {
      (multiply(smem + RN * STAGE, std::integral_constant<int, Hi>{}, ds, a,
                std::integral_constant<int, RD>{}), ...);
    }(std::make_integer_sequence<int, NH>{});
  };
  auto main_loop = [&] {
#pragma unroll
    for (int h = 0; h < NH; ++h) {
#pragma unroll
      for (int i = 0; i < TP; ++i)
        pf[h][i] = *reinterpret_cast<const v4i*>(smem + pa[h] + i * kFrag);
#pragma unroll
      for (int j = 0; j < TQ; ++j)
        qf[h][j] = *reinterpret_cast<const v4i*>(smem + qa[h] + kQBase + j * kFrag);
    }
    if constexpr (FLIP) {  // the first group's fragments
#pragma unroll
      for (int j = 0; j < TQ; ++j)
#pragma unroll
        for (int u = 0; u < 4; ++u) flip1(qf[0][j], u);
    }
    // stage 0's rows (the loop sums stage kt + 1)
#pragma unroll
    for (int n = 0; n < NSB; ++n)
#pragma unroll
      for (int g = 0; g < NSG; ++g) {
        const v4i r = *reinterpret_cast<const v4i*>(smem + sa[n][g]);
#pragma unroll
        for (int u = 0; u < 4; ++u) sum1(wsum[n], r[u]);
      }
    for (int kt0 = 0; kt0 < KT; kt0 += kStages) {
      bool done = false;
      [&]<int... R>(std::integer_sequence<int, R...>) {
        ([&] {
          if (!done) {
            if (kt0 + R < KT) stage_body(kt0 + R, std::integral_constant<int, R>{});
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
  main_loop();
  HAGO_STAMP(p, 3);
  // drain the zero-fill stages before LDS is reused and before the workgroup may exit (the
  // barriers of the channel terms below come before anything is written to the ring's memory)
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");

  // weight row sums: the two 32-lane halves hold the two halves of each 32-k group of a row.
  // Each lane has summed 16 bytes per 32-k group it covers (biased by 128 each) per stage for
  // stages 0 .. KT: the loop's last iteration added the first zero-fill stage, whose bytes are
  // all zero.  Split blocks: the second k-half's sums wait in s_mult until the terms are formed.
#pragma unroll
  for (int n = 0; n < NSB; ++n) {
    int32_t v = (int32_t)(wsum[n] - (uint32_t)(KT + 1) * ((uint32_t)NSG * 16u * 128u));
    v += __shfl_xor(v, 32);
    if constexpr (kSplitSum) {
      const int part = wave / WBLK;
      if (part < 2 && fhalf == 0) (part == 0 ? s_corr : s_mult)[(wave % WBLK) * 32 + frow] = v;
    } else {
      const int blk = wave + NW * n;
      if (blk < WBLK && fhalf == 0) s_corr[blk * 32 + frow] = v;
    }
  }
  __syncthreads();
  const bool general = finish_channel_terms<NT, CH>(p, chregs, s_corr, s_mult, s_shift, s_c64,
                                                    kSplitSum ? s_mult : nullptr, s_shm1);
  HAGO_STAMP(p, 4);
  if constexpr (!ACT_ON_P) {
    constexpr bool kCanStage = BQ * (BP + 16) <= kStages * STAGE && (BQ * BP / 16) % NT == 0;
    if constexpr (kCanStage) {
      if (p.out_mode == 0 && !p.acc_wrap_shift && p.vec16_out && !p.rs.half_away) {
        if (general)
          qgemm_epilogue_dense_staged<WP, WQ, TP, TQ, false>(p, acc, p0, q0, s_corr, s_mult, s_shift,
                                                             s_c64, s_shm1, smem);
        else
          qgemm_epilogue_dense_staged<WP, WQ, TP, TQ, true>(p, acc, p0, q0, s_corr, s_mult, s_shift,
                                                            s_c64, s_shm1, smem);
        return;
      }
    }
  }
  qgemm_epilogue<WP, WQ, TP, TQ, ACT_ON_P, kPixPerm>(p, acc, p0, q0, s_corr, s_mult, s_shift);
}

template <int WP, int WQ, int TP, int TQ, int kStages, int OCC, bool CONV, bool ACT_ON_P, bool FLIP,
          bool UNIFORM, int BK>
hipError_t launch_dma_kernel(const QgemmParams& p, hipStream_t st) {
  constexpr int BP = WP * TP * 32, BQ = WQ * TQ * 32;
  constexpr int CH = ACT_ON_P ? BQ : BP;
  constexpr size_t lds = (size_t)kStages * (BP + BQ) * BK + 1024 + 6 * CH * sizeof(int32_t);
  const int P_ext = ACT_ON_P ? p.M : p.N;
  const int Q_ext = ACT_ON_P ? p.N : p.M;
  const int64_t tiles = (int64_t)((P_ext + BP - 1) / BP) * ((Q_ext + BQ - 1) / BQ);
  auto kern = qgemm_dma_kernel<WP, WQ, TP, TQ, kStages, OCC, CONV, ACT_ON_P, FLIP, UNIFORM, BK>;
  static std::atomic<uint64_t> attr_set{0};  // per kernel: the devices whose dynamic-LDS limit is raised
  hipError_t e = raise_lds_limit(reinterpret_cast<const void*>(kern), (int)lds, attr_set);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(kern, dim3((unsigned)tiles), dim3(64 * WP * WQ), lds, st, p);
  return hipGetLastError();
}

// Picks the kernel variant: uint8 dense activations are flipped in the loop; shapes whose
// stages are uniform take the scalar-offset loop.
template <int WP, int WQ, int TP, int TQ, int kStages, int OCC, bool CONV, bool ACT_ON_P, int BK = kBK>
hipError_t launch_dma_cfg(const QgemmParams& p, hipStream_t st) {
  const bool uniform = p.K % BK == 0 && (!CONV || p.g.C % BK == 0);
  if constexpr (!CONV) {
    if (p.act_xor4 != 0)
      return uniform
                 ? launch_dma_kernel<WP, WQ, TP, TQ, kStages, OCC, CONV, ACT_ON_P, true, true, BK>(p, st)
                 : launch_dma_kernel<WP, WQ, TP, TQ, kStages, OCC, CONV, ACT_ON_P, true, false, BK>(p, st);
  }
  return uniform
             ? launch_dma_kernel<WP, WQ, TP, TQ, kStages, OCC, CONV, ACT_ON_P, false, true, BK>(p, st)
             : launch_dma_kernel<WP, WQ, TP, TQ, kStages, OCC, CONV, ACT_ON_P, false, false, BK>(p, st);
}

}  // namespace

// Requires: K % 16 == 0, K >= 16, 16-byte aligned operands, N*K and M*K below 2^31.
hipError_t launch_qdense_dma(const QgemmParams& p, int shape, hipStream_t st) {
  switch (shape) {
    case 1: return launch_dma_cfg<2, 4, 3, 2, 4, 1, false, false>(p, st);   // 192 x 256
    case 2: return launch_dma_cfg<2, 4, 2, 1, 4, 1, false, false, 128>(p, st);   // 128 x 128, 128-byte stages
    case 3: return launch_dma_cfg<2, 4, 2, 1, 4, 1, false, false>(p, st);   // 128 x 128, 64-byte stages
    case 4: return launch_dma_cfg<2, 2, 1, 1, 4, 2, false, false>(p, st);   // 64 x 64: few rows
    default: return launch_dma_cfg<2, 4, 4, 2, 4, 1, false, false>(p, st);  // 256 x 256
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
    if (p.N <= 64) {
      if (p.M <= 64 * 128) return launch_dma_cfg<2, 2, 1, 1, 4, 2, true, true>(p, st);  // 64 x 64: few pixels
      // (256 x 64 tiles were slower at every size: 36.7 vs 31.7 us for 64 -> 64 at 56 x 56, batch 64)
      return launch_dma_cfg<4, 1, 1, 2, 4, 2, true, true>(p, st);             // 128 x 64
    }
    // few pixels: 64 x 64 tiles when 128 x 128 ones would leave most of the chip idle
    const int64_t tiles128 = (int64_t)((p.M + 127) / 128) * ((p.N + 127) / 128);
    if (small_m && p.N > 64 && tiles128 < 256) return launch_dma_cfg<2, 2, 1, 1, 4, 2, true, true>(p, st);  // 64 x 64
    // (256 x 128 tiles were slower: 27.4 vs 24.6 us for 128 -> 128 at 28 x 28, batch 64)
    if (p.N <= 128) return launch_dma_cfg<2, 2, 2, 2, 4, 2, true, true>(p, st);            // 128 x 128
    return small_m ? launch_dma_cfg<2, 2, 2, 2, 4, 2, true, true>(p, st)
                   : launch_dma_cfg<4, 2, 2, 4, 4, 1, true, true>(p, st);                  // 256 x 256
  }
  // P = channels, Q = pixels
  if (p.N <= 32) return launch_dma_cfg<1, 4, 1, 2, 4, 2, true, false>(p, st);     // 32 x 256
  if (p.N <= 64) {
    if (p.M <= 64 * 128) return launch_dma_cfg<2, 2, 1, 1, 4, 2, true, false>(p, st);  // 64 x 64: few pixels
    // (64 x 256 tiles were slower: 37.9 vs 31.6 us for 64 -> 64 at 56 x 56, batch 64)
    return launch_dma_cfg<1, 4, 2, 1, 4, 2, true, false>(p, st);                  // 64 x 128
  }
  if (p.N <= 128 || small_m) return launch_dma_cfg<2, 2, 2, 2, 4, 2, true, false>(p, st);  // 128 x 128
  return launch_dma_cfg<4, 2, 2, 4, 4, 1, true, false>(p, st);                    // 256 x 256
}

}  // namespace hago
