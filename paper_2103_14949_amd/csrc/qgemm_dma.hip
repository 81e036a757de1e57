// Dense int8 GEMM, fast path: operands stream from global memory straight
// into LDS (buffer_load ... lds, 16 bytes per lane), four 64-byte k-stages
// deep, so no vector registers and no LDS-write instructions are spent on
// staging and three stages of loads are always in flight behind the one
// being multiplied.
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
// the weight fragments with v_dot4 (see qgemm.hip for the identity).
//
// Synchronisation per stage, placed between the two 32-k halves of the stage
// that is being multiplied: s_waitcnt vmcnt(2*L) (L = DMA instructions per
// wavefront per stage; two younger stages may stay in flight), one barrier
// (everybody's part of the next stage has landed and everybody has taken its
// last fragments of the current one), then the current buffer is refilled with
// the stage four ahead.
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

  // Per-lane global offset of the row this lane fetches in DMA instruction s (without the k
  // part), and the logical chunk (in bytes) it fetches inside a stage.
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
  uint32_t off[L];   // row offset of slot d
  int lck[L];        // logical chunk (bytes) inside a stage
  int ldst[L];       // LDS byte offset of the slot's 1 KB window inside a stage (< 0: spare)
  bool slot_q[L], slot_act[L];
  const int lrow = lane >> 2;  // row inside a 16-row group
  const int lslot = lane & 3;  // physical 16-byte slot
#pragma unroll
  for (int d = 0; d < L; ++d) {
    const int grp = wave + NW * d;
    const bool isq = grp >= GP;
    const int rt = (isq ? grp - GP : grp) * 16 + lrow;  // row inside its tile
    slot_q[d] = isq;
    slot_act[d] = isq ? !ACT_ON_P : ACT_ON_P;
    lck[d] = (lslot ^ swz4(rt)) * 16;
    if (grp < G) {
      off[d] = row_offset((isq ? q0 : p0) + rt, slot_act[d]);
      ldst[d] = (isq ? BP * kBK + (grp - GP) * 1024 : grp * 1024);  // wavefront-uniform
    } else {
      off[d] = kOob;
      ldst[d] = -1;
    }
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

  // DMA instruction d (0 .. L-1) of a stage: the first LP fill the P tile, the rest the Q tile.  d is a compile-time constant at every call site.
  auto issue_one = [&](int stage_idx, auto dconst) {
    constexpr int d = decltype(dconst)::value;
    const int k0 = stage_idx * kBK;
    const uint32_t base = lds0 + (uint32_t)(stage_idx % kStages) * STAGE;
    const bool tail = k0 + kBK > p.K;  // uniform: some chunks of this stage lie beyond K
    uint32_t o = off[d] + k_offset(k0 + lck[d], slot_act[d]);
    if (tail && k0 + lck[d] >= p.K) o = kOob;
    const v4i rs = slot_q[d] ? rs_q : rs_p;
    const uint32_t dst = ldst[d] >= 0 ? base + (uint32_t)ldst[d] : lds0 + (uint32_t)kStages * STAGE;
    dma16(rs, (uint32_t)__builtin_amdgcn_readfirstlane((int)dst), o);
  };
  auto issue_range = [&](int stage_idx, auto lo, auto hi) {
    constexpr int kLo = decltype(lo)::value, kHi = decltype(hi)::value;
    [&]<int... I>(std::integer_sequence<int, I...>) {
      (issue_one(stage_idx, std::integral_constant<int, kLo + I>{}), ...);
    }(std::make_integer_sequence<int, kHi - kLo>{});
  };
  constexpr int LH = (L + 1) / 2;  // a stage is issued in two parts (LH and L - LH instructions),
                                  // spread over two MFMA groups
  using IC0 = std::integral_constant<int, 0>;
  using ICH = std::integral_constant<int, LH>;
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
  int32_t wsum[TW];
#pragma unroll
  for (int i = 0; i < TW; ++i) wsum[i] = 0;

  const int KT = (p.K + kBK - 1) / kBK;
  // prologue: stages 0 .. kStages-1 (stages beyond K are all-zero fills, which keeps the
  // number of outstanding loads uniform)
#pragma unroll
  for (int s = 0; s < kStages - 1; ++s) issue_range(s, IC0{}, ICL{});
  issue_range(kStages - 1, IC0{}, ICH{});
  HAGO_STAMP(p, 1);

  const int frow = lane & 31;
  const int fhalf = lane >> 5;
  // only one wavefront per weight fragment row needs to sum it
  const bool sums_here = ACT_ON_P ? (wp == 0) : (wq == 0);
#ifdef HAGO_PHASE_TIMING
  const int x4 = (p.dbg_skip & 4) ? 0 : (int)p.act_xor4;
  const bool need_wsum = (p.corr_coef != 0) && sums_here && !(p.dbg_skip & 4);
#else
  const int x4 = (int)p.act_xor4;  // 0 in conv mode: the prepacked copy is already flipped
  const bool need_wsum = (p.corr_coef != 0) && sums_here;
#endif
  // fragment addresses inside a stage (bytes)
  int pa[TP][2], qa[TQ][2];
#pragma unroll
  for (int i = 0; i < TP; ++i) {
    const int row = (wp * TP + i) * 32 + frow;
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) pa[i][ks] = row * kBK + (((ks * 2 + fhalf) ^ swz4(row)) * 16);
  }
#pragma unroll
  for (int j = 0; j < TQ; ++j) {
    const int row = (wq * TQ + j) * 32 + frow;
#pragma unroll
    for (int ks = 0; ks < 2; ++ks)
      qa[j][ks] = BP * kBK + row * kBK + (((ks * 2 + fhalf) ^ swz4(row)) * 16);
  }

  // Fragment sets for the two 32-k halves of a stage.  While the MFMAs of one half run, the
  // fragments of the next half are already being read, and the stage barrier sits between the
  // two MFMA groups so that the matrix pipe has work queued while wavefronts wait on it.
  v4i pf0[TP], qf0[TQ], pf1[TP], qf1[TQ];
  auto read_frags = [&](const uint8_t* base, int ks, v4i (&pf)[TP], v4i (&qf)[TQ]) {
#pragma unroll
    for (int i = 0; i < TP; ++i) pf[i] = *reinterpret_cast<const v4i*>(base + pa[i][ks]);
#pragma unroll
    for (int j = 0; j < TQ; ++j) qf[j] = *reinterpret_cast<const v4i*>(base + qa[j][ks]);
  };
  // One 32-k half: per column j of the wavefront tile, flip the activation fragment, multiply it
  // with the TP weight fragments, and (HALF = 0 / 1) drop one of the stage's DMA instructions
  // behind some of the columns, so that the eight wavefronts feed the memory pipe a few
  // instructions at a time instead of all at once after the barrier.
  auto multiply = [&](v4i (&pf)[TP], v4i (&qf)[TQ], int dma_stage, auto half) {
    constexpr int kHalf = decltype(half)::value;
    if (need_wsum) {
#pragma unroll
      for (int i = 0; i < TW; ++i) {
        const v4i& f = ACT_ON_P ? qf[i < TQ ? i : 0] : pf[i < TP ? i : 0];
        wsum[i] = __builtin_amdgcn_sdot4(f.x, 0x01010101, wsum[i], false);
        wsum[i] = __builtin_amdgcn_sdot4(f.y, 0x01010101, wsum[i], false);
        wsum[i] = __builtin_amdgcn_sdot4(f.z, 0x01010101, wsum[i], false);
        wsum[i] = __builtin_amdgcn_sdot4(f.w, 0x01010101, wsum[i], false);
      }
    }
    if constexpr (ACT_ON_P && !CONV) {
#pragma unroll
      for (int i = 0; i < TP; ++i) pf[i] = v4i{pf[i].x ^ x4, pf[i].y ^ x4, pf[i].z ^ x4, pf[i].w ^ x4};
    }
    [&]<int... J>(std::integer_sequence<int, J...>) {
      ([&] {
        constexpr int j = J;
        if constexpr (!ACT_ON_P && !CONV)
          qf[j] = v4i{qf[j].x ^ x4, qf[j].y ^ x4, qf[j].z ^ x4, qf[j].w ^ x4};
#pragma unroll
        for (int i = 0; i < TP; ++i)
          acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(pf[i], qf[j], acc[i][j], 0, 0, 0);
        // DMA instructions [first, last) of this half go behind column j
        constexpr int cnt = kHalf == 0 ? LH : L - LH;   // instructions of this part
        constexpr int org = kHalf == 0 ? 0 : LH;
        constexpr int first = (j * cnt) / TQ, last = ((j + 1) * cnt) / TQ;
        if constexpr (last > first) {
#ifdef HAGO_PHASE_TIMING
          if (!(p.dbg_skip & 1))
#endif
          issue_range(dma_stage, std::integral_constant<int, org + first>{},
                      std::integral_constant<int, org + last>{});
        }
      }(), ...);
    }(std::make_integer_sequence<int, TQ>{});
  };

  // stage 0 has landed once at most the younger loads (stages 1, 2 and half of 3) are outstanding
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"((kStages - 2) * L + LH) : "memory");
  __syncthreads();
  HAGO_STAMP(p, 2);
  read_frags(smem, 0, pf0, qf0);
  for (int kt = 0; kt < KT; ++kt) {
    const uint8_t* base = smem + (kt % kStages) * STAGE;
    const uint8_t* next = smem + ((kt + 1) % kStages) * STAGE;
#ifdef HAGO_PHASE_TIMING
    if (!(p.dbg_skip & 2))
#endif
    read_frags(base, 1, pf1, qf1);
    __builtin_amdgcn_sched_barrier(0);
    multiply(pf0, qf0, kt + kStages - 1, std::integral_constant<int, 1>{});
    __builtin_amdgcn_sched_barrier(0);
    // stage kt+1 has landed once only stages kt+2, kt+3 are outstanding; after the barrier
    // every wavefront also holds its last fragments of stage kt, so that buffer can be refilled
#ifdef HAGO_PHASE_TIMING
    if (!(p.dbg_skip & 8)) {
#endif
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"((kStages - 2) * L) : "memory");
    __syncthreads();
#ifdef HAGO_PHASE_TIMING
    }
#endif
#ifdef HAGO_PHASE_TIMING
    if (!(p.dbg_skip & 2))
#endif
    read_frags(next, 0, pf0, qf0);
    __builtin_amdgcn_sched_barrier(0);
    multiply(pf1, qf1, kt + kStages, std::integral_constant<int, 0>{});
    __builtin_amdgcn_sched_barrier(0);
  }
  HAGO_STAMP(p, 3);
  // drain the zero-fill stages before LDS is reused and before the workgroup may exit
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();

  // weight row sums: the two 32-lane halves hold the two k-halves of each row
#pragma unroll
  for (int i = 0; i < TW; ++i) {
    int32_t v = wsum[i];
    v += __shfl_xor(v, 32);
    const int ci = ACT_ON_P ? (wq * TQ + i) * 32 + frow : (wp * TP + i) * 32 + frow;
    if (sums_here && fhalf == 0) s_corr[ci] = v;
  }
  __syncthreads();
  const bool any_sh0 = finish_channel_terms<NT, CH>(p, chregs, s_corr, s_mult, s_shift);
  HAGO_STAMP(p, 4);
  if constexpr (!ACT_ON_P) {
    constexpr bool kCanStage = ((BP / 16) & (BP / 16 - 1)) == 0 && BQ * BP <= kStages * STAGE &&
                               (BQ * BP / 16) % NT == 0;
    if constexpr (kCanStage) {
      if (p.out_mode == 0 && !p.acc16 && p.vec16_out && p0 + BP <= p.N && q0 + BQ <= p.M) {
        if (any_sh0)
          qgemm_epilogue_dense_staged<WP, WQ, TP, TQ, false>(p, acc, p0, q0, s_corr, s_mult, s_shift, smem);
        else
          qgemm_epilogue_dense_staged<WP, WQ, TP, TQ, true>(p, acc, p0, q0, s_corr, s_mult, s_shift, smem);
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
  constexpr size_t lds = (size_t)kStages * (BP + BQ) * kBK + 1024 + 3 * CH * sizeof(int32_t);
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
    case 1: return launch_dma_cfg<2, 2, 2, 4, 3, 2, false, false>(p, st);  // 128 x 256, 2 per CU
    case 2: return launch_dma_cfg<2, 2, 4, 2, 3, 2, false, false>(p, st);  // 256 x 128, 2 per CU
    case 3: return launch_dma_cfg<2, 2, 2, 2, 4, 2, false, false>(p, st);  // 128 x 128
    case 5: return launch_dma_cfg<2, 2, 2, 4, 4, 1, false, false>(p, st);  // 128 x 256, 1 per CU
    default: return launch_dma_cfg<4, 2, 2, 4, 4, 1, false, false>(p, st); // 256 x 256, 8 wavefronts
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
