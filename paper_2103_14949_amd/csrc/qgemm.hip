// Quantized GEMM on the gfx950 int8 matrix cores (v_mfma_i32_32x32x32_i8):
// dense layers and non-depthwise convolutions (implicit GEMM), int32
// accumulation (optionally reduced modulo 2^16), fused requantize epilogue.
//
// A workgroup of WP x WQ wavefronts computes a BP x BQ tile of
// D[i][j] = sum_k P[i][k] * Q[j][k].  Both operands are byte matrices that are
// contiguous along k, which is what the MFMA wants: lane l feeds 16
// consecutive k-bytes of row (l % 32), the upper 32 lanes the next 16 bytes.
// In the result a lane owns column j = l % 32 and, per group of four
// accumulator registers, four CONSECUTIVE rows i.  P is therefore chosen as
// the operand whose index is contiguous in the output tensor, so that four
// results pack into one 32-bit store:
//   dense, NHWC conv : P = weights (i = output channel),  Q = activations
//   NCHW conv        : P = activations (i = output pixel), Q = weights
//
// What bounds the kernel.  A CU multiplies 4096 byte pairs per clock but its
// vector memory path delivers about 64 bytes per clock and its LDS about
// 128-140, so a tile must reuse every staged byte many times: the L1 traffic of
// a tile is (BP + BQ) * K bytes for BP * BQ * K products, and each wavefront
// re-reads its fragments from LDS once per 32 k.  Hence the large tiles
// (up to 256 x 256 per workgroup, 64 x 128 per wavefront) and eight wavefronts
// per workgroup, two per SIMD, so that one can issue MFMAs while the other
// waits on LDS.
//
// Zero points and unsigned activations.  The MFMA multiplies signed bytes.
// A uint8 activation a is fed as a' = a XOR 0x80 = a - 128, an int8 one as is
// (off = 128 or 0).  Then
//   sum_k (a - z) w = sum_k a' w + (off - z) * sum_k w[n,k]
// and the weight row sums are accumulated with v_dot4 by the lanes that stage
// the weight tile, so no separate pass over the weights is needed.  Padded
// convolution taps are staged as the zero point itself, which makes them
// contribute exactly 0 under the same identity.
//
// K is processed in stages of 128 bytes (one cache line per row), double
// buffered in LDS through registers (global -> VGPR -> LDS), one barrier per
// stage; the loads of stage s+1 are in flight while stage s is multiplied.
// The eight 16-byte chunks of an LDS row are XOR-swizzled with the row index
// so that fragment reads and staging writes spread over all banks.
#include "qgemm_common.h"


namespace hago {

namespace {

constexpr int kBK = 128;           // k-bytes per LDS stage
constexpr int kChunks = kBK / 16;  // 16-byte chunks per LDS row

enum { MODE_DENSE = 0, MODE_CONV_NCHW = 1, MODE_CONV_NHWC = 2 };

__device__ __forceinline__ int lds_off(int row, int chunk) {
  return row * kBK + ((chunk ^ row ^ (row >> 3)) & (kChunks - 1)) * 16;
}

// 16 bytes of row `row` of a row-major [ext, K] byte matrix starting at k,
// zero beyond the matrix.
__device__ __forceinline__ v4i load_rowmajor(const uint8_t* __restrict__ src, int row, int ext,
                                             int K, int k, int vec_k) {
  v4i v = {0, 0, 0, 0};
  if (row < ext && k < K) {
    const uint8_t* ptr = src + (size_t)row * (size_t)K + k;
    if (vec_k && k + 16 <= K) {
      v = *reinterpret_cast<const v4i*>(ptr);
    } else {
      uint32_t d[4] = {0u, 0u, 0u, 0u};
#pragma unroll
      for (int j = 0; j < 16; ++j)
        if (k + j < K) d[j >> 2] |= (uint32_t)ptr[j] << (8 * (j & 3));
      v = v4i{(int)d[0], (int)d[1], (int)d[2], (int)d[3]};
    }
  }
  return v;
}

__device__ __forceinline__ int32_t bytesum(const v4i& v) {
  int32_t s = __builtin_amdgcn_sdot4(v.x, 0x01010101, 0, false);
  s = __builtin_amdgcn_sdot4(v.y, 0x01010101, s, false);
  s = __builtin_amdgcn_sdot4(v.z, 0x01010101, s, false);
  s = __builtin_amdgcn_sdot4(v.w, 0x01010101, s, false);
  return s;
}

// Position of one im2col row (= output pixel) in the input tensor.
struct PixelPos {
  int32_t valid;   // row index < M
  int32_t base;    // NCHW: b*C*H*W + iy0*W + ix0 ; NHWC: ((b*H + iy0)*W + ix0)*C  (may be negative)
  int32_t iy0, ix0;
};

__device__ __forceinline__ PixelPos pixel_pos(const ConvGeom& g, int m, int M, bool nhwc) {
  PixelPos pp;
  pp.valid = m < M;
  const int mm = pp.valid ? m : 0;
  const int ohw = g.OH * g.OW;
  const int b = mm / ohw;
  const int pix = mm - b * ohw;
  const int oy = pix / g.OW;
  const int ox = pix - oy * g.OW;
  pp.iy0 = oy * g.stride_h - g.pad_h;
  pp.ix0 = ox * g.stride_w - g.pad_w;
  pp.base = nhwc ? ((b * g.H + pp.iy0) * g.W + pp.ix0) * g.C
                 : b * g.C * g.H * g.W + pp.iy0 * g.W + pp.ix0;
  return pp;
}

// 16 consecutive k of one im2col row, NCHW input, k = (c*KH + ky)*KW + kx.
// k0 is wavefront-uniform, so the (c, ky, kx) walk runs on the scalar unit.
__device__ __forceinline__ v4i load_im2col_nchw(const QgemmParams& p, const PixelPos& pp, int k0) {
  const ConvGeom& g = p.g;
  uint32_t d[4] = {0u, 0u, 0u, 0u};
  if (k0 >= p.K) return v4i{0, 0, 0, 0};
  const int khw = g.KH * g.KW;
  int c = k0 / khw;
  int t = k0 - c * khw;
  int ky = t / g.KW;
  int kx = t - ky * g.KW;
  int koff = (c * g.H + ky) * g.W + kx;
  const uint32_t xor1 = p.act_xor4 & 0xffu;
#pragma unroll
  for (int j = 0; j < 16; ++j) {
    uint32_t b = 0;
    if (k0 + j < p.K) {
      const int iy = pp.iy0 + ky, ix = pp.ix0 + kx;
      const bool ok = pp.valid && (unsigned)iy < (unsigned)g.H && (unsigned)ix < (unsigned)g.W;
      b = p.pad_byte;
      if (ok) b = (uint32_t)p.act[pp.base + koff] ^ xor1;
    }
    d[j >> 2] |= b << (8 * (j & 3));
    // advance (c, ky, kx) by one tap
    ++kx; ++koff;
    if (kx == g.KW) {
      kx = 0; ++ky; koff += g.W - g.KW;
      if (ky == g.KH) { ky = 0; koff += (g.H - g.KH) * g.W; }
    }
  }
  return v4i{(int)d[0], (int)d[1], (int)d[2], (int)d[3]};
}

// 16 consecutive k of one im2col row, NHWC input, k = (ky*KW + kx)*C + c.
__device__ __forceinline__ v4i load_im2col_nhwc(const QgemmParams& p, const PixelPos& pp, int k0) {
  const ConvGeom& g = p.g;
  const uint32_t xor1 = p.act_xor4 & 0xffu;
  if (k0 >= p.K) return v4i{0, 0, 0, 0};
  int t = k0 / g.C;
  int c = k0 - t * g.C;
  int ky = t / g.KW;
  int kx = t - ky * g.KW;
  if (p.vec_k && c + 16 <= g.C) {  // whole chunk inside one tap, 16-byte aligned
    const int iy = pp.iy0 + ky, ix = pp.ix0 + kx;
    const bool ok = pp.valid && (unsigned)iy < (unsigned)g.H && (unsigned)ix < (unsigned)g.W;
    const int padw = (int)(p.pad_byte * 0x01010101u);
    v4i v = {padw, padw, padw, padw};
    if (ok) {
      v = *reinterpret_cast<const v4i*>(p.act + (pp.base + (ky * g.W + kx) * g.C + c));
      const int x4 = (int)p.act_xor4;
      v = v4i{v.x ^ x4, v.y ^ x4, v.z ^ x4, v.w ^ x4};
    }
    return v;
  }
  uint32_t d[4] = {0u, 0u, 0u, 0u};
#pragma unroll
  for (int j = 0; j < 16; ++j) {
    uint32_t b = 0;
    if (k0 + j < p.K) {
      const int iy = pp.iy0 + ky, ix = pp.ix0 + kx;
      const bool ok = pp.valid && (unsigned)iy < (unsigned)g.H && (unsigned)ix < (unsigned)g.W;
      b = p.pad_byte;
      if (ok) b = (uint32_t)p.act[pp.base + (ky * g.W + kx) * g.C + c] ^ xor1;
    }
    d[j >> 2] |= b << (8 * (j & 3));
    ++c;
    if (c == g.C) {
      c = 0; ++kx;
      if (kx == g.KW) { kx = 0; ++ky; }
    }
  }
  return v4i{(int)d[0], (int)d[1], (int)d[2], (int)d[3]};
}

// VEC: every operand row can be read as aligned 16-byte chunks (dense: K % 16 == 0; NHWC: C % 16
// == 0).  Then staging loads are unconditional (addresses clamped into the tensor, the value
// replaced afterwards where it lies outside), so that a whole stage of loads is in flight while
// the previous stage is multiplied.  Without VEC the loads are assembled bytewise (any shape).
template <int WP, int WQ, int TP, int TQ, int MODE, bool VEC>
__global__ __launch_bounds__(64 * WP * WQ) void qgemm_kernel(QgemmParams p) {
  constexpr int NT = 64 * WP * WQ;
  constexpr int BP = WP * TP * 32;
  constexpr int BQ = WQ * TQ * 32;
  constexpr int NP = (BP * kChunks + NT - 1) / NT;  // 16-byte chunks per lane per stage
  constexpr int NQ = (BQ * kChunks + NT - 1) / NT;
  constexpr bool ACT_ON_P = (MODE == MODE_CONV_NCHW);
  constexpr int CH = ACT_ON_P ? BQ : BP;  // output channels covered by the tile
  constexpr int RA = ACT_ON_P ? BP : BQ;  // rows of the activation tile
  constexpr int NA = ACT_ON_P ? NP : NQ;
  constexpr int NW = ACT_ON_P ? NQ : NP;
  constexpr int RW = ACT_ON_P ? BQ : BP;  // rows of the weight tile
  constexpr int STAGE = (BP + BQ) * kBK;  // bytes of one LDS stage
  static_assert(MODE == MODE_DENSE || (RA % 64 == 0 && (NT % RA == 0 || RA % NT == 0)),
                "im2col staging needs a fixed tile row per lane and a uniform chunk per wavefront");

  extern __shared__ __attribute__((aligned(16))) uint8_t smem[];
  uint8_t* s_tile = smem;  // 2 stages
  int32_t* s_corr = reinterpret_cast<int32_t*>(smem + 2 * STAGE);
  int32_t* s_mult = s_corr + CH;
  int32_t* s_shift = s_mult + CH;

  const int t = threadIdx.x;
  const int lane = t & 63;
  const int wave = t >> 6;
  const int wp = wave % WP;
  const int wq = wave / WP;

  const int P_ext = ACT_ON_P ? p.M : p.N;
  const int tiles_p = (P_ext + BP - 1) / BP;
  const int tile = xcd_remap(blockIdx.x, gridDim.x);
  const int tile_p = tile % tiles_p;
  const int tile_q = tile / tiles_p;
  const int p0 = tile_p * BP;
  const int q0 = tile_q * BQ;
  const int a0 = ACT_ON_P ? p0 : q0;  // first activation row (m) of the tile
  const int w0 = ACT_ON_P ? q0 : p0;  // first weight row (n) of the tile
  const int a_lds = ACT_ON_P ? 0 : BP * kBK;  // byte offset of the activation tile in a stage
  const int w_lds = ACT_ON_P ? BP * kBK : 0;

  // im2col: the lane's tile row is the same in every stage
  PixelPos pp{};
  if constexpr (MODE != MODE_DENSE) pp = pixel_pos(p.g, a0 + (t % RA), p.M, MODE == MODE_CONV_NHWC);

  v4i st_a[NA], st_w[NW];
  int32_t wsum[NW];
#pragma unroll
  for (int s = 0; s < NW; ++s) wsum[s] = 0;

  // fast path: clamped row pointers, computed once
  const uint8_t* wrow[NW];
  const uint8_t* arow[NA];
  bool wrow_ok[NW], arow_ok[NA];
  if constexpr (VEC) {
#pragma unroll
    for (int s = 0; s < NW; ++s) {
      const int q = t + NT * s;
      const int row = w0 + q / kChunks;
      wrow_ok[s] = (q < RW * kChunks) && row < p.N;
      wrow[s] = reinterpret_cast<const uint8_t*>(p.wgt) + (size_t)(wrow_ok[s] ? row : 0) * p.K +
                (q % kChunks) * 16;
    }
    if constexpr (MODE == MODE_DENSE) {
#pragma unroll
      for (int s = 0; s < NA; ++s) {
        const int q = t + NT * s;
        const int row = a0 + q / kChunks;
        arow_ok[s] = (q < RA * kChunks) && row < p.M;
        arow[s] = p.act + (size_t)(arow_ok[s] ? row : 0) * p.K + (q % kChunks) * 16;
      }
    }
  }
  const int kmax = p.K - 16;  // last chunk start that is inside a row (VEC: K % 16 == 0, K >= 16)

  auto fetch = [&](int k0) {
    if constexpr (VEC) {
#pragma unroll
      for (int s = 0; s < NW; ++s) {
        const int kc = k0 + ((t + NT * s) % kChunks) * 16;
        const int back = kc > kmax ? kc - kmax : 0;  // pull a chunk beyond K back inside the row
        st_w[s] = *reinterpret_cast<const v4i*>(wrow[s] + k0 - back);
      }
    } else {
#pragma unroll
      for (int s = 0; s < NW; ++s) {
        const int q = t + NT * s;
        st_w[s] = v4i{0, 0, 0, 0};
        if (q < RW * kChunks)
          st_w[s] = load_rowmajor(reinterpret_cast<const uint8_t*>(p.wgt), w0 + q / kChunks, p.N,
                                  p.K, k0 + (q % kChunks) * 16, p.vec_k);
      }
    }
#pragma unroll
    for (int s = 0; s < NA; ++s) {
      const int q = t + NT * s;
      if constexpr (MODE == MODE_DENSE && VEC) {
        const int kc = k0 + (q % kChunks) * 16;
        const int back = kc > kmax ? kc - kmax : 0;
        st_a[s] = *reinterpret_cast<const v4i*>(arow[s] + k0 - back);
      } else {
        st_a[s] = v4i{0, 0, 0, 0};
        if (q < RA * kChunks) {
          if constexpr (MODE == MODE_DENSE) {
            st_a[s] = load_rowmajor(p.act, a0 + q / kChunks, p.M, p.K, k0 + (q % kChunks) * 16, p.vec_k);
          } else {
            const int ch = __builtin_amdgcn_readfirstlane(q / RA);
            if constexpr (MODE == MODE_CONV_NCHW)
              st_a[s] = load_im2col_nchw(p, pp, k0 + ch * 16);
            else
              st_a[s] = load_im2col_nhwc(p, pp, k0 + ch * 16);
          }
        }
      }
    }
  };

  // registers -> LDS; the weight row sums and the uint8 -> int8 flip happen here, once per byte
  auto stash = [&](int buf, int k0) {
    uint8_t* base = s_tile + buf * STAGE;
#pragma unroll
    for (int s = 0; s < NW; ++s) {
      const int q = t + NT * s;
      if (q < RW * kChunks) {
        v4i v = st_w[s];
        if constexpr (VEC) {
          if (!(wrow_ok[s] && k0 + (q % kChunks) * 16 < p.K)) v = v4i{0, 0, 0, 0};
        }
        wsum[s] += bytesum(v);
        *reinterpret_cast<v4i*>(base + w_lds + lds_off(q / kChunks, q % kChunks)) = v;
      }
    }
#pragma unroll
    for (int s = 0; s < NA; ++s) {
      const int q = t + NT * s;
      if (q < RA * kChunks) {
        if constexpr (MODE == MODE_DENSE) {
          const int x4 = (int)p.act_xor4;
          v4i v = st_a[s];
          if constexpr (VEC) {
            if (!(arow_ok[s] && k0 + (q % kChunks) * 16 < p.K)) v = v4i{0, 0, 0, 0};
          }
          *reinterpret_cast<v4i*>(base + a_lds + lds_off(q / kChunks, q % kChunks)) =
              v4i{v.x ^ x4, v.y ^ x4, v.z ^ x4, v.w ^ x4};
        } else {
          *reinterpret_cast<v4i*>(base + a_lds + lds_off(q % RA, q / RA)) = st_a[s];
        }
      }
    }
  };

  v16i acc[TP][TQ];
#pragma unroll
  for (int i = 0; i < TP; ++i)
#pragma unroll
    for (int j = 0; j < TQ; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0;

  const int KT = (p.K + kBK - 1) / kBK;
  if (KT > 0) {
    fetch(0);
    stash(0, 0);
  }
  __syncthreads();

  const int frow = lane & 31;
  const int fhalf = lane >> 5;
  for (int kt = 0; kt < KT; ++kt) {
    const int buf = kt & 1;
    if (kt + 1 < KT) fetch((kt + 1) * kBK);
    const uint8_t* base = s_tile + buf * STAGE;
#pragma unroll
    for (int ks = 0; ks < kBK / 32; ++ks) {
      v4i pf[TP], qf[TQ];
#pragma unroll
      for (int i = 0; i < TP; ++i) {
        const int row = (wp * TP + i) * 32 + frow;
        pf[i] = *reinterpret_cast<const v4i*>(base + lds_off(row, ks * 2 + fhalf));
      }
#pragma unroll
      for (int j = 0; j < TQ; ++j) {
        const int row = (wq * TQ + j) * 32 + frow;
        qf[j] = *reinterpret_cast<const v4i*>(base + BP * kBK + lds_off(row, ks * 2 + fhalf));
      }
#pragma unroll
      for (int i = 0; i < TP; ++i)
#pragma unroll
        for (int j = 0; j < TQ; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(pf[i], qf[j], acc[i][j], 0, 0, 0);
    }
    if (kt + 1 < KT) stash(buf ^ 1, (kt + 1) * kBK);
    __syncthreads();
  }

  // ---- per-channel terms of the tile: corr = bias + (off - z_a) * sum_k w, multiplier, shift
#pragma unroll
  for (int s = 0; s < NW; ++s) {
    int32_t v = wsum[s];
    v += __shfl_xor(v, 1);
    v += __shfl_xor(v, 2);
    v += __shfl_xor(v, 4);
    const int q = t + NT * s;
    if (q < RW * kChunks && (q % kChunks) == 0) s_corr[q / kChunks] = v;
  }
  __syncthreads();
  stage_channel_terms<NT, CH>(p, w0, s_corr, s_mult, s_shift);
  qgemm_epilogue<WP, WQ, TP, TQ, ACT_ON_P>(p, acc, p0, q0, s_corr, s_mult, s_shift);
}

// ---- tile shapes ---------------------------------------------------------------------------
// A shape is (WP, WQ, TP, TQ): wavefronts along P and Q, 32x32 sub-tiles per wavefront.
struct TileShape { int wp, wq, tp, tq; };
constexpr TileShape kShapes[] = {
    {2, 2, 2, 4},  // 0: 128 x 256
    {2, 2, 4, 2},  // 1: 256 x 128
    {2, 2, 2, 2},  // 2: 128 x 128
    {1, 4, 1, 2},  // 3:  32 x 256
    {4, 1, 2, 1},  // 4: 256 x  32
    {2, 2, 1, 2},  // 5:  64 x 128
    {2, 2, 2, 1},  // 6: 128 x  64
};
constexpr int kNumShapes = sizeof(kShapes) / sizeof(kShapes[0]);

template <int WP, int WQ, int TP, int TQ, int MODE, bool VEC>
hipError_t launch_cfg(const QgemmParams& p, hipStream_t st) {
  constexpr int BP = WP * TP * 32, BQ = WQ * TQ * 32;
  constexpr int CH = (MODE == MODE_CONV_NCHW) ? BQ : BP;
  constexpr size_t lds = 2 * (size_t)(BP + BQ) * kBK + 3 * CH * sizeof(int32_t);
  const int P_ext = (MODE == MODE_CONV_NCHW) ? p.M : p.N;
  const int Q_ext = (MODE == MODE_CONV_NCHW) ? p.N : p.M;
  const int64_t tiles = (int64_t)((P_ext + BP - 1) / BP) * ((Q_ext + BQ - 1) / BQ);
  auto kern = qgemm_kernel<WP, WQ, TP, TQ, MODE, VEC>;
  static std::atomic<uint64_t> attr_set{0};  // per kernel: the devices whose dynamic-LDS limit is raised
  hipError_t e = raise_lds_limit(reinterpret_cast<const void*>(kern), (int)lds, attr_set);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(kern, dim3((unsigned)tiles), dim3(64 * WP * WQ), lds, st, p);
  return hipGetLastError();
}

// Whether a shape can be instantiated for a mode (im2col staging wants a fixed tile row per
// lane and a wavefront-uniform chunk).
constexpr bool shape_ok(int mode, int wp, int wq, int tp, int tq) {
  if (mode == MODE_DENSE) return true;
  const int nt = 64 * wp * wq;
  const int ra = (mode == MODE_CONV_NCHW) ? wp * tp * 32 : wq * tq * 32;
  return ra % 64 == 0 && (nt % ra == 0 || ra % nt == 0);
}

template <int MODE, int I>
hipError_t launch_shape_rec(int shape, const QgemmParams& p, hipStream_t st) {
  if constexpr (I >= kNumShapes) {
    return launch_cfg<2, 2, 2, 2, MODE, false>(p, st);
  } else {
    constexpr TileShape s = kShapes[I];
    if constexpr (shape_ok(MODE, s.wp, s.wq, s.tp, s.tq)) {
      if (shape == I) return launch_cfg<s.wp, s.wq, s.tp, s.tq, MODE, MODE == MODE_DENSE>(p, st);
    }
    return launch_shape_rec<MODE, I + 1>(shape, p, st);
  }
}

template <int MODE>
hipError_t launch_shape(int shape, const QgemmParams& p, hipStream_t st) {
  return launch_shape_rec<MODE, 0>(shape, p, st);
}

// Estimated cycles of the slowest CU for a tile shape: tiles are spread over 256 CUs; a tile
// costs the larger of its MFMA time and its L1 time, plus the requantize epilogue.
double shape_cost(const TileShape& s, int64_t P_ext, int64_t Q_ext, int64_t K) {
  const int64_t bp = s.wp * s.tp * 32, bq = s.wq * s.tq * 32;
  const int64_t tiles = ((P_ext + bp - 1) / bp) * ((Q_ext + bq - 1) / bq);
  const double rounds = (double)((tiles + 255) / 256);
  const double kk = (double)((K + kBK - 1) / kBK * kBK);
  const double mfma = (double)bp * bq * kk / 4096.0 / 0.85;
  const double l1 = (double)(bp + bq) * kk / 52.0;
  const double lds_rate = 128.0 * (s.tp + s.tq) / (double)(s.tp * s.tq);  // bytes per clock needed
  const double lds = mfma * (lds_rate > 110.0 ? lds_rate / 110.0 : 1.0);
  const double main = mfma > l1 ? (mfma > lds ? mfma : lds) : (l1 > lds ? l1 : lds);
  const double epi = (double)bp * bq / (64.0 * s.wp * s.wq) * 36.0 / 4.0 * 4.0;
  return rounds * (main + epi + 1500.0);
}

// Test hooks: -1 / 0 mean "choose automatically".  Plain atomics: a test sets them between calls.
std::atomic<int> g_hook[kNumHooks] = {0, -1, -1};

int pick_shape(int mode, int64_t P_ext, int64_t Q_ext, int64_t K) {
  const int v = g_hook[kHookGenericTile].load(std::memory_order_relaxed);  // forced tile (tests)
  if (v >= 0 && v < kNumShapes && shape_ok(mode, kShapes[v].wp, kShapes[v].wq, kShapes[v].tp, kShapes[v].tq))
    return v;
  int best = 2;
  double best_cost = 1e300;
  for (int i = 0; i < kNumShapes; ++i) {
    if (!shape_ok(mode, kShapes[i].wp, kShapes[i].wq, kShapes[i].tp, kShapes[i].tq)) continue;
    const double c = shape_cost(kShapes[i], P_ext, Q_ext, K);
    if (c < best_cost) { best_cost = c; best = i; }
  }
  return best;
}

}  // namespace

hipError_t launch_qdense_dma(const QgemmParams& p, int shape, hipStream_t st);

#ifdef HAGO_PHASE_TIMING
// development builds only: the timing driver hands over the buffer for the kernels' phase stamps
extern "C" void hago_debug_set_stamp_buffer(long long* buf, int skip) {
  g_stamp_buffer = buf;
  g_stamp_skip = skip;
}
#endif

void set_test_hook(int key, int value) {
  if (key >= 0 && key < kNumHooks) g_hook[key].store(value, std::memory_order_relaxed);
}

hipError_t launch_qdense(const GemmArgs& a, hipStream_t st) {
  if (a.M == 0 || a.N == 0) return hipSuccess;
  if (a.operand16) return launch_qgemm16(a, nullptr, st);
  QgemmParams p = make_qgemm_params(a, nullptr);
  p.vec_k = (a.K % 16 == 0) && ptr_aligned(a.act, 16) && ptr_aligned(a.wgt, 16);
  p.vec_out = (a.N % 4 == 0) && ptr_aligned(a.out, 4 * qgemm_out_elem_size(a));
  p.vec16_out = (a.N % 16 == 0) && ptr_aligned(a.out, 16);
  if (!p.vec_k || a.K < 16) return launch_cfg<2, 2, 2, 2, MODE_DENSE, false>(p, st);
  const bool generic = g_hook[kHookGemmPath].load(std::memory_order_relaxed) == 1;
  const bool fits32 = (int64_t)a.N * a.K < (1ll << 31) && (int64_t)a.M * a.K < (1ll << 31);
  if (fits32 && !generic) {
    const int forced = g_hook[kHookDmaTile].load(std::memory_order_relaxed);
    // Tile shape: the one whose busiest CU has the least to do (rounds of tiles over the 256
    // CUs x tile area), with larger tiles discounted for their better operand reuse.
    struct Cand { int id, bp, bq; double eff; };
    static const Cand cands[] = {{0, 256, 256, 1.0}, {1, 192, 256, 0.95}, {2, 128, 128, 0.75}, {4, 64, 64, 0.5}};
    int best = 0;
    double best_cost = 0;
    for (const Cand& c : cands) {
      const int64_t tiles = (int64_t)((a.N + c.bp - 1) / c.bp) * ((a.M + c.bq - 1) / c.bq);
      const double cost = (double)((tiles + 255) / 256) * c.bp * c.bq / c.eff;
      if (c.id == 0 || cost < best_cost) { best = c.id; best_cost = cost; }
    }
    return launch_qdense_dma(p, forced >= 0 ? forced : best, st);
  }
  return launch_shape<MODE_DENSE>(pick_shape(MODE_DENSE, a.N, a.M, a.K), p, st);
}

hipError_t launch_qconv_dma(const QgemmParams& p, bool nchw_out, hipStream_t st);

namespace {
inline int64_t round256(int64_t v) { return (v + 255) & ~(int64_t)255; }
}  // namespace

int64_t qconv_workspace_bytes(const ConvGeom& cg) {
  const int64_t Cp = (cg.C + 15) / 16 * 16;
  const int64_t Hp = cg.H + 2 * (int64_t)cg.pad_h, Wp = cg.W + 2 * (int64_t)cg.pad_w;
  const int64_t act_bytes = (int64_t)cg.B * Hp * Wp * Cp;
  const int64_t Kp = (int64_t)cg.KH * cg.KW * Cp;
  const int64_t wgt_bytes = (int64_t)cg.O * Kp;
  // 32-bit offsets into both copies; k -> (tap, channel) and tap -> (ky, kx) by multiplication
  // with ceil(2^32 / C) and ceil(2^32 / KW), which is exact while k * Cp and tap * KW stay
  // below 2^32
  if (act_bytes >= (1ll << 31) || wgt_bytes >= (1ll << 31) || Kp * Cp >= (1ll << 32) ||
      (int64_t)cg.KH * cg.KW * cg.KW >= (1ll << 32))
    return -1;
  return round256(wgt_bytes) + round256(act_bytes);
}

// Fast path: rewrite both operands into the workspace (one launch), then run the implicit GEMM
// that streams them into LDS.
static hipError_t conv_dma(const GemmArgs& a, const ConvGeom& cg, void* ws, bool weights_ready,
                           hipStream_t st) {
  const int64_t Cp = (cg.C + 15) / 16 * 16;
  const int64_t Hp = cg.H + 2 * (int64_t)cg.pad_h, Wp = cg.W + 2 * (int64_t)cg.pad_w;
  const int64_t act_bytes = (int64_t)cg.B * Hp * Wp * Cp;
  const int64_t Kp = (int64_t)cg.KH * cg.KW * Cp;
  const int64_t wgt_bytes = (int64_t)cg.O * Kp;
  int8_t* wgt_p = static_cast<int8_t*>(ws);
  uint8_t* act_p = static_cast<uint8_t*>(ws) + round256(wgt_bytes);
  hipError_t err = launch_conv_prepack(a, cg, (int32_t)Cp, act_p, wgt_p, weights_ready, st);
  if (err != hipSuccess) return err;

  ConvGeom pg = cg;  // geometry of the padded copy
  pg.H = (int32_t)Hp; pg.W = (int32_t)Wp; pg.C = (int32_t)Cp; pg.pad_h = 0; pg.pad_w = 0;
  GemmArgs b = a;
  b.act = act_p;
  b.wgt = wgt_p;
  b.K = (int32_t)Kp;
  QgemmParams p = make_qgemm_params(b, &pg);
  p.act_xor4 = 0;  // the copy is already flipped; the zero-point term is unchanged
  p.vec_k = 1;
  p.act_bytes = (uint32_t)act_bytes;
  p.inv_c = (uint32_t)(((1ull << 32) + (uint64_t)Cp - 1) / (uint64_t)Cp);
  p.inv_kw = cg.KW > 1 ? (uint32_t)(((1ull << 32) + (uint64_t)cg.KW - 1) / (uint64_t)cg.KW) : 0u;
  if (cg.nhwc) {
    p.vec_out = (a.N % 4 == 0) && ptr_aligned(a.out, 4 * qgemm_out_elem_size(a));
    p.vec16_out = (a.N % 16 == 0) && ptr_aligned(a.out, 16);
  } else {
    p.vec_out = ((cg.OH * cg.OW) % 4 == 0) && ptr_aligned(a.out, 4 * qgemm_out_elem_size(a));
  }
  return launch_qconv_dma(p, !cg.nhwc, st);
}

hipError_t launch_qconv_gemm(const GemmArgs& a, const ConvGeom& cg, void* ws, bool weights_ready,
                             hipStream_t st) {
  if (a.M == 0 || a.N == 0) return hipSuccess;
  if (a.operand16) return launch_qgemm16(a, &cg, st);
  hipError_t err = hipSuccess;
  const int path = g_hook[kHookGemmPath].load(std::memory_order_relaxed);  // 1 / 2: skip the special cases
  if (path == 0) {
    if (try_qconv_pointwise_nchw(a, cg, st, &err)) return err;
    // channel-last 1x1 stride-1 unpadded convolution is a dense layer over the pixels
    if (cg.nhwc && cg.KH == 1 && cg.KW == 1 && cg.stride_h == 1 && cg.stride_w == 1 && cg.pad_h == 0 &&
        cg.pad_w == 0)
      return launch_qdense(a, st);
    // 3x3 stride 1 over NCHW: one launch that transposes the tensor on its way into the LDS
    // (faster than rewriting it through the workspace first, and it needs none)
    if (try_qconv3x3_nchw(a, cg, st, &err)) return err;
  }
  if (ws && path != 1 && qconv_workspace_bytes(cg) >= 0) return conv_dma(a, cg, ws, weights_ready, st);
  QgemmParams p = make_qgemm_params(a, &cg);
  if (cg.nhwc) {
    p.vec_k = (cg.C % 16 == 0) && ptr_aligned(a.act, 16) && ptr_aligned(a.wgt, 16);
    p.vec_out = (a.N % 4 == 0) && ptr_aligned(a.out, 4 * qgemm_out_elem_size(a));
    return launch_shape<MODE_CONV_NHWC>(pick_shape(MODE_CONV_NHWC, a.N, a.M, a.K), p, st);
  }
  p.vec_k = (a.K % 16 == 0) && ptr_aligned(a.wgt, 16);
  p.vec_out = ((cg.OH * cg.OW) % 4 == 0) && ptr_aligned(a.out, 4 * qgemm_out_elem_size(a));
  return launch_shape<MODE_CONV_NCHW>(pick_shape(MODE_CONV_NCHW, a.M, a.N, a.K), p, st);
}

}  // namespace hago
