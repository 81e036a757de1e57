// Quantized GEMM on the gfx950 int8 matrix cores (v_mfma_i32_32x32x32_i8):
// dense layers and non-depthwise convolutions (implicit GEMM), int32
// accumulation (optionally reduced modulo 2^16), fused requantize epilogue.
//
// One workgroup = 256 lanes = 4 wavefronts computes a BP x BQ tile of
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
// Zero points and unsigned activations.  The MFMA multiplies signed bytes.
// A uint8 activation a is fed as a' = a XOR 0x80 = a - 128, an int8 one as is
// (off = 128 or 0).  Then
//   sum_k (a - z) w = sum_k a' w + (off - z) * sum_k w[n,k]
// and the weight row sums are accumulated with v_dot4 by the lanes that stage
// the weight tile, so no separate pass over the weights is needed.  Padded
// convolution taps are staged as the zero point itself, which makes them
// contribute exactly 0 under the same identity.
//
// K is processed in stages of 64 bytes, double-buffered in LDS through
// registers (global -> VGPR -> LDS), one barrier per stage.  LDS rows are 64
// bytes; the four 16-byte chunks of a row are XOR-swizzled with the row index
// so that the 128-bit fragment reads and the staging writes spread over banks.
#include "hago_device.h"
#include "launch.h"

namespace hago {

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

constexpr int kThreads = 256;
constexpr int kBK = 64;  // k-bytes per LDS stage

enum { MODE_DENSE = 0, MODE_CONV_NCHW = 1, MODE_CONV_NHWC = 2 };

struct QgemmParams {
  const uint8_t* act;
  const int8_t* wgt;
  const int32_t* bias;
  void* out;
  const int32_t* mult;
  const int32_t* shift;
  int32_t M, N, K;
  int32_t per_channel, has_rq, acc16;
  int32_t out_mode;    // 0: requantized 8-bit, 1: raw int32, 2: raw int16
  uint32_t act_xor4;   // 0x80808080 for uint8 activations, else 0
  int32_t corr_coef;   // off - z_a
  uint32_t pad_byte;   // staged value of a padded tap: (z_a XOR act_xor) & 0xff
  int32_t vec_k;       // rows of both operands can be read as aligned 16-byte chunks
  int32_t vec_out;     // four consecutive results along the packed axis form one aligned store
  RequantScalars rs;
  ConvGeom g;
};

__device__ __forceinline__ int swz(int row, int chunk) {
  return chunk ^ (((row >> 1) ^ (row >> 3)) & 3);
}

__device__ __forceinline__ int lds_off(int row, int chunk) { return row * kBK + swz(row, chunk) * 16; }

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
  const int khw = g.KH * g.KW;
  int c = k0 / khw;
  int t = k0 - c * khw;
  int ky = t / g.KW;
  int kx = t - ky * g.KW;
  int koff = (c * g.H + ky) * g.W + kx;
#pragma unroll
  for (int j = 0; j < 16; ++j) {
    uint32_t b = 0;
    if (k0 + j < p.K) {
      const int iy = pp.iy0 + ky, ix = pp.ix0 + kx;
      const bool ok = pp.valid && (unsigned)iy < (unsigned)g.H && (unsigned)ix < (unsigned)g.W;
      b = p.pad_byte;
      if (ok) b = (uint32_t)p.act[pp.base + koff] ^ (p.act_xor4 & 0xffu);
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

template <int WP, int WQ, int TP, int TQ, int MODE>
__global__ __launch_bounds__(kThreads) void qgemm_kernel(QgemmParams p) {
  static_assert(WP * WQ == 4, "four wavefronts per workgroup");
  constexpr int BP = WP * TP * 32;
  constexpr int BQ = WQ * TQ * 32;
  constexpr int NP = (BP * 4 + kThreads - 1) / kThreads;  // 16-byte chunks per lane per stage
  constexpr int NQ = (BQ * 4 + kThreads - 1) / kThreads;
  constexpr bool ACT_ON_P = (MODE == MODE_CONV_NCHW);
  constexpr int CH = ACT_ON_P ? BQ : BP;  // output channels covered by the tile
  constexpr int RA = ACT_ON_P ? BP : BQ;  // rows of the activation tile
  constexpr int NA = ACT_ON_P ? NP : NQ;
  constexpr int NW = ACT_ON_P ? NQ : NP;
  constexpr int RW = ACT_ON_P ? BQ : BP;  // rows of the weight tile

  __shared__ __attribute__((aligned(16))) uint8_t s_tile[2][(BP + BQ) * kBK];
  __shared__ int32_t s_corr[CH];
  __shared__ int32_t s_mult[CH];
  __shared__ int32_t s_shift[CH];

  const int t = threadIdx.x;
  const int lane = t & 63;
  const int wave = t >> 6;
  const int wp = wave % WP;
  const int wq = wave / WP;

  const int P_ext = ACT_ON_P ? p.M : p.N;
  const int Q_ext = ACT_ON_P ? p.N : p.M;
  const int tiles_p = (P_ext + BP - 1) / BP;
  const int tile_p = blockIdx.x % tiles_p;
  const int tile_q = blockIdx.x / tiles_p;
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

  auto fetch = [&](int k0) {
#pragma unroll
    for (int s = 0; s < NW; ++s) {
      const int q = t + kThreads * s;
      st_w[s] = v4i{0, 0, 0, 0};
      if (q < RW * 4) {
        st_w[s] = load_rowmajor(reinterpret_cast<const uint8_t*>(p.wgt), w0 + (q >> 2), p.N, p.K,
                                k0 + (q & 3) * 16, p.vec_k);
        wsum[s] += bytesum(st_w[s]);
      }
    }
#pragma unroll
    for (int s = 0; s < NA; ++s) {
      const int q = t + kThreads * s;
      st_a[s] = v4i{0, 0, 0, 0};
      if (q < RA * 4) {
        if constexpr (MODE == MODE_DENSE) {
          v4i v = load_rowmajor(p.act, a0 + (q >> 2), p.M, p.K, k0 + (q & 3) * 16, p.vec_k);
          const int x4 = (int)p.act_xor4;
          st_a[s] = v4i{v.x ^ x4, v.y ^ x4, v.z ^ x4, v.w ^ x4};
        } else {
          // chunk index is uniform over a wavefront (RA is a multiple of 64 or divides it evenly)
          const int ch = __builtin_amdgcn_readfirstlane(q / RA);
          if constexpr (MODE == MODE_CONV_NCHW)
            st_a[s] = load_im2col_nchw(p, pp, k0 + ch * 16);
          else
            st_a[s] = load_im2col_nhwc(p, pp, k0 + ch * 16);
        }
      }
    }
  };

  auto stash = [&](int buf) {
    uint8_t* base = s_tile[buf];
#pragma unroll
    for (int s = 0; s < NW; ++s) {
      const int q = t + kThreads * s;
      if (q < RW * 4) *reinterpret_cast<v4i*>(base + w_lds + lds_off(q >> 2, q & 3)) = st_w[s];
    }
#pragma unroll
    for (int s = 0; s < NA; ++s) {
      const int q = t + kThreads * s;
      if (q < RA * 4) {
        const int row = (MODE == MODE_DENSE) ? (q >> 2) : (q % RA);
        const int ch = (MODE == MODE_DENSE) ? (q & 3) : (q / RA);
        *reinterpret_cast<v4i*>(base + a_lds + lds_off(row, ch)) = st_a[s];
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
    stash(0);
  }
  __syncthreads();

  const int frow = lane & 31;
  const int fhalf = lane >> 5;
  for (int kt = 0; kt < KT; ++kt) {
    const int buf = kt & 1;
    if (kt + 1 < KT) fetch((kt + 1) * kBK);
    const uint8_t* base = s_tile[buf];
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) {
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
    if (kt + 1 < KT) stash(buf ^ 1);
    __syncthreads();
  }

  // ---- per-channel terms of the tile: corr = bias + (off - z_a) * sum_k w, multiplier, shift
#pragma unroll
  for (int s = 0; s < NW; ++s) {
    int32_t v = wsum[s];
    v += __shfl_xor(v, 1);
    v += __shfl_xor(v, 2);
    const int q = t + kThreads * s;
    if (q < RW * 4 && (q & 3) == 0) s_corr[q >> 2] = v;
  }
  __syncthreads();
  for (int ci = t; ci < CH; ci += kThreads) {
    const int n = w0 + ci;
    int32_t corr = 0, mu = 0, sh = 0;
    if (n < p.N) {
      corr = (p.bias ? p.bias[n] : 0) + p.corr_coef * s_corr[ci];
      if (p.has_rq) {
        mu = p.mult[p.per_channel ? n : 0];
        sh = p.shift[p.per_channel ? n : 0];
      }
    }
    s_corr[ci] = corr;
    s_mult[ci] = mu;
    s_shift[ci] = sh;
  }
  __syncthreads();

  // ---- epilogue: requantize and store.  Per lane: column j, rows i0 .. i0+3 per register group.
  const int ohw = p.g.OH * p.g.OW;
#pragma unroll
  for (int tj = 0; tj < TQ; ++tj) {
    const int j_loc = (wq * TQ + tj) * 32 + frow;
    const int j = q0 + j_loc;
#pragma unroll
    for (int ti = 0; ti < TP; ++ti) {
#pragma unroll
      for (int g4 = 0; g4 < 4; ++g4) {
        const int i_loc = (wp * TP + ti) * 32 + g4 * 8 + fhalf * 4;
        const int i = p0 + i_loc;
        int32_t v[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const int ci = ACT_ON_P ? j_loc : i_loc + r;
          int32_t a = acc[ti][tj][g4 * 4 + r] + s_corr[ci];
          if (p.acc16) a = (int32_t)(int16_t)a;
          if (p.has_rq) a = requant_one(a, s_mult[ci], s_shift[ci], p.rs);
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

QgemmParams make_params(const GemmArgs& a, const ConvGeom* cg) {
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
  p.out_mode = a.has_rq ? 0 : (a.acc16 ? 2 : 1);
  p.act_xor4 = a.act_unsigned ? 0x80808080u : 0u;
  p.corr_coef = (a.act_unsigned ? 128 : 0) - a.act_zero_point;
  p.pad_byte = ((uint32_t)a.act_zero_point ^ (a.act_unsigned ? 0x80u : 0u)) & 0xffu;
  p.rs = RequantScalars{a.rq.z_out, a.rq.clip_lo - a.rq.z_out, a.rq.clip_hi - a.rq.z_out};
  if (cg) p.g = *cg;
  return p;
}

inline bool aligned(const void* ptr, size_t n) { return (reinterpret_cast<uintptr_t>(ptr) & (n - 1)) == 0; }

inline size_t out_elem_size(const GemmArgs& a) { return a.has_rq ? 1 : (a.acc16 ? 2 : 4); }

template <int WP, int WQ, int TP, int TQ, int MODE>
hipError_t launch_cfg(const QgemmParams& p, hipStream_t st) {
  constexpr int BP = WP * TP * 32, BQ = WQ * TQ * 32;
  const int P_ext = (MODE == MODE_CONV_NCHW) ? p.M : p.N;
  const int Q_ext = (MODE == MODE_CONV_NCHW) ? p.N : p.M;
  const int64_t tiles = (int64_t)((P_ext + BP - 1) / BP) * ((Q_ext + BQ - 1) / BQ);
  hipLaunchKernelGGL((qgemm_kernel<WP, WQ, TP, TQ, MODE>), dim3((unsigned)tiles), dim3(kThreads), 0,
                     st, p);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_qdense(const GemmArgs& a, hipStream_t st) {
  if (a.M == 0 || a.N == 0) return hipSuccess;
  QgemmParams p = make_params(a, nullptr);
  p.vec_k = (a.K % 16 == 0) && aligned(a.act, 16) && aligned(a.wgt, 16);
  p.vec_out = (a.N % 4 == 0) && aligned(a.out, 4 * out_elem_size(a));
  if (a.N <= 32) return launch_cfg<1, 4, 1, 2, MODE_DENSE>(p, st);   // 32 x 256
  if (a.N <= 64) return launch_cfg<2, 2, 1, 2, MODE_DENSE>(p, st);   // 64 x 128
  return launch_cfg<2, 2, 2, 2, MODE_DENSE>(p, st);                  // 128 x 128
}

hipError_t launch_qconv_gemm(const GemmArgs& a, const ConvGeom& cg, hipStream_t st) {
  if (a.M == 0 || a.N == 0) return hipSuccess;
  QgemmParams p = make_params(a, &cg);
  if (cg.nhwc) {
    p.vec_k = (cg.C % 16 == 0) && aligned(a.act, 16) && aligned(a.wgt, 16);
    p.vec_out = (a.N % 4 == 0) && aligned(a.out, 4 * out_elem_size(a));
    if (a.N <= 32) return launch_cfg<1, 4, 1, 2, MODE_CONV_NHWC>(p, st);
    if (a.N <= 64) return launch_cfg<2, 2, 1, 2, MODE_CONV_NHWC>(p, st);
    return launch_cfg<2, 2, 2, 2, MODE_CONV_NHWC>(p, st);
  }
  p.vec_k = (a.K % 16 == 0) && aligned(a.wgt, 16);
  p.vec_out = ((cg.OH * cg.OW) % 4 == 0) && aligned(a.out, 4 * out_elem_size(a));
  if (a.N <= 32) return launch_cfg<4, 1, 2, 1, MODE_CONV_NCHW>(p, st);   // 256 pixels x 32 channels
  if (a.N <= 64) return launch_cfg<2, 2, 2, 1, MODE_CONV_NCHW>(p, st);   // 128 x 64
  return launch_cfg<2, 2, 2, 2, MODE_CONV_NCHW>(p, st);                  // 128 x 128
}

}  // namespace hago
