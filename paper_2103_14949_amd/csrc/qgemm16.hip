// int16 x int16 operands with 32-bit (or 24-bit) accumulation: the second operand triple the
// paper names (Introduction; Sec. 4.1 hardware specification: "conv2d operator with int16 x int16
// inputs with int32 accumulation").  gfx950 has no int16 matrix instruction, so this runs on the
// vector ALUs with v_dot2_i32_i16 (two multiply-adds per lane and instruction): a plain LDS-tiled
// GEMM, 64 x 64 outputs per workgroup, 32 reduction elements per stage, 4 x 4 outputs per
// thread.  Dense layers and groups == 1 convolutions (both layouts, as an implicit GEMM whose
// loader gathers the taps) share the kernel.
//
// The activation zero point is not subtracted from the operands (a - z need not fit int16):
// sum (a - z) w = sum a w - z sum w, with the weight row sums accumulated by the same threads.
// Padded taps are staged as the zero point itself, so they contribute exactly 0 under that
// identity.  Products are exact in 32 bits and sums wrap modulo 2^32, as in the 8-bit kernels.
#include "hago_device.h"
#include "launch.h"

namespace hago {

namespace {

constexpr int kTile = 64;     // outputs per workgroup along both axes
constexpr int kStage = 32;    // reduction elements per stage
constexpr int kRowDw = kStage / 2 + 1;  // LDS row stride in dwords (17: conflict-free column reads)

struct G16Params {
  const int16_t* act;
  const int16_t* wgt;
  const int32_t* bias;
  void* out;
  const int32_t* mult;
  const int32_t* shift;
  int32_t M, N, K;
  int32_t per_channel, has_rq, acc_wrap_shift;
  int32_t z_a;
  int32_t mode;      // 0 dense, 1 conv NCHW, 2 conv NHWC
  int32_t vec_k;     // dense rows are aligned 16-byte chunks
  RequantScalars rs;
  ConvGeom g;
};

__device__ __forceinline__ int32_t dot2(uint32_t a, uint32_t b, int32_t c) {
  return __builtin_amdgcn_sdot2(__builtin_bit_cast(__attribute__((ext_vector_type(2))) short, a),
                                __builtin_bit_cast(__attribute__((ext_vector_type(2))) short, b), c, false);
}

// Element (row m, reduction index k) of the activation operand; k >= K and rows >= M read as 0,
// taps outside the image as the zero point.
__device__ __forceinline__ int32_t act_elem(const G16Params& p, int m, int k) {
  if (m >= p.M || k >= p.K) return 0;
  if (p.mode == 0) return p.act[(int64_t)m * p.K + k];
  const ConvGeom& g = p.g;
  const int ohw = g.OH * g.OW;
  const int b = m / ohw;
  const int pix = m - b * ohw;
  const int oy = pix / g.OW, ox = pix - oy * g.OW;
  int c, ky, kx;
  if (p.mode == 1) {  // k = (c * KH + ky) * KW + kx
    kx = k % g.KW;
    const int r = k / g.KW;
    ky = r % g.KH;
    c = r / g.KH;
  } else {            // k = (ky * KW + kx) * C + c
    c = k % g.C;
    const int r = k / g.C;
    kx = r % g.KW;
    ky = r / g.KW;
  }
  const int iy = oy * g.stride_h + ky - g.pad_h, ix = ox * g.stride_w + kx - g.pad_w;
  if ((unsigned)iy >= (unsigned)g.H || (unsigned)ix >= (unsigned)g.W) return p.z_a;
  const int64_t ai = p.mode == 1 ? (((int64_t)b * g.C + c) * g.H + iy) * g.W + ix
                                 : (((int64_t)b * g.H + iy) * g.W + ix) * g.C + c;
  return p.act[ai];
}

template <bool ZP>
__global__ __launch_bounds__(256) void qgemm16_kernel(G16Params p) {
  __shared__ uint32_t sa[kTile * kRowDw];
  __shared__ uint32_t sw[kTile * kRowDw];
  const int t = threadIdx.x;
  const int tx = t & 15, ty = t >> 4;
  const int tiles_n = (p.N + kTile - 1) / kTile;
  const int tile_m = (int)(blockIdx.x / tiles_n), tile_n = (int)(blockIdx.x % tiles_n);
  const int m0 = tile_m * kTile, n0 = tile_n * kTile;

  int32_t acc[4][4];
  int32_t wsum[4] = {0, 0, 0, 0};
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) acc[i][j] = 0;

  // staging: thread t fills 8 consecutive reduction elements (4 dwords) of row t / 4
  const int lrow = t >> 2, lchunk = (t & 3) * 8;
  for (int k0 = 0; k0 < p.K; k0 += kStage) {
    uint32_t va[4], vw[4];
    const int m = m0 + lrow, n = n0 + lrow, k = k0 + lchunk;
    if (p.vec_k && p.mode == 0 && m < p.M && k + 8 <= p.K) {
      const uint4 q = *reinterpret_cast<const uint4*>(p.act + (int64_t)m * p.K + k);
      va[0] = q.x; va[1] = q.y; va[2] = q.z; va[3] = q.w;
    } else {
#pragma unroll
      for (int e = 0; e < 4; ++e)
        va[e] = ((uint32_t)act_elem(p, m, k + 2 * e) & 0xffffu) | ((uint32_t)act_elem(p, m, k + 2 * e + 1) << 16);
    }
    if (p.vec_k && n < p.N && k + 8 <= p.K) {
      const uint4 q = *reinterpret_cast<const uint4*>(p.wgt + (int64_t)n * p.K + k);
      vw[0] = q.x; vw[1] = q.y; vw[2] = q.z; vw[3] = q.w;
    } else {
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const int32_t w0 = (n < p.N && k + 2 * e < p.K) ? p.wgt[(int64_t)n * p.K + k + 2 * e] : 0;
        const int32_t w1 = (n < p.N && k + 2 * e + 1 < p.K) ? p.wgt[(int64_t)n * p.K + k + 2 * e + 1] : 0;
        vw[e] = ((uint32_t)w0 & 0xffffu) | ((uint32_t)w1 << 16);
      }
    }
    __syncthreads();  // the previous stage has been consumed
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      sa[lrow * kRowDw + (lchunk >> 1) + e] = va[e];
      sw[lrow * kRowDw + (lchunk >> 1) + e] = vw[e];
    }
    __syncthreads();
#pragma unroll
    for (int kp = 0; kp < kStage / 2; ++kp) {
      uint32_t a4[4], w4[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) a4[i] = sa[(ty * 4 + i) * kRowDw + kp];
#pragma unroll
      for (int j = 0; j < 4; ++j) w4[j] = sw[(tx * 4 + j) * kRowDw + kp];
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = dot2(a4[i], w4[j], acc[i][j]);
      if constexpr (ZP) {
#pragma unroll
        for (int j = 0; j < 4; ++j) wsum[j] = dot2(w4[j], 0x00010001u, wsum[j]);
      }
    }
  }

  // epilogue: bias, zero-point term, accumulator width, requantize, store
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int n = n0 + tx * 4 + j;
    if (n >= p.N) continue;
    const int32_t corr = (p.bias ? p.bias[n] : 0) - (ZP ? p.z_a * wsum[j] : 0);
    int32_t m = 0, sh = 0;
    if (p.has_rq) {
      m = rq_mult(p.mult, p.per_channel ? n : 0);
      sh = rq_shift(p.mult, p.shift, p.per_channel ? n : 0);
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int row = m0 + ty * 4 + i;
      if (row >= p.M) continue;
      int32_t a = acc[i][j] + corr;
      if (p.acc_wrap_shift) a = wrap_acc_bits(a, p.acc_wrap_shift);
      int64_t o;
      if (p.mode == 1) {
        const int ohw = p.g.OH * p.g.OW;
        const int b = row / ohw;
        o = ((int64_t)b * p.N + n) * ohw + (row - b * ohw);
      } else {
        o = (int64_t)row * p.N + n;
      }
      if (p.has_rq) static_cast<uint8_t*>(p.out)[o] = (uint8_t)requant_general(a, m, sh, p.rs);
      else static_cast<int32_t*>(p.out)[o] = a;
    }
  }
}

}  // namespace

hipError_t launch_qgemm16(const GemmArgs& a, const ConvGeom* cg, hipStream_t st) {
  if (a.M == 0 || a.N == 0) return hipSuccess;
  G16Params p{};
  p.act = static_cast<const int16_t*>(a.act);
  p.wgt = reinterpret_cast<const int16_t*>(a.wgt);
  p.bias = a.bias;
  p.out = a.out;
  p.mult = a.rq.multiplier;
  p.shift = a.rq.shift;
  p.M = a.M; p.N = a.N; p.K = a.K;
  p.per_channel = a.rq.per_channel;
  p.has_rq = a.has_rq;
  p.acc_wrap_shift = a.acc_wrap_shift;
  p.z_a = a.act_zero_point;
  p.mode = cg ? (cg->nhwc ? 2 : 1) : 0;
  p.vec_k = (a.K % 8 == 0) && ((reinterpret_cast<uintptr_t>(a.act) & 15u) == 0) &&
            ((reinterpret_cast<uintptr_t>(a.wgt) & 15u) == 0);
  p.rs = RequantScalars{a.rq.z_out, a.rq.clip_lo - a.rq.z_out, a.rq.clip_hi - a.rq.z_out, a.rq.half_away};
  if (cg) p.g = *cg;
  const int64_t tiles = (int64_t)((a.M + kTile - 1) / kTile) * ((a.N + kTile - 1) / kTile);
  if (tiles >= (1ll << 31)) return hipErrorInvalidValue;
  if (a.act_zero_point != 0)
    hipLaunchKernelGGL(qgemm16_kernel<true>, dim3((unsigned)tiles), dim3(256), 0, st, p);
  else
    hipLaunchKernelGGL(qgemm16_kernel<false>, dim3((unsigned)tiles), dim3(256), 0, st, p);
  return hipGetLastError();
}

}  // namespace hago
