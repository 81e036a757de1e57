// Depthwise quantized convolution (groups == C == O) with the fused requantize
// epilogue.  Bandwidth-bound: each output byte needs one input byte from HBM,
// so there is no MFMA here; the work is 9 multiply-adds per output on the
// vector ALUs (4 at a time with v_dot4).
//
//   rows3x3  : NCHW, 3x3, stride 1, pad 1, W % 4 == 0, aligned.  One WAVEFRONT per (image,
//              channel, band of rows, segment of 64 columns) and no LDS: a lane loads one
//              dword per input row and gets its neighbours' by DPP; see the kernel.
//   rows3x3s2: the same for stride 2 (two outputs per lane and row).
//   small3x3 : stride 1, W <= 16, H <= 64, any alignment: several planes per wavefront.
//   nhwc3x3  : channel-last, stride 1, pad 1, C % 4 == 0: four channels and a run of pixels per thread.
//   wave3x3  : stride 1, W <= 64, without the alignment conditions.  One WAVEFRONT per (image,
//              channel) plane, four planes per workgroup.  A lane owns a strip
//              of four output columns and a quarter of the rows and slides
//              down it, so every staged input row is read from LDS once and
//              serves three output rows; 12 v_dot4 per four outputs.
//   plane3x3 : the same geometry for wider images.  One workgroup per (image,
//              channel, band of rows).  The band plus a one-pixel halo (filled with the
//              zero point, so padded taps contribute 0) is staged in LDS with
//              the image column x at LDS column x + 4; four adjacent outputs
//              share three aligned dword reads per input row.
//   direct   : every other geometry / layout: one output per lane straight
//              from global memory (cache-served), same arithmetic.
#include "hago_device.h"
#include "launch.h"

namespace hago {

namespace {

constexpr int kThreads = 256;
constexpr int kBandRows = 64;          // output rows per workgroup (plane3x3)
constexpr int kMaxLdsBytes = 60 * 1024;

struct DwArgs {
  const uint8_t* act;
  const int8_t* wgt;
  const int32_t* bias;
  void* out;
  ConvGeom g;
  uint32_t act_xor;    // 0x80 for a uint8 container (maps it to int8 = a - 128)
  int32_t act_off;     // 128 for uint8, 0 for int8
  int32_t z_a;
  int32_t acc16;
  int32_t acc_wrap_shift;  // 32 - accumulator bits (0, 16 or 8); the register kernels know 0 and 16 only
  int32_t has_rq;
  int32_t out_mode;    // 0: requantized 8-bit, 1: raw int32, 2: raw int16
  const int32_t* mult;
  const int32_t* shift;
  int32_t per_channel;
  RequantScalars rs;
};

__device__ __forceinline__ int32_t wrap_acc(int32_t acc, int wrap_shift) {
  return wrap_shift ? wrap_acc_bits(acc, wrap_shift) : acc;
}

__device__ __forceinline__ void store_one(const DwArgs& p, int64_t idx, int32_t acc, int32_t m,
                                          int32_t sh) {
  if (p.out_mode == 0)
    static_cast<uint8_t*>(p.out)[idx] = (uint8_t)requant_general(acc, m, sh, p.rs);
  else if (p.out_mode == 1)
    static_cast<int32_t*>(p.out)[idx] = acc;
  else
    static_cast<int16_t*>(p.out)[idx] = (int16_t)acc;
}

__global__ __launch_bounds__(kThreads) void dw_direct_kernel(DwArgs p) {
  const ConvGeom& g = p.g;
  const int64_t total = (int64_t)g.B * g.O * g.OH * g.OW;
  const int64_t stride = (int64_t)gridDim.x * kThreads;
  for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < total; i += stride) {
    int32_t b, c, oy, ox;
    int64_t r = i;
    if (g.nhwc) {
      c = (int32_t)(r % g.O); r /= g.O;
      ox = (int32_t)(r % g.OW); r /= g.OW;
      oy = (int32_t)(r % g.OH); b = (int32_t)(r / g.OH);
    } else {
      ox = (int32_t)(r % g.OW); r /= g.OW;
      oy = (int32_t)(r % g.OH); r /= g.OH;
      c = (int32_t)(r % g.O); b = (int32_t)(r / g.O);
    }
    int32_t acc = p.bias ? p.bias[c] : 0;
    for (int ky = 0; ky < g.KH; ++ky) {
      const int iy = oy * g.stride_h + ky - g.pad_h;
      if (iy < 0 || iy >= g.H) continue;
      for (int kx = 0; kx < g.KW; ++kx) {
        const int ix = ox * g.stride_w + kx - g.pad_w;
        if (ix < 0 || ix >= g.W) continue;
        const int64_t ai = g.nhwc ? (((int64_t)b * g.H + iy) * g.W + ix) * g.C + c
                                  : (((int64_t)b * g.C + c) * g.H + iy) * g.W + ix;
        const int64_t wi = g.nhwc ? ((int64_t)c * g.KH + ky) * g.KW + kx
                                  : ((int64_t)c * g.KH + ky) * g.KW + kx;
        const int32_t av = (int32_t)(int8_t)(p.act[ai] ^ p.act_xor) + p.act_off - p.z_a;
        acc += av * (int32_t)p.wgt[wi];
      }
    }
    acc = wrap_acc(acc, p.acc_wrap_shift);
    const int pc = p.per_channel ? c : 0;
    store_one(p, i, acc, p.has_rq ? rq_mult(p.mult, pc) : 0, p.has_rq ? rq_shift(p.mult, p.shift, pc) : 0);
  }
}

// NCHW 3x3 stride 1 pad 1.  Dynamic LDS: (band_rows + 2) * rs bytes where
// rs = row stride (multiple of 4, >= W + 12).
__global__ __launch_bounds__(kThreads) void dw_plane3x3_kernel(DwArgs p, int32_t rs, int32_t nband,
                                                              int32_t vec_io) {
  extern __shared__ uint32_t lds[];
  const ConvGeom& g = p.g;
  const int H = g.H, W = g.W;
  const int64_t plane = blockIdx.x / nband;  // b * C + c
  const int band = (int)(blockIdx.x - plane * nband);
  const int c = (int)(plane % g.C);
  const int y0 = band * kBandRows;
  const int rows = (H - y0 < kBandRows) ? H - y0 : kBandRows;  // output rows in this band
  const int lrows = rows + 2;
  const int rs4 = rs >> 2;

  const uint32_t padb = ((uint32_t)p.z_a ^ p.act_xor) & 0xffu;
  const uint32_t pad4 = padb * 0x01010101u;
  for (int i = threadIdx.x; i < lrows * rs4; i += kThreads) lds[i] = pad4;
  __syncthreads();

  // stage input rows y0-1 .. y0+rows (clipped to the image); image column x
  // goes to LDS column x + 4 so that aligned dwords stay aligned.
  const uint8_t* src = p.act + plane * (int64_t)H * W;
  const int ya = (y0 - 1 < 0) ? 0 : y0 - 1;
  const int yb = (y0 + rows + 1 > H) ? H : y0 + rows + 1;
  if (vec_io) {
    const int w4 = W >> 2;
    const uint32_t x4 = p.act_xor * 0x01010101u;
    const uint32_t* src4 = reinterpret_cast<const uint32_t*>(src);
    for (int i = threadIdx.x; i < (yb - ya) * w4; i += kThreads) {
      const int r = i / w4, q = i - r * w4;
      lds[(ya + r - (y0 - 1)) * rs4 + 1 + q] = src4[(ya + r) * w4 + q] ^ x4;
    }
  } else {
    uint8_t* l8 = reinterpret_cast<uint8_t*>(lds);
    for (int i = threadIdx.x; i < (yb - ya) * W; i += kThreads) {
      const int r = i / W, x = i - r * W;
      l8[(ya + r - (y0 - 1)) * rs + 4 + x] = (uint8_t)(src[(int64_t)(ya + r) * W + x] ^ p.act_xor);
    }
  }

  // per-channel constants
  const int8_t* wc = p.wgt + (int64_t)c * 9;
  uint32_t wrow[3];
  int32_t wsum = 0;
#pragma unroll
  for (int ky = 0; ky < 3; ++ky) {
    const int32_t w0 = wc[ky * 3 + 0], w1 = wc[ky * 3 + 1], w2 = wc[ky * 3 + 2];
    wsum += w0 + w1 + w2;
    wrow[ky] = (uint32_t)(w0 & 0xff) | ((uint32_t)(w1 & 0xff) << 8) | ((uint32_t)(w2 & 0xff) << 16);
  }
  // sum (a - z) w = sum (a' + off - z) w = sum a' w + (off - z) * sum w, a' = staged byte
  const int32_t corr = (p.bias ? p.bias[c] : 0) + (p.act_off - p.z_a) * wsum;
  const int pc = p.per_channel ? c : 0;
  const int32_t m = p.has_rq ? rq_mult(p.mult, pc) : 0;
  const int32_t sh = p.has_rq ? rq_shift(p.mult, p.shift, pc) : 0;
  __syncthreads();

  const int gx = (W + 3) >> 2;  // groups of 4 outputs per row
  const int64_t obase = plane * (int64_t)H * W;
  for (int it = threadIdx.x; it < rows * gx; it += kThreads) {
    const int ry = it / gx, q = it - ry * gx;
    int32_t acc[4] = {corr, corr, corr, corr};
#pragma unroll
    for (int ky = 0; ky < 3; ++ky) {
      const uint32_t* row = lds + (ry + ky) * rs4 + q;  // LDS columns 4q .. 4q+11
      const uint32_t d0 = row[0], d1 = row[1], d2 = row[2];
      // output x = 4q + i reads LDS columns x + 3 .. x + 5
      const uint32_t w0 = __builtin_amdgcn_alignbyte(d1, d0, 3);
      const uint32_t w1 = d1;
      const uint32_t w2 = __builtin_amdgcn_alignbyte(d2, d1, 1);
      const uint32_t w3 = __builtin_amdgcn_alignbyte(d2, d1, 2);
      acc[0] = __builtin_amdgcn_sdot4((int)w0, (int)wrow[ky], acc[0], false);
      acc[1] = __builtin_amdgcn_sdot4((int)w1, (int)wrow[ky], acc[1], false);
      acc[2] = __builtin_amdgcn_sdot4((int)w2, (int)wrow[ky], acc[2], false);
      acc[3] = __builtin_amdgcn_sdot4((int)w3, (int)wrow[ky], acc[3], false);
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) acc[i] = wrap_acc(acc[i], p.acc_wrap_shift);
    const int x0 = q << 2;
    const int64_t o = obase + (int64_t)(y0 + ry) * W + x0;
    if (vec_io) {
      if (p.out_mode == 0) {
        reinterpret_cast<uint32_t*>(p.out)[o >> 2] =
            pack4(requant_general(acc[0], m, sh, p.rs), requant_general(acc[1], m, sh, p.rs),
                  requant_general(acc[2], m, sh, p.rs), requant_general(acc[3], m, sh, p.rs));
      } else if (p.out_mode == 1) {
        reinterpret_cast<int4*>(p.out)[o >> 2] = make_int4(acc[0], acc[1], acc[2], acc[3]);
      } else {
        reinterpret_cast<short4*>(p.out)[o >> 2] =
            make_short4((short)acc[0], (short)acc[1], (short)acc[2], (short)acc[3]);
      }
    } else {
#pragma unroll
      for (int i = 0; i < 4; ++i)
        if (x0 + i < W) store_one(p, o + i, acc[i], m, sh);
    }
  }
}


// r = floor((a * m + 2^(30+sh)) / 2^(31+sh)); sh is wavefront-uniform here.
__device__ __forceinline__ int32_t dw_mul_shift(int32_t a, int32_t m, int64_t rnd, int32_t sh) {
  const int64_t pr = (int64_t)a * (int64_t)m + rnd;
  return sh >= 1 ? ((int32_t)(pr >> 32) >> (sh - 1)) : (int32_t)(pr >> (31 + sh));
}

// NCHW 3x3 stride 1 pad 1, W <= 64.  Dynamic LDS: 4 planes x (H + 2) * rs bytes,
// rs = row stride (multiple of 4, >= W + 12).  inv_w4 = ceil(2^32 / (W / 4)) (vector path).
__global__ __launch_bounds__(kThreads) void dw_wave3x3_kernel(DwArgs p, int32_t rs, uint32_t inv_w4,
                                                             int32_t vec_io, int64_t planes) {
  extern __shared__ uint32_t lds[];
  const ConvGeom& g = p.g;
  const int H = g.H, W = g.W;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int64_t plane = (int64_t)blockIdx.x * 4 + wave;  // b * C + c
  const bool active = plane < planes;
  const int c = active ? (int)(plane % g.C) : 0;
  const int lrows = H + 2;
  const int rs4 = rs >> 2;
  uint32_t* pl = lds + wave * lrows * rs4;  // this wavefront's plane: image (y, x) at row y+1, column x+4

  const uint32_t padb = ((uint32_t)p.z_a ^ p.act_xor) & 0xffu;
  const uint32_t pad4 = padb * 0x01010101u;
  if (active) {
    const uint8_t* src = p.act + plane * (int64_t)H * W;
    if (vec_io) {
      const int w4 = W >> 2;
      const uint32_t x4 = p.act_xor * 0x01010101u;
      const uint32_t* src4 = reinterpret_cast<const uint32_t*>(src);
      // halo (and everything else) first, then the image over it; LDS operations of one
      // wavefront execute in order, so the second write wins
      for (int i = lane; i < lrows * rs4; i += 64) pl[i] = pad4;
      // image dwords in batches of 8 loads per lane, all issued before the first is used
      const int nd = H * w4;
      for (int i0 = 0; i0 < nd; i0 += 8 * 64) {
        uint32_t v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
          const int i = i0 + u * 64 + lane;
          v[u] = src4[i < nd ? i : nd - 1];
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) {
          const int i = i0 + u * 64 + lane;
          const int r = (w4 == 1) ? i : (int)__umulhi((uint32_t)i, inv_w4);  // i / w4
          const int q = i - r * w4;
          if (i < nd) pl[(r + 1) * rs4 + 1 + q] = v[u] ^ x4;
        }
      }
    } else {
      uint8_t* l8 = reinterpret_cast<uint8_t*>(pl);
      for (int i = lane; i < lrows * rs; i += 64) {
        const int r = i / rs, x = i - r * rs - 4;
        uint32_t v = padb;
        if (r >= 1 && r <= H && x >= 0 && x < W) v = (uint32_t)src[(int64_t)(r - 1) * W + x] ^ p.act_xor;
        l8[i] = (uint8_t)v;
      }
    }
  }
  __syncthreads();
  if (!active) return;

  // per-channel constants (wavefront-uniform)
  const int8_t* wc = p.wgt + (int64_t)c * 9;
  uint32_t wrow[3];
  int32_t wsum = 0;
#pragma unroll
  for (int ky = 0; ky < 3; ++ky) {
    const int32_t w0 = wc[ky * 3 + 0], w1 = wc[ky * 3 + 1], w2 = wc[ky * 3 + 2];
    wsum += w0 + w1 + w2;
    wrow[ky] = (uint32_t)(w0 & 0xff) | ((uint32_t)(w1 & 0xff) << 8) | ((uint32_t)(w2 & 0xff) << 16);
  }
  const int32_t corr = (p.bias ? p.bias[c] : 0) + (p.act_off - p.z_a) * wsum;
  const int pc = p.per_channel ? c : 0;
  const int32_t m = p.has_rq ? rq_mult(p.mult, pc) : 0;
  const int32_t sh = p.has_rq ? rq_shift(p.mult, p.shift, pc) : 0;
  const int64_t rnd = (int64_t)1 << (30 + sh);
  const int32_t lo = p.rs.lo_rel, hi = p.rs.hi_rel, z = p.rs.z_out;

  const int gx = (W + 3) >> 2;  // strips of 4 output columns (<= 16)
  const int q = lane & 15;
  const int rc = lane >> 4;
  const int rpc = (H + 3) >> 2;  // rows per lane quarter
  const int y0 = rc * rpc;
  const int y1 = (y0 + rpc < H) ? y0 + rpc : H;
  if (q >= gx || y0 >= y1) return;

  // windows of one staged row: output x = 4q + i reads LDS columns x+3 .. x+5
  auto windows = [&](int lrow, uint32_t (&w)[4]) {
    const uint32_t* row = pl + lrow * rs4 + q;
    const uint32_t d0 = row[0], d1 = row[1], d2 = row[2];
    w[0] = __builtin_amdgcn_alignbyte(d1, d0, 3);
    w[1] = d1;
    w[2] = __builtin_amdgcn_alignbyte(d2, d1, 1);
    w[3] = __builtin_amdgcn_alignbyte(d2, d1, 2);
  };
  uint32_t wa[4], wb[4], wcur[4];
  windows(y0, wa);      // image row y0 - 1
  windows(y0 + 1, wb);  // image row y0
  const int64_t obase = plane * (int64_t)H * W;
  for (int y = y0; y < y1; ++y) {
    windows(y + 2, wcur);  // image row y + 1
    int32_t acc[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      int32_t a = __builtin_amdgcn_sdot4((int)wa[i], (int)wrow[0], corr, false);
      a = __builtin_amdgcn_sdot4((int)wb[i], (int)wrow[1], a, false);
      a = __builtin_amdgcn_sdot4((int)wcur[i], (int)wrow[2], a, false);
      acc[i] = wrap_acc(a, p.acc_wrap_shift);
      wa[i] = wb[i];
      wb[i] = wcur[i];
    }
    const int x0 = q << 2;
    const int64_t o = obase + (int64_t)y * W + x0;
    if (p.out_mode == 0) {
      int32_t r[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) r[i] = med3(dw_mul_shift(acc[i], m, rnd, sh), lo, hi) + z;
      if (vec_io) {
        reinterpret_cast<uint32_t*>(p.out)[o >> 2] = pack4_perm(r[0], r[1], r[2], r[3]);
      } else {
#pragma unroll
        for (int i = 0; i < 4; ++i)
          if (x0 + i < W) static_cast<uint8_t*>(p.out)[o + i] = (uint8_t)r[i];
      }
    } else if (vec_io && p.out_mode == 1) {
      reinterpret_cast<int4*>(p.out)[o >> 2] = make_int4(acc[0], acc[1], acc[2], acc[3]);
    } else if (vec_io) {
      reinterpret_cast<short4*>(p.out)[o >> 2] =
          make_short4((short)acc[0], (short)acc[1], (short)acc[2], (short)acc[3]);
    } else {
#pragma unroll
      for (int i = 0; i < 4; ++i)
        if (x0 + i < W) store_one(p, o + i, acc[i], m, sh);
    }
  }
}


// NCHW 3x3 stride 1 pad 1, W % 4 == 0, 4-byte aligned tensors and weights, planes
// below 2 GB: no LDS.  One wavefront per (plane, band of 4 * rpc rows), rpc <= 16.  Lane (q, rc):
// strip of four output columns q, quarter rc of the band's rows.  A lane loads ONE dword per
// input row (its own strip) and takes the left and right neighbours' dwords by DPP row shifts
// (the 16 lanes of a DPP row are the strips of one image row; lanes without a strip hold the
// zero point, which is also what a shift from outside the row yields).  All rpc + 2 loads are
// in flight together.  Loads and stores go through buffer descriptors of the plane, so a lane
// that has nothing to load or store just uses an out-of-range offset.
// The kernel is bound by vector-ALU instruction issue (about 40 per row of four outputs against
// 5 bytes of traffic), so everything that is the same for the whole wavefront -- the channel's
// weights, bias and multiplier -- comes through scalar loads and scalar arithmetic, and the
// per-output work is three dot products, one 64-bit multiply-add, one shift and one clamp.
// MODE 0: requantized 8-bit, 1: raw int32, 2: raw int16; ACC16: accumulator wraps to 16 bits.
// WIDE: images wider than 64 columns are cut into segments of 64 (grid z = band * nsegs + segment);
// the lanes at the ends of a segment fetch the neighbouring segment's dword with one more load
// per row, which replaces what the DPP shift cannot deliver.
template <int MODE, bool ACC16, bool WIDE>
__global__ __launch_bounds__(kThreads) void dw_rows3x3_kernel(DwArgs p, int32_t rpc, int32_t nsegs) {
  // grid: x = groups of four channels, y = image, z = band (and column segment)
  const ConvGeom& g = p.g;
  const int H = g.H, W = g.W;
  const int lane = threadIdx.x & 63;
  const int c = (int)(blockIdx.x * 4 + __builtin_amdgcn_readfirstlane(threadIdx.x >> 6));
  if (c >= g.C) return;  // wavefront-uniform; the kernel has no barrier
  const int64_t plane = (int64_t)blockIdx.y * g.C + c;
  const int seg = WIDE ? (int)blockIdx.z % nsegs : 0;
  const int band = WIDE ? (int)blockIdx.z / nsegs : (int)blockIdx.z;
  const int cb = seg * 64;  // first column of the segment
  constexpr uint32_t kOob = 0x80000000u;
  constexpr int kEsz = MODE == 0 ? 1 : (MODE == 1 ? 4 : 2);
  constexpr int kPass = 16;  // most output rows per lane

  const int q = lane & 15;
  const int rc = lane >> 4;
  const int y0 = (band * 4 + rc) * rpc;  // first output row of the lane
  const bool has_strip = cb + (q << 2) < W;
  const uint32_t lane_off = has_strip ? (uint32_t)(cb + (q << 2)) : kOob;  // byte column of the strip
  // the dword beyond the segment's end that this lane stands in for (first lane: left, last: right)
  const bool left_edge = WIDE && q == 0 && seg > 0;
  const bool right_edge = WIDE && q == 15 && cb + 64 < W;
  const uint32_t edge_off = left_edge ? (uint32_t)(cb - 4) : (right_edge ? (uint32_t)(cb + 64) : kOob);
  const uint32_t x4 = p.act_xor * 0x01010101u;
  const uint32_t pad4 = (((uint32_t)p.z_a ^ p.act_xor) & 0xffu) * 0x01010101u;
  const int64_t pbytes = (int64_t)H * W;
  const __amdgpu_buffer_rsrc_t rin = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<uint8_t*>(p.act) + (int64_t)plane * pbytes, 0, (int)pbytes, 0x00020000);
  const __amdgpu_buffer_rsrc_t rout = __builtin_amdgcn_make_buffer_rsrc(
      static_cast<uint8_t*>(p.out) + (int64_t)plane * pbytes * kEsz, 0, (int)(pbytes * kEsz), 0x00020000);

  // Row i of the lane is image row y0 + i - 1.  A row outside the image, and a lane without a
  // strip, read as the zero point: their offsets are out of the descriptor's range (a negative
  // row wraps to a huge offset, a row >= H lies beyond the plane, a strip-less lane starts at
  // 2^31), such a load returns 0, and the flip mask turns that into the zero point's byte (in
  // range it is the plain sign flip).  The mask is opaque to the compiler: with a select on the
  // loaded value it builds a branch around every load, each followed by a full wait.
  uint32_t flip_lane = has_strip ? x4 : pad4;
  asm volatile("" : "+v"(flip_lane));
  uint32_t d[kPass + 2];  // as loaded; the flip is applied where a row is used, so that no row waits for a later one
  {
    const uint32_t off0 = lane_off + (uint32_t)((y0 - 1) * W);
#pragma unroll
    for (int i = 0; i < kPass + 2; ++i) {
      uint32_t off = off0 + (uint32_t)(i * W);
      if (i >= 3) off = (i - 1 <= rpc) ? off : kOob;  // uniform: rows beyond the lane's halo
      d[i] = __builtin_amdgcn_raw_buffer_load_b32(rin, off, 0, 0);
    }
  }
  uint32_t de[WIDE ? kPass + 2 : 1];  // the edge lanes' extra dwords, same rows
  if constexpr (WIDE) {
    const uint32_t off0 = edge_off + (uint32_t)((y0 - 1) * W);
#pragma unroll
    for (int i = 0; i < kPass + 2; ++i) {
      uint32_t off = off0 + (uint32_t)(i * W);
      if (i >= 3) off = (i - 1 <= rpc) ? off : kOob;
      de[i] = __builtin_amdgcn_raw_buffer_load_b32(rin, off, 0, 0);
    }
  }
  const int rows_in = H + 1 - y0;  // rows 1 .. rows_in - 1 of the lane lie in the image
  struct Row { uint32_t d, edge; };  // a lane's dword of a row and, for an edge lane (which has a strip: same flip), its edge dword
  auto row = [&](int i) {
    uint32_t flip = (i == 0 ? y0 > 0 : i < rows_in) ? flip_lane : pad4;
    asm volatile("" : "+v"(flip));
    return Row{d[i] ^ flip, WIDE ? de[i] ^ flip : 0u};
  };

  // The channel's constants, through scalar loads (the addresses are the same for the whole
  // wavefront; scalar loads have their own counter, so waiting for them here, behind the row
  // loads, does not wait for a row).  The nine weights: the three aligned dwords that hold bytes
  // 9c .. 9c+8.  Each of the three holds at least one of the nine bytes, and an aligned dword
  // lies within one page, so the bytes read before and after the channel's weights are never a
  // fault.  A pointer the mode does not use is replaced by the weights' address.
  const uint32_t wb = (uint32_t)c * 9u;
  const int pc = p.per_channel ? c : 0;
  const uint32_t* wp = reinterpret_cast<const uint32_t*>(p.wgt + (wb & ~3u));
  const uint32_t* bp = p.bias ? reinterpret_cast<const uint32_t*>(p.bias + c) : wp;
  const uint32_t* mp = (MODE == 0 && p.mult) ? reinterpret_cast<const uint32_t*>(p.mult + pc) : wp;
  const uint32_t* sp = MODE == 0 ? reinterpret_cast<const uint32_t*>(p.shift + pc) : wp;
  uint64_t d01;
  uint32_t d2, bias_raw, m_raw, sh_raw;
  asm volatile(
      "s_load_dwordx2 %0, %5, 0x0\n\t"
      "s_load_dword %1, %5, 0x8\n\t"
      "s_load_dword %2, %6, 0x0\n\t"
      "s_load_dword %3, %7, 0x0\n\t"
      "s_load_dword %4, %8, 0x0\n\t"
      "s_waitcnt lgkmcnt(0)"
      : "=&s"(d01), "=&s"(d2), "=&s"(bias_raw), "=&s"(m_raw), "=&s"(sh_raw)
      : "s"(wp), "s"(bp), "s"(mp), "s"(sp));
  const uint32_t d0 = (uint32_t)d01, d1 = (uint32_t)(d01 >> 32);
  const uint32_t o8 = (wb & 3u) * 8u;
  const uint32_t w03 = (uint32_t)((((uint64_t)d1 << 32) | d0) >> o8);  // weights 0..3
  const uint32_t w47 = (uint32_t)((((uint64_t)d2 << 32) | d1) >> o8);  // weights 4..7
  const uint32_t w8 = (d2 >> o8) & 0xffu;
  int32_t wrow[3];
  wrow[0] = (int32_t)(w03 & 0xffffffu);
  wrow[1] = (int32_t)((w03 >> 24) | ((w47 & 0xffffu) << 8));
  wrow[2] = (int32_t)((w47 >> 16) | (w8 << 16));
  int32_t wsum = 0;
#pragma unroll
  for (int ky = 0; ky < 3; ++ky)
#pragma unroll
    for (int kx = 0; kx < 3; ++kx) wsum += (int32_t)(int8_t)(wrow[ky] >> (8 * kx));
  const int32_t bias = p.bias ? (int32_t)bias_raw : 0;
  // (no multiplier array: power-of-two scales, i.e. multiplier one half and the shift one less)
  const int32_t m = MODE == 0 ? (p.mult ? (int32_t)m_raw : (1 << 30)) : 0;
  const int32_t sh = MODE == 0 ? (int32_t)sh_raw - (p.mult ? 0 : 1) : 0;
  // sum (a - z) w = sum (a' + off - z) w = sum a' w + (off - z) * sum w, a' = flipped byte
  const int32_t corr = bias + (p.act_off - p.z_a) * wsum;
  const int64_t rnd = (int64_t)1 << (30 + sh);
  const int32_t z = p.rs.z_out;
  const int32_t away = p.rs.half_away ? -1 : 0;  // mask of the sign-bit correction

  // the four 3-byte windows of a strip: output x = 4q + i reads input columns x-1 .. x+1
  // The shifted copies live in two registers of their own, which start as the zero point in
  // every lane: a shift never writes the lane at the end of a DPP row it has no source for, so
  // that lane keeps the zero point from one shift to the next and needs no fresh copy.
  uint32_t left = pad4, right = pad4;
  auto windows = [&](Row r, uint32_t (&w)[4]) {
    const uint32_t d1 = r.d;
    left = (uint32_t)__builtin_amdgcn_update_dpp((int)left, (int)d1, 0x111, 0xf, 0xf, false);    // row_shr:1
    right = (uint32_t)__builtin_amdgcn_update_dpp((int)right, (int)d1, 0x101, 0xf, 0xf, false);  // row_shl:1
    if constexpr (WIDE) {
      left = left_edge ? r.edge : left;
      right = right_edge ? r.edge : right;
    }
    w[0] = __builtin_amdgcn_alignbyte(d1, left, 3);
    w[1] = d1;
    w[2] = __builtin_amdgcn_alignbyte(right, d1, 1);
    w[3] = __builtin_amdgcn_alignbyte(right, d1, 2);
  };
  // (the builtin, not inline assembly: the compiler has to see the dot instructions to keep the
  // wait states they need before a dependent instruction)
  auto dot4 = [](uint32_t a, int32_t b, int32_t c) {
    return __builtin_amdgcn_sdot4((int)a, b, c, false);
  };
  // A store beyond the image lies beyond the plane, and a strip-less lane's offset starts at
  // 2^31: both are out of the descriptor's range and dropped.
  const uint32_t so0 = has_strip ? (uint32_t)(cb + (q << 2) + y0 * W) * kEsz : kOob;

  // FOLD (requantized, 32-bit accumulator, and the channel's constants small enough): the
  // correction term, the rounding term and the output zero point all go into one 64-bit
  // constant k64, so that an output is clamp((dots * m + k64) >> (31 + sh)) against the
  // absolute bounds: (acc * m + rnd) >> s + z == (acc * m + rnd + z * 2^s) >> s exactly, and
  // acc = dots + corr cannot wrap when |corr| <= 2^30 (|dots| < 2^19).  With sh <= 19 and an
  // 8-bit z nothing here leaves 63 bits.
  // PLAIN: int8 activations with zero point 0 need no flip at all (the mask is zero everywhere)
  auto rows = [&]<bool FOLD, bool PLAIN>() {
    auto rowp = [&](int i) {
      if constexpr (PLAIN) return Row{d[i], WIDE ? de[i] : 0u};
      else return row(i);
    };
    int32_t lo = p.rs.lo_rel + (FOLD ? z : 0), hi = p.rs.hi_rel + (FOLD ? z : 0);
    // vector-register copies: v_med3 takes at most one scalar operand
    asm volatile("" : "+v"(lo), "+v"(hi));
    const int64_t k64 = FOLD ? (int64_t)corr * m + rnd + ((int64_t)z << (31 + sh)) : rnd;
    const int32_t init = FOLD ? 0 : corr;
    uint32_t w[3][4];  // windows of three consecutive rows, slot = row % 3
    windows(rowp(0), w[0]);
    windows(rowp(1), w[1]);
#pragma unroll
    for (int i = 0; i < kPass; ++i) {
      if (i < rpc) {  // uniform
        windows(rowp(i + 2), w[(i + 2) % 3]);
        int32_t acc[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          int32_t a = dot4(w[i % 3][e], wrow[0], init);
          a = dot4(w[(i + 1) % 3][e], wrow[1], a);
          a = dot4(w[(i + 2) % 3][e], wrow[2], a);
          acc[e] = ACC16 ? (int32_t)(int16_t)a : a;
        }
        const uint32_t so = so0 + (uint32_t)(i * W * kEsz);
        if constexpr (MODE == 0) {
          int32_t r[4];
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            // (general form only: halves away from zero add the accumulator's sign bit)
            const int64_t pr = (int64_t)acc[e] * (int64_t)m + k64 + (FOLD ? 0 : (int64_t)((acc[e] >> 31) & away));
            r[e] = med3((int32_t)(pr >> (31 + sh)), lo, hi) + (FOLD ? 0 : z);
          }
          __builtin_amdgcn_raw_buffer_store_b32(pack4_perm(r[0], r[1], r[2], r[3]), rout, so, 0, 0);
        } else if constexpr (MODE == 1) {
          typedef int32_t v4i32 __attribute__((ext_vector_type(4)));
          __builtin_amdgcn_raw_buffer_store_b128(v4i32{acc[0], acc[1], acc[2], acc[3]}, rout, so, 0, 0);
        } else {
          typedef uint32_t v2u32 __attribute__((ext_vector_type(2)));
          __builtin_amdgcn_raw_buffer_store_b64(
              v2u32{(uint32_t)(acc[0] & 0xffff) | ((uint32_t)acc[1] << 16),
                    (uint32_t)(acc[2] & 0xffff) | ((uint32_t)acc[3] << 16)}, rout, so, 0, 0);
        }
      }
    }
  };
  const bool fold = MODE == 0 && !ACC16 && sh >= 0 && sh <= 19 && corr >= -(1 << 30) && corr <= (1 << 30) &&
                    z >= -256 && z <= 255 && !p.rs.half_away;
  if (fold && x4 == 0 && pad4 == 0)
    rows.template operator()<true, true>();
  else if (fold)
    rows.template operator()<true, false>();
  else
    rows.template operator()<false, false>();
}

// The same register scheme for stride 2 (NCHW 3x3, pad 1, W % 4 == 0): the MobileNet
// downsampling layers.  Lane (q, rc) still loads the dword of input columns 4q .. 4q+3 of each
// input row; it yields the two outputs 2q (columns 4q-1 .. 4q+1: one byte from the left
// neighbour, by DPP) and 2q+1 (columns 4q+1 .. 4q+3), so no right neighbour is needed.  Output
// row oy reads input rows 2oy-1 .. 2oy+1; consecutive output rows share one input row, so a
// lane with rpc output rows loads 2 * rpc + 1 input rows.  The two 8-bit results of a lane are
// merged with its neighbour's into one dword store when output rows are dword-aligned
// (W % 8 == 0), else stored as 16 bits.
// MODE / ACC16 as above.
template <int MODE, bool ACC16, bool WIDE>
__global__ __launch_bounds__(kThreads) void dw_rows3x3s2_kernel(DwArgs p, int32_t rpc, int32_t nsegs) {
  // grid: x = groups of four channels, y = image, z = band of 4 * rpc output rows (and column segment)
  const ConvGeom& g = p.g;
  const int H = g.H, W = g.W, OH = g.OH, OW = g.OW;
  const int lane = threadIdx.x & 63;
  const int c = (int)(blockIdx.x * 4 + __builtin_amdgcn_readfirstlane(threadIdx.x >> 6));
  if (c >= g.C) return;  // wavefront-uniform; the kernel has no barrier
  const int64_t plane = (int64_t)blockIdx.y * g.C + c;
  const int seg = WIDE ? (int)blockIdx.z % nsegs : 0;
  const int band = WIDE ? (int)blockIdx.z / nsegs : (int)blockIdx.z;
  const int cb = seg * 64;  // first input column of the segment
  constexpr uint32_t kOob = 0x80000000u;
  constexpr int kEsz = MODE == 0 ? 1 : (MODE == 1 ? 4 : 2);
  constexpr int kPass = 16;  // most output rows per lane

  const int q = lane & 15;
  const int rc = lane >> 4;
  const int oy0 = (band * 4 + rc) * rpc;  // first output row of the lane
  const int y0 = 2 * oy0 - 1;             // its first input row
  const bool has_strip = cb + (q << 2) < W;
  const uint32_t lane_off = has_strip ? (uint32_t)(cb + (q << 2)) : kOob;
  const bool left_edge = WIDE && q == 0 && seg > 0;  // this lane's left neighbour is in the previous segment
  const uint32_t edge_off = left_edge ? (uint32_t)(cb - 4) : kOob;
  const uint32_t x4 = p.act_xor * 0x01010101u;
  const uint32_t pad4 = (((uint32_t)p.z_a ^ p.act_xor) & 0xffu) * 0x01010101u;
  const int64_t ibytes = (int64_t)H * W, obytes = (int64_t)OH * OW * kEsz;
  const __amdgpu_buffer_rsrc_t rin = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<uint8_t*>(p.act) + plane * ibytes, 0, (int)ibytes, 0x00020000);
  const __amdgpu_buffer_rsrc_t rout = __builtin_amdgcn_make_buffer_rsrc(
      static_cast<uint8_t*>(p.out) + plane * obytes, 0, (int)obytes, 0x00020000);

  // input row j of the lane is image row y0 + j; out-of-image rows and strip-less lanes read 0
  // through the descriptor's range check and become the zero point's byte under the flip mask
  uint32_t flip_lane = has_strip ? x4 : pad4;
  asm volatile("" : "+v"(flip_lane));
  uint32_t d[2 * kPass + 1];
  {
    const uint32_t off0 = lane_off + (uint32_t)(y0 * W);
#pragma unroll
    for (int j = 0; j < 2 * kPass + 1; ++j) {
      uint32_t off = off0 + (uint32_t)(j * W);
      if (j >= 3) off = (j <= 2 * rpc) ? off : kOob;  // uniform: rows the lane does not need
      d[j] = __builtin_amdgcn_raw_buffer_load_b32(rin, off, 0, 0);
    }
  }
  uint32_t de[WIDE ? 2 * kPass + 1 : 1];  // the first lane's extra dwords, same rows
  if constexpr (WIDE) {
    const uint32_t off0 = edge_off + (uint32_t)(y0 * W);
#pragma unroll
    for (int j = 0; j < 2 * kPass + 1; ++j) {
      uint32_t off = off0 + (uint32_t)(j * W);
      if (j >= 3) off = (j <= 2 * rpc) ? off : kOob;
      de[j] = __builtin_amdgcn_raw_buffer_load_b32(rin, off, 0, 0);
    }
  }
  const int rows_in = H - y0;  // rows 1 .. rows_in - 1 of the lane lie in the image (y0 >= -1)
  struct Row { uint32_t d, edge; };  // a lane's dword of a row and (first lane of a later segment) its left neighbour
  auto row = [&](int j) {
    uint32_t flip = (j == 0 ? y0 >= 0 : j < rows_in) ? flip_lane : pad4;
    asm volatile("" : "+v"(flip));
    return Row{d[j] ^ flip, WIDE ? de[j] ^ flip : 0u};
  };

  // channel constants through scalar loads, as in the stride-1 kernel
  const uint32_t wb = (uint32_t)c * 9u;
  const int pc = p.per_channel ? c : 0;
  const uint32_t* wp = reinterpret_cast<const uint32_t*>(p.wgt + (wb & ~3u));
  const uint32_t* bp = p.bias ? reinterpret_cast<const uint32_t*>(p.bias + c) : wp;
  const uint32_t* mp = (MODE == 0 && p.mult) ? reinterpret_cast<const uint32_t*>(p.mult + pc) : wp;
  const uint32_t* sp = MODE == 0 ? reinterpret_cast<const uint32_t*>(p.shift + pc) : wp;
  uint64_t d01;
  uint32_t d2, bias_raw, m_raw, sh_raw;
  asm volatile(
      "s_load_dwordx2 %0, %5, 0x0\n\t"
      "s_load_dword %1, %5, 0x8\n\t"
      "s_load_dword %2, %6, 0x0\n\t"
      "s_load_dword %3, %7, 0x0\n\t"
      "s_load_dword %4, %8, 0x0\n\t"
      "s_waitcnt lgkmcnt(0)"
      : "=&s"(d01), "=&s"(d2), "=&s"(bias_raw), "=&s"(m_raw), "=&s"(sh_raw)
      : "s"(wp), "s"(bp), "s"(mp), "s"(sp));
  const uint32_t d0 = (uint32_t)d01, d1 = (uint32_t)(d01 >> 32);
  const uint32_t o8 = (wb & 3u) * 8u;
  const uint32_t w03 = (uint32_t)((((uint64_t)d1 << 32) | d0) >> o8);  // weights 0..3
  const uint32_t w47 = (uint32_t)((((uint64_t)d2 << 32) | d1) >> o8);  // weights 4..7
  const uint32_t w8 = (d2 >> o8) & 0xffu;
  int32_t wrow[3];
  wrow[0] = (int32_t)(w03 & 0xffffffu);
  wrow[1] = (int32_t)((w03 >> 24) | ((w47 & 0xffffu) << 8));
  wrow[2] = (int32_t)((w47 >> 16) | (w8 << 16));
  int32_t wsum = 0;
#pragma unroll
  for (int ky = 0; ky < 3; ++ky)
#pragma unroll
    for (int kx = 0; kx < 3; ++kx) wsum += (int32_t)(int8_t)(wrow[ky] >> (8 * kx));
  const int32_t bias = p.bias ? (int32_t)bias_raw : 0;
  // (no multiplier array: power-of-two scales, i.e. multiplier one half and the shift one less)
  const int32_t m = MODE == 0 ? (p.mult ? (int32_t)m_raw : (1 << 30)) : 0;
  const int32_t sh = MODE == 0 ? (int32_t)sh_raw - (p.mult ? 0 : 1) : 0;
  const int32_t corr = bias + (p.act_off - p.z_a) * wsum;
  const int64_t rnd = (int64_t)1 << (30 + sh);
  const int32_t z = p.rs.z_out;
  const int32_t away = p.rs.half_away ? -1 : 0;  // mask of the sign-bit correction

  // windows of one input row: A = columns 4q-1 .. 4q+2 (output 2q uses its first three bytes,
  // the fourth meets the zero byte of the packed weights), B = columns 4q+1 .. 4q+3
  uint32_t left = pad4;  // keeps the zero point in the lane a shift has no source for
  auto windows = [&](Row r, uint32_t (&w)[2]) {
    const uint32_t d1 = r.d;
    left = (uint32_t)__builtin_amdgcn_update_dpp((int)left, (int)d1, 0x111, 0xf, 0xf, false);  // row_shr:1
    if constexpr (WIDE) left = left_edge ? r.edge : left;
    w[0] = __builtin_amdgcn_alignbyte(d1, left, 3);
    w[1] = d1 >> 8;
  };
  auto dot4 = [](uint32_t a, int32_t b, int32_t c) {
    return __builtin_amdgcn_sdot4((int)a, b, c, false);
  };
  const bool merge = (OW & 3) == 0;  // output rows start on dwords: even lanes store four results
  // outputs 2q, 2q+1 of row oy0 + i; out-of-range rows lie beyond the plane (dropped)
  const uint32_t so0 = has_strip ? (uint32_t)(cb / 2 + 2 * q + oy0 * OW) * kEsz : kOob;
  const uint32_t so0_even = (has_strip && (q & 1) == 0) ? so0 : kOob;

  // PLAIN: int8 activations with zero point 0 need no flip at all (the mask is zero everywhere)
  auto rows = [&]<bool FOLD, bool PLAIN>() {
    auto rowp = [&](int i) {
      if constexpr (PLAIN) return Row{d[i], WIDE ? de[i] : 0u};
      else return row(i);
    };
    int32_t lo = p.rs.lo_rel + (FOLD ? z : 0), hi = p.rs.hi_rel + (FOLD ? z : 0);
    asm volatile("" : "+v"(lo), "+v"(hi));
    const int64_t k64 = FOLD ? (int64_t)corr * m + rnd + ((int64_t)z << (31 + sh)) : rnd;
    const int32_t init = FOLD ? 0 : corr;
    uint32_t w[3][2];  // windows of input rows 2i, 2i+1, 2i+2: slot = row % 3 over the unrolled loop
    windows(rowp(0), w[0]);
#pragma unroll
    for (int i = 0; i < kPass; ++i) {
      if (i < rpc) {  // uniform
        // rows 2i (slot a), 2i+1 (slot b), 2i+2 (slot cc); the last is the next output's first
        const int a = (2 * i) % 3, b = (2 * i + 1) % 3, cc = (2 * i + 2) % 3;
        windows(rowp(2 * i + 1), w[b]);
        windows(rowp(2 * i + 2), w[cc]);
        int32_t acc[2];
#pragma unroll
        for (int e = 0; e < 2; ++e) {
          int32_t v = dot4(w[a][e], wrow[0], init);
          v = dot4(w[b][e], wrow[1], v);
          v = dot4(w[cc][e], wrow[2], v);
          acc[e] = ACC16 ? (int32_t)(int16_t)v : v;
        }
        const uint32_t step = (uint32_t)(i * OW * kEsz);
        if constexpr (MODE == 0) {
          int32_t r[2];
#pragma unroll
          for (int e = 0; e < 2; ++e) {
            // (general form only: halves away from zero add the accumulator's sign bit)
            const int64_t pr = (int64_t)acc[e] * (int64_t)m + k64 + (FOLD ? 0 : (int64_t)((acc[e] >> 31) & away));
            r[e] = med3((int32_t)(pr >> (31 + sh)), lo, hi) + (FOLD ? 0 : z);
          }
          const uint32_t h16 = ((uint32_t)r[0] & 0xffu) | (((uint32_t)r[1] & 0xffu) << 8);
          if (merge) {
            const uint32_t nb = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)h16, 0x101, 0xf, 0xf, true);  // row_shl:1
            __builtin_amdgcn_raw_buffer_store_b32(h16 | (nb << 16), rout, so0_even + (so0_even != kOob ? step : 0u), 0, 0);
          } else {
            __builtin_amdgcn_raw_buffer_store_b16((short)h16, rout, so0 + (so0 != kOob ? step : 0u), 0, 0);
          }
        } else if constexpr (MODE == 1) {
          typedef int32_t v2i32 __attribute__((ext_vector_type(2)));
          __builtin_amdgcn_raw_buffer_store_b64(v2i32{acc[0], acc[1]}, rout, so0 + (so0 != kOob ? step : 0u), 0, 0);
        } else {
          __builtin_amdgcn_raw_buffer_store_b32(((uint32_t)acc[0] & 0xffffu) | ((uint32_t)acc[1] << 16), rout,
                                                so0 + (so0 != kOob ? step : 0u), 0, 0);
        }
      }
    }
  };
  const bool fold = MODE == 0 && !ACC16 && sh >= 0 && sh <= 19 && corr >= -(1 << 30) && corr <= (1 << 30) &&
                    z >= -256 && z <= 255 && !p.rs.half_away;
  if (fold && x4 == 0 && pad4 == 0)
    rows.template operator()<true, true>();
  else if (fold)
    rows.template operator()<true, false>();
  else
    rows.template operator()<false, false>();
}

// Small planes (NCHW 3x3 stride 1 pad 1, W <= 16, H <= 64, any alignment): the late layers of the
// mobile networks (14 x 14, 7 x 7).  With one plane per wavefront three quarters of the lanes
// would idle, so the 16 lanes of a DPP row are shared by pp = 16 / nstrips planes (nstrips =
// strips of four columns per image row); the four DPP rows are the row quarters as in the
// register kernel.  Rows start at any byte, so a lane's dword is cut out of the two aligned
// dwords around it; bytes beyond the image row and rows outside the image become the zero
// point under a byte mask; the shifts stop at plane boundaries by a select.  Everything that
// depends on the channel is per lane here (weights, bias, multiplier, shift), so the requantize
// is the general form.  Loads and stores go through descriptors of the whole tensors with
// out-of-range offsets for everything that does not exist.
template <int MODE, bool ACC16>
__global__ __launch_bounds__(kThreads) void dw_small3x3_kernel(DwArgs p, int32_t nstrips, int32_t pp, int32_t rpc,
                                                               int64_t planes, uint32_t in_bytes,
                                                               uint32_t out_bytes) {
  const ConvGeom& g = p.g;
  const int H = g.H, W = g.W;
  const int lane = threadIdx.x & 63;
  const int64_t group = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  constexpr uint32_t kOob = 0x80000000u;
  constexpr int kEsz = MODE == 0 ? 1 : (MODE == 1 ? 4 : 2);
  constexpr int kPass = 16;  // most output rows per lane

  const int q = lane & 15;
  const int rc = lane >> 4;
  const int pl = q / nstrips;        // plane of the group
  const int sq = q - pl * nstrips;   // strip of the plane
  const int64_t plane64 = group * pp + pl;
  const bool active = pl < pp && plane64 < planes;
  const uint32_t plane = active ? (uint32_t)plane64 : 0u;  // planes * H * W < 2^31
  const int c = (int)(plane % (uint32_t)g.C);
  const int x0 = sq << 2;
  const int y0 = rc * rpc;
  const uint32_t x4 = p.act_xor * 0x01010101u;
  const uint32_t pad4 = (((uint32_t)p.z_a ^ p.act_xor) & 0xffu) * 0x01010101u;
  // (the input's range ends with the aligned dword that holds its last byte: a dword that
  // reaches past the range would read as zero as a whole, and an aligned dword lies in one page)
  const __amdgpu_buffer_rsrc_t rin = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<uint8_t*>(p.act), 0, (int)((in_bytes + 3u) & ~3u), 0x00020000);
  const __amdgpu_buffer_rsrc_t rout = __builtin_amdgcn_make_buffer_rsrc(p.out, 0, (int)out_bytes, 0x00020000);

  // row i of the lane is image row y0 + i - 1: the two aligned dwords around its strip
  const uint32_t base = plane * (uint32_t)(H * W) + (uint32_t)x0;
  uint32_t dlo[kPass + 2], dhi[kPass + 2];
#pragma unroll
  for (int i = 0; i < kPass + 2; ++i) {
    const int y = y0 + i - 1;
    const bool ok = active && (uint32_t)y < (uint32_t)H && i - 1 <= rpc;
    const uint32_t a = base + (uint32_t)(y * W);
    dlo[i] = __builtin_amdgcn_raw_buffer_load_b32(rin, ok ? (a & ~3u) : kOob, 0, 0);
    dhi[i] = __builtin_amdgcn_raw_buffer_load_b32(rin, ok ? (a & ~3u) + 4u : kOob, 0, 0);
  }
  // the bytes of the strip that lie inside the image row
  const int nv = W - x0;
  const uint32_t colmask = nv >= 4 ? 0xffffffffu : (nv <= 0 ? 0u : (1u << (8 * nv)) - 1u);
  auto row = [&](int i) {
    const int y = y0 + i - 1;
    const bool ok = active && (uint32_t)y < (uint32_t)H;
    const uint32_t a = base + (uint32_t)(y * W);
    const uint32_t v = __builtin_amdgcn_alignbyte(dhi[i], dlo[i], a & 3u) ^ x4;
    const uint32_t mask = ok ? colmask : 0u;
    return (v & mask) | (pad4 & ~mask);
  };

  // per-lane channel constants
  const int8_t* wc = p.wgt + (int64_t)c * 9;
  int32_t wrow[3];
  int32_t wsum = 0;
#pragma unroll
  for (int ky = 0; ky < 3; ++ky) {
    const int32_t w0 = wc[ky * 3 + 0], w1 = wc[ky * 3 + 1], w2 = wc[ky * 3 + 2];
    wsum += w0 + w1 + w2;
    wrow[ky] = (w0 & 0xff) | ((w1 & 0xff) << 8) | ((w2 & 0xff) << 16);
  }
  const int32_t bias = p.bias ? p.bias[c] : 0;
  const int pc = p.per_channel ? c : 0;
  const int32_t m = MODE == 0 ? rq_mult(p.mult, pc) : 0;
  const int32_t sh = MODE == 0 ? rq_shift(p.mult, p.shift, pc) : 0;
  const int32_t corr = bias + (p.act_off - p.z_a) * wsum;
  const int64_t rnd = (int64_t)1 << (30 + sh);
  const int32_t z = p.rs.z_out;
  const int32_t away = p.rs.half_away ? -1 : 0;
  int32_t lo = p.rs.lo_rel, hi = p.rs.hi_rel;
  asm volatile("" : "+v"(lo), "+v"(hi));

  const bool first = sq == 0, last = sq == nstrips - 1;  // the plane's ends inside the DPP row
  auto windows = [&](uint32_t d1, uint32_t (&w)[4]) {
    uint32_t left = (uint32_t)__builtin_amdgcn_update_dpp((int)pad4, (int)d1, 0x111, 0xf, 0xf, false);   // row_shr:1
    uint32_t right = (uint32_t)__builtin_amdgcn_update_dpp((int)pad4, (int)d1, 0x101, 0xf, 0xf, false);  // row_shl:1
    left = first ? pad4 : left;
    right = last ? pad4 : right;
    w[0] = __builtin_amdgcn_alignbyte(d1, left, 3);
    w[1] = d1;
    w[2] = __builtin_amdgcn_alignbyte(right, d1, 1);
    w[3] = __builtin_amdgcn_alignbyte(right, d1, 2);
  };
  auto dot4 = [](uint32_t a, int32_t b, int32_t c) {
    return __builtin_amdgcn_sdot4((int)a, b, c, false);
  };
  uint32_t w[3][4];
  windows(row(0), w[0]);
  windows(row(1), w[1]);
#pragma unroll
  for (int i = 0; i < kPass; ++i) {
    if (i < rpc) {  // uniform
      windows(row(i + 2), w[(i + 2) % 3]);
      const int y = y0 + i;
      const bool rok = active && y < H;
      const uint32_t o0 = (plane * (uint32_t)(H * W) + (uint32_t)(y * W + x0)) * kEsz;
      int32_t v[4];
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        int32_t a = dot4(w[i % 3][e], wrow[0], corr);
        a = dot4(w[(i + 1) % 3][e], wrow[1], a);
        a = dot4(w[(i + 2) % 3][e], wrow[2], a);
        if (ACC16) a = (int32_t)(int16_t)a;
        if constexpr (MODE == 0) {
          const int64_t pr = (int64_t)a * (int64_t)m + rnd + (int64_t)((a >> 31) & away);
          a = med3((int32_t)(pr >> (31 + sh)), lo, hi) + z;
        }
        v[e] = a;
      }
      auto off = [&](int e) { return (rok && x0 + e < W) ? o0 + (uint32_t)(e * kEsz) : kOob; };
      if constexpr (MODE == 0) {
        // whole strips as one dword when rows are dword-aligned, pairs when they are 2-byte
        // aligned (a pair is inside the row or outside), else single bytes
        if ((W & 3) == 0) {
          __builtin_amdgcn_raw_buffer_store_b32(pack4_perm(v[0], v[1], v[2], v[3]), rout, off(0), 0, 0);
        } else if ((W & 1) == 0) {
          __builtin_amdgcn_raw_buffer_store_b16((short)(((uint32_t)v[0] & 0xffu) | (((uint32_t)v[1] & 0xffu) << 8)),
                                                rout, off(0), 0, 0);
          __builtin_amdgcn_raw_buffer_store_b16((short)(((uint32_t)v[2] & 0xffu) | (((uint32_t)v[3] & 0xffu) << 8)),
                                                rout, off(2), 0, 0);
        } else {
#pragma unroll
          for (int e = 0; e < 4; ++e) __builtin_amdgcn_raw_buffer_store_b8((uint8_t)v[e], rout, off(e), 0, 0);
        }
      } else if constexpr (MODE == 1) {
#pragma unroll
        for (int e = 0; e < 4; ++e) __builtin_amdgcn_raw_buffer_store_b32((uint32_t)v[e], rout, off(e), 0, 0);
      } else {
#pragma unroll
        for (int e = 0; e < 4; ++e) __builtin_amdgcn_raw_buffer_store_b16((short)v[e], rout, off(e), 0, 0);
      }
    }
  }
}

// Channel-last 3x3, stride 1, pad 1, C % 4 == 0, 4-byte aligned tensors.  A thread owns four
// consecutive channels (one dword per pixel) and a run of kRun output pixels along a row;
// consecutive threads own consecutive channel quads, so a wavefront's loads and stores are
// contiguous.  Per new output column the thread loads three dwords (the column's three rows),
// splits them into bytes once and keeps the last three columns in registers; the channel's
// weights, their sum, bias, multiplier and shift are fetched once per thread.  Taps outside
// the image read as the zero point.  There is no dot product across channels here, so the
// arithmetic is 36 multiply-adds per output dword.
constexpr int kNhwcRun = 8;

template <int MODE, bool ACC16>
__global__ __launch_bounds__(kThreads) void dw_nhwc3x3_kernel(DwArgs p, int32_t c4, int32_t xruns, int64_t threads,
                                                              uint32_t in_bytes) {
  const ConvGeom& g = p.g;
  const int H = g.H, W = g.W, C = g.C;
  const int64_t t = (int64_t)blockIdx.x * kThreads + threadIdx.x;
  if (t >= threads) return;
  const int cq = (int)(t % c4);
  int64_t r = t / c4;
  const int xr = (int)(r % xruns); r /= xruns;
  const int y = (int)(r % H);
  const int b = (int)(r / H);
  const int c = cq << 2;
  const int x0 = xr * kNhwcRun;
  constexpr uint32_t kOob = 0x80000000u;
  constexpr int kEsz = MODE == 0 ? 1 : (MODE == 1 ? 4 : 2);
  const __amdgpu_buffer_rsrc_t rin = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<uint8_t*>(p.act), 0, (int)in_bytes, 0x00020000);
  const uint32_t x4 = p.act_xor * 0x01010101u;
  const uint32_t pad4 = (((uint32_t)p.z_a ^ p.act_xor) & 0xffu) * 0x01010101u;

  // the four channels' weights: 36 consecutive bytes from byte 9c (c % 4 == 0: dword-aligned)
  const uint32_t* wp = reinterpret_cast<const uint32_t*>(p.wgt + (int64_t)c * 9);
  uint32_t wd[9];
#pragma unroll
  for (int i = 0; i < 9; ++i) wd[i] = wp[i];
  int32_t wt[4][9];  // [channel][tap]
  int32_t wsum[4] = {0, 0, 0, 0};
#pragma unroll
  for (int j = 0; j < 4; ++j)
#pragma unroll
    for (int k = 0; k < 9; ++k) {
      const int byte = j * 9 + k;
      wt[j][k] = (int32_t)(int8_t)(wd[byte >> 2] >> (8 * (byte & 3)));
      wsum[j] += wt[j][k];
    }
  int32_t corr[4], m[4], sh[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int pc = p.per_channel ? c + j : 0;
    corr[j] = (p.bias ? p.bias[c + j] : 0) + (p.act_off - p.z_a) * wsum[j];
    m[j] = MODE == 0 ? rq_mult(p.mult, pc) : 0;
    sh[j] = MODE == 0 ? rq_shift(p.mult, p.shift, pc) : 0;
  }
  const int32_t away = p.rs.half_away ? -1 : 0;

  // column x of the three rows y-1 .. y+1 as signed bytes per channel
  const uint32_t pix_stride = (uint32_t)C;
  const uint32_t row0 = ((uint32_t)b * (uint32_t)H) * (uint32_t)W;  // in pixels
  auto load_col = [&](int x, int32_t (&col)[3][4]) {
    uint32_t d[3];
#pragma unroll
    for (int ky = 0; ky < 3; ++ky) {
      const int iy = y + ky - 1;
      const bool ok = (uint32_t)iy < (uint32_t)H && (uint32_t)x < (uint32_t)W;
      const uint32_t off = ok ? (row0 + (uint32_t)(iy * W + x)) * pix_stride + (uint32_t)c : kOob;
      const uint32_t v = __builtin_amdgcn_raw_buffer_load_b32(rin, off, 0, 0);
      d[ky] = ok ? (v ^ x4) : pad4;
    }
#pragma unroll
    for (int ky = 0; ky < 3; ++ky)
#pragma unroll
      for (int j = 0; j < 4; ++j) col[ky][j] = (int32_t)(int8_t)(d[ky] >> (8 * j));
  };
  int32_t cols[3][3][4];  // ring of the last three columns, slot = (x + 1) % 3 over the unrolled loop
  load_col(x0 - 1, cols[0]);
  load_col(x0, cols[1]);
  uint8_t* out = static_cast<uint8_t*>(p.out);
#pragma unroll
  for (int i = 0; i < kNhwcRun; ++i) {
    const int x = x0 + i;
    load_col(x + 1, cols[(i + 2) % 3]);
    if (x < W) {
      int32_t v[4];
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        int32_t a = corr[j];
#pragma unroll
        for (int ky = 0; ky < 3; ++ky)
#pragma unroll
          for (int kx = 0; kx < 3; ++kx) a += cols[(i + kx) % 3][ky][j] * wt[j][ky * 3 + kx];
        if (ACC16) a = (int32_t)(int16_t)a;
        if constexpr (MODE == 0) {
          const int64_t pr = (int64_t)a * (int64_t)m[j] + ((int64_t)1 << (30 + sh[j])) + (int64_t)((a >> 31) & away);
          a = med3((int32_t)(pr >> (31 + sh[j])), p.rs.lo_rel, p.rs.hi_rel) + p.rs.z_out;
        }
        v[j] = a;
      }
      const int64_t o = ((((int64_t)b * H + y) * W + x) * C + c) * kEsz;
      if constexpr (MODE == 0)
        *reinterpret_cast<uint32_t*>(out + o) = pack4_perm(v[0], v[1], v[2], v[3]);
      else if constexpr (MODE == 1)
        *reinterpret_cast<int4*>(out + o) = make_int4(v[0], v[1], v[2], v[3]);
      else
        *reinterpret_cast<short4*>(out + o) = make_short4((short)v[0], (short)v[1], (short)v[2], (short)v[3]);
    }
  }
}

}  // namespace

hipError_t launch_qconv_depthwise(const GemmArgs& a, const ConvGeom& cg, hipStream_t st) {
  DwArgs p{};
  p.act = static_cast<const uint8_t*>(a.act);
  p.wgt = a.wgt;
  p.bias = a.bias;
  p.out = a.out;
  p.g = cg;
  p.act_xor = a.act_unsigned ? 0x80u : 0u;
  p.act_off = a.act_unsigned ? 128 : 0;
  p.z_a = a.act_zero_point;
  p.acc16 = a.acc16;
  p.acc_wrap_shift = a.acc_wrap_shift;
  p.has_rq = a.has_rq;
  p.out_mode = a.has_rq ? 0 : (a.acc16 ? 2 : 1);
  p.mult = a.rq.multiplier;
  p.shift = a.rq.shift;
  p.per_channel = a.rq.per_channel;
  p.rs = RequantScalars{a.rq.z_out, a.rq.clip_lo - a.rq.z_out, a.rq.clip_hi - a.rq.z_out, a.rq.half_away};

  const int64_t total = (int64_t)cg.B * cg.O * cg.OH * cg.OW;
  if (total == 0) return hipSuccess;

  const bool plane_ok = !cg.nhwc && cg.KH == 3 && cg.KW == 3 && cg.stride_h == 1 &&
                        cg.stride_w == 1 && cg.pad_h == 1 && cg.pad_w == 1;
  const int rs = ((cg.W + 12 + 3) / 4) * 4;
  const int band_rows = cg.H < kBandRows ? cg.H : kBandRows;
  const size_t lds_bytes = (size_t)(band_rows + 2) * rs;
  const int64_t planes = (int64_t)cg.B * cg.C;
  const int nband = (cg.H + kBandRows - 1) / kBandRows;
  const size_t wave_lds = (size_t)4 * (cg.H + 2) * rs;
  const size_t esz = a.has_rq ? 1 : (a.acc16 ? 2 : 4);
  const bool vec_io = (cg.W % 4 == 0) && ((reinterpret_cast<uintptr_t>(a.act) & 3u) == 0) &&
                      ((reinterpret_cast<uintptr_t>(a.out) & (4 * esz - 1)) == 0);
  // the register kernel: bands of 4 * rpc rows, one wavefront each
  const int32_t rpc = (cg.H + 3) / 4 < 16 ? (cg.H + 3) / 4 : 16;
  const int64_t nband_r = (cg.H + 4 * rpc - 1) / (4 * rpc);
  // (the wavefront-per-plane kernel rounds ties toward +infinity only)
  const bool upward = !(a.has_rq && a.rq.half_away);
  // stride 2: the register kernel for the downsampling layers
  const bool s2_ok = !cg.nhwc && cg.KH == 3 && cg.KW == 3 && cg.stride_h == 2 && cg.stride_w == 2 &&
                     cg.pad_h == 1 && cg.pad_w == 1;
  const int32_t rpc2 = (cg.OH + 3) / 4 < 16 ? (cg.OH + 3) / 4 : 16;
  const int64_t nband2 = (cg.OH + 4 * rpc2 - 1) / (4 * rpc2);
  // (the register kernels are compiled for 32- and 16-bit accumulators; 24-bit ones take the
  // kernels that wrap by a run-time width)
  const bool regs_ok = a.acc_wrap_shift == 0 || a.acc_wrap_shift == 16;
  // channel-last 3x3 stride 1 pad 1
  if (regs_ok && cg.nhwc && cg.KH == 3 && cg.KW == 3 && cg.stride_h == 1 && cg.stride_w == 1 && cg.pad_h == 1 &&
      cg.pad_w == 1 && cg.C % 4 == 0 && (reinterpret_cast<uintptr_t>(a.act) & 3u) == 0 &&
      (reinterpret_cast<uintptr_t>(a.wgt) & 3u) == 0 && (reinterpret_cast<uintptr_t>(a.out) & (4 * esz - 1)) == 0 &&
      (int64_t)cg.B * cg.C * cg.H * cg.W < (1ll << 31)) {
    const int32_t c4 = cg.C / 4, xruns = (cg.W + kNhwcRun - 1) / kNhwcRun;
    const int64_t threads = (int64_t)cg.B * cg.H * xruns * c4;
    if ((threads + kThreads - 1) / kThreads < (1ll << 31)) {
      auto kern = p.out_mode == 1 ? dw_nhwc3x3_kernel<1, false>
                : p.out_mode == 2 ? dw_nhwc3x3_kernel<2, true>
                : p.acc16 ? dw_nhwc3x3_kernel<0, true> : dw_nhwc3x3_kernel<0, false>;
      hipLaunchKernelGGL(kern, dim3((unsigned)((threads + kThreads - 1) / kThreads)), dim3(kThreads), 0, st, p, c4,
                         xruns, threads, (uint32_t)((int64_t)cg.B * cg.C * cg.H * cg.W));
      return hipGetLastError();
    }
  }
  // small planes: several planes share the 16 lanes of a DPP row
  if (regs_ok && plane_ok && cg.W <= 16 && cg.H <= 64 && total * (int64_t)esz < (1ll << 31) &&
      (int64_t)cg.B * cg.C * cg.H * cg.W < (1ll << 31) &&
      (reinterpret_cast<uintptr_t>(a.act) & 3u) == 0 && (reinterpret_cast<uintptr_t>(a.out) & 3u) == 0) {
    const int32_t nstrips = (cg.W + 3) / 4, pp = 16 / nstrips;
    const int64_t groups = (planes + pp - 1) / pp;
    if ((groups + 3) / 4 < (1ll << 31)) {
      auto kern = p.out_mode == 1 ? dw_small3x3_kernel<1, false>
                : p.out_mode == 2 ? dw_small3x3_kernel<2, true>
                : p.acc16 ? dw_small3x3_kernel<0, true> : dw_small3x3_kernel<0, false>;
      hipLaunchKernelGGL(kern, dim3((unsigned)((groups + 3) / 4)), dim3(kThreads), 0, st, p, nstrips, pp,
                         (int32_t)((cg.H + 3) / 4), planes, (uint32_t)((int64_t)cg.B * cg.C * cg.H * cg.W),
                         (uint32_t)(total * (int64_t)esz));
      return hipGetLastError();
    }
  }
  const int32_t nsegs = (cg.W + 63) / 64;  // column segments of the register kernels
  if (regs_ok && s2_ok && cg.W % 4 == 0 && (reinterpret_cast<uintptr_t>(a.act) & 3u) == 0 &&
      (reinterpret_cast<uintptr_t>(a.out) & 7u) == 0 && (reinterpret_cast<uintptr_t>(a.wgt) & 3u) == 0 &&
      cg.B <= 65535 && nband2 * nsegs <= 65535 && (int64_t)cg.H * cg.W * 4 < (1ll << 31) &&
      (int64_t)cg.C * 9 < (1ll << 30)) {
    auto kern = nsegs > 1 ? (p.out_mode == 1 ? dw_rows3x3s2_kernel<1, false, true>
                             : p.out_mode == 2 ? dw_rows3x3s2_kernel<2, true, true>
                             : p.acc16 ? dw_rows3x3s2_kernel<0, true, true> : dw_rows3x3s2_kernel<0, false, true>)
                          : (p.out_mode == 1 ? dw_rows3x3s2_kernel<1, false, false>
                             : p.out_mode == 2 ? dw_rows3x3s2_kernel<2, true, false>
                             : p.acc16 ? dw_rows3x3s2_kernel<0, true, false> : dw_rows3x3s2_kernel<0, false, false>);
    hipLaunchKernelGGL(kern, dim3((unsigned)((cg.C + 3) / 4), (unsigned)cg.B, (unsigned)(nband2 * nsegs)),
                       dim3(kThreads), 0, st, p, rpc2, nsegs);
    return hipGetLastError();
  }
  if (regs_ok && plane_ok && vec_io && (reinterpret_cast<uintptr_t>(a.wgt) & 3u) == 0 &&
      cg.B <= 65535 && nband_r * nsegs <= 65535 && (int64_t)cg.H * cg.W * 4 < (1ll << 31) &&
      (int64_t)cg.C * 9 < (1ll << 30)) {
    auto kern = nsegs > 1 ? (p.out_mode == 1 ? dw_rows3x3_kernel<1, false, true>
                             : p.out_mode == 2 ? dw_rows3x3_kernel<2, true, true>
                             : p.acc16 ? dw_rows3x3_kernel<0, true, true> : dw_rows3x3_kernel<0, false, true>)
                          : (p.out_mode == 1 ? dw_rows3x3_kernel<1, false, false>
                             : p.out_mode == 2 ? dw_rows3x3_kernel<2, true, false>
                             : p.acc16 ? dw_rows3x3_kernel<0, true, false> : dw_rows3x3_kernel<0, false, false>);
    hipLaunchKernelGGL(kern, dim3((unsigned)((cg.C + 3) / 4), (unsigned)cg.B, (unsigned)(nband_r * nsegs)),
                       dim3(kThreads), 0, st, p, rpc, nsegs);
  } else if (upward && plane_ok && cg.W <= 64 && wave_lds <= (size_t)kMaxLdsBytes && planes < (1ll << 32)) {
    const uint32_t w4 = vec_io ? (uint32_t)cg.W / 4 : 1u;
    const uint32_t inv_w4 = w4 > 1 ? (uint32_t)(((1ull << 32) + w4 - 1) / w4) : 0u;  // unused for w4 == 1
    hipLaunchKernelGGL(dw_wave3x3_kernel, dim3((unsigned)((planes + 3) / 4)), dim3(kThreads),
                       wave_lds, st, p, rs, inv_w4, vec_io ? 1 : 0, planes);
  } else if (plane_ok && lds_bytes <= (size_t)kMaxLdsBytes && planes * nband < (1ll << 31)) {
    hipLaunchKernelGGL(dw_plane3x3_kernel, dim3((unsigned)(planes * nband)), dim3(kThreads),
                       lds_bytes, st, p, rs, nband, vec_io ? 1 : 0);
  } else {
    const int64_t blocks = (total + kThreads - 1) / kThreads;
    const int64_t cap = 256 * 64;
    hipLaunchKernelGGL(dw_direct_kernel, dim3((unsigned)(blocks < cap ? blocks : cap)),
                       dim3(kThreads), 0, st, p);
  }
  return hipGetLastError();
}

}  // namespace hago
