// 3x3 stride-1 pad-1 convolution (groups == 1) on NCHW tensors in ONE launch, straight from the
// caller's buffers: no rewritten copy of the input, no scratch memory.
//
// The int8 matrix instruction wants 16 consecutive reduction bytes per lane, and in NCHW the
// reduction index (input channel) is the slow one.  The transposition therefore happens on the
// way into LDS: a workgroup owns TR whole output rows of one image (TR * W <= 32 * NW * AF pixels) and
// a block of up to 64 output channels.  It stages
//   - the input rows it needs, with their one-pixel halo, channel-last: [TR + 2][W + 2][C + 16]
//     bytes (uint8 inputs flipped to int8, everything outside the image filled with the zero
//     point, so padded taps contribute 0 under the zero-point identity of the GEMM kernels).  The
//     TR + 2 rows of one channel are one contiguous run in memory; a thread loads, for 16
//     channels, the dword of four pixels of that run (consecutive lanes, consecutive dwords),
//     transposes the 16 x 4 bytes in registers and writes 16 bytes per pixel;
//   - its weights, once, as [o][tap][C] (+16 bytes per o): the workgroup is persistent and walks
//     over pixel tiles with the weights resident.
// The loads of the NEXT tile are issued before the current one is multiplied and are written to
// LDS after it, so memory latency hides behind the matrix instructions and the epilogue.  The
// start-up chain is kept short the same way: the first tile's loads and the per-channel constants
// go out before the weights are fetched, and the weight sums of the zero-point term are added up
// (LDS atomics) by the threads that stage the weights, only when that term is not zero.
// The 16 bytes of padding per pixel / per output channel make the 16-byte fragment reads of 32
// consecutive pixels (or channels) conflict-free (strides of 20 or 36 dwords).  A filter tap is
// then just an address offset into the staged tile, so every input byte is fetched once.
//
// MFMA orientation: pixels are the P operand (rows of the 32x32 tile), output channels the Q
// operand, so a lane owns one output channel and, per accumulator, 16 pixels.  Row r of a 32-row
// block holds pixel perm(r) of the block, chosen so that a lane's 16 registers are 16 CONSECUTIVE
// pixels: one 16-byte store per channel.
#include "hago_device.h"
#include "launch.h"

namespace hago {

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

struct C3Params {
  const uint8_t* act;
  const int8_t* wgt;
  const int32_t* bias;
  void* out;
  const int32_t* mult;
  const int32_t* shift;
  int32_t B, C, H, W, O;
  int32_t TR;            // output rows per tile
  int32_t tiles_per_img; // ceil(H / TR)
  int32_t ntiles;        // B * tiles_per_img
  int32_t nblk;          // blocks of 64 output channels
  int32_t per_channel, has_rq, acc_wrap_shift;
  int32_t out_mode;      // 0: requantized 8-bit, 1: raw int32, 2: raw int16
  uint32_t act_xor4;     // 0x80808080 for uint8 activations
  uint32_t pad4;         // staged value of a pixel outside the image, in every byte
  int32_t corr_coef;     // off - z_a
  RequantScalars rs;
};

// row r of a 32-row block <-> pixel of the block (see the header)
__device__ __forceinline__ constexpr int pix_of_row(int r) {
  return 16 * ((r >> 2) & 1) + 4 * (r >> 3) + (r & 3);
}

// 4 channels x 4 pixels (a..d: the dwords of four consecutive channels) -> per pixel the dword
// of its four channels
__device__ __forceinline__ void transpose4(uint32_t a, uint32_t b, uint32_t c, uint32_t d, uint32_t flip,
                                           uint32_t (&o)[4]) {
  const uint32_t t0 = __builtin_amdgcn_perm(b, a, 0x05010400u);  // a0 b0 a1 b1
  const uint32_t t1 = __builtin_amdgcn_perm(b, a, 0x07030602u);  // a2 b2 a3 b3
  const uint32_t t2 = __builtin_amdgcn_perm(d, c, 0x05010400u);
  const uint32_t t3 = __builtin_amdgcn_perm(d, c, 0x07030602u);
  o[0] = __builtin_amdgcn_perm(t2, t0, 0x05040100u) ^ flip;
  o[1] = __builtin_amdgcn_perm(t2, t0, 0x07060302u) ^ flip;
  o[2] = __builtin_amdgcn_perm(t3, t1, 0x05040100u) ^ flip;
  o[3] = __builtin_amdgcn_perm(t3, t1, 0x07060302u) ^ flip;
}

// NW: wavefronts per workgroup; AF: 32-pixel MFMA row blocks per wavefront (tiles of 32 * NW * AF
// pixels); NU: staging units per thread; CK: input channels / 32.
template <int NW, int AF, int NU, int CK>
__global__ __launch_bounds__(64 * NW, NW == 4 ? 2 : 1) void conv3x3_nchw_kernel(C3Params p) {
  constexpr int NT = 64 * NW;
  extern __shared__ __attribute__((aligned(16))) uint8_t smem[];
  const int t = threadIdx.x;
  const int lane = t & 63;
  const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
  constexpr int C = 32 * CK;
  const int H = p.H, W = p.W, O = p.O;
  constexpr int Cp = C + 16;           // bytes per staged pixel
  const int Wp = W + 2;
  constexpr int wstride = 9 * C + 16;  // bytes per staged output channel
  const int HW = H * W;
  // Workgroups that share a pixel tile (one per block of output channels) read the same input,
  // and neighbouring tiles of an image share their halo rows.  Consecutive workgroup ids go round
  // the 8 XCDs, each with an L2 of its own, so the block index is taken from the id divided by 8
  // (the sharers land on one XCD) and each XCD walks a contiguous eighth of the tiles.
  int blk, tile, tile_end, tile_step;
  const int nwg = (int)gridDim.x / p.nblk;
  if (nwg % 8 == 0) {
    const int xcd = (int)blockIdx.x & 7, q = (int)blockIdx.x >> 3;
    const int per_xcd = (p.ntiles + 7) / 8;
    blk = q % p.nblk;
    tile = xcd * per_xcd + q / p.nblk;
    tile_end = (xcd + 1) * per_xcd < p.ntiles ? (xcd + 1) * per_xcd : p.ntiles;
    tile_step = nwg / 8;
  } else {
    blk = (int)blockIdx.x % p.nblk;
    tile = (int)blockIdx.x / p.nblk;
    tile_end = p.ntiles;
    tile_step = nwg;
  }
  const int o0 = blk * 64;                             // this workgroup's block of output channels

  uint8_t* s_w = smem;                                 // [64][wstride]
  uint8_t* s_in = smem + 64 * wstride;                 // [(TR + 2)][Wp][Cp]
  int32_t* s_sum = reinterpret_cast<int32_t*>(s_in + (p.TR + 2) * Wp * Cp);  // [64] weight sums

  // ---- staging units of a tile: (16-channel group, dword of the channel's run of TR + 2 rows)
  const int w4 = W >> 2;
  const int run4 = (p.TR + 2) * w4;                    // dwords per channel run
  const int units = (C >> 4) * run4;
  uint32_t raw[NU][16];                                // as loaded: [unit][channel] = four pixels
  int u_row[NU], u_off[NU];                            // row inside the tile (-1: no unit), LDS byte offset of the first pixel
  uint32_t u_src[NU];                                  // byte offset of the unit's first channel row start + column
#pragma unroll
  for (int n = 0; n < NU; ++n) {
    const int u = t + NT * n;
    u_row[n] = -1; u_off[n] = 0; u_src[n] = 0;
    if (u < units) {
      const int c16 = u / run4, d = u - c16 * run4;
      const int r = d / w4, x4 = d - r * w4;
      u_row[n] = r;
      u_off[n] = (r * Wp + 1 + 4 * x4) * Cp + 16 * c16;
      u_src[n] = (uint32_t)(c16 * 16) * (uint32_t)HW + (uint32_t)(4 * x4);   // + (y0 - 1 + r) * W
    }
  }
  auto load_tile = [&](int tile) {
    const int b = tile / p.tiles_per_img;
    const int y0 = (tile - b * p.tiles_per_img) * p.TR;
    const uint8_t* img = p.act + (int64_t)b * C * HW;
#pragma unroll
    for (int n = 0; n < NU; ++n) {
      const int iy = y0 - 1 + u_row[n];
      const bool ok = u_row[n] >= 0 && (unsigned)iy < (unsigned)H;
#pragma unroll
      for (int k = 0; k < 16; ++k)
        raw[n][k] = ok ? *reinterpret_cast<const uint32_t*>(img + u_src[n] + (uint32_t)(iy * W) + (uint32_t)k * (uint32_t)HW)
                       : p.pad4;
    }
  };
  auto store_tile = [&](int tile) {
    const int b = tile / p.tiles_per_img;
    const int y0 = (tile - b * p.tiles_per_img) * p.TR;
#pragma unroll
    for (int n = 0; n < NU; ++n) {
      if (u_row[n] < 0) continue;
      const int iy = y0 - 1 + u_row[n];
      const uint32_t flip = (unsigned)iy < (unsigned)H ? p.act_xor4 : 0u;   // padding is staged as it is
      uint32_t px[4][4];   // [channel quad][pixel]
#pragma unroll
      for (int g = 0; g < 4; ++g) transpose4(raw[n][4 * g], raw[n][4 * g + 1], raw[n][4 * g + 2], raw[n][4 * g + 3], flip, px[g]);
#pragma unroll
      for (int i = 0; i < 4; ++i)
        *reinterpret_cast<uint4*>(s_in + u_off[n] + i * Cp) = make_uint4(px[0][i], px[1][i], px[2][i], px[3][i]);
    }
    // the halo columns x = -1 and x = W
    const int c4n = C >> 2;
    for (int u = t; u < (p.TR + 2) * 2 * c4n; u += NT) {
      const int c4 = u % c4n, rs = u / c4n;
      const int r = rs >> 1, side = rs & 1;
      *reinterpret_cast<uint32_t*>(s_in + (r * Wp + (side ? W + 1 : 0)) * Cp + 4 * c4) = p.pad4;
    }
  };
  // weight sums per output channel (only the zero-point term needs them): every thread that
  // stages weights adds its four channels' nine taps
  const bool need_sum = p.corr_coef != 0;
  if (t < 64) s_sum[t] = 0;
  __syncthreads();

  if (tile < tile_end) load_tile(tile);   // in flight while the weights are staged

  // ---- per-lane constants: output channels o0 + j and o0 + 32 + j (their loads go out now too)
  const int j = lane & 31, h = lane >> 5;
  int32_t corr[2], mu[2], sh[2];
#pragma unroll
  for (int tn = 0; tn < 2; ++tn) {
    const int o = o0 + 32 * tn + j;
    corr[tn] = 0; mu[tn] = 0; sh[tn] = 1;
    if (o < O) {
      corr[tn] = p.bias ? p.bias[o] : 0;
      if (p.has_rq) {
        mu[tn] = rq_mult(p.mult, p.per_channel ? o : 0);
        sh[tn] = rq_shift(p.mult, p.shift, p.per_channel ? o : 0);
      }
    }
  }

  // ---- weights of the block: OIHW (per o: [C][9]) -> [o][tap][C]; channels beyond O are zero.
  // A unit is four channels of one output channel: 36 contiguous bytes in memory (nine dwords when
  // the tensor is 4-byte aligned), byte 9 j + k = channel j, tap k; tap k's dword is bytes
  // (k, 9 + k, 18 + k, 27 + k), picked with three byte permutes.
  const bool w_aligned = (reinterpret_cast<uintptr_t>(p.wgt) & 3u) == 0;
  for (int i = t; i < 64 * (C / 4); i += NT) {
    const int o = i / (C / 4), c4 = (i - o * (C / 4)) * 4;
    uint32_t tap[9] = {0, 0, 0, 0, 0, 0, 0, 0, 0};
    if (o0 + o < O) {
      const int8_t* src = p.wgt + ((int64_t)(o0 + o) * C + c4) * 9;
      if (w_aligned) {
        uint32_t dw[9];
#pragma unroll
        for (int k = 0; k < 9; ++k) dw[k] = reinterpret_cast<const uint32_t*>(src)[k];
#pragma unroll
        for (int k = 0; k < 9; ++k) {
          // selector bytes: 0-3 pick from the second operand, 4-7 from the first
          constexpr uint32_t kKeep = 0x0c0c0000u;  // upper half zero
          const int i0 = k, i1 = 9 + k, i2 = 18 + k, i3 = 27 + k;
          const uint32_t lo = __builtin_amdgcn_perm(dw[i1 >> 2], dw[i0 >> 2], kKeep | (uint32_t)(i0 & 3) | ((uint32_t)(4 + (i1 & 3)) << 8));
          const uint32_t hi = __builtin_amdgcn_perm(dw[i3 >> 2], dw[i2 >> 2], kKeep | (uint32_t)(i2 & 3) | ((uint32_t)(4 + (i3 & 3)) << 8));
          tap[k] = __builtin_amdgcn_perm(hi, lo, 0x05040100u);
        }
      } else {
#pragma unroll
        for (int jj = 0; jj < 4; ++jj)
#pragma unroll
          for (int k = 0; k < 9; ++k) tap[k] |= (uint32_t)(uint8_t)src[jj * 9 + k] << (8 * jj);
      }
    }
    int32_t part = 0;
#pragma unroll
    for (int k = 0; k < 9; ++k) {
      *reinterpret_cast<uint32_t*>(s_w + o * wstride + k * C + c4) = tap[k];
      part = __builtin_amdgcn_sdot4((int)tap[k], 0x01010101, part, false);
    }
    if (need_sum) atomicAdd(&s_sum[o], part);
  }
  __syncthreads();
  bool lane_ok = true;   // the folded requantize arithmetic is exact for this lane's channels
#pragma unroll
  for (int tn = 0; tn < 2; ++tn) {
    if (o0 + 32 * tn + j < O) corr[tn] += p.corr_coef * s_sum[32 * tn + j];
    lane_ok = lane_ok && sh[tn] >= 1 && sh[tn] <= 19 && corr[tn] >= -(1 << 30) && corr[tn] <= (1 << 30);
  }
  // FOLD (requantized, 32-bit accumulator, every lane's constants small enough): correction term,
  // rounding term and output zero point go into one 64-bit constant per lane and channel, the
  // result is the high dword of acc * m + k64 shifted by sh - 1 (the shift distance is >= 32),
  // clamped BEFORE that shift against limits scaled by 2^(sh-1), so that the shift can drop each
  // result straight into its byte of the output dword.  |acc| <= 9 C 2^14 < 2^30 and
  // |corr| <= 2^30, so acc + corr cannot wrap; with sh <= 19 and an 8-bit z nothing leaves 63 bits.
  const bool fold = p.out_mode == 0 && p.acc_wrap_shift == 0 && !p.rs.half_away && p.rs.z_out >= -256 &&
                    p.rs.z_out <= 255 && __builtin_amdgcn_ballot_w64(!lane_ok) == 0;   // wavefront-uniform
  int64_t k64[2];
  int32_t lo_s[2], hi_s[2], s1[2];
#pragma unroll
  for (int tn = 0; tn < 2; ++tn) {
    s1[tn] = sh[tn] - 1;
    k64[tn] = (int64_t)corr[tn] * mu[tn] + ((int64_t)1 << (30 + (sh[tn] & 31))) + ((int64_t)p.rs.z_out << (31 + (sh[tn] & 31)));
    lo_s[tn] = clip_lo_before_shift(p.rs.lo_rel + p.rs.z_out, s1[tn] & 31);
    hi_s[tn] = clip_hi_before_shift(p.rs.hi_rel + p.rs.z_out, s1[tn] & 31);
  }

  // fragment addresses: the lane's pixels of the tile as MFMA rows
  const int pt = p.TR * W;                             // pixels of a full tile (<= 32 * NW * AF)
  uint32_t a_base[AF];
#pragma unroll
  for (int f = 0; f < AF; ++f) {
    const int q = 32 * (AF * wave + f) + pix_of_row(j);  // the lane's pixel in row block f
    const int qc = q < pt ? q : 0;                       // rows beyond the tile read pixel 0 (results dropped)
    const int qr = qc / W, qx = qc - qr * W;
    a_base[f] = (uint32_t)((qr * Wp + qx) * Cp + 16 * h);
  }
  const uint32_t b_base = (uint32_t)(j * wstride + 16 * h);

  for (; tile < tile_end; tile += tile_step) {
    const int b = tile / p.tiles_per_img;
    const int y0 = (tile - b * p.tiles_per_img) * p.TR;          // first output row
    const int rows = (H - y0 < p.TR) ? H - y0 : p.TR;            // output rows of this tile
    __syncthreads();       // the previous tile has been consumed
    store_tile(tile);      // registers -> LDS (waits for this tile's loads)
    __syncthreads();
    if (tile + tile_step < tile_end) load_tile(tile + tile_step);   // the next tile's loads go out now

    // ---- implicit GEMM: 9 taps x C / 32 steps, 2 AF MFMAs (64 output channels) per step
    v16i acc[AF][2];
#pragma unroll
    for (int f = 0; f < AF; ++f)
#pragma unroll
      for (int tn = 0; tn < 2; ++tn)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[f][tn][r] = 0;
    // Fully unrolled, the fragments of step s + 1 are requested before the matrix instructions of
    // step s are issued, so the LDS latency hides behind them; all offsets of the weight
    // fragments are immediates, a tap costs one address addition per row block.
    {
      v4i bq[2][2], aq[2][AF];
      uint32_t a_addr[AF];
      auto fetch = [&](int buf, int tap, int c) {
        bq[buf][0] = *reinterpret_cast<const v4i*>(s_w + b_base + tap * C + 32 * c);
        bq[buf][1] = *reinterpret_cast<const v4i*>(s_w + b_base + 32 * wstride + tap * C + 32 * c);
#pragma unroll
        for (int f = 0; f < AF; ++f) aq[buf][f] = *reinterpret_cast<const v4i*>(s_in + a_addr[f] + 32 * c);
      };
#pragma unroll
      for (int f = 0; f < AF; ++f) a_addr[f] = a_base[f];
      fetch(0, 0, 0);
#pragma unroll
      for (int step = 0; step < 9 * CK; ++step) {
        const int cur = step & 1;
        if (step + 1 < 9 * CK) {
          const int ntap = (step + 1) / CK, nc = (step + 1) % CK;
          if (nc == 0) {
            const int ky = ntap / 3, kx = ntap - 3 * ky;
            const uint32_t a_tap = (uint32_t)((ky * Wp + kx) * Cp);
#pragma unroll
            for (int f = 0; f < AF; ++f) a_addr[f] = a_base[f] + a_tap;
          }
          fetch(cur ^ 1, ntap, nc);
        }
        __builtin_amdgcn_sched_barrier(0);   // keep the requests ahead of this step's matrix instructions
#pragma unroll
        for (int f = 0; f < AF; ++f) {
          acc[f][0] = __builtin_amdgcn_mfma_i32_32x32x32_i8(aq[cur][f], bq[cur][0], acc[f][0], 0, 0, 0);
          acc[f][1] = __builtin_amdgcn_mfma_i32_32x32x32_i8(aq[cur][f], bq[cur][1], acc[f][1], 0, 0, 0);
        }
        __builtin_amdgcn_sched_barrier(0);
      }
    }

    // ---- epilogue: the lane's 16 consecutive pixels of channel o0 + 32 tn + j, per row block
    const int npix = rows * W;                           // valid pixels of this tile
    const bool tile16 = (npix & 15) == 0 && ((y0 * W) & 15) == 0 && (HW & 15) == 0;
#pragma unroll
    for (int f = 0; f < AF; ++f) {
      const int pix0 = 32 * (AF * wave + f) + 16 * h;    // first of the 16 pixels inside the tile
      const int64_t obase = (int64_t)b * O * HW + (int64_t)y0 * W + pix0;
      const bool full16 = tile16 && pix0 + 16 <= npix;
#pragma unroll
      for (int tn = 0; tn < 2; ++tn) {
        const int o = o0 + 32 * tn + j;
        if (o >= O || pix0 >= npix) continue;
        const int64_t oo = obase + (int64_t)o * HW;
        if (p.out_mode == 0) {
          uint8_t* dst = static_cast<uint8_t*>(p.out) + oo;
          uint32_t dw[4];
          if (fold) {
#pragma unroll
            for (int g = 0; g < 4; ++g) {
              auto one = [&]<int E>() {
                const int64_t pr = (int64_t)acc[f][tn][4 * g + E] * (int64_t)mu[tn] + k64[tn];
                ashr_into_byte<E>(dw[g], med3((int32_t)(pr >> 32), lo_s[tn], hi_s[tn]), s1[tn]);
              };
              one.template operator()<0>();
              one.template operator()<1>();
              one.template operator()<2>();
              one.template operator()<3>();
            }
          } else {
#pragma unroll
            for (int g = 0; g < 4; ++g) {
              int32_t v[4];
#pragma unroll
              for (int e = 0; e < 4; ++e) {
                int32_t a = acc[f][tn][4 * g + e] + corr[tn];
                if (p.acc_wrap_shift) a = wrap_acc_bits(a, p.acc_wrap_shift);
                v[e] = requant_general(a, mu[tn], sh[tn], p.rs);
              }
              dw[g] = pack4(v[0], v[1], v[2], v[3]);
            }
          }
          if (full16 && (reinterpret_cast<uintptr_t>(dst) & 15u) == 0) {
            *reinterpret_cast<uint4*>(dst) = make_uint4(dw[0], dw[1], dw[2], dw[3]);
          } else {
#pragma unroll
            for (int r = 0; r < 16; ++r)
              if (pix0 + r < npix) dst[r] = (uint8_t)(dw[r >> 2] >> (8 * (r & 3)));
          }
        } else {
          int32_t v[16];
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            v[r] = acc[f][tn][r] + corr[tn];
            if (p.acc_wrap_shift) v[r] = wrap_acc_bits(v[r], p.acc_wrap_shift);
          }
          if (p.out_mode == 1) {
            int32_t* dst = static_cast<int32_t*>(p.out) + oo;
            if (full16 && (reinterpret_cast<uintptr_t>(dst) & 15u) == 0) {
#pragma unroll
              for (int g = 0; g < 4; ++g)
                reinterpret_cast<int4*>(dst)[g] = make_int4(v[4 * g], v[4 * g + 1], v[4 * g + 2], v[4 * g + 3]);
            } else {
#pragma unroll
              for (int r = 0; r < 16; ++r)
                if (pix0 + r < npix) dst[r] = v[r];
            }
          } else {
            int16_t* dst = static_cast<int16_t*>(p.out) + oo;
            if (full16 && (reinterpret_cast<uintptr_t>(dst) & 15u) == 0) {
#pragma unroll
              for (int g = 0; g < 2; ++g) {
                uint32_t dq[4];
#pragma unroll
                for (int x = 0; x < 4; ++x)
                  dq[x] = ((uint32_t)v[8 * g + 2 * x] & 0xffffu) | ((uint32_t)v[8 * g + 2 * x + 1] << 16);
                reinterpret_cast<uint4*>(dst)[g] = make_uint4(dq[0], dq[1], dq[2], dq[3]);
              }
            } else {
#pragma unroll
              for (int r = 0; r < 16; ++r)
                if (pix0 + r < npix) dst[r] = (int16_t)v[r];
            }
          }
        }
      }
    }
  }
}

template <int NW, int AF, int NU, int CK>
hipError_t launch_c3_ck(const C3Params& p, size_t lds, int64_t grid, hipStream_t st) {
  static std::atomic<uint64_t> attr_set{0};
  // the LDS size depends on the geometry, not only on the template arguments: raise the kernel's
  // limit to the CU's 160 KB once, whatever this call needs
  hipError_t e = raise_lds_limit(reinterpret_cast<const void*>(conv3x3_nchw_kernel<NW, AF, NU, CK>), 160 * 1024, attr_set);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL((conv3x3_nchw_kernel<NW, AF, NU, CK>), dim3((unsigned)grid), dim3(64 * NW), lds, st, p);
  return hipGetLastError();
}

template <int NW, int AF, int NU>
hipError_t launch_c3(const C3Params& p, size_t lds, int64_t grid, hipStream_t st) {
  switch (p.C / 32) {
    case 1: return launch_c3_ck<NW, AF, NU, 1>(p, lds, grid, st);
    case 2: return launch_c3_ck<NW, AF, NU, 2>(p, lds, grid, st);
    case 3: return launch_c3_ck<NW, AF, NU, 3>(p, lds, grid, st);
    default: return launch_c3_ck<NW, AF, NU, 4>(p, lds, grid, st);
  }
}

}  // namespace

// Takes NCHW 3x3 stride-1 pad-1 convolutions with C a multiple of 32 up to 128, W a multiple of 4
// up to 128 and 4-byte aligned activations; returns false (nothing launched) for anything else.
bool try_qconv3x3_nchw(const GemmArgs& a, const ConvGeom& cg, hipStream_t st, hipError_t* err) {
  if (cg.nhwc || cg.KH != 3 || cg.KW != 3 || cg.stride_h != 1 || cg.stride_w != 1 || cg.pad_h != 1 ||
      cg.pad_w != 1 || cg.C % 32 != 0 || cg.C > 128 || cg.W % 4 != 0 || cg.W > 128 ||
      (reinterpret_cast<uintptr_t>(a.act) & 3u) != 0 || (int64_t)cg.B * cg.C * cg.H * cg.W >= (1ll << 31) ||
      (int64_t)cg.B * cg.O * cg.H * cg.W >= (1ll << 31))
    return false;
  C3Params p{};
  p.act = static_cast<const uint8_t*>(a.act);
  p.wgt = a.wgt;
  p.bias = a.bias;
  p.out = a.out;
  p.mult = a.rq.multiplier;
  p.shift = a.rq.shift;
  p.B = cg.B; p.C = cg.C; p.H = cg.H; p.W = cg.W; p.O = cg.O;
  p.nblk = (cg.O + 63) / 64;
  p.per_channel = a.rq.per_channel;
  p.has_rq = a.has_rq;
  p.acc_wrap_shift = a.acc_wrap_shift;
  p.out_mode = a.has_rq ? 0 : (a.acc16 ? 2 : 1);
  p.act_xor4 = a.act_unsigned ? 0x80808080u : 0u;
  p.pad4 = ((((uint32_t)a.act_zero_point) ^ (a.act_unsigned ? 0x80u : 0u)) & 0xffu) * 0x01010101u;
  p.corr_coef = (a.act_unsigned ? 128 : 0) - a.act_zero_point;
  p.rs = RequantScalars{a.rq.z_out, a.rq.clip_lo - a.rq.z_out, a.rq.clip_hi - a.rq.z_out, a.rq.half_away};
  // Tile shapes (wavefronts x 32-pixel row blocks per wavefront).  512 pixels cost the fewest LDS
  // bytes per matrix instruction (each wavefront owns 64 pixels x 64 channels) and are taken when
  // they still leave every CU a tile; 256 pixels on eight wavefronts otherwise; 128 pixels on four
  // where the wider tiles' rows do not fit the LDS.
  struct Shape { int nw, af; };
  static const Shape shapes[] = {{8, 2}, {8, 1}, {4, 1}};
  size_t lds = 0;
  int nu = 0, pick = -1;
  int64_t ntiles = 0;
  for (int i = 0; i < 3 && pick < 0; ++i) {
    const int pixels = 32 * shapes[i].nw * shapes[i].af, threads = 64 * shapes[i].nw;
    p.TR = pixels / cg.W < cg.H ? pixels / cg.W : cg.H;
    // whole 16-pixel groups per tile where that is possible: 16-byte stores
    int gran = 16;
    for (int wv = cg.W; (wv & 1) == 0 && gran > 1; wv >>= 1) gran >>= 1;   // 16 / gcd(W, 16)
    if (p.TR >= gran) p.TR -= p.TR % gran;
    p.tiles_per_img = (cg.H + p.TR - 1) / p.TR;
    ntiles = (int64_t)cg.B * p.tiles_per_img;
    lds = (size_t)64 * (9 * cg.C + 16) + (size_t)(p.TR + 2) * (cg.W + 2) * (cg.C + 16) + 64 * sizeof(int32_t);
    nu = ((cg.C / 16) * (p.TR + 2) * (cg.W / 4) + threads - 1) / threads;
    const bool fits = lds <= 160 * 1024 && nu <= 3 && ntiles < (1ll << 31);
    if (fits && (i > 0 || ntiles * p.nblk >= 256)) pick = i;
  }
  if (pick < 0) return false;
  p.ntiles = (int32_t)ntiles;
  // persistent workgroups: as many as fit the chip at this LDS size (two per CU at most), shared
  // out evenly among the blocks of output channels
  const int fit = (int)((160 * 1024) / lds);
  const int per_cu = fit > 2 ? 2 : fit;
  int64_t per_blk = (256ll * per_cu) / p.nblk;
  if (per_blk < 1) per_blk = 1;
  if (per_blk > ntiles) per_blk = ntiles;
  const int64_t grid = per_blk * p.nblk;
#define HAGO_C3(I, NWV, AFV, NUV) if (pick == I && nu == NUV) { *err = launch_c3<NWV, AFV, NUV>(p, lds, grid, st); return true; }
  HAGO_C3(0, 8, 2, 1) HAGO_C3(0, 8, 2, 2) HAGO_C3(0, 8, 2, 3)
  HAGO_C3(1, 8, 1, 1) HAGO_C3(1, 8, 1, 2) HAGO_C3(1, 8, 1, 3)
  HAGO_C3(2, 4, 1, 1) HAGO_C3(2, 4, 1, 2) HAGO_C3(2, 4, 1, 3)
#undef HAGO_C3
  return false;
}

}  // namespace hago
