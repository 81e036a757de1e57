// 1x1 convolution (stride 1, no padding, groups == 1) on NCHW tensors, straight from the
// caller's buffers: out[b][n][p] = sum_c (a[b][c][p] - z_a) * w[n][c] + bias[n], p = y * W + x.
//
// In NCHW the reduction index c is the slow one, while the MFMA wants, per lane, 16
// consecutive k-bytes of one row.  The general convolution path therefore rewrites the input
// into a channel-last copy first, which for this operator (few output channels, so hardly any
// reuse of the input) costs more memory traffic than the convolution itself.  Here a
// wavefront owns 32 consecutive pixels of one image.  A lane loads dwords (four consecutive
// pixels of one channel); the four lanes of a quad load four consecutive channels of the same
// four pixels and transpose that 4x4 byte block among themselves (two DPP quad permutes and two
// byte permutes), after which each lane holds four consecutive channels of ITS pixel: one dword
// of its MFMA operand.  Each input byte is fetched once, 256 bytes per load instruction.
// The MFMA runs with the pixels as its P operand: a lane then owns one output channel and, per
// group of four accumulator registers, four consecutive pixels, which are packed and stored
// together.  The work is bound by memory, not by the matrix pipe (an output channel tile does
// 1/32 of an MFMA per pixel and k-step).
//
// All loads of a few k-steps (32 channels each) are issued before the first is used.
// Out-of-range channels and pixels are fetched through buffer descriptors with out-of-range
// offsets (they read as 0; the weights of padded channels are 0 as well).
#include "hago_device.h"
#include "launch.h"

namespace hago {

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

constexpr uint32_t kOob = 0x80000000u;

struct PwArgs {
  const uint8_t* act;
  const int8_t* wgt;
  const int32_t* bias;
  void* out;
  const int32_t* mult;
  const int32_t* shift;
  int32_t B, C, HW, N;
  int32_t tiles_per_img;
  int64_t tiles;
  uint32_t act_xor4;   // 0x80808080 for uint8 activations
  int32_t corr_coef;   // off - z_a
  int32_t per_channel;
  RequantScalars rs;
};

// MODE 0: requantized 8-bit, 1: raw int32, 2: raw int16; ACC16: accumulator wraps to 16 bits;
// NT: 32-channel tiles per wavefront (N <= 32 * NT).
template <int MODE, bool ACC16, int NT>
__global__ __launch_bounds__(256) void pw_nchw_kernel(PwArgs p) {
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int64_t tile = (int64_t)blockIdx.x * 4 + wave;
  if (tile >= p.tiles) return;  // wavefront-uniform; the kernel has no barrier
  const int b = (int)(tile / p.tiles_per_img);
  const int pix0 = (int)(tile - (int64_t)b * p.tiles_per_img) * 32;
  const int i = lane & 31, h = lane >> 5;
  const int C = p.C, HW = p.HW, N = p.N;

  const __amdgpu_buffer_rsrc_t rin = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<uint8_t*>(p.act) + (int64_t)b * C * HW, 0, C * HW, 0x00020000);
  const __amdgpu_buffer_rsrc_t rw = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<int8_t*>(p.wgt), 0, N * C, 0x00020000);
  // the quad's four pixels (H * W % 4 == 0: all inside the image or all outside); + channel * HW
  const int q = lane & 3;
  const uint32_t a_lane = (pix0 + (i & ~3) < HW) ? (uint32_t)(pix0 + (i & ~3)) : kOob;
  // byte selectors of the two transpose steps (own dword in S1: bytes 0-3, partner's in S0: 4-7)
  const uint32_t sel1 = (q & 2) ? 0x03020706u : 0x05040100u;  // halves swapped with lane q ^ 2
  const uint32_t sel2 = (q & 1) ? 0x03070105u : 0x06020400u;  // bytes swapped with lane q ^ 1
  uint32_t w_lane[NT];                                                    // + k
#pragma unroll
  for (int t = 0; t < NT; ++t) w_lane[t] = (t * 32 + i < N) ? (uint32_t)((t * 32 + i) * C) : kOob;

  // the lane's output channels: requantize parameters (used at the very end)
  int32_t bias_r[NT], mult_r[NT], shift_r[NT];
#pragma unroll
  for (int t = 0; t < NT; ++t) {
    const int n = t * 32 + i;
    bias_r[t] = 0; mult_r[t] = 0; shift_r[t] = 0;
    if (n < N) {
      if (p.bias) bias_r[t] = p.bias[n];
      if (MODE == 0) {
        mult_r[t] = rq_mult(p.mult, p.per_channel ? n : 0);
        shift_r[t] = rq_shift(p.mult, p.shift, p.per_channel ? n : 0);
      }
    }
  }

  v16i acc[NT];
  int32_t wsum[NT];
#pragma unroll
  for (int t = 0; t < NT; ++t) {
    wsum[t] = 0;
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[t][r] = 0;
  }
  // k-steps whose loads are in flight together (fewer with more accumulators, for registers)
  constexpr int kChunk = NT == 4 ? 4 : 6;
  const int ksteps = (C + 31) >> 5;
  for (int s0 = 0; s0 < ksteps; s0 += kChunk) {
    uint32_t ab[kChunk][4];
    v4i wb[kChunk][NT];
#pragma unroll
    for (int u = 0; u < kChunk; ++u) {
      if (s0 + u < ksteps) {  // uniform
        const int k = (s0 + u) * 32 + 16 * h;  // first channel of this lane's 16 (C % 16 == 0)
        const bool kok = k < C;
#pragma unroll
        for (int d = 0; d < 4; ++d)  // channel k + 4d + q, four pixels
          ab[u][d] = __builtin_amdgcn_raw_buffer_load_b32(
              rin, (kok && a_lane != kOob) ? a_lane + (uint32_t)((k + 4 * d + q) * HW) : kOob, 0, 0);
#pragma unroll
        for (int t = 0; t < NT; ++t)
          wb[u][t] = __builtin_amdgcn_raw_buffer_load_b128(
              rw, (kok && w_lane[t] != kOob) ? w_lane[t] + (uint32_t)k : kOob, 0, 0);
      }
    }
#pragma unroll
    for (int u = 0; u < kChunk; ++u) {
      if (s0 + u < ksteps) {  // uniform
        v4i af;
#pragma unroll
        for (int d = 0; d < 4; ++d) {
          const uint32_t x = ab[u][d];  // pixels 0..3 of channel q  ->  channels 0..3 of pixel q
          const uint32_t t = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x4E, 0xf, 0xf, true);  // quad_perm [2,3,0,1]
          const uint32_t a2 = __builtin_amdgcn_perm(t, x, sel1);
          const uint32_t v = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)a2, 0xB1, 0xf, 0xf, true);  // quad_perm [1,0,3,2]
          af[d] = (int)(__builtin_amdgcn_perm(v, a2, sel2) ^ p.act_xor4);
        }
#pragma unroll
        for (int t = 0; t < NT; ++t) {
#pragma unroll
          for (int d = 0; d < 4; ++d)
            wsum[t] = __builtin_amdgcn_sdot4(wb[u][t][d], 0x01010101, wsum[t], false);
          acc[t] = __builtin_amdgcn_mfma_i32_32x32x32_i8(af, wb[u][t], acc[t], 0, 0, 0);
        }
      }
    }
  }

  // Lane l owns channel t * 32 + l % 32; registers 4g .. 4g+3 are pixels 8g + 4 * (l / 32) + 0..3.
  const RequantScalars rs = p.rs;
  constexpr int kEsz = MODE == 0 ? 1 : (MODE == 1 ? 4 : 2);
#pragma unroll
  for (int t = 0; t < NT; ++t) {
    const int n = t * 32 + i;
    const int32_t ws = wsum[t] + __shfl_xor(wsum[t], 32);  // the two k-halves of the row sums
    const int32_t corr = bias_r[t] + p.corr_coef * ws;
    const int64_t rnd = (int64_t)1 << (30 + shift_r[t]);
    uint8_t* orow = static_cast<uint8_t*>(p.out) + ((int64_t)b * N + n) * HW * kEsz;
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      const int pg = pix0 + 8 * g + 4 * h;  // HW % 4 == 0: the group is inside the image or outside
      if (n < N && pg < HW) {
        int32_t v[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          v[e] = acc[t][4 * g + e] + corr;
          if (ACC16) v[e] = (int32_t)(int16_t)v[e];
        }
        if constexpr (MODE == 0) {
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const int64_t pr = (int64_t)v[e] * (int64_t)mult_r[t] + rnd;
            v[e] = med3((int32_t)(pr >> (31 + shift_r[t])), rs.lo_rel, rs.hi_rel) + rs.z_out;
          }
          *reinterpret_cast<uint32_t*>(orow + pg) = pack4_perm(v[0], v[1], v[2], v[3]);
        } else if constexpr (MODE == 1) {
          *reinterpret_cast<int4*>(orow + (int64_t)pg * 4) = make_int4(v[0], v[1], v[2], v[3]);
        } else {
          *reinterpret_cast<short4*>(orow + (int64_t)pg * 2) =
              make_short4((short)v[0], (short)v[1], (short)v[2], (short)v[3]);
        }
      }
    }
  }
}

// N <= 32: a wavefront owns 128 consecutive pixels of one image, as four MFMA row tiles.
// Lane (i, h) loads, for each of its 16 channels (k-half h), the dword of pixels 4i .. 4i+3:
// consecutive lanes read consecutive dwords, so a load instruction covers 128 contiguous bytes
// of a channel (two channels per instruction) and every byte is fetched once.  Four 4x4 byte
// transposes inside the lane (eight byte permutes each, no lane exchange) turn the 16 dwords
// into the 16 k-bytes of each of the lane's four pixels, and pixel 4i + j becomes row i of row
// tile j: four MFMAs share one weight operand.  On the way out lane (n, h) then holds, for its
// output channel, registers (g, e) of tile j = pixel 4 * (8g + 4h + e) + j: the four tiles pack
// into one dword and the four e into 16 contiguous bytes, so a store instruction writes 32
// contiguous bytes of each channel.
template <int MODE, bool ACC16>
__global__ __launch_bounds__(64) void pw_nchw_quad_kernel(PwArgs p) {
  const int lane = threadIdx.x;
  // Workgroups go to the eight XCDs round-robin.  A channel plane is not a multiple of the
  // 128-byte line in general, so neighbouring tiles share lines; numbering the tiles so that
  // an XCD gets a run of consecutive ones lets that XCD's L2 serve the shared lines (with the
  // plain order every such line was fetched from memory by two XCDs: 1.5 times the bytes).
  int64_t tile = blockIdx.x;
  if (gridDim.y == 1) {
    const int64_t nt = gridDim.x, x = tile & 7, slot = tile >> 3;
    const int64_t qn = nt >> 3, rn = nt & 7;
    tile = x * qn + (x < rn ? x : rn) + slot;
  }
  const int b = (int)(tile / p.tiles_per_img);
  const int pix0 = (int)(tile - (int64_t)b * p.tiles_per_img) * 128;
  const int i = lane & 31, h = lane >> 5;
  const int C = p.C, HW = p.HW, N = p.N;
  // grid y: block of 32 output channels (few input channels, many output channels: the input is
  // re-read per block, from the cache)
  const int n = (int)blockIdx.y * 32 + i;  // the lane's output channel

  const __amdgpu_buffer_rsrc_t rin = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<uint8_t*>(p.act) + (int64_t)b * C * HW, 0, C * HW, 0x00020000);
  const __amdgpu_buffer_rsrc_t rw = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<int8_t*>(p.wgt), 0, N * C, 0x00020000);
  // the lane's four pixels (H * W % 4 == 0: all inside the image or all outside); + channel * HW
  const uint32_t a_lane = (pix0 + 4 * i < HW) ? (uint32_t)(pix0 + 4 * i) : kOob;
  const uint32_t w_lane = (n < N) ? (uint32_t)(n * C) : kOob;  // + k

  // the lane's output channel: requantize parameters (used at the very end)
  int32_t bias_r = 0, mult_r = 0, shift_r = 0;
  if (n < N) {
    if (p.bias) bias_r = p.bias[n];
    if (MODE == 0) {
      mult_r = rq_mult(p.mult, p.per_channel ? n : 0);
      shift_r = rq_shift(p.mult, p.shift, p.per_channel ? n : 0);
    }
  }

  v16i acc[4];
#pragma unroll
  for (int j = 0; j < 4; ++j)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[j][r] = 0;
  int32_t wsum = 0;
  constexpr int kChunk = 5;  // k-steps (32 channels each) whose loads are in flight together
  const int ksteps = (C + 31) >> 5;
  // FULL: all kChunk steps exist, so the code has no branches and the compiler waits for each
  // step's loads separately (the first MFMAs run while later steps are still arriving)
  auto chunk = [&]<bool FULL>(int s0) {
    uint32_t ab[kChunk][16];
    v4i wb[kChunk];
#pragma unroll
    for (int u = 0; u < kChunk; ++u) {
      if (FULL || s0 + u < ksteps) {  // uniform
        const int k = (s0 + u) * 32 + 16 * h;  // first channel of this lane's 16 (C % 4 == 0)
        const bool kok = k < C;
        const uint32_t a0 = (kok && a_lane != kOob) ? a_lane + (uint32_t)(k * HW) : kOob;
#pragma unroll
        for (int d = 0; d < 16; ++d)  // channel k + d, four pixels; channels beyond C are not fetched
          ab[u][d] = __builtin_amdgcn_raw_buffer_load_b32(
              rin, (a0 != kOob && k + d < C) ? a0 + (uint32_t)(d * HW) : kOob, 0, 0);
        wb[u] = __builtin_amdgcn_raw_buffer_load_b128(
            rw, (kok && w_lane != kOob) ? w_lane + (uint32_t)k : kOob, 0, 0);
      }
    }
#pragma unroll
    for (int u = 0; u < kChunk; ++u) {
      if (FULL || s0 + u < ksteps) {  // uniform
        v4i af[4];
        const int kc = (s0 + u) * 32 + 16 * h;
#pragma unroll
        for (int m = 0; m < 4; ++m) {
          // channels 4m .. 4m+3 of this group exist or not as a whole (C % 4 == 0): the ones that
          // do not must be exactly zero on both sides (the flip would make them -128, and the
          // 16-byte weight load runs into the next row)
          const uint32_t live = kc + 4 * m < C ? 0xffffffffu : 0u;
          wb[u][m] &= (int)live;
          // rows a..d = channels 4m .. 4m+3, bytes = pixels 0..3  ->  rows = pixels, bytes = channels
          const uint32_t a = ab[u][4 * m], bq = ab[u][4 * m + 1], c = ab[u][4 * m + 2], d = ab[u][4 * m + 3];
          const uint32_t t0 = __builtin_amdgcn_perm(bq, a, 0x05010400u);  // a0 b0 a1 b1
          const uint32_t t1 = __builtin_amdgcn_perm(bq, a, 0x07030602u);  // a2 b2 a3 b3
          const uint32_t t2 = __builtin_amdgcn_perm(d, c, 0x05010400u);   // c0 d0 c1 d1
          const uint32_t t3 = __builtin_amdgcn_perm(d, c, 0x07030602u);   // c2 d2 c3 d3
          af[0][m] = (int)((__builtin_amdgcn_perm(t2, t0, 0x05040100u) ^ p.act_xor4) & live);
          af[1][m] = (int)((__builtin_amdgcn_perm(t2, t0, 0x07060302u) ^ p.act_xor4) & live);
          af[2][m] = (int)((__builtin_amdgcn_perm(t3, t1, 0x05040100u) ^ p.act_xor4) & live);
          af[3][m] = (int)((__builtin_amdgcn_perm(t3, t1, 0x07060302u) ^ p.act_xor4) & live);
        }
#pragma unroll
        for (int d = 0; d < 4; ++d) wsum = __builtin_amdgcn_sdot4(wb[u][d], 0x01010101, wsum, false);
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(af[j], wb[u], acc[j], 0, 0, 0);
      }
    }
  };
  for (int s0 = 0; s0 < ksteps; s0 += kChunk) {
    if (s0 + kChunk <= ksteps)
      chunk.template operator()<true>(s0);
    else
      chunk.template operator()<false>(s0);
  }

  const RequantScalars rs = p.rs;
  constexpr int kEsz = MODE == 0 ? 1 : (MODE == 1 ? 4 : 2);
  const int32_t ws = wsum + __shfl_xor(wsum, 32);  // the two k-halves of the row sums
  const int32_t corr = bias_r + p.corr_coef * ws;
  const int64_t rnd = (int64_t)1 << (30 + shift_r);
  uint8_t* orow = static_cast<uint8_t*>(p.out) + ((int64_t)b * N + n) * HW * kEsz;
  const bool vec16 = (HW & 15) == 0 && (reinterpret_cast<uintptr_t>(p.out) & 15u) == 0;
  // FOLD (requantized, 32-bit accumulator, every lane's constants small enough): the correction
  // term, the rounding term and the output zero point go into one 64-bit constant per lane, so
  // an output is clamp((acc * m + k64) >> (31 + sh)) against the absolute bounds:
  // ((acc + corr) * m + rnd) >> s + z == (acc * m + corr * m + rnd + z * 2^s) >> s exactly, and
  // acc + corr cannot wrap when |corr| <= 2^30 and |acc| <= 2^30 (|acc| <= C * 2^15 < 2^30 for
  // C < 2^15).  With sh <= 19 and an 8-bit z nothing leaves 63 bits.
  const int32_t away = rs.half_away ? -1 : 0;  // mask of the sign-bit correction
  auto store_all = [&]<bool FOLD>() {
    const int32_t lo = rs.lo_rel + (FOLD ? rs.z_out : 0), hi = rs.hi_rel + (FOLD ? rs.z_out : 0);
    const int64_t k64 = FOLD ? (int64_t)corr * mult_r + rnd + ((int64_t)rs.z_out << (31 + shift_r)) : rnd;
    const int32_t add = FOLD ? 0 : corr;
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      uint32_t dw[4];
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const int pq = pix0 + 4 * (8 * g + 4 * h + e);  // first of the four pixels; HW % 4 == 0
        int32_t v[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          v[j] = acc[j][4 * g + e] + add;
          if (ACC16) v[j] = (int32_t)(int16_t)v[j];
        }
        if constexpr (MODE == 0) {
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            // (general form only: halves away from zero add the accumulator's sign bit)
            const int64_t pr = (int64_t)v[j] * (int64_t)mult_r + k64 + (FOLD ? 0 : (int64_t)((v[j] >> 31) & away));
            v[j] = med3((int32_t)(pr >> (31 + shift_r)), lo, hi) + (FOLD ? 0 : rs.z_out);
          }
          dw[e] = pack4_perm(v[0], v[1], v[2], v[3]);
          if (!vec16 && n < N && pq < HW) *reinterpret_cast<uint32_t*>(orow + pq) = dw[e];
        } else if constexpr (MODE == 1) {
          if (n < N && pq < HW) *reinterpret_cast<int4*>(orow + (int64_t)pq * 4) = make_int4(v[0], v[1], v[2], v[3]);
        } else {
          if (n < N && pq < HW)
            *reinterpret_cast<short4*>(orow + (int64_t)pq * 2) =
                make_short4((short)v[0], (short)v[1], (short)v[2], (short)v[3]);
        }
      }
      if constexpr (MODE == 0) {
        const int pg = pix0 + 32 * g + 16 * h;  // HW % 16 == 0: the 16 pixels are inside the image or outside
        if (vec16 && n < N && pg < HW)
          *reinterpret_cast<uint4*>(orow + pg) = make_uint4(dw[0], dw[1], dw[2], dw[3]);
      }
    }
  };
  const bool lane_ok = shift_r >= 0 && shift_r <= 19 && corr >= -(1 << 30) && corr <= (1 << 30);
  const bool fold = MODE == 0 && !ACC16 && C < (1 << 15) && rs.z_out >= -256 && rs.z_out <= 255 &&
                    !rs.half_away && __builtin_amdgcn_ballot_w64(!lane_ok) == 0;  // wavefront-uniform
  if (fold)
    store_all.template operator()<true>();
  else
    store_all.template operator()<false>();
}

template <int MODE, bool ACC16>
hipError_t launch_nt(const PwArgs& p, hipStream_t st) {
  // 128 pixels per wavefront, one wavefront per workgroup, 32 output channels per workgroup row:
  // for up to 32 output channels, and for few input channels (the input is then cheap to re-read)
  if (p.N <= 32 || (p.C <= 64 && (p.N + 31) / 32 <= 65535)) {
    PwArgs q = p;
    q.tiles_per_img = (p.HW + 127) / 128;
    q.tiles = (int64_t)p.B * q.tiles_per_img;  // < 2^31: B and H*W are 32-bit and B * H*W fits the tensor
    hipLaunchKernelGGL((pw_nchw_quad_kernel<MODE, ACC16>), dim3((unsigned)q.tiles, (unsigned)((p.N + 31) / 32)),
                       dim3(64), 0, st, q);
    return hipGetLastError();
  }
  const unsigned grid = (unsigned)((p.tiles + 3) / 4);
  if (p.N <= 64) hipLaunchKernelGGL((pw_nchw_kernel<MODE, ACC16, 2>), dim3(grid), dim3(256), 0, st, p);
  else hipLaunchKernelGGL((pw_nchw_kernel<MODE, ACC16, 4>), dim3(grid), dim3(256), 0, st, p);
  return hipGetLastError();
}

}  // namespace

// Returns false (and launches nothing) when the geometry is not this kernel's.
bool try_qconv_pointwise_nchw(const GemmArgs& a, const ConvGeom& cg, hipStream_t st, hipError_t* err) {
  const int64_t HW = (int64_t)cg.H * cg.W;
  const size_t esz = a.has_rq ? 1 : (a.acc16 ? 2 : 4);
  const bool quad = cg.O <= 32 || cg.C <= 64;  // the 128-pixel kernel (any O when C is small)
  if (a.acc_wrap_shift != 0 && a.acc_wrap_shift != 16) return false;  // 24-bit accumulators: the general path
  if (a.has_rq && a.rq.half_away && !quad) return false;  // the wider kernel: ties toward +infinity only
  if (cg.nhwc || cg.KH != 1 || cg.KW != 1 || cg.stride_h != 1 || cg.stride_w != 1 || cg.pad_h != 0 ||
      cg.pad_w != 0 || (quad ? cg.C % 4 != 0 : cg.C % 16 != 0) || HW % 4 != 0 || (!quad && cg.O > 128) ||
      (int64_t)cg.C * HW >= (1ll << 31) ||
      (int64_t)cg.O * cg.C >= (1ll << 31) || (reinterpret_cast<uintptr_t>(a.wgt) & 15u) != 0 ||
      (reinterpret_cast<uintptr_t>(a.act) & 3u) != 0 ||
      (reinterpret_cast<uintptr_t>(a.out) & (4 * esz - 1)) != 0)
    return false;
  PwArgs p{};
  p.act = static_cast<const uint8_t*>(a.act);
  p.wgt = a.wgt;
  p.bias = a.bias;
  p.out = a.out;
  p.mult = a.rq.multiplier;
  p.shift = a.rq.shift;
  p.B = cg.B; p.C = cg.C; p.HW = (int32_t)HW; p.N = cg.O;
  p.tiles_per_img = (int32_t)((HW + 31) / 32);
  p.tiles = (int64_t)cg.B * p.tiles_per_img;
  p.act_xor4 = a.act_unsigned ? 0x80808080u : 0u;
  p.corr_coef = (a.act_unsigned ? 128 : 0) - a.act_zero_point;
  p.per_channel = a.rq.per_channel;
  p.rs = RequantScalars{a.rq.z_out, a.rq.clip_lo - a.rq.z_out, a.rq.clip_hi - a.rq.z_out, a.rq.half_away};
  if (p.tiles == 0 || p.tiles / 4 >= (1ll << 31)) return false;
  if (a.has_rq) *err = a.acc16 ? launch_nt<0, true>(p, st) : launch_nt<0, false>(p, st);
  else *err = a.acc16 ? launch_nt<2, true>(p, st) : launch_nt<1, false>(p, st);
  return true;
}

}  // namespace hago
