// Operand preparation for the implicit-GEMM convolution: the rewrite of both
// operands into the caller's workspace.
//
// The int8 matrix cores want 16 consecutive reduction elements per lane.  In
// NCHW the reduction index (input channel) is the slowest-varying one, so the
// convolution first rewrites its operands, once per call and in one launch:
//   activations -> [B][H + 2 pad_h][W + 2 pad_w][Cp]   (Cp = C rounded up to 16)
//                  uint8 inputs flipped to int8 (XOR 0x80), the padding ring
//                  filled with the zero point (so padded taps contribute 0),
//                  channels beyond C zero;
//   weights     -> [O][KH * KW][Cp], channels beyond C zero.
// After that a tap of an output pixel is 16-byte chunks of contiguous memory
// and the GEMM kernel can stream both operands straight into LDS.
#include "../../include/hago.h"
#include "hago_device.h"
#include "launch.h"

#include <atomic>

// Fixed scratch of the entry point that must not allocate (hago_qconv2d_static): static device
// memory, one copy per GPU at that GPU's own address, held until the process ends.  Host code
// never uses this name as an address; static_scratch() below asks the runtime for the device
// address once per device and hands that out.
static __device__ __align__(256) unsigned char scratch[HAGO_STATIC_SCRATCH_BYTES];

namespace hago {

namespace {

struct PrepackArgs {
  const uint8_t* act;
  const int8_t* wgt;
  uint8_t* act_out;
  int8_t* wgt_out;
  int32_t B, C, H, W, O, KH, KW, ph, pw, Hp, Wp, Cp, nhwc;
  int32_t nhwc_vec;   // channel-last input whose 16-channel chunks are aligned 16-byte loads
  uint32_t act_xor;   // 0x80 for uint8 inputs
  uint32_t pad_byte;  // (zero point XOR act_xor) & 0xff
  int64_t act_chunks, wgt_chunks;  // 16-byte chunks to produce
};

__device__ __forceinline__ uint4 pack16(const uint32_t (&b)[16]) {
  uint4 r;
  r.x = b[0] | (b[1] << 8) | (b[2] << 16) | (b[3] << 24);
  r.y = b[4] | (b[5] << 8) | (b[6] << 16) | (b[7] << 24);
  r.z = b[8] | (b[9] << 8) | (b[10] << 16) | (b[11] << 24);
  r.w = b[12] | (b[13] << 8) | (b[14] << 16) | (b[15] << 24);
  return r;
}

__device__ __forceinline__ void prepack_weight_chunk(const PrepackArgs& p, int64_t k) {
  // k = (o*KH*KW + t)*nch + cc
  const int nch = p.Cp >> 4;
  const int khw = p.KH * p.KW;
  const int cc = (int)(k % nch);
  const int64_t ot = k / nch;
  const int t = (int)(ot % khw);
  const int64_t o = ot / khw;
  const int c0 = cc << 4;
  uint32_t v[16];
#pragma unroll
  for (int j = 0; j < 16; ++j) {
    const int c = c0 + j < p.C ? c0 + j : p.C - 1;
    const int64_t src = p.nhwc ? (o * khw + t) * p.C + c : (o * p.C + c) * khw + t;
    v[j] = (uint8_t)p.wgt[src];
  }
#pragma unroll
  for (int j = 0; j < 16; ++j) v[j] = (c0 + j < p.C) ? v[j] : 0u;
  *reinterpret_cast<uint4*>(p.wgt_out + (ot * p.Cp + c0)) = pack16(v);
}

__global__ __launch_bounds__(256) void conv_prepack_kernel(PrepackArgs p) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const int nch = p.Cp >> 4;
  if (i < p.act_chunks) {
    // i = ((b*Hp + py)*nch + cc)*Wp + px : lanes run along px, which is contiguous in NCHW
    int64_t r = i;
    const int px = (int)(r % p.Wp); r /= p.Wp;
    const int cc = (int)(r % nch); r /= nch;
    const int py = (int)(r % p.Hp);
    const int b = (int)(r / p.Hp);
    const int iy = py - p.ph, ix = px - p.pw;
    const bool inside = (unsigned)iy < (unsigned)p.H && (unsigned)ix < (unsigned)p.W;
    const int c0 = cc << 4;
    uint32_t v[16];
    if (p.nhwc) {
      const int64_t base = (((int64_t)b * p.H + (inside ? iy : 0)) * p.W + (inside ? ix : 0)) * p.C;
      if (p.nhwc_vec) {  // C % 16 == 0 and a 16-byte aligned tensor: the chunk is one aligned load
        const uint4 q = *reinterpret_cast<const uint4*>(p.act + base + c0);
        const uint32_t x4 = p.act_xor * 0x01010101u, pad4 = p.pad_byte * 0x01010101u;
        const uint4 r = inside ? make_uint4(q.x ^ x4, q.y ^ x4, q.z ^ x4, q.w ^ x4) : make_uint4(pad4, pad4, pad4, pad4);
        *reinterpret_cast<uint4*>(p.act_out + ((((int64_t)b * p.Hp + py) * p.Wp + px) * p.Cp) + c0) = r;
        return;
      }
#pragma unroll
      for (int j = 0; j < 16; ++j) v[j] = p.act[base + (c0 + j < p.C ? c0 + j : p.C - 1)];
    } else {
      const int64_t hw = (int64_t)p.H * p.W;
      const int64_t base = (int64_t)b * p.C * hw + (int64_t)(inside ? iy : 0) * p.W + (inside ? ix : 0);
#pragma unroll
      for (int j = 0; j < 16; ++j) v[j] = p.act[base + (int64_t)(c0 + j < p.C ? c0 + j : p.C - 1) * hw];
    }
#pragma unroll
    for (int j = 0; j < 16; ++j)
      v[j] = (c0 + j < p.C) ? (inside ? (v[j] ^ p.act_xor) : p.pad_byte) : 0u;
    const int64_t o = ((((int64_t)b * p.Hp + py) * p.Wp + px) * p.Cp) + c0;
    *reinterpret_cast<uint4*>(p.act_out + o) = pack16(v);
    return;
  }
  const int64_t k = i - p.act_chunks;
  if (k < p.wgt_chunks) prepack_weight_chunk(p, k);
}

// NCHW activations with W % 4 == 0, transposed through LDS so that both sides are coalesced.
// A workgroup owns 64 channels x 64 pixels of one image.  Thread (cq, pq) loads, for its four
// channels, the dword of its four pixels (16 threads cover 64 contiguous bytes of a channel
// plane), transposes the 4x4 byte block in registers and writes one dword per pixel into an
// LDS tile [pixel][channel] whose rows are 17 dwords apart (conflict-free writes).  Then
// thread (pixel, chunk) reads 16 channel bytes and stores them: a wavefront writes 16 pixels x
// 64 bytes, contiguous in the padded channel-last copy.  The blocks behind the interior ones
// write the padding ring and the weights, one 16-byte chunk per thread.
__global__ __launch_bounds__(256) void conv_prepack_nchw_kernel(PrepackArgs p, int32_t ptiles, int32_t ctiles,
                                                                int32_t act_blocks, int64_t ring_chunks) {
  __shared__ uint32_t tile[64 * 17];
  const int nch = p.Cp >> 4;
  if ((int)blockIdx.x < act_blocks) {
    const int t = threadIdx.x;
    const int pt = (int)blockIdx.x % ptiles;
    const int bc = (int)blockIdx.x / ptiles;
    const int ct = bc % ctiles;
    const int b = bc / ctiles;
    const int hw = p.H * p.W;
    {
      const int pq = t & 15, cq = t >> 4;
      const int pix = pt * 64 + 4 * pq;   // four pixels, inside the plane or outside (hw % 4 == 0)
      const int c0 = ct * 64 + 4 * cq;    // four channels
      const __amdgpu_buffer_rsrc_t rin = __builtin_amdgcn_make_buffer_rsrc(
          const_cast<uint8_t*>(p.act) + (int64_t)b * p.C * hw, 0, p.C * hw, 0x00020000);
      constexpr uint32_t kOob = 0x80000000u;
      uint32_t v[4];
#pragma unroll
      for (int k = 0; k < 4; ++k)  // a channel beyond C lies beyond the image's planes: reads 0
        v[k] = __builtin_amdgcn_raw_buffer_load_b32(
            rin, (pix < hw && c0 + k < p.C) ? (uint32_t)((c0 + k) * hw + pix) : kOob, 0, 0);
      const uint32_t t0 = __builtin_amdgcn_perm(v[1], v[0], 0x05010400u);  // a0 b0 a1 b1
      const uint32_t t1 = __builtin_amdgcn_perm(v[1], v[0], 0x07030602u);  // a2 b2 a3 b3
      const uint32_t t2 = __builtin_amdgcn_perm(v[3], v[2], 0x05010400u);  // c0 d0 c1 d1
      const uint32_t t3 = __builtin_amdgcn_perm(v[3], v[2], 0x07030602u);  // c2 d2 c3 d3
      const uint32_t x4 = p.act_xor * 0x01010101u;
      const int left = p.C - c0;  // channels of this dword that exist (the others stay zero)
      const uint32_t mask = left >= 4 ? 0xffffffffu : (left <= 0 ? 0u : (1u << (8 * left)) - 1u);
      tile[(4 * pq + 0) * 17 + cq] = (__builtin_amdgcn_perm(t2, t0, 0x05040100u) ^ x4) & mask;
      tile[(4 * pq + 1) * 17 + cq] = (__builtin_amdgcn_perm(t2, t0, 0x07060302u) ^ x4) & mask;
      tile[(4 * pq + 2) * 17 + cq] = (__builtin_amdgcn_perm(t3, t1, 0x05040100u) ^ x4) & mask;
      tile[(4 * pq + 3) * 17 + cq] = (__builtin_amdgcn_perm(t3, t1, 0x07060302u) ^ x4) & mask;
    }
    __syncthreads();
    const int pl = t >> 2, ch = t & 3;
    const int pix = pt * 64 + pl;
    if (pix < hw && ct * 64 + ch * 16 < p.Cp) {
      const int iy = pix / p.W, ix = pix - iy * p.W;
      const uint32_t* src = tile + pl * 17 + 4 * ch;
      *reinterpret_cast<uint4*>(p.act_out + (((int64_t)b * p.Hp + iy + p.ph) * p.Wp + ix + p.pw) * p.Cp +
                                ct * 64 + ch * 16) = make_uint4(src[0], src[1], src[2], src[3]);
    }
    return;
  }
  const int64_t i = ((int64_t)blockIdx.x - act_blocks) * 256 + threadIdx.x;
  if (i < ring_chunks) {
    // the padding ring of image b: ph rows above, pw pixels left and right of every image row,
    // ph rows below; the zero point's byte in the channels that exist
    const int ring = p.Hp * p.Wp - p.H * p.W;
    const int cc = (int)(i % nch);
    const int64_t r = i / nch;
    const int b = (int)(r / ring);
    int rr = (int)(r - (int64_t)b * ring);
    int py, px;
    const int top = p.ph * p.Wp, mid = p.H * 2 * p.pw;
    if (rr < top) {
      py = rr / p.Wp; px = rr - py * p.Wp;
    } else if (rr < top + mid) {
      rr -= top;
      const int y = rr / (2 * p.pw), k = rr - y * 2 * p.pw;
      py = p.ph + y; px = k < p.pw ? k : p.W + k;
    } else {
      rr -= top + mid;
      const int y = rr / p.Wp;
      py = p.ph + p.H + y; px = rr - y * p.Wp;
    }
    uint32_t v[16];
#pragma unroll
    for (int j = 0; j < 16; ++j) v[j] = ((cc << 4) + j < p.C) ? p.pad_byte : 0u;
    *reinterpret_cast<uint4*>(p.act_out + ((((int64_t)b * p.Hp + py) * p.Wp + px) * p.Cp) + (cc << 4)) = pack16(v);
    return;
  }
  const int64_t k = i - ring_chunks;
  if (k < p.wgt_chunks) prepack_weight_chunk(p, k);
}

}  // namespace

hipError_t static_scratch(void** ptr, int64_t* capacity) {
  static std::atomic<void*> addr[64];  // per device; zero-initialised
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= 64) return hipErrorInvalidDevice;
  void* p = addr[dev].load(std::memory_order_acquire);
  if (!p) {
    // the current device's copy of the array (two threads may both ask; they get the same answer)
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (!p) return hipErrorInvalidSymbol;
    addr[dev].store(p, std::memory_order_release);
  }
  *ptr = p;
  *capacity = (int64_t)HAGO_STATIC_SCRATCH_BYTES;
  return hipSuccess;
}

// skip_weights: the weight copy is already in place (a previous call with the same weights
// wrote it); only the activations and their padding ring are rewritten.
hipError_t launch_conv_prepack(const GemmArgs& a, const ConvGeom& cg, int32_t Cp, uint8_t* act_out,
                               int8_t* wgt_out, bool skip_weights, hipStream_t st) {
  PrepackArgs p{};
  p.act = static_cast<const uint8_t*>(a.act);
  p.wgt = a.wgt;
  p.act_out = act_out;
  p.wgt_out = wgt_out;
  p.B = cg.B; p.C = cg.C; p.H = cg.H; p.W = cg.W; p.O = cg.O; p.KH = cg.KH; p.KW = cg.KW;
  p.ph = cg.pad_h; p.pw = cg.pad_w;
  p.Hp = cg.H + 2 * cg.pad_h; p.Wp = cg.W + 2 * cg.pad_w; p.Cp = Cp;
  p.nhwc = cg.nhwc;
  p.nhwc_vec = cg.nhwc && cg.C % 16 == 0 && (reinterpret_cast<uintptr_t>(a.act) & 15u) == 0;
  p.act_xor = a.act_unsigned ? 0x80u : 0u;
  p.pad_byte = ((uint32_t)a.act_zero_point ^ p.act_xor) & 0xffu;
  p.act_chunks = (int64_t)p.B * p.Hp * p.Wp * (Cp / 16);
  p.wgt_chunks = skip_weights ? 0 : (int64_t)p.O * p.KH * p.KW * (Cp / 16);
  const int64_t hw = (int64_t)cg.H * cg.W;
  if (!cg.nhwc && cg.W % 4 == 0 && (reinterpret_cast<uintptr_t>(a.act) & 3u) == 0 &&
      (int64_t)cg.C * hw < (1ll << 31)) {
    const int64_t ptiles = (hw + 63) / 64, ctiles = (Cp + 63) / 64;
    const int64_t act_blocks = (int64_t)cg.B * ctiles * ptiles;
    const int64_t ring_chunks = (int64_t)p.B * ((int64_t)p.Hp * p.Wp - hw) * (Cp / 16);
    const int64_t blocks = act_blocks + (ring_chunks + p.wgt_chunks + 255) / 256;
    if (blocks < (1ll << 31)) {
      hipLaunchKernelGGL(conv_prepack_nchw_kernel, dim3((unsigned)blocks), dim3(256), 0, st, p,
                         (int32_t)ptiles, (int32_t)ctiles, (int32_t)act_blocks, ring_chunks);
      return hipGetLastError();
    }
  }
  const int64_t blocks = (p.act_chunks + p.wgt_chunks + 255) / 256;
  hipLaunchKernelGGL(conv_prepack_kernel, dim3((unsigned)blocks), dim3(256), 0, st, p);
  return hipGetLastError();
}

}  // namespace hago
