// Measured ceilings for the benchmark report: what this chip delivers when a kernel does nothing
// but the bounding operation.  Not operators of the method; the benchmark prints them next to the
// published peaks so that a roofline fraction can also be read against what is reachable.
//   hago_probe_mfma_i8 : every wavefront issues v_mfma_i32_32x32x32_i8 back to back on operands it
//                        loaded once (real data: the achievable clock under matrix-core load
//                        depends on how many bits toggle).
//   hago_probe_copy    : a streaming copy with the access pattern of the elementwise kernels
//                        (128-bit nontemporal loads and stores, four per lane).
#include "../../include/hago.h"

#include <hip/hip_runtime.h>

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

__global__ __launch_bounds__(256) void probe_mfma_kernel(const v4i* __restrict__ operands, int32_t* __restrict__ sink,
                                                         int32_t iters) {
  // four independent accumulator tiles per wavefront, so the pipe never waits for a result
  const v4i a = operands[threadIdx.x], b = operands[256 + threadIdx.x];
  v16i acc[4];
#pragma unroll
  for (int j = 0; j < 4; ++j)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[j][r] = 0;
  for (int i = 0; i < iters; ++i) {
#pragma unroll
    for (int j = 0; j < 4; ++j) acc[j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, acc[j], 0, 0, 0);
  }
  int32_t s = 0;
#pragma unroll
  for (int j = 0; j < 4; ++j)
#pragma unroll
    for (int r = 0; r < 16; ++r) s += acc[j][r];
  if (s == 0x7fffffff) sink[0] = s;  // keeps the loop alive; practically never true
}

__global__ __launch_bounds__(256) void probe_copy_kernel(const v4i* __restrict__ src, v4i* __restrict__ dst, int64_t nvec) {
  const int64_t stride = (int64_t)gridDim.x * 256 * 4;
  for (int64_t base = (int64_t)blockIdx.x * 256 * 4 + threadIdx.x; base < nvec; base += stride) {
    v4i q[4];
#pragma unroll
    for (int u = 0; u < 4; ++u)
      if (base + u * 256 < nvec) q[u] = __builtin_nontemporal_load(src + base + u * 256);
#pragma unroll
    for (int u = 0; u < 4; ++u)
      if (base + u * 256 < nvec) __builtin_nontemporal_store(q[u], dst + base + u * 256);
  }
}

}  // namespace

extern "C" {

hago_status hago_probe_mfma_i8(const void* operands, void* sink, int32_t workgroups, int32_t iters, void* stream) {
  if (!operands || !sink) return HAGO_ERR_NULL;
  if (workgroups < 1 || workgroups > (1 << 20) || iters < 0) return HAGO_ERR_SHAPE;
  hipLaunchKernelGGL(probe_mfma_kernel, dim3((unsigned)workgroups), dim3(256), 0, static_cast<hipStream_t>(stream),
                     static_cast<const v4i*>(operands), static_cast<int32_t*>(sink), iters);
  return hipGetLastError() == hipSuccess ? HAGO_OK : HAGO_ERR_DEVICE;
}

hago_status hago_probe_copy(const void* src, void* dst, int64_t bytes, void* stream) {
  if (bytes < 0 || bytes % 16 != 0) return HAGO_ERR_SHAPE;
  if (bytes == 0) return HAGO_OK;
  if (!src || !dst) return HAGO_ERR_NULL;
  if ((reinterpret_cast<uintptr_t>(src) | reinterpret_cast<uintptr_t>(dst)) & 15u) return HAGO_ERR_PARAM;
  const int64_t nvec = bytes / 16;
  const int64_t blocks = (nvec + 1023) / 1024;
  hipLaunchKernelGGL(probe_copy_kernel, dim3((unsigned)(blocks < (1 << 30) ? blocks : (1 << 30))), dim3(256), 0,
                     static_cast<hipStream_t>(stream), static_cast<const v4i*>(src), static_cast<v4i*>(dst), nvec);
  return hipGetLastError() == hipSuccess ? HAGO_OK : HAGO_ERR_DEVICE;
}

}  // extern "C"
