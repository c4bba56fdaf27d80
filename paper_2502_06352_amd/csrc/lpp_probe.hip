// Measurement aid, not a step of the method: a plain streaming read of a device buffer, the
// ceiling against which the HBM-bound kernels of this library are read (their roofline is
// "bytes the method must move / time"; this says how fast the memory system delivers bytes to
// compute units when nothing else is asked of them).
#include "lpp_internal.h"

namespace {

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

// Every lane streams 16-byte chunks, eight loads in flight, and folds them into one word that is
// written only if it matches a value it cannot have by accident: the loads cannot be dropped, and
// nothing is written.
__global__ __launch_bounds__(256) void stream_read_kernel(const u32x4* src, size_t n16, uint32_t* sink) {
  const size_t stride = (size_t)gridDim.x * 256;
  size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  uint32_t acc = 0;
  for (; i + 7 * stride < n16; i += 8 * stride) {
    u32x4 v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) v[u] = __builtin_nontemporal_load(src + i + u * stride);
#pragma unroll
    for (int u = 0; u < 8; ++u) acc ^= v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
  }
  for (; i < n16; i += stride) {
    const u32x4 v = __builtin_nontemporal_load(src + i);
    acc ^= v.x ^ v.y ^ v.z ^ v.w;
  }
  if (acc == 0x9E3779B9u && sink) sink[0] = acc;
}

}  // namespace

extern "C" int32_t lpp_probe_stream_read(const void* src, size_t bytes, uint32_t* sink, int32_t blocks,
                                         void* stream) {
  if (!src || bytes < 16 || blocks < 1 || blocks > (1 << 20)) return LPP_EINVAL;
  if (reinterpret_cast<uintptr_t>(src) % 16 != 0) return LPP_EINVAL;
  hipLaunchKernelGGL(stream_read_kernel, dim3((unsigned)blocks), dim3(256), 0, reinterpret_cast<hipStream_t>(stream),
                     reinterpret_cast<const u32x4*>(src), bytes / 16, sink);
  LPP_HIP_TRY(hipGetLastError());
  return LPP_OK;
}
