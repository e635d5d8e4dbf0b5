// Measurement aids: a read-only streaming pass and a plain copy, 16 bytes per lane per step,
// grid-stride.  They show what bandwidth a trivial kernel reaches on this device and give the
// known-size reference that hardware byte counters are scaled by.
#include "rap_device.h"

namespace rap {

__global__ __launch_bounds__(256) void stream_read_kernel(const uint4* __restrict__ src, size_t n16, uint4* sink) {
  const size_t stride = static_cast<size_t>(gridDim.x) * blockDim.x;
  uint4 acc = make_uint4(0, 0, 0, 0);
  for (size_t i = static_cast<size_t>(blockIdx.x) * blockDim.x + threadIdx.x; i < n16; i += stride) {
    const uint4 v = src[i];
    acc.x ^= v.x; acc.y ^= v.y; acc.z ^= v.z; acc.w ^= v.w;
  }
  // data-dependent store so the loads cannot be dropped; practically never taken for real data
  if ((acc.x & acc.y & acc.z & acc.w) == 0x9e3779b9u) *sink = acc;
}

__global__ __launch_bounds__(256) void stream_copy_kernel(uint4* __restrict__ dst, const uint4* __restrict__ src, size_t n16) {
  const size_t stride = static_cast<size_t>(gridDim.x) * blockDim.x;
  for (size_t i = static_cast<size_t>(blockIdx.x) * blockDim.x + threadIdx.x; i < n16; i += stride) dst[i] = src[i];
}

hipError_t launch_stream_read(const void* src, size_t bytes, void* sink, hipStream_t stream) {
  const size_t n16 = bytes / 16;
  const unsigned grid = 256 * 16;
  hipLaunchKernelGGL(stream_read_kernel, dim3(grid), dim3(256), 0, stream, static_cast<const uint4*>(src), n16,
                     static_cast<uint4*>(sink));
  return hipGetLastError();
}

hipError_t launch_stream_copy(void* dst, const void* src, size_t bytes, hipStream_t stream) {
  const size_t n16 = bytes / 16;
  const unsigned grid = 256 * 16;
  hipLaunchKernelGGL(stream_copy_kernel, dim3(grid), dim3(256), 0, stream, static_cast<uint4*>(dst),
                     static_cast<const uint4*>(src), n16);
  return hipGetLastError();
}

}  // namespace rap
