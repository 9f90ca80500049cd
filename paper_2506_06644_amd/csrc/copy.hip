// A plain device-to-device copy of known size: 16 bytes per lane and step, grid-stride.  It is the
// reference the HBM byte counters (FETCH_SIZE / WRITE_SIZE) are scaled by when the traffic of the
// other kernels is measured: it reads exactly `nbytes` and writes exactly `nbytes`.
#include <algorithm>

#include "spark_device.h"
#include "spark_internal.h"

namespace spark {

namespace {

__global__ __launch_bounds__(256) void copy_bytes_kernel(u32x4* __restrict__ dst, const u32x4* __restrict__ src, size_t n16) {
  const size_t stride = (size_t)gridDim.x * 256;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += stride)
    __builtin_nontemporal_store(__builtin_nontemporal_load(src + i), dst + i);
}

}  // namespace

hipError_t launch_copy_bytes(void* dst, const void* src, size_t nbytes, hipStream_t st) {
  if (nbytes == 0) return hipSuccess;
  const size_t n16 = nbytes / 16;
  const unsigned grid = (unsigned)std::min<size_t>((n16 + 255) / 256, 256 * 32);
  hipLaunchKernelGGL(copy_bytes_kernel, dim3(grid), dim3(256), 0, st, static_cast<u32x4*>(dst),
                     static_cast<const u32x4*>(src), n16);
  return hipGetLastError();
}

}  // namespace spark
