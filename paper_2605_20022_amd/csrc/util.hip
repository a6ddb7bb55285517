// Plain streaming copy: the yard-stick for achievable HBM bandwidth and for scaling the
// FETCH_SIZE / WRITE_SIZE hardware counters (it moves exactly `bytes` in and `bytes` out).
#include "fd_common.h"

namespace fd {

__global__ __launch_bounds__(256) void stream_copy_kernel(const u32x4* __restrict__ src, u32x4* __restrict__ dst, size_t n) {
  size_t i = blockIdx.x * (size_t)256 + threadIdx.x;
  const size_t stride = (size_t)gridDim.x * 256;
  for (; i < n; i += stride) {
    u32x4 v = __builtin_nontemporal_load(src + i);
    __builtin_nontemporal_store(v, dst + i);
  }
}

hipError_t run_stream_copy(const void* src, void* dst, size_t bytes, hipStream_t st) {
  size_t n = bytes / 16;
  size_t blocks = (n + 255) / 256;
  if (blocks > 256 * 16) blocks = 256 * 16;
  hipLaunchKernelGGL(stream_copy_kernel, dim3((unsigned)blocks), dim3(256), 0, st,
                     reinterpret_cast<const u32x4*>(src), reinterpret_cast<u32x4*>(dst), n);
  return hipGetLastError();
}

}  // namespace fd
