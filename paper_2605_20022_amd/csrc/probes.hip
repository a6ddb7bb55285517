// Measurement probes: a library of their own (libfdprobes.so), used by the benchmark only and not part
// of the product library or its header.  Plain streaming copy: the yard-stick for achievable HBM
// bandwidth and for scaling the FETCH_SIZE / WRITE_SIZE hardware counters (it moves exactly `bytes` in
// and `bytes` out).  Staged read: the attention kernel's launch shape and load scheme with nothing else
// in it, i.e. what a job of a given size can reach at best.
//
//   int fdp_stream_copy(const void* src, void* dst, size_t bytes, void* hip_stream)
//       device pointers, 16-byte aligned, bytes a multiple of 16; asynchronous on the stream
//   int fdp_stream_read(const void* src, size_t bytes, uint32_t* sums, void* hip_stream)
//       bytes a multiple of 32768; sums (device, 512 * 256 words) receives one 32-bit word sum per
//       thread, their total is the sum of all 32-bit words of the buffer modulo 2^32
// Both return 0, 1 for a bad argument, 4 for a failed launch.
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace {

typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;

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

// 2 x CUs persistent work-groups of four waves; every work-group reads a contiguous run of 32 KB tiles,
// two tiles in flight in registers, each passed through an LDS double buffer (one barrier per tile) and
// read back from LDS once.  sums[blockIdx.x * 256 + tid] = 32-bit sum of the words this thread read.
constexpr int SR_TILE = 32768;
constexpr int SR_GRID = 512;

__global__ __launch_bounds__(256, 2) void stream_read_kernel(const char* __restrict__ src, long long tiles, unsigned* __restrict__ sums) {
  __shared__ __attribute__((aligned(16))) char lds[2 * SR_TILE];
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const long long per = (tiles + gridDim.x - 1) / gridDim.x;
  const long long t0 = per * blockIdx.x;
  const long long t1 = t0 + per < tiles ? t0 + per : tiles;
  const int nt = t1 > t0 ? (int)(t1 - t0) : 0;
  const char* base = src + t0 * SR_TILE + wave * (SR_TILE / 4) + lane * 16;
  u32x4 ra[8], rb[8];
  auto load = [&](int t, u32x4 (&r)[8]) {
    const u32x4* g = reinterpret_cast<const u32x4*>(base + (long long)t * SR_TILE);
#pragma unroll
    for (int i = 0; i < 8; ++i) r[i] = __builtin_nontemporal_load(g + i * 64);
  };
  auto pass = [&](int b, const u32x4 (&r)[8]) {
    u32x4* d = reinterpret_cast<u32x4*>(lds + b * SR_TILE + wave * (SR_TILE / 4) + lane * 16);
#pragma unroll
    for (int i = 0; i < 8; ++i) d[i * 64] = r[i];
  };
  auto readback = [&](int b) {
    const u32x4* d = reinterpret_cast<const u32x4*>(lds + b * SR_TILE + tid * 16);
    u32x4 s = {0u, 0u, 0u, 0u};
#pragma unroll
    for (int i = 0; i < 8; ++i) s += d[i * 256];
    return s.x + s.y + s.z + s.w;
  };
  unsigned acc = 0;
  if (nt > 0) load(0, ra);
  if (nt > 1) load(1, rb);
  for (int t = 0; t < nt; t += 2) {
    pass(0, ra);
    if (t + 2 < nt) load(t + 2, ra);
    __syncthreads();
    acc += readback(0);
    if (t + 1 < nt) {
      pass(1, rb);
      if (t + 3 < nt) load(t + 3, rb);
      __syncthreads();
      acc += readback(1);
    }
  }
  sums[blockIdx.x * 256 + tid] = acc;
}

hipError_t run_stream_read(const void* src, size_t bytes, unsigned* sums, hipStream_t st) {
  hipLaunchKernelGGL(stream_read_kernel, dim3(SR_GRID), dim3(256), 0, st,
                     reinterpret_cast<const char*>(src), (long long)(bytes / SR_TILE), sums);
  return hipGetLastError();
}

}  // namespace

extern "C" {

__attribute__((visibility("default"))) int fdp_stream_copy(const void* src, void* dst, size_t bytes, void* hip_stream) {
  if (!src || !dst || bytes % 16 || (reinterpret_cast<uintptr_t>(src) & 15) || (reinterpret_cast<uintptr_t>(dst) & 15)) return 1;
  if (bytes == 0) return 0;
  return run_stream_copy(src, dst, bytes, reinterpret_cast<hipStream_t>(hip_stream)) == hipSuccess ? 0 : 4;
}

__attribute__((visibility("default"))) int fdp_stream_read(const void* src, size_t bytes, uint32_t* sums, void* hip_stream) {
  if (!src || !sums || bytes % 32768 || (reinterpret_cast<uintptr_t>(src) & 15)) return 1;
  return run_stream_read(src, bytes, sums, reinterpret_cast<hipStream_t>(hip_stream)) == hipSuccess ? 0 : 4;
}

}  // extern "C"
