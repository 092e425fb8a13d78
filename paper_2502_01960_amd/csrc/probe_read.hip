// Streaming-read probe (measurement aid: part of libmpic_probe.so only).
//
// How fast can one launch read a buffer of the size a decode step reads?  The probe reads
// `bytes` once, 16 bytes per lane and load, four loads in flight per lane, folds the words
// into one value per lane (so that the loads cannot be dropped) and writes one float per
// workgroup.  A kernel that has to read N bytes of keys and values from HBM cannot finish
// sooner than this one does on N bytes: launch, ramp-up and drain of a short launch are
// in the figure, as they are in the decode kernel's.
#include <hip/hip_runtime.h>

#include <cstdint>

namespace mpic {
namespace {

constexpr int THREADS = 512;
typedef uint32_t rd_u32x4 __attribute__((ext_vector_type(4)));

__global__ __launch_bounds__(THREADS) void probe_read_kernel(const rd_u32x4* __restrict__ src, int64_t n16, float* sink) {
  const int64_t stride = static_cast<int64_t>(gridDim.x) * THREADS;
  int64_t i = static_cast<int64_t>(blockIdx.x) * THREADS + threadIdx.x;
  uint32_t acc = 0;
  for (; i + 3 * stride < n16; i += 4 * stride) {
    const rd_u32x4 a = __builtin_nontemporal_load(src + i);
    const rd_u32x4 b = __builtin_nontemporal_load(src + i + stride);
    const rd_u32x4 c = __builtin_nontemporal_load(src + i + 2 * stride);
    const rd_u32x4 d = __builtin_nontemporal_load(src + i + 3 * stride);
    acc ^= a.x ^ a.y ^ a.z ^ a.w ^ b.x ^ b.y ^ b.z ^ b.w ^ c.x ^ c.y ^ c.z ^ c.w ^ d.x ^ d.y ^ d.z ^ d.w;
  }
  for (; i < n16; i += stride) {
    const rd_u32x4 a = __builtin_nontemporal_load(src + i);
    acc ^= a.x ^ a.y ^ a.z ^ a.w;
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) acc ^= __shfl_xor(acc, off);
  if ((threadIdx.x & 63) == 0 && acc == 0x9E3779B9u) sink[blockIdx.x] = 1.0f;  // (practically never: keeps the loads alive)
  if (threadIdx.x == 0 && blockIdx.x == 0) sink[gridDim.x] = 0.0f;
}

}  // namespace
}  // namespace mpic

// One launch that reads `bytes` (a multiple of 16) from `src` (device).  n_wgs workgroups of
// 512 threads; sink: device float [n_wgs + 1].  Returns 0, -1 (bad arguments) or -4 (HIP error).
extern "C" int mpic_probe_read(const void* src, int64_t bytes, int n_wgs, float* sink, void* stream) {
  if (!src || !sink || bytes < 16 || (bytes & 15) || n_wgs < 1 || (reinterpret_cast<uintptr_t>(src) & 15)) return -1;
  hipLaunchKernelGGL(mpic::probe_read_kernel, dim3(n_wgs), dim3(mpic::THREADS), 0, static_cast<hipStream_t>(stream),
                     static_cast<const mpic::rd_u32x4*>(src), bytes / 16, sink);
  return hipGetLastError() == hipSuccess ? 0 : -4;
}
