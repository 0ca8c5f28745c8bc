// Read-only bandwidth probe: what a plain streaming read reaches on the device, as a yardstick
// next to the published peak.  Not part of the decode path.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "launch.h"

namespace confkv {

constexpr int kProbeThreads = 256;
constexpr int kProbeLoads = 8;     // 16-byte loads in flight per thread

// grid (G), 256 threads: workgroup g reads the g-th of G equal contiguous shares, 32 KB
// (8 loads x 256 threads x 16 bytes) per trip, and folds everything into one word per
// workgroup so that the loads cannot be dropped.
__global__ __launch_bounds__(kProbeThreads) void probe_read_kernel(const int4 *__restrict__ src, size_t n16,
                                                                   unsigned *__restrict__ out) {
  const size_t share = (n16 + gridDim.x - 1) / gridDim.x;
  const size_t lo = (size_t)blockIdx.x * share, hi = lo + share < n16 ? lo + share : n16;
  unsigned acc = 0;
  for (size_t base = lo + threadIdx.x; base < hi; base += (size_t)kProbeThreads * kProbeLoads) {
    int4 v[kProbeLoads];
#pragma unroll
    for (int k = 0; k < kProbeLoads; ++k) {
      const size_t i = base + (size_t)k * kProbeThreads;
      v[k] = src[i < hi ? i : hi - 1];               // branch-free: all loads of a trip in flight
    }
#pragma unroll
    for (int k = 0; k < kProbeLoads; ++k) {
      const bool in = base + (size_t)k * kProbeThreads < hi;     // re-read words past the share do not count
      acc ^= in ? (unsigned)(v[k].x ^ v[k].y ^ v[k].z ^ v[k].w) : 0u;
    }
  }
  for (int m = 32; m >= 1; m >>= 1) acc ^= __shfl_xor(acc, m, 64);
  if ((threadIdx.x & 63) == 0) atomicXor(&out[blockIdx.x], acc);
}

hipError_t launch_probe_read(const void *src, size_t bytes, unsigned *out, int workgroups, hipStream_t stream) {
  hipLaunchKernelGGL(probe_read_kernel, dim3(workgroups), dim3(kProbeThreads), 0, stream, (const int4 *)src,
                     bytes / 16, out);
  return hipGetLastError();
}

}  // namespace confkv
