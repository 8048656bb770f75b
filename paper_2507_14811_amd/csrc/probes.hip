// Device probes used by the benchmark to put measured ceilings next to the datasheet peaks.
#include "sq_kernels.hpp"

namespace sq {

// Register-only int8 MFMA loop: every wave multiplies operands it loaded once (so their values, not memory,
// set the switching activity) into 8 independent 32x32 accumulators.  The sustained rate depends on the
// operand data because the core clock is power-managed.
__global__ __launch_bounds__(256) void probe_mfma_kernel(const v4i* __restrict__ codes, const uint32_t nvec,
                                                         const int iters, int* __restrict__ sink) {
  const uint32_t gid = blockIdx.x * 256u + threadIdx.x;
  v4i a[4], b[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    a[i] = codes[(gid * 8u + i) % nvec];
    b[i] = codes[(gid * 8u + 4u + i) % nvec];
  }
  v16i acc[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) acc[i] = (v16i)(0);
#pragma unroll 1
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < 8; ++i) acc[i] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[i & 3], b[(i >> 1) & 3], acc[i], 0, 0, 0);
  }
  int s = 0;
#pragma unroll
  for (int i = 0; i < 8; ++i)
#pragma unroll
    for (int v = 0; v < 16; ++v) s += acc[i][v];
  if (s == 0x7E57AB1E && sink) sink[0] = s;     // keeps the loop alive; practically never true
}

hipError_t launch_probe_mfma(const void* codes, size_t bytes, int iters, int* sink, hipStream_t st) {
  hipLaunchKernelGGL(probe_mfma_kernel, dim3(device_cus()), dim3(256), 0, st, reinterpret_cast<const v4i*>(codes),
                     (uint32_t)(bytes / 16), iters, sink);
  return hipGetLastError();
}

}  // namespace sq
