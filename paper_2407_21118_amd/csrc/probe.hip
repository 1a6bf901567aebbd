// Device probes for the benchmark: what this GPU sustains on a bare matrix-core
// loop and on a bare streaming read, so that kernel rates can be quoted against
// measured ceilings as well as against the data-sheet peaks.

#include "palu_dev.h"

namespace palu {

// every wavefront issues `iters` x 4 independent v_mfma_f32_32x32x16_f16 (operands in registers)
__global__ __launch_bounds__(256) void probe_mfma_kernel(float* sink, int iters) {
  half8 a, b;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    a[i] = (_Float16)((threadIdx.x & 63) * 0.001f + i);
    b[i] = (_Float16)(i * 0.5f - (threadIdx.x & 31) * 0.01f);
  }
  float16v acc[4];
#pragma unroll
  for (int n = 0; n < 4; ++n)
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[n][i] = 0.f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int n = 0; n < 4; ++n) acc[n] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, acc[n], 0, 0, 0);
  }
  float s = 0.f;
#pragma unroll
  for (int n = 0; n < 4; ++n)
#pragma unroll
    for (int i = 0; i < 16; ++i) s += acc[n][i];
  if (s == 12345.678f) sink[0] = s;          // keeps the loop alive; practically never true
}

// grid-stride read of n16 16-byte words, four loads in flight per thread
__global__ __launch_bounds__(256) void probe_read_kernel(const uint4v* __restrict__ src, size_t n16, float* sink) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  unsigned acc = 0;
  for (; i + 3 * stride < n16; i += 4 * stride) {
    const uint4v v0 = src[i], v1 = src[i + stride], v2 = src[i + 2 * stride], v3 = src[i + 3 * stride];
    acc += v0.x ^ v1.y ^ v2.z ^ v3.w;
  }
  for (; i < n16; i += stride) acc += src[i].x;
  if (acc == 0x12345678u) sink[0] = 1.f;
}

}  // namespace palu
