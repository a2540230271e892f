// Measurement aids: a read-only streaming kernel and a plain copy.
#pragma once

#include "ears_device.h"

namespace ears {

// =================================================================================================
// Measurement aids.
// =================================================================================================
constexpr int kBenchBlocks = 4096;

__global__ __launch_bounds__(kBlock) void bench_read_kernel(const uint4* src, size_t nvec,
                                                            uint32_t* sink) {
  uint32_t acc = 0;
  const size_t stride = (size_t)gridDim.x * kBlock;
  size_t i = (size_t)blockIdx.x * kBlock + threadIdx.x;
  for (; i + 3 * stride < nvec; i += 4 * stride) {
    const uint4 a = src[i], b = src[i + stride], c = src[i + 2 * stride], d = src[i + 3 * stride];
    acc ^= a.x ^ a.y ^ a.z ^ a.w ^ b.x ^ b.y ^ b.z ^ b.w ^ c.x ^ c.y ^ c.z ^ c.w ^ d.x ^ d.y ^ d.z ^ d.w;
  }
  for (; i < nvec; i += stride) {
    const uint4 a = src[i];
    acc ^= a.x ^ a.y ^ a.z ^ a.w;
  }
#pragma unroll
  for (int d = 1; d < kWave; d <<= 1) acc ^= __shfl_xor(acc, d, 64);
  __shared__ uint32_t sh[kWavesPerBlock];
  if ((threadIdx.x & (kWave - 1)) == 0) sh[threadIdx.x / kWave] = acc;
  __syncthreads();
  if (threadIdx.x == 0) sink[blockIdx.x] = sh[0] ^ sh[1] ^ sh[2] ^ sh[3];
}

__global__ __launch_bounds__(kBlock) void bench_copy_kernel(uint4* dst, const uint4* src,
                                                            size_t nvec) {
  const size_t stride = (size_t)gridDim.x * kBlock;
  for (size_t i = (size_t)blockIdx.x * kBlock + threadIdx.x; i < nvec; i += stride) dst[i] = src[i];
}


}  // namespace ears
