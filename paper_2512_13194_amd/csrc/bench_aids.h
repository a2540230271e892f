// Measurement aids: a read-only streaming kernel and a plain copy.
#pragma once

#include "ears_device.h"

namespace ears {

// =================================================================================================
// Measurement aids.
// =================================================================================================
constexpr int kBenchBlocks = 4096;
constexpr size_t kBenchSlabVecs = 16384;  // about 256 KiB per workgroup visit, one logit row
constexpr int kBenchUnroll = 8;           // 16-byte loads in flight per lane, as in the row pass on long rows

// Read-only ceiling: every workgroup streams whole 256 KiB slabs with the same non-temporal
// 16-byte loads, eight in flight per lane, that the row-statistics pass uses, and folds them
// into a checksum.
__global__ __launch_bounds__(kBlock) void bench_read_kernel(const uint4* src, size_t nvec,
                                                            size_t slab_vecs, uint32_t* sink) {
  uint32_t acc = 0;
  const size_t nslabs = (nvec + slab_vecs - 1) / slab_vecs;
  for (size_t slab = blockIdx.x; slab < nslabs; slab += gridDim.x) {
    const size_t v0 = slab * slab_vecs;
    const size_t v1 = v0 + slab_vecs < nvec ? v0 + slab_vecs : nvec;
    for (size_t i0 = v0 + threadIdx.x; i0 < v1; i0 += (size_t)kBlock * kBenchUnroll) {
      uint4 raw[kBenchUnroll];
#pragma unroll
      for (int u = 0; u < kBenchUnroll; ++u) {
        const size_t i = i0 + (size_t)u * kBlock;
        raw[u] = i < v1 ? load_stream(src + i) : make_uint4(0u, 0u, 0u, 0u);
      }
#pragma unroll
      for (int u = 0; u < kBenchUnroll; ++u) acc ^= raw[u].x ^ raw[u].y ^ raw[u].z ^ raw[u].w;
    }
  }
#pragma unroll
  for (int d = 1; d < kWave; d <<= 1) acc ^= __shfl_xor(acc, d, 64);
  __shared__ uint32_t sh[kWavesPerBlock];
  if ((threadIdx.x & (kWave - 1)) == 0) sh[threadIdx.x / kWave] = acc;
  __syncthreads();
  if (threadIdx.x == 0) {
    uint32_t x = 0;
    for (int w = 0; w < kWavesPerBlock; ++w) x ^= sh[w];
    sink[blockIdx.x] = x;
  }
}

__global__ __launch_bounds__(kBlock) void bench_copy_kernel(uint4* dst, const uint4* src,
                                                            size_t nvec) {
  const size_t stride = (size_t)gridDim.x * kBlock;
  for (size_t i = (size_t)blockIdx.x * kBlock + threadIdx.x; i < nvec; i += stride) dst[i] = src[i];
}


}  // namespace ears
