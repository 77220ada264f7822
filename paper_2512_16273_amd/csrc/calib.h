// tslt_calibrate_read: a plain read-only streaming kernel over a caller's buffer, with the load shape of the
// dense passes (16-byte nontemporal loads, 256 threads per workgroup, four vectors in flight per thread, one
// contiguous chunk per workgroup).  It measures what this chip delivers to a kernel that does nothing but
// read: the practical ceiling the streaming kernels are held against beside the published peak.
#pragma once
#include "common.h"

namespace tslt {

constexpr int kCalibUnroll = 4;

__global__ __launch_bounds__(kBlock) void calibrate_read_kernel(const uint4* src, uint64_t vecs_per_block, uint32_t* sink) {
  const uint4* base = src + size_t(blockIdx.x) * vecs_per_block + threadIdx.x;
  uint32_t acc = 0;
  for (uint64_t i = 0; i < vecs_per_block; i += uint64_t(kCalibUnroll) * kBlock) {
    uint4 d[kCalibUnroll];
#pragma unroll
    for (int u = 0; u < kCalibUnroll; ++u) d[u] = load_vec_stream(base + i + u * kBlock);
#pragma unroll
    for (int u = 0; u < kCalibUnroll; ++u) acc += d[u].x ^ d[u].y ^ d[u].z ^ d[u].w;
  }
  // the sum is stored only if it equals a value it practically never has: the loads stay, the writes do not
  if (acc == 0x9E3779B9u) sink[0] = acc;
}

}  // namespace tslt
