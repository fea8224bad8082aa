// Measurement helper: a plain streaming read of a device buffer with 128-bit loads, the practical
// ceiling against which the attention kernel's bandwidth is reported.  Not a step of the method.
#include "common.h"

namespace absb {

constexpr int SR_THREADS = 256;
constexpr int SR_UNROLL = 8;

__global__ __launch_bounds__(SR_THREADS) void stream_read_kernel(const uint4* __restrict__ src, size_t n16,
                                                                 uint32_t* sink) {
  // work-group w reads the tiles w, w + gridDim.x, ...; a tile is SR_UNROLL x 4 KiB, every wave load
  // instruction covers 1 KiB of consecutive bytes
  const size_t tile = (size_t)SR_THREADS * SR_UNROLL;
  uint32_t acc = 0;
  for (size_t base = (size_t)blockIdx.x * tile; base < n16; base += (size_t)gridDim.x * tile) {
    uint4 v[SR_UNROLL];
#pragma unroll
    for (int u = 0; u < SR_UNROLL; ++u) {
      const size_t i = base + (size_t)u * SR_THREADS + threadIdx.x;
      v[u] = src[i < n16 ? i : n16 - 1];
    }
#pragma unroll
    for (int u = 0; u < SR_UNROLL; ++u) acc ^= v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
  }
  // keeps the loads alive; written only if every lane of a wave agrees on an unlikely value
  if (__all(acc == 0x9e3779b9u)) sink[0] = acc;
}

int launch_stream_read(const void* src, size_t bytes, uint32_t* sink, int num_cus, hipStream_t stream) {
  const size_t n16 = bytes / 16;
  if (n16 == 0) return ABSB_OK;
  const size_t tiles = (n16 + (size_t)SR_THREADS * SR_UNROLL - 1) / ((size_t)SR_THREADS * SR_UNROLL);
  size_t grid = (size_t)num_cus * 8;
  if (grid > tiles) grid = tiles;
  hipLaunchKernelGGL(stream_read_kernel, dim3((unsigned)grid), dim3(SR_THREADS), 0, stream,
                     static_cast<const uint4*>(src), n16, sink);
  return check_launch();
}

}  // namespace absb
