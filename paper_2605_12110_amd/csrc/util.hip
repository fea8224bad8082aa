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

// Attention recall of a selection (Sec. 2.3): the share of the dense softmax mass that falls on
// the selected tokens is exp(lse over the selection - lse over the whole context); per
// (request, KV head) the mean over the group's query heads, in order.
__global__ void head_recall_kernel(const float* lse_sel, const float* lse_all, float* recall, int nseg, int G) {
  const int s = blockIdx.x * blockDim.x + threadIdx.x;
  if (s >= nseg) return;
  float acc = 0.0f;
  for (int g = 0; g < G; ++g) {
    const float a = lse_sel[(size_t)s * G + g], z = lse_all[(size_t)s * G + g];
    acc += (a == -__builtin_inff()) ? 0.0f : __expf(a - z);  // an empty selection holds no mass
  }
  recall[s] = acc / (float)G;
}

int launch_head_recall(const float* lse_sel, const float* lse_all, float* recall, int nseg, int G,
                       hipStream_t stream) {
  hipLaunchKernelGGL(head_recall_kernel, dim3((unsigned)((nseg + 255) / 256)), dim3(256), 0, stream, lse_sel, lse_all,
                     recall, nseg, G);
  return check_launch();
}

}  // namespace absb
