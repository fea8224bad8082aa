// Selection stage (Sec. 3.4, kernel 2) as a launch of its own: per (request, KV head) segment of
// the score array the K_s = min(N_s, ceil(T_b / B_h)) highest-scoring blocks; the prefix-sum
// offsets of the estimation stage delimit the segments.  Equal scores go to the lower block index
// and the index list is written in ascending order, so there is exactly one correct output.
// One work-group of 1024 threads per segment; the algorithm is in topk_dev.h.
#include "topk_dev.h"

namespace absb {

constexpr int TOPK_THREADS = 1024;

// KPT > 0: keys of the segment live in registers (N <= KPT*1024).  KPT == 0: keys are re-read.
template <int KPT>
__global__ __launch_bounds__(TOPK_THREADS) void topk_kernel(TopkParams p) {
  extern __shared__ __align__(16) char s_topk[];
  TopkShared& sh = *reinterpret_cast<TopkShared*>(s_topk);
  uint32_t* bitmap = reinterpret_cast<uint32_t*>(s_topk + ((sizeof(TopkShared) + 15) & ~size_t(15)));
  topk_segment<TOPK_THREADS, KPT, false>(p, (int)blockIdx.x, sh, bitmap);
}

int launch_topk(const Geometry& g, const Plan& pl, const int32_t* scores, const int32_t* cent_off,
                const int32_t* budget, const int32_t* seq_lens, int32_t* sel_idx, int32_t* sel_cnt,
                int32_t sel_stride, int32_t* tickets, hipStream_t stream) {
  if (pl.max_blocks > TOPK_MAX_BLOCKS) return ABSB_ERR_UNSUPPORTED;
  const TopkParams p = make_topk_params(g, scores, cent_off, budget, seq_lens, sel_idx, sel_cnt, sel_stride, tickets);
  const dim3 grid((unsigned)pl.nseg), block(TOPK_THREADS);
  const size_t lds = topk_lds_bytes(pl.max_blocks);
  const int tiles = (pl.max_blocks + TOPK_THREADS - 1) / TOPK_THREADS;
  if (tiles <= 1)
    hipLaunchKernelGGL(topk_kernel<1>, grid, block, lds, stream, p);
  else if (tiles <= 2)
    hipLaunchKernelGGL(topk_kernel<2>, grid, block, lds, stream, p);
  else if (tiles <= 4)
    hipLaunchKernelGGL(topk_kernel<4>, grid, block, lds, stream, p);
  else if (tiles <= 8)
    hipLaunchKernelGGL(topk_kernel<8>, grid, block, lds, stream, p);
  else if (tiles <= 16)
    hipLaunchKernelGGL(topk_kernel<16>, grid, block, lds, stream, p);
  else
    hipLaunchKernelGGL(topk_kernel<0>, grid, block, lds, stream, p);
  return check_launch();
}

}  // namespace absb
