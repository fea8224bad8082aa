// Estimation stage (Sec. 3.4, kernel 1) as a launch of its own: one launch over the flattened code
// array delimited by the prefix-sum offsets; the arithmetic is in score_dev.h.  Compiled with
// -ffp-contract=off (every binary32 step of the weight image is a single IEEE operation).
#include "score_dev.h"

namespace absb {

template <int DT, int REP>
__global__ __launch_bounds__(256) void score_kernel(ScoreParams p) {
  __shared__ __align__(16) char s_lds[score_lds_bytes<REP>()];
  score_chunk<DT, REP, false>(p, (int)blockIdx.y, (int)blockIdx.x, s_lds);
}

int launch_score(const Geometry& g, const Plan& pl, int dtype, const void* q, const uint8_t* codes,
                 const float* qscale, const float* qmin, const int32_t* cent_off, const int32_t* seq_lens,
                 int32_t* scores, int32_t* score_exp, hipStream_t stream) {
  const ScoreParams p = make_score_params(g, pl, q, codes, qscale, qmin, cent_off, seq_lens, scores, score_exp);
  dim3 grid((unsigned)((pl.max_blocks + pl.score_chunk - 1) / pl.score_chunk), (unsigned)pl.nseg);
  if (dtype == ABSB_F16 && g.repr == ABSB_REPR_MEAN)
    hipLaunchKernelGGL((score_kernel<ABSB_F16, 0>), grid, dim3(256), 0, stream, p);
  else if (dtype == ABSB_F16)
    hipLaunchKernelGGL((score_kernel<ABSB_F16, 1>), grid, dim3(256), 0, stream, p);
  else if (g.repr == ABSB_REPR_MEAN)
    hipLaunchKernelGGL((score_kernel<ABSB_BF16, 0>), grid, dim3(256), 0, stream, p);
  else
    hipLaunchKernelGGL((score_kernel<ABSB_BF16, 1>), grid, dim3(256), 0, stream, p);
  return check_launch();
}

}  // namespace absb
