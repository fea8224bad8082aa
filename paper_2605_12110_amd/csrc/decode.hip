// Attention over the selected blocks (Sec. 3.4, kernel 3) as a launch of its own; the work of a
// work-group is in decode_dev.h.
#include "decode_dev.h"

namespace absb {

template <int DT, int G>
__global__ __launch_bounds__(DEC_THREADS, 3) void decode_kernel(DecodeParams p) {
  __shared__ __align__(16) char s_lds[DEC_LDS_BYTES];
  decode_split<DT, G, false>(p, (int)blockIdx.y, (int)blockIdx.x, s_lds);
}

// Zeroes the per-segment ticket counters when no earlier kernel of the same call has done it.
__global__ void decode_clear_tickets_kernel(int32_t* tickets, int n) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) tickets[(size_t)i * ABSB_TICKET_STRIDE] = 0;
}

template <int DT>
static void launch_partial(const DecodeParams& p, dim3 grid, hipStream_t stream) {
  switch (p.g.Gd) {
    case 1: hipLaunchKernelGGL((decode_kernel<DT, 1>), grid, dim3(DEC_THREADS), 0, stream, p); break;
    case 2: hipLaunchKernelGGL((decode_kernel<DT, 2>), grid, dim3(DEC_THREADS), 0, stream, p); break;
    case 3: hipLaunchKernelGGL((decode_kernel<DT, 3>), grid, dim3(DEC_THREADS), 0, stream, p); break;
    case 4: hipLaunchKernelGGL((decode_kernel<DT, 4>), grid, dim3(DEC_THREADS), 0, stream, p); break;
    case 5: hipLaunchKernelGGL((decode_kernel<DT, 5>), grid, dim3(DEC_THREADS), 0, stream, p); break;
    case 6: hipLaunchKernelGGL((decode_kernel<DT, 6>), grid, dim3(DEC_THREADS), 0, stream, p); break;
    case 7: hipLaunchKernelGGL((decode_kernel<DT, 7>), grid, dim3(DEC_THREADS), 0, stream, p); break;
    default: hipLaunchKernelGGL((decode_kernel<DT, 8>), grid, dim3(DEC_THREADS), 0, stream, p); break;
  }
}

int launch_decode(const Geometry& g, const Plan& pl, int dtype, float sm_scale, const void* q,
                  const void* k_cache, const void* v_cache, const int32_t* page_table, const int32_t* seq_lens,
                  const int32_t* sel_idx, const int32_t* sel_cnt, int32_t sel_stride, void* out, float* lse,
                  char* ws, bool tickets_cleared, hipStream_t stream) {
  const DecodeParams p = make_decode_params(g, pl, sm_scale, q, k_cache, v_cache, page_table, seq_lens, sel_idx, sel_cnt,
                                            sel_stride, out, lse, ws);
  if (!tickets_cleared && pl.max_splits > 1) {
    hipLaunchKernelGGL(decode_clear_tickets_kernel, dim3((unsigned)((pl.nseg + 255) / 256)), dim3(256), 0, stream,
                       p.tickets, (int)pl.nseg);
    int rc = check_launch();
    if (rc != ABSB_OK) return rc;
  }
  dim3 grid((unsigned)pl.max_splits, (unsigned)pl.nseg);
  if (dtype == ABSB_F16)
    launch_partial<ABSB_F16>(p, grid, stream);
  else
    launch_partial<ABSB_BF16>(p, grid, stream);
  return check_launch();
}

}  // namespace absb
