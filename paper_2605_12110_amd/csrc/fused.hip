// The whole decode step (score -> select -> attention over the selection, Sec. 3.4 kernels 1-3)
// in ONE launch.
//
// At batch 1 the step moves ~20 MB, i.e. a few microseconds of HBM time, so three dependent
// launches cost more in launch floors and drained pipelines than in work; and at large batches
// the selection of one segment (one CU, instruction-bound) can run under the attention of others.
// Work-groups take one of two roles by their index:
//
//   [0, n_score)        estimation of one chunk of one segment's blocks (score_dev.h).  Scores are
//                       stored device-coherently; the work-group then draws a ticket from the
//                       segment's counter, and the one that draws the last ticket runs the
//                       segment's selection (topk_dev.h): it stores the selected blocks
//                       device-coherently in the order it finds them, raises the segment's flag,
//                       and only then writes the ascending list if the caller asked for one.
//   [n_score, grid)     attention over one split of one segment's selection (decode_dev.h): the
//                       work-group loads its queries, waits for the segment's flag, reads the
//                       blocks with device-coherent loads (attention does not depend on their
//                       order beyond rounding) and proceeds as in the stand-alone kernel
//                       (partials, ticket, the last arriver merges).
//
// Progress: estimation/selection work-groups never wait for anything.  Attention work-groups wait
// only for work-groups with lower indices; the hardware starts work-groups in index order, so
// every work-group waited for is already running or done.  The wait is also bounded in time, so
// the launch ends whatever happens (a wait that ran out sets the status word; its segment's
// output rows are then set to NaN).
//
// Counters (estimation tickets, flags, attention tickets; 256 bytes apart) must be zero when the
// launch starts and are zero again when it ends: absb_workspace_init clears them once.
//
// Compiled with -ffp-contract=off, as the estimation stage requires.
#include "decode_dev.h"
#include "score_dev.h"
#include "topk_dev.h"

namespace absb {

struct FusedParams {
  ScoreParams sc;
  TopkParams tk;
  DecodeParams dc;
  int32_t* score_tickets;  // [nseg], ABSB_TICKET_STRIDE apart
  int32_t n_score, chunks_per_seg;
};

constexpr int FUSED_THREADS = DEC_THREADS;

__host__ __device__ constexpr size_t max_sz(size_t a, size_t b) { return a > b ? a : b; }

template <int DT, int G, int REP>
__global__ __launch_bounds__(FUSED_THREADS, 3) void fused_step_kernel(FusedParams p) {
  extern __shared__ __align__(16) char lds[];
  const int bid = blockIdx.x, tid = threadIdx.x;
  if (bid >= p.n_score) {
    const int id = bid - p.n_score;
    decode_split<DT, G, true>(p.dc, id / p.dc.max_splits, id % p.dc.max_splits, lds);
    return;
  }
  const int s = bid / p.chunks_per_seg;
  const int N = score_chunk<DT, REP, true>(p.sc, s, bid % p.chunks_per_seg, lds);
  if (N == 0) return;

  // ---- hand the chunk's scores over; the segment's last chunk goes on to select
  wait_stores_acknowledged();
  __syncthreads();  // every thread's scores are visible device-wide; the estimation's LDS is free
  int* s_last = reinterpret_cast<int*>(lds);
  if (tid == 0) {
    int32_t* ticket = p.score_tickets + (size_t)s * ABSB_TICKET_STRIDE;
    const int nchunks = (N + p.sc.chunk - 1) / p.sc.chunk;
    const int last =
        __hip_atomic_fetch_add(ticket, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == nchunks - 1;
    if (last) st_i32<true>(ticket, 0);
    *s_last = last;
  }
  __syncthreads();
  if (!*s_last) return;
  __syncthreads();  // everybody has read the word before the selection reuses the memory

  TopkShared& sh = *reinterpret_cast<TopkShared*>(lds);
  uint32_t* bitmap = reinterpret_cast<uint32_t*>(lds + ((sizeof(TopkShared) + 15) & ~size_t(15)));
  const int tiles = (N + FUSED_THREADS - 1) / FUSED_THREADS;
  if (tiles <= 8)
    topk_segment<FUSED_THREADS, 8, true, true>(p.tk, s, sh, bitmap);
  else if (tiles <= 16)
    topk_segment<FUSED_THREADS, 16, true, true>(p.tk, s, sh, bitmap);
  else if (tiles <= 32)
    topk_segment<FUSED_THREADS, 32, true, true>(p.tk, s, sh, bitmap);
  else if (tiles <= 64)
    topk_segment<FUSED_THREADS, 64, true, true>(p.tk, s, sh, bitmap);
  else
    topk_segment<FUSED_THREADS, 0, true, true>(p.tk, s, sh, bitmap);
  // (the selection raises the segment's flag itself, as soon as its members are known)
}

// Clears the counters at the start of a workspace (all three kinds, and the status word).
__global__ void clear_counters_kernel(int32_t* head, int nwords) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < nwords) head[i] = 0;
}

int launch_workspace_init(const Plan& pl, char* ws, hipStream_t stream) {
  const int nwords = (int)(pl.ws_head_bytes / 4);
  hipLaunchKernelGGL(clear_counters_kernel, dim3((unsigned)((nwords + 255) / 256)), dim3(256), 0, stream,
                     reinterpret_cast<int32_t*>(ws), nwords);
  return check_launch();
}

template <int DT, int G>
static void launch_fused_rep(const FusedParams& p, int repr, dim3 grid, size_t lds, hipStream_t stream) {
  if (repr == ABSB_REPR_MEAN)
    hipLaunchKernelGGL((fused_step_kernel<DT, G, 0>), grid, dim3(FUSED_THREADS), lds, stream, p);
  else
    hipLaunchKernelGGL((fused_step_kernel<DT, G, 1>), grid, dim3(FUSED_THREADS), lds, stream, p);
}

template <int DT>
static void launch_fused_group(const FusedParams& p, int repr, dim3 grid, size_t lds, hipStream_t stream) {
  switch (p.dc.g.Gd) {
    case 1: launch_fused_rep<DT, 1>(p, repr, grid, lds, stream); break;
    case 2: launch_fused_rep<DT, 2>(p, repr, grid, lds, stream); break;
    case 3: launch_fused_rep<DT, 3>(p, repr, grid, lds, stream); break;
    case 4: launch_fused_rep<DT, 4>(p, repr, grid, lds, stream); break;
    case 5: launch_fused_rep<DT, 5>(p, repr, grid, lds, stream); break;
    case 6: launch_fused_rep<DT, 6>(p, repr, grid, lds, stream); break;
    case 7: launch_fused_rep<DT, 7>(p, repr, grid, lds, stream); break;
    default: launch_fused_rep<DT, 8>(p, repr, grid, lds, stream); break;
  }
}

bool fused_one_launch_fits(const Plan& pl) {
  if (pl.max_blocks > TOPK_MAX_BLOCKS) return false;
  const int64_t cps = (pl.max_blocks + pl.score_chunk - 1) / pl.score_chunk;
  const int64_t grid = cps * pl.nseg + (int64_t)pl.nseg * pl.max_splits;
  return grid < (int64_t(1) << 31) - 1;
}

int launch_fused(const Geometry& g, const Plan& pl, int dtype, float sm_scale, const void* q, const uint8_t* codes,
                 const float* qscale, const float* qmin, const void* k_cache, const void* v_cache, const int32_t* page_table,
                 const int32_t* seq_lens, const int32_t* cent_off, const int32_t* budget, int32_t* sel_idx_out,
                 int32_t* sel_cnt, void* out, float* lse, char* ws, hipStream_t stream) {
  if (!fused_one_launch_fits(pl)) return ABSB_ERR_UNSUPPORTED;
  FusedParams p;
  int32_t* scores = reinterpret_cast<int32_t*>(ws + pl.ws_scores);
  p.sc = make_score_params(g, pl, q, codes, qscale, qmin, cent_off, seq_lens, scores, nullptr);
  // the attention reads the workspace's list (any order); the caller's, if wanted, is ascending
  int32_t* work_list = reinterpret_cast<int32_t*>(ws + pl.ws_sel_idx);
  p.tk = make_topk_params(g, scores, cent_off, budget, seq_lens, sel_idx_out, sel_cnt, pl.sel_stride, nullptr);
  p.tk.work_list = work_list;
  p.tk.flags = reinterpret_cast<int32_t*>(ws + pl.ws_flags);
  p.dc = make_decode_params(g, pl, sm_scale, q, k_cache, v_cache, page_table, seq_lens, work_list, sel_cnt,
                            pl.sel_stride, out, lse, ws);
  p.dc.budget = budget;
  p.dc.cent_off = cent_off;
  p.dc.flags = reinterpret_cast<int32_t*>(ws + pl.ws_flags);
  p.dc.status = reinterpret_cast<int32_t*>(ws + pl.ws_status);
  p.score_tickets = reinterpret_cast<int32_t*>(ws + pl.ws_score_tickets);
  p.chunks_per_seg = (pl.max_blocks + pl.score_chunk - 1) / pl.score_chunk;
  p.n_score = p.chunks_per_seg * pl.nseg;
  const dim3 grid((unsigned)(p.n_score + pl.nseg * pl.max_splits));
  const size_t lds = max_sz(max_sz((size_t)DEC_LDS_BYTES, topk_lds_bytes(pl.max_blocks)), score_lds_bytes<1>());
  if (dtype == ABSB_F16)
    launch_fused_group<ABSB_F16>(p, g.repr, grid, lds, stream);
  else
    launch_fused_group<ABSB_BF16>(p, g.repr, grid, lds, stream);
  return check_launch();
}

}  // namespace absb
