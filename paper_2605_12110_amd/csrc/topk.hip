// Selection stage (Sec. 3.4, kernel 2): per (request, KV head) segment of the score array the
// K_s = min(N_s, ceil(T_b / B_h)) highest-scoring blocks; the prefix-sum offsets of the estimation
// stage delimit the segments.  Equal scores go to the lower block index and the index list is
// written in ascending order, so there is exactly one correct output.
//
// One work-group of 1024 threads per segment runs an exact radix select in LDS:
//   1. min / max of the segment's scores -> keys relative to the minimum, so that the digits of
//      the first pass are spread over the histogram bins instead of piling up in a few;
//   2. most-significant-digit-first 8-bit histogram passes narrow down the threshold key tau and
//      the number `need` of tau-valued blocks that still fit;
//   3. one ordered compaction: block j is selected iff key_j > tau, or key_j == tau and fewer than
//      `need` tau-valued blocks precede it; its output slot is the count of selected blocks before it.
// Scores are re-read from L2 in each pass (a segment is at most a few hundred KiB).
#include "common.h"

namespace absb {

struct TopkParams {
  const int32_t* scores;
  const int32_t* cent_off;
  const int32_t* budget;  // [Bt]
  int32_t* sel_idx;
  int32_t* sel_cnt;
  int32_t sel_stride, Hkv;
  HeadTable heads;
};

constexpr int TOPK_THREADS = 1024;
constexpr int TOPK_WAVES = TOPK_THREADS / 64;

__device__ __forceinline__ uint32_t ordered_key(int32_t score) { return (uint32_t)score ^ 0x80000000u; }

__global__ __launch_bounds__(TOPK_THREADS) void topk_kernel(TopkParams p) {
  const int s = blockIdx.x;
  const int b = s / p.Hkv, h = s % p.Hkv;
  const int off = p.cent_off[s];
  const int N = p.cent_off[s + 1] - off;
  const int lb = p.heads.log2_block[h];
  const int T = p.budget[b];
  int K = (int)(((int64_t)T + (1 << lb) - 1) >> lb);
  K = min(min(K, N), p.sel_stride);
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int32_t* sc = p.scores + off;
  int32_t* out = p.sel_idx + (size_t)s * p.sel_stride;

  if (tid == 0) p.sel_cnt[s] = K;
  for (int i = K + tid; i < p.sel_stride; i += TOPK_THREADS) out[i] = -1;
  if (K >= N) {  // everything is selected
    for (int i = tid; i < N; i += TOPK_THREADS) out[i] = i;
    return;
  }

  __shared__ uint32_t s_red[2 * TOPK_WAVES];
  __shared__ uint32_t s_hist[256];
  __shared__ uint32_t s_bcast[2];
  __shared__ uint32_t s_cnt_gt[TOPK_WAVES], s_cnt_eq[TOPK_WAVES];

  // ---- 1. range of the keys
  uint32_t kmin = 0xffffffffu, kmax = 0u;
  for (int j = tid; j < N; j += TOPK_THREADS) {
    const uint32_t k = ordered_key(sc[j]);
    kmin = min(kmin, k);
    kmax = max(kmax, k);
  }
  for (int d = 32; d >= 1; d >>= 1) {
    kmin = min(kmin, (uint32_t)__shfl_xor((int)kmin, d));
    kmax = max(kmax, (uint32_t)__shfl_xor((int)kmax, d));
  }
  if (lane == 0) {
    s_red[wave] = kmin;
    s_red[TOPK_WAVES + wave] = kmax;
  }
  __syncthreads();
  kmin = s_red[0];
  kmax = s_red[TOPK_WAVES];
  for (int w = 1; w < TOPK_WAVES; ++w) {
    kmin = min(kmin, s_red[w]);
    kmax = max(kmax, s_red[TOPK_WAVES + w]);
  }
  const uint32_t range = kmax - kmin;  // relative keys live in [0, range]
  const int bits = 32 - __builtin_clz(range | 1u);
  const int passes = (bits + 7) / 8;

  // ---- 2. radix select on rel = key - kmin, most significant digit first
  uint32_t prefix = 0, mask = 0;
  int need = K;
  for (int pass = passes - 1; pass >= 0; --pass) {
    const int shift = pass * 8;
    if (tid < 256) s_hist[tid] = 0;
    __syncthreads();
    for (int j = tid; j < N; j += TOPK_THREADS) {
      const uint32_t rel = ordered_key(sc[j]) - kmin;
      if ((rel & mask) == prefix) atomicAdd(&s_hist[(rel >> shift) & 255u], 1u);
    }
    __syncthreads();
    if (wave == 0) {
      // lane owns bins 4*lane .. 4*lane+3; above = number of candidates in strictly higher bins
      const uint32_t c0 = s_hist[4 * lane], c1 = s_hist[4 * lane + 1], c2 = s_hist[4 * lane + 2],
                     c3 = s_hist[4 * lane + 3];
      const uint32_t mine = c0 + c1 + c2 + c3;
      uint32_t incl = mine;  // inclusive suffix sum over lanes (lane 63 = highest bins)
      for (int d = 1; d < 64; d <<= 1) {
        const uint32_t v = (uint32_t)__shfl_down((int)incl, d);
        if (lane + d < 64) incl += v;
      }
      uint32_t above = incl - mine;
      // walk the four bins from the top
      const uint32_t c[4] = {c0, c1, c2, c3};
#pragma unroll
      for (int i = 3; i >= 0; --i) {
        if (above < (uint32_t)need && (uint32_t)need <= above + c[i]) {
          s_bcast[0] = (uint32_t)(4 * lane + i);
          s_bcast[1] = above;
        }
        above += c[i];
      }
    }
    __syncthreads();
    prefix |= s_bcast[0] << shift;
    mask |= 255u << shift;
    need -= (int)s_bcast[1];
  }
  // tau = prefix (relative key); `need` >= 1 blocks with key == tau are taken, lowest index first

  // ---- 3. ordered compaction in tiles of 1024 consecutive indices
  int base_gt = 0, base_eq = 0;  // selected-by-gt / eq-valued blocks before the tile
  for (int t0 = 0; t0 < N; t0 += TOPK_THREADS) {
    const int j = t0 + tid;
    uint32_t rel = 0;
    bool gt = false, eq = false;
    if (j < N) {
      rel = ordered_key(sc[j]) - kmin;
      gt = rel > prefix;
      eq = rel == prefix;
    }
    const uint64_t bgt = __ballot(gt), beq = __ballot(eq);
    if (lane == 0) {
      s_cnt_gt[wave] = (uint32_t)__popcll(bgt);
      s_cnt_eq[wave] = (uint32_t)__popcll(beq);
    }
    __syncthreads();
    int gt_before = base_gt, eq_before = base_eq, gt_tile = 0, eq_tile = 0;
    for (int w = 0; w < TOPK_WAVES; ++w) {
      const int cg = (int)s_cnt_gt[w], ce = (int)s_cnt_eq[w];
      if (w < wave) {
        gt_before += cg;
        eq_before += ce;
      }
      gt_tile += cg;
      eq_tile += ce;
    }
    const uint64_t lt_mask = (1ull << lane) - 1ull;
    gt_before += __popcll(bgt & lt_mask);
    eq_before += __popcll(beq & lt_mask);
    if (gt || (eq && eq_before < need)) out[gt_before + min(eq_before, need)] = j;
    base_gt += gt_tile;
    base_eq += eq_tile;
    __syncthreads();
  }
}

int launch_topk(const Geometry& g, const Plan& pl, const int32_t* scores, const int32_t* cent_off,
                const int32_t* budget, int32_t* sel_idx, int32_t* sel_cnt, int32_t sel_stride,
                hipStream_t stream) {
  TopkParams p;
  p.scores = scores;
  p.cent_off = cent_off;
  p.budget = budget;
  p.sel_idx = sel_idx;
  p.sel_cnt = sel_cnt;
  p.sel_stride = sel_stride;
  p.Hkv = g.Hkv;
  p.heads = g.heads;
  hipLaunchKernelGGL(topk_kernel, dim3((unsigned)pl.nseg), dim3(TOPK_THREADS), 0, stream, p);
  return check_launch();
}

}  // namespace absb
