// Selection stage (Sec. 3.4, kernel 2): per (request, KV head) segment of the score array the
// K_s = min(N_s, ceil(T_b / B_h)) highest-scoring blocks; the prefix-sum offsets of the estimation
// stage delimit the segments.  Equal scores go to the lower block index and the index list is
// written in ascending order, so there is exactly one correct output.
//
// One work-group of 1024 threads per segment.  Selection is an exact threshold search:
//   1. the segment's scores are loaded once (coalesced, all loads in flight together) and kept in
//      registers as order-preserving unsigned keys relative to the segment minimum;
//   2. one 256-bin LDS histogram over the top 8 significant bits of the key range finds the bin
//      that holds the K-th largest key;
//   3. the few candidates of that bin are appended to an LDS list and ranked exactly by
//      (key desc, index asc); the candidate of rank `need`-1 fixes the threshold key tau and how
//      many tau-valued blocks are taken (a crowded bin falls back to further radix digits);
//   4. one ordered compaction: block j is selected iff key_j > tau, or key_j == tau and fewer than
//      `need_eq` tau-valued blocks precede it; its output slot is the number of selected blocks
//      before it (ballots + one scan of per-(tile, wave) counts).
// Segments with more than 16384 blocks use the same algorithm with keys re-read from L2.
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
constexpr int TOPK_MAX_CAND = 1024;  // candidates ranked by brute force
constexpr int TOPK_MAX_KPT = 16;     // keys per thread held in registers

__device__ __forceinline__ uint32_t ordered_key(int32_t score) { return (uint32_t)score ^ 0x80000000u; }

struct TopkShared {
  uint32_t red[2 * TOPK_WAVES];
  uint32_t hist[256];
  uint32_t bcast[4];
  uint32_t cand_key[TOPK_MAX_CAND];
  uint32_t cand_idx[TOPK_MAX_CAND];
  uint32_t cand_n;
  uint32_t cnt_gt[TOPK_MAX_KPT * TOPK_WAVES];
  uint32_t cnt_eq[TOPK_MAX_KPT * TOPK_WAVES];
};

// Finds, from a 256-bin histogram of the candidates' current digit, the bin holding the
// `need`-th largest candidate; run by wave 0.  bcast[0] = bin, bcast[1] = candidates above it.
__device__ __forceinline__ void pick_bin(TopkShared& sh, int lane, uint32_t need) {
  const uint32_t c0 = sh.hist[4 * lane], c1 = sh.hist[4 * lane + 1], c2 = sh.hist[4 * lane + 2],
                 c3 = sh.hist[4 * lane + 3];
  const uint32_t mine = c0 + c1 + c2 + c3;
  uint32_t incl = mine;  // inclusive suffix sum over lanes (lane 63 owns the highest bins)
  for (int d = 1; d < 64; d <<= 1) {
    const uint32_t v = (uint32_t)__shfl_down((int)incl, d);
    if (lane + d < 64) incl += v;
  }
  uint32_t above = incl - mine;
  const uint32_t c[4] = {c0, c1, c2, c3};
#pragma unroll
  for (int i = 3; i >= 0; --i) {
    if (above < need && need <= above + c[i]) {
      sh.bcast[0] = (uint32_t)(4 * lane + i);
      sh.bcast[1] = above;
      sh.bcast[2] = c[i];
    }
    above += c[i];
  }
}

// KPT > 0: keys of the segment live in registers (N <= KPT*1024).  KPT == 0: keys are re-read.
template <int KPT>
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
  constexpr int R = KPT > 0 ? KPT : 1;
  const int ntiles = KPT > 0 ? KPT : (N + TOPK_THREADS - 1) / TOPK_THREADS;

  // keys first: everything else waits on them
  uint32_t key[R];
  if (KPT > 0) {
#pragma unroll
    for (int i = 0; i < R; ++i) {
      const int j = i * TOPK_THREADS + tid;
      key[i] = j < N ? ordered_key(sc[j]) : 0u;
    }
  }
  auto key_at = [&](int i) -> uint32_t {  // valid only for i*1024+tid < N
    if (KPT > 0) return key[i];
    return ordered_key(sc[i * TOPK_THREADS + tid]);
  };

  if (tid == 0) p.sel_cnt[s] = K;
  for (int i = K + tid; i < p.sel_stride; i += TOPK_THREADS) out[i] = -1;
  if (K >= N) {  // everything is selected
    for (int i = tid; i < N; i += TOPK_THREADS) out[i] = i;
    return;
  }

  __shared__ TopkShared sh;
  if (tid < 256) sh.hist[tid] = 0;
  if (tid == 0) sh.cand_n = 0;

  // ---- 1. range of the keys
  uint32_t kmin = 0xffffffffu, kmax = 0u;
#pragma unroll
  for (int i = 0; i < (KPT > 0 ? KPT : 1); ++i) {
    if (KPT > 0) {
      if (i * TOPK_THREADS + tid < N) {
        kmin = min(kmin, key[i]);
        kmax = max(kmax, key[i]);
      }
    }
  }
  if (KPT == 0) {
    for (int i = 0; i < ntiles; ++i)
      if (i * TOPK_THREADS + tid < N) {
        const uint32_t k = key_at(i);
        kmin = min(kmin, k);
        kmax = max(kmax, k);
      }
  }
  for (int d = 32; d >= 1; d >>= 1) {
    kmin = min(kmin, (uint32_t)__shfl_xor((int)kmin, d));
    kmax = max(kmax, (uint32_t)__shfl_xor((int)kmax, d));
  }
  if (lane == 0) {
    sh.red[wave] = kmin;
    sh.red[TOPK_WAVES + wave] = kmax;
  }
  __syncthreads();
  kmin = sh.red[0];
  kmax = sh.red[TOPK_WAVES];
#pragma unroll
  for (int w = 1; w < TOPK_WAVES; ++w) {
    kmin = min(kmin, sh.red[w]);
    kmax = max(kmax, sh.red[TOPK_WAVES + w]);
  }
  const uint32_t range = kmax - kmin;  // relative keys live in [0, range]
  const int bits = 32 - __builtin_clz(range | 1u);
  int shift = bits > 8 ? bits - 8 : 0;  // first digit = the top 8 significant bits

  // ---- 2. histogram of the first digit, threshold bin
  uint32_t prefix = 0, mask = 0;  // candidates: (rel & mask) == prefix
  uint32_t need = (uint32_t)K;
#pragma unroll
  for (int i = 0; i < ntiles; ++i) {
    if (i * TOPK_THREADS + tid < N) atomicAdd(&sh.hist[((key_at(i) - kmin) >> shift) & 255u], 1u);
  }
  __syncthreads();
  if (wave == 0) pick_bin(sh, lane, need);
  __syncthreads();
  prefix = sh.bcast[0] << shift;
  mask = 255u << shift;
  need -= sh.bcast[1];
  uint32_t ncand = sh.bcast[2];

  // ---- 3. exact threshold inside the bin
  uint32_t tau = prefix, need_eq = need;  // valid as is when no bits are left (shift == 0)
  while (shift > 0) {
    if (ncand <= (uint32_t)TOPK_MAX_CAND) {
      // few candidates: list them, rank them by (key desc, index asc)
#pragma unroll
      for (int i = 0; i < ntiles; ++i) {
        const int j = i * TOPK_THREADS + tid;
        if (j < N) {
          const uint32_t rel = key_at(i) - kmin;
          if ((rel & mask) == prefix) {
            const uint32_t slot = atomicAdd(&sh.cand_n, 1u);
            sh.cand_key[slot] = rel;
            sh.cand_idx[slot] = (uint32_t)j;
          }
        }
      }
      __syncthreads();
      if ((uint32_t)tid < ncand) {
        const uint32_t mk = sh.cand_key[tid], mi = sh.cand_idx[tid];
        uint32_t rank = 0, gtk = 0;
        for (uint32_t u = 0; u < ncand; ++u) {
          const uint32_t ok = sh.cand_key[u], oi = sh.cand_idx[u];
          gtk += ok > mk;
          rank += (ok > mk) || (ok == mk && oi < mi);
        }
        if (rank == need - 1) {
          sh.bcast[0] = mk;
          sh.bcast[1] = need - gtk;  // how many blocks with key == tau are taken
        }
      }
      __syncthreads();
      tau = sh.bcast[0];
      need_eq = sh.bcast[1];
      break;
    }
    // crowded bin: next 8-bit digit
    shift = shift > 8 ? shift - 8 : 0;
    if (tid < 256) sh.hist[tid] = 0;
    __syncthreads();
#pragma unroll
    for (int i = 0; i < ntiles; ++i) {
      if (i * TOPK_THREADS + tid < N) {
        const uint32_t rel = key_at(i) - kmin;
        if ((rel & mask) == prefix) atomicAdd(&sh.hist[(rel >> shift) & 255u], 1u);
      }
    }
    __syncthreads();
    if (wave == 0) pick_bin(sh, lane, need);
    __syncthreads();
    prefix |= sh.bcast[0] << shift;
    mask |= 255u << shift;
    need -= sh.bcast[1];
    ncand = sh.bcast[2];
    tau = prefix;
    need_eq = need;
    __syncthreads();  // bcast is rewritten by the next round
  }

  // ---- 4. ordered compaction
  const uint64_t lt_mask = (1ull << lane) - 1ull;
  if (KPT > 0) {
    // per-(tile, wave) counts -> one exclusive scan in index order -> slots
#pragma unroll
    for (int i = 0; i < R; ++i) {
      const int j = i * TOPK_THREADS + tid;
      const uint32_t rel = key[i] - kmin;
      const bool v = j < N;
      const uint64_t bgt = __ballot(v && rel > tau), beq = __ballot(v && rel == tau);
      if (lane == 0) {
        sh.cnt_gt[i * TOPK_WAVES + wave] = (uint32_t)__popcll(bgt);
        sh.cnt_eq[i * TOPK_WAVES + wave] = (uint32_t)__popcll(beq);
      }
    }
    __syncthreads();
    if (wave < 2) {  // wave 0 scans cnt_gt, wave 1 scans cnt_eq; lane owns R*16/64 consecutive entries
      uint32_t* arr = wave == 0 ? sh.cnt_gt : sh.cnt_eq;
      constexpr int PER = (R * TOPK_WAVES + 63) / 64;
      uint32_t v[PER], tot = 0;
#pragma unroll
      for (int e = 0; e < PER; ++e) {
        const int idx = lane * PER + e;
        v[e] = idx < R * TOPK_WAVES ? arr[idx] : 0u;
        tot += v[e];
      }
      uint32_t incl = tot;
      for (int d = 1; d < 64; d <<= 1) {
        const uint32_t o = (uint32_t)__shfl_up((int)incl, d);
        if (lane >= d) incl += o;
      }
      uint32_t run = incl - tot;
#pragma unroll
      for (int e = 0; e < PER; ++e) {
        const int idx = lane * PER + e;
        if (idx < R * TOPK_WAVES) arr[idx] = run;
        run += v[e];
      }
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < R; ++i) {
      const int j = i * TOPK_THREADS + tid;
      const uint32_t rel = key[i] - kmin;
      const bool v = j < N;
      const bool gt = v && rel > tau, eq = v && rel == tau;
      const uint64_t bgt = __ballot(gt), beq = __ballot(eq);
      const uint32_t gt_before = sh.cnt_gt[i * TOPK_WAVES + wave] + (uint32_t)__popcll(bgt & lt_mask);
      const uint32_t eq_before = sh.cnt_eq[i * TOPK_WAVES + wave] + (uint32_t)__popcll(beq & lt_mask);
      if (gt || (eq && eq_before < need_eq)) {
        const uint32_t slot = gt_before + min(eq_before, need_eq);
        if (slot < (uint32_t)K) out[slot] = j;  // always true for consistent counts; keeps stores in bounds
      }
    }
  } else {
    // long segments: tile by tile with running bases
    uint32_t base_gt = 0, base_eq = 0;
    for (int i = 0; i < ntiles; ++i) {
      const int j = i * TOPK_THREADS + tid;
      const bool v = j < N;
      const uint32_t rel = v ? key_at(i) - kmin : 0u;
      const bool gt = v && rel > tau, eq = v && rel == tau;
      const uint64_t bgt = __ballot(gt), beq = __ballot(eq);
      if (lane == 0) {
        sh.cnt_gt[wave] = (uint32_t)__popcll(bgt);
        sh.cnt_eq[wave] = (uint32_t)__popcll(beq);
      }
      __syncthreads();
      uint32_t gt_before = base_gt, eq_before = base_eq, gt_tile = 0, eq_tile = 0;
#pragma unroll
      for (int w = 0; w < TOPK_WAVES; ++w) {
        const uint32_t cg = sh.cnt_gt[w], ce = sh.cnt_eq[w];
        if (w < wave) {
          gt_before += cg;
          eq_before += ce;
        }
        gt_tile += cg;
        eq_tile += ce;
      }
      gt_before += (uint32_t)__popcll(bgt & lt_mask);
      eq_before += (uint32_t)__popcll(beq & lt_mask);
      if (gt || (eq && eq_before < need_eq)) {
        const uint32_t slot = gt_before + min(eq_before, need_eq);
        if (slot < (uint32_t)K) out[slot] = j;
      }
      base_gt += gt_tile;
      base_eq += eq_tile;
      __syncthreads();
    }
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
  const dim3 grid((unsigned)pl.nseg), block(TOPK_THREADS);
  const int tiles = (pl.max_blocks + TOPK_THREADS - 1) / TOPK_THREADS;
  if (tiles <= 1)
    hipLaunchKernelGGL(topk_kernel<1>, grid, block, 0, stream, p);
  else if (tiles <= 2)
    hipLaunchKernelGGL(topk_kernel<2>, grid, block, 0, stream, p);
  else if (tiles <= 4)
    hipLaunchKernelGGL(topk_kernel<4>, grid, block, 0, stream, p);
  else if (tiles <= 8)
    hipLaunchKernelGGL(topk_kernel<8>, grid, block, 0, stream, p);
  else if (tiles <= 16)
    hipLaunchKernelGGL(topk_kernel<16>, grid, block, 0, stream, p);
  else
    hipLaunchKernelGGL(topk_kernel<0>, grid, block, 0, stream, p);
  return check_launch();
}

}  // namespace absb
