// Selection stage (Sec. 3.4, kernel 2): per (request, KV head) segment of the score array the
// K_s = min(N_s, ceil(T_b / B_h)) highest-scoring blocks; the prefix-sum offsets of the estimation
// stage delimit the segments.  Equal scores go to the lower block index and the index list is
// written in ascending order, so there is exactly one correct output.
//
// One work-group of 1024 threads per segment.  Selection is an exact threshold search that touches
// every key three times with a handful of instructions each (the kernel runs on one CU per
// segment, so instructions per key and dependent latencies, not bytes, bound it):
//   1. the segment's scores are loaded once (coalesced, unconditional, all loads in flight
//      together) and kept in registers as order-preserving unsigned keys; min/max give the range;
//   2. a 2048-bin LDS histogram over the top 11 significant bits of (key - min) and a work-group
//      scan find the bin d1 that holds the K-th largest key;
//   3. keys above bin d1 set their bit in an LDS bitmap of selected blocks; the few keys inside
//      d1 are appended to a candidate list, ranked exactly by (key desc, index asc), and the best
//      `need` of them set their bits too;
//   4. the bitmap is scanned in index order (popcount prefix sums) and the indices written out.
// A crowded bin (more than 1024 candidates, e.g. all scores equal) takes a slow path: further radix
// digits give the exact threshold tau, and blocks equal to tau are admitted in index order through
// a second bitmap.  Segments longer than 16384 blocks run the same code with keys re-read from L2.
// Wave-level reductions and scans use DPP row operations, not LDS-crossbar shuffles.
//
// Optional policy (off by default): the blocks that hold the first sink_tokens or the last
// recent_tokens tokens are always selected.  They form a prefix and a suffix of the segment, so
// they are written to the list directly and the blocks in between compete for what is left of K_s.
#include "common.h"

namespace absb {

struct TopkParams {
  const int32_t* scores;
  const int32_t* cent_off;
  const int32_t* budget;  // [Bt]
  const int32_t* seq_lens;  // [Bt]
  int32_t sink_tokens, recent_tokens;  // blocks holding these tokens are selected ahead of every score
  int32_t* sel_idx;
  int32_t* sel_cnt;
  int32_t* tickets;  // [nseg] or null: split counters of the attention kernel that follows, cleared here
  int32_t sel_stride, Hkv, tight;
  HeadTable heads;
};

constexpr int TOPK_THREADS = 1024;
constexpr int TOPK_WAVES = TOPK_THREADS / 64;
constexpr int TOPK_MAX_CAND = 1024;       // candidates ranked by brute force
constexpr int TOPK_MAX_BLOCKS = 1 << 17;  // bitmap capacity (2 x 16 KiB of LDS)
constexpr int TOPK_DIGIT_BITS = 11;
constexpr int TOPK_BINS = 1 << TOPK_DIGIT_BITS;  // two bins per thread

__device__ __forceinline__ uint32_t ordered_key(int32_t score) { return (uint32_t)score ^ 0x80000000u; }

struct TopkShared {
  uint32_t red[2 * TOPK_WAVES];
  uint32_t hist[TOPK_BINS];
  uint32_t bcast[4];
  uint32_t cand_key[TOPK_MAX_CAND];
  uint32_t cand_idx[TOPK_MAX_CAND];
  uint32_t cand_n;
  uint32_t wave_a[TOPK_WAVES], wave_b[TOPK_WAVES];
};

struct UMin {
  __device__ __forceinline__ uint32_t operator()(uint32_t a, uint32_t b) const { return a < b ? a : b; }
};
struct UMax {
  __device__ __forceinline__ uint32_t operator()(uint32_t a, uint32_t b) const { return a > b ? a : b; }
};

// Exclusive prefix sum of one value per thread over the work-group (thread order); *total = sum.
// `slot` is 16 words of LDS scratch.  Contains one barrier: call from uniform control flow.
__device__ __forceinline__ uint32_t block_excl_scan(uint32_t v, uint32_t* slot, int lane, int wave, uint32_t* total) {
  uint32_t wave_total;
  const uint32_t incl = wave_incl_scan_u32(v, &wave_total);
  if (lane == 0) slot[wave] = wave_total;
  __syncthreads();
  // 16 wave totals: every 16-lane row scans them again (cheaper than a second barrier)
  const uint32_t mine = slot[lane & (TOPK_WAVES - 1)];
  uint32_t s = mine;
  s += (uint32_t)dpp_i<0x111>((int)s);
  s += (uint32_t)dpp_i<0x112>((int)s);
  s += (uint32_t)dpp_i<0x114>((int)s);
  s += (uint32_t)dpp_i<0x118>((int)s);  // inclusive over the row = over waves 0..(lane&15)
  *total = (uint32_t)__builtin_amdgcn_readlane((int)s, 15);
  // exclusive prefix of this thread's wave: lane `wave` holds the sum over waves 0..wave; drop own total
  const uint32_t upto = (uint32_t)__builtin_amdgcn_readlane((int)s, __builtin_amdgcn_readfirstlane(wave));
  return upto - wave_total + incl - v;
}

// From the histogram of the current digit among the candidates: the bin holding the `need`-th
// largest candidate.  All threads take part (two bins each, highest bins first).
// bcast = {bin, candidates above it, candidates in it}.  Two barriers inside.
__device__ __forceinline__ void pick_bin(TopkShared& sh, int tid, int lane, int wave, uint32_t need) {
  const int hi = TOPK_BINS - 1 - 2 * tid;  // descending: thread 0 owns the two highest bins
  const uint32_t c0 = sh.hist[hi], c1 = sh.hist[hi - 1];
  uint32_t total;
  uint32_t above = block_excl_scan(c0 + c1, sh.wave_a, lane, wave, &total);
  if (above < need && need <= above + c0) {
    sh.bcast[0] = (uint32_t)hi;
    sh.bcast[1] = above;
    sh.bcast[2] = c0;
  }
  above += c0;
  if (above < need && need <= above + c1) {
    sh.bcast[0] = (uint32_t)(hi - 1);
    sh.bcast[1] = above;
    sh.bcast[2] = c1;
  }
  __syncthreads();
}

// KPT > 0: keys of the segment live in registers (N <= KPT*1024).  KPT == 0: keys are re-read.
template <int KPT>
__global__ __launch_bounds__(TOPK_THREADS) void topk_kernel(TopkParams p) {
  extern __shared__ uint32_t s_bitmap[];  // [2][words]: selected-by-key bits, then equal-to-tau bits
  __shared__ TopkShared sh;
  const int s = blockIdx.x;
  const int b = s / p.Hkv, h = s % p.Hkv;
  const int off = p.cent_off[s];
  const int lb = p.heads.log2_block[h];
  const int Nall = blocks_in_use(p.tight, p.cent_off[s + 1] - off, p.seq_lens, b, lb);
  const int T = p.budget[b];
  int K = (int)(((int64_t)T + (1 << lb) - 1) >> lb);
  K = min(min(K, Nall), p.sel_stride);
  // Forced blocks are a prefix [0, lo) (they hold the first sink_tokens tokens) and a suffix
  // [hi, Nall) (the last recent_tokens tokens) of the segment; they are selected ahead of every
  // score, lowest index first, and the blocks [lo, hi) compete by score for what is left of K.
  int lo = 0, hi = Nall;
  if (p.sink_tokens > 0) lo = min(Nall, (int)(((int64_t)p.sink_tokens + (1 << lb) - 1) >> lb));
  if (p.recent_tokens > 0) hi = max(lo, min(Nall, max(0, p.seq_lens[b] - p.recent_tokens) >> lb));
  const int nforced = lo + (Nall - hi);
  const int N = hi - lo;  // competing blocks; the code below indexes them from 0
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int32_t* sc = p.scores + off + (N > 0 ? lo : 0);
  int32_t* out = p.sel_idx + (size_t)s * p.sel_stride;
  constexpr int R = KPT > 0 ? KPT : 1;
  const int ntiles = KPT > 0 ? KPT : (N + TOPK_THREADS - 1) / TOPK_THREADS;
  const int nwords = (N + 31) >> 5;
  uint32_t* bm_gt = s_bitmap;
  uint32_t* bm_eq = s_bitmap + nwords;

  // keys first: everything else waits on them.  The index is clamped instead of the load being
  // predicated, so the loads issue back to back (the clamp keeps them legal when nothing competes).
  const int jlast = max(N - 1, 0);
  uint32_t key[R];
  if (KPT > 0) {
#pragma unroll
    for (int i = 0; i < R; ++i) key[i] = ordered_key(sc[min(i * TOPK_THREADS + tid, jlast)]);
  }
  auto key_at = [&](int i) -> uint32_t {  // meaningful only for i*1024+tid < N
    if (KPT > 0) return key[i];
    return ordered_key(sc[min(i * TOPK_THREADS + tid, jlast)]);
  };

  if (tid == 0) {
    p.sel_cnt[s] = K;
    if (p.tickets) p.tickets[(size_t)s * ABSB_TICKET_STRIDE] = 0;
  }
#pragma unroll 1
  for (int i = K + tid; i < p.sel_stride; i += TOPK_THREADS) out[i] = -1;
  if (K >= Nall) {  // everything is selected
#pragma unroll 1
    for (int i = tid; i < Nall; i += TOPK_THREADS) out[i] = i;
    return;
  }
  if (nforced >= K) {  // the forced blocks alone fill the list: lowest indices first
#pragma unroll 1
    for (int i = tid; i < K; i += TOPK_THREADS) out[i] = i < lo ? i : hi + (i - lo);
    return;
  }
  // list = forced prefix, then the chosen ones of [lo, hi) (written below, relative to `out`), then
  // the forced suffix
  K -= nforced;
#pragma unroll 1
  for (int i = tid; i < lo; i += TOPK_THREADS) out[i] = i;
#pragma unroll 1
  for (int i = tid; i < Nall - hi; i += TOPK_THREADS) out[lo + K + i] = hi + i;
  out += lo;

  sh.hist[tid] = 0;
  sh.hist[tid + TOPK_THREADS] = 0;
  if (tid == 0) sh.cand_n = 0;
#pragma unroll 1
  for (int w = tid; w < 2 * nwords; w += TOPK_THREADS) s_bitmap[w] = 0;

  // ---- 1. range of the keys (clamped duplicates of the last key do not change min/max)
  uint32_t kmin = 0xffffffffu, kmax = 0u;
#pragma unroll
  for (int i = 0; i < ntiles; ++i) {
    const uint32_t k = key_at(i);
    kmin = min(kmin, k);
    kmax = max(kmax, k);
  }
  kmin = wave_reduce_u32(kmin, UMin());
  kmax = wave_reduce_u32(kmax, UMax());
  if (lane == 0) {
    sh.red[wave] = kmin;
    sh.red[TOPK_WAVES + wave] = kmax;
  }
  __syncthreads();
  kmin = row16_reduce_u32(sh.red[lane & (TOPK_WAVES - 1)], UMin());
  kmax = row16_reduce_u32(sh.red[TOPK_WAVES + (lane & (TOPK_WAVES - 1))], UMax());
  const uint32_t range = kmax - kmin;  // relative keys live in [0, range]
  const int bits = 32 - __builtin_clz(range | 1u);
  int shift = bits > TOPK_DIGIT_BITS ? bits - TOPK_DIGIT_BITS : 0;  // first digit = the top significant bits

  // ---- 2. histogram of the first digit, threshold bin
  // (slots past the end hold copies of the last key: counting them would pile thousands of LDS
  // atomics on one bin, so they are skipped, not corrected for afterwards)
#pragma unroll
  for (int i = 0; i < ntiles; ++i) {
    if (i * TOPK_THREADS + tid < N) atomicAdd(&sh.hist[(key_at(i) - kmin) >> shift], 1u);
  }
  __syncthreads();
  pick_bin(sh, tid, lane, wave, (uint32_t)K);
  const uint32_t d1 = sh.bcast[0];
  uint32_t need = (uint32_t)K - sh.bcast[1];
  uint32_t ncand = sh.bcast[2];
  uint32_t need_eq = 0;

  if (shift == 0 || ncand <= (uint32_t)TOPK_MAX_CAND) {
    // ---- 3. keys above the bin are selected; keys inside it become candidates
    // (with shift == 0 the bin is a single key value: its members tie, lowest index first)
    const bool list_cands = ncand <= (uint32_t)TOPK_MAX_CAND;
#pragma unroll
    for (int i = 0; i < ntiles; ++i) {
      const int j = i * TOPK_THREADS + tid;
      const uint32_t rel = key_at(i) - kmin;
      const uint32_t dg = rel >> shift;
      if (dg >= d1 && j < N) {  // the digit test comes first: it fails for almost every key
        if (dg > d1) {
          atomicOr(&bm_gt[j >> 5], 1u << (j & 31));
        } else if (list_cands) {
          const uint32_t slot = atomicAdd(&sh.cand_n, 1u);
          sh.cand_key[slot] = rel;
          sh.cand_idx[slot] = (uint32_t)j;
        } else {
          atomicOr(&bm_eq[j >> 5], 1u << (j & 31));
        }
      }
    }
    __syncthreads();
    if (list_cands) {
      if ((uint32_t)tid < ncand) {
        const uint32_t mk = sh.cand_key[tid], mi = sh.cand_idx[tid];
        uint32_t rank = 0;
#pragma unroll 4
        for (uint32_t u = 0; u < ncand; ++u) {
          const uint32_t ok = sh.cand_key[u], oi = sh.cand_idx[u];
          rank += (ok > mk) || (ok == mk && oi < mi);
        }
        if (rank < need) atomicOr(&bm_gt[mi >> 5], 1u << (mi & 31));
      }
    } else {
      need_eq = need;  // bin == one key value: admit its first `need` members by index
    }
    __syncthreads();
  } else {
    // ---- slow path: crowded bin.  More radix digits until the bin is a single key value.
    uint32_t prefix = d1 << shift, mask = (uint32_t)(TOPK_BINS - 1) << shift;
    while (shift > 0) {
      shift = shift > TOPK_DIGIT_BITS ? shift - TOPK_DIGIT_BITS : 0;
      sh.hist[tid] = 0;
      sh.hist[tid + TOPK_THREADS] = 0;
      __syncthreads();
#pragma unroll 1
      for (int j = tid; j < N; j += TOPK_THREADS) {
        const uint32_t rel = ordered_key(sc[j]) - kmin;
        if ((rel & mask) == prefix) atomicAdd(&sh.hist[(rel >> shift) & (uint32_t)(TOPK_BINS - 1)], 1u);
      }
      __syncthreads();
      pick_bin(sh, tid, lane, wave, need);
      prefix |= sh.bcast[0] << shift;
      mask |= (uint32_t)(TOPK_BINS - 1) << shift;
      need -= sh.bcast[1];
      __syncthreads();  // bcast is rewritten by the next round
    }
    const uint32_t tau = prefix;
    need_eq = need;
#pragma unroll 1
    for (int j = tid; j < N; j += TOPK_THREADS) {
      const uint32_t rel = ordered_key(sc[j]) - kmin;
      if (rel > tau)
        atomicOr(&bm_gt[j >> 5], 1u << (j & 31));
      else if (rel == tau)
        atomicOr(&bm_eq[j >> 5], 1u << (j & 31));
    }
    __syncthreads();
  }

  // ---- 4. bitmaps -> ascending index list
  uint32_t base_gt = 0, base_eq = 0;
#pragma unroll 1
  for (int w0 = 0; w0 < nwords; w0 += TOPK_THREADS) {
    const int w = w0 + tid;
    const uint32_t g = w < nwords ? bm_gt[w] : 0u;
    const uint32_t e = (need_eq > 0 && w < nwords) ? bm_eq[w] : 0u;
    uint32_t tot_gt, tot_eq = 0;
    uint32_t G = base_gt + block_excl_scan((uint32_t)__popc(g), sh.wave_a, lane, wave, &tot_gt);
    uint32_t E = base_eq;
    if (need_eq > 0) E += block_excl_scan((uint32_t)__popc(e), sh.wave_b, lane, wave, &tot_eq);
    uint32_t bitsleft = g | e;
#pragma unroll 1
    while (bitsleft) {
      const int bpos = __builtin_ctz(bitsleft);
      bitsleft &= bitsleft - 1;
      const int idx = (w << 5) + bpos;
      if ((g >> bpos) & 1u) {
        const uint32_t slot = G + min(E, need_eq);
        if (slot < (uint32_t)K) out[slot] = idx + lo;  // always true for consistent counts; keeps stores in bounds
        ++G;
      } else {
        if (E < need_eq) {
          const uint32_t slot = G + E;
          if (slot < (uint32_t)K) out[slot] = idx + lo;
        }
        ++E;
      }
    }
    base_gt += tot_gt;
    base_eq += tot_eq;
    __syncthreads();  // the scan scratch is reused by the next tile of words
  }
}

int launch_topk(const Geometry& g, const Plan& pl, const int32_t* scores, const int32_t* cent_off,
                const int32_t* budget, const int32_t* seq_lens, int32_t* sel_idx, int32_t* sel_cnt,
                int32_t sel_stride, int32_t* tickets, hipStream_t stream) {
  if (pl.max_blocks > TOPK_MAX_BLOCKS) return ABSB_ERR_UNSUPPORTED;
  TopkParams p;
  p.scores = scores;
  p.cent_off = cent_off;
  p.budget = budget;
  p.seq_lens = seq_lens;
  p.tight = g.tight;
  p.sink_tokens = g.sink_tokens;
  p.recent_tokens = g.recent_tokens;
  p.sel_idx = sel_idx;
  p.sel_cnt = sel_cnt;
  p.tickets = tickets;
  p.sel_stride = sel_stride;
  p.Hkv = g.Hkv;
  p.heads = g.heads;
  const dim3 grid((unsigned)pl.nseg), block(TOPK_THREADS);
  const size_t lds = (size_t)2 * ((pl.max_blocks + 31) / 32) * sizeof(uint32_t);
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
