// Selection stage, device side (Sec. 3.4, kernel 2): the work a work-group does for one
// (request, KV head) segment.  Used by the stand-alone selection kernel (1024 threads) and by the
// one-launch decode step (256 threads, the segment's scores arriving from other work-groups).
//
// Selection is an exact threshold search that touches every key three times with a handful of
// instructions each (it runs on one CU per segment, so instructions per key and dependent
// latencies, not bytes, bound it):
//   1. the segment's scores are loaded once (coalesced, unconditional, all loads in flight
//      together) and kept in registers as order-preserving unsigned keys; min/max give the range;
//   2. a 2048-bin LDS histogram over the top 11 significant bits of (key - min) and a work-group
//      scan find the bin d1 that holds the K-th largest key;
//   3. keys above bin d1 set their bit in an LDS bitmap of selected blocks; the few keys inside
//      d1 are appended to a candidate list; a long list is cut down by histogram rounds over
//      further digits of the key, a short one is ranked exactly by (key desc, index asc), and the
//      best `need` candidates set their bits too;
//   4. the bitmap is scanned in index order (every thread a run of words, one popcount prefix sum over
//      the work-group) and the indices written out.
// A crowded bin (more than 1024 candidates, e.g. all scores equal) takes a slow path: further radix
// digits give the exact threshold tau, and blocks equal to tau are admitted in index order through
// a second bitmap.  Segments too long for the register tile run the same code with keys re-read.
// Wave-level reductions and scans use DPP row operations, not LDS-crossbar shuffles.
//
// Optional policy (off by default): the blocks that hold the first sink_tokens or the last
// recent_tokens tokens are always selected.  They form a prefix and a suffix of the segment, so
// they are written to the list directly and the blocks in between compete for what is left of K_s.
#pragma once
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
  // Only for the selection that runs inside the pipelined one-launch step (EARLY): the list the
  // attention work-groups read, the flag per segment that says it is complete; sel_idx is then
  // the caller's copy in ascending order and may be null.
  int32_t* work_list;  // [nseg, sel_stride]
  int32_t* flags;      // [nseg], ABSB_TICKET_STRIDE apart
  int32_t sel_stride, Hkv, tight;
  int32_t Hsel, Rk;  // selection segments per request, selection segments per KV head
  HeadTable heads;
};

inline TopkParams make_topk_params(const Geometry& g, const int32_t* scores, const int32_t* cent_off,
                                   const int32_t* budget, const int32_t* seq_lens, int32_t* sel_idx,
                                   int32_t* sel_cnt, int32_t sel_stride, int32_t* tickets) {
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
  p.work_list = nullptr;
  p.flags = nullptr;
  p.sel_stride = sel_stride;
  p.Hkv = g.Hkv;
  p.Hsel = g.Hsel;
  p.Rk = g.Rk;
  p.heads = g.heads;
  return p;
}

constexpr int TOPK_MAX_CAND = 1024;       // longest candidate list
constexpr int TOPK_RANK_MAX = 128;        // candidates ranked against each other (quadratic work)
constexpr int TOPK_MAX_BLOCKS = ABSB_MAX_SEL_BLOCKS;  // bitmap capacity (2 x 16 KiB of LDS)
constexpr int TOPK_DIGIT_BITS = 11;
constexpr int TOPK_BINS = 1 << TOPK_DIGIT_BITS;
constexpr int TOPK_SLOTS = 16;            // per-wave scratch words: up to 16 waves per work-group

__device__ __forceinline__ uint32_t ordered_key(int32_t score) { return (uint32_t)score ^ 0x80000000u; }

struct TopkShared {
  uint32_t red[2 * TOPK_SLOTS];
  uint32_t hist[TOPK_BINS + 64];  // the bins, then one dump word per lane (slots past a segment's end)
  uint32_t bcast[4];
  uint32_t cand_key[TOPK_MAX_CAND];
  uint32_t cand_idx[TOPK_MAX_CAND];
  uint32_t cand_n;
  uint32_t wave_a[TOPK_SLOTS], wave_b[TOPK_SLOTS];
};
// LDS a segment's selection needs: the fixed part, then two bitmaps of one bit per block.
__host__ __device__ constexpr size_t topk_lds_bytes(int max_blocks) {
  return ((sizeof(TopkShared) + 15) & ~size_t(15)) + (size_t)2 * ((max_blocks + 31) / 32) * sizeof(uint32_t);
}

struct UMin {
  __device__ __forceinline__ uint32_t operator()(uint32_t a, uint32_t b) const { return a < b ? a : b; }
};
struct UMax {
  __device__ __forceinline__ uint32_t operator()(uint32_t a, uint32_t b) const { return a > b ? a : b; }
};

// Exclusive prefix sum of one value per thread over the work-group (thread order); *total = sum.
// `slot` is 16 words of LDS scratch.  Contains one barrier: call from uniform control flow.
template <int NT>
__device__ __forceinline__ uint32_t block_excl_scan(uint32_t v, uint32_t* slot, int lane, int wave, uint32_t* total) {
  constexpr int WAVES = NT / 64;
  static_assert(WAVES >= 1 && WAVES <= TOPK_SLOTS, "one scratch word per wave");
  uint32_t wave_total;
  const uint32_t incl = wave_incl_scan_u32(v, &wave_total);
  if (lane == 0) slot[wave] = wave_total;
  __syncthreads();
  // the wave totals: every 16-lane row scans them again (cheaper than a second barrier)
  const int r = lane & (TOPK_SLOTS - 1);
  uint32_t s = r < WAVES ? slot[r] : 0u;
  s += (uint32_t)dpp_i<0x111>((int)s);
  s += (uint32_t)dpp_i<0x112>((int)s);
  s += (uint32_t)dpp_i<0x114>((int)s);
  s += (uint32_t)dpp_i<0x118>((int)s);  // inclusive over the row = over waves 0..(lane&15)
  *total = (uint32_t)__builtin_amdgcn_readlane((int)s, 15);
  // exclusive prefix of this thread's wave: lane `wave` holds the sum over waves 0..wave; drop own total
  const uint32_t upto = (uint32_t)__builtin_amdgcn_readlane((int)s, __builtin_amdgcn_readfirstlane(wave));
  return upto - wave_total + incl - v;
}

// A slot of an LDS list for every lane that calls it (any subset of a wave, from divergent code):
// one atomic per wave, not per lane.
__device__ __forceinline__ uint32_t append_slot(uint32_t* counter) {
  const uint64_t m = __builtin_amdgcn_ballot_w64(true);  // the lanes that are here
  const uint32_t before = __builtin_amdgcn_mbcnt_hi((uint32_t)(m >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)m, 0u));
  uint32_t base = 0;
  if (before == 0) base = atomicAdd(counter, (uint32_t)__popcll(m));
  return (uint32_t)__builtin_amdgcn_readfirstlane((int)base) + before;
}

// key[i] for an index known only at run time, without leaving the registers: a select tree over
// the bits of i (R - 1 selects).  Used on the rare paths only.
template <int R>
__device__ __forceinline__ uint32_t pick_reg(const uint32_t (&key)[R], int i) {
  uint32_t t[R];
#pragma unroll
  for (int k = 0; k < R; ++k) t[k] = key[k];
#pragma unroll
  for (int s = 1, b = 0; s < R; s <<= 1, ++b) {
    const uint32_t up = 0u - (uint32_t)((i >> b) & 1);  // a bit-mask blend: stays a register operation
#pragma unroll
    for (int k = 0; k + s < R; k += 2 * s) t[k] = (t[k + s] & up) | (t[k] & ~up);
  }
  return t[0];
}

// From the histogram of the current digit among the candidates: the bin holding the `need`-th
// largest candidate.  All threads take part (TOPK_BINS / NT bins each, highest bins first).
// bcast = {bin, candidates above it, candidates in it}.  Two barriers inside.
template <int NT>
__device__ __forceinline__ void pick_bin(TopkShared& sh, int tid, int lane, int wave, uint32_t need) {
  constexpr int BPT = TOPK_BINS / NT;
  const int hi = TOPK_BINS - 1 - BPT * tid;  // descending: thread 0 owns the highest bins
  uint32_t c[BPT], sum = 0;
#pragma unroll
  for (int k = 0; k < BPT; ++k) {
    c[k] = sh.hist[hi - k];
    sum += c[k];
  }
  uint32_t total;
  uint32_t above = block_excl_scan<NT>(sum, sh.wave_a, lane, wave, &total);
#pragma unroll
  for (int k = 0; k < BPT; ++k) {
    if (above < need && need <= above + c[k]) {
      sh.bcast[0] = (uint32_t)(hi - k);
      sh.bcast[1] = above;
      sh.bcast[2] = c[k];
    }
    above += c[k];
  }
  __syncthreads();
}

// The selection of selection segment t by one work-group of NT threads.
//   KPT > 0: keys of the segment live in registers (competing blocks <= KPT*NT); KPT == 0: re-read.
//   COH: the scores were written, and the list will be read, by other work-groups of this launch.
//   EARLY: attention work-groups of this launch are waiting for the segment's flag.  What they read is
//     p.work_list, a permutation of the selection (attention does not care about the order of its
//     blocks), raised as soon as the members are known: forced blocks, then the blocks above the
//     threshold bin in the order (thread, tile), then the admitted candidates by rank; the order is
//     a function of the scores alone.  The ascending list in p.sel_idx, if the caller wants one, is
//     written after the flag, off the path the attention waits on.  On the rare paths (a long
//     candidate list, ties, more blocks than a register tile holds) the work list is the ascending
//     list and the flag goes up at the end.
//   sh, bitmap: LDS as sized by topk_lds_bytes().
// Every thread of the work-group must call it; all of them return together.
template <int NT, int KPT, bool COH, bool EARLY = false>
__device__ __forceinline__ void topk_segment(const TopkParams& p, int t, TopkShared& sh, uint32_t* s_bitmap) {
  constexpr int WAVES = NT / 64;
  const SegMap sm = seg_map(t, p.Hsel, p.Rk, p.Hkv);
  const int b = sm.b;
  const int off = p.cent_off[sm.s];
  const int rows = p.cent_off[sm.s + 1] - off;
  const int lb = p.heads.log2_block[sm.hk];
  const int Nall = blocks_in_use(p.tight, rows, p.seq_lens, b, lb);
  int K = budget_blocks(p.budget[b], lb, Nall, p.sel_stride);
  // Forced blocks are a prefix [0, lo) (they hold the first sink_tokens tokens) and a suffix
  // [hi, Nall) (the last recent_tokens tokens) of the segment; they are selected ahead of every
  // score, lowest index first, and the blocks [lo, hi) compete by score for what is left of K.
  int lo = 0, hi = Nall;
  if (p.sink_tokens > 0) lo = min(Nall, (int)(((int64_t)p.sink_tokens + (1 << lb) - 1) >> lb));
  if (p.recent_tokens > 0) hi = max(lo, min(Nall, max(0, p.seq_lens[b] - p.recent_tokens) >> lb));
  const int nforced = lo + (Nall - hi);
  const int N = hi - lo;  // competing blocks; the code below indexes them from 0
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int32_t* sc = p.scores + score_base(sm, p.Rk, off, rows) + (N > 0 ? lo : 0);
  // `out`: the ascending list (null: not wanted; only possible with EARLY); `wl`: the work list
  int32_t* out = (!EARLY || p.sel_idx) ? p.sel_idx + (size_t)t * p.sel_stride : nullptr;
  int32_t* wl = EARLY ? p.work_list + (size_t)t * p.sel_stride : nullptr;
  auto publish = [&]() __attribute__((always_inline)) {  // EARLY: the work list is complete
    wait_stores_acknowledged();
    __syncthreads();
    if (tid == 0) st_i32<true>(p.flags + (size_t)t * ABSB_TICKET_STRIDE, 1);
  };
  constexpr int R = KPT > 0 ? KPT : 1;
  const int ntiles = KPT > 0 ? KPT : (N + NT - 1) / NT;
  const int nwords = (N + 31) >> 5;
  uint32_t* bm_gt = s_bitmap;
  uint32_t* bm_eq = s_bitmap + nwords;

  // keys first: everything else waits on them.  The index is clamped instead of the load being
  // predicated, so the loads issue back to back (the clamp keeps them legal when nothing competes).
  const int jlast = max(N - 1, 0);
  uint32_t key[R];
  if (KPT > 0) {
#pragma unroll
    for (int i = 0; i < R; ++i) key[i] = ordered_key(ld_i32<COH>(sc + min(i * NT + tid, jlast)));
  }
  auto key_at = [&](int i) -> uint32_t {  // meaningful only for i*NT+tid < N
    if (KPT > 0) return key[i];
    return ordered_key(ld_i32<COH>(sc + min(i * NT + tid, jlast)));
  };

  if (tid == 0) {
    st_i32<COH>(p.sel_cnt + t, K);
    if (p.tickets) p.tickets[(size_t)t * ABSB_TICKET_STRIDE] = 0;
  }
  // entry i of the ascending list (and of the work list, while that one is kept ascending)
  bool wl_ascending = EARLY;
  auto put = [&](int i, int v) __attribute__((always_inline)) {
    if (!EARLY || out) st_i32<COH>(out + i, v);
    if (EARLY && wl_ascending) st_i32<true>(wl + i, v);
  };
  if (!EARLY || out) {
#pragma unroll 1
    for (int i = K + tid; i < p.sel_stride; i += NT) st_i32<COH>(out + i, -1);
  }
  if (K >= Nall) {  // everything is selected
#pragma unroll 1
    for (int i = tid; i < Nall; i += NT) put(i, i);
    if (EARLY && K > 0) publish();
    return;
  }
  if (nforced >= K) {  // the forced blocks alone fill the list: lowest indices first
#pragma unroll 1
    for (int i = tid; i < K; i += NT) put(i, i < lo ? i : hi + (i - lo));
    if (EARLY && K > 0) publish();
    return;
  }
  // list = forced prefix, then the chosen ones of [lo, hi) (written below, at lo + their rank by
  // index), then the forced suffix
  K -= nforced;
#pragma unroll 1
  for (int i = tid; i < lo; i += NT) put(i, i);
  if (!EARLY || out) {
#pragma unroll 1
    for (int i = tid; i < Nall - hi; i += NT) st_i32<COH>(out + lo + K + i, hi + i);
  }

#pragma unroll
  for (int i = tid; i < TOPK_BINS; i += NT) sh.hist[i] = 0;
  if (tid == 0) sh.cand_n = 0;
#pragma unroll 1
  for (int w = tid; w < 2 * nwords; w += NT) s_bitmap[w] = 0;

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
    sh.red[TOPK_SLOTS + wave] = kmax;
  }
  __syncthreads();
  {
    const int r = lane & (TOPK_SLOTS - 1);
    kmin = row16_reduce_u32(r < WAVES ? sh.red[r] : 0xffffffffu, UMin());
    kmax = row16_reduce_u32(r < WAVES ? sh.red[TOPK_SLOTS + r] : 0u, UMax());
  }
  const uint32_t range = kmax - kmin;  // relative keys live in [0, range]
  // from here on only key - min is needed: kept in place of the key (one register per key)
  if (KPT > 0) {
#pragma unroll
    for (int i = 0; i < R; ++i) key[i] -= kmin;
  }
  auto rel_at = [&](int i) -> uint32_t {
    if (KPT > 0) return key[i];
    return ordered_key(ld_i32<COH>(sc + min(i * NT + tid, jlast))) - kmin;
  };
  const int bits = 32 - __builtin_clz(range | 1u);
  int shift = bits > TOPK_DIGIT_BITS ? bits - TOPK_DIGIT_BITS : 0;  // first digit = the top significant bits

  // ---- 2. histogram of the first digit, threshold bin
  // (slots past the end hold copies of the last key: counting them would pile thousands of LDS
  // atomics on one bin, so they are kept out, not corrected for afterwards)
  //
  // With a register tile the passes over the keys are written without branches and without
  // changes of the execution mask: a 4-wave work-group has one wave per SIMD, which cannot overlap
  // its own scalar, vector and LDS instructions across such changes (measured: ~14 cycles per
  // instruction with a predicated body per key, against ~5 for straight-line code).  Which of the
  // thread's tiles hold a block of the segment (tile i holds block i*NT + tid) is a bit mask; a
  // slot past the end is counted into a dump word of its lane instead of a bin.
  const int nvalid = N > tid ? (N - tid + NT - 1) / NT : 0;
  const uint64_t valid = nvalid >= 64 ? ~0ull : ((1ull << nvalid) - 1ull);
  if (KPT > 0) {
#pragma unroll
    for (int i = 0; i < R; ++i) {
      const uint32_t dg = key[i] >> shift;
      const uint32_t m = 0u - (uint32_t)((valid >> i) & 1ull);  // all ones for a real block
      atomicAdd(&sh.hist[(dg & m) | ((uint32_t)(TOPK_BINS + lane) & ~m)], 1u);
    }
  } else {
#pragma unroll 1
    for (int i = 0; i < ntiles; ++i) {
      if (i * NT + tid < N) atomicAdd(&sh.hist[rel_at(i) >> shift], 1u);
    }
  }
  __syncthreads();
  // The next pass over the keys recomputes its digits instead of carrying one more register per
  // key across the barrier: with a long register tile that carrying spills.  The empty statements
  // make the values opaque to the optimiser.
  if (KPT > 8) {
#pragma unroll
    for (int i = 0; i < R; ++i) asm volatile("" : "+v"(key[i]));
  }
  pick_bin<NT>(sh, tid, lane, wave, (uint32_t)K);
  const uint32_t d1 = sh.bcast[0];
  uint32_t need = (uint32_t)K - sh.bcast[1];
  uint32_t ncand = sh.bcast[2];
  uint32_t need_eq = 0;
  // The common case (a short candidate list) with EARLY: members go to the work list as they are
  // found, at places fixed by a count per thread and one scan, and the bitmaps are only needed if
  // the caller wants the ascending list.  Layout: [0, lo) forced prefix, [lo, nforced) forced
  // suffix, then the K - need blocks above the bin, then the `need` admitted candidates.
  const bool direct = EARLY && KPT > 0 && ncand <= (uint32_t)TOPK_RANK_MAX;
  const bool use_bm = !direct || out != nullptr;
  const uint32_t wl_cand0 = (uint32_t)nforced + ((uint32_t)K - need);  // first candidate's place
  if (EARLY) {
    wl_ascending = !direct;
    const int at = direct ? lo : lo + K;
#pragma unroll 1
    for (int i = tid; i < Nall - hi; i += NT) st_i32<true>(wl + at + i, hi + i);
  }

  if (shift == 0 || ncand <= (uint32_t)TOPK_MAX_CAND) {
    // ---- 3. keys above the bin are selected; keys inside it become candidates
    // (with shift == 0 the bin is a single key value: its members tie, lowest index first)
    const bool list_cands = ncand <= (uint32_t)TOPK_MAX_CAND;
    if (KPT > 0) {
      // straight-line pass: which of the thread's tiles lie above / inside the threshold bin, as two
      // bit masks built by shifting (tiles taken from the last to the first, so tile i ends up at
      // bit i of its 32-bit half); the few set bits are then worked off in two short loops
      constexpr int NW = R > 32 ? 2 : 1;  // 32-bit halves of the masks in use
      uint32_t above[NW], inside[NW];
#pragma unroll
      for (int w = 0; w < NW; ++w) above[w] = inside[w] = 0u;
#pragma unroll
      for (int i = R - 1; i >= 0; --i) {
        const uint32_t dg = key[i] >> shift;
        const int w = NW == 2 ? (i >> 5) : 0;
        above[w] = (above[w] << 1) | (uint32_t)(dg > d1);
        inside[w] = (inside[w] << 1) | (uint32_t)(dg == d1);
      }
      uint32_t wl_pos = 0;  // direct: this thread's next place in the work list
      if (direct) {
        uint32_t mine = 0, total;
#pragma unroll
        for (int w = 0; w < NW; ++w) mine += (uint32_t)__popc(above[w] & (uint32_t)(valid >> (32 * w)));
        wl_pos = (uint32_t)nforced + block_excl_scan<NT>(mine, sh.wave_b, lane, wave, &total);
      }
#pragma unroll
      for (int w = 0; w < NW; ++w) {
        const uint32_t ok = (uint32_t)(valid >> (32 * w));
        uint32_t left = above[w] & ok;
#pragma unroll 1
        while (left) {
          const int j = (__builtin_ctz(left) + 32 * w) * NT + tid;
          left &= left - 1;
          if (use_bm) atomicOr(&bm_gt[j >> 5], 1u << (j & 31));
          if (direct) {
            if (wl_pos < wl_cand0) st_i32<true>(wl + wl_pos, j + lo);  // always true for consistent counts
            ++wl_pos;
          }
        }
        left = inside[w] & ok;
#pragma unroll 1
        while (__builtin_expect(left != 0, 0)) {  // rare even per wave
          const int i = __builtin_ctz(left) + 32 * w;
          const int j = i * NT + tid;
          left &= left - 1;
          if (list_cands) {
            const uint32_t rel = pick_reg<R>(key, i);
            const uint32_t slot = append_slot(&sh.cand_n);
            sh.cand_key[slot] = rel;
            sh.cand_idx[slot] = (uint32_t)j;
          } else {
            atomicOr(&bm_eq[j >> 5], 1u << (j & 31));
          }
        }
      }
    } else {
#pragma unroll 1
      for (int i = 0; i < ntiles; ++i) {
        const int j = i * NT + tid;
        const uint32_t rel = rel_at(i);
        const uint32_t dg = rel >> shift;
        if (dg >= d1 && j < N) {  // the digit test comes first: it fails for almost every key
          if (dg > d1) {
            atomicOr(&bm_gt[j >> 5], 1u << (j & 31));
          } else if (list_cands) {
            const uint32_t slot = append_slot(&sh.cand_n);
            sh.cand_key[slot] = rel;
            sh.cand_idx[slot] = (uint32_t)j;
          } else {
            atomicOr(&bm_eq[j >> 5], 1u << (j & 31));
          }
        }
      }
    }
    __syncthreads();
    if (list_cands) {
      // A long candidate list (a range stretched by a few outliers packs the bulk of the keys into
      // few bins) is cut down by further digits of the key, a histogram round per digit over the
      // list alone: candidates above the new threshold bin are selected, those inside it form the
      // next list.  Each thread carries its candidates through a round in registers.
      constexpr int CPT = (TOPK_MAX_CAND + NT - 1) / NT;
      uint32_t cshift = (uint32_t)shift;  // bits of the key not yet looked at
      while (ncand > (uint32_t)TOPK_RANK_MAX && cshift > 0) {
        const uint32_t nshift = cshift > TOPK_DIGIT_BITS ? cshift - TOPK_DIGIT_BITS : 0;
        uint32_t ck[CPT], ci[CPT];
#pragma unroll
        for (int i = 0; i < CPT; ++i) {
          const uint32_t c = (uint32_t)(i * NT + tid);
          ck[i] = c < ncand ? sh.cand_key[c] : 0u;
          ci[i] = c < ncand ? sh.cand_idx[c] : 0u;
        }
#pragma unroll
        for (int i = tid; i < TOPK_BINS; i += NT) sh.hist[i] = 0;
        if (tid == 0) sh.cand_n = 0;
        __syncthreads();
#pragma unroll
        for (int i = 0; i < CPT; ++i)
          if ((uint32_t)(i * NT + tid) < ncand) atomicAdd(&sh.hist[(ck[i] >> nshift) & (uint32_t)(TOPK_BINS - 1)], 1u);
        __syncthreads();
        pick_bin<NT>(sh, tid, lane, wave, need);
        const uint32_t d2 = sh.bcast[0], above2 = sh.bcast[1], inbin2 = sh.bcast[2];
#pragma unroll
        for (int i = 0; i < CPT; ++i) {
          if ((uint32_t)(i * NT + tid) < ncand) {
            const uint32_t dg = (ck[i] >> nshift) & (uint32_t)(TOPK_BINS - 1);
            if (dg > d2) {
              atomicOr(&bm_gt[ci[i] >> 5], 1u << (ci[i] & 31));
            } else if (dg == d2) {
              const uint32_t slot = append_slot(&sh.cand_n);
              sh.cand_key[slot] = ck[i];
              sh.cand_idx[slot] = ci[i];
            }
          }
        }
        __syncthreads();  // the new list is complete; bcast may be rewritten
        need -= above2;
        ncand = inbin2;
        cshift = nshift;
      }
      if (ncand <= (uint32_t)TOPK_RANK_MAX) {
        // a short list: exact rank of every candidate by (key desc, index asc)
#pragma unroll 1
        for (uint32_t c = (uint32_t)tid; c < ncand; c += NT) {
          const uint32_t mk = sh.cand_key[c], mi = sh.cand_idx[c];
          uint32_t rank = 0;
#pragma unroll 4
          for (uint32_t u = 0; u < ncand; ++u) {
            const uint32_t ok = sh.cand_key[u], oi = sh.cand_idx[u];
            rank += (ok > mk) || (ok == mk && oi < mi);
          }
          if (rank < need) {
            if (use_bm) atomicOr(&bm_gt[mi >> 5], 1u << (mi & 31));
            if (direct) st_i32<true>(wl + wl_cand0 + rank, (int)mi + lo);
          }
        }
      } else {
        // every digit used up: the candidates share one key value and tie, lowest index first
#pragma unroll 1
        for (uint32_t c = (uint32_t)tid; c < ncand; c += NT) {
          const uint32_t mi = sh.cand_idx[c];
          atomicOr(&bm_eq[mi >> 5], 1u << (mi & 31));
        }
        need_eq = need;
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
#pragma unroll
      for (int i = tid; i < TOPK_BINS; i += NT) sh.hist[i] = 0;
      __syncthreads();
#pragma unroll 1
      for (int j = tid; j < N; j += NT) {
        const uint32_t rel = ordered_key(ld_i32<COH>(sc + j)) - kmin;
        if ((rel & mask) == prefix) atomicAdd(&sh.hist[(rel >> shift) & (uint32_t)(TOPK_BINS - 1)], 1u);
      }
      __syncthreads();
      pick_bin<NT>(sh, tid, lane, wave, need);
      prefix |= sh.bcast[0] << shift;
      mask |= (uint32_t)(TOPK_BINS - 1) << shift;
      need -= sh.bcast[1];
      __syncthreads();  // bcast is rewritten by the next round
    }
    const uint32_t tau = prefix;
    need_eq = need;
#pragma unroll 1
    for (int j = tid; j < N; j += NT) {
      const uint32_t rel = ordered_key(ld_i32<COH>(sc + j)) - kmin;
      if (rel > tau)
        atomicOr(&bm_gt[j >> 5], 1u << (j & 31));
      else if (rel == tau)
        atomicOr(&bm_eq[j >> 5], 1u << (j & 31));
    }
    __syncthreads();
  }
  if (direct) {
    publish();
    if (!out) return;
  }
  // ---- 4. bitmaps -> ascending index list, in one round: every thread owns a run of consecutive
  // bitmap words, counts their bits, one scan over the work-group places the run, and the thread
  // writes its blocks out in order
  const int wpt = (nwords + NT - 1) / NT;  // words per thread
  const int wa = min(tid * wpt, nwords), wb = min(wa + wpt, nwords);
  uint32_t cnt_gt = 0, cnt_eq = 0;
#pragma unroll 1
  for (int w = wa; w < wb; ++w) {
    cnt_gt += (uint32_t)__popc(bm_gt[w]);
    if (need_eq > 0) cnt_eq += (uint32_t)__popc(bm_eq[w]);
  }
  uint32_t tot_gt, tot_eq;
  uint32_t G = block_excl_scan<NT>(cnt_gt, sh.wave_a, lane, wave, &tot_gt);
  uint32_t E = 0;
  if (need_eq > 0) E = block_excl_scan<NT>(cnt_eq, sh.wave_b, lane, wave, &tot_eq);
#pragma unroll 1
  for (int w = wa; w < wb; ++w) {
    const uint32_t g = bm_gt[w];
    const uint32_t e = need_eq > 0 ? bm_eq[w] : 0u;
    uint32_t bitsleft = g | e;
#pragma unroll 1
    while (bitsleft) {
      const int bpos = __builtin_ctz(bitsleft);
      bitsleft &= bitsleft - 1;
      const int idx = (w << 5) + bpos;
      if ((g >> bpos) & 1u) {
        const uint32_t slot = G + min(E, need_eq);
        if (slot < (uint32_t)K) put(lo + (int)slot, idx + lo);  // always true for consistent counts; keeps stores in bounds
        ++G;
      } else {
        if (E < need_eq) {
          const uint32_t slot = G + E;
          if (slot < (uint32_t)K) put(lo + (int)slot, idx + lo);
        }
        ++E;
      }
    }
  }
  if (EARLY && !direct) publish();
}

}  // namespace absb
