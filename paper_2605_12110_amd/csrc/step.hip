// The whole decode step (score -> select -> attention over the selection, Sec. 3.4 kernels 1-3)
// in ONE launch, with the selection spread over the work-groups that score and attend.
//
// At batch 1 the step moves ~20 MB, a few microseconds of HBM time: what it costs is the chain of
// dependent hand-overs between its stages, and a selection that runs on one compute unit per
// segment.  Here a segment (one request, one KV head) is cut into `units` of consecutive blocks,
// and one work-group per unit does everything for its blocks:
//
//   1. it scores them (score_dev.h), keeps the scores in LDS, and counts them into a 256-bin
//      histogram over the range the scores can take at all, which follows from the query's
//      fixed-point weights alone (every 4-bit code lies in [0, 15]) and is therefore the same in
//      every unit before any code has been read; the histogram row (16-bit counts) goes to device
//      memory and the unit signs in on the segment's arrival counter;
//   2. once all units of the segment have signed in, EVERY unit reads all rows (a few KB), adds them
//      up and finds the bin d1 that holds the K_s-th largest score: all units reach the same verdict
//      without anybody having to tell them;
//   3. a unit classifies its own blocks: above the bin = selected, inside the bin = candidate.  It
//      publishes its candidates (score, index) and attends over its selected blocks right away
//      (decode_dev.h; the block list never leaves LDS, the page-table entries of its token range were
//      fetched while it waited);
//   4. then it requests its candidates' rows, and while they fly it reads the segment's candidates
//      (from the rows it knows how many every unit holds) and ranks its OWN ones exactly against
//      them (score descending, index ascending): those among the best `need` count, the others'
//      rows are dropped; a second stretch of the same online softmax;
//   5. every unit writes a split-K partial; the one that draws the segment's last ticket merges
//      (as in the stand-alone attention kernel).
// Between scores and attention there is one hand-over, and no pass over a whole segment by one
// work-group.  The selected SET is exactly that of absb_score + absb_topk (same integer scores, same
// total order); the order in which tokens enter the softmax differs, so outputs agree within
// rounding, not bit for bit.
//
// Each segment also has a COORDINATOR work-group for what is not on the way to the output: the
// ascending index list (sel_idx_out), which only the caller needs (when asked for, units publish
// their words of a selection bitmap and the coordinator turns it into the list while the partials
// are being merged), and the crowded threshold bin (more than STEP_MAX_CAND candidates: e.g. all
// scores equal), where it runs the exact selection of topk_dev.h on the segment's scores itself,
// writes the list to device memory and raises the segment's flag; the units, which see the crowded
// bin too, wait for that flag and split the list's positions among themselves as the stand-alone
// attention kernel does.  Budgets that cover the context, or forced blocks that fill the list, need
// no scores at all: every unit knows its blocks' fate from the shapes.
//
// Progress.  A segment's work-groups are consecutive in the grid: coordinator first, then its units.
// Units wait for the other units of their segment (and for the coordinator on a crowded bin), the
// coordinator waits for its units.  With work-groups started in index order and more resident
// work-groups than a segment has (at most ABSB_STEP_MAX_UNITS + 1; the chip holds 256 even at one
// per compute unit), the earliest unfinished segment always has all its work-groups running, so it
// finishes and frees its slots.  Every wait is also bounded in time: a work-group whose wait runs
// out sets the status word, writes NaN into its segment's output rows and leaves, so the grid drains
// whatever happens.
//
// Counters and flags (256 bytes apart, at the start of the workspace) must be zero when the launch
// starts and are zero again when it ends.
//
// Compiled with -ffp-contract=off, as the estimation stage requires.
#include "decode_dev.h"
#include "score_dev.h"
#include "topk_dev.h"

namespace absb {

constexpr int STEP_THREADS = DEC_THREADS;
constexpr int STEP_LOG2_BINS = 8;
constexpr int STEP_BINS = 1 << STEP_LOG2_BINS;   // histogram bins over the scores' possible range
constexpr int STEP_MAX_CAND = 512;               // candidates of a segment that units rank against
constexpr int STEP_MAX_UNIT_BLOCKS = 2048;       // blocks per unit: 2^17 blocks / 64 units
constexpr int STEP_PT_CACHE = 512;               // page-table entries a unit keeps in LDS
constexpr int STEP_SCORE_BATCH = 8;              // 512 blocks' codes requested at once
constexpr int32_t LIST_READY = 1;

struct StepParams {
  ScoreParams sc;
  TopkParams tk;   // scores, list and counts in device memory (the crowded-bin path and the list output)
  DecodeParams dc;
  // hand-over words, one per selection segment, ABSB_TICKET_STRIDE words apart
  int32_t* arrive;     // units whose scores and histogram row are out (read by the units)
  int32_t* arrive_c;   // the same count, for the coordinator (each reader clears its own)
  int32_t* cand_done;  // candidates that are out
  int32_t* listed;     // units whose words of the selection bitmap are out
  int32_t* list_flag;  // crowded bin: the coordinator's list is in device memory
  uint16_t* rows;      // [nseg][units_max][STEP_BINS]
  uint2* cand;         // (score - lowest possible score, block index); a unit's pairs start at its first score's place
  uint32_t* bitmap;    // [nseg][bitmap_words]
  int32_t units_max, unit_tokens, bitmap_words, want_list;
};

// LDS of a unit, behind the attention kernel's: what has to survive the attention loop
constexpr int STEP_LDS_LIST = DEC_LDS_BYTES;                                 // int32 [STEP_MAX_UNIT_BLOCKS]
constexpr int STEP_LDS_CAND_J = STEP_LDS_LIST + STEP_MAX_UNIT_BLOCKS * 4;    // int32 [STEP_MAX_CAND] own candidates: block
constexpr int STEP_LDS_CAND_KEY = STEP_LDS_CAND_J + STEP_MAX_CAND * 4;       // uint32 [STEP_MAX_CAND] ... and score
constexpr int STEP_LDS_PT = STEP_LDS_CAND_KEY + STEP_MAX_CAND * 4;           // int32 [STEP_PT_CACHE]
constexpr int STEP_LDS_CPRE = STEP_LDS_PT + STEP_PT_CACHE * 4;               // int32 [MAX_UNITS + 1] candidates before unit c
constexpr int STEP_LDS_MISC = STEP_LDS_CPRE + (ABSB_STEP_MAX_UNITS + 4) * 4; // 64 words of scan / broadcast scratch
constexpr int STEP_LDS_UNIT = STEP_LDS_MISC + 64 * 4;
// ... and what only lives until the attention loop starts
constexpr int STEP_LDS_SCORE = 3072;                                         // int32 [STEP_MAX_UNIT_BLOCKS], behind the estimation's
constexpr int STEP_LDS_HIST = STEP_LDS_SCORE + STEP_MAX_UNIT_BLOCKS * 4;     // uint32 [STEP_BINS]
constexpr int STEP_LDS_ROWS = STEP_LDS_HIST + STEP_BINS * 4;                 // uint16 [MAX_UNITS][STEP_BINS]: up to the page table
static_assert(score_lds_bytes<0>() <= STEP_LDS_SCORE && score_lds_bytes<1>() <= STEP_LDS_SCORE, "estimation LDS");
static_assert(STEP_LDS_ROWS + ABSB_STEP_MAX_UNITS * STEP_BINS * 2 <= STEP_LDS_PT, "rows end before the page-table copy");
static_assert(STEP_BINS == STEP_THREADS, "a work-group's threads own one bin each");
// ... and after the first attention stretch: the segment's candidates and the ranks of the unit's own
constexpr int STEP_LDS_ALL_KEY = 0;                                          // uint32 [STEP_MAX_CAND]
constexpr int STEP_LDS_ALL_IDX = STEP_LDS_ALL_KEY + STEP_MAX_CAND * 4;
constexpr int STEP_LDS_RANK = STEP_LDS_ALL_IDX + STEP_MAX_CAND * 4;          // uint32 [STEP_MAX_CAND]
// (these three share their bytes with the waves' staging areas: they are used strictly between two
// stretches of the attention loop, while the second stretch's first rows are still on their way to
// registers, with barriers on both sides)

__host__ __device__ constexpr size_t step_max_sz(size_t a, size_t b) { return a > b ? a : b; }

// Shape of a selection segment as every one of its work-groups derives it.
struct SegShape {
  SegMap sm;
  int lb, off, rows;
  int Nall, K;       // blocks in use, blocks to select
  int lo, hi;        // forced blocks are [0, lo) and [hi, Nall); [lo, hi) compete
  int nforced;
  int units, unit_blocks;
};

__device__ __forceinline__ SegShape seg_shape(const StepParams& p, int t) {
  SegShape g;
  g.sm = seg_map(t, p.tk.Hsel, p.tk.Rk, p.tk.Hkv);
  g.off = p.tk.cent_off[g.sm.s];
  g.rows = p.tk.cent_off[g.sm.s + 1] - g.off;
  g.lb = p.tk.heads.log2_block[g.sm.hk];
  g.Nall = blocks_in_use(p.tk.tight, g.rows, p.tk.seq_lens, g.sm.b, g.lb);
  g.K = budget_blocks(p.tk.budget[g.sm.b], g.lb, g.Nall, p.tk.sel_stride);
  g.lo = 0;
  g.hi = g.Nall;
  if (p.tk.sink_tokens > 0) g.lo = min(g.Nall, (int)(((int64_t)p.tk.sink_tokens + (1 << g.lb) - 1) >> g.lb));
  if (p.tk.recent_tokens > 0)
    g.hi = max(g.lo, min(g.Nall, max(0, p.tk.seq_lens[g.sm.b] - p.tk.recent_tokens) >> g.lb));
  g.nforced = g.lo + (g.Nall - g.hi);
  step_units(g.K, g.lb, g.Nall, p.unit_tokens, &g.units, &g.unit_blocks);
  return g;
}

// Waits (thread 0, bounded in time) until the counter at `ctr` reads `target`.  Every thread returns
// 1, or 0 when the wait ran into its limit (*status is then set).  Barriers inside.
__device__ __forceinline__ int wait_for_count(const int32_t* ctr, int target, int32_t* status, int* s_word) {
  if (threadIdx.x == 0) {
    int v = ld_i32<true>(ctr);
    if (v != target) {
      const uint64_t t0 = wall_clock64();
      do {
        __builtin_amdgcn_s_sleep(2);
        v = ld_i32<true>(ctr);
      } while (v != target && wall_clock64() - t0 < DEC_WAIT_LIMIT_TICKS);
    }
    if (v != target) st_i32<true>(status, 1);
    *s_word = v == target;
  }
  __syncthreads();
  const int ok = *s_word;
  __syncthreads();
  return ok;
}

// Ascending index list of the set bits of an LDS bitmap of `nwords` words: every thread owns a run of
// consecutive words, one scan over the work-group places the runs.  Writes at most `K` entries.
__device__ __forceinline__ void emit_bitmap_list(const uint32_t* bm, int nwords, int32_t* out, int K, uint32_t* slot) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wpt = (nwords + STEP_THREADS - 1) / STEP_THREADS;
  const int wa = min(tid * wpt, nwords), wb = min(wa + wpt, nwords);
  uint32_t cnt = 0;
#pragma unroll 1
  for (int w = wa; w < wb; ++w) cnt += (uint32_t)__popc(bm[w]);
  uint32_t total;
  uint32_t at = block_excl_scan<STEP_THREADS>(cnt, slot, lane, wave, &total);
#pragma unroll 1
  for (int w = wa; w < wb; ++w) {
    uint32_t left = bm[w];
#pragma unroll 1
    while (left) {
      const int bpos = __builtin_ctz(left);
      left &= left - 1;
      if (at < (uint32_t)K) st_i32<false>(out + at, (w << 5) + bpos);
      ++at;
    }
  }
}

// What the histogram rows of a segment's units say: the bin d1 that holds the Kc-th largest
// competing score, how many of its members are still needed, how many it has.
struct Verdict {
  int d1, need, n_in;
  __device__ __forceinline__ bool whole() const { return need == n_in; }                       // the bin is admitted as it is
  __device__ __forceinline__ bool crowded() const { return n_in > STEP_MAX_CAND && need < n_in; }
};

// Loads the U rows of segment t into LDS at `s_rows`, adds them up and locates the threshold bin.
// Every thread of the work-group must call; all get the same result.  `s_misc`: 32 words.
__device__ __forceinline__ Verdict read_verdict(const StepParams& p, int t, int U, int Kc, char* lds_rows, uint32_t* s_misc) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  uint16_t (*s_rows)[STEP_BINS] = reinterpret_cast<uint16_t (*)[STEP_BINS]>(lds_rows);
  {
    const uint4* src = reinterpret_cast<const uint4*>(p.rows + (size_t)t * p.units_max * STEP_BINS);
    const int nvec = U * (STEP_BINS * 2 / 16);  // 16-byte pieces
    constexpr int VPT = ABSB_STEP_MAX_UNITS * (STEP_BINS * 2 / 16) / STEP_THREADS;
    u32x4 v[VPT];
    const __amdgpu_buffer_rsrc_t rsrc =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<uint4*>(src), 0, nvec * 16, 0x00020000);
#pragma unroll
    for (int k = 0; k < VPT; ++k)  // pieces past the last row read as zero (buffer bounds) and cost no traffic
      v[k] = __builtin_amdgcn_raw_buffer_load_b128(rsrc, (k * STEP_THREADS + tid) * 16, 0, 16 /* sc1 */);
#pragma unroll
    for (int k = 0; k < VPT; ++k)
      if (k * STEP_THREADS + tid < nvec) reinterpret_cast<u32x4*>(lds_rows)[k * STEP_THREADS + tid] = v[k];
  }
  if (tid == 0) s_misc[17] = s_misc[18] = s_misc[19] = 0;
  __syncthreads();
  // thread tid owns bin STEP_BINS - 1 - tid: an exclusive scan in thread order counts the scores above
  const int bin = STEP_BINS - 1 - tid;
  uint32_t cnt = 0;
#pragma unroll 4
  for (int c = 0; c < U; ++c) cnt += s_rows[c][bin];
  uint32_t total;
  const uint32_t above = block_excl_scan<STEP_THREADS>(cnt, s_misc, lane, wave, &total);
  if (above < (uint32_t)Kc && (uint32_t)Kc <= above + cnt) {
    s_misc[17] = (uint32_t)bin;
    s_misc[18] = above;
    s_misc[19] = cnt;
  }
  __syncthreads();
  Verdict v;
  v.d1 = (int)s_misc[17];
  v.need = Kc - (int)s_misc[18];
  v.n_in = (int)s_misc[19];
  return v;
}

// Attention of this wave over positions [pos_begin, pos_end) of the virtual token sequence of the
// unit's block list in LDS, folded into `st`: the loop of attend_positions (decode_dev.h) with the
// rows of TWO steps in flight.  A unit that got more than its share of the selection works through
// several steps of 64 positions; at batch 1 every step waits a full trip to cold memory for its rows,
// and with list and page-table entries in LDS nothing keeps the step after next from being requested
// as well.  `after_first_issue` and `live` as in attend_positions.
struct StepRows {
  u32x4 k0, k1, k2, k3, v0, v1, v2, v3;
  uint32_t valid;
};
template <int DT, int G, class Hook, class Live>
__device__ __forceinline__ void attend_local(const DecodeParams& p, const SplitCtx& c, const int32_t* s_list, int last_entry,
                                             const PageRef& pages, int pos_begin, int pos_end, const uint2 (&qb)[8],
                                             AttnState& st, Hook&& after_first_issue, Live&& live) {
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, grp = lane >> 4, li = lane & 15;
  const int lb = c.lb, L = c.L, lP = c.lP;
  char* kt = c.kt;
  char* vt = c.vt;
  constexpr int STEP = DEC_WAVES * ROWS_PER_WAVE_STEP;
  auto issue = [&](int base, StepRows& r) __attribute__((always_inline)) {
    // the lane's four rows: consecutive positions from a multiple of four, in one block and one page
    const int pos = base + grp * 4;
    const int sj = s_list[min(pos >> lb, last_entry)];
    const int t = (sj << lb) + (pos & ((1 << lb) - 1));
    uint32_t vb = 0;
#pragma unroll
    for (int i = 0; i < 4; ++i) vb |= (uint32_t)(pos + i < pos_end && t + i < L) << i;  // a selected last block may be partial
    const int tcb = max(0, min(t, L - 1)) & ~3;
    const int pg = pages.at(tcb >> lP);
    const size_t row0 = (size_t)pg * p.g.s_page + c.lane_off;
    const size_t off0 = row0 + (size_t)(min(tcb + 0, L - 1) & ((1 << lP) - 1)) * p.g.s_tok;
    const size_t off1 = row0 + (size_t)(min(tcb + 1, L - 1) & ((1 << lP) - 1)) * p.g.s_tok;
    const size_t off2 = row0 + (size_t)(min(tcb + 2, L - 1) & ((1 << lP) - 1)) * p.g.s_tok;
    const size_t off3 = row0 + (size_t)(min(tcb + 3, L - 1) & ((1 << lP) - 1)) * p.g.s_tok;
    r.valid = vb;
    r.k0 = *reinterpret_cast<const u32x4*>(p.k + off0);
    r.k1 = *reinterpret_cast<const u32x4*>(p.k + off1);
    r.k2 = *reinterpret_cast<const u32x4*>(p.k + off2);
    r.k3 = *reinterpret_cast<const u32x4*>(p.k + off3);
    r.v0 = *reinterpret_cast<const u32x4*>(p.v + off0);
    r.v1 = *reinterpret_cast<const u32x4*>(p.v + off1);
    r.v2 = *reinterpret_cast<const u32x4*>(p.v + off2);
    r.v3 = *reinterpret_cast<const u32x4*>(p.v + off3);
  };
  float m = st.m, l = st.l, lx = st.lx;
  // one step: the rows in `r` go to LDS, `r` is refilled with the rows of the step after next, then
  // S = K Q^T, the online softmax and O += P V from LDS
  auto step = [&](int base, StepRows& r) __attribute__((always_inline)) {
    const uint32_t valid = live((base + grp * 4) >> lb) ? r.valid : 0u;
    *reinterpret_cast<u32x4*>(kt + (grp * 4 + 0) * K_PITCH + li * 16) = r.k0;
    *reinterpret_cast<u32x4*>(kt + (grp * 4 + 1) * K_PITCH + li * 16) = r.k1;
    *reinterpret_cast<u32x4*>(kt + (grp * 4 + 2) * K_PITCH + li * 16) = r.k2;
    *reinterpret_cast<u32x4*>(kt + (grp * 4 + 3) * K_PITCH + li * 16) = r.k3;
    stage_v_word(vt + 0 * 1024 + li * 32 + grp * 8, r.v0.x, r.v1.x, r.v2.x, r.v3.x);
    stage_v_word(vt + 1 * 1024 + li * 32 + grp * 8, r.v0.y, r.v1.y, r.v2.y, r.v3.y);
    stage_v_word(vt + 2 * 1024 + li * 32 + grp * 8, r.v0.z, r.v1.z, r.v2.z, r.v3.z);
    stage_v_word(vt + 3 * 1024 + li * 32 + grp * 8, r.v0.w, r.v1.w, r.v2.w, r.v3.w);
    if (base + 2 * STEP < pos_end) issue(base + 2 * STEP, r);
    float4_t s0 = {0.0f, 0.0f, 0.0f, 0.0f}, s1 = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
    for (int ks = 0; ks < 8; ks += 2) {
      const uint2 a0 = *reinterpret_cast<const uint2*>(kt + li * K_PITCH + (16 * ks + 4 * grp) * 2);
      const uint2 a1 = *reinterpret_cast<const uint2*>(kt + li * K_PITCH + (16 * (ks + 1) + 4 * grp) * 2);
      s0 = mma16<DT>(a0, qb[ks], s0);
      s1 = mma16<DT>(a1, qb[ks + 1], s1);
    }
    float sc[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) sc[i] = ((valid >> i) & 1u) ? (s0[i] + s1[i]) * p.scale_log2 : -__builtin_inff();
    float mx = fmaxf(fmaxf(sc[0], sc[1]), fmaxf(sc[2], sc[3]));
    mx = fmaxf(mx, __shfl_xor(mx, 16));
    mx = fmaxf(mx, __shfl_xor(mx, 32));
    const float mn = fmaxf(m, mx);
    const float alpha = fast_exp2(m - mn);
    m = mn;
    uint32_t pb[4];
    float psum = 0.0f, esum = 0.0f;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const float e = fast_exp2(sc[i] - mn);
      const uint16_t ph = Elem<DT>::narrow(e);  // the weight as the product will see it
      psum += Elem<DT>::widen(ph);
      esum += e;
      pb[i] = ph;
    }
    l = __builtin_fmaf(l, alpha, psum);
    lx = __builtin_fmaf(lx, alpha, esum);
    const uint2 pa = make_uint2(pb[0] | (pb[1] << 16), pb[2] | (pb[3] << 16));
    if (__any(alpha != 1.0f)) {  // rescale O when some head's maximum moved
      float ah[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const float a_lo = bitcast<float>(__builtin_amdgcn_readlane(bitcast<int>(alpha), i));
        const float a_hi = bitcast<float>(__builtin_amdgcn_readlane(bitcast<int>(alpha), (G > 4 ? 4 + i : i)));
        ah[i] = (G > 4 && grp == 1) ? a_hi : a_lo;
      }
#pragma unroll
      for (int j = 0; j < 8; ++j) {
#pragma unroll
        for (int i = 0; i < 4; ++i) st.oacc[j][i] *= ah[i];
      }
    }
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const uint2 bv = *reinterpret_cast<const uint2*>(vt + j * 512 + li * 32 + grp * 8);
      st.oacc[j] = mma16<DT>(pa, bv, st.oacc[j]);
    }
  };
  int base = pos_begin + wave * ROWS_PER_WAVE_STEP;
  StepRows ra, rb;
  ra.valid = rb.valid = 0;
  if (base < pos_end) issue(base, ra);
  if (base + STEP < pos_end) issue(base + STEP, rb);
  after_first_issue();
  while (base < pos_end) {  // trip count depends on the wave only: every branch here is wave-uniform
    step(base, ra);
    base += STEP;
    if (base >= pos_end) break;
    step(base, rb);
    base += STEP;
  }
  st.m = m;
  st.l = l;
  st.lx = lx;
}

// ------------------------------------------------------------------ coordinator
template <int DT, int G>
__device__ __forceinline__ void step_coordinator(const StepParams& p, int t, char* lds) {
  const SegShape g = seg_shape(p, t);
  const int tid = threadIdx.x;
  const bool compete = g.K < g.Nall && g.nforced < g.K;
  TopkShared& sh = *reinterpret_cast<TopkShared*>(lds);
  uint32_t* sel_bitmap = reinterpret_cast<uint32_t*>(lds + ((sizeof(TopkShared) + 15) & ~size_t(15)));
  if (!compete) {
    // no score decides anything: the exact selection's early exits write the list and the count
    if (p.want_list) topk_segment<STEP_THREADS, 0, true>(p.tk, t, sh, sel_bitmap);
    return;
  }
  uint32_t* s_misc = reinterpret_cast<uint32_t*>(lds + STEP_LDS_MISC);  // [0,16) scan slots, 16.. broadcast
  int32_t* arrive_c = p.arrive_c + (size_t)t * ABSB_TICKET_STRIDE;
  int32_t* listed = p.listed + (size_t)t * ABSB_TICKET_STRIDE;
  const int U = g.units;

  // ---- all units have scored: is the threshold bin crowded?
  if (!wait_for_count(arrive_c, U, p.dc.status, reinterpret_cast<int*>(s_misc + 16))) return;
  if (tid == 0) st_i32<true>(arrive_c, 0);
  const Verdict v = read_verdict(p, t, U, g.K - g.nforced, lds + STEP_LDS_ROWS, s_misc);
  if (v.crowded()) {
    // the exact selection over the segment's scores, by this work-group alone; the units wait for it
    __syncthreads();
    topk_segment<STEP_THREADS, 0, true>(p.tk, t, sh, sel_bitmap);
    wait_stores_acknowledged();
    __syncthreads();
    if (tid == 0) st_i32<true>(p.list_flag + (size_t)t * ABSB_TICKET_STRIDE, LIST_READY);
    return;
  }
  if (p.want_list) {
    // ---- the caller wants the ascending index list: from the units' bitmap words
    if (!wait_for_count(listed, U, p.dc.status, reinterpret_cast<int*>(s_misc + 16))) return;
    if (tid == 0) st_i32<true>(listed, 0);
    const int nwords = (g.Nall + 31) >> 5;
    uint32_t* s_bm = reinterpret_cast<uint32_t*>(lds);
    const uint32_t* bm = p.bitmap + (size_t)t * p.bitmap_words;
#pragma unroll 1
    for (int w = tid; w < nwords; w += STEP_THREADS) s_bm[w] = (uint32_t)ld_i32<true>(reinterpret_cast<const int32_t*>(bm + w));
    int32_t* out = p.tk.sel_idx + (size_t)t * p.tk.sel_stride;
    if (tid == 0) p.tk.sel_cnt[t] = g.K;
#pragma unroll 1
    for (int i = g.K + tid; i < p.tk.sel_stride; i += STEP_THREADS) out[i] = -1;
    __syncthreads();
    emit_bitmap_list(s_bm, nwords, out, g.K, s_misc + 32);
  }
}

// ------------------------------------------------------------------ unit
template <int DT, int G, int REP>
__device__ __forceinline__ void step_unit(const StepParams& p, int t, int c, char* lds) {
  const SegShape g = seg_shape(p, t);
  if (c >= g.units) return;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, grp = lane >> 4, li = lane & 15;
  const int b = g.sm.b, hs = g.sm.hs, hk = g.sm.hk, lb = g.lb;
  const int U = g.units;
  const int j0 = c * g.unit_blocks, j1 = min(g.Nall, j0 + g.unit_blocks), n = j1 - j0;
  const bool compete = g.K < g.Nall && g.nforced < g.K;

  int32_t* s_list = reinterpret_cast<int32_t*>(lds + STEP_LDS_LIST);
  int32_t* s_cand_j = reinterpret_cast<int32_t*>(lds + STEP_LDS_CAND_J);
  uint32_t* s_cand_key = reinterpret_cast<uint32_t*>(lds + STEP_LDS_CAND_KEY);
  int32_t* s_pt = reinterpret_cast<int32_t*>(lds + STEP_LDS_PT);
  int32_t* s_cpre = reinterpret_cast<int32_t*>(lds + STEP_LDS_CPRE);
  uint32_t* s_misc = reinterpret_cast<uint32_t*>(lds + STEP_LDS_MISC);  // [0,16) and [16,32) scan slots, 32.. broadcast
  int32_t* s_score = reinterpret_cast<int32_t*>(lds + STEP_LDS_SCORE);
  uint32_t* s_hist = reinterpret_cast<uint32_t*>(lds + STEP_LDS_HIST);
  int32_t* arrive = p.arrive + (size_t)t * ABSB_TICKET_STRIDE;
  int32_t* cand_done = p.cand_done + (size_t)t * ABSB_TICKET_STRIDE;
  int32_t* list_flag = p.list_flag + (size_t)t * ABSB_TICKET_STRIDE;

  // ---- what the attention needs and no stage produces: context length, the page-table entries of
  // the unit's token range (they land while the unit scores and waits), the queries
  SplitCtx cx;
  cx.b = b;
  cx.hs = hs;
  cx.hk = hk;
  cx.lb = lb;
  cx.L = p.dc.seq_lens[b];
  cx.lP = p.dc.g.log2_page;
  cx.lane_off = (size_t)hk * p.dc.g.s_head + (size_t)li * 8;
  cx.kt = lds + wave * STAGE_BYTES;
  cx.vt = cx.kt + K_TILE_BYTES;
  const int32_t* pt_row = p.dc.page_table + (size_t)b * p.dc.g.pt_stride;
  const int tok0 = j0 << lb, tok1 = min(cx.L, j1 << lb);
  const int page0 = tok0 >> cx.lP, npages = ((max(tok1, tok0 + 1) - 1) >> cx.lP) - page0 + 1;
  const bool pt_cached = npages <= STEP_PT_CACHE;
  if (pt_cached) {
#pragma unroll 1
    for (int i = tid; i < npages; i += STEP_THREADS) s_pt[i] = pt_row[page0 + i];
  }
  const PageRef pages{pt_row, pt_cached ? (lds_const_i32*)s_pt : (lds_const_i32*)nullptr, page0, npages};
  uint2 qb[8];
  load_q<G>(p.dc, b, hs, qb);

  int nsure = 0, ncand = 0;
  Verdict v = {0, 0, 0};
  bool list_mode = false;
  if (!compete) {
    // ---- every block's fate follows from the shapes: all selected, or the first K forced ones
    uint32_t mine = 0;
    const int per = (n + STEP_THREADS - 1) / STEP_THREADS;
    const int ia = min(tid * per, n), ib = min(ia + per, n);
    for (int i = ia; i < ib; ++i) {
      const int j = j0 + i;
      mine += (g.K >= g.Nall) || (j < g.lo ? j < g.K : (j >= g.hi && g.lo + (j - g.hi) < g.K));
    }
    uint32_t total;
    uint32_t at = block_excl_scan<STEP_THREADS>(mine, s_misc, lane, wave, &total);
    for (int i = ia; i < ib; ++i) {
      const int j = j0 + i;
      if ((g.K >= g.Nall) || (j < g.lo ? j < g.K : (j >= g.hi && g.lo + (j - g.hi) < g.K))) s_list[at++] = j;
    }
    nsure = (int)total;
    __syncthreads();
  } else {
    // ---- 1. scores of the unit's blocks: to LDS, and to device memory for the crowded-bin path
#pragma unroll
    for (int i = tid; i < STEP_BINS; i += STEP_THREADS) s_hist[i] = 0;
    int32_t* scores_t = p.sc.scores + score_base(g.sm, p.sc.Rk, g.off, g.rows);
    ScoreRange rng;
    score_blocks<DT, REP, true, STEP_SCORE_BATCH>(
        p.sc, t, j0, n, lds,
        [&](int j, int32_t sc) __attribute__((always_inline)) {
          s_score[j - j0] = sc;
          st_i32<true>(scores_t + j, sc);
        },
        &rng);
    const uint32_t rel0 = (uint32_t)rng.lo;
    const uint32_t span = (uint32_t)rng.hi - (uint32_t)rng.lo;
    const int bits = 32 - __builtin_clz(span | 1u);
    const uint32_t shift = bits > STEP_LOG2_BINS ? (uint32_t)(bits - STEP_LOG2_BINS) : 0u;
    __syncthreads();
    // ---- histogram row of the competing blocks
#pragma unroll 1
    for (int i = tid; i < n; i += STEP_THREADS) {
      const int j = j0 + i;
      if (j >= g.lo && j < g.hi) atomicAdd(&s_hist[((uint32_t)s_score[i] - rel0) >> shift], 1u);
    }
    __syncthreads();
    if (tid < STEP_BINS / 8) {
      u32x4 w;
      w.x = s_hist[8 * tid + 0] | (s_hist[8 * tid + 1] << 16);
      w.y = s_hist[8 * tid + 2] | (s_hist[8 * tid + 3] << 16);
      w.z = s_hist[8 * tid + 4] | (s_hist[8 * tid + 5] << 16);
      w.w = s_hist[8 * tid + 6] | (s_hist[8 * tid + 7] << 16);
      uint16_t* row = p.rows + ((size_t)t * p.units_max + c) * STEP_BINS;
      const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(row, 0, STEP_BINS * 2, 0x00020000);
      __builtin_amdgcn_raw_buffer_store_b128(w, rsrc, tid * 16, 0, 16 /* sc1 */);
    }
    wait_stores_acknowledged();
    __syncthreads();
    if (tid == 0) {
      __hip_atomic_fetch_add(arrive, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      __hip_atomic_fetch_add(p.arrive_c + (size_t)t * ABSB_TICKET_STRIDE, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }

    // ---- 2. once every unit has signed in: the verdict, from all rows
    if (!wait_for_count(arrive, U, p.dc.status, reinterpret_cast<int*>(s_misc + 32))) {
      poison_rows<DT, G>(p.dc, b, hs);
      return;
    }
    v = read_verdict(p, t, U, g.K - g.nforced, lds + STEP_LDS_ROWS, s_misc);
    list_mode = v.crowded();
    if (list_mode) {
      if (!wait_for_flag(list_flag, p.dc.status, reinterpret_cast<int*>(s_misc + 32))) {
        poison_rows<DT, G>(p.dc, b, hs);
        return;
      }
    } else {
      // ---- 3. classify: forced and above the bin = selected, inside the bin = candidate
      const uint32_t d1 = (uint32_t)v.d1;
      const bool whole = v.whole();
      if (!whole && tid == 0) {  // where every unit's candidates start among the segment's
        uint16_t (*s_rows)[STEP_BINS] = reinterpret_cast<uint16_t (*)[STEP_BINS]>(lds + STEP_LDS_ROWS);
        int acc = 0;
        for (int u = 0; u < U; ++u) {
          s_cpre[u] = acc;
          acc += s_rows[u][d1];
        }
        s_cpre[U] = acc;
      }
      const int per = (n + STEP_THREADS - 1) / STEP_THREADS;
      const int ia = min(tid * per, n), ib = min(ia + per, n);
      uint32_t my_sure = 0, my_cand = 0;
      for (int i = ia; i < ib; ++i) {
        const int j = j0 + i;
        const bool forced = j < g.lo || j >= g.hi;
        const uint32_t dg = ((uint32_t)s_score[i] - rel0) >> shift;
        my_sure += forced || dg > d1 || (whole && dg == d1);
        my_cand += !forced && !whole && dg == d1;
      }
      uint32_t tot_sure, tot_cand;
      uint32_t at = block_excl_scan<STEP_THREADS>(my_sure, s_misc, lane, wave, &tot_sure);
      uint32_t ct = block_excl_scan<STEP_THREADS>(my_cand, s_misc + 16, lane, wave, &tot_cand);
      nsure = (int)tot_sure;
      ncand = (int)tot_cand;
      // (the rows in LDS reach into the list's bytes: everybody is past reading them now)
      __syncthreads();
      uint64_t* cand_out = reinterpret_cast<uint64_t*>(p.cand) + score_base(g.sm, p.tk.Rk, g.off, g.rows) + j0;
      for (int i = ia; i < ib; ++i) {
        const int j = j0 + i;
        const bool forced = j < g.lo || j >= g.hi;
        const uint32_t rel = (uint32_t)s_score[i] - rel0;
        const uint32_t dg = rel >> shift;
        if (forced || dg > d1 || (whole && dg == d1)) {
          s_list[at++] = j;
        } else if (!whole && dg == d1) {
          // (a unit never holds more candidates than the segment may have in all: STEP_MAX_CAND)
          s_cand_j[ct] = j;
          s_cand_key[ct] = rel;
          s_list[nsure + ct] = j;  // behind the sure blocks: their rows are requested as if all were admitted
          __hip_atomic_store(cand_out + ct, ((uint64_t)(uint32_t)j << 32) | rel, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          ++ct;
        }
      }
      __syncthreads();
    }
  }

  AttnState st;
  st.reset();
  auto clear_words = [&]() __attribute__((always_inline)) {  // by the segment's last unit: every other one is past all its waits
    if (compete) {
      st_i32<true>(arrive, 0);
      st_i32<true>(cand_done, 0);
      st_i32<true>(list_flag, 0);
    }
  };
  if (list_mode) {
    // ---- crowded bin: the list is in device memory; unit c takes the c-th stretch of its positions
    const int ntok = g.K << lb;
    const int stretch = ((ntok + U - 1) / U + 63) & ~63;
    const int pos_begin = c * stretch, pos_end = min(ntok, pos_begin + stretch);
    if (pos_begin < pos_end) {
      const ListRef<LIST_COHERENT> list{p.tk.sel_idx + (size_t)t * p.tk.sel_stride, p.tk.sel_stride - 1};
      const PageRef anywhere{pt_row, nullptr, 0, 0};  // the stretch's tokens lie anywhere in the context
      const int sj = list.at((pos_begin + wave * ROWS_PER_WAVE_STEP + grp * 4) >> lb);
      attend_positions<DT, G, LIST_COHERENT>(p.dc, cx, list, anywhere, pos_begin, pos_end, sj, qb, st);
    }
    finish_split<DT, G>(p.dc, t, b, hs, c, U, p.units_max, st, lds, clear_words);
    return;
  }

  // ---- attention over the unit's selected blocks; the candidates' publication (their stores have
  // to be acknowledged before they are counted) waits behind the first rows, which it has to wait
  // for anyway
  {
    const int pos_end = nsure << lb;
    attend_local<DT, G>(p.dc, cx, s_list, STEP_MAX_UNIT_BLOCKS - 1, pages, 0, pos_end, qb, st, [&]() __attribute__((always_inline)) {
      if (ncand > 0) {  // the same in every wave
        wait_stores_acknowledged();
        __syncthreads();
        if (tid == 0) __hip_atomic_fetch_add(cand_done, ncand, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      }
    }, AllLive());
  }
  int nsel = nsure;
  if (ncand > 0) {
    // ---- 4. the unit's candidates: their rows are requested as if all were admitted; behind those
    // loads the unit reads the segment's candidates and ranks its own among them
    __syncthreads();  // every wave is done with its staging area
    uint32_t* s_all_key = reinterpret_cast<uint32_t*>(lds + STEP_LDS_ALL_KEY);
    uint32_t* s_all_idx = reinterpret_cast<uint32_t*>(lds + STEP_LDS_ALL_IDX);
    uint32_t* s_rank = reinterpret_cast<uint32_t*>(lds + STEP_LDS_RANK);
    bool timed_out = false;
    const int pos_begin = nsure << lb, pos_end = (nsure + ncand) << lb;
    attend_local<DT, G>(
        p.dc, cx, s_list, STEP_MAX_UNIT_BLOCKS - 1, pages, pos_begin, pos_end, qb, st,
        [&]() __attribute__((always_inline)) {
          const int n_in = v.n_in;
          if (!wait_for_count(cand_done, n_in, p.dc.status, reinterpret_cast<int*>(s_misc + 32))) {
            timed_out = true;
            return;
          }
          const uint64_t* cand_t = reinterpret_cast<const uint64_t*>(p.cand) + score_base(g.sm, p.tk.Rk, g.off, g.rows);
#pragma unroll 1
          for (int i = tid; i < n_in; i += STEP_THREADS) {
            int u = 0;  // the unit whose candidates include the i-th: largest u with s_cpre[u] <= i
#pragma unroll
            for (int sb = ABSB_STEP_MAX_UNITS / 2; sb > 0; sb >>= 1)
              if (u + sb < U && s_cpre[u + sb] <= i) u += sb;
            const uint64_t pr = __hip_atomic_load(cand_t + (size_t)u * g.unit_blocks + (i - s_cpre[u]), __ATOMIC_RELAXED,
                                                  __HIP_MEMORY_SCOPE_AGENT);
            s_all_key[i] = (uint32_t)pr;
            s_all_idx[i] = (uint32_t)(pr >> 32);
          }
          for (int i = tid; i < ncand; i += STEP_THREADS) s_rank[i] = 0;
          __syncthreads();
          // rank of own candidate k = how many of the segment's candidates come before it under
          // (score descending, index ascending); pairs spread over the work-group
#pragma unroll 1
          for (int pr = tid; pr < ncand * n_in; pr += STEP_THREADS) {
            const int k = pr / n_in, u = pr - k * n_in;
            const uint32_t mk = s_cand_key[k], mi = (uint32_t)s_cand_j[k];
            const uint32_t ok = s_all_key[u], oi = s_all_idx[u];
            if ((ok > mk) || (ok == mk && oi < mi)) atomicAdd(&s_rank[k], 1u);
          }
          __syncthreads();
          // the verdict on entry nsure + k goes where it survives the loop (which stages rows over the
          // ranks): in place of the candidate's score, which nobody needs any more
          for (int i = tid; i < ncand; i += STEP_THREADS) s_cand_key[i] = s_rank[i] < (uint32_t)v.need ? 1u : 0u;
          __syncthreads();
        },
        [&](int entry) __attribute__((always_inline)) {
          // entries before pos_begin never come here; beyond the candidates (prefetch) reads are clamped
          return s_cand_key[min(max(entry - nsure, 0), ncand - 1)] != 0u;
        });
    if (timed_out) {
      poison_rows<DT, G>(p.dc, b, hs);
      return;
    }
    nsel = nsure + ncand;  // for the bitmap below only the admitted ones count: see there
  }
  if (p.want_list && compete) {
    // ---- the unit's words of the selection bitmap (a unit's blocks start at a multiple of 32)
    __syncthreads();  // every wave is done with the staging area
    uint32_t* s_bm = reinterpret_cast<uint32_t*>(lds);
    const int nw = (n + 31) >> 5;
    for (int w = tid; w < nw; w += STEP_THREADS) s_bm[w] = 0;
    __syncthreads();
    for (int i = tid; i < nsel; i += STEP_THREADS) {
      if (i >= nsure && s_cand_key[i - nsure] == 0u) continue;  // a candidate that was not admitted
      const int r = s_list[i] - j0;
      atomicOr(&s_bm[r >> 5], 1u << (r & 31));
    }
    __syncthreads();
    uint32_t* bm = p.bitmap + (size_t)t * p.bitmap_words + (j0 >> 5);
    for (int w = tid; w < nw; w += STEP_THREADS) st_i32<true>(reinterpret_cast<int32_t*>(bm + w), (int32_t)s_bm[w]);
    wait_stores_acknowledged();
    __syncthreads();
    if (tid == 0)
      __hip_atomic_fetch_add(p.listed + (size_t)t * ABSB_TICKET_STRIDE, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
  finish_split<DT, G>(p.dc, t, b, hs, c, U, p.units_max, st, lds, clear_words);
}

template <int DT, int G, int REP>
__global__ __launch_bounds__(STEP_THREADS, 2) void step_kernel(StepParams p) {
  extern __shared__ __align__(16) char lds[];
  const int per_seg = p.units_max + 1;
  const int t = blockIdx.x / per_seg, r = blockIdx.x % per_seg;
  if (r == 0)
    step_coordinator<DT, G>(p, t, lds);
  else
    step_unit<DT, G, REP>(p, t, r - 1, lds);
}

template <int DT, int G>
static void launch_step_rep(const StepParams& p, int repr, dim3 grid, size_t lds, hipStream_t stream) {
  if (repr == ABSB_REPR_MEAN)
    hipLaunchKernelGGL((step_kernel<DT, G, 0>), grid, dim3(STEP_THREADS), lds, stream, p);
  else
    hipLaunchKernelGGL((step_kernel<DT, G, 1>), grid, dim3(STEP_THREADS), lds, stream, p);
}

template <int DT>
static void launch_step_group(const StepParams& p, int repr, dim3 grid, size_t lds, hipStream_t stream) {
  switch (p.dc.g.Gd) {
    case 1: launch_step_rep<DT, 1>(p, repr, grid, lds, stream); break;
    case 2: launch_step_rep<DT, 2>(p, repr, grid, lds, stream); break;
    case 3: launch_step_rep<DT, 3>(p, repr, grid, lds, stream); break;
    case 4: launch_step_rep<DT, 4>(p, repr, grid, lds, stream); break;
    case 5: launch_step_rep<DT, 5>(p, repr, grid, lds, stream); break;
    case 6: launch_step_rep<DT, 6>(p, repr, grid, lds, stream); break;
    case 7: launch_step_rep<DT, 7>(p, repr, grid, lds, stream); break;
    default: launch_step_rep<DT, 8>(p, repr, grid, lds, stream); break;
  }
}

bool step_fits(const Plan& pl) {
  if (pl.max_blocks > TOPK_MAX_BLOCKS) return false;
  return (int64_t)pl.nseg * (pl.units_max + 1) < (int64_t(1) << 31) - 1;
}

int launch_step(const Geometry& g, const Plan& pl, int dtype, float sm_scale, const void* q, const uint8_t* codes,
                const float* qscale, const float* qmin, const void* k_cache, const void* v_cache, const int32_t* page_table,
                const int32_t* seq_lens, const int32_t* cent_off, const int32_t* budget, int32_t* sel_idx,
                int32_t* sel_cnt, bool want_list, void* out, float* lse, char* ws, hipStream_t stream) {
  if (!step_fits(pl)) return ABSB_ERR_UNSUPPORTED;
  StepParams p;
  int32_t* scores = reinterpret_cast<int32_t*>(ws + pl.ws_scores);
  p.sc = make_score_params(g, pl, q, codes, qscale, qmin, cent_off, seq_lens, scores, nullptr);
  p.tk = make_topk_params(g, scores, cent_off, budget, seq_lens, sel_idx, sel_cnt, pl.sel_stride, nullptr);
  p.dc = make_decode_params(g, pl, sm_scale, q, k_cache, v_cache, page_table, seq_lens, sel_idx, sel_cnt,
                            pl.sel_stride, out, lse, ws);
  p.dc.part_o = reinterpret_cast<float*>(ws + pl.ws_unit_o);
  p.dc.part_ml = reinterpret_cast<float*>(ws + pl.ws_unit_ml);
  p.dc.budget = budget;
  p.dc.cent_off = cent_off;
  p.dc.status = reinterpret_cast<int32_t*>(ws + pl.ws_status);
  p.arrive = reinterpret_cast<int32_t*>(ws + pl.ws_score_tickets);
  p.arrive_c = reinterpret_cast<int32_t*>(ws + pl.ws_cutoff);
  p.cand_done = reinterpret_cast<int32_t*>(ws + pl.ws_cand_done);
  p.listed = reinterpret_cast<int32_t*>(ws + pl.ws_listed);
  p.list_flag = reinterpret_cast<int32_t*>(ws + pl.ws_flags);
  p.rows = reinterpret_cast<uint16_t*>(ws + pl.ws_rows);
  p.cand = reinterpret_cast<uint2*>(ws + pl.ws_cand);
  p.bitmap = reinterpret_cast<uint32_t*>(ws + pl.ws_bitmap);
  p.units_max = pl.units_max;
  p.unit_tokens = pl.unit_tokens;
  p.bitmap_words = pl.bitmap_words;
  p.want_list = want_list ? 1 : 0;
  const dim3 grid((unsigned)((int64_t)pl.nseg * (pl.units_max + 1)));
  const size_t lds = step_max_sz((size_t)STEP_LDS_UNIT, topk_lds_bytes(pl.max_blocks));
  if (dtype == ABSB_F16)
    launch_step_group<ABSB_F16>(p, g.repr, grid, lds, stream);
  else
    launch_step_group<ABSB_BF16>(p, g.repr, grid, lds, stream);
  return check_launch();
}

}  // namespace absb
