// Attention over the selected blocks, device side (Sec. 3.4, kernel 3; Eq. (1) restricted to the selection).
//
// A selected logical block j of KV head h covers tokens [j*B_h, (j+1)*B_h); token t sits in
// physical page page_table[b][t / P] at slot t % P.  The kernel walks the selection as a virtual
// token sequence (position -> block list entry -> token -> page/slot) and reads K and V rows in
// place: no gather, no per-head page list, any mix of block sizes in one launch.
//
// Split-K flash decoding in one kernel: work-group (split, segment) handles `split_tokens`
// consecutive positions of its segment's selection and produces an unnormalised partial (m, l, o~)
// for the G query heads of the group.  A segment with one split normalises and writes its output
// rows directly; otherwise the partial goes to the workspace, the work-group draws a ticket from
// the segment's counter, and the one that draws the last ticket merges the segment's partials with
// the log-sum-exp rule.  No work-group ever waits for another, so the grid drains whatever the
// counters hold; they must be zero at launch (the selection kernel of the fused step clears them,
// the stand-alone entry point runs a clearing kernel first).
//
// Data path of one wave step (16 rows):
//   * global -> registers: a row is 256 bytes = 16 lanes x 16 bytes; each 16-lane group loads
//     four consecutive rows with 128-bit loads, so every wave load instruction covers whole rows;
//   * registers -> LDS: K rows as they are (row pitch 272 B, conflict-free for the reads below),
//     V transposed in registers first (4 rows x 8 channels per lane -> 8 channels x 4 rows), so
//     that the four rows a matrix operand needs at one channel sit in one 8-byte LDS word;
//   * the next step's global loads are issued here, and fly while this step computes from LDS;
//   * S = K Q^T and O += P V run on the 16x16x16 matrix instruction: with G <= 8 query rows
//     per K/V row the tile is mostly padding, but the vector pipeline (q.k dots, lane reductions,
//     P.V multiply-adds) was measured to cost as much time as the HBM stream itself, and the
//     matrix pipeline is idle otherwise.  The logits tile comes out in exactly the lane layout
//     the P operand of the second product needs (head = lane % 16, rows 4*(lane/16)..+3), so the
//     softmax runs in place with two cross-group maxima per step.
#pragma once
#include "common.h"

namespace absb {

struct DecodeParams {
  const uint16_t* q;
  const uint16_t* k;
  const uint16_t* v;
  const int32_t* page_table;
  const int32_t* seq_lens;
  const int32_t* sel_idx;
  const int32_t* sel_cnt;
  float* part_o;   // [nseg][max_splits][G][128]
  float* part_ml;  // [nseg][max_splits][G][4]  (running max in log2 units, sum of the rounded weights, exact sum, -)
  int32_t* tickets;  // [nseg], zero when the kernel starts
  // one-launch step only: the list is produced by another work-group of the same launch
  const int32_t* budget;    // [Bt]
  const int32_t* cent_off;  // [nseg+1]
  int32_t* flags;    // [nseg] (ABSB_TICKET_STRIDE apart): non-zero once the segment's list is complete
  int32_t* status;   // one word: set non-zero when a wait ran into its time limit
  void* out;       // [Bt][Hq][128]
  float* lse;      // [Bt][Hq] or null
  int32_t sel_stride, split_tokens, max_splits;
  float scale_log2;  // sm_scale * log2(e)
  Geometry g;
};

inline DecodeParams make_decode_params(const Geometry& g, const Plan& pl, float sm_scale, const void* q,
                                       const void* k_cache, const void* v_cache, const int32_t* page_table,
                                       const int32_t* seq_lens, const int32_t* sel_idx, const int32_t* sel_cnt,
                                       int32_t sel_stride, void* out, float* lse, char* ws) {
  DecodeParams p;
  p.q = static_cast<const uint16_t*>(q);
  p.k = static_cast<const uint16_t*>(k_cache);
  p.v = static_cast<const uint16_t*>(v_cache);
  p.page_table = page_table;
  p.seq_lens = seq_lens;
  p.sel_idx = sel_idx;
  p.sel_cnt = sel_cnt;
  p.part_o = reinterpret_cast<float*>(ws + pl.ws_part_o);
  p.part_ml = reinterpret_cast<float*>(ws + pl.ws_part_ml);
  p.tickets = reinterpret_cast<int32_t*>(ws + pl.ws_tickets);
  p.budget = nullptr;
  p.cent_off = nullptr;
  p.flags = nullptr;
  p.status = nullptr;
  p.out = out;
  p.lse = lse;
  p.sel_stride = sel_stride;
  p.split_tokens = pl.split_tokens;
  p.max_splits = pl.max_splits;
  p.scale_log2 = sm_scale * 1.4426950408889634f;
  p.g = g;
  return p;
}

constexpr float M_INIT = -1.0e30f;  // finite stand-in for "no token seen yet"
constexpr int DEC_THREADS = 256;
constexpr int DEC_WAVES = DEC_THREADS / 64;
constexpr int ROWS_PER_WAVE_STEP = 16;        // 4 row-groups x 4 consecutive rows
constexpr int K_PITCH = 272;                  // bytes per staged K row (256 + 16: spreads rows over banks)
constexpr int K_TILE_BYTES = ROWS_PER_WAVE_STEP * K_PITCH;
constexpr int V_TILE_BYTES = 8 * 512;         // [channel % 8][channel / 8][16 rows] 16-bit
constexpr int STAGE_BYTES = K_TILE_BYTES + V_TILE_BYTES;
constexpr int MRG_UNROLL = 16;                // splits a thread merges per memory round trip
// LDS of one work-group: the waves' staging areas (reused by the epilogue), per-wave maxima and
// the two sums per head, two words for work-group broadcasts
constexpr int DEC_LDS_STATE = DEC_WAVES * STAGE_BYTES;
constexpr int DEC_LDS_BYTES = DEC_LDS_STATE + 3 * ABSB_MAX_GROUP * DEC_WAVES * 4 + 16;
// a work-group that waits for its segment's list gives up after this long (100 MHz ticks): the
// wait cannot outlast the launch whatever the rest of the grid does
constexpr uint64_t DEC_WAIT_LIMIT_TICKS = 25u * 1000u * 1000u;

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

typedef float float4_t __attribute__((ext_vector_type(4)));
typedef _Float16 half4_t __attribute__((ext_vector_type(4)));
typedef short short4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef float float2_t __attribute__((ext_vector_type(2)));

// D(16x16) += A(16x16) B(16x16), operands as four 16-bit values per lane:
// A[m = lane%16][k = 4*(lane/16)+i], B[k = 4*(lane/16)+i][n = lane%16], D[m = 4*(lane/16)+i][n = lane%16].
template <int DT>
__device__ __forceinline__ float4_t mma16(uint2 a, uint2 b, float4_t c) {
  if (DT == ABSB_F16)
    return __builtin_amdgcn_mfma_f32_16x16x16f16(bitcast<half4_t>(a), bitcast<half4_t>(b), c, 0, 0, 0);
  return __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(bitcast<short4_t>(a), bitcast<short4_t>(b), c, 0, 0, 0);
}

// The same 32-bit word (two adjacent channels) of four consecutive V rows -> two LDS words, one per
// channel, each holding that channel's four rows.  `dst` addresses the even channel's word.
__device__ __forceinline__ void stage_v_word(char* dst, uint32_t r0, uint32_t r1, uint32_t r2, uint32_t r3) {
  const uint32_t e01 = __builtin_amdgcn_perm(r1, r0, 0x05040100u);  // low halves: even channel, rows 0,1
  const uint32_t e23 = __builtin_amdgcn_perm(r3, r2, 0x05040100u);
  const uint32_t o01 = __builtin_amdgcn_perm(r1, r0, 0x07060302u);  // high halves: odd channel
  const uint32_t o23 = __builtin_amdgcn_perm(r3, r2, 0x07060302u);
  *reinterpret_cast<uint2*>(dst) = make_uint2(e01, e23);
  *reinterpret_cast<uint2*>(dst + 512) = make_uint2(o01, o23);
}

// Where the attention loop takes a segment's block list from.
enum : int {
  LIST_PLAIN = 0,     // device memory, complete before the launch
  LIST_COHERENT = 1,  // device memory, written by another work-group of this launch: device-coherent loads
  LIST_LOCAL = 2      // this work-group's LDS
};

// A block list: entry i is a block index of the segment.  Indices beyond `last` read entry `last`
// (the loop prefetches ahead of the range it works on; the clamp keeps every read inside the storage).
template <int SRC>
struct ListRef {
  const int32_t* ptr;
  int last;
  __device__ __forceinline__ int at(int i) const {
    i = min(i, last);
    if (SRC == LIST_COHERENT) return ld_i32<true>(ptr + i);
    return ptr[i];
  }
};

// Logical page -> physical page of one request: the page table row in device memory, or a copy of the
// entries [first, first + count) that the work-group holds in LDS.
typedef __attribute__((address_space(3))) const int32_t lds_const_i32;
struct PageRef {
  const int32_t* row;    // device memory
  lds_const_i32* local;  // LDS copy, or null (typed as LDS: a generic pointer would make these reads wait
                         // for every row load in flight)
  int first, count;
  __device__ __forceinline__ int at(int page) const {
    if (local) return local[min(max(page - first, 0), count - 1)];
    return row[page];
  }
};

// Running state of the online softmax of one wave: per head (= lane % 16) the running maximum, common
// to the wave's four row groups; partial sums over the lane's rows of the weights as rounded for the
// P V product (the output's normaliser: the output stays a convex combination of value rows) and of
// the weights before rounding (the log-sum-exp: rounding to bf16 would bias it by up to 2^-8 when all
// weights round the same way); O[head = 4*grp + i][channel = 8*li + j], j = 0..7.
struct AttnState {
  float m, l, lx;
  float4_t oacc[8];
  __device__ __forceinline__ void reset() {
    m = M_INIT;
    l = 0.0f;
    lx = 0.0f;
#pragma unroll
    for (int j = 0; j < 8; ++j) oacc[j] = float4_t{0.0f, 0.0f, 0.0f, 0.0f};
  }
};

// What a work-group needs to know about its segment and its place in LDS.
struct SplitCtx {
  int b, hs, hk, lb, L, lP;
  size_t lane_off;
  char* kt;  // this wave's staging areas
  char* vt;
};

// Q as the B operand of S = K Q^T: lane (head = li, k-group = grp) holds Q[head][16*ks + 4*grp + i];
// heads beyond G are zero rows of the tile.
template <int G>
__device__ __forceinline__ void load_q(const DecodeParams& p, int b, int hs, uint2 (&qb)[8]) {
  const int lane = threadIdx.x & 63, grp = lane >> 4, li = lane & 15;
#pragma unroll
  for (int ks = 0; ks < 8; ++ks) {
    qb[ks] = make_uint2(0u, 0u);
    if (li < G)
      qb[ks] = *reinterpret_cast<const uint2*>(p.q + ((size_t)b * p.g.Hq + (size_t)hs * G + li) * ABSB_HEAD_DIM + 16 * ks +
                                               4 * grp);
  }
}

// Attention of this wave over positions [pos_begin, pos_end) of the virtual token sequence of a block
// list (position -> list entry pos >> lb -> token -> page/slot), folded into `st`.  A work-group step
// covers DEC_WAVES * 16 consecutive positions, 16 per wave; pos_begin must be a multiple of 4.  `sj`:
// the list entry of this lane's first rows, fetched by the caller (so that the load is in flight early).
//
// `after_first_issue()` runs once the first step's row loads are in flight (work that has to wait for
// memory anyway can hide behind them; it may contain barriers: every wave of the work-group calls this
// function).  `live(entry)`: false for list entries whose rows were requested but must not count
// (evaluated when a step is computed, after after_first_issue()).
struct NoHook {
  __device__ __forceinline__ void operator()() const {}
};
struct AllLive {
  __device__ __forceinline__ bool operator()(int) const { return true; }
};
template <int DT, int G, int SRC, class Hook = NoHook, class Live = AllLive>
__device__ __forceinline__ void attend_positions(const DecodeParams& p, const SplitCtx& c, const ListRef<SRC>& list,
                                                 const PageRef& pages, int pos_begin, int pos_end, int sj,
                                                 const uint2 (&qb)[8], AttnState& st, Hook&& after_first_issue = Hook(),
                                                 Live&& live = Live()) {
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, grp = lane >> 4, li = lane & 15;
  const int lb = c.lb, L = c.L, lP = c.lP;
  char* kt = c.kt;
  char* vt = c.vt;
  constexpr int STEP = DEC_WAVES * ROWS_PER_WAVE_STEP;  // positions per work-group step
  u32x4 k0, k1, k2, k3, v0, v1, v2, v3;

  // The address chain list entry -> page-table entry -> row is kept two steps deep so that only
  // the row loads themselves wait on memory inside the loop: issuing step k's rows uses the page
  // requested during step k-1, requests the page of step k+1 (whose list entry has arrived by
  // then) and the list entry of step k+2.
  //   tcb: first token of the lane's four rows (clamped into the context, so every address is
  //        legal), pg: its physical page, vb: which of the four rows are real.
#define ABSB_GROUP_TOKEN(base_of_step)                                                                \
  {                                                                                                   \
    const int pos = (base_of_step) + grp * 4;                                                         \
    const int t = (sj << lb) + (pos & ((1 << lb) - 1));                                               \
    vb = 0;                                                                                           \
    _Pragma("unroll") for (int r = 0; r < 4; ++r)                                                     \
        vb |= (uint32_t)(pos + r < pos_end && t + r < L) << r; /* a selected last block may be partial */ \
    tcb = max(0, min(t, L - 1)) & ~3;                                                                 \
    pg = pages.at(tcb >> lP);                                                                         \
  }
#define ABSB_ISSUE(base_expr)                                                                         \
  {                                                                                                   \
    const int base_ = (base_expr);                                                                    \
    const size_t row0 = (size_t)pg * p.g.s_page + c.lane_off;                                         \
    const size_t off0 = row0 + (size_t)(min(tcb + 0, L - 1) & ((1 << lP) - 1)) * p.g.s_tok;           \
    const size_t off1 = row0 + (size_t)(min(tcb + 1, L - 1) & ((1 << lP) - 1)) * p.g.s_tok;           \
    const size_t off2 = row0 + (size_t)(min(tcb + 2, L - 1) & ((1 << lP) - 1)) * p.g.s_tok;           \
    const size_t off3 = row0 + (size_t)(min(tcb + 3, L - 1) & ((1 << lP) - 1)) * p.g.s_tok;           \
    valid_next = vb;                                                                                  \
    k0 = *reinterpret_cast<const u32x4*>(p.k + off0);                                                 \
    k1 = *reinterpret_cast<const u32x4*>(p.k + off1);                                                 \
    k2 = *reinterpret_cast<const u32x4*>(p.k + off2);                                                 \
    k3 = *reinterpret_cast<const u32x4*>(p.k + off3);                                                 \
    v0 = *reinterpret_cast<const u32x4*>(p.v + off0);                                                 \
    v1 = *reinterpret_cast<const u32x4*>(p.v + off1);                                                 \
    v2 = *reinterpret_cast<const u32x4*>(p.v + off2);                                                 \
    v3 = *reinterpret_cast<const u32x4*>(p.v + off3);                                                 \
    ABSB_GROUP_TOKEN(base_ + STEP)                                                                    \
    sj = list.at((base_ + 2 * STEP + grp * 4) >> lb);                                                 \
  }

  int base = pos_begin + wave * ROWS_PER_WAVE_STEP;
  uint32_t valid_next = 0, vb;
  int tcb, pg;
  ABSB_GROUP_TOKEN(base)                           // first step: entry -> page, in order
  sj = list.at((base + STEP + grp * 4) >> lb);     // second step's entry
  if (base < pos_end) ABSB_ISSUE(base)
  after_first_issue();
  float m = st.m, l = st.l, lx = st.lx;
  while (base < pos_end) {  // trip count depends on the wave only: every branch here is wave-uniform
    // ---- stage the step's rows in LDS
    const uint32_t valid = live((base + grp * 4) >> lb) ? valid_next : 0u;
    *reinterpret_cast<u32x4*>(kt + (grp * 4 + 0) * K_PITCH + li * 16) = k0;
    *reinterpret_cast<u32x4*>(kt + (grp * 4 + 1) * K_PITCH + li * 16) = k1;
    *reinterpret_cast<u32x4*>(kt + (grp * 4 + 2) * K_PITCH + li * 16) = k2;
    *reinterpret_cast<u32x4*>(kt + (grp * 4 + 3) * K_PITCH + li * 16) = k3;
    // 32-bit word d of a row = channels 2d, 2d+1 of the lane's eight
    stage_v_word(vt + 0 * 1024 + li * 32 + grp * 8, v0.x, v1.x, v2.x, v3.x);
    stage_v_word(vt + 1 * 1024 + li * 32 + grp * 8, v0.y, v1.y, v2.y, v3.y);
    stage_v_word(vt + 2 * 1024 + li * 32 + grp * 8, v0.z, v1.z, v2.z, v3.z);
    stage_v_word(vt + 3 * 1024 + li * 32 + grp * 8, v0.w, v1.w, v2.w, v3.w);
    // ---- next step's rows go in flight now; they land while this step computes
    const int next = base + STEP;
    if (next < pos_end) ABSB_ISSUE(next)

    // ---- S[row][head] = K Q^T over the 128 channels (two accumulators: shorter dependent chain)
    float4_t s0 = {0.0f, 0.0f, 0.0f, 0.0f}, s1 = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
    for (int ks = 0; ks < 8; ks += 2) {
      const uint2 a0 = *reinterpret_cast<const uint2*>(kt + li * K_PITCH + (16 * ks + 4 * grp) * 2);
      const uint2 a1 = *reinterpret_cast<const uint2*>(kt + li * K_PITCH + (16 * (ks + 1) + 4 * grp) * 2);
      s0 = mma16<DT>(a0, qb[ks], s0);
      s1 = mma16<DT>(a1, qb[ks + 1], s1);
    }
    // ---- online softmax in place: this lane holds rows 4*grp..4*grp+3 of head li
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
    // ---- rescale O when some head's maximum moved (rare once the maxima have settled)
    if (__any(alpha != 1.0f)) {
      float ah[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const float a_lo = bitcast<float>(__builtin_amdgcn_readlane(bitcast<int>(alpha), i));
        const float a_hi = bitcast<float>(__builtin_amdgcn_readlane(bitcast<int>(alpha), (G > 4 ? 4 + i : i)));
        ah[i] = (G > 4 && grp == 1) ? a_hi : a_lo;  // groups beyond the heads hold zeros: any factor does
      }
#pragma unroll
      for (int j = 0; j < 8; ++j) {
#pragma unroll
        for (int i = 0; i < 4; ++i) st.oacc[j][i] *= ah[i];
      }
    }
    // ---- O[head][channel] += P V: B operand = four rows of one channel, one LDS word
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const uint2 bv = *reinterpret_cast<const uint2*>(vt + j * 512 + li * 32 + grp * 8);
      st.oacc[j] = mma16<DT>(pa, bv, st.oacc[j]);
    }
    base = next;
  }
#undef ABSB_ISSUE
#undef ABSB_GROUP_TOKEN
  st.m = m;
  st.l = l;
  st.lx = lx;
}

// An empty selection: the output rows are zero, the log-sum-exp -inf.
template <int G>
__device__ __forceinline__ void write_empty_rows(const DecodeParams& p, int b, int hs) {
  for (int i = threadIdx.x; i < G * ABSB_HEAD_DIM; i += DEC_THREADS) {
    const size_t row = (size_t)b * p.g.Hq + (size_t)hs * G + (i >> 7);
    static_cast<uint16_t*>(p.out)[row * ABSB_HEAD_DIM + (i & 127)] = 0;
    if (p.lse && (i & 127) == 0) p.lse[row] = -__builtin_inff();
  }
}

// A wait ran out: the segment's output cannot be completed.  Its rows are set to NaN so that nobody
// takes stale values for results.
template <int DT, int G>
__device__ __forceinline__ void poison_rows(const DecodeParams& p, int b, int hs) {
  const uint16_t nan16 = DT == ABSB_F16 ? (uint16_t)0x7e00 : (uint16_t)0x7fc0;
  for (int i = threadIdx.x; i < G * ABSB_HEAD_DIM; i += DEC_THREADS) {
    const size_t row = (size_t)b * p.g.Hq + (size_t)hs * G + (i >> 7);
    static_cast<uint16_t*>(p.out)[row * ABSB_HEAD_DIM + (i & 127)] = nan16;
    if (p.lse && (i & 127) == 0) p.lse[row] = __builtin_nanf("");
  }
}

// The end of a work-group's attention: the four wave states are folded into the work-group's partial;
// with one split per segment it is normalised and written out; otherwise it goes to slot `split` of
// the segment's partials, the work-group draws a ticket, and the one that draws ticket nsplit - 1
// merges the segment's `nsplit` partials with the log-sum-exp rule and writes the output rows.
// `slots`: partial slots per segment (the stride of the partial arrays).  `on_last`: called by thread 0
// of the segment's last work-group (the merging one, or the only one), for flags of the segment that
// have to go back to zero: every other work-group of the segment has drawn its ticket by then.  Every
// thread of the work-group must call.
template <int DT, int G, class OnLast>
__device__ __forceinline__ void finish_split(const DecodeParams& p, int s, int b, int hs, int split, int nsplit, int slots,
                                             AttnState& st, char* lds, OnLast&& on_last) {
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, grp = lane >> 4, li = lane & 15;
  char* s_stage = lds;
  float (*s_m)[DEC_WAVES] = reinterpret_cast<float (*)[DEC_WAVES]>(lds + DEC_LDS_STATE);
  float (*s_l)[DEC_WAVES] = s_m + ABSB_MAX_GROUP;
  float (*s_lx)[DEC_WAVES] = s_l + ABSB_MAX_GROUP;
  int* s_bcast = reinterpret_cast<int*>(lds + DEC_LDS_STATE + 3 * ABSB_MAX_GROUP * DEC_WAVES * 4);
  float m = st.m, l = st.l, lx = st.lx;

  // ---- the wave's state: m per head (lane li), l summed over the four groups, O in groups 0 (and 1)
  l += __shfl_xor(l, 16);
  l += __shfl_xor(l, 32);
  lx += __shfl_xor(lx, 16);
  lx += __shfl_xor(lx, 32);
  if (grp == 0 && li < G) s_m[li][wave] = m;
  __syncthreads();  // also: every wave is done with its staging area, which the merge reuses below
  // work-group maximum per head; own state rescaled to it, so that the four states simply add up
  float* s_o = reinterpret_cast<float*>(s_stage);  // [DEC_WAVES][G][128]
  if (grp == 0 && li < G) {
    const float M = fmaxf(fmaxf(s_m[li][0], s_m[li][1]), fmaxf(s_m[li][2], s_m[li][3]));
    const float a = fast_exp2(m - M);
    s_l[li][wave] = l * a;
    s_lx[li][wave] = lx * a;
  }
  if (grp * 4 < G) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int hd = grp * 4 + i;
      if (hd < G) {
        const float M = fmaxf(fmaxf(s_m[hd][0], s_m[hd][1]), fmaxf(s_m[hd][2], s_m[hd][3]));
        const float a = fast_exp2(s_m[hd][wave] - M);
        float4* dst = reinterpret_cast<float4*>(s_o + ((size_t)wave * G + hd) * ABSB_HEAD_DIM + li * 8);
        dst[0] = make_float4(st.oacc[0][i] * a, st.oacc[1][i] * a, st.oacc[2][i] * a, st.oacc[3][i] * a);
        dst[1] = make_float4(st.oacc[4][i] * a, st.oacc[5][i] * a, st.oacc[6][i] * a, st.oacc[7][i] * a);
      }
    }
  }
  __syncthreads();
  // ---- the work-group's partial: thread -> column (head g, channels 4*c4..4*c4+3), G*32 columns
  constexpr int NCOL = G * 32;
  constexpr int CP = NCOL <= 32 ? 32 : NCOL <= 64 ? 64 : NCOL <= 128 ? 128 : 256;  // columns, padded to 2^k
  constexpr int SL = DEC_THREADS / CP;                                             // split lanes per column
  const int col = tid & (CP - 1), sl = tid / CP;
  const int g = min(col, NCOL - 1) >> 5, c4 = col & 31;
  float4_t O = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
  for (int w = 0; w < DEC_WAVES; ++w)
    O += *reinterpret_cast<const float4_t*>(s_o + ((size_t)w * G + g) * ABSB_HEAD_DIM + c4 * 4);
  float M = fmaxf(fmaxf(s_m[g][0], s_m[g][1]), fmaxf(s_m[g][2], s_m[g][3]));
  float Lsum = (s_l[g][0] + s_l[g][1]) + (s_l[g][2] + s_l[g][3]);
  float Lx = (s_lx[g][0] + s_lx[g][1]) + (s_lx[g][2] + s_lx[g][3]);

  if (nsplit > 1) {
    // Publish the partial, take a ticket; the work-group that draws the segment's last ticket merges.
    // Visibility across the chip's L2 slices without a cache write-back: partials are written and
    // read with device-coherent accesses (the sc1 cache policy, which the non-coherent cache levels
    // do not serve), a writer waits for its stores to be acknowledged before it draws its ticket,
    // and the merging group issues its reads only after its ticket has come back.  Nobody waits
    // for anybody.
    constexpr int COHERENT = 16;  // cache-policy operand of the buffer instructions: sc1
    const size_t slot0 = (size_t)s * slots;
    const __amdgpu_buffer_rsrc_t part_o = __builtin_amdgcn_make_buffer_rsrc(
        p.part_o + slot0 * G * ABSB_HEAD_DIM, 0, slots * G * ABSB_HEAD_DIM * 4, 0x00020000);
    const __amdgpu_buffer_rsrc_t part_ml =
        __builtin_amdgcn_make_buffer_rsrc(p.part_ml + slot0 * G * 4, 0, slots * G * 16, 0x00020000);
    if (tid < NCOL) {
      __builtin_amdgcn_raw_buffer_store_b128(bitcast<u32x4>(O), part_o, ((split * G + g) * ABSB_HEAD_DIM + c4 * 4) * 4,
                                             0, COHERENT);
      if (c4 == 0)
        __builtin_amdgcn_raw_buffer_store_b128(bitcast<u32x4>(float4_t{M, Lsum, Lx, 0.0f}), part_ml,
                                               (split * G + g) * 16, 0, COHERENT);
    }
    int& s_last = s_bcast[0];
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // this thread's stores have been acknowledged
    __syncthreads();                                   // ... and so have everybody's
    if (tid == 0)
      s_last = __hip_atomic_fetch_add(p.tickets + (size_t)s * ABSB_TICKET_STRIDE, 1, __ATOMIC_RELAXED,
                                      __HIP_MEMORY_SCOPE_AGENT) == nsplit - 1;
    __syncthreads();
    if (!s_last) return;
    // every counter a launch touches is back at zero when the launch ends
    if (tid == 0) {
      __hip_atomic_store(p.tickets + (size_t)s * ABSB_TICKET_STRIDE, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      on_last();
    }

    // log-sum-exp merge: split lane `sl` of a column takes splits sl, sl + SL, ...; MRG_UNROLL of
    // them per memory round trip, folded into a running (M, Lsum, O)
    M = M_INIT;
    Lsum = 0.0f;
    Lx = 0.0f;
    O = float4_t{0.0f, 0.0f, 0.0f, 0.0f};
    for (int i0 = sl; i0 < nsplit; i0 += SL * MRG_UNROLL) {
      float4_t mlv[MRG_UNROLL];
      float4_t ov[MRG_UNROLL];
#pragma unroll
      for (int u = 0; u < MRG_UNROLL; ++u) {
        const int i = min(i0 + u * SL, nsplit - 1);  // the tail repeats the last slot, with weight 0
        mlv[u] = bitcast<float4_t>(__builtin_amdgcn_raw_buffer_load_b128(part_ml, (i * G + g) * 16, 0, COHERENT));
        ov[u] = bitcast<float4_t>(
            __builtin_amdgcn_raw_buffer_load_b128(part_o, ((i * G + g) * ABSB_HEAD_DIM + c4 * 4) * 4, 0, COHERENT));
      }
      float bm = M;
#pragma unroll
      for (int u = 0; u < MRG_UNROLL; ++u) bm = fmaxf(bm, mlv[u].x);
      const float a = fast_exp2(M - bm);
      O *= a;
      Lsum *= a;
      Lx *= a;
      M = bm;
#pragma unroll
      for (int u = 0; u < MRG_UNROLL; ++u) {
        const float w = i0 + u * SL < nsplit ? fast_exp2(mlv[u].x - bm) : 0.0f;
        O += ov[u] * w;
        Lsum = __builtin_fmaf(mlv[u].y, w, Lsum);
        Lx = __builtin_fmaf(mlv[u].z, w, Lx);
      }
    }
    if (SL > 1) {  // fold the split lanes of a column (the staging area is free again)
      float* s_red = reinterpret_cast<float*>(s_stage);  // [SL][CP][8]
      __syncthreads();
      float* mine = s_red + ((size_t)sl * CP + col) * 8;
      *reinterpret_cast<float4_t*>(mine) = float4_t{M, Lsum, Lx, 0.0f};
      *reinterpret_cast<float4_t*>(mine + 4) = O;
      __syncthreads();
      if (sl == 0) {
        float bm = M;
#pragma unroll
        for (int k = 1; k < SL; ++k) bm = fmaxf(bm, s_red[((size_t)k * CP + col) * 8]);
        const float a = fast_exp2(M - bm);
        O *= a;
        Lsum *= a;
        Lx *= a;
        M = bm;
#pragma unroll
        for (int k = 1; k < SL; ++k) {
          const float* sr = s_red + ((size_t)k * CP + col) * 8;
          const float w = fast_exp2(sr[0] - bm);
          Lsum = __builtin_fmaf(sr[1], w, Lsum);
          Lx = __builtin_fmaf(sr[2], w, Lx);
#pragma unroll
          for (int j = 0; j < 4; ++j) O[j] = __builtin_fmaf(sr[4 + j], w, O[j]);
        }
      }
    }
  }

  if (nsplit <= 1 && tid == 0) on_last();

  // ---- normalise and write the group's output rows
  if (tid < NCOL) {
    const size_t row = (size_t)b * p.g.Hq + (size_t)hs * G + g;
    const bool any = Lsum > 0.0f;
    const float inv = any ? 1.0f / Lsum : 0.0f;
    const uint32_t lo = (uint32_t)Elem<DT>::narrow(O[0] * inv) | ((uint32_t)Elem<DT>::narrow(O[1] * inv) << 16);
    const uint32_t hi = (uint32_t)Elem<DT>::narrow(O[2] * inv) | ((uint32_t)Elem<DT>::narrow(O[3] * inv) << 16);
    *reinterpret_cast<uint2*>(static_cast<uint16_t*>(p.out) + row * ABSB_HEAD_DIM + c4 * 4) = make_uint2(lo, hi);
    if (p.lse && c4 == 0) p.lse[row] = any ? (M + __builtin_log2f(Lx)) * 0.6931471805599453f : -__builtin_inff();
  }
}

// Waits (thread 0, bounded in time) until the 32-bit word at `flag` is non-zero; every thread of the
// work-group returns the value seen (0: the wait ran into its limit; *status is then set).  Two
// barriers inside.  `s_word`: one word of LDS.
__device__ __forceinline__ int wait_for_flag(const int32_t* flag, int32_t* status, int* s_word) {
  if (threadIdx.x == 0) {
    int v = ld_i32<true>(flag);
    if (!v) {
      const uint64_t t0 = wall_clock64();
      do {
        __builtin_amdgcn_s_sleep(8);
        v = ld_i32<true>(flag);
      } while (!v && wall_clock64() - t0 < DEC_WAIT_LIMIT_TICKS);
    }
    if (!v) st_i32<true>(status, 1);
    *s_word = v;
  }
  __syncthreads();
  const int v = *s_word;
  __syncthreads();  // the word may be reused
  return v;
}

// Partial (and, for the last arriver, merged) attention of split `split` of segment s by one
// work-group of DEC_THREADS threads.  LISTED == false: the block list was complete before the
// launch.  LISTED == true (the pipelined one-launch step): the list is being produced by another work-group of
// this launch with a lower index; its length K_s is recomputed here from the budget, the
// work-group waits (bounded) for the segment's flag before it reads the list with device-coherent
// loads, and the segment's last work-group clears the flag again; a wait that ran out leaves NaN in
// the segment's rows.  `lds`: DEC_LDS_BYTES.
template <int DT, int G, bool LISTED>
__device__ __forceinline__ void decode_split(const DecodeParams& p, int s, int split, char* lds) {
  // s is a SELECTION segment: its G (= the template's) query heads start at head hs * G; hk is the
  // KV head whose rows they read
  const SegMap sm = seg_map(s, p.g.Hsel, p.g.Rk, p.g.Hkv);
  const int b = sm.b, hs = sm.hs, hk = sm.hk;
  const int lb = p.g.heads.log2_block[hk];
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, grp = lane >> 4, li = lane & 15;
  constexpr int SRC = LISTED ? LIST_COHERENT : LIST_PLAIN;
  const ListRef<SRC> list{p.sel_idx + (size_t)s * p.sel_stride, p.sel_stride - 1};
  const int pos_begin = split * p.split_tokens;

  // A lane's four rows of a step are four consecutive positions starting at a multiple of four:
  // they lie in one block (B >= 8) and one page (P >= 8), so one list entry and one page-table
  // entry serve all four.  The first step's list entry is fetched before the list length is known
  // (the index is clamped to the list's storage, so the read is always legal); this takes one
  // memory round trip off the dependent chain count -> entry -> page -> row.
  int sj = 0;
  if (!LISTED) sj = list.at((pos_begin + wave * ROWS_PER_WAVE_STEP + grp * 4) >> lb);

  // never beyond what the launch covers (a list longer than promised is cut, not overrun)
  int nsel;
  if (LISTED) {
    const int rows = p.cent_off[sm.s + 1] - p.cent_off[sm.s];
    nsel = budget_blocks(p.budget[b], lb, blocks_in_use(p.g.tight, rows, p.seq_lens, b, lb), p.sel_stride);
  } else {
    nsel = p.sel_cnt[s];
  }
  const int ntok = min(nsel << lb, p.max_splits * p.split_tokens);
  if (ntok == 0 && split == 0) write_empty_rows<G>(p, b, hs);
  if (pos_begin >= ntok) return;
  const int pos_end = min(ntok, pos_begin + p.split_tokens);

  SplitCtx c;
  c.b = b;
  c.hs = hs;
  c.hk = hk;
  c.lb = lb;
  c.L = p.seq_lens[b];
  c.lP = p.g.log2_page;
  c.lane_off = (size_t)hk * p.g.s_head + (size_t)li * 8;
  c.kt = lds + wave * STAGE_BYTES;
  c.vt = c.kt + K_TILE_BYTES;
  const PageRef pages{p.page_table + (size_t)b * p.g.pt_stride, nullptr, 0, 0};
  int* s_bcast = reinterpret_cast<int*>(lds + DEC_LDS_STATE + 3 * ABSB_MAX_GROUP * DEC_WAVES * 4);
  const int nsplit = (ntok + p.split_tokens - 1) / p.split_tokens;

  uint2 qb[8];
  load_q<G>(p, b, hs, qb);

  int32_t* flag = LISTED ? p.flags + (size_t)s * ABSB_TICKET_STRIDE : nullptr;
  if (LISTED) {
    // The list comes from a work-group with a lower index, which never waits for anything and was
    // dispatched before this one: the wait ends.  The time limit only makes that unconditional.
    if (!wait_for_flag(flag, p.status, s_bcast + 1)) {
      if (split == 0) poison_rows<DT, G>(p, b, hs);  // nobody will complete this segment's rows
      return;
    }
    sj = list.at((pos_begin + wave * ROWS_PER_WAVE_STEP + grp * 4) >> lb);
  }

  AttnState st;
  st.reset();
  attend_positions<DT, G, SRC>(p, c, list, pages, pos_begin, pos_end, sj, qb, st);
  finish_split<DT, G>(p, s, b, hs, split, nsplit, p.max_splits, st, lds, [&]() {
    if (LISTED) st_i32<true>(flag, 0);  // every reader of the list has drawn its ticket
  });
}

}  // namespace absb
