// Internal declarations shared by the translation units of libabsb.so (not installed).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "absb.h"

#define ABSB_HEAD_DIM 128
#define ABSB_MAX_KV_HEADS 64
#define ABSB_MAX_GROUP 8
#define ABSB_MAX_SEL_BLOCKS (1 << 17)  // blocks per segment the selection holds (its LDS bitmap)
#define ABSB_HIDDEN __attribute__((visibility("hidden")))
// Split counters sit 256 bytes apart: counters that share a memory line serialise each other's
// atomic updates (measured: 8 segments x 32 arrivals on one line cost 2.7 us, apart 0.x us).
#define ABSB_TICKET_STRIDE 64
#define ABSB_STEP_MAX_UNITS 64   // work-groups that share a segment in the one-launch step

namespace absb {

// Per-KV-head block sizes as log2, passed to kernels by value.
struct HeadTable {
  uint8_t log2_block[ABSB_MAX_KV_HEADS];
};

// Shape of the layer and of the paged cache, passed to kernels by value.
struct Geometry {
  int32_t Bt, Hq, Hkv, G;
  // Selection segments.  Group selection (default): one per (request, KV head), whose G query
  // heads share the list: Hsel = Hkv, Gd = G, Rk = 1.  Per-query-head selection: one per
  // (request, query head): Hsel = Hq, Gd = 1, Rk = G selection segments read each KV head's store.
  int32_t Hsel, Gd, Rk;
  int32_t agg_max;    // 1: a group's shared score is the maximum over its query heads (else their sum)
  int32_t log2_page;  // P = 1 << log2_page
  int32_t pt_stride;
  int32_t repr;       // absb_repr: vectors per block = repr + 1
  int32_t sink_tokens, recent_tokens;  // forced blocks of the selection (0 = none)
  int32_t tight;      // 1: the block layout is that of the current lengths (off[s+1] - off[s] = N_s)
  int64_t s_page, s_head, s_tok;  // element strides of the K/V caches
  HeadTable heads;
};

// Host-side sizes derived from (layer, batch).
struct Plan {
  int32_t nseg;             // selection segments: Bt * Hsel
  int32_t nstore;           // store segments: Bt * Hkv
  int64_t total;            // total centroids (rows of the store)
  int32_t max_blocks;       // max_s N_s
  int32_t sel_stride;       // max_s K_s (0 when no budget was given)
  int64_t max_tokens;       // max_s (upper bound of selected tokens of a segment)
  int64_t sum_tokens;       // sum_s of the same bound
  int32_t split_tokens;     // tokens per split-K work-group
  int32_t max_splits;       // grid.x of the decode kernels
  int32_t one_launch;       // absb_decode_fused: the whole step as one launch (else one launch per stage)
  int32_t step_form;        // absb_step_form actually used (never ABSB_STEP_AUTO)
  int32_t unit_tokens;      // one-launch step: selected tokens a unit should get
  int32_t units_max;        // max_s units of a segment
  int32_t bitmap_words;     // words of a segment's selection bitmap
  int32_t score_chunk;      // centroids per work-group in score
  int32_t build_chunk_tokens;  // tokens per work-group in build (a head's chunk: max(16, that / B_h) blocks)
  int32_t build_max_chunks;    // max_s ceil(N_s / chunk_h)
  // workspace carving (byte offsets, 256-aligned)
  size_t ws_part_o, ws_part_ml, ws_tickets;       // decode partials, per-segment split counters
  size_t ws_score_tickets, ws_flags, ws_status;   // more counters of the one-launch step
  size_t ws_cand_done, ws_listed, ws_cutoff;      // ... and of its unit form
  size_t ws_rows, ws_cand, ws_bitmap, ws_unit_o, ws_unit_ml;
  size_t ws_head_bytes;                           // all counters: the part absb_workspace_init clears
  size_t ws_scores, ws_sel_idx, ws_sel_cnt;       // fused step intermediates
  size_t ws_cent, ws_minmax, ws_qinv;             // build intermediates
  size_t ws_decode_bytes, ws_fused_bytes, ws_build_bytes, ws_bytes;
};

// Validates the host-visible arguments and fills geometry + plan.  `need_budget`: budget_host
// must be present (topk, fused); otherwise it is used when present.  `sel_stride_in` > 0 bounds
// the selected-token estimate for the stand-alone decode.
ABSB_HIDDEN int make_plan(const absb_layer* layer, const absb_batch* batch, bool need_budget,
                          int32_t sel_stride_in, Geometry* geo, Plan* plan);

// Launchers (one per stage); all enqueue on `stream` and return an absb_status.
ABSB_HIDDEN int launch_build(const Geometry& g, const Plan& pl, int dtype, const void* k_cache,
                             const int32_t* page_table, const int32_t* seq_lens, const int32_t* cent_off,
                             uint8_t* codes, float* qscale, float* qmin, char* ws, hipStream_t stream);
ABSB_HIDDEN int launch_score(const Geometry& g, const Plan& pl, int dtype, const void* q, const uint8_t* codes,
                             const float* qscale, const float* qmin, const int32_t* cent_off, const int32_t* seq_lens,
                             int32_t* scores, int32_t* score_exp, hipStream_t stream);
// append == false: only (re)compute the tail state from the cache
ABSB_HIDDEN int launch_append(const Geometry& g, const Plan& pl, int dtype, bool append, const void* k_cache,
                              const int32_t* page_table, const int32_t* seq_lens, const int32_t* cent_off,
                              uint8_t* codes, const float* qscale, const float* qmin, float* tail,
                              int32_t* clamped, hipStream_t stream);
ABSB_HIDDEN int launch_topk(const Geometry& g, const Plan& pl, const int32_t* scores, const int32_t* cent_off,
                            const int32_t* budget, const int32_t* seq_lens, int32_t* sel_idx, int32_t* sel_cnt,
                            int32_t sel_stride,
                            int32_t* tickets, hipStream_t stream);
ABSB_HIDDEN int launch_decode(const Geometry& g, const Plan& pl, int dtype, float sm_scale, const void* q,
                              const void* k_cache, const void* v_cache, const int32_t* page_table,
                              const int32_t* seq_lens, const int32_t* sel_idx, const int32_t* sel_cnt,
                              int32_t sel_stride, void* out, float* lse, char* ws, bool tickets_cleared,
                              hipStream_t stream);

// The whole step in one launch (estimation, selection and attention work-groups in one grid).
ABSB_HIDDEN bool fused_one_launch_fits(const Plan& pl);
ABSB_HIDDEN int launch_fused(const Geometry& g, const Plan& pl, int dtype, float sm_scale, const void* q,
                             const uint8_t* codes, const float* qscale, const float* qmin, const void* k_cache,
                             const void* v_cache, const int32_t* page_table, const int32_t* seq_lens, const int32_t* cent_off,
                             const int32_t* budget, int32_t* sel_idx_out, int32_t* sel_cnt, void* out, float* lse,
                             char* ws, hipStream_t stream);
ABSB_HIDDEN int launch_workspace_init(const Plan& pl, char* ws, hipStream_t stream);
// The whole step in one launch, units of a segment doing score, selection and attention for their own blocks.
ABSB_HIDDEN bool step_fits(const Plan& pl);
ABSB_HIDDEN int launch_step(const Geometry& g, const Plan& pl, int dtype, float sm_scale, const void* q,
                            const uint8_t* codes, const float* qscale, const float* qmin, const void* k_cache,
                            const void* v_cache, const int32_t* page_table, const int32_t* seq_lens, const int32_t* cent_off,
                            const int32_t* budget, int32_t* sel_idx, int32_t* sel_cnt, bool want_list, void* out, float* lse,
                            char* ws, hipStream_t stream);

// How a segment of N blocks in use, K of them to be selected, is cut into units of the one-launch step:
// enough units that each gets about `unit_tokens` selected tokens and scores at most 512 blocks, at
// most ABSB_STEP_MAX_UNITS; a unit's blocks start at a multiple of 32.  Host and device agree on it.
__host__ __device__ inline void step_units(int K, int log2_block, int N, int unit_tokens, int* units, int* unit_blocks) {
  const long long tok = (long long)K << log2_block;
  long long u = (tok + unit_tokens - 1) / unit_tokens;
  const long long by_blocks = ((long long)N + 511) / 512;
  if (u < by_blocks) u = by_blocks;
  if (u < 1) u = 1;
  if (u > ABSB_STEP_MAX_UNITS) u = ABSB_STEP_MAX_UNITS;
  int cb = (int)(((long long)N + u - 1) / u);
  cb = (cb + 31) & ~31;
  if (cb < 32) cb = 32;
  *unit_blocks = cb;
  *units = N > 0 ? (N + cb - 1) / cb : 1;
}

ABSB_HIDDEN int launch_stream_read(const void* src, size_t bytes, uint32_t* sink, int num_cus, hipStream_t stream);

ABSB_HIDDEN int launch_head_recall(const float* lse_sel, const float* lse_all, float* recall, int nseg, int G,
                                   hipStream_t stream);

inline int check_launch() { return hipGetLastError() == hipSuccess ? ABSB_OK : ABSB_ERR_HIP; }

// ------------------------------------------------------------------ device helpers
#ifdef __HIPCC__
// Selection segment t -> request b, selection head hs (first query head = hs * Gd), KV head hk,
// store segment s = b * Hkv + hk, and where the segment's scores start in the score array:
// the Rk selection segments of a store segment lie side by side, Rk * off[s] + (hs % Rk) * rows.
struct SegMap {
  int b, hs, hk, s;
};
__device__ __forceinline__ SegMap seg_map(int t, int Hsel, int Rk, int Hkv) {
  SegMap m;
  m.b = t / Hsel;
  m.hs = t % Hsel;
  m.hk = m.hs / Rk;
  m.s = m.b * Hkv + m.hk;
  return m;
}
__device__ __forceinline__ int64_t score_base(const SegMap& m, int Rk, int off, int rows) {
  return (int64_t)Rk * off + (int64_t)(m.hs % Rk) * rows;
}
// Device-coherent 32-bit accesses for data handed from one work-group to another inside a launch
// (relaxed, agent scope: served past the caches that are not coherent across the chip).  The
// hand-off protocol around them: the writer waits until its stores are acknowledged
// (s_waitcnt vmcnt(0) + work-group barrier), then publishes a counter or flag with a relaxed
// agent-scope atomic; the reader issues its loads only after it has seen that counter or flag.
template <bool COH>
__device__ __forceinline__ int32_t ld_i32(const int32_t* p) {
  if (COH) return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  return *p;
}
template <bool COH>
__device__ __forceinline__ void st_i32(int32_t* p, int32_t v) {
  if (COH)
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  else
    *p = v;
}
__device__ __forceinline__ void wait_stores_acknowledged() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

// K_s = min(N_s, ceil(T_b / B_h)) (Sec. 3.4, kernel 2), never more than the list has room for.
__device__ __forceinline__ int budget_blocks(int T, int log2_block, int blocks, int sel_stride) {
  const int K = (int)(((int64_t)T + (1 << log2_block) - 1) >> log2_block);
  return min(min(K, blocks), sel_stride);
}

// Blocks in use of a segment: all rows of a tight layout (no need to wait for the length then);
// otherwise N_s = ceil(L_b / B_h), never more than the layout has rows for.
__device__ __forceinline__ int blocks_in_use(bool tight, int rows, const int32_t* seq_lens, int b, int log2_block) {
  if (tight) return rows;
  return min(rows, (int)(((int64_t)seq_lens[b] + (1 << log2_block) - 1) >> log2_block));
}

template <typename To, typename From>
__device__ __forceinline__ To bitcast(From v) {
  return __builtin_bit_cast(To, v);
}

typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));

// Element traits of the two storage formats.  A 32-bit word holds two consecutive channels
// (low half = even channel).
template <int DT>
struct Elem;

template <>
struct Elem<ABSB_F16> {
  static __device__ __forceinline__ float dot2(uint32_t a, uint32_t b, float c) {
    return __builtin_amdgcn_fdot2(bitcast<half2_t>(a), bitcast<half2_t>(b), c, false);
  }
  static __device__ __forceinline__ float lo(uint32_t v) { return (float)bitcast<half2_t>(v).x; }
  static __device__ __forceinline__ float hi(uint32_t v) { return (float)bitcast<half2_t>(v).y; }
  static __device__ __forceinline__ float widen(uint16_t v) { return (float)bitcast<_Float16>(v); }
  static __device__ __forceinline__ uint16_t narrow(float f) { return bitcast<uint16_t>((_Float16)f); }
};

template <>
struct Elem<ABSB_BF16> {
  static __device__ __forceinline__ float dot2(uint32_t a, uint32_t b, float c) {
    return __builtin_amdgcn_fdot2_f32_bf16(bitcast<bf16x2_t>(a), bitcast<bf16x2_t>(b), c, false);
  }
  static __device__ __forceinline__ float lo(uint32_t v) { return bitcast<float>(v << 16); }
  static __device__ __forceinline__ float hi(uint32_t v) { return bitcast<float>(v & 0xffff0000u); }
  static __device__ __forceinline__ float widen(uint16_t v) { return bitcast<float>((uint32_t)v << 16); }
  static __device__ __forceinline__ uint16_t narrow(float f) {  // round to nearest, ties to even
    uint32_t u = bitcast<uint32_t>(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40u);  // NaN stays NaN
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
  }
};

// DPP controls (GFX9 encoding).
enum : int {
  DPP_QUAD_XOR1 = 0xB1,        // quad_perm:[1,0,3,2]
  DPP_QUAD_XOR2 = 0x4E,        // quad_perm:[2,3,0,1]
  DPP_ROW_MIRROR = 0x140,      // lane i <- lane 15-i within a row of 16
  DPP_ROW_HALF_MIRROR = 0x141  // lane i <- lane 7-i within a half row of 8
};

template <int CTRL>
__device__ __forceinline__ float dpp_f(float v) {
  return bitcast<float>(__builtin_amdgcn_update_dpp(0, bitcast<int>(v), CTRL, 0xf, 0xf, true));
}
template <int CTRL>
__device__ __forceinline__ int dpp_i(int v) {
  return __builtin_amdgcn_update_dpp(0, v, CTRL, 0xf, 0xf, true);
}

// Sum over the 16 lanes of a DPP row; every lane of the row ends with the same bits.
__device__ __forceinline__ float row16_sum(float v) {
  v += dpp_f<DPP_QUAD_XOR1>(v);
  v += dpp_f<DPP_QUAD_XOR2>(v);
  v += dpp_f<DPP_ROW_HALF_MIRROR>(v);
  v += dpp_f<DPP_ROW_MIRROR>(v);
  return v;
}
__device__ __forceinline__ int quad_sum(int v) {
  v += dpp_i<DPP_QUAD_XOR1>(v);
  v += dpp_i<DPP_QUAD_XOR2>(v);
  return v;
}

// Reductions and scans over a wave built from DPP row operations and four lane reads.  They
// replace ds_bpermute shuffle chains (each shuffle is an LDS-crossbar round trip of >100 cycles).
// All 64 lanes must be active.
template <typename Op>
__device__ __forceinline__ uint32_t row16_reduce_u32(uint32_t v, Op op) {  // every lane of a row gets the row's result
  v = op(v, (uint32_t)dpp_i<DPP_QUAD_XOR1>((int)v));
  v = op(v, (uint32_t)dpp_i<DPP_QUAD_XOR2>((int)v));
  v = op(v, (uint32_t)dpp_i<DPP_ROW_HALF_MIRROR>((int)v));
  v = op(v, (uint32_t)dpp_i<DPP_ROW_MIRROR>((int)v));
  return v;
}
template <typename Op>
__device__ __forceinline__ uint32_t wave_reduce_u32(uint32_t v, Op op) {  // wave-uniform result
  v = row16_reduce_u32(v, op);
  const uint32_t a = (uint32_t)__builtin_amdgcn_readlane((int)v, 0), b = (uint32_t)__builtin_amdgcn_readlane((int)v, 16),
                 c = (uint32_t)__builtin_amdgcn_readlane((int)v, 32), d = (uint32_t)__builtin_amdgcn_readlane((int)v, 48);
  return op(op(a, b), op(c, d));
}
__device__ __forceinline__ float wave_max_f32(float v) {
  v = fmaxf(v, dpp_f<DPP_QUAD_XOR1>(v));
  v = fmaxf(v, dpp_f<DPP_QUAD_XOR2>(v));
  v = fmaxf(v, dpp_f<DPP_ROW_HALF_MIRROR>(v));
  v = fmaxf(v, dpp_f<DPP_ROW_MIRROR>(v));
  const float a = bitcast<float>(__builtin_amdgcn_readlane(bitcast<int>(v), 0)),
              b = bitcast<float>(__builtin_amdgcn_readlane(bitcast<int>(v), 16)),
              c = bitcast<float>(__builtin_amdgcn_readlane(bitcast<int>(v), 32)),
              d = bitcast<float>(__builtin_amdgcn_readlane(bitcast<int>(v), 48));
  return fmaxf(fmaxf(a, b), fmaxf(c, d));
}
// Inclusive prefix sum over the wave in lane order; *total receives the wave's sum.
__device__ __forceinline__ uint32_t wave_incl_scan_u32(uint32_t v, uint32_t* total) {
  v += (uint32_t)dpp_i<0x111>((int)v);  // row_shr:1 (lanes shifted in from outside the row read 0)
  v += (uint32_t)dpp_i<0x112>((int)v);  // row_shr:2
  v += (uint32_t)dpp_i<0x114>((int)v);  // row_shr:4
  v += (uint32_t)dpp_i<0x118>((int)v);  // row_shr:8
  const uint32_t t0 = (uint32_t)__builtin_amdgcn_readlane((int)v, 15), t1 = (uint32_t)__builtin_amdgcn_readlane((int)v, 31),
                 t2 = (uint32_t)__builtin_amdgcn_readlane((int)v, 47), t3 = (uint32_t)__builtin_amdgcn_readlane((int)v, 63);
  const int row = (int)(__builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, 0u)) >> 4);
  v += (row >= 1 ? t0 : 0u) + (row >= 2 ? t1 : 0u) + (row >= 3 ? t2 : 0u);
  *total = t0 + t1 + t2 + t3;
  return v;
}
#endif  // __HIPCC__

}  // namespace absb
