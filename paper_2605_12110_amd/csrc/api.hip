// Host side of libabsb.so: argument validation, size planning, workspace carving and the
// extern "C" entry points.  Nothing here touches the device except through the launchers.
#include <algorithm>
#include <cmath>
#include <mutex>

#include "common.h"

namespace absb {

static inline bool is_pow2(int64_t v) { return v > 0 && (v & (v - 1)) == 0; }
static inline int ilog2(int64_t v) {
  int r = 0;
  while ((int64_t(1) << (r + 1)) <= v) ++r;
  return r;
}
static inline size_t align256(size_t v) { return (v + 255) & ~size_t(255); }
static inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

int make_plan(const absb_layer* layer, const absb_batch* batch, bool need_budget, int32_t sel_stride_in,
              Geometry* geo, Plan* pl) {
  if (!layer || !batch) return ABSB_ERR_NULL;
  if (!layer->block_size || !batch->seq_lens_host) return ABSB_ERR_NULL;
  if (need_budget && !batch->budget_host) return ABSB_ERR_NULL;
  if (layer->head_dim != ABSB_HEAD_DIM) return ABSB_ERR_UNSUPPORTED;
  if (layer->dtype != ABSB_F16 && layer->dtype != ABSB_BF16) return ABSB_ERR_UNSUPPORTED;
  const int Hq = layer->num_q_heads, Hkv = layer->num_kv_heads;
  if (Hq < 1 || Hkv < 1 || Hq % Hkv != 0) return ABSB_ERR_BAD_SHAPE;
  if (Hq / Hkv > ABSB_MAX_GROUP || Hkv > ABSB_MAX_KV_HEADS) return ABSB_ERR_UNSUPPORTED;
  if (layer->block_repr != ABSB_REPR_MEAN && layer->block_repr != ABSB_REPR_MINMAX) return ABSB_ERR_UNSUPPORTED;
  const int P = layer->page_size;
  if (!is_pow2(P) || P < 8 || P > 65536) return ABSB_ERR_BAD_SHAPE;
  const int64_t sp = layer->kv_stride_page, sh = layer->kv_stride_head, st = layer->kv_stride_tok;
  if (sp <= 0 || sh <= 0 || st < ABSB_HEAD_DIM || (sp % 8) || (sh % 8) || (st % 8)) return ABSB_ERR_BAD_SHAPE;
  if (!(layer->sm_scale >= 0.0f) || std::isinf(layer->sm_scale)) return ABSB_ERR_BAD_SHAPE;
  if (layer->sink_tokens < 0 || layer->recent_tokens < 0) return ABSB_ERR_BAD_SHAPE;
  if (layer->selection != ABSB_SELECT_GROUP && layer->selection != ABSB_SELECT_PER_QUERY_HEAD &&
      layer->selection != ABSB_SELECT_GROUP_MAX)
    return ABSB_ERR_UNSUPPORTED;
  if (layer->selection == ABSB_SELECT_GROUP_MAX && layer->block_repr != ABSB_REPR_MEAN) return ABSB_ERR_UNSUPPORTED;
  const bool per_q = layer->selection == ABSB_SELECT_PER_QUERY_HEAD;
  const int Hsel = per_q ? Hq : Hkv;
  const int Bt = batch->batch;
  if (Bt < 1 || (int64_t)Bt * Hsel > 65535) return ABSB_ERR_BAD_SHAPE;  // segments index grid.y

  Geometry g = {};
  g.Bt = Bt;
  g.Hq = Hq;
  g.Hkv = Hkv;
  g.G = Hq / Hkv;
  g.Hsel = Hsel;
  g.Gd = per_q ? 1 : g.G;
  g.Rk = per_q ? g.G : 1;
  g.agg_max = layer->selection == ABSB_SELECT_GROUP_MAX;
  g.log2_page = ilog2(P);
  g.pt_stride = batch->pt_stride;
  g.repr = layer->block_repr;
  g.tight = batch->cap_lens_host ? 0 : 1;
  g.sink_tokens = layer->sink_tokens;
  g.recent_tokens = layer->recent_tokens;
  g.s_page = sp;
  g.s_head = sh;
  g.s_tok = st;
  for (int h = 0; h < Hkv; ++h) {
    const int B = layer->block_size[h];
    if (!is_pow2(B) || B < 8 || B > 128) return ABSB_ERR_BAD_BLOCK_SIZE;
    // both are powers of two, so B | P or P | B holds: blocks never straddle a page partially
    g.heads.log2_block[h] = (uint8_t)ilog2(B);
  }

  Plan p = {};
  // selected tokens a unit of the one-launch step should get: two attention steps at batch 1; large
  // batches, whose work-groups queue for the compute units anyway, do better with longer units
  int64_t budget_tokens = 0;
  if (batch->budget_host)
    for (int b = 0; b < Bt; ++b) budget_tokens += (int64_t)std::min(batch->budget_host[b], batch->seq_lens_host[b]) * Hsel;
  const absb_launch_opts& opts = batch->opts;
  if (opts.step_form < ABSB_STEP_AUTO || opts.step_form > ABSB_STEP_PER_STAGE) return ABSB_ERR_BAD_SHAPE;
  if (opts.split_tokens < 0 || opts.split_tokens % 64 || opts.score_chunk < 0 || opts.score_chunk % 64 ||
      opts.unit_tokens < 0 || opts.unit_tokens % 64 || opts.counters_zero < 0 || opts.counters_zero > 1)
    return ABSB_ERR_BAD_SHAPE;
  int unit_tokens = opts.unit_tokens;
  if (unit_tokens <= 0) unit_tokens = budget_tokens >= 131072 ? 256 : 128;
  p.unit_tokens = unit_tokens;
  p.units_max = 1;
  p.nseg = Bt * Hsel;
  p.nstore = Bt * Hkv;
  p.build_chunk_tokens = 1024;
  int64_t max_len = 0;
  for (int b = 0; b < Bt; ++b) {
    const int64_t L = batch->seq_lens_host[b];
    if (L < 1) return ABSB_ERR_BAD_SHAPE;
    const int64_t cap = batch->cap_lens_host ? batch->cap_lens_host[b] : L;  // the layout's length
    if (cap < L) return ABSB_ERR_BAD_SHAPE;
    if (L > max_len) max_len = L;
    if (batch->budget_host && batch->budget_host[b] < 1) return ABSB_ERR_BAD_SHAPE;
    for (int h = 0; h < Hkv; ++h) {
      const int64_t B = layer->block_size[h];
      const int64_t N = ceil_div(L, B);
      int64_t K = N;
      if (batch->budget_host) {
        const int64_t kb = ceil_div(batch->budget_host[b], B);
        if (kb < K) K = kb;
        if (K > p.sel_stride) p.sel_stride = (int32_t)K;
      }
      if (sel_stride_in > 0 && sel_stride_in < K) K = sel_stride_in;
      p.total += ceil_div(cap, B);
      const int64_t cb = std::max<int64_t>(16, p.build_chunk_tokens / B);  // as build_chunk_blocks() on the device
      if (ceil_div(N, cb) > p.build_max_chunks) p.build_max_chunks = (int32_t)ceil_div(N, cb);
      if (N > p.max_blocks) p.max_blocks = (int32_t)N;
      const int64_t tok = K * B;
      {
        int su = 1, sb = 32;
        step_units((int)K, g.heads.log2_block[h], (int)N, unit_tokens, &su, &sb);
        if (su > p.units_max) p.units_max = su;
      }
      if (tok > p.max_tokens) p.max_tokens = tok;
      p.sum_tokens += tok * g.Rk;  // every selection segment of the KV head reads its own tokens
    }
  }
  if (!batch->budget_host) p.sel_stride = p.max_blocks;
  // entry points that select (they are the ones that need the budgets) refuse on the host what the
  // selection cannot hold, before anything is enqueued
  if (need_budget && p.max_blocks > ABSB_MAX_SEL_BLOCKS) return ABSB_ERR_UNSUPPORTED;
  if (p.total >= (int64_t(1) << 31) - 1) return ABSB_ERR_BAD_SHAPE;
  if ((int64_t)batch->pt_stride < ceil_div(max_len, P)) return ABSB_ERR_BAD_SHAPE;

  // How absb_decode_fused is enqueued.  Measured on MI355X with cold caches (every step on a copy
  // of the layer that the last-level cache has forgotten): the pipelined one-launch step wins by
  // 6-12 % (config 1: 16.6 against 18.9 us, config 2: 30.5 / 32.6, config 3: 22.2 / 24.3, config 4:
  // 52.5 / 56.5) wherever no segment is longer than 16384 blocks, the longest register tile of its
  // 256-thread selection; beyond (keys re-read) that selection takes several times longer (69 against
  // 36 us at 256K context).  Very long lists (budgets near the context) go to the per-stage path: its
  // attention kernel reads the lists through the L2.
  const bool by_shape = p.max_blocks <= 16384 && p.sel_stride <= 4096;
  // Segments beyond 16384 blocks: there the selection by one work-group costs more than everything
  // else together (measured at 256K context: 35.9 us per stage against 31.4 us),
  // and the step runs as units that select among themselves, as long as the chip holds all of a
  // batch's units at once (two work-groups per compute unit).
  const bool by_units = !by_shape && p.max_blocks > 16384 && (int64_t)p.nseg * (p.units_max + 1) <= 480;
  p.step_form = opts.step_form != ABSB_STEP_AUTO ? opts.step_form
                : by_shape ? ABSB_STEP_PIPELINED : by_units ? ABSB_STEP_UNITS : ABSB_STEP_PER_STAGE;
  p.one_launch = p.step_form != ABSB_STEP_PER_STAGE;
  p.bitmap_words = (p.max_blocks + 31) / 32;
  // split-K shape, in 64-token granules (one work-group step).  Measured on MI355X (256 CUs, three
  // resident work-groups each): the kernel is fastest with about two work-groups per CU, all
  // resident at once and each streaming as long as possible; a work-group needs at least two steps
  // to amortise its set-up; and since one work-group merges a segment's partials, a segment should
  // not be cut into more than 64.
  // (the shape follows the batch, not the enqueue knob: every form of the step then cuts the
  // segments alike and gives the same bits)
  int st_tok = opts.split_tokens;
  if (st_tok <= 0) {
    const int64_t target_wgs = 640;
    int64_t t = ceil_div(ceil_div(p.sum_tokens, target_wgs), 64) * 64;
    if (t < 128) t = p.sum_tokens / 128 >= 128 ? 128 : 64;  // one step only when two would leave the chip idle
    // In the one-launch step the attention work-groups of a large batch start segment by segment as
    // the lists come out, not all at once: sweeps there favour ~1100 work-groups of at least four
    // steps (config 4 43.5 -> 42.0 us, config 5 at budget 8192 41.4 -> 39.2).
    if (by_shape && batch->budget_host && p.sum_tokens >= 65536)
      t = std::max<int64_t>(256, ceil_div(ceil_div(p.sum_tokens, 1100), 64) * 64);
    const int64_t cap_tok = ceil_div(ceil_div(p.max_tokens, 64), 64) * 64;
    if (t < cap_tok) t = cap_tok;
    st_tok = (int)t;
  }
  p.split_tokens = st_tok;
  p.max_splits = (int32_t)ceil_div(p.max_tokens, st_tok);
  if (p.max_splits < 1) p.max_splits = 1;
  if (p.max_splits > 65535) return ABSB_ERR_BAD_SHAPE;
  if ((int64_t)p.max_splits * st_tok >= (int64_t(1) << 31)) return ABSB_ERR_BAD_SHAPE;  // positions are 32-bit

  // blocks per estimation work-group: 256 (one batch of loads per lane); in the one-launch step,
  // where estimation work-groups share the CUs with attention work-groups, a large batch does
  // better with two batches per work-group (the prologue is amortised, half as many work-groups)
  int sc = opts.score_chunk;
  p.score_chunk = sc > 0 ? sc : (p.one_launch && p.total >= 65536 ? 512 : 256);

  // workspace: the split counters of the attention kernel come first, at the same place in every
  // carving (nothing else ever writes there); behind them the three users overlap, since they
  // never run concurrently on one workspace
  p.ws_tickets = 0;
  const size_t ctr = align256((size_t)p.nseg * ABSB_TICKET_STRIDE * 4);
  p.ws_score_tickets = ctr;
  p.ws_flags = 2 * ctr;
  p.ws_status = 3 * ctr;
  p.ws_cand_done = 3 * ctr + 256;
  p.ws_listed = 4 * ctr + 256;
  p.ws_cutoff = 5 * ctr + 256;
  const size_t head = 6 * ctr + 256;
  p.ws_head_bytes = head;
  size_t o = head;
  p.ws_scores = o;
  o += align256((size_t)p.total * g.Rk * 4);
  p.ws_sel_idx = o;
  o += align256((size_t)p.nseg * (size_t)(p.sel_stride > 0 ? p.sel_stride : 1) * 4);
  p.ws_sel_cnt = o;
  o += align256((size_t)p.nseg * 4);
  const size_t fused_head = o;
  p.ws_part_o = o;
  o += align256((size_t)p.nseg * p.max_splits * g.Gd * ABSB_HEAD_DIM * 4);
  p.ws_part_ml = o;
  o += align256((size_t)p.nseg * p.max_splits * g.Gd * 4 * 4);  // (max, rounded sum, exact sum, -) per split and head
  p.ws_decode_bytes = o;  // the stand-alone decode uses the same offsets (the head is left unused)
  // the unit form of the one-launch step: histogram rows, candidates, bitmaps, one partial per unit
  p.ws_rows = o;
  o += align256((size_t)p.nseg * p.units_max * 256 * 2);
  p.ws_cand = o;
  o += align256((size_t)p.total * g.Rk * 8);
  p.ws_bitmap = o;
  o += align256((size_t)p.nseg * p.bitmap_words * 4);
  p.ws_unit_o = o;
  o += align256((size_t)p.nseg * p.units_max * g.Gd * ABSB_HEAD_DIM * 4);
  p.ws_unit_ml = o;
  o += align256((size_t)p.nseg * p.units_max * g.Gd * 4 * 4);
  p.ws_fused_bytes = o;
  (void)fused_head;
  size_t bo = head;
  p.ws_cent = bo;
  const size_t width = (size_t)ABSB_HEAD_DIM * (g.repr + 1);  // values per block
  bo += align256((size_t)p.total * width * 4);
  p.ws_minmax = bo;
  bo += align256((size_t)p.nstore * p.build_max_chunks * 2 * width * 4);
  p.ws_qinv = bo;
  bo += align256((size_t)p.nstore * width * 4);
  p.ws_build_bytes = bo;
  p.ws_bytes = p.ws_fused_bytes > p.ws_build_bytes ? p.ws_fused_bytes : p.ws_build_bytes;

  if (geo) *geo = g;
  if (pl) *pl = p;
  return ABSB_OK;
}

static int check_ws(const void* ws, size_t have, size_t need) {
  if (need == 0) return ABSB_OK;
  if (!ws || (reinterpret_cast<uintptr_t>(ws) & 255) || have < need) return ABSB_ERR_WORKSPACE;
  return ABSB_OK;
}

static float resolve_scale(const absb_layer* layer) {
  return layer->sm_scale > 0.0f ? layer->sm_scale : 1.0f / std::sqrt((float)layer->head_dim);
}

}  // namespace absb

using namespace absb;

extern "C" {

int absb_plan(const absb_layer* layer, const absb_batch* batch, int32_t* cent_off_host,
              int64_t* total_centroids, int32_t* sel_stride, size_t* workspace_bytes) {
  Geometry g;
  Plan p;
  int rc = make_plan(layer, batch, false, 0, &g, &p);
  if (rc != ABSB_OK) return rc;
  if (cent_off_host) {
    int32_t acc = 0;
    cent_off_host[0] = 0;
    for (int b = 0; b < g.Bt; ++b)
      for (int h = 0; h < g.Hkv; ++h) {
        const int64_t B = layer->block_size[h];
        const int64_t cap = batch->cap_lens_host ? batch->cap_lens_host[b] : batch->seq_lens_host[b];
        acc += (int32_t)((cap + B - 1) / B);
        cent_off_host[b * g.Hkv + h + 1] = acc;
      }
  }
  if (total_centroids) *total_centroids = p.total;
  if (sel_stride) *sel_stride = p.sel_stride;
  if (workspace_bytes) *workspace_bytes = p.ws_bytes;
  return ABSB_OK;
}

int absb_build_centroids(const absb_layer* layer, const absb_batch* batch, const void* k_cache, uint8_t* codes,
                         float* qscale, float* qmin, void* workspace, size_t workspace_bytes, void* stream) {
  Geometry g;
  Plan p;
  int rc = make_plan(layer, batch, false, 0, &g, &p);
  if (rc != ABSB_OK) return rc;
  if (!k_cache || !codes || !qscale || !qmin || !batch->seq_lens || !batch->page_table || !batch->cent_off)
    return ABSB_ERR_NULL;
  rc = check_ws(workspace, workspace_bytes, p.ws_build_bytes);
  if (rc != ABSB_OK) return rc;
  return launch_build(g, p, layer->dtype, k_cache, batch->page_table, batch->seq_lens, batch->cent_off, codes,
                      qscale, qmin, static_cast<char*>(workspace), static_cast<hipStream_t>(stream));
}

int absb_score(const absb_layer* layer, const absb_batch* batch, const void* q, const uint8_t* codes,
               const float* qscale, int32_t* scores, int32_t* score_exp, void* stream) {
  Geometry g;
  Plan p;
  int rc = make_plan(layer, batch, false, 0, &g, &p);
  if (rc != ABSB_OK) return rc;
  if (!q || !codes || !qscale || !scores || !batch->cent_off || !batch->seq_lens) return ABSB_ERR_NULL;
  if (g.agg_max && !batch->qmin) return ABSB_ERR_NULL;
  return launch_score(g, p, layer->dtype, q, codes, qscale, batch->qmin, batch->cent_off, batch->seq_lens, scores, score_exp,
                      static_cast<hipStream_t>(stream));
}

int absb_topk(const absb_layer* layer, const absb_batch* batch, const int32_t* scores, int32_t* sel_idx,
              int32_t* sel_cnt, int32_t sel_stride, void* workspace, size_t workspace_bytes, void* stream) {
  (void)workspace;
  (void)workspace_bytes;  // the selection needs no scratch memory
  Geometry g;
  Plan p;
  int rc = make_plan(layer, batch, true, 0, &g, &p);
  if (rc != ABSB_OK) return rc;
  if (!scores || !sel_idx || !sel_cnt || !batch->cent_off || !batch->budget) return ABSB_ERR_NULL;
  if (!batch->seq_lens) return ABSB_ERR_NULL;
  if (sel_stride < p.sel_stride) return ABSB_ERR_BAD_SHAPE;
  return launch_topk(g, p, scores, batch->cent_off, batch->budget, batch->seq_lens, sel_idx, sel_cnt, sel_stride, nullptr,
                     static_cast<hipStream_t>(stream));
}

int absb_sparse_decode(const absb_layer* layer, const absb_batch* batch, const void* q, const void* k_cache,
                       const void* v_cache, const int32_t* sel_idx, const int32_t* sel_cnt, int32_t sel_stride,
                       void* out, float* lse, void* workspace, size_t workspace_bytes, void* stream) {
  if (sel_stride < 1) return layer && batch ? ABSB_ERR_BAD_SHAPE : ABSB_ERR_NULL;
  Geometry g;
  Plan p;
  int rc = make_plan(layer, batch, false, sel_stride, &g, &p);
  if (rc != ABSB_OK) return rc;
  if (!q || !k_cache || !v_cache || !sel_idx || !sel_cnt || !out || !batch->seq_lens || !batch->page_table)
    return ABSB_ERR_NULL;
  rc = check_ws(workspace, workspace_bytes, p.ws_decode_bytes);
  if (rc != ABSB_OK) return rc;
  return launch_decode(g, p, layer->dtype, resolve_scale(layer), q, k_cache, v_cache, batch->page_table,
                       batch->seq_lens, sel_idx, sel_cnt, sel_stride, out, lse, static_cast<char*>(workspace),
                       batch->opts.counters_zero == 1, static_cast<hipStream_t>(stream));
}

int absb_decode_fused(const absb_layer* layer, const absb_batch* batch, const void* q, const uint8_t* codes,
                      const float* qscale, const void* k_cache, const void* v_cache, void* out, float* lse,
                      int32_t* sel_idx_out, int32_t* sel_cnt_out, void* workspace, size_t workspace_bytes,
                      void* stream) {
  Geometry g;
  Plan p;
  int rc = make_plan(layer, batch, true, 0, &g, &p);
  if (rc != ABSB_OK) return rc;
  if (!q || !codes || !qscale || !k_cache || !v_cache || !out || !batch->seq_lens || !batch->page_table ||
      !batch->cent_off || !batch->budget)
    return ABSB_ERR_NULL;
  if (g.agg_max && !batch->qmin) return ABSB_ERR_NULL;
  rc = check_ws(workspace, workspace_bytes, p.ws_fused_bytes);
  if (rc != ABSB_OK) return rc;
  char* ws = static_cast<char*>(workspace);
  hipStream_t st = static_cast<hipStream_t>(stream);
  int32_t* scores = reinterpret_cast<int32_t*>(ws + p.ws_scores);
  int32_t* sel_idx = sel_idx_out ? sel_idx_out : reinterpret_cast<int32_t*>(ws + p.ws_sel_idx);
  int32_t* sel_cnt = sel_cnt_out ? sel_cnt_out : reinterpret_cast<int32_t*>(ws + p.ws_sel_cnt);
  if (p.step_form == ABSB_STEP_UNITS && step_fits(p))
    return launch_step(g, p, layer->dtype, resolve_scale(layer), q, codes, qscale, batch->qmin, k_cache, v_cache,
                       batch->page_table, batch->seq_lens, batch->cent_off, batch->budget, sel_idx, sel_cnt,
                       sel_idx_out != nullptr, out, lse, ws, st);
  if (p.step_form == ABSB_STEP_PIPELINED && fused_one_launch_fits(p))
    return launch_fused(g, p, layer->dtype, resolve_scale(layer), q, codes, qscale, batch->qmin, k_cache, v_cache, batch->page_table,
                        batch->seq_lens, batch->cent_off, batch->budget, sel_idx_out, sel_cnt, out, lse, ws, st);
  rc = launch_score(g, p, layer->dtype, q, codes, qscale, batch->qmin, batch->cent_off, batch->seq_lens, scores, nullptr, st);
  if (rc != ABSB_OK) return rc;
  // the selection kernel also clears the split counters of the attention kernel behind it
  rc = launch_topk(g, p, scores, batch->cent_off, batch->budget, batch->seq_lens, sel_idx, sel_cnt, p.sel_stride,
                   reinterpret_cast<int32_t*>(ws + p.ws_tickets), st);
  if (rc != ABSB_OK) return rc;
  return launch_decode(g, p, layer->dtype, resolve_scale(layer), q, k_cache, v_cache, batch->page_table,
                       batch->seq_lens, sel_idx, sel_cnt, p.sel_stride, out, lse, ws, true, st);
}

int absb_step_form_used(const absb_layer* layer, const absb_batch* batch) {
  Geometry g;
  Plan p;
  int rc = make_plan(layer, batch, true, 0, &g, &p);
  if (rc != ABSB_OK) return rc;
  if (p.step_form == ABSB_STEP_UNITS && step_fits(p)) return ABSB_STEP_UNITS;
  if (p.step_form == ABSB_STEP_PIPELINED && fused_one_launch_fits(p)) return ABSB_STEP_PIPELINED;
  return ABSB_STEP_PER_STAGE;
}

int absb_status_offset(const absb_layer* layer, const absb_batch* batch, size_t* offset) {
  Geometry g;
  Plan p;
  int rc = make_plan(layer, batch, false, 0, &g, &p);
  if (rc != ABSB_OK) return rc;
  if (!offset) return ABSB_ERR_NULL;
  *offset = p.ws_status;
  return ABSB_OK;
}

int absb_workspace_init(const absb_layer* layer, const absb_batch* batch, void* workspace, size_t workspace_bytes,
                        void* stream) {
  Geometry g;
  Plan p;
  int rc = make_plan(layer, batch, false, 0, &g, &p);
  if (rc != ABSB_OK) return rc;
  rc = check_ws(workspace, workspace_bytes, p.ws_head_bytes);
  if (rc != ABSB_OK) return rc;
  return launch_workspace_init(p, static_cast<char*>(workspace), static_cast<hipStream_t>(stream));
}

int absb_tail_init(const absb_layer* layer, const absb_batch* batch, const void* k_cache, float* tail, void* stream) {
  Geometry g;
  Plan p;
  int rc = make_plan(layer, batch, false, 0, &g, &p);
  if (rc != ABSB_OK) return rc;
  if (!k_cache || !tail || !batch->seq_lens || !batch->page_table) return ABSB_ERR_NULL;
  return launch_append(g, p, layer->dtype, false, k_cache, batch->page_table, batch->seq_lens, nullptr, nullptr,
                       nullptr, nullptr, tail, nullptr, static_cast<hipStream_t>(stream));
}

int absb_append_token(const absb_layer* layer, const absb_batch* batch, const void* k_cache, uint8_t* codes,
                      const float* qscale, const float* qmin, float* tail, int32_t* clamped, void* stream) {
  Geometry g;
  Plan p;
  int rc = make_plan(layer, batch, false, 0, &g, &p);
  if (rc != ABSB_OK) return rc;
  if (!k_cache || !codes || !qscale || !qmin || !tail || !batch->seq_lens || !batch->page_table || !batch->cent_off)
    return ABSB_ERR_NULL;
  return launch_append(g, p, layer->dtype, true, k_cache, batch->page_table, batch->seq_lens, batch->cent_off, codes,
                       qscale, qmin, tail, clamped, static_cast<hipStream_t>(stream));
}

int absb_head_recall(const absb_layer* layer, const absb_batch* batch, const float* lse_selected,
                     const float* lse_dense, float* recall, void* stream) {
  Geometry g;
  Plan p;
  int rc = make_plan(layer, batch, false, 0, &g, &p);
  if (rc != ABSB_OK) return rc;
  if (!lse_selected || !lse_dense || !recall) return ABSB_ERR_NULL;
  return launch_head_recall(lse_selected, lse_dense, recall, p.nstore, g.G, static_cast<hipStream_t>(stream));
}

int absb_assign_block_sizes(int32_t n_samples, int32_t n_heads, int32_t n_cand, const float* recall_host,
                            const int32_t* cand, double tau, int32_t* block_size_out, double* mean_out) {
  if (!recall_host || !cand || !block_size_out) return ABSB_ERR_NULL;
  if (n_samples < 1 || n_heads < 1 || n_cand < 1 || n_cand > 64 || !(tau >= 0.0)) return ABSB_ERR_BAD_SHAPE;
  if (!is_pow2(cand[0]) || cand[0] < 8 || cand[0] > 128) return ABSB_ERR_BAD_BLOCK_SIZE;
  for (int k = 1; k < n_cand; ++k) {
    if (!is_pow2(cand[k]) || cand[k] > 128) return ABSB_ERR_BAD_BLOCK_SIZE;
    if (cand[k] <= cand[k - 1]) return ABSB_ERR_BAD_SHAPE;
  }
  // Eq. (2), head by head.  First Recall(h, B) for every candidate: the mean over the samples (which
  // are whatever the caller measured recall on: one row per request of every calibration input),
  // accumulated in binary64 in sample order.  Then the candidates are tried from the largest down:
  // the set {B : Recall(h, B) >= tau * Recall(h, B_min)} is read as written, so the first one that
  // passes is its maximum, whatever the candidates below it do; B_min is in the set for tau <= 1 and
  // is the answer when nothing passes.
  const size_t row = (size_t)n_heads * n_cand;
  for (int h = 0; h < n_heads; ++h) {
    double recall_of[64];
    for (int k = 0; k < n_cand; ++k) recall_of[k] = 0.0;
    const float* sample = recall_host + (size_t)h * n_cand;
    for (int i = 0; i < n_samples; ++i, sample += row)
      for (int k = 0; k < n_cand; ++k) recall_of[k] += (double)sample[k];
    for (int k = 0; k < n_cand; ++k) {
      recall_of[k] /= (double)n_samples;
      if (mean_out) mean_out[(size_t)h * n_cand + k] = recall_of[k];
    }
    const double floor_of_head = tau * recall_of[0];
    int chosen = n_cand - 1;
    while (chosen > 0 && !(recall_of[chosen] >= floor_of_head)) --chosen;
    block_size_out[h] = cand[chosen];
  }
  return ABSB_OK;
}

int absb_stream_read(const void* src, size_t bytes, void* sink, void* stream) {
  if (!src || !sink) return ABSB_ERR_NULL;
  if (reinterpret_cast<uintptr_t>(src) & 15) return ABSB_ERR_BAD_SHAPE;
  int dev = 0, cus = 0;
  if (hipGetDevice(&dev) != hipSuccess ||
      hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1)
    return ABSB_ERR_HIP;
  return launch_stream_read(src, bytes, static_cast<uint32_t*>(sink), cus, static_cast<hipStream_t>(stream));
}

const char* absb_strerror(int status) {
  switch (status) {
    case ABSB_OK: return "ok";
    case ABSB_ERR_NULL: return "a required pointer is NULL";
    case ABSB_ERR_BAD_SHAPE: return "invalid shape, length, stride, budget or list width";
    case ABSB_ERR_BAD_BLOCK_SIZE: return "block size must be a power of two in [8,128]";
    case ABSB_ERR_UNSUPPORTED: return "unsupported configuration (head_dim, group size, head count or dtype)";
    case ABSB_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
    case ABSB_ERR_HIP: return "HIP launch failed";
    case ABSB_ERR_STATIC_WORKSPACE:
      return "the batch needs more scratch memory than the library's built-in array holds (ABSB_STATIC_WORKSPACE_BYTES); "
             "use absb_decode_fused with a workspace of the caller's";
    default: return "unknown status";
  }
}

}  // extern "C"

// ------------------------------------------------------------------ the step for callers that cannot allocate
//
// absb_decode_fused with the workspace taken from device memory that the library's code object
// holds: a file-scope array, one copy per GPU, there from the moment the library is loaded on that
// GPU until the process ends.  Nothing is allocated or freed by the call, by the library or by any
// runtime routine it uses.
namespace absb {

static __device__ __align__(256) unsigned char scratch[ABSB_STATIC_WORKSPACE_BYTES];

constexpr int kMaxDevices = 64;
struct StaticWorkspace {
  char* ptr = nullptr;        // this device's copy of `scratch` (a device address; the array's name is not one)
  size_t head_bytes = 0;      // counters cleared for a batch shape whose counters take this many bytes
};
static StaticWorkspace g_static_ws[kMaxDevices];
static std::mutex g_static_ws_lock;

// Device address of the current device's scratch array, resolved once per device.
static int static_workspace(int* dev_out, StaticWorkspace** slot) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return ABSB_ERR_HIP;
  StaticWorkspace& w = g_static_ws[dev];
  if (!w.ptr) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return ABSB_ERR_HIP;
    w.ptr = static_cast<char*>(p);
    w.head_bytes = 0;
  }
  *dev_out = dev;
  *slot = &w;
  return ABSB_OK;
}

}  // namespace absb

extern "C" {

int absb_decode_fused_static(const absb_layer* layer, const absb_batch* batch, const void* q, const uint8_t* codes,
                             const float* qscale, const void* k_cache, const void* v_cache, void* out, float* lse,
                             int32_t* sel_idx_out, int32_t* sel_cnt_out, void* stream) {
  Geometry g;
  Plan p;
  int rc = make_plan(layer, batch, true, 0, &g, &p);
  if (rc != ABSB_OK) return rc;
  if (p.ws_fused_bytes > (size_t)ABSB_STATIC_WORKSPACE_BYTES) return ABSB_ERR_STATIC_WORKSPACE;
  std::lock_guard<std::mutex> hold(g_static_ws_lock);
  int dev = 0;
  StaticWorkspace* w = nullptr;
  rc = static_workspace(&dev, &w);
  if (rc != ABSB_OK) return rc;
  // The array keeps what the last call left.  The counters at its start are zero after every
  // completed step, but where they sit follows the batch shape: a first call on this device, or a
  // call whose counters take a different number of bytes than the last one's, clears them first
  // (a small fill kernel on the caller's stream, ordered before the step).
  if (w->head_bytes != p.ws_head_bytes) {
    rc = launch_workspace_init(p, w->ptr, static_cast<hipStream_t>(stream));
    if (rc != ABSB_OK) return rc;
    w->head_bytes = p.ws_head_bytes;
  }
  return absb_decode_fused(layer, batch, q, codes, qscale, k_cache, v_cache, out, lse, sel_idx_out, sel_cnt_out, w->ptr,
                           (size_t)ABSB_STATIC_WORKSPACE_BYTES, stream);
}

}  // extern "C"
