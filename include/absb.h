/*
 * absb - adaptive-block sparse decode attention for AMD MI355X (gfx950).
 *
 * C ABI of libabsb.so.  The library implements the decode-step hot path of AB-Sparse:
 * block-sparse attention in which every KV head has its own block size B_h.
 *
 *   build  : block centroids (mean pooling, Sec. 2.2) quantized to INT4, asymmetric,
 *            one scale and one zero-point offset per head-dim channel (Sec. 3.3),
 *            stored in a flattened 1-D array delimited by prefix sums (Sec. 3.4, kernel 1)
 *   score  : importance of every block, r_j = q . c_j^T (Sec. 2.2), dequantization fused,
 *            all heads of all requests in one launch (Sec. 3.4, kernel 1)
 *   topk   : per head the K_h = ceil(T / B_h) best blocks under a token budget T
 *            (Sec. 3.4, kernel 2)
 *   decode : softmax attention, Eq. (1), over the selected blocks only, read in place
 *            from a paged KV cache through the page table (Sec. 3.4, kernel 3), as
 *            split-K partials merged by log-sum-exp
 *
 * Conventions
 *   - Every function returns ABSB_OK (0) or a negative absb_status.  No exceptions, no exit.
 *   - Host-visible arguments are validated before anything is launched; on error nothing
 *     has been enqueued.
 *   - All device work is enqueued on the caller's stream (`stream` is a hipStream_t passed
 *     as void*; NULL = the default stream).  No call synchronises, allocates or frees.
 *   - The caller owns every buffer.  Pointers are DEVICE pointers unless the comment says
 *     "host".  Host arrays are read during the call only.  Device buffers must stay valid
 *     until the enqueued work has finished.
 *   - Contents of device arrays (page indices, lengths, selected indices) are trusted:
 *     out-of-range values are undefined behaviour.  The device copies `seq_lens`/`budget`
 *     must hold the same values as their host twins.
 *   - One segment per (request b, KV head h): s = b*num_kv_heads + h, request-major.  The
 *     G = num_q_heads/num_kv_heads query heads of a KV head share its blocks and its
 *     selection; their scores are summed (the score is linear in q).
 *   - Workspace: `absb_plan` reports the size that suffices for every entry point on that
 *     (layer, batch); 256-byte aligned.  Its first bytes hold the counters through which the
 *     work-groups of absb_decode_fused hand work to each other: they must be zero when that
 *     call starts.  absb_workspace_init clears them (a workspace allocated zero-filled needs no
 *     call), and every entry point leaves them zero.  Where they sit depends on the number of
 *     selection segments of the batch, and the other stages' data lies right behind them: when a
 *     workspace is reused for a batch with a different number of segments (requests joining or
 *     leaving), call absb_workspace_init again (one small launch), or keep a workspace per batch
 *     shape.  Nothing else in the workspace needs initialisation or survives a call.  Calls that
 *     share a workspace must be ordered on one stream.
 *   - Limits: at most 65535 selection segments per batch (ABSB_ERR_BAD_SHAPE beyond); the selection
 *     (absb_topk, absb_decode_fused) holds at most 2^17 blocks per segment (ABSB_ERR_UNSUPPORTED
 *     beyond: 1 Mi tokens at B_h = 8, 16 Mi at B_h = 128); fewer than 2^31 blocks in all.
 */
#ifndef ABSB_H
#define ABSB_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#if defined(__GNUC__)
#define ABSB_API __attribute__((visibility("default")))
#else
#define ABSB_API
#endif

typedef enum absb_dtype { ABSB_F16 = 0, ABSB_BF16 = 1 } absb_dtype;

/* How a block of keys is represented for the estimation stage (Sec. 2.2, footnote on pooling):
 *   ABSB_REPR_MEAN   : the mean of the block's keys, scored by q . c^T (the paper's running example);
 *   ABSB_REPR_MINMAX : the channel-wise maxima and minima of the block's keys (the max-min pooling
 *                      of the baseline the paper's evaluation builds on, Sec. 4.1), scored by the
 *                      channel-wise upper bound sum_c max(q_c * max_c, q_c * min_c) of q . k.
 * R below is the number of vectors per block: 1 for MEAN, 2 for MINMAX (maxima first). */
typedef enum absb_repr { ABSB_REPR_MEAN = 0, ABSB_REPR_MINMAX = 1 } absb_repr;

/* Who shares a selection (the paper selects "per head" and leaves grouped-query models open):
 *   ABSB_SELECT_GROUP          : one selection per (request, KV head), shared by its G query heads,
 *                                ranked by the sum of their scores; K and V rows are read once per
 *                                KV head.  The default.
 *   ABSB_SELECT_PER_QUERY_HEAD : one selection per (request, query head), ranked by that head's own
 *                                score; every query head reads the K and V rows of its own list
 *                                (G times the traffic).  The centroid store stays one per KV head.
 *   ABSB_SELECT_GROUP_MAX      : as GROUP, but ranked by the maximum over the group's query heads of
 *                                q_g . c^ (the dequantized centroid) instead of their sum.  Comparing
 *                                heads needs each head's zero-point term sum_c q_g[c]*qmin[c]: the
 *                                score stage then reads batch->qmin.  Mean pooling only.
 * Below, a "selection segment" is t = b*Hsel + hs with Hsel = Hkv (GROUP) or Hq (PER_QUERY_HEAD);
 * with PER_QUERY_HEAD hs is the query head, its KV head is hs / G, and everything the default mode
 * does for a KV head and its group is done for the query head alone. */
typedef enum absb_select {
  ABSB_SELECT_GROUP = 0,
  ABSB_SELECT_PER_QUERY_HEAD = 1,
  ABSB_SELECT_GROUP_MAX = 2
} absb_select;

typedef enum absb_status {
  ABSB_OK = 0,
  ABSB_ERR_NULL = -1,           /* a required pointer is NULL                                   */
  ABSB_ERR_BAD_SHAPE = -2,      /* head counts, lengths, strides, budgets or list width invalid */
  ABSB_ERR_BAD_BLOCK_SIZE = -3, /* block size not a power of two in [8,128], or not nesting with
                                   the page size                                                */
  ABSB_ERR_UNSUPPORTED = -4,    /* head_dim != 128, group size > 8, more than 64 KV heads, dtype */
  ABSB_ERR_WORKSPACE = -5,      /* workspace NULL, misaligned or smaller than absb_plan reports  */
  ABSB_ERR_HIP = -6,            /* a HIP launch failed (see hipGetLastError)                     */
  ABSB_ERR_STATIC_WORKSPACE = -7 /* absb_decode_fused_static: the batch needs more scratch memory
                                   than the library's built-in array (ABSB_STATIC_WORKSPACE_BYTES) */
} absb_status;

/* Static description of one attention layer.  Host memory. */
typedef struct absb_layer {
  int32_t num_q_heads;       /* Hq                                                              */
  int32_t num_kv_heads;      /* Hkv; Hq % Hkv == 0; G = Hq/Hkv <= 8; Hkv <= 64                   */
  int32_t head_dim;          /* d; 128                                                          */
  int32_t page_size;         /* P tokens per physical page; power of two, >= 8                  */
  int32_t dtype;             /* absb_dtype of q, K, V and out                                   */
  int32_t block_repr;        /* absb_repr; 0 = mean pooling                                     */
  const int32_t* block_size; /* host [Hkv]: B_h, power of two in [8,128]; B_h | P or P | B_h    */
  /* K/V cache addressing, in elements: element (page, head, slot, c) of either cache is at
     page*kv_stride_page + head*kv_stride_head + slot*kv_stride_tok + c (channels contiguous).
     Every stride must be a multiple of 8 elements (16-byte rows).  "HND" pages
     [page][Hkv][P][d] are {Hkv*P*d, P*d, d}. */
  int64_t kv_stride_page, kv_stride_head, kv_stride_tok;
  float sm_scale;            /* softmax scale; 0 selects 1/sqrt(head_dim) as in Eq. (1)         */
  /* Selection policy on top of the paper's pure Top-K (both 0 = pure Top-K): every block that holds
     one of the first sink_tokens or of the last recent_tokens tokens of the context ranks ahead of
     every score (lowest index first among themselves).  Forced blocks count towards K_s.        */
  int32_t sink_tokens;       /* >= 0                                                            */
  int32_t recent_tokens;     /* >= 0                                                            */
  int32_t selection;         /* absb_select; 0 = one selection per KV head                      */
} absb_layer;

/* How a call is enqueued: launch shapes that never change what is computed (selections stay
 * bit-identical, outputs stay within rounding).  All zero = the library's choices, which is what
 * correct use needs; the fields exist for measurements and for callers that know their shapes.  They
 * are read from the batch of the call they are passed with and from nowhere else: nothing
 * process-wide, two callers cannot change each other's launches.  An invalid value makes the entry
 * point return ABSB_ERR_BAD_SHAPE before anything is enqueued. */
typedef enum absb_step_form {
  ABSB_STEP_AUTO = 0,       /* by shape (see absb_decode_fused)                                    */
  ABSB_STEP_PIPELINED = 1,  /* one launch: estimation work-groups, a segment's last one selects, then
                               attention work-groups that start on the segment's flag              */
  ABSB_STEP_UNITS = 2,      /* one launch: every work-group scores, selects and attends for its own
                               stretch of a segment's blocks                                       */
  ABSB_STEP_PER_STAGE = 3   /* one launch per stage: score, top-k, sparse decode                   */
} absb_step_form;
typedef struct absb_launch_opts {
  int32_t step_form;     /* absb_step_form; read by absb_decode_fused(_static), absb_step_form_used */
  int32_t split_tokens;  /* tokens per split-K work-group of the attention kernel; multiple of 64    */
  int32_t score_chunk;   /* blocks per estimation work-group; multiple of 64                        */
  int32_t unit_tokens;   /* ABSB_STEP_UNITS: selected tokens a work-group should get; multiple of 64 */
  int32_t counters_zero; /* absb_sparse_decode only: 1 = the split counters at the start of the
                            workspace are known to be zero, the kernel that clears them is skipped.
                            That holds after any completed absb_sparse_decode / absb_decode_fused call
                            for the same number of segments on that workspace (the counters sit at its
                            start, no other stage writes there, every kernel leaves the ones it used
                            at zero).  0 = clear them (default).                                    */
} absb_launch_opts;

/* One decode step's batch. */
typedef struct absb_batch {
  int32_t batch;                /* Bt >= 1                                                      */
  int32_t pt_stride;            /* row pitch of page_table, >= ceil(max L_b / P)                */
  const int32_t* seq_lens_host; /* host [Bt]: context length L_b >= 1 (includes the new token)  */
  const int32_t* seq_lens;      /* device [Bt], same values                                     */
  const int32_t* page_table;    /* device [Bt][pt_stride]: logical page -> physical page        */
  const int32_t* cent_off;      /* device [Bt*Hkv+1]: off[s+1] = off[s] + ceil(L_b/B_h)
                                   (Sec. 3.4 kernel 1); absb_plan computes the host copy        */
  const int32_t* budget_host;   /* host [Bt]: token budget T_b >= 1 per KV head                 */
  const int32_t* budget;        /* device [Bt], same values                                     */
  const int32_t* cap_lens_host; /* host [Bt] or NULL: the lengths the block layout is sized for,
                                   >= seq_lens_host.  With it, cent_off is laid out for
                                   ceil(cap_b/B_h) blocks per segment, of which the first
                                   N_s = ceil(L_b/B_h) are in use: contexts can then grow in place
                                   (absb_append_token).  NULL = the tight layout of Sec. 3.4.   */
  const float* qmin;            /* device [Bt*Hkv][d] or NULL: the store's zero-point offsets as
                                   written by absb_build_centroids; read by absb_score and
                                   absb_decode_fused only with ABSB_SELECT_GROUP_MAX            */
  absb_launch_opts opts;        /* all zero = the library's choices                             */
} absb_batch;

/* Sizes derived on the host from a (layer, batch) pair.  Only the host fields of `batch`
 * are read (seq_lens_host, budget_host); device pointers may be NULL here.
 *   cent_off_host [Bt*Hkv+1] : prefix sums of N_s = ceil(L_b/B_h), or of ceil(cap_b/B_h) when
 *                              cap_lens_host is given                          (may be NULL)
 *   total_centroids          : off[Bt*Hkv] (rows of the code array, used or not)
 *   sel_stride               : max_s K_s, K_s = min(N_s, ceil(T_b/B_h)) (Sec. 3.4 kernel 2)
 *   workspace_bytes          : enough for any entry point below on this (layer, batch) */
ABSB_API int absb_plan(const absb_layer* layer, const absb_batch* batch, int32_t* cent_off_host,
                       int64_t* total_centroids, int32_t* sel_stride, size_t* workspace_bytes);

/* Centroid store build (Sec. 2.2 pooling; Sec. 3.3 INT4 asymmetric per-channel; Sec. 3.4
 * flattened layout).  Reads every key of every request once.  With R vectors per block
 * (see absb_repr) a block is a row of R*d values:
 *   k_cache          : paged K cache (layout above)
 *   codes [total][R*d/2] u8 : block j of segment s at byte (off[s]+j)*(R*d/2); byte i holds
 *                      value 2i in its low nibble and value 2i+1 in its high nibble
 *   qscale [Bt*Hkv][R*d] f32: per (segment, value) step (max-min)/15 over that segment's blocks
 *   qmin   [Bt*Hkv][R*d] f32: per (segment, value) minimum (the asymmetric zero-point offset)
 * A last block shorter than B_h is pooled over its valid keys.  Arithmetic is binary32 in a
 * fixed order (keys summed in token order, one division, round-half-even codes), so the codes
 * are reproducible bit for bit. */
ABSB_API int absb_build_centroids(const absb_layer* layer, const absb_batch* batch, const void* k_cache,
                                  uint8_t* codes, float* qscale, float* qmin, void* workspace,
                                  size_t workspace_bytes, void* stream);

/* Estimation (Sec. 2.2 r = q . c^T; Sec. 3.4 kernel 1): one launch over the flattened code array.
 *   q [Bt][Hq][d]     : queries of this step
 *   scores [total] i32: S_j = sum_c wq_c * code_jc, where wq is the 16-bit fixed-point image
 *                       (largest magnitude in [2^14, 2^15]) of w_c = (sum_g q_g[c]) * qscale[s][c].
 *                       Within a segment S_j ranks the blocks exactly as the dequantized
 *                       score does (the zero-point term is constant per segment).
 *                       ABSB_REPR_MINMAX: the same over 2d weights, w = (P * qscale[s][0..d),
 *                       Q * qscale[s][d..2d)), P_c / Q_c the sums of the group's positive /
 *                       negative q_g[c]: the bound's larger product is the one whose extremum
 *                       matches the sign of q_c, which keeps the group score linear in the codes.
 *   score_exp [Bt*Hkv] i32, optional (NULL ok): e with w ~= wq * 2^e
 * Reads batch->seq_lens and batch->cent_off.
 * ABSB_SELECT_GROUP_MAX (mean pooling): S_j = max_g ( sum_c wq_gc * code_jc + zq_g ) on one exponent
 * e per group: w_gc = q_g[c] * qscale[s][c], e from the largest |w_gc| of the group, zq_g =
 * rint(z_g * 2^-e) clamped to +-2^30, z_g = sum_c q_g[c] * qmin[s][c] in binary32 (products summed
 * pairwise within runs of 16 consecutive channels, the runs then in increasing order).
 * ABSB_SELECT_PER_QUERY_HEAD: w_c = q_hs[c] * qscale[s][c] for the one query head; scores holds
 * G*total values, the G selection segments of store segment s side by side: block j of query head
 * hs at G*off[s] + (hs % G)*(off[s+1]-off[s]) + j; score_exp [Bt*Hq]. */
ABSB_API int absb_score(const absb_layer* layer, const absb_batch* batch, const void* q, const uint8_t* codes,
                        const float* qscale, int32_t* scores, int32_t* score_exp, void* stream);

/* Selection (Sec. 3.4 kernel 2): per segment the K_s = min(N_s, ceil(T_b/B_h)) blocks with the
 * highest score; equal scores go to the lower block index.
 *   sel_idx [Bt*Hkv][sel_stride] i32: chosen block indices in ascending order, padded with -1
 *   sel_cnt [Bt*Hkv] i32            : K_s
 *   sel_stride >= the value absb_plan reports, else ABSB_ERR_BAD_SHAPE
 * With layer->sink_tokens / recent_tokens set, the blocks holding those tokens are selected first
 * (lowest index first if there are more of them than K_s), the rest of K_s by score.
 * ABSB_SELECT_PER_QUERY_HEAD: one list per selection segment, sel_idx [Bt*Hq][sel_stride],
 * sel_cnt [Bt*Hq]; scores laid out as absb_score writes them. */
ABSB_API int absb_topk(const absb_layer* layer, const absb_batch* batch, const int32_t* scores,
                       int32_t* sel_idx, int32_t* sel_cnt, int32_t sel_stride, void* workspace,
                       size_t workspace_bytes, void* stream);

/* Attention over selected blocks (Eq. (1) restricted to the selection; Sec. 3.4 kernel 3).
 * Block j of segment (b,h) covers tokens [j*B_h, min((j+1)*B_h, L_b)); token t lives in
 * physical page page_table[b][t / P], slot t % P.  K and V rows are read in place.
 *   sel_idx/sel_cnt : any block list per segment (order free, no duplicates), sel_cnt[s] <=
 *                     sel_stride; when batch->budget_host is non-NULL also sel_cnt[s] <= K_s
 *   out [Bt][Hq][d] : attention output in the K/V dtype
 *   lse [Bt][Hq] f32, optional (NULL ok): natural-log sum of exp of the scaled logits
 * An empty selection yields out = 0 and lse = -inf.  Accumulation is binary32; the softmax weights
 * enter the P V product rounded to the K/V dtype and out is normalised by the sum of the rounded
 * weights, lse is taken from the weights before rounding.
 * ABSB_SELECT_PER_QUERY_HEAD: sel_idx [Bt*Hq][sel_stride], sel_cnt [Bt*Hq], one list per query head. */
ABSB_API int absb_sparse_decode(const absb_layer* layer, const absb_batch* batch, const void* q,
                                const void* k_cache, const void* v_cache, const int32_t* sel_idx,
                                const int32_t* sel_cnt, int32_t sel_stride, void* out, float* lse,
                                void* workspace, size_t workspace_bytes, void* stream);

/* Clears the counters at the start of `workspace` (see "Workspace" above).  One small launch. */
ABSB_API int absb_workspace_init(const absb_layer* layer, const absb_batch* batch, void* workspace,
                                 size_t workspace_bytes, void* stream);

/* The whole step: score -> topk -> sparse decode (Sec. 3.4, kernels 1-3) through one call, with the
 * fewest launches that are fastest for the shape.  Produces exactly the selection of absb_score +
 * absb_topk, and the output of absb_sparse_decode on it up to the rounding of a different summation
 * order (same tolerance against exact arithmetic).  Three ways to enqueue it (batch->opts.step_form;
 * ABSB_STEP_AUTO picks by shape):
 *   ABSB_STEP_PIPELINED  one launch.  The grid holds the estimation work-groups, then the attention
 *                        work-groups; a segment's last estimation work-group runs its selection and
 *                        raises a flag, the segment's attention work-groups start on that flag.
 *                        Chosen while no segment exceeds 16384 blocks and no list 4096 blocks.
 *   ABSB_STEP_UNITS      one launch.  Every segment is cut into units of consecutive blocks; a unit's
 *                        work-group scores its blocks, publishes a histogram row of its scores,
 *                        derives the segment's threshold from all rows, and attends over its own
 *                        selected blocks; blocks inside the threshold bin are settled by an exact
 *                        ranking among the segment's candidates.  No work-group ever passes over a
 *                        whole segment, so the cost hardly grows with the context.  Chosen for
 *                        segments beyond 16384 blocks when the chip holds all units at once.
 *   ABSB_STEP_PER_STAGE  three launches (score, top-k, sparse decode).  Otherwise.
 * The one-launch forms hand work between work-groups through the counters at the start of the
 * workspace: they must be zero when the call starts (absb_workspace_init) and are zero again when its
 * work has finished.  ABSB_STEP_PER_STAGE does not need them cleared.
 *   sel_idx_out [Bt*Hkv][plan's sel_stride], sel_cnt_out [Bt*Hkv]: optional copies of the
 *   selection (NULL ok).
 * Status word (one-launch forms): every wait of a work-group for another is bounded in time (0.25 s).
 * A wait that runs out can only mean that the contract was broken (counters not zero at the start,
 * device lengths or budgets that differ from their host twins) or that the device was taken away
 * from the launch for that long; the work-group then sets the int32 at absb_status_offset() to 1,
 * writes NaN into its segment's rows of `out` (and `lse`) and leaves, so the launch always ends.  The
 * call itself has long returned ABSB_OK by then: a caller that cannot rule those causes out reads
 * the status word after synchronising with the stream (or looks for NaN in `out`), and when it is
 * set calls absb_workspace_init before the workspace is used again and repeats the step. */
ABSB_API int absb_decode_fused(const absb_layer* layer, const absb_batch* batch, const void* q,
                               const uint8_t* codes, const float* qscale, const void* k_cache,
                               const void* v_cache, void* out, float* lse, int32_t* sel_idx_out,
                               int32_t* sel_cnt_out, void* workspace, size_t workspace_bytes, void* stream);

/* For callers that cannot allocate device memory (code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc): absb_decode_fused without a workspace argument.  The
 * scratch memory (counters, scores, lists, split-K partials) is a fixed array of
 * ABSB_STATIC_WORKSPACE_BYTES inside the library's code object: every GPU the library runs on holds
 * its own copy from the first use until the process ends.  The call allocates and frees nothing and
 * calls no runtime routine that does; inputs and outputs are still the caller's.  Same results as
 * absb_decode_fused with a cleared workspace of the caller's.
 *   - A (layer, batch) whose absb_plan workspace_bytes exceeds ABSB_STATIC_WORKSPACE_BYTES is refused
 *     with ABSB_ERR_STATIC_WORKSPACE before anything is enqueued.
 *   - The array keeps what the last call left; the call clears what must start at zero itself (a
 *     small fill kernel on `stream` whenever the batch shape's counter area differs from the last
 *     call's on that GPU), so no absb_workspace_init is needed.
 *   - All calls on one GPU share that GPU's array: calls whose device work can overlap (different
 *     streams, or threads that do not order their streams) race.  Order them on one stream.
 *   - The device is the one current at the call (hipGetDevice); `stream` must belong to it. */
#define ABSB_STATIC_WORKSPACE_BYTES (16u << 20)
ABSB_API int absb_decode_fused_static(const absb_layer* layer, const absb_batch* batch, const void* q,
                                      const uint8_t* codes, const float* qscale, const void* k_cache,
                                      const void* v_cache, void* out, float* lse, int32_t* sel_idx_out,
                                      int32_t* sel_cnt_out, void* stream);

/* How absb_decode_fused will enqueue the step for this (layer, batch, batch->opts): the absb_step_form
 * it will use (ABSB_STEP_PIPELINED, ABSB_STEP_UNITS: one launch; ABSB_STEP_PER_STAGE: three), never
 * ABSB_STEP_AUTO; a negative absb_status on invalid arguments.  A form asked for in batch->opts that
 * cannot hold the shape falls back to ABSB_STEP_PER_STAGE.  Pure host helper; reads the host fields
 * only. */
ABSB_API int absb_step_form_used(const absb_layer* layer, const absb_batch* batch);

/* Where the one-launch forms report a wait that ran out (see absb_decode_fused): byte offset, inside
 * the workspace, of an int32 status word that absb_workspace_init clears and that stays zero in
 * normal operation.  Pure host helper. */
ABSB_API int absb_status_offset(const absb_layer* layer, const absb_batch* batch, size_t* offset);

/* Keeping the store current while decoding, without a rebuild (the paper notes that recomputing
 * every centroid is too expensive, Sec. 1 and 3.2, and leaves the mechanism open; this is the
 * reading taken here).  The pooled state of each segment's LAST block is kept in binary32 in
 * `tail` [Bt*Hkv][R*d]: the running sum of its keys in token order (mean pooling), or its running
 * maxima then minima (max-min pooling).
 *
 * absb_tail_init: computes `tail` from the K cache at the lengths in batch->seq_lens (call once
 * after absb_build_centroids).
 *
 * absb_append_token: every request has grown by ONE token: batch->seq_lens(_host) already count
 * it and its key is in the K cache at position L_b - 1.  The key is folded into `tail` with the
 * single binary32 operations a rebuild would use (so the block's value is bit-identical to a
 * rebuild's), and the 4-bit row of the block that holds it is re-emitted under the store's FROZEN
 * qscale/qmin: code = clamp(rint((value - qmin) * (1/qscale)), 0, 15), 0 where qscale is 0.  Rows
 * of closed blocks never change; qscale/qmin are only refreshed by absb_build_centroids.  When the
 * token opens a new block the row off[s] + N_s - 1 is written for the first time: the layout must
 * have room for it (batch->cap_lens_host).
 *   clamped [Bt*Hkv] i32, optional (NULL ok): the signal for a re-ranging policy.  When the token
 *   completes its block (L_b % B_h == 0; the row is final from then on), the number of the row's R*d
 *   values that the frozen range does not hold is ADDED to clamped[s]: values whose unclamped code
 *   falls outside [0, 15], and values that differ from qmin where qscale is 0.  The caller zeroes
 *   the array after absb_build_centroids and rebuilds when the counts (at most R*d per completed
 *   block) exceed what it tolerates.  One request is re-ranged without touching the others by
 *   absb_build_centroids on a batch of one: that request's length, capacity, page-table row and its
 *   own prefix sums (those of the batch minus off[b*Hkv]), with codes + off[b*Hkv]*(R*d/2),
 *   qscale + b*Hkv*R*d and qmin + b*Hkv*R*d as outputs, and a workspace of its own (the counters at
 *   the start of a workspace belong to one batch shape). */
ABSB_API int absb_tail_init(const absb_layer* layer, const absb_batch* batch, const void* k_cache, float* tail,
                            void* stream);
ABSB_API int absb_append_token(const absb_layer* layer, const absb_batch* batch, const void* k_cache,
                               uint8_t* codes, const float* qscale, const float* qmin, float* tail,
                               int32_t* clamped, void* stream);

/* Offline calibration of the per-head block sizes (Sec. 3.2).  Two pieces; the loop over
 * calibration samples and candidate sizes around them uses the entry points above.
 *
 * absb_head_recall: attention recall (Sec. 2.3) of a selection per (request, KV head), from two
 * log-sum-exp arrays of the same queries over the same cache: `lse_selected` as written by
 * absb_sparse_decode / absb_decode_fused for the selection, `lse_dense` as written by the same
 * entry points with a budget >= the context length.  recall[s] = mean over the group's query heads
 * of exp(lse_selected - lse_dense).  All three device arrays: lse [Bt][Hq] f32, recall [Bt*Hkv] f32.
 *
 * absb_assign_block_sizes (host only, no device work): Eq. (2).  recall_host
 * [n_samples][n_heads][n_cand] f32 holds Recall(h, B) per calibration sample, candidates ascending
 * (cand[0] = B_min); block_size_out[h] = the largest candidate whose mean recall over the samples is
 * >= tau * the mean recall at B_min.  mean_out [n_heads][n_cand] f64 (NULL ok) receives the means. */
ABSB_API int absb_head_recall(const absb_layer* layer, const absb_batch* batch, const float* lse_selected,
                              const float* lse_dense, float* recall, void* stream);
ABSB_API int absb_assign_block_sizes(int32_t n_samples, int32_t n_heads, int32_t n_cand, const float* recall_host,
                                     const int32_t* cand, double tau, int32_t* block_size_out, double* mean_out);

/* Measurement helper, not a step of the method: reads `bytes` (a multiple of 16; the tail is
 * ignored) of the device buffer `src` (16-byte aligned) once with 128-bit loads and discards them.
 * Timing it gives the practical streaming-read ceiling of the device, against which the attention
 * kernel's bandwidth can be stated.  `sink`: 4 bytes of device memory (practically never written). */
ABSB_API int absb_stream_read(const void* src, size_t bytes, void* sink, void* stream);

/* Static string for a status code. */
ABSB_API const char* absb_strerror(int status);

#ifdef __cplusplus
}
#endif
#endif /* ABSB_H */
