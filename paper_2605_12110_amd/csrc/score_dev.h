// Estimation stage, device side (Sec. 3.4, kernel 1): importance score of every block of every
// (request, KV head) from the INT4 centroid codes, dequantization fused, one launch over the
// flattened code array delimited by the prefix-sum offsets.
//
// The G query heads of a KV head are folded into one weight vector w_c = (sum_g q_g[c]) * scale_c
// (the score r = q . c^T of Sec. 2.2 is linear in q; the zero-point term is constant within a
// segment and cannot change the ranking).  w is imaged on integers wq with the largest magnitude
// in [2^14, 2^15]; S_j = sum_c wq_c * code_jc is then exact in int32 in any summation order, so the
// ranking has one answer on every machine.  The binary32 steps (sum over g in order, one multiply,
// max, power-of-two scaling, round-half-even) are single IEEE operations: this file is compiled
// with -ffp-contract=off.
//
// Memory: a block is 64 bytes of codes per vector (one vector for mean pooling; maxima then minima
// for max-min pooling, whose score is the same dot over 256 weights: the maxima weighted by the sum
// of the group's positive q_g, the minima by the sum of its negative q_g).  Four lanes share one
// block (16 bytes = 32 values of each vector), so one wave load instruction reads 16 whole vectors.
//
// Arithmetic: the codes are unsigned 4-bit, so the dot product runs on the packed 4-bit dot
// instruction (8 multiply-adds per lane and instruction).  The biased weight wq + 2^15 (17 bits,
// unsigned) is cut into five 4-bit planes; S = sum_k 16^k * dot(plane_k, codes) - 2^15 * sum(codes).
// Six packed dots per 8 channels replace 16 unpack-and-multiply steps, and the kernel stays short:
// it is launched with one batch of work per lane, so instruction count is what bounds it.
#pragma once
#include "common.h"

namespace absb {

struct ScoreParams {
  const uint16_t* q;        // [Bt][Hq][128]
  const uint8_t* codes;     // [total][64 * R], R vectors per block
  const float* qscale;      // [nseg][128 * R]
  const float* qmin;        // [nseg][128]: read only when agg_max
  const int32_t* cent_off;  // [nseg+1]
  const int32_t* seq_lens;  // [Bt]
  HeadTable heads;
  int32_t* scores;          // [total]
  int32_t* score_exp;       // [nseg] or null
  int32_t Hq, Hkv, G, chunk, tight;  // G: query heads folded into one selection segment (Gd)
  int32_t Hsel, Rk;
  int32_t agg_max;  // the group's score is the maximum over its query heads (mean pooling only)
};

constexpr int SCORE_PLANES = 5;

inline ScoreParams make_score_params(const Geometry& g, const Plan& pl, const void* q, const uint8_t* codes,
                                     const float* qscale, const float* qmin, const int32_t* cent_off,
                                     const int32_t* seq_lens, int32_t* scores, int32_t* score_exp) {
  ScoreParams p;
  p.q = static_cast<const uint16_t*>(q);
  p.codes = codes;
  p.qscale = qscale;
  p.qmin = qmin;
  p.agg_max = g.agg_max;
  p.cent_off = cent_off;
  p.seq_lens = seq_lens;
  p.heads = g.heads;
  p.tight = g.tight;
  p.scores = scores;
  p.score_exp = score_exp;
  p.Hq = g.Hq;
  p.Hkv = g.Hkv;
  p.G = g.Gd;
  p.Hsel = g.Hsel;
  p.Rk = g.Rk;
  p.chunk = pl.score_chunk;
  return p;
}

__device__ __forceinline__ uint32_t or8(uint32_t v) {  // OR over aligned groups of 8 lanes
  v |= (uint32_t)dpp_i<DPP_QUAD_XOR1>((int)v);
  v |= (uint32_t)dpp_i<DPP_QUAD_XOR2>((int)v);
  v |= (uint32_t)dpp_i<DPP_ROW_HALF_MIRROR>((int)v);
  return v;
}

// LDS of one work-group: the four wave maxima, then the digit planes of the weights.  The
// group-maximum score keeps a set of planes per query head, the run sums of the heads' zero-point
// products and their fixed-point offsets.
constexpr size_t SCORE_GMAX_PLANES_AT = 16 + ABSB_MAX_GROUP * 8 * 4 + ABSB_MAX_GROUP * 4;
constexpr size_t SCORE_GMAX_RANGE_AT =
    SCORE_GMAX_PLANES_AT + (size_t)ABSB_MAX_GROUP * SCORE_PLANES * (ABSB_HEAD_DIM / 8) * sizeof(uint32_t);
template <int REP>
__host__ __device__ constexpr size_t score_range_at() {  // per-wave sums of the negative / positive weights
  return 16 + (size_t)SCORE_PLANES * (ABSB_HEAD_DIM * (REP + 1) / 8) * sizeof(uint32_t);
}
template <int REP>
__host__ __device__ constexpr size_t score_lds_bytes() {
  const size_t plain = score_range_at<REP>() + 4 * 2 * sizeof(int32_t);
  const size_t gmax = SCORE_GMAX_RANGE_AT + 2 * ABSB_MAX_GROUP * 2 * sizeof(int32_t);
  return REP == 0 && gmax > plain ? gmax : plain;
}

// Bounds of a segment's scores that follow from the weights alone (every code lies in [0, 15]):
// lo = 15 * sum_c min(wq_c, 0) <= S_j <= 15 * sum_c max(wq_c, 0) = hi.  The same for every work-group
// that scores a part of the segment, before any code has been read.
struct ScoreRange {
  int32_t lo, hi;
};
struct IAdd {
  __device__ __forceinline__ uint32_t operator()(uint32_t a, uint32_t b) const { return a + b; }
};

// Group-maximum score (mean pooling): S_j = max_g ( sum_c wq_gc * code_jc + zq_g ) with one exponent
// for the group; see absb_score.  Same work split as score_chunk below: four lanes per block, the
// packed 4-bit dots once per query head against that head's digit planes (read from LDS per head),
// the sum of the codes shared by all heads.
template <int DT, bool RANGE, int PF, class Sink>
__device__ __forceinline__ int score_blocks_groupmax(const ScoreParams& p, int t, int j0, int jcount, char* lds,
                                                     Sink&& sink, ScoreRange* range) {
  constexpr int W = ABSB_HEAD_DIM, ROW_BYTES = W / 2;
  const SegMap sm = seg_map(t, p.Hsel, p.Rk, p.Hkv);
  const int b = sm.b, s = sm.s;
  const int tid = threadIdx.x, G = p.G;
  uint16_t qraw[ABSB_MAX_GROUP];
  float scale = 0.0f, zero = 0.0f;
  if (tid < W) {
    const uint16_t* qrow = p.q + ((size_t)b * p.Hq + (size_t)sm.hs * G) * ABSB_HEAD_DIM + tid;
#pragma unroll
    for (int g = 0; g < ABSB_MAX_GROUP; ++g) qraw[g] = g < G ? qrow[(size_t)g * ABSB_HEAD_DIM] : (uint16_t)0;
    scale = p.qscale[(size_t)s * W + tid];
    zero = p.qmin[(size_t)s * W + tid];
  }
  const int off = p.cent_off[s];
  const int rows = p.cent_off[s + 1] - off;
  const int N = blocks_in_use(p.tight, rows, p.seq_lens, b, p.heads.log2_block[sm.hk]);
  if (j0 >= N) return 0;

  float* s_absmax = reinterpret_cast<float*>(lds);                                   // [4]
  float (*s_zrun)[8] = reinterpret_cast<float (*)[8]>(lds + 16);                     // [G][8 runs of 16 channels]
  int32_t* s_zq = reinterpret_cast<int32_t*>(lds + 16 + ABSB_MAX_GROUP * 8 * 4);     // [G]
  uint32_t (*s_plane)[SCORE_PLANES][W / 8] =
      reinterpret_cast<uint32_t (*)[SCORE_PLANES][W / 8]>(lds + SCORE_GMAX_PLANES_AT);  // [G][planes][16]

  int32_t (*s_rng)[ABSB_MAX_GROUP][2] =
      reinterpret_cast<int32_t (*)[ABSB_MAX_GROUP][2]>(lds + SCORE_GMAX_RANGE_AT);     // [2 waves][G][neg, pos]

  const int quarter = tid & 3;
  const int jend = min(N, j0 + jcount);
  const uint8_t* base = p.codes + (size_t)off * ROW_BYTES + quarter * 16;
  uint4 pre[PF];
#pragma unroll
  for (int u = 0; u < PF; ++u) {
    const int j = min(j0 + u * 64 + (tid >> 2), jend - 1);
    pre[u] = *reinterpret_cast<const uint4*>(base + (size_t)j * ROW_BYTES);
  }

  // ---- prologue (threads 0..127, one channel each): weights of every head, their largest
  // magnitude, and the heads' zero-point products summed pairwise over each run of 16 channels
  float w[ABSB_MAX_GROUP];
  if (tid < W) {
    float a = 0.0f;
#pragma unroll
    for (int g = 0; g < ABSB_MAX_GROUP; ++g) {
      const float qv = Elem<DT>::widen(qraw[g]);
      w[g] = qv * scale;
      float ag = __builtin_fabsf(w[g]);
      ag = (ag != ag) ? 0.0f : ag;
      a = fmaxf(a, g < G ? ag : 0.0f);
      const float run = row16_sum(qv * zero);  // ((p0+p1)+(p2+p3))+... over the row's 16 channels
      if (g < G && (tid & 15) == 0) s_zrun[g][tid >> 4] = run;
    }
    a = wave_max_f32(a);
    if ((tid & 63) == 0) s_absmax[tid >> 6] = a;
  }
  __syncthreads();
  const float A = fmaxf(s_absmax[0], s_absmax[1]);
  int ex = 0;
  const bool live = (A >= 0x1p-100f) && (A <= 3.4028234663852886e38f);
  if (live) ex = (int)((bitcast<uint32_t>(A) >> 23) & 0xffu) - 127 - 14;
  if (tid < G) {  // the head's offset on the group's scale: the 8 run sums in order
    float z = s_zrun[tid][0];
#pragma unroll
    for (int k = 1; k < 8; ++k) z = z + s_zrun[tid][k];
    float zs = live ? __builtin_rintf(__builtin_ldexpf(z, -ex)) : 0.0f;
    zs = (zs != zs) ? 0.0f : zs;
    zs = fminf(fmaxf(zs, -0x1p30f), 0x1p30f);
    s_zq[tid] = (int32_t)zs;
  }
  if (tid < W) {
    const int sh = 4 * (tid & 7);
#pragma unroll
    for (int g = 0; g < ABSB_MAX_GROUP; ++g) {
      int32_t wq = 0;
      if (live && w[g] == w[g]) wq = (int32_t)__builtin_rintf(__builtin_ldexpf(w[g], -ex));  // a NaN weight images to 0
      const uint32_t wo = (uint32_t)(wq + 32768);
#pragma unroll
      for (int k = 0; k < SCORE_PLANES; ++k) {
        const uint32_t packed = or8(((wo >> (4 * k)) & 15u) << sh);
        if (g < G && (tid & 7) == 0) s_plane[g][k][tid >> 3] = packed;
      }
      if (RANGE) {  // per head: sums of its negative and of its positive weights (exact, order-free)
        const uint32_t neg = wave_reduce_u32((uint32_t)min(wq, 0), IAdd()), pos = wave_reduce_u32((uint32_t)max(wq, 0), IAdd());
        if (g < G && (tid & 63) == 0) {
          s_rng[tid >> 6][g][0] = (int32_t)neg;
          s_rng[tid >> 6][g][1] = (int32_t)pos;
        }
      }
    }
  }
  if (tid == 0 && j0 == 0 && p.score_exp) p.score_exp[t] = ex;
  __syncthreads();
  if (RANGE) {  // S_j = max_g (dot_g + zq_g), and dot_g lies in 15 * [sum of negative, sum of positive weights]
    int32_t lo = INT32_MIN, hi = INT32_MIN;
    for (int g = 0; g < G; ++g) {
      lo = max(lo, 15 * (s_rng[0][g][0] + s_rng[1][g][0]) + s_zq[g]);
      hi = max(hi, 15 * (s_rng[0][g][1] + s_rng[1][g][1]) + s_zq[g]);
    }
    range->lo = lo;
    range->hi = hi;
  }

#pragma unroll 1
  for (int jb = j0;;) {
    uint32_t ones[PF];
    int32_t best[PF];
#pragma unroll
    for (int u = 0; u < PF; ++u) {
      uint32_t o = __builtin_amdgcn_udot8(pre[u].x, 0x11111111u, 0u, false);
      o = __builtin_amdgcn_udot8(pre[u].y, 0x11111111u, o, false);
      o = __builtin_amdgcn_udot8(pre[u].z, 0x11111111u, o, false);
      ones[u] = __builtin_amdgcn_udot8(pre[u].w, 0x11111111u, o, false);
      best[u] = 0;
    }
#pragma unroll 1
    for (int g = 0; g < G; ++g) {
      uint4 wp[SCORE_PLANES];
#pragma unroll
      for (int k = 0; k < SCORE_PLANES; ++k) wp[k] = *reinterpret_cast<const uint4*>(&s_plane[g][k][quarter * 4]);
      const int32_t zq = s_zq[g];
#pragma unroll
      for (int u = 0; u < PF; ++u) {
        uint32_t acc = 0;
#pragma unroll
        for (int k = 0; k < SCORE_PLANES; ++k) {
          uint32_t d = __builtin_amdgcn_udot8(pre[u].x, wp[k].x, 0u, false);
          d = __builtin_amdgcn_udot8(pre[u].y, wp[k].y, d, false);
          d = __builtin_amdgcn_udot8(pre[u].z, wp[k].z, d, false);
          d = __builtin_amdgcn_udot8(pre[u].w, wp[k].w, d, false);
          acc += d << (4 * k);
        }
        acc -= ones[u] << 15;
        const int32_t sc = quad_sum((int32_t)acc) + zq;
        best[u] = g == 0 ? sc : max(best[u], sc);
      }
    }
#pragma unroll
    for (int u = 0; u < PF; ++u) {
      const int j = jb + u * 64 + (tid >> 2);
      if (j < jend && quarter == 0) sink(j, best[u]);
    }
    jb += PF * 64;
    if (jb >= jend) break;
#pragma unroll
    for (int u = 0; u < PF; ++u) {
      const int j = min(jb + u * 64 + (tid >> 2), jend - 1);
      pre[u] = *reinterpret_cast<const uint4*>(base + (size_t)j * ROW_BYTES);
    }
  }
  return N;
}

// Scores of blocks [j0, j0 + jcount) of selection segment t by one work-group of 256 threads; every score is
// handed to sink(block index, score) by one lane.  Returns the segment's block count N_s, or 0 (nothing
// done, *range untouched) when the segment has no such blocks.  RANGE: *range receives the bounds of the
// segment's scores.  PF: steps of 64 blocks whose codes are requested at once (a batch).
// `lds`: score_lds_bytes<REP>() bytes, 16-byte aligned.
template <int DT, int REP, bool RANGE, int PF, class Sink>
__device__ __forceinline__ int score_blocks(const ScoreParams& p, int t, int j0, int jcount, char* lds, Sink&& sink,
                                            ScoreRange* range) {
  if (REP == 0 && p.agg_max) return score_blocks_groupmax<DT, RANGE, PF>(p, t, j0, jcount, lds, sink, range);
  constexpr int R = REP + 1;                 // vectors per block: the mean, or maxima and minima
  constexpr int W = ABSB_HEAD_DIM * R;       // weights = values per block
  constexpr int ROW_BYTES = W / 2;
  const SegMap sm = seg_map(t, p.Hsel, p.Rk, p.Hkv);
  const int b = sm.b, s = sm.s;
  const int tid = threadIdx.x;
  // ---- the group's query values and the scale of this thread's weight go in flight first, all at
  // once: their addresses need nothing from memory, and everything below waits for them
  uint16_t qraw[ABSB_MAX_GROUP];
  float scale = 0.0f;
  if (tid < W) {
    const uint16_t* qrow =
        p.q + ((size_t)b * p.Hq + (size_t)sm.hs * p.G) * ABSB_HEAD_DIM + (tid & (ABSB_HEAD_DIM - 1));
#pragma unroll
    for (int g = 0; g < ABSB_MAX_GROUP; ++g) qraw[g] = g < p.G ? qrow[(size_t)g * ABSB_HEAD_DIM] : (uint16_t)0;
    scale = p.qscale[(size_t)s * W + tid];
  }
  const int off = p.cent_off[s];
  const int rows = p.cent_off[s + 1] - off;
  const int N = blocks_in_use(p.tight, rows, p.seq_lens, b, p.heads.log2_block[sm.hk]);
  if (j0 >= N) return 0;

  float* s_absmax = reinterpret_cast<float*>(lds);
  uint32_t (*s_plane)[W / 8] = reinterpret_cast<uint32_t (*)[W / 8]>(lds + 16);
  int32_t (*s_rng)[2] = reinterpret_cast<int32_t (*)[2]>(lds + score_range_at<REP>());  // [wave][neg, pos]

  // ---- the work-group's first batch of codes goes in flight before anything else: the loads do
  // not depend on the query, so their latency overlaps the prologue below
  // 64 blocks per work-group step, PF steps per batch
  const int quarter = tid & 3;
  const int jend = min(N, j0 + jcount);
  const uint8_t* base = p.codes + (size_t)off * ROW_BYTES + quarter * 16;
  uint4 pre[PF][R];
#pragma unroll
  for (int u = 0; u < PF; ++u) {
    const int j = min(j0 + u * 64 + (tid >> 2), jend - 1);  // clamped, not predicated: loads issue back to back
#pragma unroll
    for (int v = 0; v < R; ++v) pre[u][v] = *reinterpret_cast<const uint4*>(base + (size_t)j * ROW_BYTES + v * 64);
  }

  // ---- prologue: fixed-point image of the weights, by threads 0..W-1 (weight index = tid).
  // Mean pooling: w = (sum_g q_g) * scale.  Maxima / minima: the maxima meet the sum of the
  // group's positive q_g, the minima the sum of its negative q_g (each in order of g, from +0).
  float w = 0.0f;
  if (tid < W) {
    const int v = tid >> 7;
    float u;
    if (REP == 0) {
      u = Elem<DT>::widen(qraw[0]);
#pragma unroll
      for (int g = 1; g < ABSB_MAX_GROUP; ++g)
        if (g < p.G) u = u + Elem<DT>::widen(qraw[g]);
    } else {
      u = 0.0f;
#pragma unroll
      for (int g = 0; g < ABSB_MAX_GROUP; ++g) {
        const float x = Elem<DT>::widen(qraw[g]);
        if (g < p.G && (v == 0 ? x > 0.0f : x < 0.0f)) u = u + x;
      }
    }
    w = u * scale;
    float a = __builtin_fabsf(w);
    a = (a != a) ? 0.0f : a;  // a NaN never wins the maximum
    a = wave_max_f32(a);  // exact, order-free
    if ((tid & 63) == 0) s_absmax[tid >> 6] = a;
  }
  __syncthreads();
  float A = fmaxf(s_absmax[0], s_absmax[1]);
  if (REP) A = fmaxf(A, fmaxf(s_absmax[2], s_absmax[3]));
  int ex = 0;
  const bool live = (A >= 0x1p-100f) && (A <= 3.4028234663852886e38f);
  if (live) ex = (int)((bitcast<uint32_t>(A) >> 23) & 0xffu) - 127 - 14;
  if (tid < W) {
    int32_t wq = 0;
    if (live && w == w) wq = (int32_t)__builtin_rintf(__builtin_ldexpf(w, -ex));  // a NaN weight images to 0
    // biased weight in [0, 2^16]; its five 4-bit digits, packed over 8 consecutive values
    const uint32_t wo = (uint32_t)(wq + 32768);
    const int sh = 4 * (tid & 7);
#pragma unroll
    for (int k = 0; k < SCORE_PLANES; ++k) {
      const uint32_t packed = or8(((wo >> (4 * k)) & 15u) << sh);
      if ((tid & 7) == 0) s_plane[k][tid >> 3] = packed;
    }
    if (RANGE) {  // sums of the negative and of the positive weights (exact, order-free)
      const uint32_t neg = wave_reduce_u32((uint32_t)min(wq, 0), IAdd()), pos = wave_reduce_u32((uint32_t)max(wq, 0), IAdd());
      if ((tid & 63) == 0) {
        s_rng[tid >> 6][0] = (int32_t)neg;
        s_rng[tid >> 6][1] = (int32_t)pos;
      }
    }
  }
  if (tid == 0 && j0 == 0 && p.score_exp) p.score_exp[t] = ex;
  __syncthreads();
  if (RANGE) {
    int32_t neg = s_rng[0][0] + s_rng[1][0], pos = s_rng[0][1] + s_rng[1][1];
    if (REP) {
      neg += s_rng[2][0] + s_rng[3][0];
      pos += s_rng[2][1] + s_rng[3][1];
    }
    range->lo = 15 * neg;
    range->hi = 15 * pos;
  }

  // ---- each lane: the digit planes of its quarter of each vector (4 words of 8 values)
  uint4 wp[R][SCORE_PLANES];
#pragma unroll
  for (int v = 0; v < R; ++v)
#pragma unroll
    for (int k = 0; k < SCORE_PLANES; ++k)
      wp[v][k] = *reinterpret_cast<const uint4*>(&s_plane[k][v * (ABSB_HEAD_DIM / 8) + quarter * 4]);

  auto dot = [&](const uint4 (&cv)[R]) -> int32_t {
    uint32_t acc = 0, ones = 0;
#pragma unroll
    for (int v = 0; v < R; ++v) {
      const uint4 c = cv[v];
#pragma unroll
      for (int k = 0; k < SCORE_PLANES; ++k) {
        uint32_t d = __builtin_amdgcn_udot8(c.x, wp[v][k].x, 0u, false);
        d = __builtin_amdgcn_udot8(c.y, wp[v][k].y, d, false);
        d = __builtin_amdgcn_udot8(c.z, wp[v][k].z, d, false);
        d = __builtin_amdgcn_udot8(c.w, wp[v][k].w, d, false);
        acc += d << (4 * k);
      }
      ones = __builtin_amdgcn_udot8(c.x, 0x11111111u, ones, false);
      ones = __builtin_amdgcn_udot8(c.y, 0x11111111u, ones, false);
      ones = __builtin_amdgcn_udot8(c.z, 0x11111111u, ones, false);
      ones = __builtin_amdgcn_udot8(c.w, 0x11111111u, ones, false);
    }
    acc -= ones << 15;                 // two's complement: exact sum_c wq_c * code_c of this quarter
    return quad_sum((int32_t)acc);     // the four lanes of a quad hold the four quarters of one block
  };

  // ---- main loop: 64 blocks per work-group step (16 per wave), PF steps per batch.
  // Every lane of a quad shares j, so the quad reduction always sees four live lanes.
#pragma unroll 1
  for (int jb = j0;;) {
#pragma unroll
    for (int u = 0; u < PF; ++u) {
      const int j = jb + u * 64 + (tid >> 2);
      const int32_t sc = dot(pre[u]);
      if (j < jend && quarter == 0) sink(j, sc);
    }
    jb += PF * 64;
    if (jb >= jend) break;
#pragma unroll
    for (int u = 0; u < PF; ++u) {
      const int j = min(jb + u * 64 + (tid >> 2), jend - 1);
#pragma unroll
      for (int v = 0; v < R; ++v) pre[u][v] = *reinterpret_cast<const uint4*>(base + (size_t)j * ROW_BYTES + v * 64);
    }
  }
  return N;
}

// Where selection segment t's scores start in the score array.
__device__ __forceinline__ int32_t* scores_of(const ScoreParams& p, int t) {
  const SegMap sm = seg_map(t, p.Hsel, p.Rk, p.Hkv);
  const int off = p.cent_off[sm.s];
  return p.scores + score_base(sm, p.Rk, off, p.cent_off[sm.s + 1] - off);
}

// The stand-alone form: blocks [chunk_idx * p.chunk, + p.chunk), scores stored to the score array.
// COH: they are read by another work-group of the same launch.
template <int DT, int REP, bool COH>
__device__ __forceinline__ int score_chunk(const ScoreParams& p, int t, int chunk_idx, char* lds) {
  int32_t* scores_t = scores_of(p, t);
  return score_blocks<DT, REP, false, 4>(
      p, t, chunk_idx * p.chunk, p.chunk, lds, [&](int j, int32_t sc) { st_i32<COH>(scores_t + j, sc); }, nullptr);
}

}  // namespace absb
