// Estimation stage (Sec. 3.4, kernel 1): importance score of every block of every
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
// Memory: a centroid is 64 bytes of codes.  Four lanes share one centroid (16 bytes = 32 channels
// each), so one wave load instruction reads 1 KiB of consecutive codes; each lane keeps its 32
// integer weights in registers for the whole work-group.
#include "common.h"

namespace absb {

struct ScoreParams {
  const uint16_t* q;        // [Bt][Hq][128]
  const uint8_t* codes;     // [total][64]
  const float* qscale;      // [nseg][128]
  const int32_t* cent_off;  // [nseg+1]
  int32_t* scores;          // [total]
  int32_t* score_exp;       // [nseg] or null
  int32_t Hq, Hkv, G, chunk;
};

template <int DT>
__global__ __launch_bounds__(256) void score_kernel(ScoreParams p) {
  const int s = blockIdx.y;
  const int off = p.cent_off[s];
  const int N = p.cent_off[s + 1] - off;
  const int j0 = blockIdx.x * p.chunk;
  if (j0 >= N) return;
  const int b = s / p.Hkv, h = s % p.Hkv;
  const int tid = threadIdx.x;

  __shared__ float s_absmax[2];
  __shared__ int32_t s_wq[ABSB_HEAD_DIM];

  // ---- the work-group's first batch of codes goes in flight before anything else: the loads do
  // not depend on the query, so their latency overlaps the prologue below
  constexpr int PF = 4;  // 64 centroids per work-group step, PF steps per batch
  const int quarter = tid & 3;
  const int jend = min(N, j0 + p.chunk);
  const uint8_t* base = p.codes + (size_t)off * 64 + quarter * 16;
  uint4 pre[PF];
#pragma unroll
  for (int u = 0; u < PF; ++u) {
    const int j = j0 + u * 64 + (tid >> 2);
    pre[u] = j < jend ? *reinterpret_cast<const uint4*>(base + (size_t)j * 64) : make_uint4(0, 0, 0, 0);
  }

  // ---- prologue: fixed-point image of w = (sum_g q_g) * scale, by threads 0..127
  float w = 0.0f;
  if (tid < ABSB_HEAD_DIM) {
    const uint16_t* qrow = p.q + ((size_t)b * p.Hq + (size_t)h * p.G) * ABSB_HEAD_DIM + tid;
    float u = Elem<DT>::widen(qrow[0]);
    for (int g = 1; g < p.G; ++g) u = u + Elem<DT>::widen(qrow[(size_t)g * ABSB_HEAD_DIM]);
    w = u * p.qscale[(size_t)s * ABSB_HEAD_DIM + tid];
    float a = __builtin_fabsf(w);
    a = (a != a) ? 0.0f : a;  // a NaN never wins the maximum
    // wave-wide maximum (exact, order-free)
    for (int d = 32; d >= 1; d >>= 1) a = fmaxf(a, __shfl_xor(a, d));
    if ((tid & 63) == 0) s_absmax[tid >> 6] = a;
  }
  __syncthreads();
  const float A = fmaxf(s_absmax[0], s_absmax[1]);
  int ex = 0;
  const bool live = (A >= 0x1p-100f) && (A <= 3.4028234663852886e38f);
  if (live) ex = (int)((bitcast<uint32_t>(A) >> 23) & 0xffu) - 127 - 14;
  if (tid < ABSB_HEAD_DIM) {
    int32_t wq = 0;
    if (live) wq = (int32_t)__builtin_rintf(__builtin_ldexpf(w, -ex));
    s_wq[tid] = wq;
  }
  if (tid == 0 && blockIdx.x == 0 && p.score_exp) p.score_exp[s] = ex;
  __syncthreads();

  // ---- each lane: the 32 weights of its quarter of the channels
  int32_t wq[32];
#pragma unroll
  for (int i = 0; i < 32; ++i) wq[i] = s_wq[quarter * 32 + i];

  auto dot = [&](const uint4& c) -> int32_t {
    const uint32_t dw[4] = {c.x, c.y, c.z, c.w};
    int32_t acc = 0;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
#pragma unroll
      for (int n = 0; n < 8; ++n) acc += wq[k * 8 + n] * (int32_t)((dw[k] >> (4 * n)) & 15u);
    }
    return quad_sum(acc);  // the four lanes of a quad hold the four quarters of one centroid
  };

  // ---- main loop: 64 centroids per work-group step (16 per wave), PF steps per batch.
  // Every lane of a quad shares j, so the quad reduction always sees four live lanes.
  for (int jb = j0;;) {
#pragma unroll
    for (int u = 0; u < PF; ++u) {
      const int j = jb + u * 64 + (tid >> 2);
      const int32_t sc = dot(pre[u]);
      if (j < jend && quarter == 0) p.scores[off + j] = sc;
    }
    jb += PF * 64;
    if (jb >= jend) break;
#pragma unroll
    for (int u = 0; u < PF; ++u) {
      const int j = jb + u * 64 + (tid >> 2);
      pre[u] = j < jend ? *reinterpret_cast<const uint4*>(base + (size_t)j * 64) : make_uint4(0, 0, 0, 0);
    }
  }
}

int launch_score(const Geometry& g, const Plan& pl, int dtype, const void* q, const uint8_t* codes,
                 const float* qscale, const int32_t* cent_off, int32_t* scores, int32_t* score_exp,
                 hipStream_t stream) {
  ScoreParams p;
  p.q = static_cast<const uint16_t*>(q);
  p.codes = codes;
  p.qscale = qscale;
  p.cent_off = cent_off;
  p.scores = scores;
  p.score_exp = score_exp;
  p.Hq = g.Hq;
  p.Hkv = g.Hkv;
  p.G = g.G;
  p.chunk = pl.score_chunk;
  dim3 grid((unsigned)((pl.max_blocks + pl.score_chunk - 1) / pl.score_chunk), (unsigned)pl.nseg);
  if (dtype == ABSB_F16)
    hipLaunchKernelGGL(score_kernel<ABSB_F16>, grid, dim3(256), 0, stream, p);
  else
    hipLaunchKernelGGL(score_kernel<ABSB_BF16>, grid, dim3(256), 0, stream, p);
  return check_launch();
}

}  // namespace absb
