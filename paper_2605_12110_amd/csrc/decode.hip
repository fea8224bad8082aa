// Attention over the selected blocks (Sec. 3.4, kernel 3; Eq. (1) restricted to the selection).
//
// A selected logical block j of KV head h covers tokens [j*B_h, (j+1)*B_h); token t sits in
// physical page page_table[b][t / P] at slot t % P.  The kernel walks the selection as a virtual
// token sequence (position -> block list entry -> token -> page/slot) and reads K and V rows in
// place: no gather, no per-head page list, any mix of block sizes in one launch.
//
// Split-K flash decoding: work-group (split, segment) handles `split_tokens` consecutive positions
// of its segment's selection and emits an unnormalised partial (m, l, o~) for the G query heads
// of the group; a second kernel merges the partials with the log-sum-exp rule.
//
// Thread mapping: a K/V row is 256 bytes = 16 lanes x 16 bytes, so one wave load instruction
// covers four whole rows with 128-bit loads.  Each 16-lane row-group owns one row per step, keeps
// its own online-softmax state for the G heads (no cross-lane traffic in the main loop except the
// 16-lane DPP reduction of q.k), and each lane accumulates the 8 output channels it loaded.
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
  float* part_ml;  // [nseg][max_splits][G][2]  (running max in log2 units, sum)
  void* out;       // [Bt][Hq][128]
  float* lse;      // [Bt][Hq] or null
  int32_t sel_stride, split_tokens, max_splits;
  float scale_log2;  // sm_scale * log2(e)
  Geometry g;
};

constexpr float M_INIT = -1.0e30f;  // finite stand-in for "no token seen yet"
constexpr int DEC_THREADS = 256;
constexpr int DEC_WAVES = DEC_THREADS / 64;
constexpr int ROWS_PER_WAVE_STEP = 16;  // 4 row-groups x 4 rows

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

template <int DT, int G>
__global__ __launch_bounds__(DEC_THREADS) void decode_partial_kernel(DecodeParams p) {
  const int s = blockIdx.y, split = blockIdx.x;
  const int b = s / p.g.Hkv, h = s % p.g.Hkv;
  const int lb = p.g.heads.log2_block[h];
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, grp = lane >> 4, li = lane & 15;
  const int32_t* sel = p.sel_idx + (size_t)s * p.sel_stride;
  const int pos_begin = split * p.split_tokens;

  // The first step's list entries are fetched before the list length is known (the address is
  // clamped to the list's storage, so the read is always legal); this takes one memory round
  // trip off the dependent chain count -> entry -> page -> row.
  const int maxpos = (p.sel_stride << lb) - 1;
  int selj[4];
#pragma unroll
  for (int r = 0; r < 4; ++r)
    selj[r] = sel[min(pos_begin + wave * ROWS_PER_WAVE_STEP + r * 4 + grp, maxpos) >> lb];

  // never beyond what the launch covers (a list longer than promised is cut, not overrun)
  const int ntok = min(p.sel_cnt[s] << lb, p.max_splits * p.split_tokens);
  if (pos_begin >= ntok) return;
  const int pos_end = min(ntok, pos_begin + p.split_tokens);
  const int L = p.seq_lens[b];
  const int lP = p.g.log2_page;

  const int32_t* pt = p.page_table + (size_t)b * p.g.pt_stride;
  const size_t lane_off = (size_t)h * p.g.s_head + (size_t)li * 8;

  // the lane's 8 channels of the G queries, as packed pairs
  uint32_t qr[G][4];
#pragma unroll
  for (int g = 0; g < G; ++g) {
    const uint4 t = *reinterpret_cast<const uint4*>(p.q + ((size_t)b * p.g.Hq + (size_t)h * G + g) * ABSB_HEAD_DIM +
                                                    li * 8);
    qr[g][0] = t.x;
    qr[g][1] = t.y;
    qr[g][2] = t.z;
    qr[g][3] = t.w;
  }

  float m[G], l[G], o[G][8];
#pragma unroll
  for (int g = 0; g < G; ++g) {
    m[g] = M_INIT;
    l[g] = 0.0f;
#pragma unroll
    for (int c = 0; c < 8; ++c) o[g][c] = 0.0f;
  }

  for (int base = pos_begin + wave * ROWS_PER_WAVE_STEP; base < pos_end; base += DEC_WAVES * ROWS_PER_WAVE_STEP) {
    // ---- block -> page mapping for this group's four rows
    size_t off[4];
    bool valid[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int pos = base + r * 4 + grp;
      const bool in = pos < pos_end;
      const int t = (selj[r] << lb) + (pos & ((1 << lb) - 1));
      valid[r] = in && t < L;                // a selected last block may be partial
      const int tc = max(0, min(t, L - 1));  // addresses stay inside the request's pages
      const int page = pt[tc >> lP];
      off[r] = (size_t)page * p.g.s_page + lane_off + (size_t)(tc & ((1 << lP) - 1)) * p.g.s_tok;
    }
    uint4 kk[4], vv[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) kk[r] = *reinterpret_cast<const uint4*>(p.k + off[r]);
#pragma unroll
    for (int r = 0; r < 4; ++r) vv[r] = *reinterpret_cast<const uint4*>(p.v + off[r]);
    // list entries of the next step, in flight behind the rows
#pragma unroll
    for (int r = 0; r < 4; ++r)
      selj[r] = sel[min(base + DEC_WAVES * ROWS_PER_WAVE_STEP + r * 4 + grp, maxpos) >> lb];

    // ---- logits (log2 units) of the four rows for the G heads
    float sc[G][4];
#pragma unroll
    for (int r = 0; r < 4; ++r) {
#pragma unroll
      for (int g = 0; g < G; ++g) {
        float a = Elem<DT>::dot2(qr[g][0], kk[r].x, 0.0f);
        a = Elem<DT>::dot2(qr[g][1], kk[r].y, a);
        a = Elem<DT>::dot2(qr[g][2], kk[r].z, a);
        a = Elem<DT>::dot2(qr[g][3], kk[r].w, a);
        a = row16_sum(a);
        sc[g][r] = valid[r] ? a * p.scale_log2 : -__builtin_inff();
      }
    }

    // ---- online softmax over the tile and P.V
#pragma unroll
    for (int g = 0; g < G; ++g) {
      const float mn = fmaxf(fmaxf(m[g], fmaxf(sc[g][0], sc[g][1])), fmaxf(sc[g][2], sc[g][3]));
      const float alpha = fast_exp2(m[g] - mn);
      float pr[4];
#pragma unroll
      for (int r = 0; r < 4; ++r) pr[r] = fast_exp2(sc[g][r] - mn);
      l[g] = __builtin_fmaf(l[g], alpha, (pr[0] + pr[1]) + (pr[2] + pr[3]));
      m[g] = mn;
#pragma unroll
      for (int c = 0; c < 8; ++c) o[g][c] *= alpha;
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const uint32_t vw[4] = {vv[r].x, vv[r].y, vv[r].z, vv[r].w};
#pragma unroll
        for (int c = 0; c < 4; ++c) {
          o[g][2 * c] = __builtin_fmaf(pr[r], Elem<DT>::lo(vw[c]), o[g][2 * c]);
          o[g][2 * c + 1] = __builtin_fmaf(pr[r], Elem<DT>::hi(vw[c]), o[g][2 * c + 1]);
        }
      }
    }
  }

  // ---- merge the work-group's 16 row-group states through LDS and write the split's partial.
  // Three short phases, each a batch of independent LDS accesses (one round trip each): publish
  // the maxima; rescale the own state to the common maximum and publish it; add the 16 states up.
  constexpr int PARTS = DEC_WAVES * 4;
  constexpr int GC = G < 4 ? G : 4;  // heads staged per pass (bounds LDS at 32 KiB)
  __shared__ float s_o[PARTS][GC][ABSB_HEAD_DIM];
  __shared__ float s_m[G][PARTS], s_l[G][PARTS];
  const int part = wave * 4 + grp;
  if (li == 0) {
#pragma unroll
    for (int g = 0; g < G; ++g) s_m[g][part] = m[g];
  }
  __syncthreads();
  // every lane: the work-group maximum per head, and its own state rescaled to it, so that the
  // 16 states can then be added up as they are (all LDS reads below are independent: one round trip)
  float Mg[G];
#pragma unroll
  for (int g = 0; g < G; ++g) {
    float mx = s_m[g][0];
#pragma unroll
    for (int q = 1; q < PARTS; ++q) mx = fmaxf(mx, s_m[g][q]);
    Mg[g] = mx;
    const float a = fast_exp2(m[g] - mx);
    l[g] *= a;
#pragma unroll
    for (int c = 0; c < 8; ++c) o[g][c] *= a;
  }
  if (li == 0) {
#pragma unroll
    for (int g = 0; g < G; ++g) s_l[g][part] = l[g];  // own slot: nobody else reads or writes it before the barrier
  }
  const size_t slot = (size_t)s * p.max_splits + split;
#pragma unroll
  for (int g0 = 0; g0 < G; g0 += GC) {
    if (g0 > 0) __syncthreads();
#pragma unroll
    for (int k = 0; k < GC; ++k) {
      if (g0 + k < G) {
        float4* dst = reinterpret_cast<float4*>(&s_o[part][k][li * 8]);
        dst[0] = make_float4(o[g0 + k][0], o[g0 + k][1], o[g0 + k][2], o[g0 + k][3]);
        dst[1] = make_float4(o[g0 + k][4], o[g0 + k][5], o[g0 + k][6], o[g0 + k][7]);
      }
    }
    __syncthreads();
    constexpr int NOUT = (G - 0 < GC ? G : GC) * ABSB_HEAD_DIM;  // outputs of a full pass
    const int nout = (G - g0 < GC ? G - g0 : GC) * ABSB_HEAD_DIM;
#pragma unroll
    for (int i0 = 0; i0 < NOUT; i0 += DEC_THREADS) {
      const int i = i0 + tid;
      if (i < nout) {
        const int k = i >> 7, c = i & 127, g = g0 + k;
        float O = s_o[0][k][c], Lsum = s_l[g][0];
#pragma unroll
        for (int q = 1; q < PARTS; ++q) {
          O += s_o[q][k][c];
          Lsum += s_l[g][q];
        }
        p.part_o[(slot * G + g) * ABSB_HEAD_DIM + c] = O;
        if (c == 0) {
          float mx = Mg[0];
#pragma unroll
          for (int gg = 1; gg < G; ++gg) mx = (gg == g) ? Mg[gg] : mx;
          p.part_ml[(slot * G + g) * 2 + 0] = mx;
          p.part_ml[(slot * G + g) * 2 + 1] = Lsum;
        }
      }
    }
  }
}

// Log-sum-exp merge of a segment's split partials.  One work-group per (query head, segment):
// 128 channels x 8 split lanes; a thread takes every 8th split, with up to MRG_UNROLL independent
// loads in flight, so the whole merge costs about one memory round trip.
constexpr int MRG_THREADS = 1024;
constexpr int MRG_LANES = MRG_THREADS / ABSB_HEAD_DIM;
constexpr int MRG_UNROLL = 8;

template <int DT>
__global__ __launch_bounds__(MRG_THREADS) void decode_merge_kernel(DecodeParams p) {
  const int s = blockIdx.y, g = blockIdx.x;
  const int G = p.g.G;
  const int b = s / p.g.Hkv, h = s % p.g.Hkv;
  const int lb = p.g.heads.log2_block[h];
  const int tid = threadIdx.x, c = tid & 127, sl = tid >> 7, lane = tid & 63, wave = tid >> 6;
  const size_t slot0 = (size_t)s * p.max_splits;
  const float2* ml = reinterpret_cast<const float2*>(p.part_ml);

  // first batch of partials: issued before the split count is known (slots up to max_splits
  // exist for every segment; unused ones hold stale bytes and are masked out below)
  float2 mlv[MRG_UNROLL];
  float ov[MRG_UNROLL];
#pragma unroll
  for (int u = 0; u < MRG_UNROLL; ++u) {
    const int i = min(sl + u * MRG_LANES, p.max_splits - 1);
    mlv[u] = ml[(slot0 + i) * G + g];
    ov[u] = p.part_o[((slot0 + i) * G + g) * ABSB_HEAD_DIM + c];
  }
  const int ntok = min(p.sel_cnt[s] << lb, p.max_splits * p.split_tokens);
  const int nsplit = (ntok + p.split_tokens - 1) / p.split_tokens;
#pragma unroll
  for (int u = 0; u < MRG_UNROLL; ++u) {
    const bool in = sl + u * MRG_LANES < nsplit;
    mlv[u] = in ? mlv[u] : make_float2(M_INIT, 0.0f);
    ov[u] = in ? ov[u] : 0.0f;
  }

  // global maximum over the splits
  float M = M_INIT;
#pragma unroll
  for (int u = 0; u < MRG_UNROLL; ++u) M = fmaxf(M, mlv[u].x);  // the work-group's lanes cover splits 0..63
  for (int i = MRG_UNROLL * MRG_LANES + tid; i < nsplit; i += MRG_THREADS) M = fmaxf(M, ml[(slot0 + i) * G + g].x);
  for (int d = 32; d >= 1; d >>= 1) M = fmaxf(M, __shfl_xor(M, d));
  __shared__ float s_max[MRG_THREADS / 64];
  __shared__ float s_acc[MRG_LANES][ABSB_HEAD_DIM], s_l[MRG_LANES];
  if (lane == 0) s_max[wave] = M;
  __syncthreads();
#pragma unroll
  for (int w = 0; w < MRG_THREADS / 64; ++w) M = fmaxf(M, s_max[w]);

  float acc = 0.0f, lacc = 0.0f;
#pragma unroll
  for (int u = 0; u < MRG_UNROLL; ++u) {
    const float w = fast_exp2(mlv[u].x - M);
    acc = __builtin_fmaf(ov[u], w, acc);
    lacc = __builtin_fmaf(mlv[u].y, w, lacc);
  }
  for (int i0 = sl + MRG_UNROLL * MRG_LANES; i0 < nsplit; i0 += MRG_UNROLL * MRG_LANES) {
#pragma unroll
    for (int u = 0; u < MRG_UNROLL; ++u) {
      const int i = i0 + u * MRG_LANES;
      const bool in = i < nsplit;
      mlv[u] = in ? ml[(slot0 + i) * G + g] : make_float2(M_INIT, 0.0f);
      ov[u] = in ? p.part_o[((slot0 + i) * G + g) * ABSB_HEAD_DIM + c] : 0.0f;
    }
#pragma unroll
    for (int u = 0; u < MRG_UNROLL; ++u) {
      const float w = fast_exp2(mlv[u].x - M);
      acc = __builtin_fmaf(ov[u], w, acc);
      lacc = __builtin_fmaf(mlv[u].y, w, lacc);
    }
  }
  s_acc[sl][c] = acc;
  if (c == 0) s_l[sl] = lacc;
  __syncthreads();
  if (sl == 0) {
    float O = s_acc[0][c], Lsum = s_l[0];
#pragma unroll
    for (int k = 1; k < MRG_LANES; ++k) {
      O += s_acc[k][c];
      Lsum += s_l[k];
    }
    const bool any = Lsum > 0.0f;
    const float res = any ? O / Lsum : 0.0f;
    const size_t row = (size_t)b * p.g.Hq + (size_t)h * G + g;
    static_cast<uint16_t*>(p.out)[row * ABSB_HEAD_DIM + c] = Elem<DT>::narrow(res);
    if (p.lse && c == 0)
      p.lse[row] = any ? (M + __builtin_log2f(Lsum)) * 0.6931471805599453f : -__builtin_inff();
  }
}

template <int DT>
static void launch_partial(const DecodeParams& p, dim3 grid, hipStream_t stream) {
  switch (p.g.G) {
    case 1: hipLaunchKernelGGL((decode_partial_kernel<DT, 1>), grid, dim3(DEC_THREADS), 0, stream, p); break;
    case 2: hipLaunchKernelGGL((decode_partial_kernel<DT, 2>), grid, dim3(DEC_THREADS), 0, stream, p); break;
    case 3: hipLaunchKernelGGL((decode_partial_kernel<DT, 3>), grid, dim3(DEC_THREADS), 0, stream, p); break;
    case 4: hipLaunchKernelGGL((decode_partial_kernel<DT, 4>), grid, dim3(DEC_THREADS), 0, stream, p); break;
    case 5: hipLaunchKernelGGL((decode_partial_kernel<DT, 5>), grid, dim3(DEC_THREADS), 0, stream, p); break;
    case 6: hipLaunchKernelGGL((decode_partial_kernel<DT, 6>), grid, dim3(DEC_THREADS), 0, stream, p); break;
    case 7: hipLaunchKernelGGL((decode_partial_kernel<DT, 7>), grid, dim3(DEC_THREADS), 0, stream, p); break;
    default: hipLaunchKernelGGL((decode_partial_kernel<DT, 8>), grid, dim3(DEC_THREADS), 0, stream, p); break;
  }
}

int launch_decode(const Geometry& g, const Plan& pl, int dtype, float sm_scale, const void* q,
                  const void* k_cache, const void* v_cache, const int32_t* page_table, const int32_t* seq_lens,
                  const int32_t* sel_idx, const int32_t* sel_cnt, int32_t sel_stride, void* out, float* lse,
                  char* ws, hipStream_t stream) {
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
  p.out = out;
  p.lse = lse;
  p.sel_stride = sel_stride;
  p.split_tokens = pl.split_tokens;
  p.max_splits = pl.max_splits;
  p.scale_log2 = sm_scale * 1.4426950408889634f;
  p.g = g;
  dim3 grid((unsigned)pl.max_splits, (unsigned)pl.nseg);
  if (dtype == ABSB_F16)
    launch_partial<ABSB_F16>(p, grid, stream);
  else
    launch_partial<ABSB_BF16>(p, grid, stream);
  int rc = check_launch();
  if (rc != ABSB_OK) return rc;
  if (dtype == ABSB_F16)
    hipLaunchKernelGGL(decode_merge_kernel<ABSB_F16>, dim3((unsigned)g.G, (unsigned)pl.nseg), dim3(MRG_THREADS), 0, stream, p);
  else
    hipLaunchKernelGGL(decode_merge_kernel<ABSB_BF16>, dim3((unsigned)g.G, (unsigned)pl.nseg), dim3(MRG_THREADS), 0, stream, p);
  return check_launch();
}

}  // namespace absb
