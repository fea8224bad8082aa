// Centroid store build: block pooling (mean pooling, or channel-wise maxima and minima: Sec. 2.2 and
// its footnote), per-channel asymmetric INT4 quantization (Sec. 3.3) and the flattened,
// prefix-sum-delimited code array (Sec. 3.4, kernel 1).  Runs once per context (prefill side), reads
// every key once.
//
// A block is a row of W = 128 * R values: R = 1 the mean, R = 2 the maxima followed by the minima.
//
// Arithmetic is fixed so that the 4-bit codes are reproducible bit for bit: binary32 running sum
// of a block's keys in token order, one IEEE division by the number of valid tokens (extrema need
// comparisons only), exact min/max per (segment, value), scale = (max-min)/15 and 15/(max-min) as two
// IEEE divisions, code = clamp(round-half-even((c - min) * (15/(max-min)))).  Compiled with
// -ffp-contract=off.
//
// Three launches:
//   1. pool: a work-group owns `chunk_tokens` consecutive tokens of a segment (a power-of-two number
//      of whole blocks, at least one per 16-lane row-group), so work per group is the same for every
//      block size.  A row-group (each lane 8 channels = one 128-bit load per key) streams its 64+
//      consecutive tokens eight rows at a time, the next eight in flight while these are pooled,
//      closes a block whenever the running token index reaches a block boundary, writes the binary32
//      row to the workspace and folds it into per-work-group minima/maxima per value;
//   2. params: reduces the partial extrema per segment and writes qscale, qmin (and 15/range);
//   3. codes: quantizes the rows, eight values per lane packed into one 32-bit store.
#include "common.h"

namespace absb {

struct BuildParams {
  const uint16_t* k;
  const int32_t* page_table;
  const int32_t* seq_lens;
  const int32_t* cent_off;
  float* cent;     // [total][W]
  float* minmax;   // [nseg][max_chunks][2][W]
  float* qinv;     // [nseg][W]
  float* qscale;   // [nseg][W]
  float* qmin;     // [nseg][W]
  uint8_t* codes;  // [total][W/2]
  int32_t chunk_tokens, max_chunks;
  Geometry g;
};

constexpr int BUILD_THREADS = 256;
constexpr int BUILD_GROUPS = BUILD_THREADS / 16;
constexpr int BUILD_ROWS = 8;  // rows per step: B >= 8 and P >= 8, so a step never straddles a block or a page

// blocks per work-group for a head with blocks of 2^lb tokens
__device__ __forceinline__ int build_chunk_blocks(int chunk_tokens, int lb) {
  return max(BUILD_GROUPS, chunk_tokens >> lb);
}

template <int DT, int REP>
__global__ __launch_bounds__(BUILD_THREADS) void build_pool_kernel(BuildParams p) {
  constexpr int W = ABSB_HEAD_DIM * (REP + 1);
  const int s = blockIdx.y, chunk = blockIdx.x;
  const int off = p.cent_off[s];
  const int b = s / p.g.Hkv, h = s % p.g.Hkv;
  const int lb = p.g.heads.log2_block[h], lP = p.g.log2_page;
  const int L = p.seq_lens[b];
  const int N = blocks_in_use(p.g.tight, p.cent_off[s + 1] - off, p.seq_lens, b, lb);
  const int cb = build_chunk_blocks(p.chunk_tokens, lb);
  const int j0 = chunk * cb;
  if (j0 >= N) return;
  const int jend = min(N, j0 + cb);
  const int B = 1 << lb;
  const int tid = threadIdx.x, grp = tid >> 4, li = tid & 15;
  const int32_t* pt = p.page_table + (size_t)b * p.g.pt_stride;
  const size_t lane_off = (size_t)h * p.g.s_head + (size_t)li * 8;

  // running extrema over this row-group's blocks, per vector of the row (v = 0: mean or maxima, 1: minima)
  float mn[REP + 1][8], mx[REP + 1][8];
#pragma unroll
  for (int v = 0; v <= REP; ++v)
#pragma unroll
    for (int c = 0; c < 8; ++c) {
      mn[v][c] = __builtin_inff();
      mx[v][c] = -__builtin_inff();
    }

  // this row-group's blocks [ja, jb) = consecutive tokens [tA, tB)
  const int per = cb / BUILD_GROUPS;
  const int ja = min(jend, j0 + grp * per), jb = min(jend, ja + per);
  const int tA = ja << lb, tB = min(jb << lb, L);

  auto row_base = [&](int t) -> const uint16_t* {  // first row of the 8-row step at token t (t < L)
    const int page = pt[t >> lP];
    return p.k + (size_t)page * p.g.s_page + lane_off + (size_t)(t & ((1 << lP) - 1)) * p.g.s_tok;
  };

  if (tA < tB) {
    uint4 cur[BUILD_ROWS], nxt[BUILD_ROWS];
    const uint16_t* base = row_base(tA);
#pragma unroll
    for (int r = 0; r < BUILD_ROWS; ++r)  // rows past the end repeat the last one (a legal address), masked below
      cur[r] = *reinterpret_cast<const uint4*>(base + (size_t)min(r, tB - 1 - tA) * p.g.s_tok);
#pragma unroll
    for (int r = 0; r < BUILD_ROWS; ++r) nxt[r] = cur[r];
    const uint16_t* base_next = row_base(min(tA + BUILD_ROWS, tB - 1));

    // the open block: its running sum (mean pooling) or its maxima / minima so far
    float acc[REP + 1][8];
    auto reset = [&]() {
#pragma unroll
      for (int c = 0; c < 8; ++c) {
        acc[0][c] = REP ? -__builtin_inff() : 0.0f;
        if (REP) acc[REP][c] = __builtin_inff();
      }
    };
    reset();
    for (int i = tA; i < tB; i += BUILD_ROWS) {
      const int in = i + BUILD_ROWS;
      if (in < tB) {
#pragma unroll
        for (int r = 0; r < BUILD_ROWS; ++r)
          nxt[r] = *reinterpret_cast<const uint4*>(base_next + (size_t)min(r, tB - 1 - in) * p.g.s_tok);
        base_next = row_base(min(in + BUILD_ROWS, tB - 1));
      }
#pragma unroll
      for (int r = 0; r < BUILD_ROWS; ++r) {
        if (i + r < tB) {
          const uint32_t w[4] = {cur[r].x, cur[r].y, cur[r].z, cur[r].w};
#pragma unroll
          for (int c = 0; c < 4; ++c) {
            const float lo = Elem<DT>::lo(w[c]), hi = Elem<DT>::hi(w[c]);
            if (REP) {
              acc[0][2 * c] = fmaxf(acc[0][2 * c], lo);
              acc[0][2 * c + 1] = fmaxf(acc[0][2 * c + 1], hi);
              acc[REP][2 * c] = fminf(acc[REP][2 * c], lo);
              acc[REP][2 * c + 1] = fminf(acc[REP][2 * c + 1], hi);
            } else {
              acc[0][2 * c] = acc[0][2 * c] + lo;
              acc[0][2 * c + 1] = acc[0][2 * c + 1] + hi;
            }
          }
        }
      }
      if ((in & (B - 1)) == 0 || in >= tB) {  // the block that holds token i is complete
        const int j = i >> lb;
        const float fn = (float)min(B, L - (j << lb));
#pragma unroll
        for (int v = 0; v <= REP; ++v) {
          float val[8];
#pragma unroll
          for (int c = 0; c < 8; ++c) {
            val[c] = REP ? acc[v][c] : acc[v][c] / fn;
            mn[v][c] = fminf(mn[v][c], val[c]);
            mx[v][c] = fmaxf(mx[v][c], val[c]);
          }
          float4* dst = reinterpret_cast<float4*>(p.cent + ((size_t)off + j) * W + v * ABSB_HEAD_DIM + li * 8);
          dst[0] = make_float4(val[0], val[1], val[2], val[3]);
          dst[1] = make_float4(val[4], val[5], val[6], val[7]);
        }
        reset();
      }
#pragma unroll
      for (int r = 0; r < BUILD_ROWS; ++r) cur[r] = nxt[r];
    }
  }

  // fold the 16 row-groups: value index = v*128 + li*8 + c
  __shared__ float s_mn[BUILD_GROUPS][W], s_mx[BUILD_GROUPS][W];
#pragma unroll
  for (int v = 0; v <= REP; ++v)
#pragma unroll
    for (int c = 0; c < 8; ++c) {
      s_mn[grp][v * ABSB_HEAD_DIM + li * 8 + c] = mn[v][c];
      s_mx[grp][v * ABSB_HEAD_DIM + li * 8 + c] = mx[v][c];
    }
  __syncthreads();
  if (tid < W) {
    float a = s_mn[0][tid], z = s_mx[0][tid];
#pragma unroll
    for (int g2 = 1; g2 < BUILD_GROUPS; ++g2) {
      a = fminf(a, s_mn[g2][tid]);
      z = fmaxf(z, s_mx[g2][tid]);
    }
    float* dst = p.minmax + ((size_t)s * p.max_chunks + chunk) * 2 * W;
    dst[tid] = a;
    dst[W + tid] = z;
  }
}

// One work-group per (segment, vector of the row): 128 values x 8 chunk lanes; min/max are exact
// in any order.
constexpr int PARAMS_THREADS = 1024;
constexpr int PARAMS_LANES = PARAMS_THREADS / ABSB_HEAD_DIM;

__global__ __launch_bounds__(PARAMS_THREADS) void build_params_kernel(BuildParams p) {
  const int W = ABSB_HEAD_DIM * (p.g.repr + 1);
  const int s = blockIdx.x, cl = threadIdx.x / ABSB_HEAD_DIM;
  const int ch = blockIdx.y * ABSB_HEAD_DIM + (threadIdx.x & (ABSB_HEAD_DIM - 1));  // value index in the row
  const int h = s % p.g.Hkv;
  const int N = blocks_in_use(p.g.tight, p.cent_off[s + 1] - p.cent_off[s], p.seq_lens, s / p.g.Hkv,
                              p.g.heads.log2_block[h]);
  const int cb = build_chunk_blocks(p.chunk_tokens, p.g.heads.log2_block[h]);
  const int nchunks = (N + cb - 1) / cb;
  float mn = __builtin_inff(), mx = -__builtin_inff();
  for (int i0 = cl; i0 < nchunks; i0 += 4 * PARAMS_LANES) {
    float a[4], z[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int i = min(i0 + u * PARAMS_LANES, nchunks - 1);  // the tail repeats a chunk: harmless for min/max
      const float* src = p.minmax + ((size_t)s * p.max_chunks + i) * 2 * W;
      a[u] = src[ch];
      z[u] = src[W + ch];
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      mn = fminf(mn, a[u]);
      mx = fmaxf(mx, z[u]);
    }
  }
  __shared__ float s_mn[PARAMS_LANES][ABSB_HEAD_DIM], s_mx[PARAMS_LANES][ABSB_HEAD_DIM];
  const int c = threadIdx.x & (ABSB_HEAD_DIM - 1);
  s_mn[cl][c] = mn;
  s_mx[cl][c] = mx;
  __syncthreads();
  if (cl != 0) return;
#pragma unroll
  for (int k = 1; k < PARAMS_LANES; ++k) {
    mn = fminf(mn, s_mn[k][c]);
    mx = fmaxf(mx, s_mx[k][c]);
  }
  const float rng = mx - mn;
  float sc = 0.0f, inv = 0.0f;
  if (rng > 0.0f) {
    sc = rng / 15.0f;
    inv = 15.0f / rng;
  }
  if (N == 0) mn = 0.0f;
  p.qscale[(size_t)s * W + ch] = sc;
  p.qmin[(size_t)s * W + ch] = mn;
  p.qinv[(size_t)s * W + ch] = inv;
}

// grid (chunk, segment, vector of the row)
__global__ __launch_bounds__(BUILD_THREADS) void build_codes_kernel(BuildParams p) {
  const int W = ABSB_HEAD_DIM * (p.g.repr + 1);
  const int s = blockIdx.y, v = blockIdx.z;
  const int off = p.cent_off[s];
  const int lb = p.g.heads.log2_block[s % p.g.Hkv];
  const int N = blocks_in_use(p.g.tight, p.cent_off[s + 1] - off, p.seq_lens, s / p.g.Hkv, lb);
  const int cb = build_chunk_blocks(p.chunk_tokens, lb);
  const int j0 = blockIdx.x * cb;
  if (j0 >= N) return;
  const int jend = min(N, j0 + cb);
  const int tid = threadIdx.x, grp = tid >> 4, li = tid & 15;
  const int col = v * ABSB_HEAD_DIM + li * 8;  // first of this lane's eight values in the row
  float mn[8], inv[8];
#pragma unroll
  for (int c = 0; c < 8; ++c) {
    mn[c] = p.qmin[(size_t)s * W + col + c];
    inv[c] = p.qinv[(size_t)s * W + col + c];
  }
  for (int j = j0 + grp; j < jend; j += BUILD_GROUPS) {
    const float4* src = reinterpret_cast<const float4*>(p.cent + ((size_t)off + j) * W + col);
    const float4 a = src[0], z = src[1];
    const float cen[8] = {a.x, a.y, a.z, a.w, z.x, z.y, z.z, z.w};
    uint32_t packed = 0;
#pragma unroll
    for (int c = 0; c < 8; ++c) {
      const float x = cen[c] - mn[c];
      const float y = x * inv[c];
      float r = __builtin_rintf(y);
      r = fminf(fmaxf(r, 0.0f), 15.0f);
      packed |= (uint32_t)r << (4 * c);
    }
    // byte i of a row holds value 2i (low nibble) and 2i+1 (high nibble): little-endian nibble n
    // of this word is value col + n
    *reinterpret_cast<uint32_t*>(p.codes + ((size_t)off + j) * (W / 2) + col / 2) = packed;
  }
}

// Decode-time maintenance.  A 16-lane row-group per segment (each lane 8 channels): folds the key
// of the newest token (position L - 1) into the pooled state of the segment's last block and
// re-emits that block's 4-bit row under the store's frozen ranges; with APPEND == false it only
// recomputes the state from the cache (the tokens of the last block, in order).  When the new token
// completes its block the row is final: the number of its values that the frozen range does not
// hold is then added to the segment's counter (the signal for a re-ranging policy).
struct AppendParams {
  const uint16_t* k;
  const int32_t* page_table;
  const int32_t* seq_lens;
  const int32_t* cent_off;
  uint8_t* codes;
  const float* qscale;
  const float* qmin;
  float* tail;  // [nseg][W]
  int32_t* clamped;  // [nseg] or null
  int32_t nseg;
  Geometry g;
};

template <int DT, int REP, bool APPEND>
__global__ __launch_bounds__(BUILD_THREADS) void append_kernel(AppendParams p) {
  constexpr int W = ABSB_HEAD_DIM * (REP + 1);
  const int tid = threadIdx.x, grp = tid >> 4, li = tid & 15;
  const int s = blockIdx.x * BUILD_GROUPS + grp;
  if (s >= p.nseg) return;
  const int b = s / p.g.Hkv, h = s % p.g.Hkv;
  const int lb = p.g.heads.log2_block[h], lP = p.g.log2_page;
  const int L = p.seq_lens[b];
  const int t_new = L - 1, j = t_new >> lb, t0 = j << lb;
  const int32_t* pt = p.page_table + (size_t)b * p.g.pt_stride;
  const size_t lane_off = (size_t)h * p.g.s_head + (size_t)li * 8;
  float* tail = p.tail + (size_t)s * W + li * 8;

  float st[REP + 1][8];
  const int t_first = APPEND ? t_new : t0;  // APPEND: one key on top of the stored state
  if (APPEND && t_new != t0) {
#pragma unroll
    for (int v = 0; v <= REP; ++v) {
      const float4 a = *reinterpret_cast<const float4*>(tail + v * ABSB_HEAD_DIM);
      const float4 z = *reinterpret_cast<const float4*>(tail + v * ABSB_HEAD_DIM + 4);
      st[v][0] = a.x, st[v][1] = a.y, st[v][2] = a.z, st[v][3] = a.w;
      st[v][4] = z.x, st[v][5] = z.y, st[v][6] = z.z, st[v][7] = z.w;
    }
  }
  for (int t = t_first; t <= t_new; ++t) {
    const int page = pt[t >> lP];
    const uint4 row = *reinterpret_cast<const uint4*>(p.k + (size_t)page * p.g.s_page + lane_off +
                                                      (size_t)(t & ((1 << lP) - 1)) * p.g.s_tok);
    const uint32_t w[4] = {row.x, row.y, row.z, row.w};
    const bool first = t == t0;  // the block's first key starts the state
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      const float lo = Elem<DT>::lo(w[c]), hi = Elem<DT>::hi(w[c]);
      if (REP) {
        st[0][2 * c] = first ? lo : fmaxf(st[0][2 * c], lo);
        st[0][2 * c + 1] = first ? hi : fmaxf(st[0][2 * c + 1], hi);
        st[REP][2 * c] = first ? lo : fminf(st[REP][2 * c], lo);
        st[REP][2 * c + 1] = first ? hi : fminf(st[REP][2 * c + 1], hi);
      } else {
        st[0][2 * c] = first ? lo : st[0][2 * c] + lo;
        st[0][2 * c + 1] = first ? hi : st[0][2 * c + 1] + hi;
      }
    }
  }
#pragma unroll
  for (int v = 0; v <= REP; ++v) {
    *reinterpret_cast<float4*>(tail + v * ABSB_HEAD_DIM) = make_float4(st[v][0], st[v][1], st[v][2], st[v][3]);
    *reinterpret_cast<float4*>(tail + v * ABSB_HEAD_DIM + 4) = make_float4(st[v][4], st[v][5], st[v][6], st[v][7]);
  }
  if (!APPEND) return;

  const float fn = (float)(t_new - t0 + 1);
  const size_t row_at = ((size_t)p.cent_off[s] + j) * (W / 2);
  int outside = 0;
#pragma unroll
  for (int v = 0; v <= REP; ++v) {
    const int col = v * ABSB_HEAD_DIM + li * 8;
    uint32_t packed = 0;
#pragma unroll
    for (int c = 0; c < 8; ++c) {
      const float value = REP ? st[v][c] : st[v][c] / fn;
      const float sc = p.qscale[(size_t)s * W + col + c];
      float r = 0.0f;
      if (sc > 0.0f) {
        const float inv = 1.0f / sc;
        const float x = value - p.qmin[(size_t)s * W + col + c];
        r = __builtin_rintf(x * inv);
        outside += !(r >= 0.0f && r <= 15.0f);
        r = fminf(fmaxf(r, 0.0f), 15.0f);  // a NaN ends up at 0
      } else {
        outside += value != p.qmin[(size_t)s * W + col + c];  // a channel that was constant at build time
      }
      packed |= (uint32_t)r << (4 * c);
    }
    *reinterpret_cast<uint32_t*>(p.codes + row_at + col / 2) = packed;
  }
  if (p.clamped && ((t_new + 1) & ((1 << lb) - 1)) == 0) {  // the block is complete (wave-uniform per row-group)
    outside += __shfl_xor(outside, 1);
    outside += __shfl_xor(outside, 2);
    outside += __shfl_xor(outside, 4);
    outside += __shfl_xor(outside, 8);
    // this row-group is the segment's only writer; an add without return value, so that nothing waits for it
    if (li == 0 && outside)
      __hip_atomic_fetch_add(p.clamped + s, outside, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
}

template <int DT, int REP>
static void launch_append_kernel(bool append, const AppendParams& p, hipStream_t stream) {
  const dim3 grid((unsigned)((p.nseg + BUILD_GROUPS - 1) / BUILD_GROUPS)), block(BUILD_THREADS);
  if (append)
    hipLaunchKernelGGL((append_kernel<DT, REP, true>), grid, block, 0, stream, p);
  else
    hipLaunchKernelGGL((append_kernel<DT, REP, false>), grid, block, 0, stream, p);
}

int launch_append(const Geometry& g, const Plan& pl, int dtype, bool append, const void* k_cache,
                  const int32_t* page_table, const int32_t* seq_lens, const int32_t* cent_off, uint8_t* codes,
                  const float* qscale, const float* qmin, float* tail, int32_t* clamped, hipStream_t stream) {
  AppendParams p;
  p.k = static_cast<const uint16_t*>(k_cache);
  p.page_table = page_table;
  p.seq_lens = seq_lens;
  p.cent_off = cent_off;
  p.codes = codes;
  p.qscale = qscale;
  p.qmin = qmin;
  p.tail = tail;
  p.clamped = clamped;
  p.nseg = pl.nstore;
  p.g = g;
  if (dtype == ABSB_F16 && g.repr == ABSB_REPR_MEAN)
    launch_append_kernel<ABSB_F16, 0>(append, p, stream);
  else if (dtype == ABSB_F16)
    launch_append_kernel<ABSB_F16, 1>(append, p, stream);
  else if (g.repr == ABSB_REPR_MEAN)
    launch_append_kernel<ABSB_BF16, 0>(append, p, stream);
  else
    launch_append_kernel<ABSB_BF16, 1>(append, p, stream);
  return check_launch();
}

int launch_build(const Geometry& g, const Plan& pl, int dtype, const void* k_cache, const int32_t* page_table,
                 const int32_t* seq_lens, const int32_t* cent_off, uint8_t* codes, float* qscale, float* qmin,
                 char* ws, hipStream_t stream) {
  BuildParams p;
  p.k = static_cast<const uint16_t*>(k_cache);
  p.page_table = page_table;
  p.seq_lens = seq_lens;
  p.cent_off = cent_off;
  p.cent = reinterpret_cast<float*>(ws + pl.ws_cent);
  p.minmax = reinterpret_cast<float*>(ws + pl.ws_minmax);
  p.qinv = reinterpret_cast<float*>(ws + pl.ws_qinv);
  p.qscale = qscale;
  p.qmin = qmin;
  p.codes = codes;
  p.chunk_tokens = pl.build_chunk_tokens;
  p.max_chunks = pl.build_max_chunks;
  p.g = g;
  const unsigned R = (unsigned)g.repr + 1;
  const dim3 grid((unsigned)pl.build_max_chunks, (unsigned)pl.nstore), block(BUILD_THREADS);
  if (dtype == ABSB_F16 && g.repr == ABSB_REPR_MEAN)
    hipLaunchKernelGGL((build_pool_kernel<ABSB_F16, 0>), grid, block, 0, stream, p);
  else if (dtype == ABSB_F16)
    hipLaunchKernelGGL((build_pool_kernel<ABSB_F16, 1>), grid, block, 0, stream, p);
  else if (g.repr == ABSB_REPR_MEAN)
    hipLaunchKernelGGL((build_pool_kernel<ABSB_BF16, 0>), grid, block, 0, stream, p);
  else
    hipLaunchKernelGGL((build_pool_kernel<ABSB_BF16, 1>), grid, block, 0, stream, p);
  int rc = check_launch();
  if (rc != ABSB_OK) return rc;
  hipLaunchKernelGGL(build_params_kernel, dim3((unsigned)pl.nstore, R), dim3(PARAMS_THREADS), 0, stream, p);
  rc = check_launch();
  if (rc != ABSB_OK) return rc;
  hipLaunchKernelGGL(build_codes_kernel, dim3(grid.x, grid.y, R), block, 0, stream, p);
  return check_launch();
}

}  // namespace absb
