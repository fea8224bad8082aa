/*
 * CPU oracle for adaptive-block sparse decode attention (AB-Sparse).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the plain, slow, obviously-correct statement
 * of what the decode path computes.  It shares no code, header, table or helper with
 * the HIP library, is never linked into it, and may be used only by the tests, by the
 * smoke check and by the benchmark's CPU-baseline leg.
 *
 * What it follows, step by step, in the paper's order and notation:
 *   - block-sparse workflow (Sec. 2.2): partition each head's keys into blocks of size
 *     B_h, one centroid c_j per block, importance r_j = q . c_j^T, Top-K blocks, attention
 *     over the selected blocks only;
 *   - centroid = mean pooling of the block's keys (Sec. 2.2, footnote on pooling); as a
 *     second representation, the max-min pooling the same footnote names (channel-wise
 *     maxima and minima of the block, scored by their channel-wise upper bound of q . k);
 *   - INT4 asymmetric per-channel centroid quantization: one scale and one zero-point
 *     offset per head-dim channel, shared by all blocks of a head (Sec. 3.3);
 *   - flattened 1-D centroid layout, offset[s+1] = offset[s] + N_s (Sec. 3.4, kernel 1);
 *   - per-head K_h = ceil(T / B_h) under a token budget T (Sec. 3.4, kernel 2);
 *   - a selected logical block maps onto fixed-size physical pages through the page
 *     table with no data movement (Sec. 3.4, kernel 3);
 *   - softmax attention, Eq. (1), restricted to the selected tokens; GQA: G = Hq/Hkv
 *     query heads share one KV head.
 *
 * Where the paper is silent the reading is fixed here once (and listed in the design
 * notes): one segment per (request, KV head), request-major; the G query heads of a
 * group are folded by summation before scoring (the score is linear in q); the last
 * block may be partial and its centroid is the mean of its valid keys only; ties in
 * Top-K go to the lowest block index and the index list is emitted ascending; scoring
 * is carried out in exact integers on a 16-bit fixed-point image of (q * scale) so that
 * the ranking has exactly one correct answer on any machine.
 *
 * Arithmetic: steps that decide integers (codes, scores, selected indices) use IEEE
 * binary32 single operations in the stated order (compile with -ffp-contract=off, no
 * fast-math); attention is evaluated in binary64 from the exactly widened inputs.
 *
 * Parity pins (tests/test_oracle_*.py): every function here is pinned to something
 * other than itself - fp64 means, quantization error bound/idempotence/extremes,
 * an independent fp64 dot-product bound for the scores, numpy lexsort and exhaustive
 * tiny cases for Top-K, an independent numpy dense softmax (Eq. 1) for attention with
 * K = all blocks, page-permutation invariance, and single-token / equal-key closed forms;
 * the max-min representation to numpy extrema, to the bound property q . k_t <= score for
 * every token of the block, and to an fp64 evaluation of the max formula.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

enum { ORC_F16 = 0, ORC_BF16 = 1 };

/* ---- exact widening of the 16-bit storage formats -------------------------------- */
static float widen_f16(uint16_t h) {
    uint32_t sign = (uint32_t)(h & 0x8000u) << 16;
    uint32_t ex = (h >> 10) & 0x1Fu;
    uint32_t man = h & 0x3FFu;
    uint32_t out;
    if (ex == 0) {
        if (man == 0) {
            out = sign;
        } else { /* subnormal: value = man * 2^-24, exact in binary32 */
            float v = (float)man * 0x1p-24f;
            memcpy(&out, &v, 4);
            out |= sign;
        }
    } else if (ex == 31) {
        out = sign | 0x7F800000u | (man << 13);
    } else {
        out = sign | ((ex + 112u) << 23) | (man << 13);
    }
    float f;
    memcpy(&f, &out, 4);
    return f;
}

static float widen_bf16(uint16_t h) {
    uint32_t out = (uint32_t)h << 16;
    float f;
    memcpy(&f, &out, 4);
    return f;
}

static float widen(uint16_t bits, int dtype) { return dtype == ORC_F16 ? widen_f16(bits) : widen_bf16(bits); }

/* row of logical token t of (request b, KV head h) in a paged cache */
typedef struct {
    const uint16_t *base;
    const int32_t *page_table; /* [Bt][pt_stride] */
    int32_t pt_stride, P;
    int64_t s_page, s_head, s_tok; /* element strides; channels contiguous */
} paged_t;

static const uint16_t *row_of(const paged_t *c, int b, int h, int64_t t) {
    int64_t page = c->page_table[(int64_t)b * c->pt_stride + t / c->P];
    return c->base + page * c->s_page + (int64_t)h * c->s_head + (t % c->P) * c->s_tok;
}

static int64_t ceil_div64(int64_t a, int64_t b) { return (a + b - 1) / b; }

int orc_num_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

void orc_set_threads(int n) {
#ifdef _OPENMP
    if (n > 0) omp_set_num_threads(n);
#else
    (void)n;
#endif
}

/* ---- segment layout: offset[s+1] = offset[s] + N_s, N_s = ceil(L_b / B_h) ----------
 * (Sec. 3.4, kernel 1; one segment per (request, KV head), s = b*Hkv + h).
 * Returns the total number of centroids. */
int64_t orc_offsets(int Bt, int Hkv, const int32_t *seq_lens, const int32_t *block_size, int64_t *off) {
    off[0] = 0;
    for (int b = 0; b < Bt; ++b)
        for (int h = 0; h < Hkv; ++h) {
            int s = b * Hkv + h;
            off[s + 1] = off[s] + ceil_div64(seq_lens[b], block_size[h]);
        }
    return off[Bt * Hkv];
}

/* ---- O1: block centroid = mean of the block's keys (binary32, tokens in order) ------ */
void orc_centroids(int dtype, int Bt, int Hkv, int d, int P, int64_t s_page, int64_t s_head, int64_t s_tok,
                   const uint16_t *k_cache, const int32_t *page_table, int pt_stride, const int32_t *seq_lens,
                   const int32_t *block_size, const int64_t *off, float *cent /* [total][d] */) {
    paged_t kc = {k_cache, page_table, pt_stride, P, s_page, s_head, s_tok};
#pragma omp parallel for schedule(dynamic, 1)
    for (int s = 0; s < Bt * Hkv; ++s) {
        int b = s / Hkv, h = s % Hkv;
        int64_t L = seq_lens[b], B = block_size[h];
        int64_t N = off[s + 1] - off[s];
        for (int64_t j = 0; j < N; ++j) {
            int64_t t0 = j * B;
            int64_t n = (L - t0 < B) ? (L - t0) : B; /* the last block may be partial */
            float *c = cent + (off[s] + j) * d;
            for (int ch = 0; ch < d; ++ch) c[ch] = 0.0f;
            for (int64_t t = t0; t < t0 + n; ++t) {
                const uint16_t *row = row_of(&kc, b, h, t);
                for (int ch = 0; ch < d; ++ch) c[ch] = c[ch] + widen(row[ch], dtype);
            }
            float fn = (float)n;
            for (int ch = 0; ch < d; ++ch) c[ch] = c[ch] / fn;
        }
    }
}

/* ---- O2: per-(segment, channel) range: scale = (max-min)/15, zero-point offset = min */
void orc_quant_params(int nseg, int d, const int64_t *off, const float *cent, float *qscale, float *qmin,
                      float *qinv /* [nseg][d] each */) {
#pragma omp parallel for schedule(dynamic, 1)
    for (int s = 0; s < nseg; ++s) {
        for (int ch = 0; ch < d; ++ch) {
            float mn = INFINITY, mx = -INFINITY;
            for (int64_t j = off[s]; j < off[s + 1]; ++j) {
                float v = cent[j * d + ch];
                if (v < mn) mn = v;
                if (v > mx) mx = v;
            }
            float rng = mx - mn;
            float sc = 0.0f, inv = 0.0f;
            if (rng > 0.0f) {
                sc = rng / 15.0f;
                inv = 15.0f / rng;
            }
            if (off[s + 1] == off[s]) mn = 0.0f;
            qscale[(int64_t)s * d + ch] = sc;
            qinv[(int64_t)s * d + ch] = inv;
            qmin[(int64_t)s * d + ch] = mn;
        }
    }
}

/* ---- O3: 4-bit codes, round-half-to-even, two channels per byte (even = low nibble) - */
void orc_quantize(int nseg, int d, const int64_t *off, const float *cent, const float *qmin, const float *qinv,
                  uint8_t *codes /* [total][d/2] */) {
#pragma omp parallel for schedule(dynamic, 1)
    for (int s = 0; s < nseg; ++s) {
        const float *mn = qmin + (int64_t)s * d, *inv = qinv + (int64_t)s * d;
        for (int64_t j = off[s]; j < off[s + 1]; ++j) {
            for (int ch = 0; ch < d; ++ch) {
                float x = cent[j * d + ch] - mn[ch];
                float y = x * inv[ch];
                float r = rintf(y); /* default rounding mode: to nearest, ties to even */
                if (r < 0.0f) r = 0.0f;
                if (r > 15.0f) r = 15.0f;
                uint8_t code = (uint8_t)r;
                uint8_t *byte = codes + j * (d / 2) + ch / 2;
                if (ch % 2 == 0)
                    *byte = code;
                else
                    *byte = (uint8_t)(*byte | (code << 4));
            }
        }
    }
}

/* dequantized centroid (diagnostics): c^ = code * scale + min */
void orc_dequantize(int nseg, int d, const int64_t *off, const uint8_t *codes, const float *qscale,
                    const float *qmin, float *out /* [total][d] */) {
    for (int s = 0; s < nseg; ++s)
        for (int64_t j = off[s]; j < off[s + 1]; ++j)
            for (int ch = 0; ch < d; ++ch) {
                uint8_t byte = codes[j * (d / 2) + ch / 2];
                int code = (ch % 2 == 0) ? (byte & 15) : (byte >> 4);
                out[j * d + ch] = fmaf((float)code, qscale[(int64_t)s * d + ch], qmin[(int64_t)s * d + ch]);
            }
}

/* ---- O4: fixed-point importance score --------------------------------------------
 * r_j = sum_g q_g . c^_j (Sec. 2.2) = sum_c u_c * (code_jc * scale_c + min_c), u = sum_g q_g.
 * The min term is the same for every block of the segment, so the ranking is that of
 * sum_c (u_c * scale_c) * code_jc.  w_c = u_c*scale_c is imaged on integers wq_c with the
 * largest |w_c| placed in [2^14, 2^15]; S_j = sum_c wq_c * code_jc is exact in int32. */
/* Fixed-point image of one weight on the scale 2^ex: rint(w * 2^-ex) as an integer.  Inputs are
 * finite by contract; a NaN weight next to finite ones (its magnitude never enters the maximum the
 * scale comes from) images to 0 instead of reaching a float-to-integer conversion. */
static int32_t fixed_image(float w, int ex) {
    if (w != w) return 0;
    return (int32_t)rintf(ldexpf(w, -ex));
}

void orc_score(int dtype, int Bt, int Hq, int Hkv, int d, const uint16_t *q /* [Bt][Hq][d] */,
               const uint8_t *codes, const float *qscale, const int64_t *off, int32_t *scores /* [total] */,
               int32_t *score_exp /* [Bt*Hkv] */, int32_t *wq_out /* [Bt*Hkv][d] or NULL */) {
    int G = Hq / Hkv;
#pragma omp parallel for schedule(dynamic, 1)
    for (int s = 0; s < Bt * Hkv; ++s) {
        int b = s / Hkv, h = s % Hkv;
        float w[1024];
        int32_t wq[1024];
        float A = 0.0f;
        for (int ch = 0; ch < d; ++ch) {
            float u = widen(q[((int64_t)b * Hq + h * G) * d + ch], dtype);
            for (int g = 1; g < G; ++g) u = u + widen(q[((int64_t)b * Hq + h * G + g) * d + ch], dtype);
            w[ch] = u * qscale[(int64_t)s * d + ch];
            float a = fabsf(w[ch]);
            if (a > A) A = a;
        }
        int ex = 0;
        if (!(A >= 0x1p-100f) || isinf(A)) {
            for (int ch = 0; ch < d; ++ch) wq[ch] = 0;
        } else {
            ex = ilogbf(A) - 14;
            for (int ch = 0; ch < d; ++ch) wq[ch] = fixed_image(w[ch], ex);
        }
        score_exp[s] = ex;
        if (wq_out)
            for (int ch = 0; ch < d; ++ch) wq_out[(int64_t)s * d + ch] = wq[ch];
        for (int64_t j = off[s]; j < off[s + 1]; ++j) {
            int32_t acc = 0;
            for (int ch = 0; ch < d; ++ch) {
                uint8_t byte = codes[j * (d / 2) + ch / 2];
                int32_t code = (ch % 2 == 0) ? (byte & 15) : (byte >> 4);
                acc += wq[ch] * code;
            }
            scores[j] = acc;
        }
    }
}

/* ---- block representation by channel-wise extrema (max-min pooling, the other pooling the
 * footnote of Sec. 2.2 names; the baseline of Sec. 4.1 scores blocks with it).
 * rep[j] = (max_t k_t[0..d-1], min_t k_t[0..d-1]) over the block's valid tokens: 2d values,
 * maxima first.  Exact (comparisons only). */
void orc_minmax_pool(int dtype, int Bt, int Hkv, int d, int P, int64_t s_page, int64_t s_head, int64_t s_tok,
                     const uint16_t *k_cache, const int32_t *page_table, int pt_stride, const int32_t *seq_lens,
                     const int32_t *block_size, const int64_t *off, float *rep /* [total][2d] */) {
    paged_t kc = {k_cache, page_table, pt_stride, P, s_page, s_head, s_tok};
#pragma omp parallel for schedule(dynamic, 1)
    for (int s = 0; s < Bt * Hkv; ++s) {
        int b = s / Hkv, h = s % Hkv;
        int64_t L = seq_lens[b], B = block_size[h];
        int64_t N = off[s + 1] - off[s];
        for (int64_t j = 0; j < N; ++j) {
            int64_t t0 = j * B;
            int64_t n = (L - t0 < B) ? (L - t0) : B;
            float *mx = rep + (off[s] + j) * 2 * d, *mn = mx + d;
            for (int ch = 0; ch < d; ++ch) {
                mx[ch] = -INFINITY;
                mn[ch] = INFINITY;
            }
            for (int64_t t = t0; t < t0 + n; ++t) {
                const uint16_t *row = row_of(&kc, b, h, t);
                for (int ch = 0; ch < d; ++ch) {
                    float v = widen(row[ch], dtype);
                    if (v > mx[ch]) mx[ch] = v;
                    if (v < mn[ch]) mn[ch] = v;
                }
            }
        }
    }
}

/* ---- importance score for the max-min representation ------------------------------
 * Per query head the block's score is the channel-wise upper bound of q . k over the block,
 *   sum_c max(q_c * M^_jc, q_c * m^_jc),
 * M^, m^ the dequantized maxima and minima; the group's score is the sum over its heads.
 * For M^ >= m^ the larger product is the one whose bound matches the sign of q_c; that
 * sign-matched product is what is taken here also where quantization makes M^ and m^ cross
 * (by less than a quantization step), so that the group score stays linear in the codes:
 *   sum_c [ P_c * (codeM_jc * scaleM_c + minM_c) + Q_c * (codem_jc * scalem_c + minm_c) ],
 * P_c = sum of the group's positive q_gc, Q_c = sum of its negative q_gc.  The offset terms
 * are constant within a segment.  What remains is the fixed-point dot of O4 over 2d weights
 * w = (P * scaleM, Q * scalem) and 2d codes (maxima first). */
void orc_score_minmax(int dtype, int Bt, int Hq, int Hkv, int d, const uint16_t *q /* [Bt][Hq][d] */,
                      const uint8_t *codes /* [total][d] bytes: d/2 of maxima, d/2 of minima */,
                      const float *qscale /* [Bt*Hkv][2d] */, const int64_t *off, int32_t *scores,
                      int32_t *score_exp, int32_t *wq_out /* [Bt*Hkv][2d] or NULL */) {
    int G = Hq / Hkv, d2 = 2 * d;
#pragma omp parallel for schedule(dynamic, 1)
    for (int s = 0; s < Bt * Hkv; ++s) {
        int b = s / Hkv, h = s % Hkv;
        float w[2048];
        int32_t wq[2048];
        float A = 0.0f;
        for (int ch = 0; ch < d; ++ch) {
            float pos = 0.0f, neg = 0.0f;
            for (int g = 0; g < G; ++g) {
                float v = widen(q[((int64_t)b * Hq + h * G + g) * d + ch], dtype);
                if (v > 0.0f) pos = pos + v;
                if (v < 0.0f) neg = neg + v;
            }
            w[ch] = pos * qscale[(int64_t)s * d2 + ch];
            w[d + ch] = neg * qscale[(int64_t)s * d2 + d + ch];
        }
        for (int c = 0; c < d2; ++c) {
            float a = fabsf(w[c]);
            if (a > A) A = a;
        }
        int ex = 0;
        if (!(A >= 0x1p-100f) || isinf(A)) {
            for (int c = 0; c < d2; ++c) wq[c] = 0;
        } else {
            ex = ilogbf(A) - 14;
            for (int c = 0; c < d2; ++c) wq[c] = fixed_image(w[c], ex);
        }
        score_exp[s] = ex;
        if (wq_out)
            for (int c = 0; c < d2; ++c) wq_out[(int64_t)s * d2 + c] = wq[c];
        for (int64_t j = off[s]; j < off[s + 1]; ++j) {
            int32_t acc = 0;
            for (int c = 0; c < d2; ++c) {
                uint8_t byte = codes[j * d + c / 2];
                int32_t code = (c % 2 == 0) ? (byte & 15) : (byte >> 4);
                acc += wq[c] * code;
            }
            scores[j] = acc;
        }
    }
}

/* ---- group score = the MAXIMUM over the group's query heads of r_j = q_g . c^_j (Sec. 2.2), a
 * second way of sharing one selection among the G query heads of a KV head (the paper selects per
 * head and leaves grouped-query models open).  Unlike the sum, the maximum compares heads, so the
 * zero-point term of each head matters:
 *   q_g . c^_j = sum_c (q_gc * scale_c) * code_jc + z_g,   z_g = sum_c q_gc * min_c.
 * Fixed point, one exponent for the whole group so that heads are comparable:
 *   w_gc = q_gc * scale_c (one binary32 multiply);  A = max_{g,c} |w_gc|;  e = ilogb(A) - 14;
 *   wq_gc = rint(w_gc * 2^-e);
 *   z_g in binary32: products q_gc * min_c (one multiply each) summed pairwise within each run of 16
 *   consecutive channels ((p0+p1)+(p2+p3))+... , the 8 run sums then added in increasing order;
 *   zq_g = rint(z_g * 2^-e) clamped to [-2^30, 2^30] (0 for a NaN);
 *   S_j = max_g ( sum_c wq_gc * code_jc + zq_g )   (int32; |sum| <= 128*15*2^15 < 2^26).
 * A < 2^-100, Inf or NaN: every weight and offset is 0, e = 0.  Mean pooling only. */
static float sum16_pairwise(const float *p) {
    float a[16];
    for (int i = 0; i < 16; ++i) a[i] = p[i];
    for (int n = 16; n > 1; n /= 2)
        for (int i = 0; i < n / 2; ++i) a[i] = a[2 * i] + a[2 * i + 1];
    return a[0];
}

void orc_score_groupmax(int dtype, int Bt, int Hq, int Hkv, int d, const uint16_t *q /* [Bt][Hq][d] */,
                        const uint8_t *codes, const float *qscale, const float *qmin, const int64_t *off,
                        int32_t *scores /* [total] */, int32_t *score_exp /* [Bt*Hkv] */,
                        int32_t *wq_out /* [Bt*Hkv][G][d] or NULL */, int32_t *zq_out /* [Bt*Hkv][G] or NULL */) {
    int G = Hq / Hkv;
#pragma omp parallel for schedule(dynamic, 1)
    for (int s = 0; s < Bt * Hkv; ++s) {
        int b = s / Hkv, h = s % Hkv;
        float w[8][256], prod[256];
        int32_t wq[8][256], zq[8];
        float z[8];
        float A = 0.0f;
        for (int g = 0; g < G; ++g) {
            const uint16_t *qrow = q + ((int64_t)b * Hq + h * G + g) * d;
            for (int ch = 0; ch < d; ++ch) {
                float qv = widen(qrow[ch], dtype);
                w[g][ch] = qv * qscale[(int64_t)s * d + ch];
                prod[ch] = qv * qmin[(int64_t)s * d + ch];
                float a = fabsf(w[g][ch]);
                if (a > A) A = a;
            }
            float acc = sum16_pairwise(prod);
            for (int k = 1; k < d / 16; ++k) acc = acc + sum16_pairwise(prod + 16 * k);
            z[g] = acc;
        }
        int ex = 0;
        int live = (A >= 0x1p-100f) && !isinf(A);
        if (live) ex = ilogbf(A) - 14;
        for (int g = 0; g < G; ++g) {
            for (int ch = 0; ch < d; ++ch) wq[g][ch] = live ? fixed_image(w[g][ch], ex) : 0;
            float zs = live ? rintf(ldexpf(z[g], -ex)) : 0.0f;
            if (!(zs == zs)) zs = 0.0f;
            if (zs > 0x1p30f) zs = 0x1p30f;
            if (zs < -0x1p30f) zs = -0x1p30f;
            zq[g] = (int32_t)zs;
        }
        score_exp[s] = ex;
        if (wq_out)
            for (int g = 0; g < G; ++g)
                for (int ch = 0; ch < d; ++ch) wq_out[((int64_t)s * G + g) * d + ch] = wq[g][ch];
        if (zq_out)
            for (int g = 0; g < G; ++g) zq_out[(int64_t)s * G + g] = zq[g];
        for (int64_t j = off[s]; j < off[s + 1]; ++j) {
            int32_t best = 0;
            for (int g = 0; g < G; ++g) {
                int32_t acc = 0;
                for (int ch = 0; ch < d; ++ch) {
                    uint8_t byte = codes[j * (d / 2) + ch / 2];
                    int32_t code = (ch % 2 == 0) ? (byte & 15) : (byte >> 4);
                    acc += wq[g][ch] * code;
                }
                acc += zq[g];
                if (g == 0 || acc > best) best = acc;
            }
            scores[j] = best;
        }
    }
}

/* ---- O5: Top-K_s per segment, K_s = min(N_s, ceil(T_b / B_h)) ----------------------- */
typedef struct {
    int32_t score;
    int32_t idx;
    int32_t forced;
} pair_t;

static int by_score_desc_then_index(const void *a, const void *b) {
    const pair_t *x = (const pair_t *)a, *y = (const pair_t *)b;
    if (x->forced != y->forced) return x->forced > y->forced ? -1 : 1; /* forced blocks ahead of every score */
    if (x->forced) return x->idx < y->idx ? -1 : (x->idx > y->idx ? 1 : 0);
    if (x->score != y->score) return x->score > y->score ? -1 : 1;
    if (x->idx != y->idx) return x->idx < y->idx ? -1 : 1;
    return 0;
}

static int by_index(const void *a, const void *b) {
    int32_t x = *(const int32_t *)a, y = *(const int32_t *)b;
    return (x > y) - (x < y);
}

/* Forced blocks (a selection policy on top of the paper's pure Top-K, off by default): the
 * blocks that hold any of the first `sink_tokens` or of the last `recent_tokens` tokens of the
 * context rank ahead of every score, lowest index first among themselves; they still count
 * towards K_s.  seq_lens may be NULL when recent_tokens is 0. */
void orc_topk(int Bt, int Hkv, const int64_t *off, const int32_t *block_size, const int32_t *budget,
              const int32_t *scores, int32_t *sel_idx /* [Bt*Hkv][sel_stride] */, int32_t *sel_cnt,
              int sel_stride, const int32_t *seq_lens, int sink_tokens, int recent_tokens) {
#pragma omp parallel for schedule(dynamic, 1)
    for (int s = 0; s < Bt * Hkv; ++s) {
        int b = s / Hkv, h = s % Hkv;
        int64_t N = off[s + 1] - off[s];
        int64_t B = block_size[h];
        int64_t K = ceil_div64(budget[b], B);
        if (K > N) K = N;
        if (K > sel_stride) K = sel_stride;
        pair_t *p = (pair_t *)malloc(sizeof(pair_t) * (size_t)(N > 0 ? N : 1));
        for (int64_t j = 0; j < N; ++j) {
            int forced = j * B < sink_tokens; /* the block's first token is among the first sink_tokens */
            if (recent_tokens > 0) {
                int64_t L = seq_lens[b];
                int64_t last = (j + 1) * B < L ? (j + 1) * B : L; /* one past the block's last token */
                if (last > L - recent_tokens) forced = 1;        /* it holds one of the last recent_tokens */
            }
            p[j].score = scores[off[s] + j];
            p[j].forced = forced;
            p[j].idx = (int32_t)j;
        }
        qsort(p, (size_t)N, sizeof(pair_t), by_score_desc_then_index);
        int32_t *out = sel_idx + (int64_t)s * sel_stride;
        for (int64_t i = 0; i < K; ++i) out[i] = p[i].idx;
        qsort(out, (size_t)K, sizeof(int32_t), by_index);
        for (int64_t i = K; i < sel_stride; ++i) out[i] = -1;
        sel_cnt[s] = (int32_t)K;
        free(p);
    }
}

/* ---- O6: attention over the selected tokens, Eq. (1) restricted to the selection ----
 * For query head hq of KV head h: z_t = sm_scale * q . k_t, a = softmax(z), o = sum a_t v_t,
 * all in binary64; lse = max z + ln sum exp(z - max z).  A selected last block contributes
 * only its valid tokens.  An empty selection gives o = 0, lse = -inf. */
static void attend_tokens(int dtype, int d, const paged_t *kc, const paged_t *vc, int b, int h,
                          const uint16_t *qrow, const int64_t *tok, int64_t ntok, double sm_scale,
                          double *z /* scratch [ntok] */, double *o /* [d] */, double *lse) {
    double m = -INFINITY;
    for (int64_t i = 0; i < ntok; ++i) {
        const uint16_t *kr = row_of(kc, b, h, tok[i]);
        double dot = 0.0;
        for (int ch = 0; ch < d; ++ch) dot += (double)widen(qrow[ch], dtype) * (double)widen(kr[ch], dtype);
        z[i] = sm_scale * dot;
        if (z[i] > m) m = z[i];
    }
    for (int ch = 0; ch < d; ++ch) o[ch] = 0.0;
    if (ntok == 0) {
        *lse = -INFINITY;
        return;
    }
    double l = 0.0;
    for (int64_t i = 0; i < ntok; ++i) {
        double p = exp(z[i] - m);
        const uint16_t *vr = row_of(vc, b, h, tok[i]);
        l += p;
        for (int ch = 0; ch < d; ++ch) o[ch] += p * (double)widen(vr[ch], dtype);
    }
    for (int ch = 0; ch < d; ++ch) o[ch] /= l;
    *lse = m + log(l);
}

void orc_sparse_attention(int dtype, int Bt, int Hq, int Hkv, int d, int P, int64_t s_page, int64_t s_head,
                          int64_t s_tok, const uint16_t *q, const uint16_t *k_cache, const uint16_t *v_cache,
                          const int32_t *page_table, int pt_stride, const int32_t *seq_lens,
                          const int32_t *block_size, const int32_t *sel_idx, const int32_t *sel_cnt,
                          int sel_stride, double sm_scale, double *out /* [Bt][Hq][d] */,
                          double *lse /* [Bt][Hq] */) {
    paged_t kc = {k_cache, page_table, pt_stride, P, s_page, s_head, s_tok};
    paged_t vc = {v_cache, page_table, pt_stride, P, s_page, s_head, s_tok};
    int G = Hq / Hkv;
#pragma omp parallel for schedule(dynamic, 1)
    for (int s = 0; s < Bt * Hkv; ++s) {
        int b = s / Hkv, h = s % Hkv;
        int64_t L = seq_lens[b], B = block_size[h];
        int64_t cnt = sel_cnt[s];
        int64_t *tok = (int64_t *)malloc(sizeof(int64_t) * (size_t)(cnt * B + 1));
        int64_t ntok = 0;
        for (int64_t i = 0; i < cnt; ++i) {
            int64_t j = sel_idx[(int64_t)s * sel_stride + i];
            if (j < 0) continue;
            for (int64_t t = j * B; t < (j + 1) * B && t < L; ++t) tok[ntok++] = t;
        }
        double *z = (double *)malloc(sizeof(double) * (size_t)(ntok + 1));
        for (int g = 0; g < G; ++g) {
            int hq = h * G + g;
            attend_tokens(dtype, d, &kc, &vc, b, h, q + ((int64_t)b * Hq + hq) * d, tok, ntok, sm_scale, z,
                          out + ((int64_t)b * Hq + hq) * d, lse + (int64_t)b * Hq + hq);
        }
        free(z);
        free(tok);
    }
}

/* ---- dense reference: Eq. (1) over every token of the context ---------------------- */
void orc_dense_attention(int dtype, int Bt, int Hq, int Hkv, int d, int P, int64_t s_page, int64_t s_head,
                         int64_t s_tok, const uint16_t *q, const uint16_t *k_cache, const uint16_t *v_cache,
                         const int32_t *page_table, int pt_stride, const int32_t *seq_lens, double sm_scale,
                         double *out, double *lse) {
    paged_t kc = {k_cache, page_table, pt_stride, P, s_page, s_head, s_tok};
    paged_t vc = {v_cache, page_table, pt_stride, P, s_page, s_head, s_tok};
    int G = Hq / Hkv;
#pragma omp parallel for schedule(dynamic, 1)
    for (int s = 0; s < Bt * Hkv; ++s) {
        int b = s / Hkv, h = s % Hkv;
        int64_t L = seq_lens[b];
        int64_t *tok = (int64_t *)malloc(sizeof(int64_t) * (size_t)(L + 1));
        for (int64_t t = 0; t < L; ++t) tok[t] = t;
        double *z = (double *)malloc(sizeof(double) * (size_t)(L + 1));
        for (int g = 0; g < G; ++g) {
            int hq = h * G + g;
            attend_tokens(dtype, d, &kc, &vc, b, h, q + ((int64_t)b * Hq + hq) * d, tok, L, sm_scale, z,
                          out + ((int64_t)b * Hq + hq) * d, lse + (int64_t)b * Hq + hq);
        }
        free(z);
        free(tok);
    }
}

/* ---- attention recall (Sec. 2.3): share of the dense softmax mass that falls on the
 * selected tokens, per query head.  Diagnostic only. */
void orc_attention_recall(int dtype, int Bt, int Hq, int Hkv, int d, int P, int64_t s_page, int64_t s_head,
                          int64_t s_tok, const uint16_t *q, const uint16_t *k_cache, const int32_t *page_table,
                          int pt_stride, const int32_t *seq_lens, const int32_t *block_size,
                          const int32_t *sel_idx, const int32_t *sel_cnt, int sel_stride, double sm_scale,
                          double *recall /* [Bt][Hq] */) {
    paged_t kc = {k_cache, page_table, pt_stride, P, s_page, s_head, s_tok};
    int G = Hq / Hkv;
#pragma omp parallel for schedule(dynamic, 1)
    for (int s = 0; s < Bt * Hkv; ++s) {
        int b = s / Hkv, h = s % Hkv;
        int64_t L = seq_lens[b], B = block_size[h];
        int64_t N = ceil_div64(L, B);
        uint8_t *picked = (uint8_t *)calloc((size_t)(N + 1), 1);
        for (int64_t i = 0; i < sel_cnt[s]; ++i) {
            int64_t j = sel_idx[(int64_t)s * sel_stride + i];
            if (j >= 0 && j < N) picked[j] = 1;
        }
        double *z = (double *)malloc(sizeof(double) * (size_t)(L + 1));
        for (int g = 0; g < G; ++g) {
            const uint16_t *qrow = q + ((int64_t)b * Hq + h * G + g) * d;
            double m = -INFINITY;
            for (int64_t t = 0; t < L; ++t) {
                const uint16_t *kr = row_of(&kc, b, h, t);
                double dot = 0.0;
                for (int ch = 0; ch < d; ++ch) dot += (double)widen(qrow[ch], dtype) * (double)widen(kr[ch], dtype);
                z[t] = sm_scale * dot;
                if (z[t] > m) m = z[t];
            }
            double all = 0.0, in = 0.0;
            for (int64_t t = 0; t < L; ++t) {
                double p = exp(z[t] - m);
                all += p;
                if (picked[t / B]) in += p;
            }
            recall[(int64_t)b * Hq + h * G + g] = in / all;
        }
        free(z);
        free(picked);
    }
}

/* ---- offline calibration (Sec. 3.2, Eq. (2)): per head the largest candidate block size whose
 * recall keeps at least the share tau of the recall at the smallest candidate,
 *   B*_h = max { B : Recall(h, B) >= tau * Recall(h, B_min) }.
 * recall[i][h][k] is the attention recall of head h on calibration sample i with candidate k
 * (candidates ascending, cand[0] = B_min); Recall(h, B) is its mean over the samples, taken in
 * binary64 in sample order.  The set is read literally: a larger candidate that passes wins even
 * if a smaller one in between fails.  mean_out [nh][nB] (may be NULL) receives the means. */
void orc_assign_block_sizes(int n_samples, int nh, int nB, const double *recall, const int32_t *cand, double tau,
                            int32_t *block_size /* [nh] */, double *mean_out) {
    for (int h = 0; h < nh; ++h) {
        double base = 0.0;
        int best = 0;
        for (int k = 0; k < nB; ++k) {
            double acc = 0.0;
            for (int i = 0; i < n_samples; ++i) acc += recall[((int64_t)i * nh + h) * nB + k];
            double mean = acc / (double)n_samples;
            if (mean_out) mean_out[(int64_t)h * nB + k] = mean;
            if (k == 0) base = mean;
            if (mean >= tau * base) best = k;
        }
        block_size[h] = cand[best];
    }
}

/* ---- keeping the store current while decoding (upstream of the per-step path; the paper only
 * notes that recomputing every centroid is too expensive, Sec. 1 and Sec. 3.2, and leaves the
 * mechanism open).  Reading taken: the pooled state of each segment's LAST block is kept in
 * binary32 (running sum in token order for mean pooling; running maxima then minima for max-min
 * pooling); a new token is folded into it with the same single operations a rebuild would use,
 * so the block's value is bit-identical to a rebuild's; its 4-bit row is re-emitted under the
 * FROZEN per-channel (scale, min) of the store with clamping to [0, 15]:
 *   code = clamp(rint((value - min) * (1 / scale))), 0 where scale == 0.
 * Rows of closed blocks never change.  The ranges are only refreshed by a rebuild.
 *
 * orc_tail_state: state [nseg][R*d] of the last block of every segment at the given lengths. */
void orc_tail_state(int dtype, int repr, int Bt, int Hkv, int d, int P, int64_t s_page, int64_t s_head,
                    int64_t s_tok, const uint16_t *k_cache, const int32_t *page_table, int pt_stride,
                    const int32_t *seq_lens, const int32_t *block_size, float *tail) {
    paged_t kc = {k_cache, page_table, pt_stride, P, s_page, s_head, s_tok};
    int W = d * (repr + 1);
    for (int s = 0; s < Bt * Hkv; ++s) {
        int b = s / Hkv, h = s % Hkv;
        int64_t L = seq_lens[b], B = block_size[h];
        int64_t t0 = ((L - 1) / B) * B;
        float *st = tail + (int64_t)s * W;
        for (int64_t t = t0; t < L; ++t) {
            const uint16_t *row = row_of(&kc, b, h, t);
            for (int ch = 0; ch < d; ++ch) {
                float v = widen(row[ch], dtype);
                if (repr == 0) {
                    st[ch] = (t == t0) ? v : st[ch] + v;
                } else {
                    st[ch] = (t == t0 || v > st[ch]) ? v : st[ch];
                    st[d + ch] = (t == t0 || v < st[d + ch]) ? v : st[d + ch];
                }
            }
        }
    }
}

/* orc_append_token: the token at position L_b - 1 (lengths already include it) joins the store.
 * tail: in/out state as above.  row_out [nseg][R*d/2]: the re-emitted 4-bit row of the block that
 * holds the token; value_out [nseg][R*d] (may be NULL): that block's pooled value (mean, or
 * maxima and minima).  clamped [nseg] (may be NULL): when the token completes its block (the row is
 * final from then on), the number of the row's values that the frozen range does not hold is ADDED:
 * values whose unclamped code rint((value - min) / scale) falls outside [0, 15], and values that
 * differ from min where the scale is 0. */
void orc_append_token(int dtype, int repr, int Bt, int Hkv, int d, int P, int64_t s_page, int64_t s_head,
                      int64_t s_tok, const uint16_t *k_cache, const int32_t *page_table, int pt_stride,
                      const int32_t *seq_lens, const int32_t *block_size, const float *qscale,
                      const float *qmin, float *tail, uint8_t *row_out, float *value_out, int32_t *clamped) {
    paged_t kc = {k_cache, page_table, pt_stride, P, s_page, s_head, s_tok};
    int W = d * (repr + 1);
    for (int s = 0; s < Bt * Hkv; ++s) {
        int b = s / Hkv, h = s % Hkv;
        int64_t L = seq_lens[b], B = block_size[h];
        int64_t t = L - 1, t0 = (t / B) * B;
        const uint16_t *row = row_of(&kc, b, h, t);
        float *st = tail + (int64_t)s * W;
        float n = (float)(t - t0 + 1);
        uint8_t *codes = row_out + (int64_t)s * (W / 2);
        int outside = 0;
        for (int c = 0; c < W; ++c) {
            int ch = c % d;
            float v = widen(row[ch], dtype);
            if (repr == 0)
                st[c] = (t == t0) ? v : st[c] + v;
            else if (c < d)
                st[c] = (t == t0 || v > st[c]) ? v : st[c];
            else
                st[c] = (t == t0 || v < st[c]) ? v : st[c];
            float value = (repr == 0) ? st[c] / n : st[c];
            if (value_out) value_out[(int64_t)s * W + c] = value;
            float sc = qscale[(int64_t)s * W + c];
            float r = 0.0f;
            if (sc > 0.0f) {
                float inv = 1.0f / sc;
                float x = value - qmin[(int64_t)s * W + c];
                r = rintf(x * inv);
                if (!(r >= 0.0f && r <= 15.0f)) ++outside;
                if (!(r >= 0.0f)) r = 0.0f;
                if (r > 15.0f) r = 15.0f;
            } else if (value != qmin[(int64_t)s * W + c]) {
                ++outside;
            }
            uint8_t code = (uint8_t)r;
            if (c % 2 == 0)
                codes[c / 2] = code;
            else
                codes[c / 2] = (uint8_t)(codes[c / 2] | (code << 4));
        }
        if (clamped && L % B == 0) clamped[s] += outside;
    }
}

/* ---- quantization variants for the design-space study of Sec. 3.3 (bit widths 2 / 4 / 8,
 * symmetric or asymmetric, always one scale per (segment, channel)).  Codes are kept one per
 * byte.  Asymmetric: code in [0, 2^bits - 1], value ~= code * scale + min, scale = (max - min) /
 * (2^bits - 1): with bits = 4 this is O2/O3 above.  Symmetric: zero-centred, code in
 * [-(2^(bits-1) - 1), 2^(bits-1) - 1] stored with that offset added, value ~= signed code * scale,
 * scale = max|x| / (2^(bits-1) - 1), no zero-point.  Same binary32 steps as O2/O3. */
void orc_quantize_variant(int nseg, int d, const int64_t *off, const float *cent, int bits, int symmetric,
                          float *qscale, float *qmin /* [nseg][d]; 0 when symmetric */,
                          uint8_t *codes /* [total][d] */) {
#pragma omp parallel for schedule(dynamic, 1)
    for (int s = 0; s < nseg; ++s) {
        for (int ch = 0; ch < d; ++ch) {
            float mn = INFINITY, mx = -INFINITY;
            for (int64_t j = off[s]; j < off[s + 1]; ++j) {
                float v = cent[j * d + ch];
                if (v < mn) mn = v;
                if (v > mx) mx = v;
            }
            float top, rng, base;
            if (symmetric) {
                top = (float)((1 << (bits - 1)) - 1);
                rng = fabsf(mn) > fabsf(mx) ? fabsf(mn) : fabsf(mx);
                base = 0.0f;
            } else {
                top = (float)((1 << bits) - 1);
                rng = mx - mn;
                base = mn;
            }
            float sc = 0.0f, inv = 0.0f;
            if (off[s + 1] > off[s] && rng > 0.0f) {
                sc = rng / top;
                inv = top / rng;
            }
            if (off[s + 1] == off[s]) base = 0.0f;
            qscale[(int64_t)s * d + ch] = sc;
            qmin[(int64_t)s * d + ch] = base;
            for (int64_t j = off[s]; j < off[s + 1]; ++j) {
                float r = rintf((cent[j * d + ch] - base) * inv);
                float lo = symmetric ? -top : 0.0f;
                if (r < lo) r = lo;
                if (r > top) r = top;
                codes[j * d + ch] = (uint8_t)(int)(symmetric ? r + top : r);
            }
        }
    }
}

/* Fixed-point score (as O4) on one-code-per-byte stores of either kind.  `zero` is the stored
 * code that stands for 0 (2^(bits-1) - 1 for symmetric stores, 0 for asymmetric ones). */
void orc_score_variant(int dtype, int Bt, int Hq, int Hkv, int d, const uint16_t *q, const uint8_t *codes,
                       const float *qscale, int zero, const int64_t *off, int32_t *scores, int32_t *score_exp) {
    int G = Hq / Hkv;
#pragma omp parallel for schedule(dynamic, 1)
    for (int s = 0; s < Bt * Hkv; ++s) {
        int b = s / Hkv, h = s % Hkv;
        float w[1024];
        int32_t wq[1024];
        float A = 0.0f;
        for (int ch = 0; ch < d; ++ch) {
            float u = widen(q[((int64_t)b * Hq + h * G) * d + ch], dtype);
            for (int g = 1; g < G; ++g) u = u + widen(q[((int64_t)b * Hq + h * G + g) * d + ch], dtype);
            w[ch] = u * qscale[(int64_t)s * d + ch];
            float a = fabsf(w[ch]);
            if (a > A) A = a;
        }
        int ex = 0;
        if (!(A >= 0x1p-100f) || isinf(A)) {
            for (int ch = 0; ch < d; ++ch) wq[ch] = 0;
        } else {
            ex = ilogbf(A) - 14;
            for (int ch = 0; ch < d; ++ch) wq[ch] = fixed_image(w[ch], ex);
        }
        score_exp[s] = ex;
        for (int64_t j = off[s]; j < off[s + 1]; ++j) {
            int64_t acc = 0;
            for (int ch = 0; ch < d; ++ch) acc += (int64_t)wq[ch] * ((int)codes[j * d + ch] - zero);
            scores[j] = (int32_t)acc; /* |acc| <= 128 * 2^15 * 255 < 2^31 */
        }
    }
}
