/*
 * CPU oracle for the SwiftPrune per-layer pruning path.
 *
 * TEST INFRASTRUCTURE ONLY: a plain, slow, single-threaded statement of what
 * the method computes, used by the tests, the smoke check and the CPU-baseline
 * leg of the benchmark.  It shares no code with the HIP library and the
 * product path never calls it.
 *
 * Source of every step: "SwiftPrune: Hessian-Free Weight Pruning for Large
 * Language Models" (arXiv 2501.16376) - Sec. 3.1 (contribution score, the
 * state-update table), Algorithm 1, Sec. 3.2 (EWMA), Sec. 3.3 (N:M).
 *
 * Precision: calibration statistics are accumulated in double and rounded to
 * float once; the selection walk is provided in float (the precision the
 * decisions are defined in for parity) and in double (for closed-form pins).
 * Build with:  gcc -O2 -ffp-contract=off -fno-fast-math -shared -fPIC
 *
 * Pins (tests, CPU only): closed forms of the two recurrences, constant/step
 * inputs, a hand-worked row, threshold monotonicity, scale and permutation
 * invariances, reduction of N:M to per-group magnitude top-N under uniform
 * channel energy, per-group exact sort, the rank-one inverse identity behind
 * the score, statistics against a library sum, the binary16 decoder against a
 * library's half type on all 65536 bit patterns.
 * Parity unpinned (the paper gives no value that fixes them): the reading
 * "x_q^2 is summed over all calibration tokens", the N:M ranking key and
 * tie-break, the degenerate-input conventions (S == 0, 1 - x_q^2/S <= 0).
 */
#include <float.h>
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { ORC_F32 = 0, ORC_BF16 = 1, ORC_F16 = 2 };

/* bf16 and IEEE binary16 are both stored in 16 bits. */
static inline int is_16bit(int dt) { return dt != ORC_F32; }

/* bf16 is the upper half of an IEEE binary32. */
static inline float bf16_to_f32(uint16_t b)
{
    uint32_t u = (uint32_t)b << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return f;
}

/* IEEE 754 binary16: 1 sign, 5 exponent (bias 15), 10 fraction bits.  Every
 * binary16 value is exactly representable in binary32. */
static inline float f16_to_f32(uint16_t h)
{
    const uint32_t sign = (uint32_t)(h & 0x8000u) << 16;
    const uint32_t e = (h >> 10) & 0x1fu;
    const uint32_t m = h & 0x3ffu;
    uint32_t u;
    float f;
    if (e == 0) {                       /* zero or subnormal: m * 2^-24 */
        f = (float)m * 0x1p-24f;
        memcpy(&u, &f, sizeof u);
        u |= sign;
    } else if (e == 31) {               /* infinity or NaN */
        u = sign | 0x7f800000u | (m << 13);
    } else {                            /* normal: rebias 15 -> 127 */
        u = sign | ((e + 112u) << 23) | (m << 13);
    }
    memcpy(&f, &u, sizeof f);
    return f;
}

static inline float load_elem(const void *base, int64_t idx, int dt)
{
    if (dt == ORC_BF16)
        return bf16_to_f32(((const uint16_t *)base)[idx]);
    if (dt == ORC_F16)
        return f16_to_f32(((const uint16_t *)base)[idx]);
    return ((const float *)base)[idx];
}

/* ------------------------------------------------------------------ */
/* Step 1: calibration statistics (Algorithm 1, first statement;        */
/* Sec. 3.1 defines S as the sum of the squared activations).           */
/* ------------------------------------------------------------------ */

/*
 * acc[q] += sum over t (ascending) of X[t,q]^2, in double.  X is
 * [tokens, in] row-major with row pitch ldx (elements).  Calling it again with
 * the next chunk of tokens continues the same sum.  With many calibration
 * tokens x_q^2 is read as the q-th diagonal entry of X X^T (the paper's
 * H = 2 X X^T), i.e. the SUM over tokens.
 */
void oracle_stats_accumulate(const void *X, int64_t tokens, int64_t in, int64_t ldx,
                             int dt, double *acc)
{
    for (int64_t t = 0; t < tokens; ++t) {
        for (int64_t q = 0; q < in; ++q) {
            double x = (double)load_elem(X, t * ldx + q, dt);
            acc[q] += x * x;
        }
    }
}

/*
 * The same sums when the producer of X has already added up the squares of its own share of the
 * tokens (Algorithm 1, first statement, with the sum over tokens cut in `parts` pieces):
 * P[p*ld + q] = sum of X[t,q]^2 over the tokens of piece p, stored as float.
 *     acc[q] += (double)P[p][q],  p ascending.
 */
void oracle_stats_accumulate_partials(const float *P, int64_t parts, int64_t in, int64_t ld, double *acc)
{
    for (int64_t p = 0; p < parts; ++p) {
        for (int64_t q = 0; q < in; ++q) {
            acc[q] += (double)P[p * ld + q];
        }
    }
}

/*
 * xsq[q] = (float)acc[q];  S = (float)(sum_q acc[q]) summed in double, q ascending.
 */
void oracle_stats_finalize(const double *acc, int64_t in, float *xsq, float *S)
{
    double s = 0.0;
    for (int64_t q = 0; q < in; ++q) {
        xsq[q] = (float)acc[q];
        s += acc[q];
    }
    *S = (float)s;
}

/*
 * Per-channel factor of the score:  hr[q] = 1/2 / (1 - xsq[q]/S)  (the score
 * equation of Sec. 3.1 with w^2 taken out).  Float version: three roundings
 * (divide, subtract, divide).
 * Conventions where the paper is silent: S == 0 -> hr = 1/2 (score = w^2/2);
 * a denominator that rounds to <= 0 is replaced by FLT_EPSILON.
 */
void oracle_channel_factor_f32(const float *xsq, float S, int64_t in, float *hr)
{
    for (int64_t q = 0; q < in; ++q) {
        if (S == 0.0f) {
            hr[q] = 0.5f;
            continue;
        }
        float rho = xsq[q] / S;
        float den = 1.0f - rho;
        if (!(den > 0.0f))
            den = FLT_EPSILON;
        hr[q] = 0.5f / den;
    }
}

/* Double version, straight from the double accumulators (no float rounding). */
void oracle_channel_factor_f64(const double *acc, int64_t in, double *hr)
{
    double s = 0.0;
    for (int64_t q = 0; q < in; ++q)
        s += acc[q];
    for (int64_t q = 0; q < in; ++q) {
        if (s == 0.0) {
            hr[q] = 0.5;
            continue;
        }
        double den = 1.0 - acc[q] / s;
        if (!(den > 0.0))
            den = DBL_EPSILON;
        hr[q] = 0.5 / den;
    }
}

/* ------------------------------------------------------------------ */
/* Steps 2-4: score, EWMA selection, N:M selection - float and double.  */
/* ------------------------------------------------------------------ */

#define REAL float
#define FN(x) x##_f32
#define FABS fabsf
#include "ewma_body.inc"
#undef REAL
#undef FN
#undef FABS

#define REAL double
#define FN(x) x##_f64
#define FABS fabs
#include "ewma_body.inc"
#undef REAL
#undef FN
#undef FABS

/* Scores of a whole layer, float: scores[r*in + q] = (w*w) * hr[q]. */
void oracle_score_f32(const void *W, int64_t out, int64_t in, int64_t ldw, int dt,
                      const float *hr, float *scores)
{
    for (int64_t r = 0; r < out; ++r)
        score_row_f32(W, dt, r * ldw, in, hr, scores + r * in);
}

void oracle_score_f64(const void *W, int64_t out, int64_t in, int64_t ldw, int dt,
                      const double *hr, double *scores)
{
    for (int64_t r = 0; r < out; ++r)
        score_row_f64(W, dt, r * ldw, in, hr, scores + r * in);
}

/*
 * Algorithm 1 exactly as printed, float: the sum S is part of the per-row
 * state and loses w_i^2 whenever element i is pruned (third row of the
 * state-update table), and the score is evaluated per element with the
 * current S:  L_i = (0.5*w*w) / (1 - xsq[i]/S_r).
 * Used as a cross-check of the fixed-S form above.  n_effective (nullable)
 * receives how many of the subtractions changed the bits of S_r, summed over rows;
 * scores (nullable, [out, in]) the score of every element as it was evaluated,
 * S_rows (nullable, [out]) the value of S_r after the last element of each row.
 */
void oracle_ewma_select_literal_f32(const void *W, int64_t out, int64_t in, int64_t ldw,
                                    int dt, const float *xsq, float S,
                                    float alpha, float beta, float la,
                                    uint32_t *keep_mask, int32_t *row_pruned,
                                    int64_t *n_effective, float *scores, float *S_rows)
{
    const int64_t words = (in + 31) / 32;
    const float A = 1.0f - alpha;
    const float B = 1.0f - beta;
    int64_t eff = 0;
    for (int64_t r = 0; r < out; ++r) {
        float S_r = S;
        float est = 0.0f, dev = 0.0f;
        int32_t cnt = 0;
        for (int64_t w = 0; w < words; ++w) keep_mask[r * words + w] = 0u;
        for (int64_t i = 0; i < in; ++i) {
            float w = load_elem(W, r * ldw + i, dt);
            float w2 = w * w;
            float half_w2 = 0.5f * w2;
            float L;
            if (S_r == 0.0f) {
                L = half_w2;
            } else {
                float rho = xsq[i] / S_r;
                float den = 1.0f - rho;
                if (!(den > 0.0f))
                    den = FLT_EPSILON;
                L = half_w2 / den;
            }
            if (scores) scores[r * in + i] = L;
            if (i == 0)
                est = L;
            float t = la * dev;
            float thr = est - t;
            if (L < thr) {
                float S_new = S_r - w2;
                if (S_new != S_r) ++eff;
                S_r = S_new;
                ++cnt;
            } else {
                keep_mask[r * words + (i >> 5)] |= (uint32_t)1 << (i & 31);
            }
            float a_est = A * est;
            float a_new = alpha * L;
            est = a_est + a_new;
            float diff = est - L;
            float b_dev = B * dev;
            float b_new = beta * fabsf(diff);
            dev = b_dev + b_new;
        }
        if (row_pruned) row_pruned[r] = cnt;
        if (S_rows) S_rows[r] = S_r;
    }
    if (n_effective) *n_effective = eff;
}

/* ------------------------------------------------------------------ */
/* Exact selection by sorting (Sec. 3.1: order a row's scores and drop  */
/* the lowest ones) - the O(n log n) rule the EWMA walk replaces; used  */
/* as a comparator.                                                     */
/* ------------------------------------------------------------------ */

typedef struct {
    float score;
    int64_t index;
} scored_t;

static int scored_cmp(const void *a, const void *b)
{
    const scored_t *x = (const scored_t *)a, *y = (const scored_t *)b;
    if (x->score < y->score) return -1;
    if (x->score > y->score) return 1;
    return (x->index > y->index) - (x->index < y->index); /* equal scores: lower index first */
}

/*
 * Per row r: sort (L, index) ascending and prune the first k_r entries, where
 * k_r = k_per_row[r] if k_per_row != NULL, else k_uniform (clamped to [0, in]).
 * NaN scores are ordered after everything else (never pruned before a number).
 */
void oracle_topk_select_f32(const void *W, int64_t out, int64_t in, int64_t ldw, int dt,
                            const float *hr, const int32_t *k_per_row, int64_t k_uniform,
                            uint32_t *keep_mask)
{
    const int64_t words = (in + 31) / 32;
    float *L = (float *)malloc((size_t)in * sizeof(float));
    scored_t *s = (scored_t *)malloc((size_t)in * sizeof(scored_t));
    for (int64_t r = 0; r < out; ++r) {
        score_row_f32(W, dt, r * ldw, in, hr, L);
        for (int64_t q = 0; q < in; ++q) {
            s[q].score = (L[q] != L[q]) ? INFINITY : L[q];
            s[q].index = (L[q] != L[q]) ? q + in : q;   /* NaN after +inf, in index order */
        }
        qsort(s, (size_t)in, sizeof(scored_t), scored_cmp);
        int64_t k = k_per_row ? (int64_t)k_per_row[r] : k_uniform;
        if (k < 0) k = 0;
        if (k > in) k = in;
        for (int64_t w = 0; w < words; ++w) keep_mask[r * words + w] = 0u;
        for (int64_t j = k; j < in; ++j) {
            int64_t q = s[j].index >= in ? s[j].index - in : s[j].index;
            keep_mask[r * words + (q >> 5)] |= (uint32_t)1 << (q & 31);
        }
    }
    free(L);
    free(s);
}

/* ------------------------------------------------------------------ */
/* Compact storage of an N:M-pruned matrix (Sec. 3.3 motivates N:M by   */
/* hardware formats that store only the kept values plus their          */
/* positions).  Open layout defined here, not a vendor format:          */
/*   values[r, g*N + j]  = j-th kept entry (ascending column) of group g */
/*   meta: the position (0..M-1) of that entry inside its group, as a    */
/*         field of b bits (b = 2 for M = 4, else 4), field number       */
/*         g*N + j of the row, packed little-endian into uint32 words;   */
/*         meta_words = ceil(in/M * N * b / 32) per row.                 */
/* A group with fewer than N kept entries is padded with +0 / position 0.*/
/* ------------------------------------------------------------------ */

static int nm_index_bits(int m_group) { return m_group == 4 ? 2 : 4; }

void oracle_compact_nm(const void *W, int64_t out, int64_t in, int64_t ldw, int dt,
                       const uint32_t *keep_mask, int n_keep, int m_group,
                       void *values, uint32_t *meta)
{
    const int64_t words = (in + 31) / 32;
    const int b = nm_index_bits(m_group);
    const int64_t per_row = in / m_group * n_keep;
    const int64_t meta_words = (per_row * b + 31) / 32;
    for (int64_t r = 0; r < out; ++r) {
        for (int64_t w = 0; w < meta_words; ++w) meta[r * meta_words + w] = 0u;
        for (int64_t g = 0; g < in / m_group; ++g) {
            int j = 0;
            for (int i = 0; i < m_group && j < n_keep; ++i) {
                int64_t q = g * m_group + i;
                if (!((keep_mask[r * words + (q >> 5)] >> (q & 31)) & 1u)) continue;
                int64_t f = g * n_keep + j;
                if (is_16bit(dt))
                    ((uint16_t *)values)[r * per_row + f] = ((const uint16_t *)W)[r * ldw + q];
                else
                    ((uint32_t *)values)[r * per_row + f] = ((const uint32_t *)W)[r * ldw + q];
                meta[r * meta_words + (f * b >> 5)] |= (uint32_t)i << ((f * b) & 31);
                ++j;
            }
            for (; j < n_keep; ++j) {
                int64_t f = g * n_keep + j;
                if (is_16bit(dt)) ((uint16_t *)values)[r * per_row + f] = 0;
                else ((uint32_t *)values)[r * per_row + f] = 0u;
            }
        }
    }
}

/* Inverse: a dense [out, in] matrix (pitch in) with the stored values at their positions, +0 elsewhere. */
void oracle_expand_nm(const void *values, const uint32_t *meta, int64_t out, int64_t in, int dt,
                      int n_keep, int m_group, void *W_out)
{
    const int b = nm_index_bits(m_group);
    const int64_t per_row = in / m_group * n_keep;
    const int64_t meta_words = (per_row * b + 31) / 32;
    for (int64_t r = 0; r < out; ++r) {
        for (int64_t q = 0; q < in; ++q) {
            if (is_16bit(dt)) ((uint16_t *)W_out)[r * in + q] = 0;
            else ((uint32_t *)W_out)[r * in + q] = 0u;
        }
        for (int64_t f = 0; f < per_row; ++f) {
            uint32_t pos = (meta[r * meta_words + (f * b >> 5)] >> ((f * b) & 31)) & ((1u << b) - 1u);
            int64_t q = f / n_keep * m_group + pos;
            /* the output is already +0 everywhere: only non-zero bit patterns are placed, so a
               padding entry (+0 at position 0) can never overwrite a stored value */
            if (is_16bit(dt)) {
                uint16_t v = ((const uint16_t *)values)[r * per_row + f];
                if (v != 0) ((uint16_t *)W_out)[r * in + q] = v;
            } else {
                uint32_t v = ((const uint32_t *)values)[r * per_row + f];
                if (v != 0) ((uint32_t *)W_out)[r * in + q] = v;
            }
        }
    }
}

/* ------------------------------------------------------------------ */
/* Step 5: apply (Algorithm 1: w_i = 0 for pruned entries, c_i = w_i).  */
/* ------------------------------------------------------------------ */

/* W[r,q] <- +0 where the keep bit is 0; kept entries are left bit-for-bit. */
void oracle_apply(void *W, int64_t out, int64_t in, int64_t ldw, int dt,
                  const uint32_t *keep_mask)
{
    const int64_t words = (in + 31) / 32;
    for (int64_t r = 0; r < out; ++r) {
        for (int64_t q = 0; q < in; ++q) {
            int keep = (keep_mask[r * words + (q >> 5)] >> (q & 31)) & 1u;
            if (keep) continue;
            if (is_16bit(dt))
                ((uint16_t *)W)[r * ldw + q] = 0;
            else
                ((float *)W)[r * ldw + q] = 0.0f;
        }
    }
}
