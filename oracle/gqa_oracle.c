/*
 * Reference ("oracle") for grouped-query decode-step attention.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the
 * GPU library is checked against.  It shares no code, header, table or helper
 * with the HIP path and nothing in the product may call it.
 *
 * What it computes (textbook softmax attention of one query token per
 * sequence over that sequence's cached keys/values; the paper fixes only the
 * workload -- a 32B grouped-query reasoning model decoding traces of several
 * thousand tokens, Section 3.3 and Table 3 -- not the operator, whose
 * definition is the standard one):
 *
 *   for every sequence b, query head h, with kv head g = h / (Hq / Hkv) and
 *   L = kv_lens[b]:
 *       s_j  = scale * sum_d Q[b,h,d] * K[b,j,g,d]            j in [0, L)
 *       m    = max_j s_j
 *       Z    = sum_j exp(s_j - m)
 *       p_j  = exp(s_j - m) / Z
 *       O[b,h,d] = sum_j p_j * V[b,j,g,d]
 *       LSE[b,h] = m + ln Z
 *
 * All arithmetic is IEEE double on the bf16 inputs widened exactly.  The two
 * passes over j (scores and maximum first, then the sums) are written out as
 * such: no running maximum, no chunking, no blocking.  L = 0 gives a zero row
 * and LSE = -inf.
 *
 * Addressing.  Contiguous cache (page_size == 0): token j of sequence b, kv
 * head g starts at  base + b*stride_b + g*stride_h + j*stride_t  (strides in
 * elements, the D elements of a row are adjacent).  Paged cache
 * (page_size > 0): token j lives in physical block
 * block_table[b*block_table_stride + j / page_size] at slot j % page_size,
 * i.e. at  base + block*stride_b + g*stride_h + slot*stride_t.
 *
 * Every function here is pinned by tests/test_oracle_pins.py (attention: brute
 * force in fsum arithmetic on tiny inputs, closed forms, invariants, a float64
 * library cross-check; append/rotary: identity at angle zero, quarter turns,
 * norm and relative-position invariants, bf16 rounding against exact cases).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

static double widen_bf16(uint16_t bits)
{
    uint32_t w = (uint32_t)bits << 16;
    float f;
    memcpy(&f, &w, sizeof f);
    return (double)f;
}

typedef struct {
    int32_t batch, num_q_heads, num_kv_heads, head_dim;
    int32_t page_size;            /* 0: contiguous cache */
    int32_t block_table_stride;   /* entries per sequence row (paged only) */
    int64_t q_stride_b, q_stride_h;
    int64_t k_stride_b, k_stride_h, k_stride_t;
    int64_t v_stride_b, v_stride_h, v_stride_t;
    double  scale;
} gqa_oracle_shape;

static const uint16_t *token_row(const uint16_t *base, const gqa_oracle_shape *s,
                                 int64_t sb, int64_t sh, int64_t st,
                                 const int32_t *block_table, int b, int g, int64_t j)
{
    if (s->page_size == 0)
        return base + (int64_t)b * sb + (int64_t)g * sh + j * st;
    int64_t blk = block_table[(int64_t)b * s->block_table_stride + j / s->page_size];
    int64_t slot = j % s->page_size;
    return base + blk * sb + (int64_t)g * sh + slot * st;
}

/*
 * out     [batch, num_q_heads, head_dim] double, contiguous
 * lse     [batch, num_q_heads] double, may be NULL
 * weights optional [batch, num_q_heads, weights_stride] double: p_j for
 *         j < kv_lens[b] (rest untouched); for inspection on tiny cases
 * returns the number of threads that worked, or -1 on a bad argument
 */
int gqa_oracle_decode_attn(const gqa_oracle_shape *s,
                           const uint16_t *q, const uint16_t *k, const uint16_t *v,
                           const int32_t *kv_lens, const int32_t *block_table,
                           double *out, double *lse,
                           double *weights, int64_t weights_stride,
                           int num_threads)
{
    if (!s || !q || !out || !kv_lens) return -1;
    if (s->batch < 0 || s->num_q_heads <= 0 || s->num_kv_heads <= 0 || s->head_dim <= 0) return -1;
    if (s->num_q_heads % s->num_kv_heads != 0) return -1;
    if (s->page_size < 0 || (s->page_size > 0 && !block_table)) return -1;
    const int group = s->num_q_heads / s->num_kv_heads;
    const int D = s->head_dim;
    const int rows = s->batch * s->num_q_heads;
    int used = 1;
    if (num_threads < 1) num_threads = 1;

#ifdef _OPENMP
#pragma omp parallel num_threads(num_threads)
#endif
    {
#ifdef _OPENMP
#pragma omp single
        used = omp_get_num_threads();
#endif
        double *qd = (double *)malloc(sizeof(double) * (size_t)D);
        double *acc = (double *)malloc(sizeof(double) * (size_t)D);
        double *score = NULL;
        int64_t score_cap = 0;
#ifdef _OPENMP
#pragma omp for schedule(dynamic, 1)
#endif
        for (int row = 0; row < rows; ++row) {
            const int b = row / s->num_q_heads;
            const int h = row % s->num_q_heads;
            const int g = h / group;
            const int64_t L = kv_lens[b];
            double *o = out + (int64_t)row * D;
            if (L <= 0) {
                for (int d = 0; d < D; ++d) o[d] = 0.0;
                if (lse) lse[row] = -INFINITY;
                continue;
            }
            if (L > score_cap) {
                free(score);
                score = (double *)malloc(sizeof(double) * (size_t)L);
                score_cap = L;
            }
            const uint16_t *qrow = q + (int64_t)b * s->q_stride_b + (int64_t)h * s->q_stride_h;
            for (int d = 0; d < D; ++d) qd[d] = widen_bf16(qrow[d]);

            /* pass 1: scores and their maximum */
            double m = -INFINITY;
            for (int64_t j = 0; j < L; ++j) {
                const uint16_t *kr = token_row(k, s, s->k_stride_b, s->k_stride_h, s->k_stride_t,
                                               block_table, b, g, j);
                double dot = 0.0;
                for (int d = 0; d < D; ++d) dot += qd[d] * widen_bf16(kr[d]);
                score[j] = s->scale * dot;
                if (score[j] > m) m = score[j];
            }
            /* pass 2: normaliser and weighted sum of value rows */
            double Z = 0.0;
            for (int64_t j = 0; j < L; ++j) {
                score[j] = exp(score[j] - m);
                Z += score[j];
            }
            for (int d = 0; d < D; ++d) acc[d] = 0.0;
            for (int64_t j = 0; j < L; ++j) {
                const uint16_t *vr = token_row(v, s, s->v_stride_b, s->v_stride_h, s->v_stride_t,
                                               block_table, b, g, j);
                const double p = score[j] / Z;
                if (weights) weights[(int64_t)row * weights_stride + j] = p;
                for (int d = 0; d < D; ++d) acc[d] += p * widen_bf16(vr[d]);
            }
            for (int d = 0; d < D; ++d) o[d] = acc[d];
            if (lse) lse[row] = m + log(Z);
        }
        free(qd);
        free(acc);
        free(score);
    }
    return used;
}

/* ------------------------------------------------------------------------
 * Reference for the step that precedes attention in a decode layer: rotate
 * the new token's query and key by its position (optional) and append the
 * new key/value rows to the cache at position kv_lens[b] - 1.
 *
 * Rotary embedding, "rotate-half" pairing of the 32B model family the paper
 * samples from: column d < D/2 is paired with column d + D/2,
 *     x'[d]       = x[d] * cos[pos][d] - x[d + D/2] * sin[pos][d]
 *     x'[d + D/2] = x[d + D/2] * cos[pos][d] + x[d] * sin[pos][d]
 * with pos = kv_lens[b] - 1 and the caller's table cos_sin[pos][0..D/2) = cos,
 * cos_sin[pos][D/2..D) = sin (fp32, widened exactly).  Arithmetic in double,
 * result rounded to bf16 with round-to-nearest-even on the whole bf16 grid
 * (sub-normal spacing 2^-133 below 2^-126, signed zeros, overflow to infinity);
 * a NaN result is stored as the quiet NaN 0x7FC0.  cos_sin == NULL copies
 * q and k unchanged.  V is always copied bit for bit.  For a sequence with
 * kv_lens[b] <= 0 the query is copied unchanged and nothing is written to the
 * cache.  Cache addressing as in the attention oracle.
 * ---------------------------------------------------------------------- */
static uint16_t round_to_bf16(double x)
{
    /* double -> float is exact enough here only if we round once: go through
     * the exact integer representation of the bf16 grid instead. */
    if (isnan(x)) return 0x7FC0;            /* one quiet NaN, whatever the sign and payload */
    if (x == 0.0 || isinf(x)) {
        float f = (float)x;
        uint32_t w;
        memcpy(&w, &f, sizeof w);
        return (uint16_t)(w >> 16);
    }
    int e;
    double m = frexp(fabs(x), &e);          /* |x| = m * 2^e, m in [0.5, 1) */
    if (e < -125) {                         /* bf16 subnormal range: fixed spacing 2^-133 */
        double q = nearbyint(ldexp(fabs(x), 133));
        float f = (float)ldexp(q, -133);
        if (x < 0) f = -f;
        uint32_t w;
        memcpy(&w, &f, sizeof w);
        return (uint16_t)(w >> 16);
    }
    double q = nearbyint(ldexp(m, 8));      /* 8 significant bits, ties to even (default rounding mode) */
    float f = (float)ldexp(q, e - 8);
    if (x < 0) f = -f;
    uint32_t w;
    memcpy(&w, &f, sizeof w);
    return (uint16_t)(w >> 16);
}

int gqa_oracle_kv_append(const gqa_oracle_shape *s,
                         const uint16_t *q_in, uint16_t *q_out,          /* [B, Hq, D] via q strides */
                         const uint16_t *k_new, const uint16_t *v_new,   /* [B, Hkv, D] dense */
                         uint16_t *k_cache, uint16_t *v_cache,
                         const int32_t *kv_lens, const int32_t *block_table,
                         const float *cos_sin)                           /* [positions, D] or NULL */
{
    if (!s || !q_in || !q_out || !k_new || !v_new || !k_cache || !v_cache || !kv_lens) return -1;
    const int D = s->head_dim, half = D / 2;
    if (D % 2 != 0) return -1;
    for (int b = 0; b < s->batch; ++b) {
        const int64_t pos = (int64_t)kv_lens[b] - 1;
        for (int h = 0; h < s->num_q_heads; ++h) {
            const uint16_t *src = q_in + (int64_t)b * s->q_stride_b + (int64_t)h * s->q_stride_h;
            uint16_t *dst = q_out + (int64_t)b * s->q_stride_b + (int64_t)h * s->q_stride_h;
            for (int d = 0; d < half; ++d) {
                if (!cos_sin || pos < 0) { dst[d] = src[d]; dst[d + half] = src[d + half]; continue; }
                const double c = (double)cos_sin[pos * D + d], sn = (double)cos_sin[pos * D + half + d];
                const double x = widen_bf16(src[d]), y = widen_bf16(src[d + half]);
                dst[d] = round_to_bf16(x * c - y * sn);
                dst[d + half] = round_to_bf16(y * c + x * sn);
            }
        }
        if (pos < 0) continue;
        for (int g = 0; g < s->num_kv_heads; ++g) {
            const uint16_t *ks = k_new + ((int64_t)b * s->num_kv_heads + g) * D;
            const uint16_t *vs = v_new + ((int64_t)b * s->num_kv_heads + g) * D;
            uint16_t *kd = (uint16_t *)token_row(k_cache, s, s->k_stride_b, s->k_stride_h, s->k_stride_t,
                                                 block_table, b, g, pos);
            uint16_t *vd = (uint16_t *)token_row(v_cache, s, s->v_stride_b, s->v_stride_h, s->v_stride_t,
                                                 block_table, b, g, pos);
            for (int d = 0; d < half; ++d) {
                if (!cos_sin) { kd[d] = ks[d]; kd[d + half] = ks[d + half]; continue; }
                const double c = (double)cos_sin[pos * D + d], sn = (double)cos_sin[pos * D + half + d];
                const double x = widen_bf16(ks[d]), y = widen_bf16(ks[d + half]);
                kd[d] = round_to_bf16(x * c - y * sn);
                kd[d + half] = round_to_bf16(y * c + x * sn);
            }
            for (int d = 0; d < D; ++d) vd[d] = vs[d];
        }
    }
    return 0;
}
