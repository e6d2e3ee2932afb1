/*
 * Runs the C oracle over a fixed set of cases and prints one line per case with
 * a digest of its outputs.  Built twice by tests/test_sanitizers.py: plainly, and
 * with -fsanitize=address,undefined; the two builds must print the same lines
 * and the sanitized one must report nothing.  Test infrastructure only.
 *
 * -DPLANT_OVERRUN makes the driver itself hand the oracle a cache that is one
 * token row too short, to show that the sanitized build would notice.
 */
#include "../../oracle/gqa_oracle.c"

#include <inttypes.h>
#include <stdio.h>

static uint64_t lcg = 0x9E3779B97F4A7C15ull;
static uint32_t next_u32(void) { lcg = lcg * 6364136223846793005ull + 1442695040888963407ull; return (uint32_t)(lcg >> 32); }
/* bf16 bit pattern of a value in about [-2, 2]: sign, exponent 125..128, random mantissa */
static uint16_t next_bf16(void) { uint32_t r = next_u32(); return (uint16_t)(((r & 1u) << 15) | ((125u + ((r >> 1) & 3u)) << 7) | ((r >> 3) & 0x7Fu)); }

static uint16_t *bf16_array(size_t n) { uint16_t *p = malloc(n * sizeof *p); for (size_t i = 0; i < n; ++i) p[i] = next_bf16(); return p; }

static void digest(const char *name, const double *out, size_t n_out, const double *lse, size_t n_lse, int rc)
{
    double s = 0.0, a = 0.0, l = 0.0;
    for (size_t i = 0; i < n_out; ++i) { s += out[i]; a += fabs(out[i]) * (double)(1 + i % 7); }
    for (size_t i = 0; i < n_lse; ++i) if (!isinf(lse[i])) l += lse[i];
    printf("%s rc=%d sum=%.17g wsum=%.17g lse=%.17g\n", name, rc, s, a, l);
}

static void run_contiguous(const char *name, int token_major, int B, int Hq, int Hkv, int D, int T, const int32_t *lens, int want_w)
{
    gqa_oracle_shape s;
    memset(&s, 0, sizeof s);
    s.batch = B; s.num_q_heads = Hq; s.num_kv_heads = Hkv; s.head_dim = D; s.scale = 0.25;
    s.q_stride_b = (int64_t)Hq * D; s.q_stride_h = D;
    if (token_major) { s.k_stride_b = (int64_t)T * Hkv * D; s.k_stride_t = (int64_t)Hkv * D; s.k_stride_h = D; }
    else             { s.k_stride_b = (int64_t)Hkv * T * D; s.k_stride_h = (int64_t)T * D; s.k_stride_t = D; }
    s.v_stride_b = s.k_stride_b; s.v_stride_h = s.k_stride_h; s.v_stride_t = s.k_stride_t;
    size_t cache = (size_t)B * Hkv * T * D;
#ifdef PLANT_OVERRUN
    cache -= (size_t)D;                       /* the last token row of the last sequence is missing */
#endif
    uint16_t *q = bf16_array((size_t)B * Hq * D), *k = bf16_array(cache), *v = bf16_array(cache);
    double *out = malloc(sizeof(double) * B * Hq * D), *lse = malloc(sizeof(double) * B * Hq);
    int maxlen = 1;
    for (int b = 0; b < B; ++b) if (lens[b] > maxlen) maxlen = lens[b];
    double *w = want_w ? calloc((size_t)B * Hq * maxlen, sizeof(double)) : NULL;
    int rc = gqa_oracle_decode_attn(&s, q, k, v, lens, NULL, out, lse, w, maxlen, 3);
    digest(name, out, (size_t)B * Hq * D, lse, (size_t)B * Hq, rc > 0);
    free(q); free(k); free(v); free(out); free(lse); free(w);
}

static void run_paged(const char *name, int B, int Hq, int Hkv, int D, int page, int table_width, const int32_t *lens)
{
    int blocks = 0;
    for (int b = 0; b < B; ++b) blocks += (lens[b] + page - 1) / page;
    gqa_oracle_shape s;
    memset(&s, 0, sizeof s);
    s.batch = B; s.num_q_heads = Hq; s.num_kv_heads = Hkv; s.head_dim = D; s.scale = -0.125;
    s.page_size = page; s.block_table_stride = table_width;
    s.q_stride_b = (int64_t)Hq * D; s.q_stride_h = D;
    s.k_stride_b = (int64_t)Hkv * page * D; s.k_stride_h = (int64_t)page * D; s.k_stride_t = D;
    s.v_stride_b = s.k_stride_b; s.v_stride_h = s.k_stride_h; s.v_stride_t = s.k_stride_t;
    uint16_t *q = bf16_array((size_t)B * Hq * D);
    uint16_t *k = bf16_array((size_t)blocks * Hkv * page * D), *v = bf16_array((size_t)blocks * Hkv * page * D);
    int32_t *table = malloc(sizeof(int32_t) * B * table_width);
    for (int i = 0; i < B * table_width; ++i) table[i] = -1;
    /* blocks handed out from the top of the pool downwards, interleaved between the sequences */
    int next = blocks - 1;
    for (int i = 0; i < table_width; ++i)
        for (int b = 0; b < B; ++b)
            if (i < (lens[b] + page - 1) / page) table[b * table_width + i] = next--;
    double *out = malloc(sizeof(double) * B * Hq * D), *lse = malloc(sizeof(double) * B * Hq);
    int rc = gqa_oracle_decode_attn(&s, q, k, v, lens, table, out, lse, NULL, 0, 2);
    digest(name, out, (size_t)B * Hq * D, lse, (size_t)B * Hq, rc > 0);

    /* the append step on the same paged cache, with a rotation table */
    int maxlen = 1;
    for (int b = 0; b < B; ++b) if (lens[b] > maxlen) maxlen = lens[b];
    float *cs = malloc(sizeof(float) * maxlen * D);
    for (int i = 0; i < maxlen * D; ++i) cs[i] = (float)((int)(next_u32() % 2001) - 1000) / 1000.0f;
    uint16_t *kn = bf16_array((size_t)B * Hkv * D), *vn = bf16_array((size_t)B * Hkv * D);
    uint16_t *qo = malloc(sizeof(uint16_t) * B * Hq * D);
    rc = gqa_oracle_kv_append(&s, q, qo, kn, vn, k, v, lens, table, cs);
    uint64_t h = 1469598103934665603ull;
    for (size_t i = 0; i < (size_t)B * Hq * D; ++i) h = (h ^ qo[i]) * 1099511628211ull;
    for (size_t i = 0; i < (size_t)blocks * Hkv * page * D; ++i) h = (h ^ k[i] ^ ((uint64_t)v[i] << 16)) * 1099511628211ull;
    printf("%s_append rc=%d hash=%016" PRIx64 "\n", name, rc, h);
    free(q); free(k); free(v); free(table); free(out); free(lse); free(cs); free(kn); free(vn); free(qo);
}

int main(void)
{
    const int32_t a[] = {5, 0, 1, 33, 64};
    run_contiguous("head_major", 0, 5, 6, 2, 16, 64, a, 1);
    run_contiguous("token_major", 1, 5, 6, 3, 8, 64, a, 0);
    const int32_t one[] = {1};
    run_contiguous("single_token", 0, 1, 4, 4, 128, 1, one, 1);
    const int32_t p[] = {17, 16, 1, 40, 0, 31};
    run_paged("paged16", 6, 8, 2, 16, 16, 4, p);
    const int32_t p2[] = {3, 4, 9};
    run_paged("paged2", 3, 4, 1, 4, 2, 5, p2);
    return 0;
}
