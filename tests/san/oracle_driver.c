/*
 * Sanitizer driver of the CPU oracle (test infrastructure): includes the oracle's source, so that its static helpers
 * are instrumented too, and runs one small case of every entry point with every buffer allocated at its exact size,
 * so that any access past a pool, a page-table row or an output is an AddressSanitizer report.  Built by
 * tests/test_sanitizers_host.py with gcc -fsanitize=address,undefined; exit status 0 means no report and the
 * cross-checks below held.
 */
#include "../../oracle/nexus_oracle.c"

#include <stdio.h>

static unsigned long long rng_state = 88172645463325252ull;
static float rnd(void)
{ /* xorshift: uniform in (-1, 1) */
    rng_state ^= rng_state << 13;
    rng_state ^= rng_state >> 7;
    rng_state ^= rng_state << 17;
    return (float)((double)(rng_state >> 11) / 9007199254740992.0 * 2.0 - 1.0);
}
static float *vec(size_t n, float scale)
{
    float *p = (float *)malloc(sizeof(float) * n);
    for (size_t i = 0; i < n; ++i) p[i] = rnd() * scale;
    return p;
}
#define CHECK(c)                                                   \
    do {                                                           \
        if (!(c)) {                                                \
            fprintf(stderr, "check failed: %s (line %d)\n", #c, __LINE__); \
            return 1;                                              \
        }                                                          \
    } while (0)

int main(void)
{
    oracle_model m = {32, 4, 2, 8, 24, 4, 1e-5f, 10000.0f};
    int d = m.hidden, qd = m.n_q_heads * m.head_dim, kvd = m.n_kv_heads * m.head_dim, nqkv = qd + 2 * kvd, F = m.ffn;
    oracle_weights w;
    float *g1 = vec(d, 0.1f), *g2 = vec(d, 0.1f);
    for (int i = 0; i < d; ++i) g1[i] += 1.f, g2[i] += 1.f;
    w.attn_norm_g = g1, w.ffn_norm_g = g2;
    w.w_qkv = vec((size_t)nqkv * d, 0.2f), w.b_qkv = vec(nqkv, 0.2f), w.w_o = vec((size_t)d * qd, 0.2f);
    w.w_gate_up = vec((size_t)2 * F * d, 0.2f), w.w_down = vec((size_t)d * F, 0.2f);

    /* prefill: request 0 = 5 tokens over a prefix of 6 (3 pages), request 1 = 7 tokens from scratch (2 pages);
       decode: contexts 0, 3 and 4 (1, 1 and 2 pages).  The pool holds exactly these 9 pages, permuted. */
    int32_t cu[3] = {0, 5, 12}, prefix[2] = {6, 0};
    int32_t pt_p[2 * 3] = {7, 2, 5, 0, 8, -1};
    int32_t ctx[3] = {0, 3, 4};
    int32_t pt_d[3 * 2] = {4, -1, 1, -1, 6, 3};
    int n_pages = 9, T = 12;
    size_t pool_elems = (size_t)n_pages * m.n_kv_heads * m.page_size * m.head_dim;
    float *kp = vec(pool_elems, 1.f), *vp = vec(pool_elems, 1.f);
    float *kp2 = (float *)malloc(sizeof(float) * pool_elems), *vp2 = (float *)malloc(sizeof(float) * pool_elems);
    memcpy(kp2, kp, sizeof(float) * pool_elems), memcpy(vp2, vp, sizeof(float) * pool_elems);
    float *x = vec((size_t)T * d, 1.f), *y = (float *)malloc(sizeof(float) * T * d);
    float *q = (float *)malloc(sizeof(float) * T * qd), *at = (float *)malloc(sizeof(float) * T * qd), *x1 = (float *)malloc(sizeof(float) * T * d);
    oracle_layer_prefill(&m, &w, x, 2, cu, prefix, pt_p, 3, kp, vp, y, q, at, x1);
    for (int i = 0; i < T * d; ++i) CHECK(isfinite(y[i]));

    /* the row-subset entry on the same batch: identical rows, identical pools */
    int32_t rows[4] = {11, 0, 4, 5};
    float *yr = (float *)malloc(sizeof(float) * 4 * d);
    oracle_layer_prefill_rows(&m, &w, x, 2, cu, prefix, pt_p, 3, kp2, vp2, 4, rows, 0, yr);
    for (int i = 0; i < 4; ++i) CHECK(memcmp(yr + (size_t)i * d, y + (size_t)rows[i] * d, sizeof(float) * d) == 0);
    CHECK(memcmp(kp, kp2, sizeof(float) * pool_elems) == 0 && memcmp(vp, vp2, sizeof(float) * pool_elems) == 0);
    oracle_layer_prefill_rows(&m, &w, x, 2, cu, prefix, pt_p, 3, kp2, vp2, 4, rows, 1, yr); /* bf16 cache storage */
    for (int i = 0; i < 4 * d; ++i) CHECK(isfinite(yr[i]));

    float *xd = vec((size_t)3 * d, 1.f), *yd = (float *)malloc(sizeof(float) * 3 * d);
    oracle_layer_decode(&m, &w, xd, 3, ctx, pt_d, 2, kp, vp, yd, NULL, NULL, NULL);
    for (int i = 0; i < 3 * d; ++i) CHECK(isfinite(yd[i]));

    /* primitives with exact-size buffers */
    float *kc = (float *)malloc(sizeof(float) * 11 * kvd), *vc = (float *)malloc(sizeof(float) * 11 * kvd);
    oracle_kv_gather(&m, kp, vp, pt_p, 11, kc, vc);
    float *a1 = (float *)malloc(sizeof(float) * qd), *a2 = (float *)malloc(sizeof(float) * qd), *pr = (float *)malloc(sizeof(float) * m.n_q_heads * 11);
    oracle_attention_contig(&m, q + (size_t)4 * qd, 10, kc, vc, a1, pr);
    oracle_attention_paged(&m, q + (size_t)4 * qd, 10, kp, vp, pt_p, a2, NULL);
    CHECK(memcmp(a1, a2, sizeof(float) * qd) == 0);
    for (int h = 0; h < m.n_q_heads; ++h) {
        double s = 0;
        for (int u = 0; u < 11; ++u) s += pr[h * 11 + u];
        CHECK(fabs(s - 1.0) < 1e-5);
    }
    float tp[3] = {3.f, 2.f, 1.f}, td[3] = {1.f, 2.f, 4.f}, ts[3] = {3.f, 2.5f, 4.f};
    CHECK(oracle_choose_split(3, tp, td, ts, 1.f, 1.f, 2, 1.3f, 1.1f) == 1);
    CHECK(oracle_choose_split(3, tp, td, ts, 1.f, 1.f, 0, 1.3f, 1.1f) == 0);
    CHECK(oracle_num_threads() >= 1);
    free(g1), free(g2), free((void *)w.w_qkv), free((void *)w.b_qkv), free((void *)w.w_o), free((void *)w.w_gate_up), free((void *)w.w_down);
    free(kp), free(vp), free(kp2), free(vp2), free(x), free(y), free(q), free(at), free(x1), free(yr), free(xd), free(yd);
    free(kc), free(vc), free(a1), free(a2), free(pr);
    puts("oracle sanitizer driver: ok");
    return 0;
}
