/*
 * nexus_oracle.c -- TEST INFRASTRUCTURE, NOT PRODUCT CODE.
 *
 * A plain, slow, obviously-correct CPU implementation of one decoder layer as
 * it is evaluated by the two phases of the intra-GPU prefill/decode
 * disaggregated step (paper Sec. 2.2 Eq. 1-3, Sec. 2.3 Eq. 4): a chunked
 * prefill sub-batch and a decode sub-batch over a shared paged KV cache.
 * The partitioned concurrent step changes where and when the layer runs, not
 * what it computes, so the oracle is the plain definition of the layer.
 *
 * Only tests, the smoke check and the benchmark's cpu_baseline leg may call
 * this file.  It shares no code, header, table or constant with the HIP path.
 *
 * Arithmetic: every array that crosses a function boundary is fp32; every
 * reduction (dot products, sums of squares, softmax sums) and every
 * transcendental is carried in fp64 and rounded to fp32 once, when stored.
 * There is no blocking, fusion or reordering: loops run in index order.
 * OpenMP is used over tokens / heads only (independent outputs).
 *
 * Readings of the paper taken here (the text leaves these open):
 *   - layer family: pre-norm RMSNorm, rotary embedding, grouped-query
 *     attention, SwiGLU feed-forward, no biases except an optional QKV bias
 *     (the evaluated models of Sec. 6.1 are of this family; Fig. 2 omits the
 *     normalisation, Eq. 3 prints a GELU two-matrix FFN);
 *   - softmax scale 1/sqrt(head_dim) (Eq. 4 overloads d);
 *   - causal visibility: query at absolute position pos sees keys 0..pos;
 *   - rotary pairing (j, j + head_dim/2), angle pos * theta^(-2j/head_dim);
 *   - keys are cached after rotation; q head h uses kv head h / G;
 *   - KV cache: pages of page_size tokens, canonical pool layout
 *     [n_pages][n_kv_heads][page_size][head_dim]; token at position pos of
 *     request r lives in page page_table[r][pos / page_size], slot
 *     pos % page_size;
 *   - a decode request with context length c holds c cached tokens; its new
 *     token sits at position c and attends to c + 1 keys;
 *   - a prefill chunk appends all its tokens' K/V before attention is read.
 *
 * Parity pins live in tests/test_oracle_*.py.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

#define ORACLE_API __attribute__((visibility("default")))

typedef struct {
    int32_t hidden, n_q_heads, n_kv_heads, head_dim, ffn, page_size;
    float rms_eps, rope_theta;
} oracle_model;

typedef struct {
    const float *attn_norm_g; /* [hidden]                         */
    const float *w_qkv;       /* [(Hq + 2 Hkv) * hd][hidden]      */
    const float *b_qkv;       /* [(Hq + 2 Hkv) * hd] or NULL      */
    const float *w_o;         /* [hidden][Hq * hd]                */
    const float *ffn_norm_g;  /* [hidden]                         */
    const float *w_gate_up;   /* [2 * ffn][hidden], gate rows first */
    const float *w_down;      /* [hidden][ffn]                    */
} oracle_weights;

ORACLE_API int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

ORACLE_API void oracle_set_num_threads(int n)
{
#ifdef _OPENMP
    if (n > 0) omp_set_num_threads(n);
#else
    (void)n;
#endif
}

/* RMSNorm of one row: out = x * rsqrt(mean(x^2) + eps) * g. */
ORACLE_API void oracle_rmsnorm_row(const float *x, const float *g, int d, float eps, float *out)
{
    double ss = 0.0;
    for (int i = 0; i < d; ++i) ss += (double)x[i] * (double)x[i];
    double inv = 1.0 / sqrt(ss / (double)d + (double)eps);
    for (int i = 0; i < d; ++i) out[i] = (float)((double)x[i] * inv * (double)g[i]);
}

ORACLE_API void oracle_rmsnorm(const float *x, const float *g, int T, int d, float eps, float *out)
{
#pragma omp parallel for schedule(static)
    for (int t = 0; t < T; ++t) oracle_rmsnorm_row(x + (size_t)t * d, g, d, eps, out + (size_t)t * d);
}

/* y[t][o] = sum_i x[t][i] * W[o][i] (+ b[o]); W is [n_out][n_in] (Eq. 1-3: Y = X W with W stored transposed). */
ORACLE_API void oracle_linear(const float *x, const float *W, const float *b, int T, int n_in, int n_out, float *y)
{
#pragma omp parallel for collapse(2) schedule(static)
    for (int t = 0; t < T; ++t) {
        for (int o = 0; o < n_out; ++o) {
            const float *xr = x + (size_t)t * n_in;
            const float *wr = W + (size_t)o * n_in;
            double acc = 0.0;
            for (int i = 0; i < n_in; ++i) acc += (double)xr[i] * (double)wr[i];
            if (b) acc += (double)b[o];
            y[(size_t)t * n_out + o] = (float)acc;
        }
    }
}

/* Rotary embedding of n_heads vectors of length hd (contiguous) at position pos, in place. */
ORACLE_API void oracle_rope(float *u, int n_heads, int hd, int pos, float theta)
{
    int half = hd / 2;
    for (int h = 0; h < n_heads; ++h) {
        float *v = u + (size_t)h * hd;
        for (int j = 0; j < half; ++j) {
            double freq = pow((double)theta, -2.0 * (double)j / (double)hd);
            double phi = (double)pos * freq;
            double c = cos(phi), s = sin(phi);
            double a = v[j], bb = v[j + half];
            v[j] = (float)(a * c - bb * s);
            v[j + half] = (float)(bb * c + a * s);
        }
    }
}

/* Paged addressing: where the token at position pos of a request lives. */
ORACLE_API void oracle_kv_slot(const int32_t *page_table_row, int pos, int page_size, int32_t *page, int32_t *slot)
{
    *page = page_table_row[pos / page_size];
    *slot = pos % page_size;
}

static inline size_t pool_index(const oracle_model *m, int page, int kvh, int slot)
{
    return (((size_t)page * m->n_kv_heads + kvh) * m->page_size + slot) * (size_t)m->head_dim;
}

/* Store one token's K (already rotated) and V, [Hkv][hd] each, at position pos. */
ORACLE_API void oracle_kv_append(const oracle_model *m, float *k_pool, float *v_pool, const int32_t *page_table_row,
                                 int pos, const float *k, const float *v)
{
    int32_t page, slot;
    oracle_kv_slot(page_table_row, pos, m->page_size, &page, &slot);
    for (int h = 0; h < m->n_kv_heads; ++h) {
        size_t o = pool_index(m, page, h, slot);
        memcpy(k_pool + o, k + (size_t)h * m->head_dim, sizeof(float) * m->head_dim);
        memcpy(v_pool + o, v + (size_t)h * m->head_dim, sizeof(float) * m->head_dim);
    }
}

/* Copy positions [0, len) of a request out of the pools into contiguous [len][Hkv][hd] arrays. */
ORACLE_API void oracle_kv_gather(const oracle_model *m, const float *k_pool, const float *v_pool,
                                 const int32_t *page_table_row, int len, float *k_out, float *v_out)
{
    for (int u = 0; u < len; ++u) {
        int32_t page, slot;
        oracle_kv_slot(page_table_row, u, m->page_size, &page, &slot);
        for (int h = 0; h < m->n_kv_heads; ++h) {
            size_t o = pool_index(m, page, h, slot);
            size_t d = ((size_t)u * m->n_kv_heads + h) * m->head_dim;
            memcpy(k_out + d, k_pool + o, sizeof(float) * m->head_dim);
            memcpy(v_out + d, v_pool + o, sizeof(float) * m->head_dim);
        }
    }
}

/*
 * Attention of one query token (all Hq heads) at absolute position pos over
 * keys 0..pos held contiguously: K, V are [>= pos+1][Hkv][hd] (Eq. 4 with the
 * causal bound and the 1/sqrt(head_dim) scale).  p_out (nullable) receives the
 * softmax probabilities, [Hq][pos + 1].
 */
ORACLE_API void oracle_attention_contig(const oracle_model *m, const float *q, int pos, const float *K, const float *V,
                                        float *a, float *p_out)
{
    int hd = m->head_dim, G = m->n_q_heads / m->n_kv_heads, n = pos + 1;
    double scale = 1.0 / sqrt((double)hd);
    double *s = (double *)malloc(sizeof(double) * (size_t)n);
    for (int hq = 0; hq < m->n_q_heads; ++hq) {
        int kvh = hq / G;
        const float *qh = q + (size_t)hq * hd;
        double mx = -INFINITY;
        for (int u = 0; u < n; ++u) {
            const float *ku = K + ((size_t)u * m->n_kv_heads + kvh) * hd;
            double acc = 0.0;
            for (int i = 0; i < hd; ++i) acc += (double)qh[i] * (double)ku[i];
            s[u] = acc * scale;
            if (s[u] > mx) mx = s[u];
        }
        double denom = 0.0;
        for (int u = 0; u < n; ++u) {
            s[u] = exp(s[u] - mx);
            denom += s[u];
        }
        for (int u = 0; u < n; ++u) s[u] /= denom;
        if (p_out)
            for (int u = 0; u < n; ++u) p_out[(size_t)hq * n + u] = (float)s[u];
        for (int i = 0; i < hd; ++i) {
            double acc = 0.0;
            for (int u = 0; u < n; ++u) acc += s[u] * (double)V[((size_t)u * m->n_kv_heads + kvh) * hd + i];
            a[(size_t)hq * hd + i] = (float)acc;
        }
    }
    free(s);
}

/* The same attention with keys and values read through the page table. */
ORACLE_API void oracle_attention_paged(const oracle_model *m, const float *q, int pos, const float *k_pool,
                                       const float *v_pool, const int32_t *page_table_row, float *a, float *p_out)
{
    int hd = m->head_dim, G = m->n_q_heads / m->n_kv_heads, n = pos + 1;
    double scale = 1.0 / sqrt((double)hd);
    double *s = (double *)malloc(sizeof(double) * (size_t)n);
    for (int hq = 0; hq < m->n_q_heads; ++hq) {
        int kvh = hq / G;
        const float *qh = q + (size_t)hq * hd;
        double mx = -INFINITY;
        for (int u = 0; u < n; ++u) {
            int32_t page, slot;
            oracle_kv_slot(page_table_row, u, m->page_size, &page, &slot);
            const float *ku = k_pool + pool_index(m, page, kvh, slot);
            double acc = 0.0;
            for (int i = 0; i < hd; ++i) acc += (double)qh[i] * (double)ku[i];
            s[u] = acc * scale;
            if (s[u] > mx) mx = s[u];
        }
        double denom = 0.0;
        for (int u = 0; u < n; ++u) {
            s[u] = exp(s[u] - mx);
            denom += s[u];
        }
        for (int u = 0; u < n; ++u) s[u] /= denom;
        if (p_out)
            for (int u = 0; u < n; ++u) p_out[(size_t)hq * n + u] = (float)s[u];
        for (int i = 0; i < hd; ++i) {
            double acc = 0.0;
            for (int u = 0; u < n; ++u) {
                int32_t page, slot;
                oracle_kv_slot(page_table_row, u, m->page_size, &page, &slot);
                acc += s[u] * (double)v_pool[pool_index(m, page, kvh, slot) + i];
            }
            a[(size_t)hq * hd + i] = (float)acc;
        }
    }
    free(s);
}

/* SwiGLU: act[f] = silu(gu[f]) * gu[F + f], silu(z) = z / (1 + exp(-z)). */
ORACLE_API void oracle_swiglu(const float *gu, int T, int F, float *act)
{
#pragma omp parallel for schedule(static)
    for (int t = 0; t < T; ++t)
        for (int f = 0; f < F; ++f) {
            double z = gu[(size_t)t * 2 * F + f], up = gu[(size_t)t * 2 * F + F + f];
            act[(size_t)t * F + f] = (float)(z / (1.0 + exp(-z)) * up);
        }
}

/*
 * Everything after attention: x1 = x + a W_o^T (Eq. 2); y = x1 + W_d(silu(W_g h2) * (W_u h2)),
 * h2 = RMSNorm(x1) (Eq. 3 in its SwiGLU form).  x1_out is nullable.
 */
static void post_attention(const oracle_model *m, const oracle_weights *w, const float *x, const float *a, int T,
                           float *y, float *x1_out)
{
    int d = m->hidden, qd = m->n_q_heads * m->head_dim, F = m->ffn;
    float *x1 = (float *)malloc(sizeof(float) * (size_t)T * d);
    float *h2 = (float *)malloc(sizeof(float) * (size_t)T * d);
    float *gu = (float *)malloc(sizeof(float) * (size_t)T * 2 * F);
    float *act = (float *)malloc(sizeof(float) * (size_t)T * F);
    oracle_linear(a, w->w_o, NULL, T, qd, d, x1);
    for (size_t i = 0; i < (size_t)T * d; ++i) x1[i] = (float)((double)x[i] + (double)x1[i]);
    if (x1_out) memcpy(x1_out, x1, sizeof(float) * (size_t)T * d);
    oracle_rmsnorm(x1, w->ffn_norm_g, T, d, m->rms_eps, h2);
    oracle_linear(h2, w->w_gate_up, NULL, T, d, 2 * F, gu);
    oracle_swiglu(gu, T, F, act);
    oracle_linear(act, w->w_down, NULL, T, F, d, y);
    for (size_t i = 0; i < (size_t)T * d; ++i) y[i] = (float)((double)x1[i] + (double)y[i]);
    free(x1);
    free(h2);
    free(gu);
    free(act);
}

/*
 * One layer over a batch of tokens whose absolute positions and owning
 * requests are given.  Shared by the two phases: a prefill chunk is a run of
 * consecutive positions of one request, a decode step is one position per
 * request.  All tokens' K/V are appended first, then every token attends to
 * keys 0..pos of its own request through that request's page-table row.
 *
 * Nullable debug outputs: q_out [T][Hq*hd] (rotated queries), attn_out
 * [T][Hq*hd], x1_out [T][hidden].
 */
static void layer_tokens(const oracle_model *m, const oracle_weights *w, const float *x, int T, const int32_t *tok_req,
                         const int32_t *tok_pos, const int32_t *page_table, int max_pages, float *k_pool,
                         float *v_pool, float *y, float *q_out, float *attn_out, float *x1_out)
{
    int d = m->hidden, hd = m->head_dim, Hq = m->n_q_heads, Hkv = m->n_kv_heads;
    int qd = Hq * hd, kvd = Hkv * hd, nqkv = qd + 2 * kvd;
    float *h = (float *)malloc(sizeof(float) * (size_t)T * d);
    float *qkv = (float *)malloc(sizeof(float) * (size_t)T * nqkv);
    float *a = (float *)malloc(sizeof(float) * (size_t)T * qd);

    oracle_rmsnorm(x, w->attn_norm_g, T, d, m->rms_eps, h);
    oracle_linear(h, w->w_qkv, w->b_qkv, T, d, nqkv, qkv);
    for (int t = 0; t < T; ++t) {
        float *row = qkv + (size_t)t * nqkv;
        oracle_rope(row, Hq, hd, tok_pos[t], m->rope_theta);
        oracle_rope(row + qd, Hkv, hd, tok_pos[t], m->rope_theta);
        oracle_kv_append(m, k_pool, v_pool, page_table + (size_t)tok_req[t] * max_pages, tok_pos[t], row + qd,
                         row + qd + kvd);
    }
#pragma omp parallel for schedule(dynamic, 1)
    for (int t = 0; t < T; ++t)
        oracle_attention_paged(m, qkv + (size_t)t * nqkv, tok_pos[t], k_pool, v_pool,
                               page_table + (size_t)tok_req[t] * max_pages, a + (size_t)t * qd, NULL);
    if (q_out)
        for (int t = 0; t < T; ++t) memcpy(q_out + (size_t)t * qd, qkv + (size_t)t * nqkv, sizeof(float) * qd);
    if (attn_out) memcpy(attn_out, a, sizeof(float) * (size_t)T * qd);
    post_attention(m, w, x, a, T, y, x1_out);
    free(h);
    free(qkv);
    free(a);
}

/*
 * Chunked-prefill phase of one layer.  Requests are packed: request r owns
 * tokens cu_chunk[r] .. cu_chunk[r+1]-1, which sit at absolute positions
 * prefix_len[r] + 0, 1, ...; positions below prefix_len[r] are already cached.
 */
ORACLE_API void oracle_layer_prefill(const oracle_model *m, const oracle_weights *w, const float *x, int n_reqs,
                                     const int32_t *cu_chunk, const int32_t *prefix_len, const int32_t *page_table,
                                     int max_pages, float *k_pool, float *v_pool, float *y, float *q_out,
                                     float *attn_out, float *x1_out)
{
    int T = cu_chunk[n_reqs];
    int32_t *req = (int32_t *)malloc(sizeof(int32_t) * (size_t)(T > 0 ? T : 1));
    int32_t *pos = (int32_t *)malloc(sizeof(int32_t) * (size_t)(T > 0 ? T : 1));
    for (int r = 0; r < n_reqs; ++r)
        for (int t = cu_chunk[r]; t < cu_chunk[r + 1]; ++t) {
            req[t] = r;
            pos[t] = prefix_len[r] + (t - cu_chunk[r]);
        }
    layer_tokens(m, w, x, T, req, pos, page_table, max_pages, k_pool, v_pool, y, q_out, attn_out, x1_out);
    free(req);
    free(pos);
}

/*
 * The chunked-prefill phase of one layer evaluated for a listed subset of the
 * batch's rows only (Eq. 1-4, same steps as oracle_layer_prefill): the keys
 * and values of EVERY token of the batch are projected, rotated and appended
 * first (a listed row attends to all earlier rows of its chunk), then the
 * query projection, the attention and everything after it run for the rows
 * in rows[0..n_rows) alone.  y receives [n_rows][hidden] in the order of
 * rows[].  Row t of the result equals row rows[t] of oracle_layer_prefill:
 * every output row of the layer depends on the other rows only through the
 * cache.  This is what lets a test afford the last rows of a long chunk.
 */
/* fp32 -> nearest bfloat16 (ties to even) -> fp32: what a cache that stores bf16 keeps of a value. */
static float bf16_round(float f)
{
    uint32_t u;
    memcpy(&u, &f, 4);
    if ((u & 0x7fffffffu) > 0x7f800000u) return f; /* NaN */
    u += 0x7fffu + ((u >> 16) & 1u);
    u &= 0xffff0000u;
    memcpy(&f, &u, 4);
    return f;
}

/*
 * kv_store_bf16 != 0 applies the storage format of a bf16 KV cache and nothing else: the rotated keys and the values
 * are rounded to bf16 as they are stored.  It exists to MEASURE what that format alone costs against the exact
 * layer (kv_store_bf16 == 0, which is what every parity gate compares with); no gate uses the rounded variant.
 */
ORACLE_API void oracle_layer_prefill_rows(const oracle_model *m, const oracle_weights *w, const float *x, int n_reqs,
                                          const int32_t *cu_chunk, const int32_t *prefix_len,
                                          const int32_t *page_table, int max_pages, float *k_pool, float *v_pool,
                                          int n_rows, const int32_t *rows, int kv_store_bf16, float *y)
{
    int d = m->hidden, hd = m->head_dim, Hq = m->n_q_heads, Hkv = m->n_kv_heads;
    int qd = Hq * hd, kvd = Hkv * hd;
    int T = cu_chunk[n_reqs];
    int32_t *req = (int32_t *)malloc(sizeof(int32_t) * (size_t)(T > 0 ? T : 1));
    int32_t *pos = (int32_t *)malloc(sizeof(int32_t) * (size_t)(T > 0 ? T : 1));
    for (int r = 0; r < n_reqs; ++r)
        for (int t = cu_chunk[r]; t < cu_chunk[r + 1]; ++t) {
            req[t] = r;
            pos[t] = prefix_len[r] + (t - cu_chunk[r]);
        }
    /* keys and values of all tokens: the k and v rows of W_qkv follow its Hq * hd query rows */
    float *h = (float *)malloc(sizeof(float) * (size_t)T * d);
    float *kv = (float *)malloc(sizeof(float) * (size_t)T * 2 * kvd);
    oracle_rmsnorm(x, w->attn_norm_g, T, d, m->rms_eps, h);
    oracle_linear(h, w->w_qkv + (size_t)qd * d, w->b_qkv ? w->b_qkv + qd : NULL, T, d, 2 * kvd, kv);
    for (int t = 0; t < T; ++t) {
        float *row = kv + (size_t)t * 2 * kvd;
        oracle_rope(row, Hkv, hd, pos[t], m->rope_theta);
        if (kv_store_bf16)
            for (int i = 0; i < 2 * kvd; ++i) row[i] = bf16_round(row[i]);
        oracle_kv_append(m, k_pool, v_pool, page_table + (size_t)req[t] * max_pages, pos[t], row, row + kvd);
    }
    /* the listed rows: query, attention over the cache, rest of the layer */
    float *xs = (float *)malloc(sizeof(float) * (size_t)n_rows * d);
    float *hs = (float *)malloc(sizeof(float) * (size_t)n_rows * d);
    float *q = (float *)malloc(sizeof(float) * (size_t)n_rows * qd);
    float *a = (float *)malloc(sizeof(float) * (size_t)n_rows * qd);
    for (int i = 0; i < n_rows; ++i) {
        memcpy(xs + (size_t)i * d, x + (size_t)rows[i] * d, sizeof(float) * d);
        memcpy(hs + (size_t)i * d, h + (size_t)rows[i] * d, sizeof(float) * d);
    }
    oracle_linear(hs, w->w_qkv, w->b_qkv, n_rows, d, qd, q);
#pragma omp parallel for schedule(dynamic, 1)
    for (int i = 0; i < n_rows; ++i) {
        int t = rows[i];
        oracle_rope(q + (size_t)i * qd, Hq, hd, pos[t], m->rope_theta);
        oracle_attention_paged(m, q + (size_t)i * qd, pos[t], k_pool, v_pool,
                               page_table + (size_t)req[t] * max_pages, a + (size_t)i * qd, NULL);
    }
    post_attention(m, w, xs, a, n_rows, y, NULL);
    free(req);
    free(pos);
    free(h);
    free(kv);
    free(xs);
    free(hs);
    free(q);
    free(a);
}

/* Decode phase of one layer: request j contributes one token at position ctx_len[j]. */
ORACLE_API void oracle_layer_decode(const oracle_model *m, const oracle_weights *w, const float *x, int n_reqs,
                                    const int32_t *ctx_len, const int32_t *page_table, int max_pages, float *k_pool,
                                    float *v_pool, float *y, float *q_out, float *attn_out, float *x1_out)
{
    int32_t *req = (int32_t *)malloc(sizeof(int32_t) * (size_t)(n_reqs > 0 ? n_reqs : 1));
    for (int j = 0; j < n_reqs; ++j) req[j] = j;
    layer_tokens(m, w, x, n_reqs, req, ctx_len, page_table, max_pages, k_pool, v_pool, y, q_out, attn_out, x1_out);
    free(req);
}

/*
 * Split selection from measured latency curves (Sec. 4.1.2 applied to
 * measurements instead of the cost model).  Candidate i gives the prefill
 * phase cand_prefill[i] units and the decode phase the rest.  t_p_min and
 * t_d_min are the phase latencies with the whole GPU.
 *   policy 0, prefill-prioritised: minimise t_p subject to t_d <= beta * t_d_min;
 *   policy 1, decode-prioritised:  minimise t_d subject to t_p <= alpha * t_p_min;
 *   policy 2, minimum measured concurrent step time.
 * Returns the index of the chosen candidate; when no candidate meets the
 * constraint, the one violating it least.  Ties go to the lower index.
 */
ORACLE_API int oracle_choose_split(int n, const float *t_p, const float *t_d, const float *t_step, float t_p_min,
                                   float t_d_min, int policy, float alpha, float beta)
{
    int best = -1;
    if (policy == 2) {
        for (int i = 0; i < n; ++i)
            if (best < 0 || t_step[i] < t_step[best]) best = i;
        return best;
    }
    const float *obj = policy == 0 ? t_p : t_d;
    const float *con = policy == 0 ? t_d : t_p;
    double bound = policy == 0 ? (double)beta * t_d_min : (double)alpha * t_p_min;
    for (int i = 0; i < n; ++i)
        if ((double)con[i] <= bound && (best < 0 || obj[i] < obj[best])) best = i;
    if (best >= 0) return best;
    for (int i = 0; i < n; ++i)
        if (best < 0 || con[i] < con[best]) best = i;
    return best;
}
