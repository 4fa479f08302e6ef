/*
 * ukv_oracle.c -- plain CPU oracle for the unified-KV decode path.
 *
 * TEST INFRASTRUCTURE ONLY.  Nothing on the product path may include, link or
 * call this file: it exists so that tests, the smoke check and the benchmark's
 * cpu_baseline leg have an independent statement of what the path computes.
 * It shares no code, header, table or helper with the HIP library.
 *
 * What it states (SeaLLM, arXiv 2504.15720):
 *   - Decode phase (section 2.1, "LLM Service"): one new token per request per
 *     step; its query attends to every cached key/value pair of the request.
 *     The result has a plain definition, out = softmax(q K^T * scale) V per
 *     query head, which is written out here directly in fp64: gather, scores,
 *     max, exponentials, normalise, weighted sum.  No tiling, no running
 *     maximum, no split/merge.
 *   - Unified KV cache with merged blocks (section 4.4): all services share
 *     one pool of equal-sized blocks ("pages"); a per-request block table
 *     names the physical block and a second index gives the place inside it.
 *     Reading taken here (the paper's figure of the block is not available):
 *     a request's cache is one byte stream, token-major, then kv-head-major,
 *     then K[d] followed by V[d] in bf16 (one "head-row" of 4*d bytes); page
 *     slot = stream_offset / page_bytes names the table entry, and the second
 *     index is stream_offset % page_bytes.  A token occupies
 *     n_kv_heads*head_dim*2*2 bytes (the paper's 4 GB example for Llama2-7B,
 *     section 2.3, is 8192 tokens * 32 layers of exactly this).  Head-rows never
 *     straddle pages (page_bytes % head_row_bytes == 0 is required); token rows may.
 *   - Query head a reads kv head a / (n_q_heads / n_kv_heads).
 *   - Prefill phase (section 2.1): all tokens of the prompt (or of a chunk of
 *     it) are processed in one pass that also leaves their key/value pairs in
 *     the cache.  Reading taken here (the paper serves decoder-only models and
 *     does not restate the mask): the pass is causal, i.e. the query of the
 *     token at position p attends to the cached pairs of positions 0..p, so
 *     that its result is what a decode step at that position would compute.
 *     ukv_oracle_prefill writes that definition out position by position.
 *
 * Pins (tests/, -m "not gpu"): brute force on contiguous arrays, torch's fp64
 * scaled_dot_product_attention, closed forms (constant V, one token, equal
 * keys, two-token logistic, zero query), invariances (page renaming, token
 * order, score shift, batch composition), hand-worked address fixtures, the
 * 4 GiB closed form, and sentinel checks for append.  Prefill: the masked-matrix
 * formulation in numpy, torch's fp64 SDPA with is_causal, position 0 = value 0,
 * last position = the decode entry point, zero queries = running means, and
 * causality (rewriting later tokens leaves earlier positions bit-identical).
 *
 * Parallelism: OpenMP over requests only.  fp64 throughout; bf16 inputs are
 * widened exactly.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ORC_OK 0
#define ORC_EINVAL (-1)
#define ORC_ERANGE (-2) /* table entry missing / page id outside the pool */
#define ORC_ENOMEM (-3)

static double bf16_to_f64(uint16_t bits)
{
    uint32_t w = (uint32_t)bits << 16;
    float f;
    memcpy(&f, &w, sizeof f);
    return (double)f;
}

/* Byte address, inside the pool image, of the head-row of (token t, kv head h).
 * Returns UINT64_MAX if the table has no valid page for it. */
static uint64_t head_row_address(uint64_t page_bytes, uint64_t n_pages, const int32_t *table,
                                 uint64_t table_len, uint64_t token_bytes, uint64_t head_row_bytes,
                                 uint64_t t, uint64_t h)
{
    uint64_t stream = t * token_bytes + h * head_row_bytes;
    uint64_t slot = stream / page_bytes;
    uint64_t second_index = stream % page_bytes;
    if (slot >= table_len)
        return UINT64_MAX;
    int64_t page = table[slot];
    if (page < 0 || (uint64_t)page >= n_pages)
        return UINT64_MAX;
    return (uint64_t)page * page_bytes + second_index;
}

static int shape_ok(uint32_t page_bytes, uint32_t n_q, uint32_t n_kv, uint32_t d)
{
    if (n_q == 0 || n_kv == 0 || d == 0 || n_q % n_kv != 0)
        return 0;
    uint64_t row = 4ull * d;
    return page_bytes != 0 && page_bytes % row == 0;
}

/* Copy the first n_tokens of one request out of the pool into contiguous
 * k_out[n][H][d], v_out[n][H][d] (bf16 bit patterns, unchanged). */
int ukv_oracle_gather(const uint8_t *pool, uint64_t pool_bytes, uint32_t page_bytes, const int32_t *table,
                      uint64_t table_len, uint32_t n_kv_heads, uint32_t head_dim, uint64_t n_tokens,
                      uint16_t *k_out, uint16_t *v_out)
{
    if (!shape_ok(page_bytes, n_kv_heads, n_kv_heads, head_dim))
        return ORC_EINVAL;
    uint64_t n_pages = pool_bytes / page_bytes;
    uint64_t row = 4ull * head_dim, tok = row * n_kv_heads;
    for (uint64_t t = 0; t < n_tokens; ++t)
        for (uint64_t h = 0; h < n_kv_heads; ++h) {
            uint64_t a = head_row_address(page_bytes, n_pages, table, table_len, tok, row, t, h);
            if (a == UINT64_MAX)
                return ORC_ERANGE;
            memcpy(k_out + (t * n_kv_heads + h) * head_dim, pool + a, 2ull * head_dim);
            memcpy(v_out + (t * n_kv_heads + h) * head_dim, pool + a + 2ull * head_dim, 2ull * head_dim);
        }
    return ORC_OK;
}

/* The inverse of gather, for a run of tokens: write contiguous k_in[n][H][d], v_in[n][H][d] as tokens
 * [first_token, first_token + n) of one request's stream.  first_token = 0 is the bulk store after a
 * whole-prompt prefill or the receiving side of a migration; first_token > 0 is the bulk append of a
 * chunk in chunked prefill (section 2.1: the pass over a chunk leaves its KV pairs in the cache behind
 * those of the earlier chunks). */
int ukv_oracle_scatter(uint8_t *pool, uint64_t pool_bytes, uint32_t page_bytes, const int32_t *table,
                       uint64_t table_len, uint32_t n_kv_heads, uint32_t head_dim, uint64_t first_token,
                       uint64_t n_tokens, const uint16_t *k_in, const uint16_t *v_in)
{
    if (!shape_ok(page_bytes, n_kv_heads, n_kv_heads, head_dim))
        return ORC_EINVAL;
    uint64_t n_pages = pool_bytes / page_bytes;
    uint64_t row = 4ull * head_dim, tok = row * n_kv_heads;
    for (uint64_t t = 0; t < n_tokens; ++t)
        for (uint64_t h = 0; h < n_kv_heads; ++h) {
            uint64_t a = head_row_address(page_bytes, n_pages, table, table_len, tok, row, first_token + t, h);
            if (a == UINT64_MAX)
                return ORC_ERANGE;
            memcpy(pool + a, k_in + (t * n_kv_heads + h) * head_dim, 2ull * head_dim);
            memcpy(pool + a + 2ull * head_dim, v_in + (t * n_kv_heads + h) * head_dim, 2ull * head_dim);
        }
    return ORC_OK;
}

/* Append: for request i write new_k[i][H][d], new_v[i][H][d] as token index
 * ctx_len[i]-1 of its stream (ctx_len already counts the new token). */
int ukv_oracle_append(uint8_t *pool, uint64_t pool_bytes, uint32_t page_bytes, uint32_t n_requests,
                      const uint32_t *n_kv_heads, const uint32_t *head_dim, const uint32_t *ctx_len,
                      const uint64_t *table_off, const uint64_t *table_len, const int32_t *page_table,
                      const uint16_t *new_k, const uint16_t *new_v, const uint64_t *new_off)
{
    uint64_t n_pages = pool_bytes / page_bytes;
    for (uint32_t i = 0; i < n_requests; ++i) {
        uint32_t H = n_kv_heads[i], d = head_dim[i];
        if (!shape_ok(page_bytes, H, H, d))
            return ORC_EINVAL;
        if (ctx_len[i] == 0)
            continue;
        uint64_t row = 4ull * d, tok = row * H, t = (uint64_t)ctx_len[i] - 1;
        for (uint64_t h = 0; h < H; ++h) {
            uint64_t a = head_row_address(page_bytes, n_pages, page_table + table_off[i], table_len[i], tok,
                                          row, t, h);
            if (a == UINT64_MAX)
                return ORC_ERANGE;
            memcpy(pool + a, new_k + new_off[i] + h * d, 2ull * d);
            memcpy(pool + a + 2ull * d, new_v + new_off[i] + h * d, 2ull * d);
        }
    }
    return ORC_OK;
}

/* One request, tokens [t0, t1): for every query head, the maximum score m, the
 * sum l of exp(s - m), and acc[j] = sum_t exp(s_t - m) V[t][j].  Full attention
 * is acc / l over [0, n).  Scores use natural exp; scale multiplies q.K. */
static int attend_range(const uint8_t *pool, uint64_t n_pages, uint32_t page_bytes, const int32_t *table,
                        uint64_t table_len, uint32_t Q, uint32_t H, uint32_t d, double scale, uint64_t t0,
                        uint64_t t1, const uint16_t *q, double *m_out, double *l_out, double *acc_out)
{
    uint64_t n = t1 - t0, row = 4ull * d, tok = row * H;
    uint32_t G = Q / H;
    double *K = (double *)malloc(sizeof(double) * (n ? n : 1) * d);
    double *V = (double *)malloc(sizeof(double) * (n ? n : 1) * d);
    double *s = (double *)malloc(sizeof(double) * (n ? n : 1));
    double *qf = (double *)malloc(sizeof(double) * d);
    int rc = ORC_OK;
    if (!K || !V || !s || !qf) {
        rc = ORC_ENOMEM;
        goto done;
    }
    for (uint32_t h = 0; h < H && rc == ORC_OK; ++h) {
        /* gather this kv head's keys and values into contiguous fp64 */
        for (uint64_t t = 0; t < n; ++t) {
            uint64_t a = head_row_address(page_bytes, n_pages, table, table_len, tok, row, t0 + t, h);
            if (a == UINT64_MAX) {
                rc = ORC_ERANGE;
                break;
            }
            const uint16_t *kr = (const uint16_t *)(pool + a);
            const uint16_t *vr = (const uint16_t *)(pool + a + 2ull * d);
            for (uint32_t j = 0; j < d; ++j) {
                K[t * d + j] = bf16_to_f64(kr[j]);
                V[t * d + j] = bf16_to_f64(vr[j]);
            }
        }
        if (rc != ORC_OK)
            break;
        for (uint32_t g = 0; g < G; ++g) {
            uint32_t a = h * G + g; /* query head a reads kv head a / G */
            for (uint32_t j = 0; j < d; ++j)
                qf[j] = bf16_to_f64(q[(uint64_t)a * d + j]);
            double m = -INFINITY;
            for (uint64_t t = 0; t < n; ++t) {
                double dot = 0.0;
                for (uint32_t j = 0; j < d; ++j)
                    dot += qf[j] * K[t * d + j];
                s[t] = dot * scale;
                if (s[t] > m)
                    m = s[t];
            }
            double l = 0.0;
            for (uint32_t j = 0; j < d; ++j)
                acc_out[(uint64_t)a * d + j] = 0.0;
            for (uint64_t t = 0; t < n; ++t) {
                double e = exp(s[t] - m);
                l += e;
                for (uint32_t j = 0; j < d; ++j)
                    acc_out[(uint64_t)a * d + j] += e * V[t * d + j];
            }
            m_out[a] = m;
            l_out[a] = l;
        }
    }
done:
    free(K);
    free(V);
    free(s);
    free(qf);
    return rc;
}

/* Decode attention for a mixed-service batch.  out is fp64 [Q_i][d_i] per request at out_off[i].
 * ctx_len == 0 gives zeros.  n_threads <= 0 means the OpenMP default. */
int ukv_oracle_attention(const uint8_t *pool, uint64_t pool_bytes, uint32_t page_bytes, uint32_t n_requests,
                         const uint32_t *n_q_heads, const uint32_t *n_kv_heads, const uint32_t *head_dim,
                         const double *scale, const uint32_t *ctx_len, const uint64_t *table_off,
                         const uint64_t *table_len, const int32_t *page_table, const uint16_t *q,
                         const uint64_t *q_off, double *out, const uint64_t *out_off, int n_threads)
{
    uint64_t n_pages = pool_bytes / page_bytes;
    int rc_all = ORC_OK;
    for (uint32_t i = 0; i < n_requests; ++i)
        if (!shape_ok(page_bytes, n_q_heads[i], n_kv_heads[i], head_dim[i]))
            return ORC_EINVAL;
#ifdef _OPENMP
    if (n_threads > 0)
        omp_set_num_threads(n_threads);
#else
    (void)n_threads;
#endif
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t i = 0; i < (int64_t)n_requests; ++i) {
        uint32_t Q = n_q_heads[i], H = n_kv_heads[i], d = head_dim[i];
        double *o = out + out_off[i];
        if (ctx_len[i] == 0) {
            for (uint64_t e = 0; e < (uint64_t)Q * d; ++e)
                o[e] = 0.0;
            continue;
        }
        double *m = (double *)malloc(sizeof(double) * Q);
        double *l = (double *)malloc(sizeof(double) * Q);
        int rc = (m && l) ? attend_range(pool, n_pages, page_bytes, page_table + table_off[i], table_len[i], Q,
                                         H, d, scale[i], 0, ctx_len[i], q + q_off[i], m, l, o)
                          : ORC_ENOMEM;
        if (rc == ORC_OK) {
            for (uint32_t a = 0; a < Q; ++a)
                for (uint32_t j = 0; j < d; ++j)
                    o[(uint64_t)a * d + j] /= l[a];
        } else {
#pragma omp critical
            rc_all = rc;
        }
        free(m);
        free(l);
    }
    return rc_all;
}

/* Un-normalised statistics of one request over the token range [t0, t1): used to state, in
 * fp64, the rule by which disjoint ranges combine (see ukv_oracle_merge). */
int ukv_oracle_attention_range(const uint8_t *pool, uint64_t pool_bytes, uint32_t page_bytes,
                               const int32_t *table, uint64_t table_len, uint32_t n_q_heads,
                               uint32_t n_kv_heads, uint32_t head_dim, double scale, uint64_t t0, uint64_t t1,
                               const uint16_t *q, double *m_out, double *l_out, double *acc_out)
{
    if (!shape_ok(page_bytes, n_q_heads, n_kv_heads, head_dim) || t1 < t0)
        return ORC_EINVAL;
    return attend_range(pool, pool_bytes / page_bytes, page_bytes, table, table_len, n_q_heads, n_kv_heads,
                        head_dim, scale, t0, t1, q, m_out, l_out, acc_out);
}

/* Prefill phase of one request (section 2.1), causal: for each listed position pos[k] (< ctx_len),
 * the query row q_rows[k] ([Q][d] bf16) attends to tokens 0..pos[k] of the request's cache, exactly
 * as the decode definition above with a context of pos[k]+1 tokens.  out: fp64 [n_pos][Q][d]. */
int ukv_oracle_prefill(const uint8_t *pool, uint64_t pool_bytes, uint32_t page_bytes, const int32_t *table,
                       uint64_t table_len, uint32_t n_q_heads, uint32_t n_kv_heads, uint32_t head_dim,
                       double scale, uint32_t ctx_len, uint32_t n_pos, const uint32_t *pos,
                       const uint16_t *q_rows, double *out, int n_threads)
{
    if (!shape_ok(page_bytes, n_q_heads, n_kv_heads, head_dim))
        return ORC_EINVAL;
    for (uint32_t k = 0; k < n_pos; ++k)
        if (pos[k] >= ctx_len)
            return ORC_EINVAL;
    uint64_t n_pages = pool_bytes / page_bytes, row = (uint64_t)n_q_heads * head_dim;
    int rc_all = ORC_OK;
#ifdef _OPENMP
    if (n_threads > 0)
        omp_set_num_threads(n_threads);
#else
    (void)n_threads;
#endif
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t k = 0; k < (int64_t)n_pos; ++k) {
        double *o = out + (uint64_t)k * row;
        double *m = (double *)malloc(sizeof(double) * n_q_heads);
        double *l = (double *)malloc(sizeof(double) * n_q_heads);
        int rc = (m && l) ? attend_range(pool, n_pages, page_bytes, table, table_len, n_q_heads, n_kv_heads,
                                         head_dim, scale, 0, (uint64_t)pos[k] + 1, q_rows + (uint64_t)k * row, m,
                                         l, o)
                          : ORC_ENOMEM;
        if (rc == ORC_OK) {
            for (uint32_t a = 0; a < n_q_heads; ++a)
                for (uint32_t j = 0; j < head_dim; ++j)
                    o[(uint64_t)a * head_dim + j] /= l[a];
        } else {
#pragma omp critical
            rc_all = rc;
        }
        free(m);
        free(l);
    }
    return rc_all;
}

/* Combine n_parts range statistics of one query head: with M = max_c m_c,
 * out = sum_c acc_c exp(m_c - M) / sum_c l_c exp(m_c - M).  Parts with l == 0 are empty. */
int ukv_oracle_merge(uint32_t n_parts, uint32_t head_dim, const double *m, const double *l, const double *acc,
                     double *out)
{
    double M = -INFINITY, L = 0.0;
    for (uint32_t c = 0; c < n_parts; ++c)
        if (l[c] > 0.0 && m[c] > M)
            M = m[c];
    for (uint32_t j = 0; j < head_dim; ++j)
        out[j] = 0.0;
    if (M == -INFINITY)
        return ORC_OK;
    for (uint32_t c = 0; c < n_parts; ++c) {
        if (!(l[c] > 0.0))
            continue;
        double w = exp(m[c] - M);
        L += l[c] * w;
        for (uint32_t j = 0; j < head_dim; ++j)
            out[j] += acc[(uint64_t)c * head_dim + j] * w;
    }
    for (uint32_t j = 0; j < head_dim; ++j)
        out[j] /= L;
    return ORC_OK;
}

int ukv_oracle_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
