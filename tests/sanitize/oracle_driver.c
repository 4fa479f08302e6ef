/* Sanitizer driver for the CPU oracle (oracle/ukv_oracle.c is compiled into this program with
 * -fsanitize=address,undefined): small seeded cases through every entry point, with exactly sized buffers so that an
 * out-of-bounds access in the oracle is reported; a few identities are checked on the way (gather after scatter
 * returns the input, a one-token context returns that token's V, split and merged = whole). */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

int ukv_oracle_gather(const uint8_t *, uint64_t, uint32_t, const int32_t *, uint64_t, uint32_t, uint32_t, uint64_t,
                      uint16_t *, uint16_t *);
int ukv_oracle_scatter(uint8_t *, uint64_t, uint32_t, const int32_t *, uint64_t, uint32_t, uint32_t, uint64_t, uint64_t,
                       const uint16_t *, const uint16_t *);
int ukv_oracle_append(uint8_t *, uint64_t, uint32_t, uint32_t, const uint32_t *, const uint32_t *, const uint32_t *,
                      const uint64_t *, const uint64_t *, const int32_t *, const uint16_t *, const uint16_t *,
                      const uint64_t *);
int ukv_oracle_attention(const uint8_t *, uint64_t, uint32_t, uint32_t, const uint32_t *, const uint32_t *,
                         const uint32_t *, const double *, const uint32_t *, const uint64_t *, const uint64_t *,
                         const int32_t *, const uint16_t *, const uint64_t *, double *, const uint64_t *, int);
int ukv_oracle_attention_range(const uint8_t *, uint64_t, uint32_t, const int32_t *, uint64_t, uint32_t, uint32_t,
                               uint32_t, double, uint64_t, uint64_t, const uint16_t *, double *, double *, double *);
int ukv_oracle_prefill(const uint8_t *, uint64_t, uint32_t, const int32_t *, uint64_t, uint32_t, uint32_t, uint32_t,
                       double, uint32_t, uint32_t, const uint32_t *, const uint16_t *, double *, int);
int ukv_oracle_merge(uint32_t, uint32_t, const double *, const double *, const double *, double *);
int ukv_oracle_threads(void);

static uint64_t g_s = 88172645463325252ull;
static uint64_t rnd(void) { g_s ^= g_s << 13; g_s ^= g_s >> 7; g_s ^= g_s << 17; return g_s; }
static uint16_t rnd_bf16(void) { /* a finite bf16 in (-2, 2) */
    float f = (float)((double)(rnd() % 4001) / 1000.0 - 2.0);
    uint32_t u;
    memcpy(&u, &f, 4);
    return (uint16_t)(u >> 16);
}
#define CHECK(c) do { if (!(c)) { fprintf(stderr, "%s:%d: %s\n", __FILE__, __LINE__, #c); exit(1); } } while (0)

static void one_case(uint32_t Q, uint32_t H, uint32_t d, uint32_t P, uint32_t n) {
    const uint64_t T = 4ull * d * H, n_tab = (n * T + P - 1) / P + ((n + 1) * T + P - 1) / P - (n * T + P - 1) / P;
    const uint64_t n_pages = n_tab + 5;
    uint8_t *pool = malloc(n_pages * P);
    memset(pool, 0xff, n_pages * P); /* NaN bit patterns outside what gets written */
    int32_t *table = malloc((n_tab ? n_tab : 1) * sizeof *table);
    for (uint64_t i = 0; i < n_tab; ++i) /* a seeded permutation of distinct pages */
        table[i] = (int32_t)((i * 7 + 3) % n_pages);
    for (uint64_t i = 0; i < n_tab; ++i)
        for (uint64_t j = 0; j < i; ++j)
            if (table[i] == table[j])
                table[i] = -1;
    for (uint64_t i = 0, next = 0; i < n_tab; ++i)
        if (table[i] < 0) {
            for (;; ++next) {
                int used = 0;
                for (uint64_t j = 0; j < n_tab; ++j)
                    used |= table[j] == (int32_t)next;
                if (!used)
                    break;
            }
            table[i] = (int32_t)next;
        }
    const uint64_t el = (uint64_t)n * H * d;
    uint16_t *k = malloc((el ? el : 1) * 2), *v = malloc((el ? el : 1) * 2), *k2 = malloc((el ? el : 1) * 2),
             *v2 = malloc((el ? el : 1) * 2), *q = malloc((uint64_t)Q * d * 2), *nk = malloc((uint64_t)H * d * 2),
             *nv = malloc((uint64_t)H * d * 2);
    for (uint64_t i = 0; i < el; ++i) k[i] = rnd_bf16(), v[i] = rnd_bf16();
    for (uint64_t i = 0; i < (uint64_t)Q * d; ++i) q[i] = rnd_bf16();
    for (uint64_t i = 0; i < (uint64_t)H * d; ++i) nk[i] = rnd_bf16(), nv[i] = rnd_bf16();
    const uint64_t n_tab0 = (n * T + P - 1) / P;
    CHECK(ukv_oracle_scatter(pool, n_pages * P, P, table, n_tab0, H, d, 0, n, k, v) == 0);
    CHECK(ukv_oracle_gather(pool, n_pages * P, P, table, n_tab0, H, d, n, k2, v2) == 0);
    CHECK(memcmp(k, k2, el * 2) == 0 && memcmp(v, v2, el * 2) == 0);
    const double scale = 1.0 / sqrt((double)d);
    uint32_t ctx = n, Qs = Q, Hs = H, ds = d;
    uint64_t zero = 0, tlen = n_tab;
    double *out = malloc((uint64_t)Q * d * sizeof *out), *out2 = malloc((uint64_t)Q * d * sizeof *out);
    CHECK(ukv_oracle_attention(pool, n_pages * P, P, 1, &Qs, &Hs, &ds, &scale, &ctx, &zero, &tlen, table, q, &zero, out,
                               &zero, 1) == 0);
    if (n == 0)
        for (uint64_t i = 0; i < (uint64_t)Q * d; ++i) CHECK(out[i] == 0.0);
    if (n >= 2) { /* split anywhere and merged = whole */
        const uint64_t cut = 1 + rnd() % (n - 1);
        double *m = malloc(2 * Q * sizeof *m), *l = malloc(2 * Q * sizeof *l), *acc = malloc(2ull * Q * d * sizeof *acc);
        CHECK(ukv_oracle_attention_range(pool, n_pages * P, P, table, n_tab0, Q, H, d, scale, 0, cut, q, m, l, acc) == 0);
        CHECK(ukv_oracle_attention_range(pool, n_pages * P, P, table, n_tab0, Q, H, d, scale, cut, n, q, m + Q, l + Q,
                                         acc + (uint64_t)Q * d) == 0);
        for (uint32_t a = 0; a < Q; ++a) {
            double mm[2] = {m[a], m[Q + a]}, ll[2] = {l[a], l[Q + a]};
            double *aa = malloc(2ull * d * sizeof *aa);
            memcpy(aa, acc + (uint64_t)a * d, d * sizeof *aa);
            memcpy(aa + d, acc + (uint64_t)Q * d + (uint64_t)a * d, d * sizeof *aa);
            CHECK(ukv_oracle_merge(2, d, mm, ll, aa, out2 + (uint64_t)a * d) == 0);
            for (uint32_t j = 0; j < d; ++j) CHECK(fabs(out2[(uint64_t)a * d + j] - out[(uint64_t)a * d + j]) < 1e-12);
            free(aa);
        }
        free(m), free(l), free(acc);
    }
    if (n >= 1) { /* causal rows: the last row is the decode result, row 0 is token 0's V */
        uint32_t pos[2] = {0, n - 1};
        uint16_t *qr = malloc(2ull * Q * d * 2);
        memcpy(qr, q, (uint64_t)Q * d * 2), memcpy(qr + (uint64_t)Q * d, q, (uint64_t)Q * d * 2);
        double *po = malloc(2ull * Q * d * sizeof *po);
        CHECK(ukv_oracle_prefill(pool, n_pages * P, P, table, n_tab0, Q, H, d, scale, n, 2, pos, qr, po, 1) == 0);
        for (uint64_t i = 0; i < (uint64_t)Q * d; ++i) CHECK(fabs(po[(uint64_t)Q * d + i] - out[i]) < 1e-12);
        free(qr), free(po);
    }
    /* append token n, then a one-token-longer attention */
    ctx = n + 1;
    CHECK(ukv_oracle_append(pool, n_pages * P, P, 1, &Hs, &ds, &ctx, &zero, &tlen, table, nk, nv, &zero) == 0);
    CHECK(ukv_oracle_attention(pool, n_pages * P, P, 1, &Qs, &Hs, &ds, &scale, &ctx, &zero, &tlen, table, q, &zero, out,
                               &zero, 2) == 0);
    if (n == 0) /* one token: its V, exactly */
        for (uint32_t a = 0; a < Q; ++a)
            for (uint32_t j = 0; j < d; ++j) {
                uint32_t u = (uint32_t)nv[(a / (Q / H)) * d + j] << 16;
                float f;
                memcpy(&f, &u, 4);
                CHECK(out[(uint64_t)a * d + j] == (double)f);
            }
    /* errors are reported, not executed: a table that is too short, a page id outside the pool */
    CHECK(ukv_oracle_gather(pool, n_pages * P, P, table, n_tab0 ? n_tab0 - 1 : 0, H, d, n ? n : 1, k2, v2) != 0 || n == 0);
    if (n_tab0) {
        const int32_t keep = table[0];
        table[0] = (int32_t)n_pages;
        CHECK(ukv_oracle_gather(pool, n_pages * P, P, table, n_tab0, H, d, n, k2, v2) != 0);
        table[0] = keep;
    }
    free(pool), free(table), free(k), free(v), free(k2), free(v2), free(q), free(nk), free(nv), free(out), free(out2);
}

int main(void) {
    static const uint32_t shapes[][3] = {{8, 8, 64}, {12, 12, 64}, {32, 32, 128}, {40, 40, 128}, {32, 8, 128}, {64, 8, 128}};
    static const uint32_t pages[] = {1024, 4096, 16384};
    int cases = 0;
    for (int s = 0; s < 6; ++s)
        for (int p = 0; p < 3; ++p)
            for (int r = 0; r < 4; ++r) {
                const uint32_t n = r == 0 ? 0 : r == 1 ? 1 : 2 + (uint32_t)(rnd() % 40);
                one_case(shapes[s][0], shapes[s][1], shapes[s][2], pages[p], n);
                ++cases;
            }
    printf("oracle driver ok: %d cases, %d threads\n", cases, ukv_oracle_threads());
    return 0;
}
