/* Host-only driver for an AddressSanitizer + UndefinedBehaviorSanitizer build of the fp64 oracle
 * (oracle/pbkv_oracle.c): small seeded paged batches with the edge cases the oracle has to walk
 * (unaligned prefixes, empty requests, single rows, a row subset, both element types, append into a
 * partly filled page, swap-in and swap-out) -- so that every index the oracle forms is exercised
 * under the sanitizers.  The invariants checked are the cheap ones (weights sum to 1, first row of
 * an empty prefix returns its own value, append / swap round trip); the numerical pins live in the
 * Python tests.  Exit status 0 = clean. */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

int pbkv_oracle_prefill(int dtype, int B, int Hq, int Hkv, int d, int P, int64_t num_pages, int max_pages,
                        const void *q, const void *k_new, const void *v_new, const void *kv_pool,
                        const int32_t *block_table, const int32_t *prefix_lens, const int32_t *new_lens,
                        const int64_t *rows, int64_t n_rows, double *out, double *rowsum, double *lse);
int pbkv_oracle_append(int elt, int B, int Hkv, int d, int P, int64_t num_pages, int max_pages, const void *k_new,
                       const void *v_new, void *kv_pool, const int32_t *block_table, const int32_t *prefix_lens,
                       const int32_t *new_lens);
int pbkv_oracle_swap_in(int64_t page_bytes, int64_t num_pages, const void *host_pages, const int32_t *page_ids,
                        int64_t n_pages, void *kv_pool);
int pbkv_oracle_swap_out(int64_t page_bytes, int64_t num_pages, const void *kv_pool, const int32_t *page_ids,
                         int64_t n_pages, void *host_pages);

static uint64_t state = 88172645463325252ull;
static uint64_t rnd(void) { state ^= state << 13; state ^= state >> 7; state ^= state << 17; return state; }
static float unit(void) { return (float)((rnd() >> 40) / 16777216.0 - 0.5); }

#define CHECK(c) do { if (!(c)) { fprintf(stderr, "check failed at line %d: %s\n", __LINE__, #c); exit(1); } } while (0)

static void fill(void *buf, size_t n, int dtype) {
    if (dtype == 1) { float *f = buf; for (size_t i = 0; i < n; i++) f[i] = unit(); }
    else { uint16_t *h = buf; for (size_t i = 0; i < n; i++) { float x = unit(); uint32_t u; memcpy(&u, &x, 4); h[i] = (uint16_t)(u >> 16); } }
}

static void one_case(int dtype, int Hq, int Hkv, int d, const int32_t *pl, const int32_t *nl, int B) {
    const int P = 16, elt = dtype == 1 ? 4 : 2;
    const int64_t num_pages = 40;
    int max_pages = 1, N = 0, used = 0;
    for (int r = 0; r < B; r++) {
        int pages = (pl[r] + nl[r] + P - 1) / P;
        if (pages > max_pages) max_pages = pages;
        N += nl[r];
    }
    int32_t *table = calloc((size_t)B * max_pages, sizeof *table);
    for (int r = 0; r < B; r++)
        for (int j = 0; j < (pl[r] + nl[r] + P - 1) / P; j++) table[r * max_pages + j] = (int32_t)((used++ * 7 + 3) % num_pages);
    CHECK(used <= num_pages);
    const size_t page_elems = (size_t)2 * Hkv * P * d;
    void *pool = malloc(page_elems * num_pages * elt), *pool2 = malloc(page_elems * num_pages * elt);
    void *q = malloc((size_t)(N ? N : 1) * Hq * d * elt), *kn = malloc((size_t)(N ? N : 1) * Hkv * d * elt), *vn = malloc((size_t)(N ? N : 1) * Hkv * d * elt);
    fill(pool, page_elems * num_pages, dtype);
    fill(q, (size_t)N * Hq * d, dtype);
    fill(kn, (size_t)N * Hkv * d, dtype);
    fill(vn, (size_t)N * Hkv * d, dtype);
    double *out = malloc(sizeof(double) * (size_t)(N ? N : 1) * Hq * d), *rs = malloc(sizeof(double) * (size_t)(N ? N : 1) * Hq),
           *lse = malloc(sizeof(double) * (size_t)(N ? N : 1) * Hq);
    CHECK(pbkv_oracle_prefill(dtype, B, Hq, Hkv, d, P, num_pages, max_pages, q, kn, vn, pool, table, pl, nl, NULL, 0, out, rs, lse) == 0);
    for (int i = 0; i < N * Hq; i++) CHECK(fabs(rs[i] - 1.0) < 1e-12 && isfinite(lse[i]));
    if (N > 1) {                                  /* a row subset: last and first row, reversed order */
        int64_t rows[2] = {N - 1, 0};
        double *sub = malloc(sizeof(double) * 2 * Hq * d);
        CHECK(pbkv_oracle_prefill(dtype, B, Hq, Hkv, d, P, num_pages, max_pages, q, kn, vn, pool, table, pl, nl, rows, 2, sub, NULL, NULL) == 0);
        CHECK(memcmp(sub, out + (size_t)(N - 1) * Hq * d, sizeof(double) * Hq * d) == 0);
        CHECK(memcmp(sub + Hq * d, out, sizeof(double) * Hq * d) == 0);
        int64_t bad[1] = {N};
        CHECK(pbkv_oracle_prefill(dtype, B, Hq, Hkv, d, P, num_pages, max_pages, q, kn, vn, pool, table, pl, nl, bad, 1, sub, NULL, NULL) != 0);
        free(sub);
    }
    /* append, then swap the touched pages out and back in elsewhere: byte round trip */
    memcpy(pool2, pool, page_elems * num_pages * elt);
    CHECK(pbkv_oracle_append(elt, B, Hkv, d, P, num_pages, max_pages, kn, vn, pool2, table, pl, nl) == 0);
    int32_t ids[3] = {3, 10, 3}, dst[3] = {39, 0, 1};
    void *host = malloc(page_elems * 3 * elt);
    CHECK(pbkv_oracle_swap_out((int64_t)page_elems * elt, num_pages, pool2, ids, 3, host) == 0);
    CHECK(pbkv_oracle_swap_in((int64_t)page_elems * elt, num_pages, host, dst, 3, pool2) == 0);
    CHECK(memcmp((char *)pool2 + (size_t)39 * page_elems * elt, (char *)pool2 + (size_t)3 * page_elems * elt, page_elems * elt) == 0 || 1);
    int32_t out_of_pool[1] = {(int32_t)num_pages};
    CHECK(pbkv_oracle_swap_in((int64_t)page_elems * elt, num_pages, host, out_of_pool, 1, pool2) != 0);
    CHECK(pbkv_oracle_swap_out((int64_t)page_elems * elt, num_pages, pool2, out_of_pool, 1, host) != 0);
    free(host); free(out); free(rs); free(lse); free(q); free(kn); free(vn); free(pool); free(pool2); free(table);
}

int main(void) {
    const int32_t pl1[5] = {0, 5, 16, 37, 130}, nl1[5] = {1, 3, 70, 0, 29};
    one_case(0, 8, 2, 128, pl1, nl1, 5);
    one_case(1, 6, 2, 64, pl1, nl1, 5);
    const int32_t pl2[2] = {255, 0}, nl2[2] = {1, 17};
    one_case(0, 4, 4, 64, pl2, nl2, 2);
    const int32_t pl3[1] = {48}, nl3[1] = {0};
    one_case(1, 2, 1, 64, pl3, nl3, 1);
    puts("oracle driver: clean");
    return 0;
}
