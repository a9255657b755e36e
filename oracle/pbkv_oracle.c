/*
 * pbkv_oracle.c -- TEST INFRASTRUCTURE, not product code.
 *
 * Plain, slow, fp64 CPU statement of what the prefix-reuse prefill path
 * computes.  Only tests, the smoke check and the benchmark's cpu_baseline leg
 * may call it; the GPU library never does and shares no code with it.
 *
 * What is computed (paper Sec. 2, "Radix Tree" / HiCache paragraphs, and the
 * introduction's description of workflow-level cache reuse): an agent request
 * whose prompt prefix is already cached only prefills its uncached suffix.
 * Each suffix token attends to every cached prefix token -- found through a
 * block table of page ids in a paged pool -- and causally to the suffix
 * tokens up to and including itself.  The paper gives no formula for the
 * attention itself; it is standard scaled dot-product attention,
 *     out = softmax(q K^T / sqrt(d)) V,
 * taken over the logical concatenation prefix + suffix[0..i].
 *
 * The definition is written out directly: two passes per output row (scores
 * and their maximum, then weights and the weighted sum), ascending key order,
 * no tiling, no online rescaling, no reordering.  Inputs are the same bits
 * the GPU sees, widened exactly to double.
 *
 * Pins (tests/test_oracle_*.py): contiguous brute force written with numpy
 * matmul that never sees the block table; a hand-derived rational example in
 * tests/golden/; closed forms (equal keys -> mean of V, equal V rows,
 * dominant key, first row of an empty prefix); invariants (physical page
 * permutation, prefix-reuse == from-scratch prefill, weights sum to one,
 * causality, GQA head mapping).  No function here is "parity unpinned".
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

enum { ORACLE_BF16 = 0, ORACLE_F32 = 1 };

/* Sets the number of threads of the row loop (the benchmark times the tiny configuration on one
 * thread); no effect on any result: rows are independent and each is summed by one thread. */
void pbkv_oracle_set_threads(int n)
{
#ifdef _OPENMP
    if (n > 0) omp_set_num_threads(n);
#else
    (void)n;
#endif
}

/* Threads the row loop of pbkv_oracle_prefill runs on (rows are independent). */
int pbkv_oracle_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* bf16 is the upper half of an IEEE binary32: widening is exact. */
static double widen(const void *base, int64_t idx, int dtype)
{
    if (dtype == ORACLE_F32)
        return (double)((const float *)base)[idx];
    uint32_t bits = (uint32_t)((const uint16_t *)base)[idx] << 16;
    float f;
    memcpy(&f, &bits, sizeof f);
    return (double)f;
}

/*
 * Attention of the suffix rows over prefix pages + own suffix.
 *
 * Layouts (row-major, innermost last):
 *   q        [N][Hq][d]        N = sum of new_lens, requests packed in order
 *   k_new    [N][Hkv][d]       v_new likewise
 *   kv_pool  [num_pages][2][Hkv][P][d]   index 0 = K, 1 = V
 *   block_table [B][max_pages] physical page id of each logical page
 *   rows     optional list of packed row indices in [0,N) to evaluate; NULL = all
 *   out      [n_out][Hq][d] doubles, rowsum/lse [n_out][Hq] (either may be NULL)
 * Query head h reads KV head h / (Hq/Hkv).
 * Returns 0, or a negative value for an argument the definition cannot use.
 */
int pbkv_oracle_prefill(int dtype, int B, int Hq, int Hkv, int d, int P,
                        int64_t num_pages, int max_pages,
                        const void *q, const void *k_new, const void *v_new,
                        const void *kv_pool, const int32_t *block_table,
                        const int32_t *prefix_lens, const int32_t *new_lens,
                        const int64_t *rows, int64_t n_rows,
                        double *out, double *rowsum, double *lse)
{
    if (Hkv <= 0 || Hq % Hkv != 0 || d <= 0 || P <= 0) return -2;
    const int G = Hq / Hkv;
    int64_t N = 0, Lmax = 1;
    int64_t *off = (int64_t *)malloc(sizeof(int64_t) * (size_t)(B + 1));
    for (int r = 0; r < B; r++) {
        if (prefix_lens[r] < 0 || new_lens[r] < 0) { free(off); return -4; }
        if ((int64_t)(prefix_lens[r] + P - 1) / P > max_pages) { free(off); return -4; }
        off[r] = N;
        N += new_lens[r];
        if ((int64_t)prefix_lens[r] + new_lens[r] > Lmax) Lmax = (int64_t)prefix_lens[r] + new_lens[r];
    }
    off[B] = N;
    for (int r = 0; r < B; r++)
        for (int j = 0; j < (prefix_lens[r] + P - 1) / P; j++) {
            int32_t pg = block_table[(int64_t)r * max_pages + j];
            if (pg < 0 || pg >= num_pages) { free(off); return -4; }
        }
    const int64_t n_out = rows ? n_rows : N;
    const double scale = 1.0 / sqrt((double)d);
    int bad = 0;

#pragma omp parallel
    {
        double *s = (double *)malloc(sizeof(double) * (size_t)Lmax);
        double *acc = (double *)malloc(sizeof(double) * (size_t)d);
#pragma omp for collapse(2) schedule(dynamic, 1)
        for (int64_t io = 0; io < n_out; io++) {
            for (int h = 0; h < Hq; h++) {
                const int64_t row = rows ? rows[io] : io;
                if (row < 0 || row >= N) {
#pragma omp atomic write
                    bad = 1;
                    continue;
                }
                int r = 0;
                while (!(row >= off[r] && row < off[r + 1])) r++;
                const int64_t i = row - off[r];          /* position inside the suffix */
                const int64_t p = prefix_lens[r];
                const int64_t L = p + i + 1;             /* visible keys: prefix + suffix[0..i] */
                const int g = h / G;
                const int64_t qbase = (row * Hq + h) * d;

                /* pass 1: scaled scores and their maximum */
                double m = -INFINITY;
                for (int64_t t = 0; t < L; t++) {
                    const void *kb; int64_t kidx;
                    if (t < p) {
                        int64_t pg = block_table[(int64_t)r * max_pages + t / P];
                        kb = kv_pool;
                        kidx = (((pg * 2 + 0) * Hkv + g) * P + t % P) * d;
                    } else {
                        kb = k_new;
                        kidx = ((off[r] + (t - p)) * Hkv + g) * d;
                    }
                    double dot = 0.0;
                    for (int c = 0; c < d; c++)
                        dot += widen(q, qbase + c, dtype) * widen(kb, kidx + c, dtype);
                    s[t] = dot * scale;
                    if (s[t] > m) m = s[t];
                }
                /* pass 2: weights, normaliser, weighted sum of values */
                double Z = 0.0;
                for (int c = 0; c < d; c++) acc[c] = 0.0;
                for (int64_t t = 0; t < L; t++) {
                    const void *vb; int64_t vidx;
                    if (t < p) {
                        int64_t pg = block_table[(int64_t)r * max_pages + t / P];
                        vb = kv_pool;
                        vidx = (((pg * 2 + 1) * Hkv + g) * P + t % P) * d;
                    } else {
                        vb = v_new;
                        vidx = ((off[r] + (t - p)) * Hkv + g) * d;
                    }
                    const double w = exp(s[t] - m);
                    s[t] = w;
                    Z += w;
                    for (int c = 0; c < d; c++)
                        acc[c] += w * widen(vb, vidx + c, dtype);
                }
                for (int c = 0; c < d; c++)
                    out[(io * Hq + h) * d + c] = acc[c] / Z;
                if (rowsum) {
                    double sum = 0.0;
                    for (int64_t t = 0; t < L; t++) sum += s[t] / Z;
                    rowsum[io * Hq + h] = sum;
                }
                if (lse) lse[io * Hq + h] = m + log(Z);
            }
        }
        free(s);
        free(acc);
    }
    free(off);
    return bad ? -4 : 0;
}

/*
 * Paged append (the KV an agent produces is kept for downstream agents):
 * suffix token t of request r goes to logical position prefix_lens[r] + t,
 * i.e. page block_table[r][(p+t)/P], slot (p+t)%P, for K and V and every KV
 * head.  Byte move on a caller-owned copy of the pool; elt = bytes per element.
 */
int pbkv_oracle_append(int elt, int B, int Hkv, int d, int P,
                       int64_t num_pages, int max_pages,
                       const void *k_new, const void *v_new, void *kv_pool,
                       const int32_t *block_table,
                       const int32_t *prefix_lens, const int32_t *new_lens)
{
    int64_t off = 0;
    const size_t rowb = (size_t)d * (size_t)elt;
    for (int r = 0; r < B; r++) {
        for (int64_t t = 0; t < new_lens[r]; t++) {
            const int64_t pos = (int64_t)prefix_lens[r] + t;
            if (pos / P >= max_pages) return -4;
            const int64_t pg = block_table[(int64_t)r * max_pages + pos / P];
            if (pg < 0 || pg >= num_pages) return -4;
            for (int kv = 0; kv < 2; kv++)
                for (int g = 0; g < Hkv; g++) {
                    const char *src = (const char *)(kv ? v_new : k_new) +
                                      (size_t)((off + t) * Hkv + g) * rowb;
                    char *dst = (char *)kv_pool +
                                (size_t)((((pg * 2 + kv) * Hkv + g) * P) + pos % P) * rowb;
                    memcpy(dst, src, rowb);
                }
        }
        off += new_lens[r];
    }
    return 0;
}

/*
 * Host -> pool swap-in (a host-tier hit, or a prefetch): the i-th host page
 * becomes pool page page_ids[i].  Whole pages, byte move.
 */
int pbkv_oracle_swap_in(int64_t page_bytes, int64_t num_pages,
                        const void *host_pages, const int32_t *page_ids,
                        int64_t n_pages, void *kv_pool)
{
    for (int64_t i = 0; i < n_pages; i++) {
        if (page_ids[i] < 0 || page_ids[i] >= num_pages) return -4;
        memcpy((char *)kv_pool + (size_t)page_ids[i] * (size_t)page_bytes,
               (const char *)host_pages + (size_t)i * (size_t)page_bytes,
               (size_t)page_bytes);
    }
    return 0;
}

/*
 * Pool -> host page swap-out (Sec. 2, HiCache: cache evicted from the GPU is retained in
 * host memory): host page i becomes a copy of pool page page_ids[i].  Whole pages, byte move;
 * the pool is only read.
 */
int pbkv_oracle_swap_out(int64_t page_bytes, int64_t num_pages,
                         const void *kv_pool, const int32_t *page_ids,
                         int64_t n_pages, void *host_pages)
{
    for (int64_t i = 0; i < n_pages; i++) {
        if (page_ids[i] < 0 || page_ids[i] >= num_pages) return -4;
        memcpy((char *)host_pages + (size_t)i * (size_t)page_bytes,
               (const char *)kv_pool + (size_t)page_ids[i] * (size_t)page_bytes,
               (size_t)page_bytes);
    }
    return 0;
}
