/*
 * pbkv.h -- C boundary of the MI355X prefix-reuse prefill library (libpbkv.so).
 *
 * The operations are the GPU-side work that the paper's cache policy exists to
 * make cheap (Sec. 1 and Sec. 2 of arxiv 2605.06472, "PBKV"): a request whose
 * prompt prefix is cached in the radix tree prefills only its uncached suffix
 * against the cached KV pages; the KV it produces is kept for downstream
 * agents; pages evicted to the host tier are swapped back on a hit or loaded
 * ahead of time by the prefetcher (Sec. 4.3).
 *
 * Conventions common to all calls
 *   - Plain pointers and sizes only.  "device" = memory of the current HIP
 *     device; "host" = ordinary host memory read during the call; "pinned" =
 *     page-locked host memory (hipHostMalloc, or a pinned torch tensor) that
 *     the GPU reads while the stream runs.
 *   - The caller owns every buffer and the stream.  The library keeps no
 *     caller pointer after the call returns.  Per device it owns a ring of
 *     pinned descriptor memory (8 MiB) and, per stream it has seen (up to 8; a
 *     ninth replaces the one used longest ago, after draining the device), 2 MiB
 *     of device memory holding the work lists of recent calls, so that a call
 *     that repeats the shape and lengths of an earlier call on that stream (the
 *     next layer of the same batch) builds and uploads nothing.  All of it is
 *     created on first use and released at process exit.
 *   - `stream` is a hipStream_t passed as void*; NULL is the default stream.
 *     Calls validate on the host, enqueue on `stream`, and return without
 *     waiting.  Buffers must stay valid until the stream has run the work.
 *     A stream that is being captured into a graph is refused
 *     (PBKV_ERR_DEVICE): the work lists live in library memory that later
 *     calls reuse, so a replay would read lists that are gone.
 *   - Device pointers are checked for their kind (device / pinned) the first
 *     time the calling thread passes an address; later calls trust it.
 *   - Return value: PBKV_OK or a negative pbkv_status.  On an argument error
 *     nothing is enqueued.  pbkv_last_error() gives a thread-local message.
 *   - Layouts are row-major, innermost dimension last:
 *       q, out        [N][num_q_heads][head_dim]   N = sum(new_lens), requests
 *                                                  packed in batch order
 *       k_new, v_new  [N][num_kv_heads][head_dim]
 *       kv_pool       [num_pages][2][num_kv_heads][page_size][head_dim]
 *                     (index 0 = K, 1 = V): one page is one contiguous block
 *                     of pbkv_page_bytes() bytes
 *       block_table   [batch][max_pages_per_req] int32: physical page of each
 *                     logical page of the request (prefix pages first, then
 *                     the pages the suffix is appended to)
 *   - Supported shapes: page_size 16; head_dim 64 or 128; num_q_heads a
 *     multiple of num_kv_heads with ratio 1, 2, 4, 8 or 16 for PBKV_BF16 and
 *     any ratio for PBKV_F32.  Anything else returns PBKV_ERR_SHAPE; there is
 *     no slow fallback.
 */
#ifndef PBKV_H
#define PBKV_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    PBKV_OK = 0,
    PBKV_ERR_NULL = -1,    /* a required pointer is NULL                          */
    PBKV_ERR_SHAPE = -2,   /* unsupported or inconsistent shape                   */
    PBKV_ERR_DTYPE = -3,   /* unknown dtype                                       */
    PBKV_ERR_RANGE = -4,   /* a length or page id does not fit the table / pool   */
    PBKV_ERR_ALIAS = -5,   /* duplicate destination pages in a swap-in            */
    PBKV_ERR_DEVICE = -6,  /* HIP runtime error, or a pointer of the wrong kind   */
    PBKV_ERR_LIMIT = -7    /* the call needs more descriptor space than the library
                              can provide at once, or the pool is 1 TiB or more   */
} pbkv_status;

typedef enum { PBKV_BF16 = 0, PBKV_F32 = 1 } pbkv_dtype;

typedef struct {
    int32_t batch;              /* B: requests in this call (0 is a valid no-op)   */
    int32_t num_q_heads;        /* H_q                                             */
    int32_t num_kv_heads;       /* H_kv                                            */
    int32_t head_dim;           /* d                                               */
    int32_t page_size;          /* P: tokens per page (16)                         */
    int32_t num_pages;          /* pages in kv_pool                                */
    int32_t max_pages_per_req;  /* row length of block_table                       */
    int32_t dtype;              /* pbkv_dtype of q, k_new, v_new, kv_pool, out     */
} pbkv_shape;

/* Bytes of one pool page for this shape (2 * H_kv * P * d * element size); 0 if the
 * shape is unsupported. */
int64_t pbkv_page_bytes(const pbkv_shape *shape);

/*
 * Prefix-reuse prefill attention (Sec. 1: a cache hit turns prefill of the shared
 * context into a lookup; Sec. 2: radix-tree prefix sharing).  For request r with
 * cached prefix length p = prefix_lens[r] and n = new_lens[r] new tokens, suffix row
 * i and query head h:
 *     out = sum_t softmax_t(q . k_t / sqrt(d)) v_t
 * over t in [0, p) read from kv_pool through block_table[r] with KV head
 * h / (H_q / H_kv), followed by the request's own suffix tokens 0..i read from
 * k_new / v_new (causal, diagonal included).  The suffix is NOT read from the pool,
 * so pbkv_append_kv may run concurrently on another stream.
 *
 *   q, k_new, v_new, kv_pool, block_table : device, read only
 *   prefix_lens, new_lens                 : host int32 [batch], read during the call
 *   out                                   : device, written; rows of other calls untouched
 * bf16: fp32 accumulation, probabilities rounded to bf16 before the PV product, one
 * final rounding to bf16.  f32: fp32 throughout.
 * Page ids read from block_table are clamped to [0, num_pages) on the device, so a
 * corrupt table gives wrong numbers, never an out-of-bounds access.
 * Errors: NULL pointers, unsupported shape, negative lengths, or
 * ceil((p + n) / P) > max_pages_per_req  ->  negative status, nothing enqueued.
 */
int pbkv_prefix_prefill(const pbkv_shape *shape, const void *q, const void *k_new,
                        const void *v_new, const void *kv_pool, const int32_t *block_table,
                        const int32_t *prefix_lens, const int32_t *new_lens, void *out,
                        void *stream);

/*
 * Paged KV append (Sec. 1: the KV-Cache an agent produces is retained for downstream
 * agents).  Suffix token t of request r is copied, for K and V and every KV head, to
 * page block_table[r][(p + t) / P], slot (p + t) % P.  Byte-exact copy; no other pool
 * byte is written.
 *   k_new, v_new, block_table : device, read only;  kv_pool : device, written
 *   prefix_lens, new_lens     : host int32 [batch]
 * Requests must not share a destination slot (their suffix pages are private).
 */
int pbkv_append_kv(const pbkv_shape *shape, const void *k_new, const void *v_new,
                   void *kv_pool, const int32_t *block_table, const int32_t *prefix_lens,
                   const int32_t *new_lens, void *stream);

/*
 * Host -> pool page swap-in (Sec. 2: HiCache keeps evicted cache in host memory and
 * swaps it back on a hit; Sec. 4.3: the prefetcher loads host nodes into free or
 * retired GPU space ahead of the hit).  Pool page page_ids[i] := host page i, whole
 * pages, byte-exact.
 *   host_pages : pinned host memory, [n_pages][pbkv_page_bytes], read by the GPU while
 *                the stream runs (must stay valid and unmodified until then)
 *   page_ids   : host int32 [n_pages], read during the call; each in [0, num_pages),
 *                all distinct (else PBKV_ERR_RANGE / PBKV_ERR_ALIAS, nothing enqueued)
 *   kv_pool    : device, written
 * Only shape->num_kv_heads, head_dim, page_size, num_pages and dtype are used.
 */
int pbkv_swap_in_pages(const pbkv_shape *shape, const void *host_pages,
                       const int32_t *page_ids, int32_t n_pages, void *kv_pool,
                       void *stream);

/*
 * Paged decode attention (Sec. 4.3: prefetch transfers are hidden behind pure-decode steps, so
 * the decode step is what the transfer budget Bandwidth * StepDuration is measured against).
 * One query row per request: for request r and query head h,
 *     out[r][h] = sum_t softmax_t(q[r][h] . k_t / sqrt(d)) v_t   over t in [0, context_lens[r])
 * with k_t, v_t read from kv_pool through block_table[r] (KV head h / (H_q / H_kv)); the row's own
 * token is expected to be in the pool already (append first).  context_lens[r] == 0 gives a zero row.
 *   q, out      : device, [batch][H_q][d], bf16 (other dtypes: PBKV_ERR_DTYPE)
 *   kv_pool, block_table : device, read only;   context_lens : host int32 [batch]
 * fp32 accumulation, probabilities kept in fp32, one final rounding to bf16.  The library keeps,
 * per stream, a device scratch buffer for the partial results of context slices (8 MiB on first
 * use; a call that needs more drains that stream and re-allocates); calls on different streams
 * use different buffers and may overlap.
 * Errors: NULL pointers, unsupported shape, negative lengths, ceil(len / P) > max_pages_per_req.
 */
int pbkv_paged_decode(const pbkv_shape *shape, const void *q, const void *kv_pool,
                      const int32_t *block_table, const int32_t *context_lens, void *out,
                      void *stream);

/*
 * pbkv_paged_decode for callers that cannot allocate device memory: code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same result bit for bit
 * (the same kernels and the same slicing of the contexts), but the partial results of the context
 * slices and the work lists live in one device array that is part of the library's image (8 MiB +
 * 192 KiB per GPU, held until the process ends) and the lists reach it through kernel arguments:
 * the call allocates nothing, records no event and copies nothing, so it may also be captured.
 * Limits: at most 4096 requests, 4096 context slices (about 2048 / (work-groups per slice) plus one
 * per request) and 8 MiB of partial results (520 floats per slice, KV head and group of eight query
 * heads at d = 128 and a head ratio of 4); beyond them PBKV_ERR_LIMIT and nothing is enqueued.
 * Every call on a GPU uses that GPU's one array: calls that overlap on one GPU (two streams, two
 * threads) race and give wrong results; nothing in it has to be cleared between calls.
 */
int pbkv_paged_decode_static(const pbkv_shape *shape, const void *q, const void *kv_pool,
                             const int32_t *block_table, const int32_t *context_lens, void *out,
                             void *stream);

/*
 * Pool -> host page swap-out (Sec. 2: with HiCache, cache evicted from the GPU is retained
 * in host memory), the mirror of pbkv_swap_in_pages: host page i := pool page
 * page_ids[i], whole pages, byte-exact; the pool is not modified.
 *   kv_pool    : device, read only
 *   page_ids   : host int32 [n_pages], read during the call; each in [0, num_pages)
 *                (else PBKV_ERR_RANGE, nothing enqueued); a page may be named more than once
 *   host_pages : pinned host memory, [n_pages][pbkv_page_bytes], written by the GPU while the
 *                stream runs; its content is defined once the stream has reached this call
 * Only shape->num_kv_heads, head_dim, page_size, num_pages and dtype are used.
 */
int pbkv_swap_out_pages(const pbkv_shape *shape, const void *kv_pool, const int32_t *page_ids,
                        int32_t n_pages, void *host_pages, void *stream);

/*
 * Gather diagnostic (measurement aid, not a step of the method): runs the page gather of
 * pbkv_prefix_prefill on bf16 inputs -- the same work units, the same walk through
 * block_table, the same loads of K/V rows into on-chip memory -- without the arithmetic,
 * and XORs the 32-bit words of every K and V row a unit stages.  A unit is (block of
 * *unit_tokens suffix tokens of one request, group of <= 4 query heads of one KV head, KV
 * head); units are numbered in that nesting order, requests and token blocks ascending.
 * Unit u covering suffix tokens [t0, t1) of request r and KV head g stages K and V of
 * prefix tokens [0, p_r) and suffix tokens [0, t1) of head g; unit_xor[u] is the XOR of
 * all their words.
 *   k_new, v_new, kv_pool, block_table : device, read only
 *   prefix_lens, new_lens              : host int32 [batch]
 *   unit_xor                           : device uint32 [unit_capacity], first *n_units written
 *   n_units, unit_tokens               : host, written (also when unit_xor is too small:
 *                                        PBKV_ERR_RANGE, nothing enqueued)
 * unit_xor == NULL with unit_capacity == 0 only asks for *n_units and *unit_tokens.
 */
int pbkv_gather_probe(const pbkv_shape *shape, const void *k_new, const void *v_new,
                      const void *kv_pool, const int32_t *block_table,
                      const int32_t *prefix_lens, const int32_t *new_lens, uint32_t *unit_xor,
                      int64_t unit_capacity, int64_t *n_units, int32_t *unit_tokens, void *stream);

/*
 * Work-group shape of the bf16 attention kernel, for tests and tuning: 4 or 8 makes every later
 * pbkv_prefix_prefill / pbkv_gather_probe launch of this process use work-groups of that many
 * waves of 32 query rows (32 or 64 suffix tokens per unit at a query/KV head ratio of 4), 64 the
 * form with four waves of 64 query rows (64 suffix tokens per unit at that ratio; the gather probe
 * then runs as for 8, which stages the same tiles), 0 returns to the library's own choice per
 * launch (4 or 64).  Results do not depend on it bit for bit.  Any other value: PBKV_ERR_SHAPE.
 */
int pbkv_set_attn_waves(int waves);

/* Thread-local, library-owned description of the last error on this thread ("" if none). */
const char *pbkv_last_error(void);

/* Library version string, e.g. "pbkv 0.1 gfx950". */
const char *pbkv_version(void);

#ifdef __cplusplus
}
#endif
#endif /* PBKV_H */
