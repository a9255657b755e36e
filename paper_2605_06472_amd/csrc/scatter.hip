// Page-granular byte movers: paged KV append and host->pool page swap-in.
// Both are pure copies (bit-exact) bound by memory bandwidth: HBM for the append,
// the host link for the swap-in.  Every access is a 16-byte vector access and every
// (token, K|V, head) row or page is a run of whole 128-byte lines on both sides.
#include "pbkv_internal.h"

namespace pbkv {

static __device__ __forceinline__ int clamp_page(int pg, int num_pages) {
    return pg < 0 ? 0 : (pg >= num_pages ? num_pages - 1 : pg);
}

// Append: the runs (AppendDesc: up to 16 consecutive suffix tokens of one request that fall in one
// pool page) are cut into parts of APPEND_CHUNKS 16-byte chunks, and a grid sized to the chip strides
// over (run, part).  Chunk index order = source order (token, K|V, head, 16B chunk), so a wave reads
// contiguous memory and writes whole rows; every thread has four independent loads in flight before
// its first store.
constexpr int APPEND_CHUNKS = 1024;   // 16 KiB per work-group and pass
constexpr int APPEND_MAX_WGS = 2048;  // 8 work-groups of 4 waves per CU
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;

__global__ __launch_bounds__(256) void append_kernel(AppendParams p, int row_chunks, int page_size, int parts_per_run) {
    const int per_tok = 2 * p.Hkv * row_chunks;               // 16-byte chunks per token (K and V)
    const int64_t page_chunks = (int64_t)per_tok * page_size;
    const u32x4 *ksrc = (const u32x4 *)p.k_new;
    const u32x4 *vsrc = (const u32x4 *)p.v_new;
    for (int64_t item = blockIdx.x; item < (int64_t)p.n_descs * parts_per_run; item += gridDim.x) {
        const int run = (int)(item / parts_per_run), part = (int)(item % parts_per_run);
        const AppendDesc d = p.descs[run];
        if (p.mirror != nullptr && part == 0 && threadIdx.x == 0) p.mirror[run] = d;
        const int total = d.count * per_tok;
        if (part * APPEND_CHUNKS >= total) continue;
        const int pg = clamp_page(p.block_table[(int64_t)d.req * p.max_pages + d.logical_page], p.num_pages);
        u32x4 *pool = (u32x4 *)p.kv_pool + (int64_t)pg * page_chunks;
        u32x4 v[4];
        int64_t dst[4];
#pragma unroll
        for (int i = 0; i < 4; i++) {
            const int idx = part * APPEND_CHUNKS + i * 256 + threadIdx.x;
            dst[i] = -1;
            if (idx < total) {
                const int c = idx % row_chunks;
                const int g = (idx / row_chunks) % p.Hkv;
                const int kv = (idx / (row_chunks * p.Hkv)) & 1;
                const int t = idx / per_tok;
                const int64_t s = ((d.src_row + t) * p.Hkv + g) * row_chunks + c;
                v[i] = __builtin_nontemporal_load((kv ? vsrc : ksrc) + s);
                dst[i] = ((int64_t)(kv * p.Hkv + g) * page_size + d.slot0 + t) * row_chunks + c;
            }
        }
#pragma unroll
        for (int i = 0; i < 4; i++)
            if (dst[i] >= 0) pool[dst[i]] = v[i];
    }
}

hipError_t launch_append(const AppendParams &p, int head_dim, int elt_bytes, hipStream_t s) {
    if (p.n_descs == 0) return hipSuccess;
    const int row_chunks = head_dim * elt_bytes / 16;
    const int parts = (16 * 2 * p.Hkv * row_chunks + APPEND_CHUNKS - 1) / APPEND_CHUNKS;
    const int64_t items = (int64_t)p.n_descs * parts;
    hipLaunchKernelGGL(append_kernel, dim3((unsigned)(items < APPEND_MAX_WGS ? items : APPEND_MAX_WGS)), dim3(256), 0, s,
                       p, row_chunks, 16, parts);
    return hipGetLastError();
}

// Swap-in: a work-group moves SWAP_CHUNKS 16-byte chunks of one page at a time from pinned host
// memory (read over the host link through the mapped pointer) into the page's pool slot.
// Four independent loads per thread are in flight before the first store.  The grid is small
// and persistent (SWAP_MAX_WGS work-groups stride over the page parts): 512 KiB in flight
// saturates the link, and a transfer that runs beside attention or decode (Sec. 4.3: prefetch
// hidden behind compute) must not park thousands of waves, each waiting microseconds on the
// link, on the CUs and memory queues the compute kernel needs.
constexpr int SWAP_CHUNKS = 1024;   // 16 KiB per work-group and pass
constexpr int SWAP_MAX_WGS = 32;

__global__ __launch_bounds__(256) void swap_in_kernel(const u32x4 *__restrict__ host_pages,
                                                      const int32_t *__restrict__ page_ids,
                                                      u32x4 *__restrict__ pool, int page_chunks,
                                                      int wgs_per_page, int n_pages) {
    for (int64_t item = blockIdx.x; item < (int64_t)n_pages * wgs_per_page; item += gridDim.x) {
        const int page = (int)(item / wgs_per_page);
        const int part = (int)(item % wgs_per_page);
        const int64_t dst_page = page_ids[page];
        const u32x4 *src = host_pages + (int64_t)page * page_chunks;
        u32x4 *dst = pool + dst_page * page_chunks;
        const int base = part * SWAP_CHUNKS + threadIdx.x;
        u32x4 v[4];
#pragma unroll
        for (int i = 0; i < 4; i++) {
            const int c = base + i * 256;
            if (c < page_chunks) v[i] = __builtin_nontemporal_load(src + c);
        }
#pragma unroll
        for (int i = 0; i < 4; i++) {
            const int c = base + i * 256;
            if (c < page_chunks) dst[c] = v[i];
        }
    }
}

hipError_t launch_swap_in(const void *host_pages, const int32_t *page_ids_dev, int32_t n_pages,
                          void *kv_pool, int64_t page_bytes, hipStream_t s) {
    if (n_pages == 0) return hipSuccess;
    const int page_chunks = (int)(page_bytes / 16);
    const int wgs_per_page = (page_chunks + SWAP_CHUNKS - 1) / SWAP_CHUNKS;
    const int64_t items = (int64_t)n_pages * wgs_per_page;
    hipLaunchKernelGGL(swap_in_kernel, dim3((unsigned)(items < SWAP_MAX_WGS ? items : SWAP_MAX_WGS)), dim3(256), 0, s,
                       (const u32x4 *)host_pages, page_ids_dev, (u32x4 *)kv_pool, page_chunks,
                       wgs_per_page, n_pages);
    return hipGetLastError();
}

// Swap-out: the mirror image -- pool page page_ids[i] is copied to host page i, read from HBM
// and written over the host link through the mapped pointer (posted writes, so the link is
// kept full without many loads in flight).
__global__ __launch_bounds__(256) void swap_out_kernel(const u32x4 *__restrict__ pool,
                                                       const int32_t *__restrict__ page_ids,
                                                       u32x4 *__restrict__ host_pages, int page_chunks,
                                                       int wgs_per_page, int n_pages) {
    for (int64_t item = blockIdx.x; item < (int64_t)n_pages * wgs_per_page; item += gridDim.x) {
        const int page = (int)(item / wgs_per_page);
        const int part = (int)(item % wgs_per_page);
        const int64_t src_page = page_ids[page];
        const u32x4 *src = pool + src_page * page_chunks;
        u32x4 *dst = host_pages + (int64_t)page * page_chunks;
        const int base = part * SWAP_CHUNKS + threadIdx.x;
        u32x4 v[4];
#pragma unroll
        for (int i = 0; i < 4; i++) {
            const int c = base + i * 256;
            if (c < page_chunks) v[i] = src[c];
        }
#pragma unroll
        for (int i = 0; i < 4; i++) {
            const int c = base + i * 256;
            if (c < page_chunks) __builtin_nontemporal_store(v[i], dst + c);
        }
    }
}

hipError_t launch_swap_out(const void *kv_pool, const int32_t *page_ids_dev, int32_t n_pages,
                           void *host_pages, int64_t page_bytes, hipStream_t s) {
    if (n_pages == 0) return hipSuccess;
    const int page_chunks = (int)(page_bytes / 16);
    const int wgs_per_page = (page_chunks + SWAP_CHUNKS - 1) / SWAP_CHUNKS;
    const int64_t items = (int64_t)n_pages * wgs_per_page;
    hipLaunchKernelGGL(swap_out_kernel, dim3((unsigned)(items < SWAP_MAX_WGS ? items : SWAP_MAX_WGS)), dim3(256), 0, s,
                       (const u32x4 *)kv_pool, page_ids_dev, (u32x4 *)host_pages, page_chunks,
                       wgs_per_page, n_pages);
    return hipGetLastError();
}

}  // namespace pbkv
