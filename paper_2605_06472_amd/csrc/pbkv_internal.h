// Internal declarations shared by the host API and the kernel translation units.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace pbkv {

// Sets the thread's last-error text (returned by pbkv_last_error) and hands back `code`.
int set_error(int code, const char *fmt, ...) __attribute__((format(printf, 2, 3)));
void clear_error();

// One unit of attention work: a block of consecutive suffix tokens of one request.
// Written by the host into pinned memory and read by the kernel through the mapped
// pointer (32 bytes, two 16-byte loads).
struct TileDesc {
    int32_t req;         // request index inside this call (row of block_table)
    int32_t tok0;        // first suffix token of the tile
    int32_t prefix_len;  // p_r
    int32_t new_len;     // n_r
    int64_t row0;        // packed row (into q / k_new / v_new / out) of the request's token 0
    int64_t pad;         // index of the tile in request order (before the longest-first sort)
};
static_assert(sizeof(TileDesc) == 32, "TileDesc is read as two 16-byte words");

// A run of consecutive suffix tokens of one request that land in one pool page.
struct AppendDesc {
    int64_t src_row;     // packed row of the first token of the run
    int32_t req;         // request index (row of block_table)
    int32_t logical_page;
    int32_t slot0;       // first slot inside the page
    int32_t count;       // tokens in the run (1..page_size)
    int64_t pad;
};
static_assert(sizeof(AppendDesc) == 32, "AppendDesc is read as two 16-byte words");

struct AttnParams {
    const void *q, *k_new, *v_new, *kv_pool;
    void *out;
    const int32_t *block_table;
    const TileDesc *tiles;
    int32_t n_tiles, Hq, Hkv, max_pages, num_pages;
    int32_t waves;   // bf16 kernel: waves per work-group (attn_bf16_waves); the tiles were cut for it
    TileDesc *mirror;   // device memory that receives a copy of the tiles the launch read, or null
};

// Decode: one slice of a request's context pages, shared by its KV heads and head groups.
struct DecodeUnit {
    int32_t req;         // request index (row of q / out / block_table)
    int32_t ctx_len;     // tokens the request's row attends to
    int32_t page0, page1;  // logical pages [page0, page1) of this slice
    int32_t split;       // running index of the slice over the whole call (addresses the scratch)
    int32_t pad[3];
};
static_assert(sizeof(DecodeUnit) == 32, "DecodeUnit is read as two 16-byte words");

struct DecodeReq {
    int32_t split0, n_splits;   // the request's slices are split0 .. split0 + n_splits - 1
    int32_t pad[2];
};
static_assert(sizeof(DecodeReq) == 16, "DecodeReq is read as one 16-byte word");

struct DecodeParams {
    const void *q, *kv_pool;
    void *out;
    const int32_t *block_table;
    const DecodeUnit *units;
    const DecodeReq *reqs;
    DecodeUnit *mirror_units;   // device memory that receives a copy of units / reqs, or null
    DecodeReq *mirror_reqs;
    float *scratch;
    int32_t n_units, n_reqs, Hq, Hkv, max_pages, num_pages;
};

struct AppendParams {
    const void *k_new, *v_new;
    void *kv_pool;
    const int32_t *block_table;
    const AppendDesc *descs;
    AppendDesc *mirror;         // device memory that receives a copy of descs, or null
    int32_t n_descs, Hkv, max_pages, num_pages;
};

// Waves per work-group the bf16 kernel runs this batch with, and the tokens per attention tile
// that follow from it (what the host cuts the suffix into).
int attn_bf16_waves(const int32_t *prefix_lens, const int32_t *new_lens, int batch);
void attn_bf16_force_waves(int waves);   // 4 or 8: every later launch uses that shape; anything else: automatic
int attn_bf16_forced_waves();
int attn_bf16_tile_tokens(int head_dim, int group, int waves);
int attn_f32_tile_tokens();

// Launchers: all arguments already validated.  Return the hipError of the launch.
hipError_t launch_attn_bf16(const AttnParams &p, int head_dim, hipStream_t s);
hipError_t launch_attn_f32(const AttnParams &p, int head_dim, hipStream_t s);
// Gather diagnostic: p.out is a uint32 array with one word per work unit, units ordered
// (tile in request order, query-head split, KV head); attn_bf16_units_per_tile gives the
// number of units of one tile.
hipError_t launch_gather_probe(const AttnParams &p, int head_dim, hipStream_t s);
int attn_bf16_units_per_tile(int num_kv_heads, int group);
hipError_t launch_append(const AppendParams &p, int head_dim, int elt_bytes, hipStream_t s);
hipError_t launch_swap_in(const void *host_pages, const int32_t *page_ids_dev, int32_t n_pages,
                          void *kv_pool, int64_t page_bytes, hipStream_t s);

// Paged decode attention (bf16): main kernel + merge of the partials in p.scratch.
hipError_t launch_decode_bf16(const DecodeParams &p, int head_dim, hipStream_t s);
int decode_heads_per_group(int group);
int64_t decode_partial_floats(int head_dim, int group);   // floats one work-group's partial occupies

hipError_t launch_swap_out(const void *kv_pool, const int32_t *page_ids_dev, int32_t n_pages,
                           void *host_pages, int64_t page_bytes, hipStream_t s);

}  // namespace pbkv
