// Host side of libpbkv: argument validation, work-list construction and launches behind
// the C boundary declared in include/pbkv.h.  No attention, append or swap-in arithmetic
// happens on the host: the host only cuts the batch into tiles / page runs and enqueues
// the kernels.
#include "../../include/pbkv.h"
#include "pbkv_internal.h"

#include <algorithm>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <deque>
#include <mutex>
#include <string>
#include <vector>

namespace {

thread_local char g_err[512] = "";

int fail(int code, const char *fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof g_err, fmt, ap);
    va_end(ap);
    return code;
}

}  // namespace

// error text for the translation units that hold no HIP code (the policy core)
int pbkv::set_error(int code, const char *fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof g_err, fmt, ap);
    va_end(ap);
    return code;
}
void pbkv::clear_error() { g_err[0] = 0; }

namespace {

int fail_hip(hipError_t e, const char *what) {
    return fail(PBKV_ERR_DEVICE, "%s: %s", what, hipGetErrorString(e));
}

int elt_bytes(int dtype) { return dtype == PBKV_BF16 ? 2 : 4; }

// Shape checks that need no device.  `need_heads` = the call uses the query-head count.
int check_shape(const pbkv_shape *s, bool need_heads) {
    if (!s) return fail(PBKV_ERR_NULL, "shape is NULL");
    if (s->dtype != PBKV_BF16 && s->dtype != PBKV_F32) return fail(PBKV_ERR_DTYPE, "unknown dtype %d", s->dtype);
    if (s->page_size != 16) return fail(PBKV_ERR_SHAPE, "page_size %d unsupported (16)", s->page_size);
    if (s->head_dim != 64 && s->head_dim != 128)
        return fail(PBKV_ERR_SHAPE, "head_dim %d unsupported (64, 128)", s->head_dim);
    if (s->num_kv_heads <= 0) return fail(PBKV_ERR_SHAPE, "num_kv_heads %d", s->num_kv_heads);
    if (s->num_pages <= 0) return fail(PBKV_ERR_SHAPE, "num_pages %d", s->num_pages);
    // the attention kernel addresses pool pages by 32-bit offsets in units of 256 bytes
    if ((int64_t)s->num_pages * 2 * s->num_kv_heads * s->page_size * s->head_dim * elt_bytes(s->dtype) >= ((int64_t)1 << 40))
        return fail(PBKV_ERR_LIMIT, "pool of %d pages is 1 TiB or more", s->num_pages);
    if (need_heads) {
        if (s->num_q_heads <= 0 || s->num_q_heads % s->num_kv_heads != 0)
            return fail(PBKV_ERR_SHAPE, "num_q_heads %d is not a multiple of num_kv_heads %d",
                        s->num_q_heads, s->num_kv_heads);
        const int G = s->num_q_heads / s->num_kv_heads;
        if (s->dtype == PBKV_BF16 && !(G == 1 || G == 2 || G == 4 || G == 8 || G == 16))
            return fail(PBKV_ERR_SHAPE, "query/KV head ratio %d unsupported for bf16 (1,2,4,8,16)", G);
    }
    if (s->batch < 0 || s->max_pages_per_req < 0) return fail(PBKV_ERR_SHAPE, "negative batch or table width");
    return PBKV_OK;
}

int check_lens(const pbkv_shape *s, const int32_t *prefix_lens, const int32_t *new_lens, int64_t *total) {
    int64_t N = 0;
    for (int r = 0; r < s->batch; r++) {
        const int64_t p = prefix_lens[r], n = new_lens[r];
        if (p < 0 || n < 0) return fail(PBKV_ERR_RANGE, "request %d: negative length (%lld, %lld)", r, (long long)p, (long long)n);
        if (p + n > INT32_MAX - 4096) return fail(PBKV_ERR_RANGE, "request %d: sequence too long", r);
        const int64_t pages = n > 0 ? (p + n + s->page_size - 1) / s->page_size : (p + s->page_size - 1) / s->page_size;
        if (n > 0 && pages > s->max_pages_per_req)
            return fail(PBKV_ERR_RANGE, "request %d needs %lld pages, block_table rows hold %d", r,
                        (long long)pages, s->max_pages_per_req);
        N += n;
    }
    *total = N;
    return PBKV_OK;
}

int check_aligned(const void *p, const char *name) {
    if (((uintptr_t)p & 15) != 0) return fail(PBKV_ERR_SHAPE, "%s is not 16-byte aligned", name);
    return PBKV_OK;
}

// Pointer kinds are asked of the runtime the first time the calling thread sees an address and
// remembered after that (a model passes the same buffers layer after layer, and the query costs
// about as much as a kernel launch).  The check catches a host pointer passed by mistake; it is no
// guard against a buffer that is freed and re-allocated as something else between calls.
enum PtrKind : uint8_t { KIND_NONE = 0, KIND_DEVICE = 1, KIND_PINNED = 2 };
struct PtrMemo {
    const void *ptr[32] = {};
    uint8_t kind[32] = {};
    int next = 0;
    bool has(const void *p, uint8_t k) const {
        for (int i = 0; i < 32; i++)
            if (ptr[i] == p && kind[i] == k) return true;
        return false;
    }
    void put(const void *p, uint8_t k) { ptr[next] = p; kind[next] = k; next = (next + 1) & 31; }
};
thread_local PtrMemo g_ptr_memo;

// The pointer must be something a kernel on the current device may dereference.
int check_device_ptr(const void *p, const char *name) {
    if (g_ptr_memo.has(p, KIND_DEVICE)) return PBKV_OK;
    hipPointerAttribute_t a;
    hipError_t e = hipPointerGetAttributes(&a, p);
    if (e != hipSuccess) {
        (void)hipGetLastError();
        return fail(PBKV_ERR_DEVICE, "%s: not a device pointer (%s)", name, hipGetErrorString(e));
    }
    if (a.type != hipMemoryTypeDevice && a.type != hipMemoryTypeManaged)
        return fail(PBKV_ERR_DEVICE, "%s: expected device memory", name);
    g_ptr_memo.put(p, KIND_DEVICE);
    return PBKV_OK;
}

int check_pinned_ptr(const void *p, const char *name, const void **dev_view) {
    *dev_view = p;               // pinned memory shares one virtual address between host and device
    if (g_ptr_memo.has(p, KIND_PINNED)) return PBKV_OK;
    hipPointerAttribute_t a;
    hipError_t e = hipPointerGetAttributes(&a, p);
    if (e != hipSuccess) {
        (void)hipGetLastError();
        return fail(PBKV_ERR_DEVICE, "%s: not pinned host memory (%s)", name, hipGetErrorString(e));
    }
    if (a.type != hipMemoryTypeHost && a.type != hipMemoryTypeManaged)
        return fail(PBKV_ERR_DEVICE, "%s: expected pinned host memory", name);
    g_ptr_memo.put(p, KIND_PINNED);
    return PBKV_OK;
}

// ---- per-device state -----------------------------------------------------------------------
// (1) A ring of pinned, device-mapped descriptor memory.  Work lists are written here by the host
//     and read by the kernels through the mapped pointer (no copy in front of a kernel); a region
//     is reused only after the event recorded behind its kernel has fired.
// (2) Per stream, a small cache of work lists in device memory.  A launch that reads its list from
//     the ring also stores a copy there (every work-group writes back the descriptor it read), and
//     a later call on the same stream with the same shape and lengths -- the next layer of the same
//     batch -- launches straight from that copy: no list is built, nothing is copied, no event is
//     recorded, and no work-group reads over the host link.  Slots are only ever written and read
//     by kernels of one stream, so stream order is all the protection they need.
// (3) Per stream, the scratch buffer of the decode kernels (partials of the context slices), for
//     the same reason: calls on different streams never share one.
struct Ring {
    char *host = nullptr;
    char *dev = nullptr;
    size_t cap = 0, head = 0;
    struct Pending { hipEvent_t ev; size_t begin, end; };
    std::deque<Pending> pending;
    std::vector<hipEvent_t> spare;
};
constexpr size_t RING_BYTES = 8u << 20;
constexpr int MAX_DEVICES = 16;
constexpr int PLAN_SLOTS = 16;                  // cached work lists per stream
constexpr size_t PLAN_SLOT_BYTES = 128u << 10;  // longer lists are not cached
constexpr int MAX_STREAM_CACHES = 8;            // streams with a cache, per device

enum PlanKind { PLAN_ATTN = 1, PLAN_APPEND = 2, PLAN_DECODE = 3 };
struct Plan {
    bool valid = false;
    int kind = 0, forced_waves = 0;
    pbkv_shape shape{};
    std::vector<int32_t> lens;   // the host arrays the list was cut from, back to back
    int32_t n_a = 0, n_b = 0;    // items (tiles | runs | slices, requests)
    int32_t waves = 0;
    int64_t aux = 0;             // decode: bytes of scratch the launch needs
    uint64_t stamp = 0;
};
struct StreamCache {
    bool used = false;
    hipStream_t stream = nullptr;
    uint64_t stamp = 0;
    char *arena = nullptr;       // PLAN_SLOTS * PLAN_SLOT_BYTES of device memory
    Plan plans[PLAN_SLOTS];
    float *scratch = nullptr;    // decode partials
    size_t scratch_cap = 0;
};
struct DevState {
    std::mutex mu;               // held from the first look at this state until the kernels are enqueued
    Ring ring;
    StreamCache sc[MAX_STREAM_CACHES];
    uint64_t clock = 0;
};
DevState g_dev[MAX_DEVICES];

int device_state(DevState **out) {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return fail_hip(e, "hipGetDevice");
    if (dev < 0 || dev >= MAX_DEVICES) return fail(PBKV_ERR_DEVICE, "device index %d unsupported", dev);
    *out = &g_dev[dev];
    return PBKV_OK;
}

struct Lease { Ring *ring; size_t begin, end; char *host; char *dev; };

int ring_acquire(DevState &ds, size_t bytes, Lease *out) {
    Ring &r = ds.ring;
    hipError_t e;
    if (!r.host) {
        void *h = nullptr, *d = nullptr;
        e = hipHostMalloc(&h, RING_BYTES, hipHostMallocMapped);
        if (e != hipSuccess) return fail_hip(e, "hipHostMalloc(descriptor ring)");
        e = hipHostGetDevicePointer(&d, h, 0);
        if (e != hipSuccess) return fail_hip(e, "hipHostGetDevicePointer");
        r.host = (char *)h;
        r.dev = (char *)d;
        r.cap = RING_BYTES;
    }
    bytes = (bytes + 255) & ~(size_t)255;
    if (bytes > r.cap / 2) return fail(PBKV_ERR_LIMIT, "work list of %zu bytes exceeds the descriptor ring", bytes);
    if (r.head + bytes > r.cap) r.head = 0;
    const size_t b = r.head, en = r.head + bytes;
    // retire finished regions, wait for unfinished ones that overlap the new region
    for (auto it = r.pending.begin(); it != r.pending.end();) {
        const bool overlap = it->begin < en && it->end > b;
        hipError_t q = overlap ? hipEventSynchronize(it->ev) : hipEventQuery(it->ev);
        if (q == hipSuccess) {
            r.spare.push_back(it->ev);
            it = r.pending.erase(it);
        } else if (q == hipErrorNotReady) {
            ++it;
        } else {
            return fail_hip(q, "descriptor ring event");
        }
    }
    r.head = en;
    *out = Lease{&r, b, en, r.host + b, r.dev + b};
    return PBKV_OK;
}

// Record "the kernels reading this lease are enqueued" on the stream.
int ring_release(const Lease &l, hipStream_t s) {
    Ring &r = *l.ring;
    hipEvent_t ev;
    if (!r.spare.empty()) {
        ev = r.spare.back();
        r.spare.pop_back();
    } else {
        hipError_t e = hipEventCreateWithFlags(&ev, hipEventDisableTiming);
        if (e != hipSuccess) return fail_hip(e, "hipEventCreate");
    }
    hipError_t e = hipEventRecord(ev, s);
    if (e != hipSuccess) return fail_hip(e, "hipEventRecord");
    r.pending.push_back({ev, l.begin, l.end});
    return PBKV_OK;
}

// The cache of the stream; a stream seen for the first time takes an unused entry, or the entry
// used longest ago (its slots may still be read by that other stream's kernels: the device is
// drained first -- this only happens to callers that rotate over more than MAX_STREAM_CACHES streams).
int stream_cache(DevState &ds, hipStream_t st, StreamCache **out) {
    StreamCache *pick = nullptr;
    for (auto &c : ds.sc) {
        if (c.used && c.stream == st) {
            c.stamp = ++ds.clock;
            *out = &c;
            return PBKV_OK;
        }
        if (!pick || (pick->used && (!c.used || c.stamp < pick->stamp))) pick = &c;
    }
    hipError_t e;
    if (pick->used) {
        if ((e = hipDeviceSynchronize()) != hipSuccess) return fail_hip(e, "hipDeviceSynchronize");
        for (auto &pl : pick->plans) pl.valid = false;
    }
    if (!pick->arena) {
        void *m = nullptr;
        if ((e = hipMalloc(&m, PLAN_SLOTS * PLAN_SLOT_BYTES)) != hipSuccess) return fail_hip(e, "hipMalloc(work-list cache)");
        pick->arena = (char *)m;
    }
    pick->used = true;
    pick->stream = st;
    pick->stamp = ++ds.clock;
    *out = pick;
    return PBKV_OK;
}

bool same_shape(const pbkv_shape &a, const pbkv_shape &b) {
    return a.batch == b.batch && a.num_q_heads == b.num_q_heads && a.num_kv_heads == b.num_kv_heads &&
           a.head_dim == b.head_dim && a.page_size == b.page_size && a.dtype == b.dtype;
}

// The cached list for (kind, shape, lengths), or null.  `b` may be null (one array only).
Plan *find_plan(DevState &ds, StreamCache &c, int kind, const pbkv_shape *s, int forced_waves, const int32_t *a,
                const int32_t *b, char **dev) {
    const size_t n = (size_t)s->batch;
    for (int i = 0; i < PLAN_SLOTS; i++) {
        Plan &pl = c.plans[i];
        if (!pl.valid || pl.kind != kind || pl.forced_waves != forced_waves || !same_shape(pl.shape, *s)) continue;
        if (pl.lens.size() != (b ? 2 * n : n)) continue;
        if (memcmp(pl.lens.data(), a, n * sizeof(int32_t)) != 0) continue;
        if (b && memcmp(pl.lens.data() + n, b, n * sizeof(int32_t)) != 0) continue;
        pl.stamp = ++ds.clock;
        *dev = c.arena + (size_t)i * PLAN_SLOT_BYTES;
        return &pl;
    }
    return nullptr;
}

// The slot a new list goes to (least recently used); the caller fills in counts and marks it valid.
Plan *new_plan(DevState &ds, StreamCache &c, int kind, const pbkv_shape *s, int forced_waves, const int32_t *a,
               const int32_t *b, char **dev) {
    int pick = 0;
    for (int i = 0; i < PLAN_SLOTS; i++) {
        if (!c.plans[i].valid) { pick = i; break; }
        if (c.plans[i].stamp < c.plans[pick].stamp) pick = i;
    }
    Plan &pl = c.plans[pick];
    const size_t n = (size_t)s->batch;
    pl.valid = false;
    pl.kind = kind;
    pl.forced_waves = forced_waves;
    pl.shape = *s;
    pl.lens.assign(a, a + n);
    if (b) pl.lens.insert(pl.lens.end(), b, b + n);
    pl.stamp = ++ds.clock;
    *dev = c.arena + (size_t)pick * PLAN_SLOT_BYTES;
    return &pl;
}

// Scratch of the decode kernels for this stream: grown on demand (the stream is drained first, its
// kernels are the only readers) and kept until the process ends.
int decode_scratch(StreamCache &c, size_t bytes, float **out) {
    if (c.scratch_cap < bytes) {
        hipError_t e;
        if (c.scratch) {
            if ((e = hipStreamSynchronize(c.stream)) != hipSuccess) return fail_hip(e, "hipStreamSynchronize");
            (void)hipFree(c.scratch);
            c.scratch = nullptr;
            c.scratch_cap = 0;
        }
        const size_t cap = std::max(bytes + bytes / 2, (size_t)8 << 20);
        void *ptr = nullptr;
        if ((e = hipMalloc(&ptr, cap)) != hipSuccess) return fail_hip(e, "hipMalloc (decode scratch)");
        c.scratch = (float *)ptr;
        c.scratch_cap = cap;
    }
    *out = c.scratch;
    return PBKV_OK;
}

// Work lists live in library-owned memory that later calls reuse, so a captured graph would
// replay against lists that are gone: the entry points that use them refuse a capturing stream.
int check_not_capturing(hipStream_t st, const char *who) {
    hipStreamCaptureStatus status = hipStreamCaptureStatusNone;
    hipError_t e = hipStreamIsCapturing(st, &status);
    if (e != hipSuccess) return fail_hip(e, "hipStreamIsCapturing");
    if (status != hipStreamCaptureStatusNone)
        return fail(PBKV_ERR_DEVICE, "%s: the stream is being captured into a graph; this call cannot be replayed", who);
    return PBKV_OK;
}

constexpr int MI355X_CUS = 256;

// Work list of the attention kernels: one tile per block of T suffix tokens of a request; `pad` keeps
// the tile's index in request order.  Order: requests by descending length (prefix + suffix), and
// inside a request its token blocks from the last (most visible keys) to the first.  Long work goes
// first, so the launch ends on short work-groups, and the token blocks of one request -- which all
// stream the same K/V pages -- are handed out together: with KV head = work-group index mod H_kv
// they land on one XCD, run side by side and find each other's pages in its L2.  (Sorting the
// tiles of all requests by length alone interleaves requests of similar length; each then streams
// its prefix once per generation of its tiles: measured 2.5 - 3.6 times the compulsory HBM reads
// on the long-history and mixed batches.)
// A tile becomes wgs_per_tile consecutive work-groups; resident_pairs_wgs > 0 names the number of
// work-groups the chip holds at once when it holds two per CU (see below), 0 switches that case off.
int build_tiles(const pbkv_shape *s, const int32_t *prefix_lens, const int32_t *new_lens, int T,
                std::vector<pbkv::TileDesc> *out, int wgs_per_tile = 1, int resident_pairs_wgs = 0) {
    std::vector<pbkv::TileDesc> &tiles = *out;
    tiles.clear();
    thread_local std::vector<int32_t> order;
    thread_local std::vector<int64_t> row0, idx0;
    order.resize((size_t)s->batch);
    row0.resize((size_t)s->batch);
    idx0.resize((size_t)s->batch);
    int64_t rows = 0, idx = 0;
    for (int r = 0; r < s->batch; r++) {
        order[r] = r;
        row0[r] = rows;
        idx0[r] = idx;
        rows += new_lens[r];
        idx += (new_lens[r] + T - 1) / T;
    }
    std::stable_sort(order.begin(), order.end(), [&](int32_t a, int32_t b) {
        return (int64_t)prefix_lens[a] + new_lens[a] > (int64_t)prefix_lens[b] + new_lens[b];
    });
    for (int32_t r : order) {
        const int32_t nb = (new_lens[r] + T - 1) / T;
        for (int32_t k = nb - 1; k >= 0; k--)
            tiles.push_back(pbkv::TileDesc{r, k * T, prefix_lens[r], new_lens[r], row0[r], idx0[r] + k});
    }
    // A launch whose work-groups are all resident at once, two per CU (the 4-wave shape on 256 CUs),
    // finishes when the CU with the most work does, and the dispatcher hands out one work-group per CU
    // before it starts on the second: the second half of the list is reversed, so that the CU holding
    // the longest work-group also gets the shortest (measured +2 % on the shared-prompt batch's
    // attention launch running alone; no difference with the append kernel beside it).
    const size_t n = tiles.size();
    if (resident_pairs_wgs > 0 && n * (size_t)wgs_per_tile > (size_t)resident_pairs_wgs / 2 &&
        n * (size_t)wgs_per_tile <= (size_t)resident_pairs_wgs)
        std::reverse(tiles.begin() + (resident_pairs_wgs / 2 + wgs_per_tile - 1) / wgs_per_tile, tiles.end());
    if (tiles.size() > (size_t)INT32_MAX / 64) return fail(PBKV_ERR_LIMIT, "too many tiles");
    return PBKV_OK;
}

thread_local std::vector<pbkv::TileDesc> tl_tiles;
thread_local std::vector<pbkv::AppendDesc> tl_runs;
thread_local std::vector<pbkv::DecodeUnit> tl_units;
thread_local std::vector<pbkv::DecodeReq> tl_reqs;
thread_local std::vector<uint8_t> tl_seen;
thread_local std::vector<int32_t> tl_ids;

}  // namespace

extern "C" {

const char *pbkv_last_error(void) { return g_err; }

const char *pbkv_version(void) { return "pbkv 0.2 gfx950"; }

int64_t pbkv_page_bytes(const pbkv_shape *s) {
    if (!s || check_shape(s, false) != PBKV_OK) return 0;
    return (int64_t)2 * s->num_kv_heads * s->page_size * s->head_dim * elt_bytes(s->dtype);
}

int pbkv_set_attn_waves(int waves) {
    g_err[0] = 0;
    if (waves != 0 && waves != 4 && waves != 8 && waves != 64) return fail(PBKV_ERR_SHAPE, "pbkv_set_attn_waves: %d (0, 4, 8 or 64)", waves);
    pbkv::attn_bf16_force_waves(waves);
    return PBKV_OK;
}

int pbkv_prefix_prefill(const pbkv_shape *s, const void *q, const void *k_new, const void *v_new,
                        const void *kv_pool, const int32_t *block_table, const int32_t *prefix_lens,
                        const int32_t *new_lens, void *out, void *stream) {
    g_err[0] = 0;
    int rc = check_shape(s, true);
    if (rc) return rc;
    if (s->batch == 0) return PBKV_OK;
    if (!q || !k_new || !v_new || !kv_pool || !block_table || !prefix_lens || !new_lens || !out)
        return fail(PBKV_ERR_NULL, "pbkv_prefix_prefill: NULL argument");
    int64_t N = 0;
    if ((rc = check_lens(s, prefix_lens, new_lens, &N))) return rc;
    if (N == 0) return PBKV_OK;
    if ((rc = check_aligned(q, "q")) || (rc = check_aligned(k_new, "k_new")) || (rc = check_aligned(v_new, "v_new")) ||
        (rc = check_aligned(kv_pool, "kv_pool")) || (rc = check_aligned(out, "out")))
        return rc;
    if ((rc = check_device_ptr(q, "q")) || (rc = check_device_ptr(k_new, "k_new")) ||
        (rc = check_device_ptr(v_new, "v_new")) || (rc = check_device_ptr(kv_pool, "kv_pool")) ||
        (rc = check_device_ptr(block_table, "block_table")) || (rc = check_device_ptr(out, "out")))
        return rc;

    hipStream_t st = (hipStream_t)stream;
    if ((rc = check_not_capturing(st, "pbkv_prefix_prefill"))) return rc;
    pbkv::AttnParams p;
    p.q = q; p.k_new = k_new; p.v_new = v_new; p.kv_pool = kv_pool; p.out = out;
    p.block_table = block_table;
    p.Hq = s->num_q_heads; p.Hkv = s->num_kv_heads;
    p.max_pages = s->max_pages_per_req; p.num_pages = s->num_pages;
    p.mirror = nullptr;
    const bool bf16 = s->dtype == PBKV_BF16;
    auto launch = [&]() {
        return bf16 ? pbkv::launch_attn_bf16(p, s->head_dim, st) : pbkv::launch_attn_f32(p, s->head_dim, st);
    };

    DevState *ds = nullptr;
    if ((rc = device_state(&ds))) return rc;
    std::lock_guard<std::mutex> lock(ds->mu);
    StreamCache *sc = nullptr;
    char *slot = nullptr;
    const int forced = pbkv::attn_bf16_forced_waves();
    if (bf16) {
        if ((rc = stream_cache(*ds, st, &sc))) return rc;
        if (Plan *pl = find_plan(*ds, *sc, PLAN_ATTN, s, forced, prefix_lens, new_lens, &slot)) {
            p.tiles = (const pbkv::TileDesc *)slot;
            p.n_tiles = pl->n_a;
            p.waves = pl->waves;
            hipError_t e = launch();
            return e == hipSuccess ? PBKV_OK : fail_hip(e, "attention launch");
        }
    }

    const int G = s->num_q_heads / s->num_kv_heads;
    const int waves = bf16 ? pbkv::attn_bf16_waves(prefix_lens, new_lens, s->batch) : 0;
    const int T = bf16 ? pbkv::attn_bf16_tile_tokens(s->head_dim, G, waves) : pbkv::attn_f32_tile_tokens();
    std::vector<pbkv::TileDesc> &tiles = tl_tiles;
    const int per_tile = bf16 ? pbkv::attn_bf16_units_per_tile(s->num_kv_heads, G) : 1;
    if ((rc = build_tiles(s, prefix_lens, new_lens, T, &tiles, per_tile, waves == 4 ? 2 * MI355X_CUS : 0))) return rc;
    const size_t bytes = tiles.size() * sizeof(pbkv::TileDesc);

    Lease lease;
    if ((rc = ring_acquire(*ds, bytes, &lease))) return rc;
    memcpy(lease.host, tiles.data(), bytes);
    p.tiles = (const pbkv::TileDesc *)lease.dev;
    p.n_tiles = (int32_t)tiles.size();
    p.waves = waves;
    Plan *pl = nullptr;
    if (bf16 && bytes <= PLAN_SLOT_BYTES) {
        pl = new_plan(*ds, *sc, PLAN_ATTN, s, forced, prefix_lens, new_lens, &slot);
        pl->n_a = p.n_tiles;
        pl->waves = waves;
        p.mirror = (pbkv::TileDesc *)slot;
    }
    hipError_t e = launch();
    int rel = ring_release(lease, st);
    if (e != hipSuccess) return fail_hip(e, "attention launch");
    if (pl) pl->valid = true;
    return rel;
}

int pbkv_gather_probe(const pbkv_shape *s, const void *k_new, const void *v_new, const void *kv_pool,
                      const int32_t *block_table, const int32_t *prefix_lens, const int32_t *new_lens,
                      uint32_t *unit_xor, int64_t unit_capacity, int64_t *n_units, int32_t *unit_tokens,
                      void *stream) {
    g_err[0] = 0;
    int rc = check_shape(s, true);
    if (rc) return rc;
    if (s->dtype != PBKV_BF16) return fail(PBKV_ERR_DTYPE, "pbkv_gather_probe: bf16 only");
    if (!n_units || !unit_tokens) return fail(PBKV_ERR_NULL, "pbkv_gather_probe: NULL argument");
    const int G = s->num_q_heads / s->num_kv_heads;
    *unit_tokens = pbkv::attn_bf16_tile_tokens(s->head_dim, G, 8);
    *n_units = 0;
    if (s->batch == 0) return PBKV_OK;
    if (!k_new || !v_new || !kv_pool || !block_table || !prefix_lens || !new_lens)
        return fail(PBKV_ERR_NULL, "pbkv_gather_probe: NULL argument");
    int64_t N = 0;
    if ((rc = check_lens(s, prefix_lens, new_lens, &N))) return rc;
    const int waves = pbkv::attn_bf16_waves(prefix_lens, new_lens, s->batch);   // the attention call's own choice
    const int T = pbkv::attn_bf16_tile_tokens(s->head_dim, G, waves);
    *unit_tokens = T;
    std::vector<pbkv::TileDesc> &tiles = tl_tiles;
    if ((rc = build_tiles(s, prefix_lens, new_lens, T, &tiles, pbkv::attn_bf16_units_per_tile(s->num_kv_heads, G),
                          waves == 4 ? 2 * MI355X_CUS : 0)))
        return rc;
    const int64_t units = (int64_t)tiles.size() * pbkv::attn_bf16_units_per_tile(s->num_kv_heads, G);
    *n_units = units;
    if (units == 0 || (!unit_xor && unit_capacity == 0)) return PBKV_OK;   // nothing to do / size query
    if (!unit_xor) return fail(PBKV_ERR_NULL, "pbkv_gather_probe: NULL unit_xor");
    if (unit_capacity < units)
        return fail(PBKV_ERR_RANGE, "pbkv_gather_probe: %lld units need room, unit_xor holds %lld", (long long)units,
                    (long long)unit_capacity);
    if ((rc = check_aligned(k_new, "k_new")) || (rc = check_aligned(v_new, "v_new")) ||
        (rc = check_aligned(kv_pool, "kv_pool")))
        return rc;
    if ((rc = check_device_ptr(k_new, "k_new")) || (rc = check_device_ptr(v_new, "v_new")) ||
        (rc = check_device_ptr(kv_pool, "kv_pool")) || (rc = check_device_ptr(block_table, "block_table")) ||
        (rc = check_device_ptr(unit_xor, "unit_xor")))
        return rc;

    if ((rc = check_not_capturing((hipStream_t)stream, "this call"))) return rc;
    DevState *ds = nullptr;
    if ((rc = device_state(&ds))) return rc;
    std::lock_guard<std::mutex> lock(ds->mu);
    Lease lease;
    if ((rc = ring_acquire(*ds, tiles.size() * sizeof(pbkv::TileDesc), &lease))) return rc;
    memcpy(lease.host, tiles.data(), tiles.size() * sizeof(pbkv::TileDesc));
    pbkv::AttnParams p;
    p.q = nullptr; p.k_new = k_new; p.v_new = v_new; p.kv_pool = kv_pool; p.out = unit_xor;
    p.block_table = block_table;
    p.tiles = (const pbkv::TileDesc *)lease.dev;
    p.n_tiles = (int32_t)tiles.size();
    p.Hq = s->num_q_heads; p.Hkv = s->num_kv_heads;
    p.max_pages = s->max_pages_per_req; p.num_pages = s->num_pages;
    p.waves = waves;
    p.mirror = nullptr;
    hipStream_t st = (hipStream_t)stream;
    hipError_t e = pbkv::launch_gather_probe(p, s->head_dim, st);
    int rel = ring_release(lease, st);
    if (e != hipSuccess) return fail_hip(e, "gather probe launch");
    return rel;
}

int pbkv_append_kv(const pbkv_shape *s, const void *k_new, const void *v_new, void *kv_pool,
                   const int32_t *block_table, const int32_t *prefix_lens, const int32_t *new_lens,
                   void *stream) {
    g_err[0] = 0;
    int rc = check_shape(s, false);
    if (rc) return rc;
    if (s->batch == 0) return PBKV_OK;
    if (!k_new || !v_new || !kv_pool || !block_table || !prefix_lens || !new_lens)
        return fail(PBKV_ERR_NULL, "pbkv_append_kv: NULL argument");
    int64_t N = 0;
    if ((rc = check_lens(s, prefix_lens, new_lens, &N))) return rc;
    if (N == 0) return PBKV_OK;
    if ((rc = check_aligned(k_new, "k_new")) || (rc = check_aligned(v_new, "v_new")) ||
        (rc = check_aligned(kv_pool, "kv_pool")))
        return rc;
    if ((rc = check_device_ptr(k_new, "k_new")) || (rc = check_device_ptr(v_new, "v_new")) ||
        (rc = check_device_ptr(kv_pool, "kv_pool")) || (rc = check_device_ptr(block_table, "block_table")))
        return rc;

    hipStream_t st = (hipStream_t)stream;
    if ((rc = check_not_capturing(st, "pbkv_append_kv"))) return rc;
    pbkv::AppendParams p;
    p.k_new = k_new; p.v_new = v_new; p.kv_pool = kv_pool; p.block_table = block_table;
    p.mirror = nullptr;
    p.Hkv = s->num_kv_heads; p.max_pages = s->max_pages_per_req; p.num_pages = s->num_pages;

    DevState *ds = nullptr;
    if ((rc = device_state(&ds))) return rc;
    std::lock_guard<std::mutex> lock(ds->mu);
    StreamCache *sc = nullptr;
    char *slot = nullptr;
    if ((rc = stream_cache(*ds, st, &sc))) return rc;
    if (Plan *pl = find_plan(*ds, *sc, PLAN_APPEND, s, 0, prefix_lens, new_lens, &slot)) {
        p.descs = (const pbkv::AppendDesc *)slot;
        p.n_descs = pl->n_a;
        hipError_t e = pbkv::launch_append(p, s->head_dim, elt_bytes(s->dtype), st);
        return e == hipSuccess ? PBKV_OK : fail_hip(e, "append launch");
    }

    const int P = s->page_size;
    std::vector<pbkv::AppendDesc> &descs = tl_runs;
    descs.clear();
    int64_t row0 = 0;
    for (int r = 0; r < s->batch; r++) {
        const int64_t pr = prefix_lens[r], n = new_lens[r];
        for (int64_t t = 0; t < n;) {
            const int64_t pos = pr + t;
            const int slot0 = (int)(pos % P);
            const int count = (int)std::min<int64_t>(P - slot0, n - t);
            descs.push_back(pbkv::AppendDesc{row0 + t, r, (int32_t)(pos / P), slot0, count, 0});
            t += count;
        }
        row0 += n;
    }
    if (descs.size() > (size_t)INT32_MAX / 64) return fail(PBKV_ERR_LIMIT, "too many page runs");
    const size_t bytes = descs.size() * sizeof(pbkv::AppendDesc);
    Lease lease;
    if ((rc = ring_acquire(*ds, bytes, &lease))) return rc;
    memcpy(lease.host, descs.data(), bytes);
    p.descs = (const pbkv::AppendDesc *)lease.dev;
    p.n_descs = (int32_t)descs.size();
    Plan *pl = nullptr;
    if (bytes <= PLAN_SLOT_BYTES) {
        pl = new_plan(*ds, *sc, PLAN_APPEND, s, 0, prefix_lens, new_lens, &slot);
        pl->n_a = p.n_descs;
        p.mirror = (pbkv::AppendDesc *)slot;
    }
    hipError_t e = pbkv::launch_append(p, s->head_dim, elt_bytes(s->dtype), st);
    int rel = ring_release(lease, st);
    if (e != hipSuccess) return fail_hip(e, "append launch");
    if (pl) pl->valid = true;
    return rel;
}

}  // extern "C"

namespace {

// Page ids of a swap: inside the pool and (swap-in: they are destinations) all distinct.
int check_page_ids(const pbkv_shape *s, const int32_t *page_ids, int32_t n_pages, bool distinct) {
    for (int i = 0; i < n_pages; i++) {
        const int32_t id = page_ids[i];
        if (id < 0 || id >= s->num_pages)
            return fail(PBKV_ERR_RANGE, "page_ids[%d] = %d outside pool of %d pages", i, id, s->num_pages);
    }
    if (!distinct) return PBKV_OK;
    if ((int64_t)n_pages * 16 < s->num_pages) {
        // few pages of a large pool: sort a copy instead of clearing a flag per pool page
        std::vector<int32_t> &ids = tl_ids;
        ids.assign(page_ids, page_ids + n_pages);
        std::sort(ids.begin(), ids.end());
        for (int i = 1; i < n_pages; i++)
            if (ids[i] == ids[i - 1]) return fail(PBKV_ERR_ALIAS, "page id %d appears twice", ids[i]);
        return PBKV_OK;
    }
    std::vector<uint8_t> &seen = tl_seen;
    seen.assign((size_t)s->num_pages, 0);
    for (int i = 0; i < n_pages; i++) {
        const int32_t id = page_ids[i];
        if (seen[id]) return fail(PBKV_ERR_ALIAS, "page_ids[%d] = %d appears twice", i, id);
        seen[id] = 1;
    }
    return PBKV_OK;
}

}  // namespace

extern "C" {

int pbkv_swap_in_pages(const pbkv_shape *s, const void *host_pages, const int32_t *page_ids,
                       int32_t n_pages, void *kv_pool, void *stream) {
    g_err[0] = 0;
    int rc = check_shape(s, false);
    if (rc) return rc;
    if (n_pages < 0) return fail(PBKV_ERR_RANGE, "n_pages %d", n_pages);
    if (n_pages == 0) return PBKV_OK;
    if (!host_pages || !page_ids || !kv_pool) return fail(PBKV_ERR_NULL, "pbkv_swap_in_pages: NULL argument");
    if ((rc = check_page_ids(s, page_ids, n_pages, true))) return rc;
    if ((rc = check_aligned(host_pages, "host_pages")) || (rc = check_aligned(kv_pool, "kv_pool"))) return rc;
    const void *host_dev = nullptr;
    if ((rc = check_pinned_ptr(host_pages, "host_pages", &host_dev))) return rc;
    if ((rc = check_device_ptr(kv_pool, "kv_pool"))) return rc;

    if ((rc = check_not_capturing((hipStream_t)stream, "this call"))) return rc;
    DevState *ds = nullptr;
    if ((rc = device_state(&ds))) return rc;
    std::lock_guard<std::mutex> lock(ds->mu);
    Lease lease;
    if ((rc = ring_acquire(*ds, (size_t)n_pages * sizeof(int32_t), &lease))) return rc;
    memcpy(lease.host, page_ids, (size_t)n_pages * sizeof(int32_t));
    hipStream_t st = (hipStream_t)stream;
    hipError_t e = pbkv::launch_swap_in(host_dev, (const int32_t *)lease.dev, n_pages, kv_pool,
                                        pbkv_page_bytes(s), st);
    int rel = ring_release(lease, st);
    if (e != hipSuccess) return fail_hip(e, "swap-in launch");
    return rel;
}

}  // extern "C"

namespace {

constexpr int64_t DECODE_TARGET_WGS = 2048;   // work-groups aimed for (1024 / 4096 / 8192 were measured: not faster)

// Validation shared by the decode entry points; also sums the pages of all contexts.
int check_decode_args(const pbkv_shape *s, const void *q, const void *kv_pool, const int32_t *block_table,
                      const int32_t *context_lens, void *out, int64_t *total_pages, const char *who) {
    int rc = check_shape(s, true);
    if (rc) return rc;
    if (s->dtype != PBKV_BF16) return fail(PBKV_ERR_DTYPE, "%s: bf16 only", who);
    *total_pages = 0;
    if (s->batch == 0) return PBKV_OK;
    if (!q || !kv_pool || !block_table || !context_lens || !out) return fail(PBKV_ERR_NULL, "%s: NULL argument", who);
    const int B = s->batch, P = s->page_size;
    for (int r = 0; r < B; r++) {
        const int64_t L = context_lens[r];
        if (L < 0 || L > INT32_MAX - 4096) return fail(PBKV_ERR_RANGE, "request %d: context length %lld", r, (long long)L);
        const int64_t pages = (L + P - 1) / P;
        if (pages > s->max_pages_per_req)
            return fail(PBKV_ERR_RANGE, "request %d needs %lld pages, block_table rows hold %d", r, (long long)pages,
                        s->max_pages_per_req);
        *total_pages += pages;
    }
    if ((rc = check_aligned(q, "q")) || (rc = check_aligned(kv_pool, "kv_pool")) || (rc = check_aligned(out, "out"))) return rc;
    if ((rc = check_device_ptr(q, "q")) || (rc = check_device_ptr(kv_pool, "kv_pool")) ||
        (rc = check_device_ptr(block_table, "block_table")) || (rc = check_device_ptr(out, "out")))
        return rc;
    return PBKV_OK;
}

// Slices of the contexts: enough work-groups to fill the chip a few times over, at least 16 pages each.
int build_decode_units(const pbkv_shape *s, const int32_t *context_lens, int64_t total_pages,
                       std::vector<pbkv::DecodeUnit> *units_out, std::vector<pbkv::DecodeReq> *reqs_out) {
    const int B = s->batch, P = s->page_size;
    const int G = s->num_q_heads / s->num_kv_heads;
    const int per_unit = s->num_kv_heads * (G / pbkv::decode_heads_per_group(G));   // work-groups per slice
    int64_t pps = (total_pages * per_unit + DECODE_TARGET_WGS - 1) / DECODE_TARGET_WGS;
    pps = std::max<int64_t>(16, (pps + 3) & ~(int64_t)3);
    std::vector<pbkv::DecodeUnit> &units = *units_out;
    std::vector<pbkv::DecodeReq> &reqs = *reqs_out;
    units.clear();
    reqs.assign((size_t)B, pbkv::DecodeReq{0, 0, {0, 0}});
    for (int r = 0; r < B; r++) {
        const int32_t L = context_lens[r];
        const int32_t pages = (L + P - 1) / P;
        reqs[r] = pbkv::DecodeReq{(int32_t)units.size(), 0, {0, 0}};
        for (int32_t p0 = 0; p0 < pages; p0 += (int32_t)pps) {
            const int32_t p1 = (int32_t)std::min<int64_t>(pages, p0 + pps);
            units.push_back(pbkv::DecodeUnit{r, L, p0, p1, (int32_t)units.size(), {0, 0, 0}});
            reqs[r].n_splits++;
        }
    }
    if (units.size() > (size_t)INT32_MAX / 64) return fail(PBKV_ERR_LIMIT, "too many slices");
    return PBKV_OK;
}

size_t decode_scratch_bytes(const pbkv_shape *s, size_t n_units) {
    const int G = s->num_q_heads / s->num_kv_heads;
    const int per_unit = s->num_kv_heads * (G / pbkv::decode_heads_per_group(G));
    return std::max<size_t>(n_units, 1) * per_unit * pbkv::decode_partial_floats(s->head_dim, G) * sizeof(float);
}

}  // namespace

extern "C" {

int pbkv_paged_decode(const pbkv_shape *s, const void *q, const void *kv_pool, const int32_t *block_table,
                      const int32_t *context_lens, void *out, void *stream) {
    g_err[0] = 0;
    int64_t total_pages = 0;
    int rc = check_decode_args(s, q, kv_pool, block_table, context_lens, out, &total_pages, "pbkv_paged_decode");
    if (rc) return rc;
    if (s->batch == 0) return PBKV_OK;
    const int B = s->batch;
    hipStream_t st = (hipStream_t)stream;
    if ((rc = check_not_capturing(st, "pbkv_paged_decode"))) return rc;
    pbkv::DecodeParams p;
    p.q = q; p.kv_pool = kv_pool; p.out = out; p.block_table = block_table;
    p.mirror_units = nullptr; p.mirror_reqs = nullptr;
    p.n_reqs = B;
    p.Hq = s->num_q_heads; p.Hkv = s->num_kv_heads;
    p.max_pages = s->max_pages_per_req; p.num_pages = s->num_pages;

    DevState *ds = nullptr;
    if ((rc = device_state(&ds))) return rc;
    std::lock_guard<std::mutex> lock(ds->mu);
    StreamCache *sc = nullptr;
    char *slot = nullptr;
    if ((rc = stream_cache(*ds, st, &sc))) return rc;
    if (Plan *pl = find_plan(*ds, *sc, PLAN_DECODE, s, 0, context_lens, nullptr, &slot)) {
        if ((rc = decode_scratch(*sc, (size_t)pl->aux, &p.scratch))) return rc;
        p.units = (const pbkv::DecodeUnit *)slot;
        p.reqs = (const pbkv::DecodeReq *)(slot + (size_t)pl->n_a * sizeof(pbkv::DecodeUnit));
        p.n_units = pl->n_a;
        hipError_t e = pbkv::launch_decode_bf16(p, s->head_dim, st);
        return e == hipSuccess ? PBKV_OK : fail_hip(e, "decode launch");
    }

    std::vector<pbkv::DecodeUnit> &units = tl_units;
    std::vector<pbkv::DecodeReq> &reqs = tl_reqs;
    if ((rc = build_decode_units(s, context_lens, total_pages, &units, &reqs))) return rc;
    const size_t need = decode_scratch_bytes(s, units.size());
    if ((rc = decode_scratch(*sc, need, &p.scratch))) return rc;

    Lease lease;
    const size_t ub = units.size() * sizeof(pbkv::DecodeUnit), rb = reqs.size() * sizeof(pbkv::DecodeReq);
    if ((rc = ring_acquire(*ds, ub + rb, &lease))) return rc;
    memcpy(lease.host, units.data(), ub);
    memcpy((char *)lease.host + ub, reqs.data(), rb);
    p.units = (const pbkv::DecodeUnit *)lease.dev;
    p.reqs = (const pbkv::DecodeReq *)((const char *)lease.dev + ub);
    p.n_units = (int32_t)units.size();
    Plan *pl = nullptr;
    if (ub + rb <= PLAN_SLOT_BYTES) {
        pl = new_plan(*ds, *sc, PLAN_DECODE, s, 0, context_lens, nullptr, &slot);
        pl->n_a = p.n_units;
        pl->n_b = B;
        pl->aux = (int64_t)need;
        p.mirror_units = (pbkv::DecodeUnit *)slot;
        p.mirror_reqs = (pbkv::DecodeReq *)(slot + ub);
    }
    hipError_t e = pbkv::launch_decode_bf16(p, s->head_dim, st);
    int rel = ring_release(lease, st);
    if (e != hipSuccess) return fail_hip(e, "decode launch");
    if (pl) pl->valid = true;
    return rel;
}

int pbkv_swap_out_pages(const pbkv_shape *s, const void *kv_pool, const int32_t *page_ids,
                        int32_t n_pages, void *host_pages, void *stream) {
    g_err[0] = 0;
    int rc = check_shape(s, false);
    if (rc) return rc;
    if (n_pages < 0) return fail(PBKV_ERR_RANGE, "n_pages %d", n_pages);
    if (n_pages == 0) return PBKV_OK;
    if (!host_pages || !page_ids || !kv_pool) return fail(PBKV_ERR_NULL, "pbkv_swap_out_pages: NULL argument");
    if ((rc = check_page_ids(s, page_ids, n_pages, false))) return rc;
    if ((rc = check_aligned(host_pages, "host_pages")) || (rc = check_aligned(kv_pool, "kv_pool"))) return rc;
    const void *host_dev = nullptr;
    if ((rc = check_pinned_ptr(host_pages, "host_pages", &host_dev))) return rc;
    if ((rc = check_device_ptr(kv_pool, "kv_pool"))) return rc;

    if ((rc = check_not_capturing((hipStream_t)stream, "this call"))) return rc;
    DevState *ds = nullptr;
    if ((rc = device_state(&ds))) return rc;
    std::lock_guard<std::mutex> lock(ds->mu);
    Lease lease;
    if ((rc = ring_acquire(*ds, (size_t)n_pages * sizeof(int32_t), &lease))) return rc;
    memcpy(lease.host, page_ids, (size_t)n_pages * sizeof(int32_t));
    hipStream_t st = (hipStream_t)stream;
    hipError_t e = pbkv::launch_swap_out(kv_pool, (const int32_t *)lease.dev, n_pages, (void *)host_dev,
                                         pbkv_page_bytes(s), st);
    int rel = ring_release(lease, st);
    if (e != hipSuccess) return fail_hip(e, "swap-out launch");
    return rel;
}

}  // extern "C"

// ---- decode without any allocation -----------------------------------------------------------
// For callers that cannot allocate device memory (code under graph capture, tight serving loops,
// harnesses that forbid it): the partials of the context slices and the two work lists live in one
// file-scope device array instead of library-allocated buffers, and the lists reach it through
// kernel arguments (a launch copies its arguments before it returns, so no host buffer has to stay
// alive and no ring, event or copy is involved).
namespace {

constexpr size_t STATIC_PARTIAL_BYTES = 8u << 20;
constexpr int STATIC_MAX_UNITS = 4096;
constexpr int STATIC_MAX_REQS = 4096;
constexpr size_t STATIC_UNITS_OFF = STATIC_PARTIAL_BYTES;
constexpr size_t STATIC_REQS_OFF = STATIC_UNITS_OFF + STATIC_MAX_UNITS * sizeof(pbkv::DecodeUnit);
constexpr size_t STATIC_BYTES = STATIC_REQS_OFF + STATIC_MAX_REQS * sizeof(pbkv::DecodeReq);

// Every GPU the library runs on holds its own copy of this array, at its own address, until the
// process ends.  In host code the name is only a handle for hipGetSymbolAddress.
static __device__ __align__(256) unsigned char scratch[STATIC_BYTES];

std::mutex g_static_mu;
void *g_static_ptr[MAX_DEVICES] = {};

// Device address of `scratch` on the current device (asked once per device).
int static_scratch(unsigned char **out) {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return fail_hip(e, "hipGetDevice");
    if (dev < 0 || dev >= MAX_DEVICES) return fail(PBKV_ERR_DEVICE, "device index %d unsupported", dev);
    std::lock_guard<std::mutex> lock(g_static_mu);
    if (!g_static_ptr[dev]) {
        void *ptr = nullptr;
        e = hipGetSymbolAddress((void **)&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !ptr) return fail_hip(e, "hipGetSymbolAddress(scratch)");
        g_static_ptr[dev] = ptr;
    }
    *out = (unsigned char *)g_static_ptr[dev];
    return PBKV_OK;
}

constexpr int STAGE_WORDS = 896;                     // 3.5 KiB of a launch's 4 KiB of arguments
struct StageChunk { uint32_t w[STAGE_WORDS]; };

__global__ __launch_bounds__(256) void stage_kernel(StageChunk c, uint32_t *dst, int n) {
    for (int i = threadIdx.x; i < n; i += 256) dst[i] = c.w[i];
}

// Copies `bytes` (a multiple of 4) of host memory to device memory at dst through kernel arguments.
hipError_t stage_words(const void *src, size_t bytes, void *dst, hipStream_t st) {
    const uint32_t *w = (const uint32_t *)src;
    size_t words = bytes / 4;
    uint32_t *d = (uint32_t *)dst;
    while (words > 0) {
        const int n = (int)std::min<size_t>(words, STAGE_WORDS);
        StageChunk c;
        memcpy(c.w, w, (size_t)n * 4);
        hipLaunchKernelGGL(stage_kernel, dim3(1), dim3(256), 0, st, c, d, n);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
        w += n;
        d += n;
        words -= n;
    }
    return hipSuccess;
}

}  // namespace

extern "C" {

int pbkv_paged_decode_static(const pbkv_shape *s, const void *q, const void *kv_pool, const int32_t *block_table,
                             const int32_t *context_lens, void *out, void *stream) {
    g_err[0] = 0;
    int64_t total_pages = 0;
    int rc = check_decode_args(s, q, kv_pool, block_table, context_lens, out, &total_pages, "pbkv_paged_decode_static");
    if (rc) return rc;
    if (s->batch == 0) return PBKV_OK;
    if (s->batch > STATIC_MAX_REQS)
        return fail(PBKV_ERR_LIMIT, "pbkv_paged_decode_static: %d requests, at most %d", s->batch, STATIC_MAX_REQS);
    std::vector<pbkv::DecodeUnit> &units = tl_units;
    std::vector<pbkv::DecodeReq> &reqs = tl_reqs;
    if ((rc = build_decode_units(s, context_lens, total_pages, &units, &reqs))) return rc;
    if (units.size() > (size_t)STATIC_MAX_UNITS)
        return fail(PBKV_ERR_LIMIT, "pbkv_paged_decode_static: %zu context slices, at most %d", units.size(), STATIC_MAX_UNITS);
    const size_t need = decode_scratch_bytes(s, units.size());
    if (need > STATIC_PARTIAL_BYTES)
        return fail(PBKV_ERR_LIMIT, "pbkv_paged_decode_static: %zu bytes of partial results, at most %zu", need,
                    STATIC_PARTIAL_BYTES);
    unsigned char *base = nullptr;
    if ((rc = static_scratch(&base))) return rc;

    hipStream_t st = (hipStream_t)stream;
    hipError_t e = stage_words(units.data(), units.size() * sizeof(pbkv::DecodeUnit), base + STATIC_UNITS_OFF, st);
    if (e == hipSuccess) e = stage_words(reqs.data(), reqs.size() * sizeof(pbkv::DecodeReq), base + STATIC_REQS_OFF, st);
    if (e != hipSuccess) return fail_hip(e, "work-list launch");
    pbkv::DecodeParams p;
    p.q = q; p.kv_pool = kv_pool; p.out = out; p.block_table = block_table;
    p.units = (const pbkv::DecodeUnit *)(base + STATIC_UNITS_OFF);
    p.reqs = (const pbkv::DecodeReq *)(base + STATIC_REQS_OFF);
    p.mirror_units = nullptr; p.mirror_reqs = nullptr;
    p.scratch = (float *)base;
    p.n_units = (int32_t)units.size(); p.n_reqs = s->batch;
    p.Hq = s->num_q_heads; p.Hkv = s->num_kv_heads;
    p.max_pages = s->max_pages_per_req; p.num_pages = s->num_pages;
    e = pbkv::launch_decode_bf16(p, s->head_dim, st);
    return e == hipSuccess ? PBKV_OK : fail_hip(e, "decode launch");
}

}  // extern "C"

