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

// The pointer must be something a kernel on the current device may dereference.
int check_device_ptr(const void *p, const char *name) {
    hipPointerAttribute_t a;
    hipError_t e = hipPointerGetAttributes(&a, p);
    if (e != hipSuccess) {
        (void)hipGetLastError();
        return fail(PBKV_ERR_DEVICE, "%s: not a device pointer (%s)", name, hipGetErrorString(e));
    }
    if (a.type != hipMemoryTypeDevice && a.type != hipMemoryTypeManaged)
        return fail(PBKV_ERR_DEVICE, "%s: expected device memory", name);
    return PBKV_OK;
}

int check_pinned_ptr(const void *p, const char *name, const void **dev_view) {
    hipPointerAttribute_t a;
    hipError_t e = hipPointerGetAttributes(&a, p);
    if (e != hipSuccess) {
        (void)hipGetLastError();
        return fail(PBKV_ERR_DEVICE, "%s: not pinned host memory (%s)", name, hipGetErrorString(e));
    }
    if (a.type != hipMemoryTypeHost && a.type != hipMemoryTypeManaged && a.type != hipMemoryTypeDevice)
        return fail(PBKV_ERR_DEVICE, "%s: expected pinned host memory", name);
    // pinned memory shares one virtual address between host and device
    *dev_view = p;
    return PBKV_OK;
}

// ---- per-device ring of pinned, device-mapped descriptor memory ---------------------------
// Work lists are written here by the host and read by the kernels through the mapped
// pointer; a region is reused only after the event recorded behind its kernel has fired.
struct Ring {
    char *host = nullptr;
    char *dev = nullptr;
    char *mirror = nullptr;          // device-memory copy of the ring (descriptor placement "device")
    size_t cap = 0, head = 0;
    struct Pending { hipEvent_t ev; size_t begin, end; };
    std::deque<Pending> pending;
    std::vector<hipEvent_t> spare;
    std::mutex mu;
};
constexpr size_t RING_BYTES = 8u << 20;
constexpr int MAX_DEVICES = 16;
Ring g_rings[MAX_DEVICES];

struct Lease { Ring *ring; size_t begin, end; char *host; char *dev; };

// Where kernels read their work lists from.  Default: the pinned ring itself, through its
// device-mapped address (no copy in front of a kernel).  PBKV_DESCRIPTORS=device: a
// device-memory mirror, filled by a small stream-ordered copy per call -- for callers that run
// kernels beside bulk host-link traffic, where a work-group's descriptor read over the link
// would queue behind that traffic.
bool descriptors_in_device_memory() {
    static const bool v = [] { const char *e = getenv("PBKV_DESCRIPTORS"); return e && std::string(e) == "device"; }();
    return v;
}

int ring_acquire(size_t bytes, Lease *out) {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return fail_hip(e, "hipGetDevice");
    if (dev < 0 || dev >= MAX_DEVICES) return fail(PBKV_ERR_DEVICE, "device index %d unsupported", dev);
    Ring &r = g_rings[dev];
    std::lock_guard<std::mutex> lk(r.mu);
    if (!r.host) {
        void *h = nullptr, *d = nullptr;
        e = hipHostMalloc(&h, RING_BYTES, hipHostMallocMapped);
        if (e != hipSuccess) return fail_hip(e, "hipHostMalloc(descriptor ring)");
        e = hipHostGetDevicePointer(&d, h, 0);
        if (e != hipSuccess) return fail_hip(e, "hipHostGetDevicePointer");
        r.host = (char *)h;
        r.dev = (char *)d;
        r.cap = RING_BYTES;
        if (descriptors_in_device_memory()) {
            void *m = nullptr;
            e = hipMalloc(&m, RING_BYTES);
            if (e != hipSuccess) return fail_hip(e, "hipMalloc(descriptor ring mirror)");
            r.mirror = (char *)m;
        }
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
    *out = Lease{&r, b, en, r.host + b, (r.mirror ? r.mirror : r.dev) + b};
    return PBKV_OK;
}

// Make what the host wrote into the lease visible at lease.dev: nothing to do when the kernels
// read the pinned ring through its mapped address, one small copy on the stream when they read
// the device-memory mirror.
int ring_commit(const Lease &l, size_t bytes, hipStream_t s) {
    if (!l.ring->mirror || bytes == 0) return PBKV_OK;
    hipError_t e = hipMemcpyAsync(l.dev, l.host, bytes, hipMemcpyHostToDevice, s);
    return e == hipSuccess ? PBKV_OK : fail_hip(e, "hipMemcpyAsync(descriptors)");
}

// Record "the kernels reading this lease are enqueued" on the stream.
int ring_release(const Lease &l, hipStream_t s) {
    Ring &r = *l.ring;
    std::lock_guard<std::mutex> lk(r.mu);
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

// Device scratch of the decode kernels (partials of the context slices): one buffer per device,
// grown on demand and kept until the process ends.  Calls that use it must not overlap on
// different streams of one device.
int decode_scratch(size_t bytes, float **out) {
    static std::mutex mu;
    static std::vector<std::pair<void *, size_t>> per_device;
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return fail_hip(e, "hipGetDevice");
    std::lock_guard<std::mutex> lock(mu);
    if ((int)per_device.size() <= dev) per_device.resize(dev + 1, {nullptr, 0});
    auto &slot = per_device[dev];
    if (slot.second < bytes) {
        if (slot.first) {
            if ((e = hipDeviceSynchronize()) != hipSuccess) return fail_hip(e, "hipDeviceSynchronize");
            (void)hipFree(slot.first);
            slot = {nullptr, 0};
        }
        const size_t cap = std::max(bytes + bytes / 2, (size_t)4 << 20);
        void *ptr = nullptr;
        if ((e = hipMalloc(&ptr, cap)) != hipSuccess) return fail_hip(e, "hipMalloc (decode scratch)");
        slot = {ptr, cap};
    }
    *out = (float *)slot.first;
    return PBKV_OK;
}

constexpr int MI355X_CUS = 256;

// Work list of the attention kernels: one tile per block of T suffix tokens of a request,
// longest (most visible keys) first; `pad` keeps the tile's index in request order.  A tile becomes
// wgs_per_tile consecutive work-groups; resident_pairs_wgs > 0 names the number of work-groups the
// chip holds at once when it holds two per CU (see below), 0 switches that case off.
int build_tiles(const pbkv_shape *s, const int32_t *prefix_lens, const int32_t *new_lens, int T,
                std::vector<pbkv::TileDesc> *out, int wgs_per_tile = 1, int resident_pairs_wgs = 0) {
    std::vector<pbkv::TileDesc> &tiles = *out;
    int64_t row0 = 0;
    for (int r = 0; r < s->batch; r++) {
        for (int t0 = 0; t0 < new_lens[r]; t0 += T) {
            const int64_t idx = (int64_t)tiles.size();
            tiles.push_back(pbkv::TileDesc{r, t0, prefix_lens[r], new_lens[r], row0, idx});
        }
        row0 += new_lens[r];
    }
    std::stable_sort(tiles.begin(), tiles.end(), [T](const pbkv::TileDesc &a, const pbkv::TileDesc &b) {
        const int64_t ka = (int64_t)a.prefix_len + std::min(a.tok0 + T, a.new_len);
        const int64_t kb = (int64_t)b.prefix_len + std::min(b.tok0 + T, b.new_len);
        return ka > kb;
    });
    // Longest-first is the right order when work-groups queue for the CUs.  A launch whose
    // work-groups are all resident at once, two per CU (the 4-wave shape on 256 CUs), finishes when
    // the CU with the most work does, and the dispatcher hands out one work-group per CU before it
    // starts on the second: the second half then runs shortest-first, so that the CU holding the
    // longest work-group also gets the shortest (measured +2 % on the benchmark workload's attention
    // launch running alone; no difference with the append kernel beside it).
    const size_t n = tiles.size();
    if (resident_pairs_wgs > 0 && n * (size_t)wgs_per_tile > (size_t)resident_pairs_wgs / 2 &&
        n * (size_t)wgs_per_tile <= (size_t)resident_pairs_wgs)
        std::reverse(tiles.begin() + (resident_pairs_wgs / 2 + wgs_per_tile - 1) / wgs_per_tile, tiles.end());
    if (tiles.size() > (size_t)INT32_MAX / 64) return fail(PBKV_ERR_LIMIT, "too many tiles");
    return PBKV_OK;
}

}  // namespace

extern "C" {

const char *pbkv_last_error(void) { return g_err; }

const char *pbkv_version(void) { return "pbkv 0.1 gfx950"; }

int64_t pbkv_page_bytes(const pbkv_shape *s) {
    if (!s || check_shape(s, false) != PBKV_OK) return 0;
    return (int64_t)2 * s->num_kv_heads * s->page_size * s->head_dim * elt_bytes(s->dtype);
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

    const int G = s->num_q_heads / s->num_kv_heads;
    const int waves = s->dtype == PBKV_BF16 ? pbkv::attn_bf16_waves(prefix_lens, new_lens, s->batch) : 0;
    const int T = s->dtype == PBKV_BF16 ? pbkv::attn_bf16_tile_tokens(s->head_dim, G, waves) : pbkv::attn_f32_tile_tokens();
    std::vector<pbkv::TileDesc> tiles;
    const int per_tile = s->dtype == PBKV_BF16 ? pbkv::attn_bf16_units_per_tile(s->num_kv_heads, G) : 1;
    if ((rc = build_tiles(s, prefix_lens, new_lens, T, &tiles, per_tile, waves == 4 ? 2 * MI355X_CUS : 0))) return rc;

    Lease lease;
    if ((rc = ring_acquire(tiles.size() * sizeof(pbkv::TileDesc), &lease))) return rc;
    memcpy(lease.host, tiles.data(), tiles.size() * sizeof(pbkv::TileDesc));

    pbkv::AttnParams p;
    p.q = q; p.k_new = k_new; p.v_new = v_new; p.kv_pool = kv_pool; p.out = out;
    p.block_table = block_table;
    p.tiles = (const pbkv::TileDesc *)lease.dev;
    p.n_tiles = (int32_t)tiles.size();
    p.Hq = s->num_q_heads; p.Hkv = s->num_kv_heads;
    p.max_pages = s->max_pages_per_req; p.num_pages = s->num_pages;
    p.waves = waves;
    p.trace = nullptr;
    hipStream_t st = (hipStream_t)stream;
    if ((rc = ring_commit(lease, tiles.size() * sizeof(pbkv::TileDesc), st))) return rc;
    hipError_t e = s->dtype == PBKV_BF16 ? pbkv::launch_attn_bf16(p, s->head_dim, st)
                                         : pbkv::launch_attn_f32(p, s->head_dim, st);
    int rel = ring_release(lease, st);
    if (e != hipSuccess) return fail_hip(e, "attention launch");
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
    std::vector<pbkv::TileDesc> tiles;
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

    Lease lease;
    if ((rc = ring_acquire(tiles.size() * sizeof(pbkv::TileDesc), &lease))) return rc;
    memcpy(lease.host, tiles.data(), tiles.size() * sizeof(pbkv::TileDesc));
    pbkv::AttnParams p;
    p.q = nullptr; p.k_new = k_new; p.v_new = v_new; p.kv_pool = kv_pool; p.out = unit_xor;
    p.block_table = block_table;
    p.tiles = (const pbkv::TileDesc *)lease.dev;
    p.n_tiles = (int32_t)tiles.size();
    p.Hq = s->num_q_heads; p.Hkv = s->num_kv_heads;
    p.max_pages = s->max_pages_per_req; p.num_pages = s->num_pages;
    p.waves = waves;
    p.trace = nullptr;
    hipStream_t st = (hipStream_t)stream;
    if ((rc = ring_commit(lease, tiles.size() * sizeof(pbkv::TileDesc), st))) return rc;
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

    const int P = s->page_size;
    std::vector<pbkv::AppendDesc> descs;
    int64_t row0 = 0;
    for (int r = 0; r < s->batch; r++) {
        const int64_t p = prefix_lens[r], n = new_lens[r];
        for (int64_t t = 0; t < n;) {
            const int64_t pos = p + t;
            const int slot0 = (int)(pos % P);
            const int count = (int)std::min<int64_t>(P - slot0, n - t);
            descs.push_back(pbkv::AppendDesc{row0 + t, r, (int32_t)(pos / P), slot0, count, 0});
            t += count;
        }
        row0 += n;
    }
    Lease lease;
    if ((rc = ring_acquire(descs.size() * sizeof(pbkv::AppendDesc), &lease))) return rc;
    memcpy(lease.host, descs.data(), descs.size() * sizeof(pbkv::AppendDesc));
    pbkv::AppendParams p;
    p.k_new = k_new; p.v_new = v_new; p.kv_pool = kv_pool; p.block_table = block_table;
    p.descs = (const pbkv::AppendDesc *)lease.dev;
    p.n_descs = (int32_t)descs.size();
    p.Hkv = s->num_kv_heads; p.max_pages = s->max_pages_per_req; p.num_pages = s->num_pages;
    hipStream_t st = (hipStream_t)stream;
    if ((rc = ring_commit(lease, descs.size() * sizeof(pbkv::AppendDesc), st))) return rc;
    hipError_t e = pbkv::launch_append(p, s->head_dim, elt_bytes(s->dtype), st);
    int rel = ring_release(lease, st);
    if (e != hipSuccess) return fail_hip(e, "append launch");
    return rel;
}

int pbkv_swap_in_pages(const pbkv_shape *s, const void *host_pages, const int32_t *page_ids,
                       int32_t n_pages, void *kv_pool, void *stream) {
    g_err[0] = 0;
    int rc = check_shape(s, false);
    if (rc) return rc;
    if (n_pages < 0) return fail(PBKV_ERR_RANGE, "n_pages %d", n_pages);
    if (n_pages == 0) return PBKV_OK;
    if (!host_pages || !page_ids || !kv_pool) return fail(PBKV_ERR_NULL, "pbkv_swap_in_pages: NULL argument");
    std::vector<uint8_t> seen((size_t)s->num_pages, 0);
    for (int i = 0; i < n_pages; i++) {
        const int32_t id = page_ids[i];
        if (id < 0 || id >= s->num_pages)
            return fail(PBKV_ERR_RANGE, "page_ids[%d] = %d outside pool of %d pages", i, id, s->num_pages);
        if (seen[id]) return fail(PBKV_ERR_ALIAS, "page_ids[%d] = %d appears twice", i, id);
        seen[id] = 1;
    }
    if ((rc = check_aligned(host_pages, "host_pages")) || (rc = check_aligned(kv_pool, "kv_pool"))) return rc;
    const void *host_dev = nullptr;
    if ((rc = check_pinned_ptr(host_pages, "host_pages", &host_dev))) return rc;
    if ((rc = check_device_ptr(kv_pool, "kv_pool"))) return rc;

    Lease lease;
    if ((rc = ring_acquire((size_t)n_pages * sizeof(int32_t), &lease))) return rc;
    memcpy(lease.host, page_ids, (size_t)n_pages * sizeof(int32_t));
    hipStream_t st = (hipStream_t)stream;
    if ((rc = ring_commit(lease, (size_t)n_pages * sizeof(int32_t), st))) return rc;
    hipError_t e = pbkv::launch_swap_in(host_dev, (const int32_t *)lease.dev, n_pages, kv_pool,
                                        pbkv_page_bytes(s), st);
    int rel = ring_release(lease, st);
    if (e != hipSuccess) return fail_hip(e, "swap-in launch");
    return rel;
}

int pbkv_paged_decode(const pbkv_shape *s, const void *q, const void *kv_pool, const int32_t *block_table,
                      const int32_t *context_lens, void *out, void *stream) {
    g_err[0] = 0;
    int rc = check_shape(s, true);
    if (rc) return rc;
    if (s->dtype != PBKV_BF16) return fail(PBKV_ERR_DTYPE, "pbkv_paged_decode: bf16 only");
    if (s->batch == 0) return PBKV_OK;
    if (!q || !kv_pool || !block_table || !context_lens || !out)
        return fail(PBKV_ERR_NULL, "pbkv_paged_decode: NULL argument");
    const int B = s->batch, P = s->page_size;
    int64_t total_pages = 0;
    for (int r = 0; r < B; r++) {
        const int64_t L = context_lens[r];
        if (L < 0 || L > INT32_MAX - 4096) return fail(PBKV_ERR_RANGE, "request %d: context length %lld", r, (long long)L);
        const int64_t pages = (L + P - 1) / P;
        if (pages > s->max_pages_per_req)
            return fail(PBKV_ERR_RANGE, "request %d needs %lld pages, block_table rows hold %d", r, (long long)pages,
                        s->max_pages_per_req);
        total_pages += pages;
    }
    if ((rc = check_aligned(q, "q")) || (rc = check_aligned(kv_pool, "kv_pool")) || (rc = check_aligned(out, "out"))) return rc;
    if ((rc = check_device_ptr(q, "q")) || (rc = check_device_ptr(kv_pool, "kv_pool")) ||
        (rc = check_device_ptr(block_table, "block_table")) || (rc = check_device_ptr(out, "out")))
        return rc;

    // slices: enough work-groups to fill the chip a few times over, at least 16 pages each
    const int G = s->num_q_heads / s->num_kv_heads;
    const int per_unit = s->num_kv_heads * (G / pbkv::decode_heads_per_group(G));   // work-groups per slice
    static const int64_t target_wgs = [] { const char *e = getenv("PBKV_DECODE_WGS"); return e && atoi(e) > 0 ? (int64_t)atoi(e) : (int64_t)2048; }();
    int64_t pps = (total_pages * per_unit + target_wgs - 1) / target_wgs;
    pps = std::max<int64_t>(16, (pps + 3) & ~(int64_t)3);
    std::vector<pbkv::DecodeUnit> units;
    std::vector<pbkv::DecodeReq> reqs((size_t)B);
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

    hipStream_t st = (hipStream_t)stream;
    float *scratch = nullptr;
    const size_t need = std::max<size_t>(units.size(), 1) * per_unit * pbkv::decode_partial_floats(s->head_dim, G) * sizeof(float);
    if ((rc = decode_scratch(need, &scratch))) return rc;

    Lease lease;
    const size_t ub = units.size() * sizeof(pbkv::DecodeUnit), rb = reqs.size() * sizeof(pbkv::DecodeReq);
    if ((rc = ring_acquire(ub + rb, &lease))) return rc;
    memcpy(lease.host, units.data(), ub);
    memcpy((char *)lease.host + ub, reqs.data(), rb);
    if ((rc = ring_commit(lease, ub + rb, st))) return rc;
    pbkv::DecodeParams p;
    p.q = q; p.kv_pool = kv_pool; p.out = out; p.block_table = block_table;
    p.units = (const pbkv::DecodeUnit *)lease.dev;
    p.reqs = (const pbkv::DecodeReq *)((const char *)lease.dev + ub);
    p.scratch = scratch;
    p.n_units = (int32_t)units.size(); p.n_reqs = B;
    p.Hq = s->num_q_heads; p.Hkv = s->num_kv_heads;
    p.max_pages = s->max_pages_per_req; p.num_pages = s->num_pages;
    hipError_t e = pbkv::launch_decode_bf16(p, s->head_dim, st);
    int rel = ring_release(lease, st);
    if (e != hipSuccess) return fail_hip(e, "decode launch");
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
    for (int i = 0; i < n_pages; i++) {
        const int32_t id = page_ids[i];
        if (id < 0 || id >= s->num_pages)
            return fail(PBKV_ERR_RANGE, "page_ids[%d] = %d outside pool of %d pages", i, id, s->num_pages);
    }
    if ((rc = check_aligned(host_pages, "host_pages")) || (rc = check_aligned(kv_pool, "kv_pool"))) return rc;
    const void *host_dev = nullptr;
    if ((rc = check_pinned_ptr(host_pages, "host_pages", &host_dev))) return rc;
    if ((rc = check_device_ptr(kv_pool, "kv_pool"))) return rc;

    Lease lease;
    if ((rc = ring_acquire((size_t)n_pages * sizeof(int32_t), &lease))) return rc;
    memcpy(lease.host, page_ids, (size_t)n_pages * sizeof(int32_t));
    hipStream_t st = (hipStream_t)stream;
    if ((rc = ring_commit(lease, (size_t)n_pages * sizeof(int32_t), st))) return rc;
    hipError_t e = pbkv::launch_swap_out(kv_pool, (const int32_t *)lease.dev, n_pages, (void *)host_dev,
                                         pbkv_page_bytes(s), st);
    int rel = ring_release(lease, st);
    if (e != hipSuccess) return fail_hip(e, "swap-out launch");
    return rel;
}

}  // extern "C"
