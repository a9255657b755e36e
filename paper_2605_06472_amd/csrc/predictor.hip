// Forward pass of the workflow predictor (App. B) for gfx950.
//
// prepare (once per set of weights)
//   predictor_tables_kernel   H^(2) by the two GraphSAGE layers, the |V| x |V| table
//                             S[v][u] = (W_q H2[v]) . H2[u] / sqrt(d) of attention scores between
//                             agents, transposed head weights: everything request-independent
//   predictor_split_kernel    W_t = hi + lo, two bf16 matrices (16 significand bits together), stored in
//                             the order the projection's MFMA operands are read
// forward (per batch)
//   predictor_project_kernel  W_t x on the matrix cores: work-group = 32 requests x one slice of
//                             d_x, operands straight from global memory into the MFMA registers
//                             (x is row-major along d_x, which is the MFMA's k direction), the waves
//                             split the slice, partial sums to the workspace
//   predictor_head_kernel     eight requests per work-group: h_txt = ReLU(sum of the slices), h_cur,
//                             the history attention by table look-up, the two head layers, K softmaxes
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <math.h>

#include "../../include/pbkv.h"
#include "../../include/pbkv_predictor.h"
#include "pbkv_internal.h"

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;

constexpr int KS_MAX = 16;          // most slices of d_x a batch is split into
constexpr int TARGET_WGS = 256;     // projection work-groups aimed for (one per CU)

int64_t align256(int64_t v) { return (v + 255) & ~(int64_t)255; }

// Workspace layout (byte offsets, each 256-byte aligned).
struct Layout {
    int64_t h2, s, wat, ba, wbt, bb, ah1, h1, ah2, q, wp, partial, total;
    int bpad;
};

Layout layout(const pbkv_predictor_shape *p, int32_t max_batch) {
    const int64_t V = p->num_agents, d = p->d, hid = p->hidden, kv1 = (int64_t)p->horizon * (V + 1);
    Layout L;
    int64_t o = 0;
    auto take = [&](int64_t bytes) { int64_t at = o; o = align256(o + bytes); return at; };
    L.h2 = take(V * d * 4);
    L.s = take(V * V * 4);
    L.wat = take(3 * d * hid * 4);
    L.ba = take(hid * 4);
    L.wbt = take(hid * kv1 * 4);
    L.bb = take(kv1 * 4);
    L.ah1 = take(V * d * 4);      // intermediates of the table kernel, each written once
    L.h1 = take(V * d * 4);
    L.ah2 = take(V * d * 4);
    L.q = take(V * d * 4);
    L.wp = take(2 * d * (int64_t)p->d_x * 2);      // W_t as hi + lo bf16 in operand order
    L.bpad = (max_batch + 31) / 32 * 32;
    L.partial = take((int64_t)KS_MAX * L.bpad * d * 4);
    L.total = o;
    return L;
}

int check_shape(const pbkv_predictor_shape *p) {
    if (!p) return pbkv::set_error(PBKV_ERR_NULL, "predictor shape is NULL");
    if (p->num_agents < 1 || p->num_agents > 64) return pbkv::set_error(PBKV_ERR_SHAPE, "num_agents %d not in [1, 64]", p->num_agents);
    if (p->d != 32 && p->d != 64 && p->d != 128) return pbkv::set_error(PBKV_ERR_SHAPE, "d %d is not 32, 64 or 128", p->d);
    if (p->d_x < 64 || p->d_x % 16) return pbkv::set_error(PBKV_ERR_SHAPE, "d_x %d is not a multiple of 16 >= 64", p->d_x);
    if (p->hidden < 1 || p->hidden > 256) return pbkv::set_error(PBKV_ERR_SHAPE, "hidden %d not in [1, 256]", p->hidden);
    if (p->horizon < 1 || p->horizon > 8) return pbkv::set_error(PBKV_ERR_SHAPE, "horizon %d not in [1, 8]", p->horizon);
    if (p->max_prefix < 0 || p->max_prefix > 64) return pbkv::set_error(PBKV_ERR_SHAPE, "max_prefix %d not in [0, 64]", p->max_prefix);
    return PBKV_OK;
}

int check_dev(const void *ptr, const char *name, int align) {
    if (!ptr) return pbkv::set_error(PBKV_ERR_NULL, "%s is NULL", name);
    if ((uintptr_t)ptr & (uintptr_t)(align - 1)) return pbkv::set_error(PBKV_ERR_SHAPE, "%s is not %d-byte aligned", name, align);
    hipPointerAttribute_t a;
    hipError_t e = hipPointerGetAttributes(&a, ptr);
    if (e != hipSuccess) {
        (void)hipGetLastError();
        return pbkv::set_error(PBKV_ERR_DEVICE, "%s: not a device pointer (%s)", name, hipGetErrorString(e));
    }
    if (a.type != hipMemoryTypeDevice && a.type != hipMemoryTypeManaged)
        return pbkv::set_error(PBKV_ERR_DEVICE, "%s: expected device memory", name);
    return PBKV_OK;
}

struct TablesParams {
    const float *emb, *trans, *w1, *w2, *wq, *wa, *ba, *wb, *bb;
    float *h2, *s, *wat, *ba_out, *wbt, *bb_out, *ah1, *h1, *ah2, *q;
    int V, d, hidden, kv1;
};

// One work-group.  Phases are separated by barriers; every intermediate array is written in one
// phase and only read in later ones.
__global__ __launch_bounds__(256) void predictor_tables_kernel(TablesParams p) {
    const int t = threadIdx.x, V = p.V, d = p.d;
    // A H for a [V][d] matrix H
    auto propagate = [&](const float *H, float *AH) {
        for (int e = t; e < V * d; e += 256) {
            const int v = e / d, f = e % d;
            float acc = 0.f;
            for (int u = 0; u < V; u++) acc = fmaf(p.trans[v * V + u], H[u * d + f], acc);
            AH[e] = acc;
        }
    };
    // ReLU([H || AH] W^T), W [d][2d]   (GraphSAGE equation, App. B)
    auto layer = [&](const float *H, const float *AH, const float *Wm, float *out) {
        for (int e = t; e < V * d; e += 256) {
            const int v = e / d, g = e % d;
            float acc = 0.f;
            for (int c = 0; c < d; c++) acc = fmaf(Wm[g * 2 * d + c], H[v * d + c], acc);
            for (int c = 0; c < d; c++) acc = fmaf(Wm[g * 2 * d + d + c], AH[v * d + c], acc);
            out[e] = fmaxf(acc, 0.f);
        }
    };
    propagate(p.emb, p.ah1);
    __syncthreads();
    layer(p.emb, p.ah1, p.w1, p.h1);
    __syncthreads();
    propagate(p.h1, p.ah2);
    __syncthreads();
    layer(p.h1, p.ah2, p.w2, p.h2);
    __syncthreads();
    // queries W_q H2[v] of every agent (history-attention equation, App. B)
    for (int e = t; e < V * d; e += 256) {
        const int v = e / d, g = e % d;
        float acc = 0.f;
        for (int c = 0; c < d; c++) acc = fmaf(p.wq[g * d + c], p.h2[v * d + c], acc);
        p.q[e] = acc;
    }
    __syncthreads();
    const float inv_sqrt_d = 1.0f / sqrtf((float)d);
    for (int e = t; e < V * V; e += 256) {
        const int v = e / V, u = e % V;
        float acc = 0.f;
        for (int g = 0; g < d; g++) acc = fmaf(p.q[v * d + g], p.h2[u * d + g], acc);
        p.s[e] = acc * inv_sqrt_d;
    }
    // head weights: W_a as it is, W_b transposed so that consecutive lanes read consecutive words
    for (int e = t; e < 3 * d * p.hidden; e += 256) p.wat[e] = p.wa[e];
    for (int e = t; e < p.hidden * p.kv1; e += 256) {
        const int j = e / p.kv1, o = e % p.kv1;
        p.wbt[e] = p.wb[o * p.hidden + j];
    }
    for (int e = t; e < p.hidden; e += 256) p.ba_out[e] = p.ba[e];
    for (int e = t; e < p.kv1; e += 256) p.bb_out[e] = p.bb[e];
}

// W_t in the order the projection reads it.  w = hi + lo with hi = bf16(w), lo = bf16(w - hi): the
// sum is w to 2^-17 relative.  For k-step s (16 columns of d_x) and feature block cb (32 rows) the
// 64 lanes' hi operands are 1 KiB contiguous, then the 64 lo operands:
//   wp[(((s * DB + cb) * 2 + part) * 64 + lane) * 8 + e] = part(W_t[32 cb + lane % 32][16 s + 8 (lane / 32) + e])
__global__ __launch_bounds__(256) void predictor_split_kernel(const float *w, __bf16 *wp, int d, int d_x) {
    const int DB = d / 32, ksteps = d_x / 16;
    const int64_t n = (int64_t)ksteps * DB * 64;
    for (int64_t i = blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256) {
        const int lane = (int)(i % 64), cb = (int)(i / 64 % DB), st = (int)(i / 64 / DB);
        const float *src = w + (int64_t)(32 * cb + lane % 32) * d_x + 16 * st + 8 * (lane / 32);
        bf16x8 hi, lo;
#pragma unroll
        for (int e = 0; e < 8; e++) {
            const float v = src[e];
            hi[e] = (__bf16)v;
            lo[e] = (__bf16)(v - (float)hi[e]);
        }
        bf16x8 *dst = (bf16x8 *)wp + ((int64_t)(st * DB + cb) * 2) * 64 + lane;
        dst[0] = hi;
        dst[64] = lo;
    }
}

struct ProjectParams {
    const __bf16 *x, *wp;
    float *partial;
    int batch, bpad, d_x, steps_per_slice, ksteps;
};

// Work-group (rb, slice): requests 32*rb .. +31, k-steps [slice*sps, (slice+1)*sps) of 16 columns
// of d_x each, handed to the waves in groups of a few consecutive k-steps.  out^T = W_t x^T: the A operand is a 32 x 16 block of W_t (rows = features), read
// from the prepared operand-order copy (1 KiB contiguous per wave load); the B operand is a 16 x 32
// block of x^T (columns = requests): lane (i = l%32, h = l/32) holds the 8 consecutive d_x entries
// 8h .. 8h+7 of row i, one 16-byte load from the row-major x.  The kernel is bound by memory
// latency, so a wave issues all loads of a group before its first MFMA; the waves' sums meet in
// LDS by a binary tree.
template <int DB, int NW>     // d / 32, waves per work-group
__global__ __launch_bounds__(64 * NW) void predictor_project_kernel(ProjectParams p) {
#if defined(__HIP_DEVICE_COMPILE__)
    constexpr int D = 32 * DB;
    constexpr int CH = DB == 4 ? 3 : 5;                   // consecutive k-steps per group: all their operands are held at once
    __shared__ float red[NW / 2][32][D + 4];
    const int l = threadIdx.x & 63, li = l & 31, lh = l >> 5;
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int rb = blockIdx.x, slice = blockIdx.y;
    const int s0 = slice * p.steps_per_slice;
    const int s1 = min(s0 + p.steps_per_slice, p.ksteps);
    const int row = rb * 32 + li;
    const bool valid = row < p.batch;
    const __bf16 *xp = p.x + (int64_t)(valid ? row : 0) * p.d_x + 8 * lh;
    const bf16x8 *wp = (const bf16x8 *)p.wp + l;
    f32x16 acc[DB];
#pragma unroll
    for (int cb = 0; cb < DB; cb++)
#pragma unroll
        for (int r = 0; r < 16; r++) acc[cb][r] = 0.f;
    bf16x8 zero;
#pragma unroll
    for (int e = 0; e < 8; e++) zero[e] = (__bf16)0.f;
    for (int base = s0 + CH * w; base < s1; base += CH * NW) {
        bf16x8 xo[CH], ho[CH][DB], lo[CH][DB];
#pragma unroll
        for (int c = 0; c < CH; c++) {
            const int sc = base + c < s1 ? base + c : base;   // past the slice: a valid address, operand zeroed below
            xo[c] = *(const bf16x8 *)(xp + sc * 16);
#pragma unroll
            for (int cb = 0; cb < DB; cb++) {
                ho[c][cb] = wp[((int64_t)(sc * DB + cb) * 2) * 64];
                lo[c][cb] = wp[((int64_t)(sc * DB + cb) * 2 + 1) * 64];
            }
        }
#pragma unroll
        for (int c = 0; c < CH; c++) {
            const bool on = valid && base + c < s1;
            const bf16x8 xb = on ? xo[c] : zero;
#pragma unroll
            for (int cb = 0; cb < DB; cb++) {
                acc[cb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ho[c][cb], xb, acc[cb], 0, 0, 0);
                acc[cb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(lo[c][cb], xb, acc[cb], 0, 0, 0);
            }
        }
    }
    // register r of lane (li, lh) is feature 32*cb + 8*(r/4) + 4*lh + r%4 of request li
    for (int half = NW / 2; half >= 1; half >>= 1) {
        if (w >= half && w < 2 * half) {
#pragma unroll
            for (int cb = 0; cb < DB; cb++)
#pragma unroll
                for (int g = 0; g < 4; g++) {
                    f32x4 v;
#pragma unroll
                    for (int c = 0; c < 4; c++) v[c] = acc[cb][4 * g + c];
                    *(f32x4 *)&red[w - half][li][32 * cb + 8 * g + 4 * lh] = v;
                }
        }
        __syncthreads();
        if (w < half) {
#pragma unroll
            for (int cb = 0; cb < DB; cb++)
#pragma unroll
                for (int g = 0; g < 4; g++) {
                    const f32x4 v = *(const f32x4 *)&red[w][li][32 * cb + 8 * g + 4 * lh];
#pragma unroll
                    for (int c = 0; c < 4; c++) acc[cb][4 * g + c] += v[c];
                }
        }
        __syncthreads();
    }
    if (w == 0) {
        float *out = p.partial + ((int64_t)slice * p.bpad + row) * D;
#pragma unroll
        for (int cb = 0; cb < DB; cb++)
#pragma unroll
            for (int g = 0; g < 4; g++) {
                f32x4 v;
#pragma unroll
                for (int c = 0; c < 4; c++) v[c] = acc[cb][4 * g + c];
                *(f32x4 *)(out + 32 * cb + 8 * g + 4 * lh) = v;
            }
    }
#endif
}

struct HeadParams {
    const float *partial, *h2, *s, *wat, *ba, *wbt, *bb;
    const int32_t *cur_agent, *prefix, *prefix_len;
    float *probs;
    int batch, bpad, n_slices, V, d, hidden, K, L;
};

__device__ inline float wave_max(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
    return v;
}
__device__ inline float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}

constexpr int RPB = 8;              // requests per work-group of the head kernel
constexpr int WBUF1 = 12544;        // most floats of W_a staged in LDS at a time (all of it at d = hidden = 64: 64 rows of 192 + 4)
constexpr int WBUF2 = 1728;         // floats of W_b^T staged at a time (all of it at hidden = 64, K (|V|+1) = 27)

// LDS of the head kernel, in floats (dynamic: it grows with |V| d and exceeds 64 KiB for large shapes).
struct HeadLds {
    int w1, w1_size, w2, zl, ha, h2, s, bias, ints, total;
};
__host__ __device__ inline HeadLds head_lds(int V, int d, int hidden, int kv1) {
    HeadLds o;
    int at = 0;
    auto take = [&](int n) { int r = at; at += (n + 3) & ~3; return r; };
    const int after = RPB * kv1 + RPB * hidden;           // logits and hidden activations reuse z's place
    o.w2 = take(WBUF2);
    o.zl = take(RPB * 3 * d > after ? RPB * 3 * d : after);
    o.ha = take(4 * RPB * (hidden > 32 ? hidden : 32));   // alpha [RPB][64] + prefix agents [RPB][64], later the waves' partial sums [4][RPB][hidden]
    o.h2 = take(V * d);
    o.s = take(V * V);
    o.bias = take(hidden + kv1);
    o.ints = take(2 * RPB);
    // the rest of the 160 KiB, up to WBUF1, holds rows of W_a (the largest shape leaves room for 29 of them)
    const int room = 160 * 1024 / 4 - at;
    o.w1_size = (room < WBUF1 ? room : WBUF1) & ~3;
    o.w1 = take(o.w1_size);
    o.total = at;
    return o;
}

constexpr int HNT = 1024;           // threads of a head work-group: 16 waves, four per SIMD

// Staging through registers: every load of a work-group's first phase is issued before the first
// LDS store, so the phase costs one memory round trip and not one per array.  src is 16-byte aligned
// and n <= 4 HNT N.
template <int N>
struct Staged {
    f32x4 v[N];
    float tail;
};
template <int N>
__device__ inline void stage_load(Staged<N> &st, const float *src, int n, int t) {
    const int n4 = n >> 2;
#pragma unroll
    for (int k = 0; k < N; k++) {
        const int e = t + HNT * k;
        st.v[k] = e < n4 ? ((const f32x4 *)src)[e] : f32x4{0.f, 0.f, 0.f, 0.f};
    }
    st.tail = 4 * n4 + t < n ? src[4 * n4 + t] : 0.f;
}
template <int N>
__device__ inline void stage_store(const Staged<N> &st, float *dst, int n, int t) {
    const int n4 = n >> 2;
#pragma unroll
    for (int k = 0; k < N; k++) {
        const int e = t + HNT * k;
        if (e < n4) ((f32x4 *)dst)[e] = st.v[k];
    }
    if (4 * n4 + t < n) dst[4 * n4 + t] = st.tail;
}

// the same for rows of `len` floats (a multiple of 4) that land `pitch` floats apart
template <int N>
__device__ inline void stage_store_rows(const Staged<N> &st, float *dst, int n, int len, int pitch, int t) {
    const int n4 = n >> 2, len4 = len >> 2;
#pragma unroll
    for (int k = 0; k < N; k++) {
        const int e = t + HNT * k;
        if (e < n4) *(f32x4 *)&dst[(e / len4) * pitch + 4 * (e % len4)] = st.v[k];
    }
}
__device__ inline void stage_rows(float *dst, const float *src, int rows, int len, int pitch, int t) {
    const int len4 = len >> 2;
    for (int e = t; e < rows * len4; e += HNT) *(f32x4 *)&dst[(e / len4) * pitch + 4 * (e % len4)] = ((const f32x4 *)src)[e];
}

// 16-byte copies where the source offset allows, single words otherwise (all loads in flight at once)
__device__ inline void stage(float *dst, const float *src, int n, int t) {
    if ((((uintptr_t)src | (uintptr_t)dst) & 15) == 0) {
        const int n4 = n >> 2;
        for (int e = t; e < n4; e += HNT) ((f32x4 *)dst)[e] = ((const f32x4 *)src)[e];
        for (int e = 4 * n4 + t; e < n; e += HNT) dst[e] = src[e];
    } else {
        for (int e = t; e < n; e += HNT) dst[e] = src[e];
    }
}


// Work-group = RPB requests, 1024 threads.  The work per request is tiny; what the kernel costs is
// the issue time of its instructions and the latency of its dependent steps.  So every step is
// spread over sixteen waves (four per SIMD, which overlap one another's latencies), and everything
// that comes from global memory and does not depend on another load -- the slices of the
// projection, the indices, the H2 and score tables, the first chunks of both head layers' weights --
// is fetched in the first phase with all loads in flight at once; the later phases work out of LDS.
// A request past the end of the batch is computed as request batch-1 again and stores nothing, so
// that all threads walk the same barriers.
__global__ __launch_bounds__(HNT) void predictor_head_kernel(HeadParams p) {
    extern __shared__ __attribute__((aligned(16))) float lds[];
    const int t = threadIdx.x, l = t & 63, w = t >> 6;
    const int b0 = blockIdx.x * RPB;
    const int V = p.V, d = p.d, d3 = 3 * p.d, hidden = p.hidden, kv1 = p.K * (V + 1);
    const int dsh = d == 32 ? 5 : (d == 64 ? 6 : 7);      // d is 32, 64 or 128
    const HeadLds o = head_lds(V, d, hidden, kv1);
    float *wbuf1 = lds + o.w1, *wbuf2 = lds + o.w2;
    float *z = lds + o.zl;                                // z[r][i], r < RPB, i < 3d
    float *logit = lds + o.zl, *hid = lds + o.zl + RPB * kv1;
    float *alpha = lds + o.ha, *red = lds + o.ha, *h2 = lds + o.h2, *stab = lds + o.s;
    float *ba = lds + o.bias, *bb = lds + o.bias + hidden;
    int *pre = (int *)(lds + o.ha) + RPB * 64, *curs = (int *)(lds + o.ints), *lens = curs + RPB;
    auto request = [&](int r) { return min(b0 + r, p.batch - 1); };
    const int P1 = d3 + 4;                                // LDS pitch of a row of W_a: 16-byte reads of consecutive rows do not collide
    const int rpc1 = o.w1_size / P1;                      // rows (hidden units) of W_a [hidden][3d] per chunk
    const int rpc2 = WBUF2 / kv1;                         // rows of W_b^T [hidden][kv1] per chunk

    // ---- phase 1: every independent global load, all issued before the first LDS store ------------
    int cur_raw = 0, len_raw = 0, pre_raw = 0;
    if (t < RPB) {
        cur_raw = p.cur_agent[request(t)];
        len_raw = p.prefix_len[request(t)];
    }
    if (t < RPB * 64 && (t & 63) < p.L)                   // prefix agents; slots past the row are agent 0
        pre_raw = p.prefix[(int64_t)request(t >> 6) * p.L + (t & 63)];
    // (iii) the slices of the projection: thread t = (request t / d, feature t % d)
    const bool has_part = t < RPB * d;
    float part[KS_MAX];
    {
        const float *src = p.partial + (int64_t)request(has_part ? t >> dsh : 0) * d + (has_part ? t & (d - 1) : 0);
#pragma unroll
        for (int sl = 0; sl < KS_MAX; sl++) part[sl] = has_part && sl < p.n_slices ? src[(int64_t)sl * p.bpad * d] : 0.f;
    }
    Staged<2> st_h2;
    Staged<1> st_s, st_w2, st_ba, st_bb;
    Staged<3> st_w1;
    const int n_w1 = min(rpc1, hidden) * d3, n_w2 = min(rpc2, hidden) * kv1;
    stage_load(st_h2, p.h2, V * d, t);
    stage_load(st_s, p.s, V * V, t);
    stage_load(st_w1, p.wat, n_w1, t);
    stage_load(st_w2, p.wbt, n_w2, t);
    stage_load(st_ba, p.ba, hidden, t);
    stage_load(st_bb, p.bb, kv1, t);
    // ... and now the stores
    if (t < RPB) {
        curs[t] = cur_raw < 0 ? 0 : (cur_raw >= V ? V - 1 : cur_raw);
        lens[t] = len_raw < 0 ? 0 : (len_raw > p.L ? p.L : len_raw);
    }
    if (t < RPB * 64) pre[t] = pre_raw < 0 ? 0 : (pre_raw >= V ? V - 1 : pre_raw);
    if (has_part) {
        float acc = 0.f;
#pragma unroll
        for (int sl = 0; sl < KS_MAX; sl++) acc += part[sl];
        z[(t >> dsh) * d3 + 2 * d + (t & (d - 1))] = fmaxf(acc, 0.f);      // h_txt = ReLU(W_t x)
    }
    stage_store(st_h2, h2, V * d, t);
    stage_store(st_s, stab, V * V, t);
    stage_store_rows(st_w1, wbuf1, n_w1, d3, P1, t);
    stage_store(st_w2, wbuf2, n_w2, t);
    stage_store(st_ba, ba, hidden, t);
    stage_store(st_bb, bb, kv1, t);
    __syncthreads();

    // ---- (i) h_cur = H2[v_t]; (ii) attention over the prefix agents: wave r < RPB serves request r, lane i = position i
    if (has_part) z[(t >> dsh) * d3 + (t & (d - 1))] = h2[curs[t >> dsh] * d + (t & (d - 1))];
    if (w < RPB) {
        const int n = lens[w];
        const float sc = l < n ? stab[curs[w] * V + pre[w * 64 + l]] : -INFINITY;
        const float mx = wave_max(sc);
        const float e = l < n ? expf(sc - mx) : 0.f;
        const float den = wave_sum(e);
        alpha[w * 64 + l] = n > 0 ? e / den : 0.f;        // zero past the prefix: the sum below may overrun it
    }
    __syncthreads();
    if (has_part) {
        const int r = t >> dsh, f = t & (d - 1), n = lens[r];
        float acc = 0.f;
        for (int i = 0; i < n; i += 4) {
            const f32x4 al = *(const f32x4 *)&alpha[r * 64 + i];
            const int4 ag = *(const int4 *)&pre[r * 64 + i];
            const float v0 = h2[ag.x * d + f], v1 = h2[ag.y * d + f], v2 = h2[ag.z * d + f], v3 = h2[ag.w * d + f];
            acc = fmaf(al[0], v0, acc);
            acc = fmaf(al[1], v1, acc);
            acc = fmaf(al[2], v2, acc);
            acc = fmaf(al[3], v3, acc);
        }
        z[r * d3 + d + f] = acc;
    }

    // ---- head layer 1: hidden = ReLU(W_a z + b_a).  Wave w = (g = w % 4, h = w / 4) takes the g-th
    // quarter of the inputs and the requests 2h, 2h+1; lane l the hidden units l, l+64, ..; weights
    // and inputs are read 16 bytes (four inputs) at a time.  The four sums of a (request, unit) meet
    // in LDS.  W_a passes through LDS whole, or in chunks of rows (hidden units) if it is too large.
    const int g = w & 3, hq = w >> 2, qlen = d3 >> 2;     // qlen = 24, 48 or 96 inputs per quarter
    const float *za = z + (2 * hq) * d3 + g * qlen, *zb = za + d3;
    for (int u0 = 0; u0 < hidden; u0 += rpc1) {
        const int nu = min(rpc1, hidden - u0);
        __syncthreads();                                  // z complete / previous chunk consumed
        if (u0 > 0) {
            stage_rows(wbuf1, p.wat + (int64_t)u0 * d3, nu, d3, P1, t);
            __syncthreads();
        }
#pragma unroll
        for (int q = 0; q < 4; q++) {
            const int ul = l + 64 * q;                    // unit inside the chunk
            if (64 * q < nu) {                            // uniform
                const float *wr = wbuf1 + min(ul, nu - 1) * P1 + g * qlen;
                float s0 = 0.f, s1 = 0.f;
                for (int i = 0; i < qlen; i += 12) {      // three 16-byte reads of each operand in flight
                    f32x4 wv[3], a4[3], b4[3];
#pragma unroll
                    for (int k = 0; k < 3; k++) {
                        wv[k] = *(const f32x4 *)&wr[i + 4 * k];
                        a4[k] = *(const f32x4 *)&za[i + 4 * k];
                        b4[k] = *(const f32x4 *)&zb[i + 4 * k];
                    }
#pragma unroll
                    for (int k = 0; k < 3; k++)
#pragma unroll
                        for (int c = 0; c < 4; c++) {
                            s0 = fmaf(wv[k][c], a4[k][c], s0);
                            s1 = fmaf(wv[k][c], b4[k][c], s1);
                        }
                }
                if (ul < nu) {
                    red[(g * RPB + 2 * hq) * hidden + u0 + ul] = s0;
                    red[(g * RPB + 2 * hq + 1) * hidden + u0 + ul] = s1;
                }
            }
        }
    }
    __syncthreads();                                      // the partial sums are complete; z is dead from here on
    // (the logits start from their bias: one thread per (request, output), accumulated in place)
    for (int e = t; e < RPB * kv1; e += HNT) logit[e] = bb[e % kv1];
    for (int e = t; e < RPB * hidden; e += HNT) {
        const int j = e % hidden;
        const float sum = ((red[e] + red[RPB * hidden + e]) + red[2 * RPB * hidden + e]) + red[3 * RPB * hidden + e];
        hid[e] = fmaxf(sum + ba[j], 0.f);
    }
    // ---- head layer 2: logits = W_b hidden + b_b
    for (int j0 = 0; j0 < hidden; j0 += rpc2) {
        const int nrow = min(rpc2, hidden - j0);
        __syncthreads();                                  // hidden complete / previous chunk consumed
        if (j0 > 0) {
            stage(wbuf2, p.wbt + (int64_t)j0 * kv1, nrow * kv1, t);
            __syncthreads();
        }
        for (int e = t; e < RPB * kv1; e += HNT) {
            const int r = e / kv1, oo = e % kv1;
            float acc = logit[e];
#pragma unroll 16
            for (int j = 0; j < nrow; j++) acc = fmaf(wbuf2[j * kv1 + oo], hid[r * hidden + j0 + j], acc);
            logit[e] = acc;
        }
    }
    __syncthreads();
    // ---- one softmax per step over the |V| agents and END
    for (int e = t; e < RPB * kv1; e += HNT) {
        const int r = e / kv1, oo = e % kv1;
        const int k0 = oo / (V + 1) * (V + 1);
        float m = -INFINITY;
#pragma unroll 8
        for (int i = 0; i <= V; i++) m = fmaxf(m, logit[r * kv1 + k0 + i]);
        float sum = 0.f;
#pragma unroll 8
        for (int i = 0; i <= V; i++) sum += expf(logit[r * kv1 + k0 + i] - m);
        if (b0 + r < p.batch) p.probs[(int64_t)(b0 + r) * kv1 + oo] = expf(logit[e] - m) / sum;
    }
}

}  // namespace

extern "C" {

int64_t pbkv_predictor_workspace_bytes(const pbkv_predictor_shape *shape, int32_t max_batch) {
    pbkv::clear_error();
    if (check_shape(shape) != PBKV_OK) return 0;
    if (max_batch < 1) {
        pbkv::set_error(PBKV_ERR_RANGE, "max_batch %d is not positive", max_batch);
        return 0;
    }
    return layout(shape, max_batch).total;
}

int pbkv_predictor_prepare(const pbkv_predictor_shape *shape, const pbkv_predictor_weights *wts,
                           void *workspace, int64_t workspace_bytes, int32_t max_batch, void *stream) {
    pbkv::clear_error();
    if (int rc = check_shape(shape)) return rc;
    if (!wts) return pbkv::set_error(PBKV_ERR_NULL, "weights is NULL");
    if (max_batch < 1) return pbkv::set_error(PBKV_ERR_RANGE, "max_batch %d is not positive", max_batch);
    const Layout L = layout(shape, max_batch);
    if (workspace_bytes < L.total)
        return pbkv::set_error(PBKV_ERR_RANGE, "workspace of %lld bytes, %lld needed", (long long)workspace_bytes, (long long)L.total);
    if (int rc = check_dev(workspace, "workspace", 256)) return rc;
    const struct { const float *p; const char *n; } ptrs[] = {
        {wts->emb, "emb"}, {wts->trans, "trans"}, {wts->w1, "w1"}, {wts->w2, "w2"}, {wts->wq, "wq"},
        {wts->wt, "wt"}, {wts->wa, "wa"}, {wts->ba, "ba"}, {wts->wb, "wb"}, {wts->bb, "bb"}};
    for (const auto &e : ptrs)
        if (int rc = check_dev(e.p, e.n, 16)) return rc;
    char *ws = (char *)workspace;
    hipStream_t s = (hipStream_t)stream;
    TablesParams t;
    t.emb = wts->emb; t.trans = wts->trans; t.w1 = wts->w1; t.w2 = wts->w2; t.wq = wts->wq;
    t.wa = wts->wa; t.ba = wts->ba; t.wb = wts->wb; t.bb = wts->bb;
    t.h2 = (float *)(ws + L.h2); t.s = (float *)(ws + L.s); t.wat = (float *)(ws + L.wat);
    t.ba_out = (float *)(ws + L.ba); t.wbt = (float *)(ws + L.wbt); t.bb_out = (float *)(ws + L.bb);
    t.ah1 = (float *)(ws + L.ah1); t.h1 = (float *)(ws + L.h1); t.ah2 = (float *)(ws + L.ah2); t.q = (float *)(ws + L.q);
    t.V = shape->num_agents; t.d = shape->d; t.hidden = shape->hidden; t.kv1 = shape->horizon * (shape->num_agents + 1);
    hipLaunchKernelGGL(predictor_tables_kernel, dim3(1), dim3(256), 0, s, t);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return pbkv::set_error(PBKV_ERR_DEVICE, "predictor tables launch: %s", hipGetErrorString(e));
    const int64_t n = (int64_t)(shape->d_x / 16) * (shape->d / 32) * 64;
    const unsigned grid = (unsigned)((n + 255) / 256 < 1024 ? (n + 255) / 256 : 1024);
    hipLaunchKernelGGL(predictor_split_kernel, dim3(grid), dim3(256), 0, s, wts->wt, (__bf16 *)(ws + L.wp), shape->d, shape->d_x);
    e = hipGetLastError();
    if (e != hipSuccess) return pbkv::set_error(PBKV_ERR_DEVICE, "predictor split launch: %s", hipGetErrorString(e));
    return PBKV_OK;
}

int pbkv_predictor_forward(const pbkv_predictor_shape *shape, void *workspace, int64_t workspace_bytes,
                           int32_t max_batch, const void *x, const int32_t *cur_agent, const int32_t *prefix,
                           const int32_t *prefix_len, int32_t batch, float *probs, void *stream) {
    pbkv::clear_error();
    if (int rc = check_shape(shape)) return rc;
    if (max_batch < 1) return pbkv::set_error(PBKV_ERR_RANGE, "max_batch %d is not positive", max_batch);
    if (batch < 0 || batch > max_batch) return pbkv::set_error(PBKV_ERR_RANGE, "batch %d not in [0, max_batch = %d]", batch, max_batch);
    const Layout L = layout(shape, max_batch);
    if (workspace_bytes < L.total)
        return pbkv::set_error(PBKV_ERR_RANGE, "workspace of %lld bytes, %lld needed", (long long)workspace_bytes, (long long)L.total);
    if (int rc = check_dev(workspace, "workspace", 256)) return rc;
    if (batch == 0) return PBKV_OK;
    if (int rc = check_dev(x, "x", 16)) return rc;
    if (int rc = check_dev(cur_agent, "cur_agent", 4)) return rc;
    if (int rc = check_dev(prefix_len, "prefix_len", 4)) return rc;
    if (shape->max_prefix > 0)
        if (int rc = check_dev(prefix, "prefix", 4)) return rc;
    if (int rc = check_dev(probs, "probs", 4)) return rc;

    char *ws = (char *)workspace;
    hipStream_t s = (hipStream_t)stream;
    // cut d_x into slices: about one work-group per CU (never more: a CU holds one), a slice being
    // whole rounds of the waves' groups of k-steps
    const int nw = shape->d == 128 ? 4 : 8, ch = shape->d == 128 ? 3 : 5;
    const int ksteps = shape->d_x / 16, rbs = (batch + 31) / 32;
    int ks = (TARGET_WGS + rbs - 1) / rbs;
    ks = ks > KS_MAX ? KS_MAX : ks;
    const int round_steps = ch * nw;
    const int sps = ((ksteps + ks - 1) / ks + round_steps - 1) / round_steps * round_steps;
    ks = (ksteps + sps - 1) / sps;

    ProjectParams pp;
    pp.x = (const __bf16 *)x; pp.wp = (const __bf16 *)(ws + L.wp);
    pp.partial = (float *)(ws + L.partial);
    pp.batch = batch; pp.bpad = L.bpad; pp.d_x = shape->d_x; pp.steps_per_slice = sps; pp.ksteps = ksteps;
    const dim3 grid(rbs, ks);
    switch (shape->d) {
        case 32: hipLaunchKernelGGL((predictor_project_kernel<1, 8>), grid, dim3(512), 0, s, pp); break;
        case 64: hipLaunchKernelGGL((predictor_project_kernel<2, 8>), grid, dim3(512), 0, s, pp); break;
        default: hipLaunchKernelGGL((predictor_project_kernel<4, 4>), grid, dim3(256), 0, s, pp); break;
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return pbkv::set_error(PBKV_ERR_DEVICE, "predictor projection launch: %s", hipGetErrorString(e));

    HeadParams hp;
    hp.partial = pp.partial; hp.h2 = (const float *)(ws + L.h2); hp.s = (const float *)(ws + L.s);
    hp.wat = (const float *)(ws + L.wat); hp.ba = (const float *)(ws + L.ba);
    hp.wbt = (const float *)(ws + L.wbt); hp.bb = (const float *)(ws + L.bb);
    hp.cur_agent = cur_agent; hp.prefix = prefix; hp.prefix_len = prefix_len; hp.probs = probs;
    hp.batch = batch; hp.bpad = L.bpad; hp.n_slices = ks; hp.V = shape->num_agents; hp.d = shape->d;
    hp.hidden = shape->hidden; hp.K = shape->horizon; hp.L = shape->max_prefix;
    const size_t lds_bytes = (size_t)head_lds(hp.V, hp.d, hp.hidden, hp.K * (hp.V + 1)).total * 4;
    if (lds_bytes > 64 * 1024) {      // above the default limit the kernel has to be told (gfx950 has 160 KiB per work-group)
        hipError_t ea = hipFuncSetAttribute((const void *)predictor_head_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
        if (ea != hipSuccess) return pbkv::set_error(PBKV_ERR_DEVICE, "predictor head LDS size %zu: %s", lds_bytes, hipGetErrorString(ea));
    }
    hipLaunchKernelGGL(predictor_head_kernel, dim3((batch + RPB - 1) / RPB), dim3(HNT), lds_bytes, s, hp);
    e = hipGetLastError();
    if (e != hipSuccess) return pbkv::set_error(PBKV_ERR_DEVICE, "predictor head launch: %s", hipGetErrorString(e));
    return PBKV_OK;
}

}  // extern "C"
