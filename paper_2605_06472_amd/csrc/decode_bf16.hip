// Paged decode attention, bf16 (one query row per request over its paged context): the
// pure-decode step behind which prefetch transfers are hidden.  HBM-bound: every K and V row of
// the context is read exactly once, 4 KiB at a time, and nothing else of size moves.
//
// Work decomposition
//   work-group = 4 waves = (request, slice of its pages, KV head, group of <= 8 query heads).
//   A wave takes every fourth page of the slice and keeps the K and V rows of the NEXT page in
//   flight (in registers) while it works on the current one: 8 KiB per wave, 64 per CU, enough
//   outstanding bytes to cover the HBM latency.  No LDS traffic and no barrier inside the loop.
//
//   scores     S[token][head] = K Q^T on the 16x16x32 bf16 MFMA: the A operand (16 tokens x 32 d)
//              is exactly 16 bytes per lane of a row-major K page, so K goes from global memory
//              into the MFMA without any shuffle; the query heads of the GQA group are the columns.
//   softmax    the 16-lane group g owns tokens 4g..4g+3 of the page (that is where the MFMA leaves
//              their scores); one reference maximum per head for the whole wave, moved only when a
//              score exceeds it by 2^8.
//   P V        on the vector ALU: V has d contiguous and the MFMA wants tokens contiguous, and an
//              HBM-bound kernel has the ALU time: lane (g, x) holds 8 d-values of its group's
//              tokens and gets their probabilities by ds_bpermute from the lanes that own them.
//   The four waves merge their partials (reference, row sum, unnormalised output) in LDS at the
//   very end and the work-group writes one partial to a scratch buffer; a small second kernel
//   merges the slices of a request.
#include "pbkv_internal.h"

namespace pbkv {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) unsigned u32x4;

constexpr int DEC_WAVES = 4;
[[maybe_unused]] constexpr int DEC_NBUF = 2;            // page buffers per wave (three were measured: not faster)
[[maybe_unused]] constexpr float DEC_RESCALE_LOG2 = 8.0f;

int decode_heads_per_group(int group) { return group < 8 ? group : 8; }

// floats per partial: [GW][D] output, [GW] reference, [GW] row sum, padded to 16 bytes
int64_t decode_partial_floats(int head_dim, int group) {
    return ((int64_t)decode_heads_per_group(group) * (head_dim + 2) + 3) & ~(int64_t)3;
}

template <int D, int GW>
__global__ __launch_bounds__(64 * DEC_WAVES) __attribute__((amdgpu_waves_per_eu(2, 2)))
void decode_bf16_kernel(DecodeParams p, int G) {
#if defined(__HIP_DEVICE_COMPILE__)
    constexpr int ROWB = D * 2;            // bytes per K/V row
    constexpr int CPR = D / 8;             // 16-byte chunks per row
    constexpr int NJ = D / 32;             // MFMAs (and K loads) per page
    constexpr int RPL = 256 / ROWB;        // V rows one 16-lane group fetches per load
    constexpr int NLV = 4 / RPL;           // V loads per page
    static_assert(RPL == 1 || RPL == 2, "head dim 64 or 128");

    const int l = threadIdx.x & 63;
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int nsplit_g = G / GW;
    int bid = blockIdx.x;
    const int hs = bid % nsplit_g;
    bid /= nsplit_g;
    const int kvh = bid % p.Hkv;
    const DecodeUnit un = p.units[bid / p.Hkv];
    if (p.mirror_units != nullptr && kvh == 0 && hs == 0 && threadIdx.x == 0) p.mirror_units[bid / p.Hkv] = un;
    const int g = l >> 4, c = l & 15;
    const int head0 = kvh * G + hs * GW;

    // Q^T operand of step j: lane (g, c) holds q[head c][32j + 8g .. +7]; columns >= GW are zero
    bf16x8 qB[NJ];
    {
        const __bf16 *qp = (const __bf16 *)p.q + ((int64_t)un.req * p.Hq + head0 + (c < GW ? c : 0)) * D + 8 * g;
#pragma unroll
        for (int j = 0; j < NJ; j++) {
            qB[j] = *(const bf16x8 *)(qp + 32 * j);
            if (c >= GW) {
#pragma unroll
                for (int e = 0; e < 8; e++) qB[j][e] = (__bf16)0.f;
            }
        }
    }
    const float sc = 1.4426950408889634f * rsqrtf((float)D);   // scores in log2 units

    const int64_t page_bytes = 2 * (int64_t)p.Hkv * 16 * ROWB;
    const char *pool_k = (const char *)p.kv_pool + (int64_t)kvh * 16 * ROWB;
    const int64_t v_in_page = (int64_t)p.Hkv * 16 * ROWB;
    const int sub = RPL == 2 ? (c >> 3) : 0;                    // which of the group's two rows (d = 64)
    const int koff = c * ROWB + g * 16;                         // + 64 j
    const int voff = (4 * g + sub) * ROWB + (l % CPR) * 16;     // + i * RPL * ROWB
    const int bp_base = (l & 48) * 4;                           // byte address of lane (g, 0) for ds_bpermute

    // this wave's pages: un.page0 + w, + 4, ...; their ids sit 64 at a time in one register
    const int32_t *bt = p.block_table + (int64_t)un.req * p.max_pages;
    const int n_mine = un.page1 - un.page0 > w ? (un.page1 - un.page0 - w + DEC_WAVES - 1) / DEC_WAVES : 0;
    auto load_ids = [&](int blk) {
        const int k = blk * 64 + l;
        int pg = k < n_mine ? bt[un.page0 + w + DEC_WAVES * k] : 0;
        return pg < 0 ? 0 : (pg >= p.num_pages ? p.num_pages - 1 : pg);
    };
    int ids = load_ids(0);

    struct PageRegs { bf16x8 k[NJ]; u32x4 v[NLV]; };
    auto load_page = [&](int k, PageRegs &r) {
        const int pg = __builtin_amdgcn_readlane(ids, k & 63);
        const char *kb = pool_k + pg * page_bytes;
#pragma unroll
        for (int j = 0; j < NJ; j++) {
            // K and V are read exactly once: streaming loads
            const u32x4 raw = __builtin_nontemporal_load((const u32x4 *)(kb + koff + 64 * j));
            __builtin_memcpy(&r.k[j], &raw, 16);
        }
#pragma unroll
        for (int i = 0; i < NLV; i++) {
            r.v[i] = __builtin_nontemporal_load((const u32x4 *)(kb + v_in_page + voff + i * RPL * ROWB));
        }
    };

    float acc[GW][8];
#pragma unroll
    for (int h = 0; h < GW; h++)
#pragma unroll
        for (int e = 0; e < 8; e++) acc[h][e] = 0.f;
    float M = -INFINITY, lsum = 0.f;       // lane (g, c): reference and partial row sum of head c

    auto compute_page = [&](int k, const PageRegs &r) {
        const int valid = un.ctx_len - (un.page0 + w + DEC_WAVES * k) * 16;   // >= 1 tokens of this page count
        f32x4 s = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int j = 0; j < NJ; j++) s = __builtin_amdgcn_mfma_f32_16x16x32_bf16(r.k[j], qB[j], s, 0, 0, 0);
        // lane (g, c): s[i] = score of token 4g + i for head c
        float t[4];
#pragma unroll
        for (int i = 0; i < 4; i++) t[i] = 4 * g + i < valid ? fmaf(s[i], sc, -M) : -INFINITY;
        const float tm = fmaxf(fmaxf(t[0], t[1]), fmaxf(t[2], t[3]));
        if (__any(c < GW && tm > DEC_RESCALE_LOG2)) {
            // move the reference of every head to the largest score the wave has seen
            float mx = -INFINITY;
#pragma unroll
            for (int i = 0; i < 4; i++) mx = fmaxf(mx, 4 * g + i < valid ? s[i] * sc : -INFINITY);
            mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
            mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
            const float newM = fmaxf(M, mx);
            const float alpha = newM == -INFINITY ? 1.f : __builtin_amdgcn_exp2f(M - newM);   // 0 on the first page
            M = newM;
            lsum *= alpha;
#pragma unroll
            for (int i = 0; i < 4; i++) t[i] = 4 * g + i < valid ? fmaf(s[i], sc, -M) : -INFINITY;
#pragma unroll
            for (int h = 0; h < GW; h++) {
                const float a = __int_as_float(__builtin_amdgcn_ds_bpermute(bp_base + 4 * h, __float_as_int(alpha)));
#pragma unroll
                for (int e = 0; e < 8; e++) acc[h][e] *= a;
            }
        }
        float pr[4];
#pragma unroll
        for (int i = 0; i < 4; i++) {
            pr[i] = __builtin_amdgcn_exp2f(t[i]);
            lsum += pr[i];
        }
#pragma unroll
        for (int i = 0; i < NLV; i++) {
            // this lane's row of load i is token 4g + i*RPL + sub; rows past the context hold
            // arbitrary pool bytes and must not reach the product
            const bool live = 4 * g + i * RPL + sub < valid;
            float v[8];
#pragma unroll
            for (int q4 = 0; q4 < 4; q4++) {
                const unsigned u = live ? r.v[i][q4] : 0u;
                v[2 * q4] = __uint_as_float(u << 16);
                v[2 * q4 + 1] = __uint_as_float(u & 0xffff0000u);
            }
#pragma unroll
            for (int h = 0; h < GW; h++) {
                float ph;
                if constexpr (RPL == 1) {
                    ph = __int_as_float(__builtin_amdgcn_ds_bpermute(bp_base + 4 * h, __float_as_int(pr[i])));
                } else {
                    const float pa = __int_as_float(__builtin_amdgcn_ds_bpermute(bp_base + 4 * h, __float_as_int(pr[2 * i])));
                    const float pb = __int_as_float(__builtin_amdgcn_ds_bpermute(bp_base + 4 * h, __float_as_int(pr[2 * i + 1])));
                    ph = sub ? pb : pa;
                }
#pragma unroll
                for (int e = 0; e < 8; e++) acc[h][e] = fmaf(ph, v[e], acc[h][e]);
            }
        }
    };

    // the pages DEC_NBUF-1 ahead are in flight while one is being worked on
    PageRegs rg[DEC_NBUF];
#pragma unroll
    for (int b = 0; b < DEC_NBUF - 1; b++)
        if (b < n_mine) load_page(b, rg[b]);
    for (int k0 = 0; k0 < n_mine; k0 += DEC_NBUF) {
#pragma unroll
        for (int b = 0; b < DEC_NBUF; b++) {
            const int k = k0 + b;
            if (k < n_mine) {
                const int kn = k + DEC_NBUF - 1;
                if (kn < n_mine) {
                    if ((kn & 63) == 0) ids = load_ids(kn >> 6);
                    load_page(kn, rg[(b + DEC_NBUF - 1) % DEC_NBUF]);
                }
                compute_page(k, rg[b]);
            }
        }
    }

    // merge the four 16-lane groups (and, for d = 64, the two rows a group fetched per load)
#pragma unroll
    for (int h = 0; h < GW; h++)
#pragma unroll
        for (int e = 0; e < 8; e++) {
            float x = acc[h][e];
            x += __shfl_xor(x, 16, 64);
            x += __shfl_xor(x, 32, 64);
            if constexpr (RPL == 2) x += __shfl_xor(x, 8, 64);
            acc[h][e] = x;
        }
    lsum += __shfl_xor(lsum, 16, 64);
    lsum += __shfl_xor(lsum, 32, 64);

    // the four waves of the work-group meet in LDS; the work-group stores ONE partial:
    // [GW][D] unnormalised output, [GW] reference, [GW] row sum
    constexpr int PS = (GW * (D + 2) + 3) & ~3;
    __shared__ __attribute__((aligned(16))) float part[DEC_WAVES][PS];
    {
        float *ps = part[w];
        if (g == 0 && sub == 0) {
#pragma unroll
            for (int h = 0; h < GW; h++) {
                float *o = ps + h * D + 8 * (l % CPR);
                *(f32x4 *)o = f32x4{acc[h][0], acc[h][1], acc[h][2], acc[h][3]};
                *(f32x4 *)(o + 4) = f32x4{acc[h][4], acc[h][5], acc[h][6], acc[h][7]};
            }
        }
        if (g == 0 && c < GW) {
            ps[GW * D + c] = M;
            ps[GW * D + GW + c] = lsum;
        }
    }
    __syncthreads();
    const int64_t slot = (((int64_t)un.split * p.Hkv + kvh) * nsplit_g + hs);
    float *dst = p.scratch + slot * PS;
    for (int idx = threadIdx.x; idx < GW * D + GW; idx += 64 * DEC_WAVES) {
        const int h = idx < GW * D ? idx / D : idx - GW * D;
        float Mx = -INFINITY;
#pragma unroll
        for (int ww = 0; ww < DEC_WAVES; ww++) Mx = fmaxf(Mx, part[ww][GW * D + h]);
        float num = 0.f, den = 0.f;
#pragma unroll
        for (int ww = 0; ww < DEC_WAVES; ww++) {
            const float m = part[ww][GW * D + h];
            const float f = m == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(m - Mx);   // a wave without pages
            num += f * (idx < GW * D ? part[ww][idx] : 0.f);
            den += f * part[ww][GW * D + GW + h];
        }
        if (idx < GW * D) {
            dst[idx] = num;
        } else {
            dst[GW * D + h] = Mx;
            dst[GW * D + GW + h] = den;
        }
    }
#endif
}

// One work-group per (request, KV head, head group), one thread per (head, d): merges the
// partials of the request's slices, normalises and rounds once to bf16.
template <int D, int GW>
__global__ __launch_bounds__(D * GW) void decode_merge_kernel(DecodeParams p, int G) {
    const int nsplit_g = G / GW;
    int bid = blockIdx.x;
    const int hs = bid % nsplit_g;
    bid /= nsplit_g;
    const int kvh = bid % p.Hkv;
    const int req = bid / p.Hkv;
    const DecodeReq rq = p.reqs[req];
    if (p.mirror_reqs != nullptr && kvh == 0 && hs == 0 && threadIdx.x == 0) p.mirror_reqs[req] = rq;
    const int d = threadIdx.x % D, h = threadIdx.x / D;
    constexpr int PS = (GW * (D + 2) + 3) & ~3;
    const int64_t stride = (int64_t)p.Hkv * nsplit_g * PS;             // between consecutive slices
    const float *base = p.scratch + (((int64_t)rq.split0 * p.Hkv + kvh) * nsplit_g + hs) * PS;
    float Mx = -INFINITY;
    for (int s = 0; s < rq.n_splits; s++) Mx = fmaxf(Mx, base[s * stride + GW * D + h]);
    float num = 0.f, den = 0.f;
    for (int s = 0; s < rq.n_splits; s++) {
        const float *ps = base + s * stride;
        const float m = ps[GW * D + h];
        const float f = m == -INFINITY ? 0.f : exp2f(m - Mx);
        num += f * ps[h * D + d];
        den += f * ps[GW * D + GW + h];
    }
    __bf16 *o = (__bf16 *)p.out + ((int64_t)req * p.Hq + kvh * G + hs * GW + h) * D + d;
    *o = (__bf16)(den > 0.f ? num / den : 0.f);
}

template <int D, int GW>
static hipError_t launch_decode_one(const DecodeParams &p, int G, hipStream_t s) {
    const int nsplit_g = G / GW;
    if (p.n_units > 0) {
        hipLaunchKernelGGL((decode_bf16_kernel<D, GW>), dim3((unsigned)p.n_units * p.Hkv * nsplit_g),
                           dim3(64 * DEC_WAVES), 0, s, p, G);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL((decode_merge_kernel<D, GW>), dim3((unsigned)p.n_reqs * p.Hkv * nsplit_g), dim3(D * GW), 0, s, p, G);
    return hipGetLastError();
}

hipError_t launch_decode_bf16(const DecodeParams &p, int head_dim, hipStream_t s) {
    const int G = p.Hq / p.Hkv;
    const int GW = decode_heads_per_group(G);
    if (head_dim == 128) {
        switch (GW) {
            case 1: return launch_decode_one<128, 1>(p, G, s);
            case 2: return launch_decode_one<128, 2>(p, G, s);
            case 4: return launch_decode_one<128, 4>(p, G, s);
            default: return launch_decode_one<128, 8>(p, G, s);
        }
    }
    switch (GW) {
        case 1: return launch_decode_one<64, 1>(p, G, s);
        case 2: return launch_decode_one<64, 2>(p, G, s);
        case 4: return launch_decode_one<64, 4>(p, G, s);
        default: return launch_decode_one<64, 8>(p, G, s);
    }
}

}  // namespace pbkv
