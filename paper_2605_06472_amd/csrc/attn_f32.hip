// fp32 prefix-reuse prefill attention: plain FMA arithmetic, one query row per lane.
// Exists for fp32 inputs, where the result must agree with the fp64 definition to
// 1e-5: there is no reduced-precision contraction anywhere on this path.  K/V rows are
// staged through LDS 32 keys at a time and read back as broadcasts.
#include "pbkv_internal.h"

namespace pbkv {

constexpr int F32_TOK = 64;    // suffix tokens (= lanes) per work-group
constexpr int F32_KEYS = 32;   // keys per LDS stage

int attn_f32_tile_tokens() { return F32_TOK; }

template <int D>
__global__ __launch_bounds__(F32_TOK) void attn_f32_kernel(AttnParams p) {
    __shared__ __attribute__((aligned(16))) float sK[F32_KEYS][D];
    __shared__ __attribute__((aligned(16))) float sV[F32_KEYS][D];
    const int tile = blockIdx.x / p.Hq;
    const int h = blockIdx.x % p.Hq;
    const TileDesc td = p.tiles[tile];
    const int G = p.Hq / p.Hkv;
    const int g = h / G;
    const int lane = threadIdx.x;
    const int tok_raw = td.tok0 + lane;
    const bool live = tok_raw < td.new_len;
    const int tok = live ? tok_raw : td.new_len - 1;
    const int tok_end = min(td.tok0 + F32_TOK, td.new_len);
    const int n_keys = td.prefix_len + tok_end;           // keys visible to the tile's last row
    const int my_keys = td.prefix_len + tok + 1;          // keys visible to this row
    const float *qf = (const float *)p.q + ((td.row0 + tok) * p.Hq + h) * D;
    const float *kn = (const float *)p.k_new;
    const float *vn = (const float *)p.v_new;
    const float *pool = (const float *)p.kv_pool;
    const int32_t *bt = p.block_table + (int64_t)td.req * p.max_pages;
    const float c = 1.4426950408889634f * rsqrtf((float)D);

    float q[D], o[D];
#pragma unroll
    for (int i = 0; i < D; i += 4) {
        const float4 t = *(const float4 *)(qf + i);
        q[i] = t.x; q[i + 1] = t.y; q[i + 2] = t.z; q[i + 3] = t.w;
    }
#pragma unroll
    for (int i = 0; i < D; i++) o[i] = 0.f;
    float m = -INFINITY, l = 0.f;

    for (int k0 = 0; k0 < n_keys; k0 += F32_KEYS) {
        __syncthreads();
        // stage 32 key/value rows: 32 * D/4 float4 each, 64 lanes
        for (int idx = lane; idx < F32_KEYS * (D / 4); idx += F32_TOK) {
            const int r = idx / (D / 4), c4 = idx % (D / 4);
            const int j = k0 + r;
            float4 kk = make_float4(0.f, 0.f, 0.f, 0.f), vv = kk;
            if (j < n_keys) {
                if (j < td.prefix_len) {
                    int pg = bt[j >> 4];
                    pg = pg < 0 ? 0 : (pg >= p.num_pages ? p.num_pages - 1 : pg);
                    const int64_t base = ((((int64_t)pg * 2) * p.Hkv + g) * 16 + (j & 15)) * D + c4 * 4;
                    kk = *(const float4 *)(pool + base);
                    vv = *(const float4 *)(pool + base + (int64_t)p.Hkv * 16 * D);
                } else {
                    const int64_t base = ((td.row0 + (j - td.prefix_len)) * p.Hkv + g) * D + c4 * 4;
                    kk = *(const float4 *)(kn + base);
                    vv = *(const float4 *)(vn + base);
                }
            }
            *(float4 *)&sK[r][c4 * 4] = kk;
            *(float4 *)&sV[r][c4 * 4] = vv;
        }
        __syncthreads();
        float s[F32_KEYS];
        float mx = m;
#pragma unroll
        for (int r = 0; r < F32_KEYS; r++) {
            float a0 = 0.f, a1 = 0.f, a2 = 0.f, a3 = 0.f;
#pragma unroll
            for (int i = 0; i < D; i += 4) {
                const float4 kk = *(const float4 *)&sK[r][i];
                a0 = fmaf(q[i], kk.x, a0);
                a1 = fmaf(q[i + 1], kk.y, a1);
                a2 = fmaf(q[i + 2], kk.z, a2);
                a3 = fmaf(q[i + 3], kk.w, a3);
            }
            const float dot = (a0 + a1) + (a2 + a3);
            s[r] = (k0 + r < my_keys) ? dot : -INFINITY;
            mx = fmaxf(mx, s[r]);
        }
        // key 0 is visible to every row, so mx is finite from the first stage on
        const float alpha = exp2f((m - mx) * c);
        m = mx;
        l *= alpha;
#pragma unroll
        for (int i = 0; i < D; i++) o[i] *= alpha;
#pragma unroll
        for (int r = 0; r < F32_KEYS; r++) {
            const float w = exp2f((s[r] - m) * c);
            l += w;
#pragma unroll
            for (int i = 0; i < D; i += 4) {
                const float4 vv = *(const float4 *)&sV[r][i];
                o[i] = fmaf(w, vv.x, o[i]);
                o[i + 1] = fmaf(w, vv.y, o[i + 1]);
                o[i + 2] = fmaf(w, vv.z, o[i + 2]);
                o[i + 3] = fmaf(w, vv.w, o[i + 3]);
            }
        }
    }
    if (live) {
        const float inv = 1.0f / l;
        float *of = (float *)p.out + ((td.row0 + tok) * p.Hq + h) * D;
#pragma unroll
        for (int i = 0; i < D; i += 4)
            *(float4 *)(of + i) = make_float4(o[i] * inv, o[i + 1] * inv, o[i + 2] * inv, o[i + 3] * inv);
    }
}

hipError_t launch_attn_f32(const AttnParams &p, int head_dim, hipStream_t s) {
    if (p.n_tiles == 0) return hipSuccess;
    const dim3 grid((unsigned)p.n_tiles * p.Hq), block(F32_TOK);
    if (head_dim == 64)
        hipLaunchKernelGGL(attn_f32_kernel<64>, grid, block, 0, s, p);
    else
        hipLaunchKernelGGL(attn_f32_kernel<128>, grid, block, 0, s, p);
    return hipGetLastError();
}

}  // namespace pbkv
