// bf16 prefix-reuse prefill attention for gfx950 (CDNA4): flash-style online softmax
// over KV tiles gathered page by page through the block table, QK^T and PV on the
// 32x32x16 bf16 MFMA, fp32 accumulation.
//
// Work decomposition
//   work-group = 4 waves = (request, KV head, block of suffix tokens).  The query heads
//   of a GQA group share every K/V tile staged in LDS: wave w takes query head
//   w % Gw (Gw = min(G,4)) and token sub-block w / Gw, 32*QB tokens per wave.
//   blockIdx -> KV head is the fastest index, so with round-robin dispatch over the 8
//   XCDs and 8 KV heads every tile of one KV head runs on one XCD and re-reads of its
//   pages hit that XCD's L2.
//
// Orientation
//   S^T = K Q^T (keys are MFMA rows, queries are MFMA columns).  A lane then owns ONE
//   query column and 16 key scores per 32x32 block, so the row max / row sum of the
//   softmax are in-lane reductions plus one exchange between lanes l and l^32, and
//   the probabilities are already in the B-operand layout of the second product
//   O^T = V^T P^T -- no LDS round trip for P.  The contraction index of PV (keys) is
//   only a label, so the key order the accumulator layout induces is matched on the
//   V side: V^T operands come from ds_read_b64_tr_b16 (transposing LDS read) on a
//   row-major [key][d] tile.
//
// LDS: K rows padded to 2d+16 bytes (16 consecutive rows x 16 B hit distinct banks for
// ds_read_b128), V rows padded to 2d+64 bytes (the 8 rows x 64 B of one transposing read
// hit distinct banks).  Two buffers each; the next tile's global loads are issued
// before the current tile's math and written to LDS after it.
#include "pbkv_internal.h"

namespace pbkv {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((address_space(3))) bf16x4 lds_bf16x4;

constexpr int BN = 64;   // keys per LDS tile (two 32-key MFMA row blocks)
constexpr int KB = BN / 32;

template <int D>
struct Geom {
    static constexpr int DC = D / 16;         // contraction steps of QK^T
    static constexpr int DB = D / 32;         // 32-row blocks of O^T
    static constexpr int KS = D * 2 + 16;     // K row stride in LDS, bytes
    static constexpr int VS = D * 2 + 64;     // V row stride in LDS, bytes
    static constexpr int KBUF = BN * KS;
    static constexpr int VBUF = BN * VS;
    static constexpr int LDS_BYTES = 2 * (KBUF + VBUF);
    static constexpr int CPR = D / 8;         // 16-byte chunks per row
    static constexpr int RPP = 256 / CPR;     // rows loaded per pass of the work-group
    static constexpr int NP = BN / RPP;       // passes per tile
};

static __device__ __forceinline__ float xmax32(float x) {
    auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
static __device__ __forceinline__ float xsum32(float x) {
    auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

int attn_bf16_tile_tokens(int /*head_dim*/, int group) {
    const int gw = group < 4 ? group : 4;
    return 64 * (4 / gw);   // QB = 2 instantiation
}

template <int D, int QB>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, 1)))
void attn_bf16_kernel(AttnParams p, int G, int Gw) {
    using Gm = Geom<D>;
    extern __shared__ __attribute__((aligned(16))) char smem[];
    char *const sK = smem;
    char *const sV = smem + 2 * Gm::KBUF;

    const int tid = threadIdx.x, w = tid >> 6, l = tid & 63, li = l & 31, lh = l >> 5;
    const int kvh = blockIdx.x % p.Hkv;
    const int rest = blockIdx.x / p.Hkv;
    const int nsplit = G / Gw;
    const int split = rest % nsplit;
    const TileDesc td = p.tiles[rest / nsplit];
    const int head = kvh * G + split * Gw + (w % Gw);
    constexpr int WTOK = 32 * QB;
    const int tile_tok = WTOK * (4 / Gw);
    const int tok_base = td.tok0 + (w / Gw) * WTOK;
    const int tok_end = min(td.tok0 + tile_tok, td.new_len);
    const int n_keys = td.prefix_len + tok_end;          // keys visible to the tile's last row
    const int n_tiles = (n_keys + BN - 1) / BN;
    const int wave_min_limit = td.prefix_len + min(tok_base, td.new_len - 1);

    const __bf16 *qg = (const __bf16 *)p.q;
    const __bf16 *kn = (const __bf16 *)p.k_new;
    const __bf16 *vn = (const __bf16 *)p.v_new;
    const __bf16 *pool = (const __bf16 *)p.kv_pool;
    const int32_t *bt = p.block_table + (int64_t)td.req * p.max_pages;

    // ---- Q^T operands: lane (li, lh) holds Q[token li][16*dc + 8*lh .. +7] -------------
    bf16x8 qreg[QB][Gm::DC];
    int my_limit[QB];                                     // last visible key of this lane's row
    int my_tok[QB];
#pragma unroll
    for (int qb = 0; qb < QB; qb++) {
        const int tr = tok_base + 32 * qb + li;
        my_tok[qb] = tr;
        const int tok = min(tr, td.new_len - 1);
        my_limit[qb] = td.prefix_len + tok;
        const __bf16 *qp = qg + ((td.row0 + tok) * p.Hq + head) * D + 8 * lh;
#pragma unroll
        for (int dc = 0; dc < Gm::DC; dc++) qreg[qb][dc] = *(const bf16x8 *)(qp + dc * 16);
    }

    // ---- cooperative tile loader --------------------------------------------------------
    const int lr = tid / Gm::CPR, lc = tid % Gm::CPR;
    uint4 kst[Gm::NP], vst[Gm::NP];
    auto issue_loads = [&](int k0) {
#pragma unroll
        for (int i = 0; i < Gm::NP; i++) {
            const int j = k0 + i * Gm::RPP + lr;
            kst[i] = make_uint4(0, 0, 0, 0);
            vst[i] = make_uint4(0, 0, 0, 0);
            if (j < n_keys) {
                if (j < td.prefix_len) {
                    int pg = bt[j >> 4];
                    pg = pg < 0 ? 0 : (pg >= p.num_pages ? p.num_pages - 1 : pg);
                    const int64_t base = (((int64_t)pg * 2 * p.Hkv + kvh) * 16 + (j & 15)) * D + lc * 8;
                    kst[i] = *(const uint4 *)(pool + base);
                    vst[i] = *(const uint4 *)(pool + base + (int64_t)p.Hkv * 16 * D);
                } else {
                    const int64_t base = ((td.row0 + (j - td.prefix_len)) * p.Hkv + kvh) * D + lc * 8;
                    kst[i] = *(const uint4 *)(kn + base);
                    vst[i] = *(const uint4 *)(vn + base);
                }
            }
        }
    };
    auto store_lds = [&](int buf) {
#pragma unroll
        for (int i = 0; i < Gm::NP; i++) {
            const int row = i * Gm::RPP + lr;
            *(uint4 *)(sK + buf * Gm::KBUF + row * Gm::KS + lc * 16) = kst[i];
            *(uint4 *)(sV + buf * Gm::VBUF + row * Gm::VS + lc * 16) = vst[i];
        }
    };

    // ---- running state --------------------------------------------------------------------
    f32x16 O[Gm::DB][QB];
#pragma unroll
    for (int db = 0; db < Gm::DB; db++)
#pragma unroll
        for (int qb = 0; qb < QB; qb++)
#pragma unroll
            for (int r = 0; r < 16; r++) O[db][qb][r] = 0.f;
    float m_run[QB], l_part[QB];
#pragma unroll
    for (int qb = 0; qb < QB; qb++) { m_run[qb] = -INFINITY; l_part[qb] = 0.f; }
    const float c = 1.4426950408889634f * rsqrtf((float)D);

    // per-lane constant parts of the LDS addresses
    const int k_lane_off = li * Gm::KS + lh * 16;
    const int v_lane_off = (4 * lh + ((l & 15) >> 2)) * Gm::VS + (16 * ((l >> 4) & 1) + 4 * (l & 3)) * 2;

    issue_loads(0);
    store_lds(0);
    __syncthreads();

    for (int t = 0; t < n_tiles; t++) {
        const int buf = t & 1;
        const int k0 = t * BN;
        const bool more = t + 1 < n_tiles;
        if (more) issue_loads(k0 + BN);

        // ---- S^T = K Q^T -------------------------------------------------------------------
        f32x16 S[KB][QB];
#pragma unroll
        for (int kb = 0; kb < KB; kb++)
#pragma unroll
            for (int qb = 0; qb < QB; qb++)
#pragma unroll
                for (int r = 0; r < 16; r++) S[kb][qb][r] = 0.f;
        const char *kbuf = sK + buf * Gm::KBUF + k_lane_off;
#pragma unroll
        for (int kb = 0; kb < KB; kb++)
#pragma unroll
            for (int dc = 0; dc < Gm::DC; dc++) {
                const bf16x8 a = *(const bf16x8 *)(kbuf + kb * 32 * Gm::KS + dc * 32);
#pragma unroll
                for (int qb = 0; qb < QB; qb++)
                    S[kb][qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qreg[qb][dc], S[kb][qb], 0, 0, 0);
            }

        // ---- online softmax (per query column = per lane) ---------------------------------
        const bool need_mask = k0 + BN - 1 > wave_min_limit;
        bf16x8 P[QB][KB][2];
#pragma unroll
        for (int qb = 0; qb < QB; qb++) {
            if (need_mask) {
#pragma unroll
                for (int kb = 0; kb < KB; kb++)
#pragma unroll
                    for (int r = 0; r < 16; r++) {
                        const int key = k0 + 32 * kb + 8 * (r >> 2) + 4 * lh + (r & 3);
                        if (key > my_limit[qb]) S[kb][qb][r] = -INFINITY;
                    }
            }
            float mx = S[0][qb][0];
#pragma unroll
            for (int kb = 0; kb < KB; kb++)
#pragma unroll
                for (int r = 0; r < 16; r++) mx = fmaxf(mx, S[kb][qb][r]);
            mx = xmax32(mx);
            const float m_new = fmaxf(m_run[qb], mx);
            // rescale lazily: a stale maximum is kept while it is within 2^8 of the true one
            if (__any((m_new - m_run[qb]) * c > 8.0f)) {
                const float alpha = __builtin_amdgcn_exp2f((m_run[qb] - m_new) * c);
                m_run[qb] = m_new;
                l_part[qb] *= alpha;
#pragma unroll
                for (int db = 0; db < Gm::DB; db++)
#pragma unroll
                    for (int r = 0; r < 16; r++) O[db][qb][r] *= alpha;
            }
            const float mc = m_run[qb] * c;
            float ls = 0.f;
#pragma unroll
            for (int kb = 0; kb < KB; kb++)
#pragma unroll
                for (int u = 0; u < 2; u++)
#pragma unroll
                    for (int e = 0; e < 8; e++) {
                        const float pv = __builtin_amdgcn_exp2f(fmaf(S[kb][qb][8 * u + e], c, -mc));
                        ls += pv;
                        P[qb][kb][u][e] = (__bf16)pv;
                    }
            l_part[qb] += ls;
        }

        // ---- O^T += V^T P^T ----------------------------------------------------------------
        const char *vbuf = sV + buf * Gm::VBUF + v_lane_off;
#pragma unroll
        for (int kb = 0; kb < KB; kb++)
#pragma unroll
            for (int u = 0; u < 2; u++)
#pragma unroll
                for (int db = 0; db < Gm::DB; db++) {
                    const char *vp = vbuf + (32 * kb + 16 * u) * Gm::VS + db * 64;
                    const bf16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4 *)vp);
                    const bf16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4 *)(vp + 8 * Gm::VS));
                    const bf16x8 a = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
#pragma unroll
                    for (int qb = 0; qb < QB; qb++)
                        O[db][qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, P[qb][kb][u], O[db][qb], 0, 0, 0);
                }

        if (more) store_lds(buf ^ 1);
        __syncthreads();
    }

    // ---- epilogue: normalise, round once to bf16, store -----------------------------------
    __bf16 *og = (__bf16 *)p.out;
#pragma unroll
    for (int qb = 0; qb < QB; qb++) {
        const float inv = 1.0f / xsum32(l_part[qb]);
        if (my_tok[qb] < td.new_len) {
            __bf16 *op = og + ((td.row0 + my_tok[qb]) * p.Hq + head) * D + 4 * lh;
#pragma unroll
            for (int db = 0; db < Gm::DB; db++)
#pragma unroll
                for (int b4 = 0; b4 < 4; b4++) {
                    bf16x4 v;
#pragma unroll
                    for (int cc = 0; cc < 4; cc++) v[cc] = (__bf16)(O[db][qb][4 * b4 + cc] * inv);
                    *(bf16x4 *)(op + 32 * db + 8 * b4) = v;
                }
        }
    }
}

template <int D, int QB>
static hipError_t launch_one(const AttnParams &p, int G, int Gw, hipStream_t s) {
    static bool attr_set = false;
    auto kern = attn_bf16_kernel<D, QB>;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize,
                                           Geom<D>::LDS_BYTES);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    const unsigned grid = (unsigned)p.n_tiles * (G / Gw) * p.Hkv;
    hipLaunchKernelGGL(kern, dim3(grid), dim3(256), Geom<D>::LDS_BYTES, s, p, G, Gw);
    return hipGetLastError();
}

hipError_t launch_attn_bf16(const AttnParams &p, int head_dim, hipStream_t s) {
    if (p.n_tiles == 0) return hipSuccess;
    const int G = p.Hq / p.Hkv;
    const int Gw = G < 4 ? G : 4;
    if (head_dim == 128) return launch_one<128, 2>(p, G, Gw, s);
    return launch_one<64, 2>(p, G, Gw, s);
}

}  // namespace pbkv
