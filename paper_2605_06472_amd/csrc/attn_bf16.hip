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
// Page gather
//   K/V rows go from global memory straight into LDS (global_load_lds_dwordx4, 16 bytes
//   per lane, 1 KiB contiguous in LDS per wave instruction) -- no staging registers and
//   no LDS store instructions.  Rows are unpadded; bank conflicts are avoided by an XOR
//   swizzle of the 16-byte chunk index that is applied on the global-address side:
//   the lane that owns LDS chunk position c' of row r fetches global chunk c'^swz(r).
//
// Software pipeline (one wave does both MFMA and VALU work; the two are interleaved
// with scheduling-group barriers):
//   phase A   S(j+1) = K(j+1) Q^T  on the MFMA  ||  P(j) = exp2(S(j) c - m c), row sums
//   phase B   O += V(j)^T P(j)     on the MFMA  ||  row max of S(j+1)
// so K runs one tile ahead of V, and the score registers ping-pong between two sets.
#include "pbkv_internal.h"

#include <cstdlib>

namespace pbkv {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((address_space(3))) bf16x4 lds_bf16x4;
typedef __attribute__((address_space(3))) void lds_void;

constexpr int BN = 64;   // keys per LDS tile (two 32-key MFMA row blocks)
constexpr int KB = BN / 32;
constexpr int PF = 3;    // LDS operand prefetch distance, in pipeline steps

template <int D>
struct Geom {
    static constexpr int DC = D / 16;         // contraction steps of QK^T per key block
    static constexpr int DB = D / 32;         // 32-row blocks of O^T
    static constexpr int NS = D / 8;          // pipeline steps per phase (KB*DC = KB*2*DB)
    static constexpr int ROWB = D * 2;        // bytes per K/V row
    static constexpr int TILEB = BN * ROWB;   // bytes per K or V tile
    static constexpr int CPR = D / 8;         // 16-byte chunks per row
    static constexpr int RPI = 64 / CPR;      // rows covered by one wave-wide 1 KiB load
    static constexpr int NI = BN / (4 * RPI); // loads per wave per tile
    // XOR applied to the chunk index of row `row` (conflict-free ds_read_b128 of 16
    // consecutive rows for K; conflict-free 4-row x 32-byte transposing reads for V)
    static __device__ __forceinline__ int swz_k(int row) { return D == 128 ? (row & 15) : ((row >> 1) & 7); }
    static __device__ __forceinline__ int swz_v(int row) { return D == 128 ? ((row & 7) << 1) : (((row >> 1) & 3) << 1); }
};

static __device__ __forceinline__ float xmax32(float x) {
    auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
static __device__ __forceinline__ float xsum32(float x) {
    auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

// Query blocks (of 32 rows) per wave: 2 = one wave per SIMD with 64 rows each, 1 = two
// work-groups per CU with 32 rows per wave.
static int query_blocks() {
    static int qb = [] {
        const char *e = getenv("PBKV_ATTN_QB");
        return (e && e[0] == '1') ? 1 : 2;
    }();
    return qb;
}

int attn_bf16_tile_tokens(int /*head_dim*/, int group) {
    const int gw = group < 4 ? group : 4;
    return 32 * query_blocks() * (4 / gw);
}

// Keeps a value (and so the code that computes it) at this point of the program; the
// constraint names a vector register, which only exists in the device pass.
#if defined(__HIP_DEVICE_COMPILE__)
#define PIN_V(x) asm volatile("" : "+v"(x))
#else
#define PIN_V(x) (void)(x)
#endif

// scheduling-group masks
#define SG_VALU 0x402   // VALU or transcendental
#define SG_MFMA 0x008
#define SG_DSRD 0x100

template <int D, int QB>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(3 - QB, 3 - QB)))
void attn_bf16_kernel(AttnParams p, int G, int Gw) {
#if defined(__HIP_DEVICE_COMPILE__)   // the body uses gfx950-only builtins and types; the host pass only needs the stub
    using Gm = Geom<D>;
    constexpr int NS = Gm::NS;
    constexpr int SPS = QB * 32 / NS;     // scores per lane handled in one pipeline step
    static_assert(SPS >= 2 && SPS % 2 == 0, "scores are converted in pairs");
    // four separate arrays: the direct-to-LDS loads of one buffer provably do not alias
    // the operand reads of the others
    __shared__ __attribute__((aligned(1024))) char sK0[Gm::TILEB];
    __shared__ __attribute__((aligned(1024))) char sK1[Gm::TILEB];
    __shared__ __attribute__((aligned(1024))) char sV0[Gm::TILEB];
    __shared__ __attribute__((aligned(1024))) char sV1[Gm::TILEB];

    const int tid = threadIdx.x, l = tid & 63, li = l & 31, lh = l >> 5;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave index, kept in a scalar register
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

    // zero the V buffers once: rows past the last key are never loaded, and 0 * stale bits
    // must not be able to produce a NaN in the PV product
    for (int i = tid; i < Gm::TILEB / 16; i += 256) {
        *(uint4 *)(sV0 + i * 16) = make_uint4(0, 0, 0, 0);
        *(uint4 *)(sV1 + i * 16) = make_uint4(0, 0, 0, 0);
    }

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

    // ---- tile loader: global -> LDS, 16 bytes per lane ------------------------------------
    // Block-table entries are held 64 at a time (16 tiles) in one vector register, lane i =
    // logical page 64*blk + i, clamped to the pool; the block after the current one is
    // loaded 16 tiles early.  A tile's four page ids are then lane reads into scalar
    // registers: no K/V address ever waits on the table.
    const int n_prefix_pages = (td.prefix_len + 15) >> 4;
    auto load_id_block = [&](int blk) {
        const int lp = blk * 64 + l;
        int pg = lp < n_prefix_pages ? bt[lp] : 0;
        pg = pg < 0 ? 0 : (pg >= p.num_pages ? p.num_pages - 1 : pg);
        return pg;
    };
    int ids_cur = load_id_block(0), ids_next = load_id_block(1);
    struct PageIds { int v[BN / 16]; };
    // page ids of tile t; tiles must be asked for in ascending order (t = 0, 1, 2, ...)
    auto fetch_page_ids = [&](int t) {
        if ((t & 15) == 0 && t > 0) {
            ids_cur = ids_next;
            ids_next = load_id_block((t >> 4) + 1);
        }
        PageIds r;
#pragma unroll
        for (int g = 0; g < BN / 16; g++) r.v[g] = __builtin_amdgcn_readlane(ids_cur, (t & 15) * 4 + g);
        return r;
    };
    // One wave-wide load = RPI consecutive rows of one page (or of the suffix), 1 KiB.  The
    // source is addressed as a raw buffer: a wave-uniform descriptor built with scalar
    // arithmetic (page base, or the suffix row base) plus a per-lane byte offset that does
    // not change from tile to tile, so the gather costs no vector address arithmetic.
    const int ld_lrow = l / Gm::CPR;                       // row inside this wave's row group
    const int ld_cpos = l % Gm::CPR;                       // chunk position this lane fills
    const int ld_slot = ((w * Gm::RPI) & 15) + ld_lrow;    // slot inside the page (same for all groups)
    const int ld_ck = ld_cpos ^ Gm::swz_k(w * Gm::RPI + ld_lrow);   // global chunk this lane fetches (K)
    const int ld_cv = ld_cpos ^ Gm::swz_v(w * Gm::RPI + ld_lrow);   // ... (V)
    const int row_pitch = p.Hkv * Gm::ROWB;                // bytes between suffix tokens
    const int voff_pk = ld_slot * Gm::ROWB + ld_ck * 16;
    const int voff_pv = ld_slot * Gm::ROWB + ld_cv * 16 + p.Hkv * 16 * Gm::ROWB;
    const int voff_sk = ld_lrow * row_pitch + ld_ck * 16;
    const int voff_sv = ld_lrow * row_pitch + ld_cv * 16;
    const int page_bytes = 2 * p.Hkv * 16 * Gm::ROWB;
    const char *pool_head = (const char *)pool + (int64_t)kvh * 16 * Gm::ROWB;
    constexpr int RSRC_FLAGS = 0x00020000;                 // raw buffer, 32-bit data format
    auto load_tile = [&](int k0, const PageIds &pid, char *buf, const __bf16 *fresh, bool is_v) {
        const int voff_p = is_v ? voff_pv : voff_pk, voff_s = is_v ? voff_sv : voff_sk;
        if (k0 + BN <= td.prefix_len) {
            // the whole tile lies in the cached prefix: one descriptor per page
#pragma unroll
            for (int i = 0; i < Gm::NI; i++) {
                // page of this row group inside the tile: i for d=128, 2i + w/2 for d=64
                const int pg = Gm::RPI == 4 ? pid.v[i] : ((w >> 1) ? pid.v[(2 * i + 1) % (BN / 16)] : pid.v[(2 * i) % (BN / 16)]);
                const auto rsrc = __builtin_amdgcn_make_buffer_rsrc(
                    (void *)(pool_head + (int64_t)pg * page_bytes), 0, page_bytes, RSRC_FLAGS);
                __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, (lds_void *)(buf + (i * 4 + w) * 1024), 16, voff_p, 0, 0, 0);
            }
            asm volatile("; tile from prefix pages");   // distinct block ends: keeps the three paths' loads apart
        } else if (k0 >= td.prefix_len && k0 + BN <= n_keys) {
            // the whole tile lies in the suffix: one descriptor, a scalar offset per row group
            const char *base = (const char *)fresh + ((td.row0 + (k0 - td.prefix_len)) * p.Hkv + kvh) * (int64_t)Gm::ROWB;
            const auto rsrc = __builtin_amdgcn_make_buffer_rsrc((void *)base, 0, BN * row_pitch, RSRC_FLAGS);
#pragma unroll
            for (int i = 0; i < Gm::NI; i++)
                __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, (lds_void *)(buf + (i * 4 + w) * 1024), 16, voff_s,
                                                         (i * 4 + w) * Gm::RPI * row_pitch, 0, 0);
            asm volatile("; tile from the suffix");
        } else {
            // the prefix ends inside this tile, or the tile holds the last visible keys
#pragma unroll
            for (int i = 0; i < Gm::NI; i++) {
                const int g0 = k0 + (i * 4 + w) * Gm::RPI;    // first key of this wave's row group
                if (g0 >= n_keys) continue;
                lds_void *dst = (lds_void *)(buf + (i * 4 + w) * 1024);
                const int pg = Gm::RPI == 4 ? pid.v[i] : ((w >> 1) ? pid.v[(2 * i + 1) % (BN / 16)] : pid.v[(2 * i) % (BN / 16)]);
                const int split = td.prefix_len - g0;          // rows [0, split) of the group are prefix rows
                if (split > 0) {
                    const auto rp = __builtin_amdgcn_make_buffer_rsrc(
                        (void *)(pool_head + (int64_t)pg * page_bytes), 0, page_bytes, RSRC_FLAGS);
                    if (ld_lrow < split) __builtin_amdgcn_raw_ptr_buffer_load_lds(rp, dst, 16, voff_p, 0, 0, 0);
                    asm volatile("; prefix rows of a mixed group");
                }
                if (split < Gm::RPI) {
                    const char *sbase = (const char *)fresh +
                                        ((td.row0 + (g0 - td.prefix_len)) * p.Hkv + kvh) * (int64_t)Gm::ROWB;
                    const auto rs = __builtin_amdgcn_make_buffer_rsrc((void *)sbase, 0, Gm::RPI * row_pitch, RSRC_FLAGS);
                    if (ld_lrow >= split && g0 + ld_lrow < n_keys)
                        __builtin_amdgcn_raw_ptr_buffer_load_lds(rs, dst, 16, voff_s, 0, 0, 0);
                    asm volatile("; suffix rows of a mixed group");
                }
            }
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
    float m_run[QB], m_new[QB], l_part[QB];
#pragma unroll
    for (int qb = 0; qb < QB; qb++) { m_run[qb] = -INFINITY; m_new[qb] = -INFINITY; l_part[qb] = 0.f; }
    const float c = 1.4426950408889634f * rsqrtf((float)D);

    // ---- per-lane LDS operand offsets (the swizzle makes them lane- and chunk-specific) ---
    // K operand of step (kb, dc): row 32*kb + li, chunk 2*dc + lh
    int k_off[Gm::DC];
#pragma unroll
    for (int dc = 0; dc < Gm::DC; dc++) k_off[dc] = li * Gm::ROWB + (((2 * dc + lh) ^ Gm::swz_k(li)) << 4);
    // V operand of step (kb, u, db): rows 32*kb + 16*u + 4*lh + (l&15)/4 (+8), 8 bytes at
    // d = 16*db + (D/2)*((l>>4)&1) + 4*(l&3): MFMA rows 0-15 take d in [16db, 16db+16),
    // rows 16-31 take d in D/2 + [16db, 16db+16)
    int v_off_l[Gm::DB];
    {
        const int vrow = 4 * lh + ((l & 15) >> 2);
#pragma unroll
        for (int db = 0; db < Gm::DB; db++) {
            const int d0 = 16 * db + (D / 2) * ((l >> 4) & 1) + 4 * (l & 3);
            v_off_l[db] = vrow * Gm::ROWB + ((((d0 >> 3)) ^ Gm::swz_v(vrow)) << 4) + ((d0 & 4) << 1);
        }
    }
    auto k_operand = [&](const char *kbuf, int s) {       // step s = (kb, dc)
        return *(const bf16x8 *)(kbuf + k_off[s % Gm::DC] + (s / Gm::DC) * 32 * Gm::ROWB);
    };
    auto v_operand = [&](const char *vbuf, int s) {       // step s = (kb, u, db)
        const int kb = s / (2 * Gm::DB), u = (s / Gm::DB) & 1, db = s % Gm::DB;
        const char *vp = vbuf + v_off_l[db] + (32 * kb + 16 * u) * Gm::ROWB;
        const bf16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4 *)vp);
        const bf16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4 *)(vp + 8 * Gm::ROWB));
        return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    };
    auto mask_scores = [&](f32x16 (&S)[KB][QB], int k0) {
#pragma unroll
        for (int qb = 0; qb < QB; qb++) {
            const int rel = my_limit[qb] - k0 - 4 * lh;
#pragma unroll
            for (int kb = 0; kb < KB; kb++)
#pragma unroll
                for (int r = 0; r < 16; r++)
                    if (32 * kb + 8 * (r >> 2) + (r & 3) > rel) S[kb][qb][r] = -INFINITY;
        }
    };

    // ---- prologue: K(0), V(0), K(1) into LDS, S(0) and its row max ---------------------------
    PageIds pid1, pid2;                                   // page ids of tiles j+1 and j+2
    __syncthreads();                                      // V buffers zeroed
    {
        const PageIds pid0 = fetch_page_ids(0);
        pid1 = fetch_page_ids(1);
        pid2 = fetch_page_ids(2);
        load_tile(0, pid0, sK0, kn, false);
        load_tile(0, pid0, sV0, vn, true);
        load_tile(BN, pid1, sK1, kn, false);
    }
    __builtin_amdgcn_s_waitcnt(0x0F70);                   // vmcnt(0): the loads have landed in LDS
    __syncthreads();
    f32x16 Sa[KB][QB], Sb[KB][QB];
#pragma unroll
    for (int kb = 0; kb < KB; kb++)
#pragma unroll
        for (int qb = 0; qb < QB; qb++)
#pragma unroll
            for (int r = 0; r < 16; r++) { Sa[kb][qb][r] = 0.f; Sb[kb][qb][r] = 0.f; }
#pragma unroll
    for (int s = 0; s < NS; s++) {
        const bf16x8 a = k_operand(sK0, s);
#pragma unroll
        for (int qb = 0; qb < QB; qb++)
            Sa[s / Gm::DC][qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qreg[qb][s % Gm::DC], Sa[s / Gm::DC][qb], 0, 0, 0);
    }
    if (BN - 1 > wave_min_limit) mask_scores(Sa, 0);
#pragma unroll
    for (int qb = 0; qb < QB; qb++) {
        float mx = Sa[0][qb][0];
#pragma unroll
        for (int kb = 0; kb < KB; kb++)
#pragma unroll
            for (int r = 0; r < 16; r++) mx = fmaxf(mx, Sa[kb][qb][r]);
        m_new[qb] = xmax32(mx);
    }

    // ---- one pipelined iteration: tile j, scores Sc = S(j) ready, Sn receives S(j+1) ----------
    auto body = [&](int j, f32x16 (&Sc)[KB][QB], f32x16 (&Sn)[KB][QB], char *kread, char *vread,
                    char *kwrite, char *vwrite) __attribute__((always_inline)) {
        // rescale lazily: a stale maximum is kept while it is within 2^8 of the true one
        bool need = false;
#pragma unroll
        for (int qb = 0; qb < QB; qb++) need |= (m_new[qb] - m_run[qb]) * c > 8.0f;
        if (__any(need)) {
#pragma unroll
            for (int qb = 0; qb < QB; qb++) {
                const float alpha = __builtin_amdgcn_exp2f((m_run[qb] - m_new[qb]) * c);
                m_run[qb] = m_new[qb];
                l_part[qb] *= alpha;
#pragma unroll
                for (int db = 0; db < Gm::DB; db++)
#pragma unroll
                    for (int r = 0; r < 16; r++) O[db][qb][r] *= alpha;
            }
        }
        // prefetch: page ids three tiles ahead, K two tiles ahead, V one tile ahead
        const PageIds pid3 = fetch_page_ids(j + 3);
#ifndef ABL_NOLOAD
        load_tile((j + 2) * BN, pid2, kwrite, kn, false);
        load_tile((j + 1) * BN, pid1, vwrite, vn, true);
#endif
        float mc[QB], ls[QB];
#pragma unroll
        for (int qb = 0; qb < QB; qb++) { mc[qb] = m_run[qb] * c; ls[qb] = 0.f; }
        bf16x8 P[QB][KB][2];

        // ---- phase A: S(j+1) = K(j+1) Q^T  ||  P = exp2(S(j) c - m c) ---------------------------
        __builtin_amdgcn_sched_barrier(0);
        bf16x8 kop[PF + 1];
#pragma unroll
        for (int s = 0; s < PF; s++) kop[s] = k_operand(kread, s);
#pragma unroll
        for (int s = 0; s < NS; s++) {
            if (s + PF < NS) kop[(s + PF) % (PF + 1)] = k_operand(kread, s + PF);
            const int kb = s / Gm::DC, dc = s % Gm::DC;
#pragma unroll
            for (int qb = 0; qb < QB; qb++) {
#ifdef ABL_NOQK
                if (dc == 0) Sn[kb][qb] = Sc[kb][qb];
                continue;
#endif
                if (dc == 0) {
                    f32x16 z;
#pragma unroll
                    for (int r = 0; r < 16; r++) z[r] = 0.f;
                    Sn[kb][qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kop[s % (PF + 1)], qreg[qb][dc], z, 0, 0, 0);
                } else {
                    Sn[kb][qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kop[s % (PF + 1)], qreg[qb][dc], Sn[kb][qb], 0, 0, 0);
                }
            }
#pragma unroll
            for (int t = 0; t < SPS; t += 2) {
                const int idx = s * SPS + t;              // flattened (qb, kb, r)
                const int qb = idx / 32, kb2 = (idx % 32) / 16, r = idx % 16;
                f32x2 pv;
#ifdef ABL_NOEXP
                pv[0] = Sc[kb2][qb][r];
                pv[1] = Sc[kb2][qb][r + 1];
#else
                pv[0] = __builtin_amdgcn_exp2f(fmaf(Sc[kb2][qb][r], c, -mc[qb]));
                pv[1] = __builtin_amdgcn_exp2f(fmaf(Sc[kb2][qb][r + 1], c, -mc[qb]));
                ls[qb] += pv[0];
                ls[qb] += pv[1];
#endif
                const bf16x2 pk = __builtin_convertvector(pv, bf16x2);
                P[qb][kb2][r / 8][r % 8] = pk[0];
                P[qb][kb2][r / 8][r % 8 + 1] = pk[1];
            }
        }
        // interleave: per step, one K operand read, then per MFMA its share of the exp work
        __builtin_amdgcn_sched_group_barrier(SG_DSRD, PF, 0);
#pragma unroll
        for (int s = 0; s < NS; s++) {
#pragma unroll
            for (int qb = 0; qb < QB; qb++) {
                __builtin_amdgcn_sched_group_barrier(SG_MFMA, 1, 0);
                __builtin_amdgcn_sched_group_barrier(SG_VALU, (7 * SPS) / (2 * QB), 0);
            }
            if (s + PF < NS) __builtin_amdgcn_sched_group_barrier(SG_DSRD, 1, 0);
        }
        // keep the probabilities in this block (they are only consumed in phase B, and the
        // optimiser would otherwise sink their computation out of the MFMA shadow)
#pragma unroll
        for (int qb = 0; qb < QB; qb++) {
#pragma unroll
            for (int kb = 0; kb < KB; kb++) {
                PIN_V(P[qb][kb][0]);
                PIN_V(P[qb][kb][1]);
            }
            PIN_V(ls[qb]);
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int qb = 0; qb < QB; qb++) l_part[qb] += ls[qb];

        // ---- phase B: O += V(j)^T P  ||  row max of S(j+1) ----------------------------------------
        const int k0n = (j + 1) * BN;
        if (k0n + BN - 1 > wave_min_limit) mask_scores(Sn, k0n);
        __builtin_amdgcn_sched_barrier(0);
        float mx[QB];
#pragma unroll
        for (int qb = 0; qb < QB; qb++) mx[qb] = Sn[0][qb][0];
        bf16x8 vop[PF + 1];
#pragma unroll
        for (int s = 0; s < PF; s++) vop[s] = v_operand(vread, s);
#pragma unroll
        for (int s = 0; s < NS; s++) {
            if (s + PF < NS) vop[(s + PF) % (PF + 1)] = v_operand(vread, s + PF);
            const int kb = s / (2 * Gm::DB), u = (s / Gm::DB) & 1, db = s % Gm::DB;
#pragma unroll
            for (int qb = 0; qb < QB; qb++) {
#ifdef ABL_NOPV
                if (s == 0) O[db][qb][0] += (float)P[qb][kb][u][0] + (float)vop[s % (PF + 1)][0];
                continue;
#endif
                O[db][qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vop[s % (PF + 1)], P[qb][kb][u], O[db][qb], 0, 0, 0);
            }
#pragma unroll
            for (int t = 0; t < SPS; t++) {
                const int idx = s * SPS + t;
                const int qb = idx / 32, kb2 = (idx % 32) / 16, r = idx % 16;
                mx[qb] = fmaxf(mx[qb], Sn[kb2][qb][r]);
            }
        }
        __builtin_amdgcn_sched_group_barrier(SG_DSRD, 2 * PF, 1);
#pragma unroll
        for (int s = 0; s < NS; s++) {
#pragma unroll
            for (int qb = 0; qb < QB; qb++) {
                __builtin_amdgcn_sched_group_barrier(SG_MFMA, 1, 1);
                __builtin_amdgcn_sched_group_barrier(SG_VALU, (SPS + 3) / (2 * QB), 1);
            }
            if (s + PF < NS) __builtin_amdgcn_sched_group_barrier(SG_DSRD, 2, 1);
        }
#pragma unroll
        for (int qb = 0; qb < QB; qb++) PIN_V(mx[qb]);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int qb = 0; qb < QB; qb++) m_new[qb] = fmaxf(m_run[qb], xmax32(mx[qb]));
        pid1 = pid2;
        pid2 = pid3;
#ifndef ABL_NOBAR
        __builtin_amdgcn_s_waitcnt(0x0F70);               // vmcnt(0): K(j+2), V(j+1) are in LDS
        __syncthreads();
#endif
    };

    for (int j = 0; j < n_tiles; j += 2) {
        body(j, Sa, Sb, sK1, sV0, sK0, sV1);
        if (j + 1 < n_tiles) body(j + 1, Sb, Sa, sK0, sV1, sK1, sV0);
    }

    // ---- epilogue: normalise, round once to bf16, store -----------------------------------
    // register r of O[db] is MFMA row 8*(r/4) + 4*lh + r%4; rows 0-15 are d = 16*db + row,
    // rows 16-31 are d = D/2 + 16*db + (row - 16)
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
                    *(bf16x4 *)(op + 16 * db + 8 * (b4 & 1) + (D / 2) * (b4 >> 1)) = v;
                }
        }
    }
#endif
}

template <int D, int QB>
static hipError_t launch_one(const AttnParams &p, int G, int Gw, hipStream_t s) {
    const unsigned grid = (unsigned)p.n_tiles * (G / Gw) * p.Hkv;
    hipLaunchKernelGGL((attn_bf16_kernel<D, QB>), dim3(grid), dim3(256), 0, s, p, G, Gw);
    return hipGetLastError();
}

hipError_t launch_attn_bf16(const AttnParams &p, int head_dim, hipStream_t s) {
    if (p.n_tiles == 0) return hipSuccess;
    const int G = p.Hq / p.Hkv;
    const int Gw = G < 4 ? G : 4;
    if (query_blocks() == 1)
        return head_dim == 128 ? launch_one<128, 1>(p, G, Gw, s) : launch_one<64, 1>(p, G, Gw, s);
    return head_dim == 128 ? launch_one<128, 2>(p, G, Gw, s) : launch_one<64, 2>(p, G, Gw, s);
}

}  // namespace pbkv
