// bf16 prefix-reuse prefill attention for gfx950 (CDNA4): flash-style online softmax
// over KV tiles gathered page by page through the block table, QK^T and PV on the
// 32x32x16 bf16 MFMA, fp32 accumulation.
//
// Work decomposition
//   work-group = NW waves = (request, KV head, block of suffix tokens).  The query heads
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
//   K/V rows go from global memory straight into LDS (buffer_load_dwordx4 ... lds, 16
//   bytes per lane, 1 KiB contiguous in LDS per wave instruction) -- no staging registers
//   and no LDS store instructions.  Rows are unpadded; bank conflicts are avoided by an
//   XOR swizzle of the 16-byte chunk index that is applied on the global-address side:
//   the lane that owns LDS chunk position c' of row r fetches global chunk c'^swz(r).
//
// Software pipeline.  Measured on gfx950: the vector-ALU issue port, not the MFMA pipe,
// limits a wave that mixes both (each MFMA costs ~11 port cycles, each VALU op 4, each
// transcendental 8), so the softmax arithmetic is split evenly over the two MFMA phases:
//   phase A   S(j+1) = K(j+1) Q^T on the MFMA  ||  P(j) = exp2(t(j)), row sums, bf16 pack
//   phase B   O += V(j)^T P(j)    on the MFMA  ||  t(j+1) = S(j+1) c - M, row max of t
// where M is the running reference maximum in log2 units.  K runs one tile ahead of V,
// and the score registers ping-pong between two sets.  The reference is only moved
// (and O rescaled) when a row maximum exceeds it by more than 2^8.
#include "pbkv_internal.h"

#include <cstdio>
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
#ifndef PBKV_PF
#define PBKV_PF 3
#endif
constexpr int PF = PBKV_PF;    // LDS operand prefetch distance, in pipeline steps
constexpr float RESCALE_LOG2 = 8.0f;   // the reference maximum may lag by this much (log2)

template <int D, int NW>
struct Geom {
    static constexpr int DC = D / 16;         // contraction steps of QK^T per key block
    static constexpr int DB = D / 32;         // 32-row blocks of O^T
    static constexpr int NS = D / 8;          // pipeline steps per phase (KB*DC = KB*2*DB)
    static constexpr int ROWB = D * 2;        // bytes per K/V row
    static constexpr int TILEB = BN * ROWB;   // bytes per K or V tile
    static constexpr int CPR = D / 8;         // 16-byte chunks per row
    static constexpr int RPI = 64 / CPR;      // rows covered by one wave-wide 1 KiB load
    static constexpr int NI = BN / (NW * RPI);// loads per wave per tile
    static_assert(NI >= 1, "too many waves for this tile");
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

// Launch shape, "QN": Q = 32-row query blocks per wave, N = waves per work-group.
//   14: 4 waves x 32 rows, two work-groups per CU
//   18: 8 waves x 32 rows, two waves per SIMD share one set of K/V tiles (default)
//   24: 4 waves x 64 rows, one wave per SIMD
static int launch_shape() {
    static int v = [] {
        const char *e = getenv("PBKV_ATTN_SHAPE");
        const int x = e ? atoi(e) : 18;
        return (x == 14 || x == 24) ? x : 18;
    }();
    return v;
}

int attn_bf16_tile_tokens(int /*head_dim*/, int group) {
    const int gw = group < 4 ? group : 4;
    const int s = launch_shape();
    return 32 * (s / 10) * ((s % 10) / gw);
}

// Keeps a value (and so the code that computes it) at this point of the program; the
// constraint names a vector register, which only exists in the device pass.
#if defined(__HIP_DEVICE_COMPILE__)
#define PIN_V(x) asm volatile("" : "+v"(x))
#define PIN_A(x) asm volatile("" : "+a"(x))   // accumulation register: usable only by the MFMA
#else
#define PIN_V(x) (void)(x)
#define PIN_A(x) (void)(x)
#endif

// scheduling-group masks
#define SG_VALU 0x402   // VALU or transcendental
#define SG_MFMA 0x008
#define SG_DSRD 0x100

template <int D, int QB, int NW>
__global__ __launch_bounds__(64 * NW) __attribute__((amdgpu_waves_per_eu(3 - QB, 3 - QB)))
void attn_bf16_kernel(AttnParams p, int G, int Gw) {
#if defined(__HIP_DEVICE_COMPILE__)   // the body uses gfx950-only builtins and types; the host pass only needs the stub
    using Gm = Geom<D, NW>;
    constexpr int NS = Gm::NS;
    constexpr int NT = 64 * NW;
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
    const int tile_tok = WTOK * (NW / Gw);
    const int tok_base = td.tok0 + (w / Gw) * WTOK;
    const int tok_end = min(td.tok0 + tile_tok, td.new_len);
    // KV tiles: TP tiles over the cached prefix (the last may be partial), then tiles over
    // the suffix starting at its first token, so that every tile is read either through
    // the block table or from k_new / v_new, never both.
    const int TP = (td.prefix_len + BN - 1) / BN;
    const int n_tiles = TP + (tok_end + BN - 1) / BN;
    const int wave_min_tok = min(tok_base, td.new_len - 1);   // smallest token index in this wave

    const __bf16 *qg = (const __bf16 *)p.q;
    const __bf16 *kn = (const __bf16 *)p.k_new;
    const __bf16 *vn = (const __bf16 *)p.v_new;
    const __bf16 *pool = (const __bf16 *)p.kv_pool;
    const int32_t *bt = p.block_table + (int64_t)td.req * p.max_pages;

    // zero the V buffers once: rows past the last key are never loaded, and 0 * stale bits
    // must not be able to produce a NaN in the PV product
    for (int i = tid; i < Gm::TILEB / 16; i += NT) {
        *(uint4 *)(sV0 + i * 16) = make_uint4(0, 0, 0, 0);
        *(uint4 *)(sV1 + i * 16) = make_uint4(0, 0, 0, 0);
    }

    // ---- Q^T operands: lane (li, lh) holds Q[token li][16*dc + 8*lh .. +7] -------------
    bf16x8 qreg[QB][Gm::DC];
    int my_tokc[QB];                                      // this lane's token, clamped to the request
    int my_tok[QB];
#pragma unroll
    for (int qb = 0; qb < QB; qb++) {
        const int tr = tok_base + 32 * qb + li;
        my_tok[qb] = tr;
        const int tok = min(tr, td.new_len - 1);
        my_tokc[qb] = tok;
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
    // not change from tile to tile, so the gather costs no vector address arithmetic.  The
    // descriptor's size is the valid part of the row group: lanes of rows past the prefix
    // end / past the last visible token are out of range and read nothing.
    // Row group g = i*NW + w of a tile (i = 0..NI-1) holds rows g*RPI .. g*RPI + RPI-1.
    const int ld_lrow = l / Gm::CPR;                       // row inside this wave's row group
    const int ld_cpos = l % Gm::CPR;                       // chunk position this lane fills
    const int ld_slot = ((w * Gm::RPI) & 15) + ld_lrow;    // slot inside the page (same for all groups)
    const int ld_ck = ld_cpos ^ Gm::swz_k(w * Gm::RPI + ld_lrow);   // global chunk this lane fetches (K)
    const int ld_cv = ld_cpos ^ Gm::swz_v(w * Gm::RPI + ld_lrow);   // ... (V)
    const int row_pitch = p.Hkv * Gm::ROWB;                // bytes between suffix tokens
    const int voff_pk = ld_slot * Gm::ROWB + ld_ck * 16;
    const int voff_pv = ld_slot * Gm::ROWB + ld_cv * 16;
    const int voff_sk = ld_lrow * row_pitch + ld_ck * 16;
    const int voff_sv = ld_lrow * row_pitch + ld_cv * 16;
    const int page_bytes = 2 * p.Hkv * 16 * Gm::ROWB;
    const char *pool_k = (const char *)pool + (int64_t)kvh * 16 * Gm::ROWB;    // K rows of this head in page 0
    const char *pool_v = pool_k + (int64_t)p.Hkv * 16 * Gm::ROWB;             // V rows
    constexpr int RSRC_FLAGS = 0x00020000;                 // raw buffer, 32-bit data format
    // page (inside the tile) of row group i*NW + w: the NW groups of one pass cover
    // NW*RPI/16 consecutive pages, GPP groups per page
    constexpr int GPP = 16 / Gm::RPI;
    static_assert(NW % GPP == 0, "the waves of one pass cover whole pages");
    constexpr int RUN = NW / GPP;                          // pages per pass
    auto group_page = [&](const PageIds &pid, int i) {
        int pg = pid.v[(i * RUN) % (BN / 16)];
#pragma unroll
        for (int r = 1; r < RUN; r++)
            if (w / GPP == r) pg = pid.v[(i * RUN + r) % (BN / 16)];
        return pg;
    };
    // pass i (0..NI-1) of the gather of tile t into buf: this wave's row group i*NW + w
    auto load_group = [&](int t, const PageIds &pid, char *buf, const __bf16 *fresh, bool is_v, int i) {
        lds_void *dst = (lds_void *)(buf + (i * NW + w) * 1024);
        if (t < TP) {
            // rows of one of the logical pages 4t .. 4t+3, valid up to the prefix end
            const int lp = t * (BN / 16) + (i * RUN) % (BN / 16) + (w / GPP) % RUN;
            const int prows = max(td.prefix_len - lp * 16, 0);     // >= 16: the whole page (no lane reaches further)
            const char *pbase = (is_v ? pool_v : pool_k) + (int64_t)group_page(pid, i) * page_bytes;
            const auto rsrc = __builtin_amdgcn_make_buffer_rsrc((void *)pbase, 0, prows * Gm::ROWB, RSRC_FLAGS);
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, dst, 16, is_v ? voff_pv : voff_pk, 0, 0, 0);
            asm volatile("; rows from a prefix page");   // distinct block ends keep the two paths' loads apart
        } else {
            // RPI suffix tokens, valid up to the last visible token
            const int s0 = (t - TP) * BN + (i * NW + w) * Gm::RPI;
            const int srows = max(tok_end - s0, 0);                // >= RPI: the whole group
            const int sbytes = srows > 0 ? (srows - 1) * row_pitch + Gm::ROWB : 0;
            const char *sbase = (const char *)fresh + ((td.row0 + s0) * p.Hkv + kvh) * (int64_t)Gm::ROWB;
            const auto rsrc = __builtin_amdgcn_make_buffer_rsrc((void *)sbase, 0, sbytes, RSRC_FLAGS);
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, dst, 16, is_v ? voff_sv : voff_sk, 0, 0, 0);
            asm volatile("; rows from the suffix");
        }
    };
    auto load_tile = [&](int t, const PageIds &pid, char *buf, const __bf16 *fresh, bool is_v) {
#pragma unroll
        for (int i = 0; i < Gm::NI; i++) load_group(t, pid, buf, fresh, is_v, i);
    };

    // ---- running state --------------------------------------------------------------------
    f32x16 O[Gm::DB][QB];
#pragma unroll
    for (int db = 0; db < Gm::DB; db++)
#pragma unroll
        for (int qb = 0; qb < QB; qb++)
#pragma unroll
            for (int r = 0; r < 16; r++) O[db][qb][r] = 0.f;
    float M[QB], tmax[QB], l_part[QB];      // reference maximum (log2 units), max of pending t, row sum
#pragma unroll
    for (int qb = 0; qb < QB; qb++) { M[qb] = 0.f; tmax[qb] = 0.f; l_part[qb] = 0.f; }
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
    // Tile t holds prefix keys 64t.. (valid below the prefix end) or suffix tokens
    // 64(t-TP).. (valid up to the row's own token).  lim = last valid row of the tile for
    // this lane's query row; needs_mask is wave-uniform.
    auto needs_mask = [&](int t) {
        return t < TP ? (t + 1) * BN > td.prefix_len : (t - TP) * BN + BN - 1 > wave_min_tok;
    };
    auto mask_scores = [&](f32x16 (&S)[KB][QB], int t) {
#pragma unroll
        for (int qb = 0; qb < QB; qb++) {
            const int lim = t < TP ? td.prefix_len - 1 - t * BN : my_tokc[qb] - (t - TP) * BN;
            const int rel = lim - 4 * lh;
#pragma unroll
            for (int kb = 0; kb < KB; kb++)
#pragma unroll
                for (int r = 0; r < 16; r++)
                    if (32 * kb + 8 * (r >> 2) + (r & 3) > rel) S[kb][qb][r] = -INFINITY;
        }
    };

    // ---- prologue: K(0), V(0), K(1) into LDS; S(0), its row max, t(0) -------------------------
    PageIds pid1, pid2;                                   // page ids of tiles j+1 and j+2
    __syncthreads();                                      // V buffers zeroed
    {
        const PageIds pid0 = fetch_page_ids(0);
        pid1 = fetch_page_ids(1);
        pid2 = fetch_page_ids(2);
        load_tile(0, pid0, sK0, kn, false);
        load_tile(0, pid0, sV0, vn, true);
        load_tile(1, pid1, sK1, kn, false);
    }
    __builtin_amdgcn_s_waitcnt(0x0F70);                   // vmcnt(0): the loads have landed in LDS
    __syncthreads();
#ifdef PBKV_TRACE
    unsigned long long tr_acc[6] = {0, 0, 0, 0, 0, 0};
    unsigned long long tr_last = __builtin_amdgcn_s_memtime();
    const unsigned long long tr_t0 = tr_last, tr_r0 = __builtin_amdgcn_s_memrealtime();
#define TRACE_MARK(k) do { unsigned long long now_ = __builtin_amdgcn_s_memtime(); tr_acc[k] += now_ - tr_last; tr_last = now_; } while (0)
#else
#define TRACE_MARK(k) do {} while (0)
#endif
    if constexpr (QB == 2) {
    // ---- 32-key pipeline for the 64-column wave ------------------------------------------------
    // With 64 query columns per wave a 64-key score block is 64 registers, twice over for the
    // ping-pong; pipelining 32 keys at a time halves that, so the score pipeline, the Q
    // operands and the LDS operand windows fit the vector half of the register file while
    // the 128 output accumulators stay in the accumulation half.  Per 64-key tile there
    // are two sub-steps and two barriers: the second half of K(j) is consumed in the first
    // sub-step, after which its buffer is refilled with K(j+2).
    constexpr int NS2 = Gm::DC;                          // steps per phase (DC = 2*DB)
    constexpr int SPS2 = QB * 16 / NS2;                  // scores per lane per step
    static_assert(SPS2 % 2 == 0, "scores are converted in pairs");
    constexpr int WAIT_OLDER = 0x0F70 | (Gm::NI & 15);   // vmcnt(NI): all but the newest tile load have landed
    static_assert(Gm::NI < 16, "vmcnt immediate");
    f32x16 Ta[QB], Tb[QB];
    auto needs_mask_blk = [&](int t, int kb) {
        return t < TP ? t * BN + 32 * kb + 32 > td.prefix_len : (t - TP) * BN + 32 * kb + 31 > wave_min_tok;
    };
    auto mask_blk = [&](f32x16 (&S)[QB], int t, int kb) {
#pragma unroll
        for (int qb = 0; qb < QB; qb++) {
            const int lim = t < TP ? td.prefix_len - 1 - t * BN : my_tokc[qb] - (t - TP) * BN;
            const int rel = lim - 4 * lh - 32 * kb;
#pragma unroll
            for (int r = 0; r < 16; r++)
                if (8 * (r >> 2) + (r & 3) > rel) S[qb][r] = -INFINITY;
        }
    };
#pragma unroll
    for (int qb = 0; qb < QB; qb++)
#pragma unroll
        for (int r = 0; r < 16; r++) { Ta[qb][r] = 0.f; Tb[qb][r] = 0.f; }
#pragma unroll
    for (int dc = 0; dc < Gm::DC; dc++) {
        const bf16x8 a = k_operand(sK0, dc);
#pragma unroll
        for (int qb = 0; qb < QB; qb++)
            Ta[qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qreg[qb][dc], Ta[qb], 0, 0, 0);
    }
    if (needs_mask_blk(0, 0)) mask_blk(Ta, 0, 0);
#pragma unroll
    for (int qb = 0; qb < QB; qb++) {
        float mx0 = Ta[qb][0];                            // key 0 is visible to every row: finite
#pragma unroll
        for (int r = 1; r < 16; r++) mx0 = fmaxf(mx0, Ta[qb][r]);
        M[qb] = xmax32(mx0) * c;
#pragma unroll
        for (int r = 0; r < 16; r++) Ta[qb][r] = fmaf(Ta[qb][r], c, -M[qb]);
    }
    // one sub-step: Tc = pending t of a 32-key block; Tn receives the next block's scores
    // (block kbn of the tile in ksrc, tile index tn); the PV product uses block kbv of vsrc
    auto sub = [&](f32x16 (&Tc)[QB], f32x16 (&Tn)[QB], const char *ksrc, int kbn, int tn, const char *vsrc,
                   int kbv, auto &&issue_loads) __attribute__((always_inline)) {
#pragma unroll
        for (int db = 0; db < Gm::DB; db++)
#pragma unroll
            for (int qb = 0; qb < QB; qb++) PIN_A(O[db][qb]);
        TRACE_MARK(5);
        bool need = false;
#pragma unroll
        for (int qb = 0; qb < QB; qb++) need |= tmax[qb] > RESCALE_LOG2;
        if (__any(need)) {
#pragma unroll
            for (int qb = 0; qb < QB; qb++) {
                const float d = fmaxf(tmax[qb], 0.f);      // never lower the reference
                const float alpha = __builtin_amdgcn_exp2f(-d);
                M[qb] += d;
                l_part[qb] *= alpha;
#pragma unroll
                for (int db = 0; db < Gm::DB; db++)
#pragma unroll
                    for (int r = 0; r < 16; r++) O[db][qb][r] *= alpha;
#pragma unroll
                for (int r = 0; r < 16; r++) Tc[qb][r] -= d;
            }
        }
        float ls[QB];
#pragma unroll
        for (int qb = 0; qb < QB; qb++) ls[qb] = 0.f;
        bf16x8 P[QB][2];
        __builtin_amdgcn_sched_barrier(0);
#ifndef ABL_NOLOAD
        issue_loads();
#endif
        __builtin_amdgcn_sched_barrier(0);
        TRACE_MARK(0);
        __builtin_amdgcn_sched_barrier(0);
        // phase A: next block's S^T on the MFMA beside exp2 / row sum / bf16 pack of this block
        bf16x8 kop[PF + 1];
#pragma unroll
        for (int s = 0; s < PF; s++) kop[s] = k_operand(ksrc, kbn * Gm::DC + s);
#pragma unroll
        for (int s = 0; s < NS2; s++) {
            if (s + PF < NS2) kop[(s + PF) % (PF + 1)] = k_operand(ksrc, kbn * Gm::DC + s + PF);
#pragma unroll
            for (int qb = 0; qb < QB; qb++) {
                if (s == 0) {
                    f32x16 z;
#pragma unroll
                    for (int r = 0; r < 16; r++) z[r] = 0.f;
                    Tn[qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kop[s % (PF + 1)], qreg[qb][s], z, 0, 0, 0);
                } else {
                    Tn[qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kop[s % (PF + 1)], qreg[qb][s], Tn[qb], 0, 0, 0);
                }
            }
#pragma unroll
            for (int t = 0; t < SPS2; t += 2) {
                const int idx = s * SPS2 + t, qb = idx / 16, r = idx % 16;
                f32x2 pv;
                pv[0] = __builtin_amdgcn_exp2f(Tc[qb][r]);
                pv[1] = __builtin_amdgcn_exp2f(Tc[qb][r + 1]);
                ls[qb] += pv[0];
                ls[qb] += pv[1];
                const bf16x2 pk = __builtin_convertvector(pv, bf16x2);
                P[qb][r / 8][r % 8] = pk[0];
                P[qb][r / 8][r % 8 + 1] = pk[1];
            }
        }
        __builtin_amdgcn_sched_group_barrier(SG_DSRD, PF, 0);
#pragma unroll
        for (int s = 0; s < NS2; s++) {
#pragma unroll
            for (int qb = 0; qb < QB; qb++) {
                __builtin_amdgcn_sched_group_barrier(SG_MFMA, 1, 0);
                __builtin_amdgcn_sched_group_barrier(SG_VALU, (5 * SPS2) / (2 * QB), 0);
            }
            if (s + PF < NS2) __builtin_amdgcn_sched_group_barrier(SG_DSRD, 1, 0);
        }
#pragma unroll
        for (int qb = 0; qb < QB; qb++) {
            PIN_V(P[qb][0]);
            PIN_V(P[qb][1]);
            PIN_V(ls[qb]);
        }
        __builtin_amdgcn_sched_barrier(0);
        TRACE_MARK(1);
#pragma unroll
        for (int qb = 0; qb < QB; qb++) l_part[qb] += ls[qb];
        // phase B: O += V^T P on the MFMA beside t = S c - M and its row max for the next block
        if (needs_mask_blk(tn, kbn)) mask_blk(Tn, tn, kbn);
        __builtin_amdgcn_sched_barrier(0);
        TRACE_MARK(2);
        __builtin_amdgcn_sched_barrier(0);
        float mx[QB];
#pragma unroll
        for (int qb = 0; qb < QB; qb++) mx[qb] = -INFINITY;
        bf16x8 vop[PF + 1];
#pragma unroll
        for (int s = 0; s < PF; s++) vop[s] = v_operand(vsrc, kbv * 2 * Gm::DB + s);
#pragma unroll
        for (int s = 0; s < NS2; s++) {
            if (s + PF < NS2) vop[(s + PF) % (PF + 1)] = v_operand(vsrc, kbv * 2 * Gm::DB + s + PF);
            const int u = s / Gm::DB, db = s % Gm::DB;
#pragma unroll
            for (int qb = 0; qb < QB; qb++)
                O[db][qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vop[s % (PF + 1)], P[qb][u], O[db][qb], 0, 0, 0);
#pragma unroll
            for (int t = 0; t < SPS2; t++) {
                const int idx = s * SPS2 + t, qb = idx / 16, r = idx % 16;
                const float tv = fmaf(Tn[qb][r], c, -M[qb]);
                Tn[qb][r] = tv;
                mx[qb] = fmaxf(mx[qb], tv);
            }
        }
        __builtin_amdgcn_sched_group_barrier(SG_DSRD, 2 * PF, 1);
#pragma unroll
        for (int s = 0; s < NS2; s++) {
#pragma unroll
            for (int qb = 0; qb < QB; qb++) {
                __builtin_amdgcn_sched_group_barrier(SG_MFMA, 1, 1);
                __builtin_amdgcn_sched_group_barrier(SG_VALU, (3 * SPS2) / (2 * QB), 1);
            }
            if (s + PF < NS2) __builtin_amdgcn_sched_group_barrier(SG_DSRD, 2, 1);
        }
#pragma unroll
        for (int qb = 0; qb < QB; qb++) {
            PIN_V(mx[qb]);
            PIN_V(Tn[qb]);
        }
        __builtin_amdgcn_sched_barrier(0);
        TRACE_MARK(3);
#pragma unroll
        for (int qb = 0; qb < QB; qb++) tmax[qb] = xmax32(mx[qb]);
    };
    auto tile_iter = [&](int j, char *kcur, char *knext, char *vcur, char *vnext) __attribute__((always_inline)) {
        const PageIds pid3 = fetch_page_ids(j + 3);
        // keys 0-31 of tile j are pending in Ta; S(j, keys 32-63) comes from kcur
        sub(Ta, Tb, kcur, 1, j, vcur, 0, [&] { load_tile(j + 1, pid1, vnext, vn, true); });
        __builtin_amdgcn_s_waitcnt(WAIT_OLDER);          // K(j+1) has landed; V(j+1) may be in flight
        __syncthreads();                                  // ... and every wave is done with kcur
        TRACE_MARK(4);
        sub(Tb, Ta, knext, 0, j + 1, vcur, 1, [&] { load_tile(j + 2, pid2, kcur, kn, false); });
        __builtin_amdgcn_s_waitcnt(WAIT_OLDER);          // V(j+1) has landed; K(j+2) may be in flight
        __syncthreads();
        TRACE_MARK(4);
        pid1 = pid2;
        pid2 = pid3;
    };
    for (int j = 0; j < n_tiles; j += 2) {
        tile_iter(j, sK0, sK1, sV0, sV1);
        if (j + 1 < n_tiles) tile_iter(j + 1, sK1, sK0, sV1, sV0);
    }
    __builtin_amdgcn_s_waitcnt(0x0F70);                   // nothing may still be writing LDS at exit
    } else {
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
    if (needs_mask(0)) mask_scores(Sa, 0);
#pragma unroll
    for (int qb = 0; qb < QB; qb++) {
        // key 0 is visible to every row, so the first tile's row maximum is finite
        float mx = Sa[0][qb][0];
#pragma unroll
        for (int kb = 0; kb < KB; kb++)
#pragma unroll
            for (int r = 0; r < 16; r++) mx = fmaxf(mx, Sa[kb][qb][r]);
        M[qb] = xmax32(mx) * c;
#pragma unroll
        for (int kb = 0; kb < KB; kb++)
#pragma unroll
            for (int r = 0; r < 16; r++) Sa[kb][qb][r] = fmaf(Sa[kb][qb][r], c, -M[qb]);
    }

    // ---- one pipelined iteration: tile j; Tc = t(j) ready; Tn receives S(j+1), then t(j+1) ----
    auto body = [&](int j, f32x16 (&Tc)[KB][QB], f32x16 (&Tn)[KB][QB], char *kread, char *vread,
                    char *kwrite, char *vwrite) __attribute__((always_inline)) {
        // move the reference only when a row maximum ran ahead of it by more than 2^8
        TRACE_MARK(5);
        bool need = false;
#pragma unroll
        for (int qb = 0; qb < QB; qb++) need |= tmax[qb] > RESCALE_LOG2;
        if (__any(need)) {
#pragma unroll
            for (int qb = 0; qb < QB; qb++) {
                const float d = fmaxf(tmax[qb], 0.f);      // never lower the reference
                const float alpha = __builtin_amdgcn_exp2f(-d);
                M[qb] += d;
                l_part[qb] *= alpha;
#pragma unroll
                for (int db = 0; db < Gm::DB; db++)
#pragma unroll
                    for (int r = 0; r < 16; r++) O[db][qb][r] *= alpha;
#pragma unroll
                for (int kb = 0; kb < KB; kb++)
#pragma unroll
                    for (int r = 0; r < 16; r++) Tc[kb][qb][r] -= d;
            }
        }
        // prefetch: page ids three tiles ahead, K two tiles ahead, V one tile ahead
        const PageIds pid3 = fetch_page_ids(j + 3);
        float ls[QB];
#pragma unroll
        for (int qb = 0; qb < QB; qb++) ls[qb] = 0.f;
        bf16x8 P[QB][KB][2];

        // ---- phase A: S(j+1) = K(j+1) Q^T  ||  P = exp2(t(j)), row sums ---------------------------
        // The phase is cut into (up to) four scheduling regions, each preceded by one or two
        // wave-wide loads of the coming tiles (the NI row groups of K(j+2), then those of
        // V(j+1)).  A burst of loads from every wave of the CU queues behind the 64 B/clk
        // vector-memory port and stalls the issuing waves; a load every few MFMAs is absorbed
        // in the background.  (Shorter regions than four steps cost more than they save.)
        constexpr int LPR = NW == 4 ? Gm::NI : (2 * Gm::NI > 4 ? 2 * Gm::NI / 4 : 1);    // loads in front of each region
        constexpr int NREG = 2 * Gm::NI / LPR, RS = NS / NREG;
        static_assert(NS % NREG == 0 && (2 * Gm::NI) % LPR == 0, "regions hold whole steps");
        bf16x8 kop[PF + 1];
#pragma unroll
        for (int rg = 0; rg < NREG; rg++) {
            __builtin_amdgcn_sched_barrier(0);
#ifndef ABL_NOLOAD
#pragma unroll
            for (int q = rg * LPR; q < (rg + 1) * LPR; q++) {
                if (q < Gm::NI) load_group(j + 2, pid2, kwrite, kn, false, q);
                else load_group(j + 1, pid1, vwrite, vn, true, q - Gm::NI);
            }
#endif
            __builtin_amdgcn_sched_barrier(0);
            const int s0 = rg * RS, s1 = s0 + RS;
            if (rg == 0) {
#pragma unroll
                for (int s = 0; s < PF; s++) kop[s] = k_operand(kread, s);
            }
#pragma unroll
            for (int s = s0; s < s1; s++) {
                if (s + PF < NS) kop[(s + PF) % (PF + 1)] = k_operand(kread, s + PF);
                const int kb = s / Gm::DC, dc = s % Gm::DC;
#pragma unroll
                for (int qb = 0; qb < QB; qb++) {
                    if (dc == 0) {
                        f32x16 z;
#pragma unroll
                        for (int r = 0; r < 16; r++) z[r] = 0.f;
                        Tn[kb][qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kop[s % (PF + 1)], qreg[qb][dc], z, 0, 0, 0);
                    } else {
                        Tn[kb][qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kop[s % (PF + 1)], qreg[qb][dc], Tn[kb][qb], 0, 0, 0);
                    }
                }
#pragma unroll
                for (int t = 0; t < SPS; t += 2) {
                    const int idx = s * SPS + t;              // flattened (qb, kb, r)
                    const int qb = idx / 32, kb2 = (idx % 32) / 16, r = idx % 16;
                    f32x2 pv;
                    pv[0] = __builtin_amdgcn_exp2f(Tc[kb2][qb][r]);
                    pv[1] = __builtin_amdgcn_exp2f(Tc[kb2][qb][r + 1]);
                    ls[qb] += pv[0];
                    ls[qb] += pv[1];
                    const bf16x2 pk = __builtin_convertvector(pv, bf16x2);
                    P[qb][kb2][r / 8][r % 8] = pk[0];
                    P[qb][kb2][r / 8][r % 8 + 1] = pk[1];
                }
            }
            // interleave: per MFMA its share of the exp work, one K operand read per step
            if (rg == 0) __builtin_amdgcn_sched_group_barrier(SG_DSRD, PF, 0);
#pragma unroll
            for (int s = s0; s < s1; s++) {
#pragma unroll
                for (int qb = 0; qb < QB; qb++) {
                    __builtin_amdgcn_sched_group_barrier(SG_MFMA, 1, 0);
                    __builtin_amdgcn_sched_group_barrier(SG_VALU, (5 * SPS) / (2 * QB), 0);
                }
                if (s + PF < NS) __builtin_amdgcn_sched_group_barrier(SG_DSRD, 1, 0);
            }
            // keep this region's probabilities, row sums and prefetched operands in this block
            // (the probabilities are only consumed in phase B, and the optimiser would otherwise
            // sink their computation out of the MFMA shadow)
#pragma unroll
            for (int idx = s0 * SPS; idx < s1 * SPS; idx += 2) {
                const int qb = idx / 32, kb2 = (idx % 32) / 16, u = (idx % 16) / 8;
                if (idx % 8 == 0 || idx == s0 * SPS) PIN_V(P[qb][kb2][u]);
            }
#pragma unroll
            for (int qb = 0; qb < QB; qb++) PIN_V(ls[qb]);
            if (rg + 1 < NREG) {
#pragma unroll
                for (int s = 0; s < PF + 1; s++) PIN_V(kop[s]);
            }
        }
        __builtin_amdgcn_sched_barrier(0);
        TRACE_MARK(1);
#pragma unroll
        for (int qb = 0; qb < QB; qb++) l_part[qb] += ls[qb];

        // ---- phase B: O += V(j)^T P  ||  t(j+1) = S(j+1) c - M and its row max --------------------
        if (needs_mask(j + 1)) mask_scores(Tn, j + 1);
        __builtin_amdgcn_sched_barrier(0);
        TRACE_MARK(2);
        __builtin_amdgcn_sched_barrier(0);
        float mx[QB];
#pragma unroll
        for (int qb = 0; qb < QB; qb++) mx[qb] = -INFINITY;
        bf16x8 vop[PF + 1];
#pragma unroll
        for (int s = 0; s < PF; s++) vop[s] = v_operand(vread, s);
#pragma unroll
        for (int s = 0; s < NS; s++) {
            if (s + PF < NS) vop[(s + PF) % (PF + 1)] = v_operand(vread, s + PF);
            const int kb = s / (2 * Gm::DB), u = (s / Gm::DB) & 1, db = s % Gm::DB;
#pragma unroll
            for (int qb = 0; qb < QB; qb++)
                O[db][qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vop[s % (PF + 1)], P[qb][kb][u], O[db][qb], 0, 0, 0);
#pragma unroll
            for (int t = 0; t < SPS; t++) {
                const int idx = s * SPS + t;
                const int qb = idx / 32, kb2 = (idx % 32) / 16, r = idx % 16;
                const float tv = fmaf(Tn[kb2][qb][r], c, -M[qb]);
                Tn[kb2][qb][r] = tv;
                mx[qb] = fmaxf(mx[qb], tv);
            }
        }
        __builtin_amdgcn_sched_group_barrier(SG_DSRD, 2 * PF, 1);
#pragma unroll
        for (int s = 0; s < NS; s++) {
#pragma unroll
            for (int qb = 0; qb < QB; qb++) {
                __builtin_amdgcn_sched_group_barrier(SG_MFMA, 1, 1);
                __builtin_amdgcn_sched_group_barrier(SG_VALU, (3 * SPS) / (2 * QB), 1);
            }
            if (s + PF < NS) __builtin_amdgcn_sched_group_barrier(SG_DSRD, 2, 1);
        }
#pragma unroll
        for (int qb = 0; qb < QB; qb++) {
            PIN_V(mx[qb]);
#pragma unroll
            for (int kb = 0; kb < KB; kb++) PIN_V(Tn[kb][qb]);
        }
        __builtin_amdgcn_sched_barrier(0);
        TRACE_MARK(3);
#pragma unroll
        for (int qb = 0; qb < QB; qb++) tmax[qb] = xmax32(mx[qb]);
        pid1 = pid2;
        pid2 = pid3;
#ifndef ABL_NOBAR
        __builtin_amdgcn_s_waitcnt(0x0F70);               // vmcnt(0): K(j+2), V(j+1) are in LDS
        __syncthreads();
#endif
        TRACE_MARK(4);
    };

    for (int j = 0; j < n_tiles; j += 2) {
        body(j, Sa, Sb, sK1, sV0, sK0, sV1);
        if (j + 1 < n_tiles) body(j + 1, Sb, Sa, sK0, sV1, sK1, sV0);
    }
    }   // 64-key pipeline

#ifdef PBKV_TRACE
    if (p.trace && l == 0 && w == 0 && blockIdx.x < 4096) {
        unsigned long long *sp = (unsigned long long *)p.trace + 64 * 8 * 8 + blockIdx.x * 2;
        sp[0] = tr_r0;
        sp[1] = __builtin_amdgcn_s_memrealtime();
    }
    if (p.trace && l == 0 && blockIdx.x < 64) {
        unsigned long long *tp = (unsigned long long *)p.trace + (blockIdx.x * NW + w) * 8;
        for (int k = 0; k < 6; k++) tp[k] = tr_acc[k];
        tp[6] = n_tiles;
        tp[7] = ((__builtin_amdgcn_s_memtime() - tr_t0) << 24) | ((__builtin_amdgcn_s_memrealtime() - tr_r0) & 0xffffff);
    }
#endif
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

template <int D, int QB, int NW>
static hipError_t launch_one(const AttnParams &p, int G, int Gw, hipStream_t s) {
    const unsigned grid = (unsigned)p.n_tiles * (G / Gw) * p.Hkv;
    hipLaunchKernelGGL((attn_bf16_kernel<D, QB, NW>), dim3(grid), dim3(64 * NW), 0, s, p, G, Gw);
    return hipGetLastError();
}

#ifdef PBKV_TRACE
static void trace_dump(void *dev, int nw) {
    static int calls = 0;
    if (++calls != 3) return;
    hipDeviceSynchronize();
    static unsigned long long h[64 * 8 * 8 + 8192];
    hipMemcpy(h, dev, sizeof h, hipMemcpyDeviceToHost);
    {
        unsigned long long *sp = h + 64 * 8 * 8, t0 = ~0ull, t1 = 0; int nb = 0;
        for (int b = 0; b < 4096; b++) if (sp[2 * b]) { nb++; if (sp[2 * b] < t0) t0 = sp[2 * b]; if (sp[2 * b + 1] > t1) t1 = sp[2 * b + 1]; }
        int late = 0; double sum_life = 0;
        for (int b = 0; b < 4096; b++) if (sp[2 * b]) { if (sp[2 * b] - t0 > 2000) late++; sum_life += sp[2 * b + 1] - sp[2 * b]; }
        printf("trace: %d blocks, span %.1f us, mean block life %.1f us, blocks starting >20us late: %d\n", nb, (t1 - t0) / 100.0, sum_life / nb / 100.0, late);
        for (int b = 0; b < nb; b += nb / 16) printf("  block %d start %.1f end %.1f\n", b, (sp[2 * b] - t0) / 100.0, (sp[2 * b + 1] - t0) / 100.0);
    }
    const char *names[6] = {"top+loads", "phaseA", "between", "phaseB", "tail+barrier", "loop-carry"};
    for (int b = 0; b < 64; b += 21)
        for (int w = 0; w < nw; w += 3) {
            unsigned long long *t = h + (b * nw + w) * 8;
            printf("trace block %d wave %d tiles %llu:", b, w, t[6]);
            for (int k = 0; k < 6; k++) printf(" %s=%.0f", names[k], t[6] ? (double)t[k] / t[6] : 0.0);
            printf(" | life %llu ticks, %.1f us real, clock %.2f GHz", t[7] >> 24, (t[7] & 0xffffff) / 100.0, (t[7] >> 24) / ((t[7] & 0xffffff) * 10.0));
            printf("\n");
        }
}
#endif

hipError_t launch_attn_bf16(const AttnParams &p0, int head_dim, hipStream_t s) {
    AttnParams p = p0;
#ifdef PBKV_TRACE
    static void *trace_buf = nullptr;
    if (!trace_buf) { hipMalloc(&trace_buf, (64 * 8 * 8 + 8192) * 8); hipMemset(trace_buf, 0, (64 * 8 * 8 + 8192) * 8); }
    p.trace = trace_buf;
    struct Dump { void *b; int nw; ~Dump() { trace_dump(b, nw); } } dump{trace_buf, launch_shape() % 10};
#endif
    if (p.n_tiles == 0) return hipSuccess;
    const int G = p.Hq / p.Hkv;
    const int Gw = G < 4 ? G : 4;
    switch (launch_shape()) {
        case 14: return head_dim == 128 ? launch_one<128, 1, 4>(p, G, Gw, s) : launch_one<64, 1, 4>(p, G, Gw, s);
        case 24: return head_dim == 128 ? launch_one<128, 2, 4>(p, G, Gw, s) : launch_one<64, 2, 4>(p, G, Gw, s);
        default: return head_dim == 128 ? launch_one<128, 1, 8>(p, G, Gw, s) : launch_one<64, 1, 8>(p, G, Gw, s);
    }
}

}  // namespace pbkv
