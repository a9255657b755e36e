// bf16 prefix-reuse prefill attention for gfx950 (CDNA4): flash-style online softmax
// over KV tiles gathered page by page through the block table, QK^T and PV on the
// 32x32x16 bf16 MFMA, fp32 accumulation.
//
// Work decomposition
//   work-group = NW waves = (request, KV head, block of suffix tokens).  The query heads
//   of a GQA group share every K/V tile staged in LDS: wave w takes query head
//   w % Gw (Gw = min(G,4)) and token sub-block w / Gw, 32 tokens per wave.
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
//   and no LDS store instructions.  Wave w fetches rows [w*RW, (w+1)*RW) of every tile
//   (RW = 64/NW, a part of ONE page), so a tile costs a wave one buffer descriptor and
//   RW*D/512 load instructions that differ only in their immediate offset (which moves
//   the global and the LDS address alike).  Rows are unpadded; bank conflicts are avoided
//   by an XOR swizzle of the 16-byte chunk index that is applied on the global-address
//   side: the lane that owns LDS chunk position c' of row r fetches global chunk c'^swz(r).
//
// Software pipeline.  A wave issues one instruction per 4-cycle slot and an MFMA occupies
// the matrix pipe for 32 cycles, so the instruction count per MFMA -- and in particular
// the vector-ALU count, since MFMA and VALU share one issue port -- decides whether the
// matrix pipe stays fed.  Hence:
//   * the scale log2(e)/sqrt(D) is folded into Q once, and the score MFMA chain starts
//     from -M (M = running reference maximum, log2 units) instead of 0: the accumulator
//     holds t = s - M directly and the softmax costs one exp2 per score, plus half a
//     bf16 pack and half a dot2 (row sum of the ROUNDED probabilities).  The dot2 runs in
//     the matrix pipe's order: one placed between two MFMAs holds the second one back
//     until it has gone through, so the eight of a block are issued together, after the
//     block's last MFMA, where they cost one such gap instead of eight;
//   * that arithmetic is dealt out evenly over ALL MFMAs by working on 32-key blocks with
//     the PV product two blocks behind the score product.  Iteration b:
//         first half   t(b+1) = K(b+1) Q^T - M   on the MFMA  ||  exp2 of half of t(b)
//         second half  O += V(b-1)^T P(b-1)      on the MFMA  ||  other half, row max of t(b+1)
//   * tile loads are spread over the first halves, one every few MFMAs.
// A 64-key tile step is two iterations; it reads only K(j) and V(j-1), so two LDS buffers
// of each suffice while K(j+1) and V(j) are in flight.  The reference M is moved (and O
// rescaled, one iteration later, once the product formed under the old M has been added)
// only when a row maximum exceeds it by more than 2^8.
#include "pbkv_internal.h"

#include <algorithm>
#include <atomic>
#include <utility>

namespace pbkv {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((address_space(3))) bf16x4 lds_bf16x4;
typedef __attribute__((address_space(3))) void lds_void;

constexpr int BN = 64;   // keys per LDS tile (two 32-key blocks)
constexpr int PF = 3;    // LDS operand prefetch distance, in MFMA steps
[[maybe_unused]] constexpr float RESCALE_SUM = 4096.0f;  // a lane's probability sum over one block above this moves the reference

template <int D, int NW>
struct Geom {
    static constexpr int DC = D / 16;         // contraction steps of QK^T per key block
    static constexpr int DB = D / 32;         // 32-row blocks of O^T
    static constexpr int H = DC;              // MFMA steps per half iteration (DC = 2*DB)
    static constexpr int ROWB = D * 2;        // bytes per K/V row
    static constexpr int TILEB = BN * ROWB;   // bytes per K or V tile
    static constexpr int CPR = D / 8;         // 16-byte chunks per row
    static constexpr int RPI = 64 / CPR;      // rows covered by one wave-wide 1 KiB load
    static constexpr int RW = BN / NW;        // tile rows gathered by one wave
    static constexpr int NI = RW / RPI;       // loads per wave per tile
    static_assert(RW % RPI == 0 && NI >= 1, "a wave loads whole 1 KiB row groups");
    static_assert(16 % RW == 0, "a wave's rows of a tile lie in one page");
    static_assert(H % NI == 0 && PF < 4 * H, "loads and operand prefetch fit the tile step");
    // XOR applied to the chunk index of row `row` (conflict-free ds_read_b128 of 16
    // consecutive rows for K; conflict-free 4-row x 32-byte transposing reads for V)
    static __device__ __forceinline__ int swz_k(int row) { return D == 128 ? (row & 15) : ((row >> 1) & 7); }
    static __device__ __forceinline__ int swz_v(int row) { return D == 128 ? ((row & 7) << 1) : (((row >> 1) & 3) << 1); }
};

template <int I> struct IntC { static constexpr int value = I; };
template <class F, int... Is>
static __device__ __forceinline__ void static_for(F &&f, std::integer_sequence<int, Is...>) { (f(IntC<Is>{}), ...); }

[[maybe_unused]] static __device__ __forceinline__ float xmax32(float x) {
    auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
[[maybe_unused]] static __device__ __forceinline__ float xsum32(float x) {
    auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

// Three shapes of work-group.
//   4 waves, 32 rows each:  two work-groups per CU, each staging its own K/V tiles.  They overlap one
//       work-group's prologue and epilogue (dependent fetches before the first tile step, the output
//       stores after the last) with the other's arithmetic and cut the work twice as fine: the shape
//       for short work units.
//   8 waves, 32 rows each:  one work-group per CU, two waves per SIMD sharing one set of tiles.
//   64 (four waves of 64 rows each, attn_bf16_w64_kernel below): one wave per SIMD; every LDS operand
//       feeds two MFMAs and a tile is staged once per 256 rows, so a tile step reads half the LDS
//       bytes per FLOP of either 32-row shape and stages as the 8-wave shape does (half of what
//       the 4-wave shape stages).  The chip is power-limited under this
//       kernel, so that is speed: measured against the better of the other two, under sustained
//       load, -1 % / -1.5 % / +4.5 % / +3 % on launches whose 64-token blocks average 37 / 70 / 152 /
//       545 tile steps.  The switch from 4 waves is at 100.
// attn_bf16_force_waves(4|8|64) overrides the choice for the whole process (0: automatic).
static std::atomic<int> g_forced_waves{0};
void attn_bf16_force_waves(int waves) { g_forced_waves.store(waves == 4 || waves == 8 || waves == 64 ? waves : 0); }
int attn_bf16_forced_waves() { return g_forced_waves.load(); }

int attn_bf16_waves(const int32_t *prefix_lens, const int32_t *new_lens, int batch) {
    const int forced = g_forced_waves.load();
    if (forced == 4 || forced == 8 || forced == 64) return forced;
    int64_t steps = 0, blocks = 0;
    for (int r = 0; r < batch; r++) {
        const int64_t tp = (prefix_lens[r] + BN - 1) / BN;
        for (int t0 = 0; t0 < new_lens[r]; t0 += 64) {
            steps += tp + (std::min(t0 + 64, new_lens[r]) + BN - 1) / BN + 1;
            blocks++;
        }
    }
    return blocks > 0 && steps < 100 * blocks ? 4 : 64;
}

int attn_bf16_tile_tokens(int /*head_dim*/, int group, int waves) {
    const int gw = group < 4 ? group : 4;
    return 32 * ((waves == 64 ? 8 : waves) / gw);     // the 64-row form cuts the suffix as the eight-wave form does
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
#define SG_VMRD 0x020
#define SG_DSRD 0x100

// Two waves share a SIMD's issue port, and the arbiter serves the older wave first: its softmax
// arithmetic would keep the younger wave's MFMAs off the matrix pipe.  Every MFMA is therefore
// issued at raised wave priority, so that a waiting MFMA of either wave goes before VALU work.
#define MFMA_PRIO(x) __builtin_amdgcn_s_setprio(x)

// PROBE = true builds the gather diagnostic: the same work units, block-table walk, buffer
// descriptors, loads into LDS and barriers, but instead of the arithmetic every wave XORs the
// 32-bit words of the valid rows it finds staged, and the work-group stores one word.
template <int D, int NW, bool PROBE>
__global__ __launch_bounds__(64 * NW) __attribute__((amdgpu_waves_per_eu(2, 2)))
void attn_bf16_kernel(AttnParams p, int G, int Gw) {
#if defined(__HIP_DEVICE_COMPILE__)   // the body uses gfx950-only builtins and types; the host pass only needs the stub
    using Gm = Geom<D, NW>;
    constexpr int H = Gm::H;
    constexpr int NT = 64 * NW;
    constexpr int ROWB = Gm::ROWB;

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
    // a launch that read its work list from the host's descriptor ring leaves a copy in device
    // memory for later launches over the same batch
    if (p.mirror != nullptr && kvh == 0 && split == 0 && tid == 0) p.mirror[rest / nsplit] = td;
    const int head = kvh * G + split * Gw + (w % Gw);
    const int tile_tok = 32 * (NW / Gw);
    const int tok_base = td.tok0 + (w / Gw) * 32;
    const int tok_end = min(td.tok0 + tile_tok, td.new_len);
    // KV tiles: TP tiles over the cached prefix (the last may be partial), then tiles over
    // the suffix starting at its first token, so that every tile is read either through
    // the block table or from k_new / v_new, never both.
    const int TP = (td.prefix_len + BN - 1) / BN;
    const int TPF = td.prefix_len / BN;                    // full prefix tiles
    const int n_tiles = TP + (tok_end + BN - 1) / BN;
    const int wave_min_tok = min(tok_base, td.new_len - 1);   // smallest token index in this wave

    // ---- Q^T operands, pre-scaled: lane (li, lh) holds c * Q[token li][16*dc + 8*lh .. +7] ----
    // c = log2(e)/sqrt(D), so the MFMA result is the score in log2 units (Eq. softmax(QK^T/sqrt(d)))
    const float c = 1.4426950408889634f * rsqrtf((float)D);
    bf16x8 qreg[Gm::DC];
    const int my_tok = tok_base + li;
    const int my_tokc = min(my_tok, td.new_len - 1);      // clamped to the request
    {
        const __bf16 *qp = (const __bf16 *)p.q + ((td.row0 + my_tokc) * p.Hq + head) * D + 8 * lh;
#pragma unroll
        for (int dc = 0; dc < Gm::DC; dc++) {
            const bf16x8 raw = *(const bf16x8 *)(qp + dc * 16);
#pragma unroll
            for (int e = 0; e < 8; e++) qreg[dc][e] = (__bf16)((float)raw[e] * c);
        }
    }

    // ---- tile sources ---------------------------------------------------------------------
    // Block-table entries are held 64 at a time (16 tiles) in one vector register, lane i =
    // logical page 64*blk + i, clamped to the pool; the block after the current one is
    // loaded 16 tiles early, so a page id is one lane read into a scalar register.
    constexpr int PPT = BN / 16;                           // pages per tile
    const int pw = (w * Gm::RW) >> 4;                      // page (inside a tile) of this wave's rows
    const int slot0 = (w * Gm::RW) & 15;                   // first slot of this wave's rows in that page
    const int32_t *bt = p.block_table + (int64_t)td.req * p.max_pages;
    const int n_prefix_pages = (td.prefix_len + 15) >> 4;
    auto load_id_block = [&](int blk) {
        const int lp = blk * 64 + l;
        int pg = lp < n_prefix_pages ? bt[lp] : 0;
        pg = pg < 0 ? 0 : (pg >= p.num_pages ? p.num_pages - 1 : pg);
        return pg;
    };
    int ids_cur = load_id_block(0), ids_next = load_id_block(1);
    // The source of a wave's rows of tile t is a raw buffer: a wave-uniform descriptor (page
    // base, or the suffix row base; size = the valid part, so lanes of rows past the prefix
    // end / past the last visible token are out of range and read nothing) plus per-lane
    // byte offsets that never change.  Tiles are asked for in ascending order.
    struct Src { const char *k, *v; int nrec; };
    const int row_pitch = p.Hkv * ROWB;                    // bytes between suffix tokens
    const int64_t page_bytes = 2 * (int64_t)p.Hkv * 16 * ROWB;
    const int64_t v_in_page = (int64_t)p.Hkv * 16 * ROWB;   // V rows follow the K rows of all heads
    const char *pool_k = (const char *)p.kv_pool + (int64_t)kvh * 16 * ROWB;   // K rows of this head in page 0
    const char *kn_h = (const char *)p.k_new + (int64_t)kvh * ROWB;
    const char *vn_h = (const char *)p.v_new + (int64_t)kvh * ROWB;
    auto tile_src = [&](int t) {
        Src s;
        if (t < TP) {
            if (__builtin_expect((t & 15) == 0 && t > 0, 0)) {
                ids_cur = ids_next;
                ids_next = load_id_block((t >> 4) + 1);
            }
            const int pg = __builtin_amdgcn_readlane(ids_cur, (t & 15) * PPT + pw);
            // only the last prefix tile can hold a partly filled (or unused) page
            const int rows = t < TP - 1 ? 16 : max(td.prefix_len - (t * PPT + pw) * 16, 0);
            s.k = pool_k + pg * page_bytes;
            s.v = s.k + v_in_page;
            s.nrec = rows * ROWB;
            asm volatile("; source: prefix page");
        } else {
            const int s0 = (t - TP) * BN + w * Gm::RW;         // first suffix token of this wave's rows
            const int srows = min(tok_end - s0, Gm::RW);       // the wave's own rows (no lane reaches further)
            const int64_t off = (td.row0 + s0) * (int64_t)row_pitch;
            s.k = kn_h + off;
            s.v = vn_h + off;
            s.nrec = srows > 0 ? (srows - 1) * row_pitch + ROWB : 0;
            asm volatile("; source: suffix rows");
        }
        return s;
    };
    // per-lane byte offsets of load i (rows w*RW + i*RPI + l/CPR of the tile); the instruction's
    // immediate offset i*1024 moves both addresses, so the suffix offsets take it back out
    int vk_p[Gm::NI], vk_s[Gm::NI], vv_p[Gm::NI], vv_s[Gm::NI];
    {
        const int lrow = l / Gm::CPR, cpos = l % Gm::CPR;
#pragma unroll
        for (int i = 0; i < Gm::NI; i++) {
            const int row = w * Gm::RW + i * Gm::RPI + lrow;
            const int ck = (cpos ^ Gm::swz_k(row)) << 4, cv = (cpos ^ Gm::swz_v(row)) << 4;
            vk_p[i] = (slot0 + lrow) * ROWB + ck;
            vv_p[i] = (slot0 + lrow) * ROWB + cv;
            vk_s[i] = (i * Gm::RPI + lrow) * row_pitch - i * 1024 + ck;
            vv_s[i] = (i * Gm::RPI + lrow) * row_pitch - i * 1024 + cv;
        }
    }
    constexpr int RSRC_FLAGS = 0x00020000;                 // raw buffer, 32-bit data format
    struct Offs { int v[Gm::NI]; };
    // the NI loads of this wave's rows of one tile into buf
    auto issue_loads = [&](const char *base, int nrec, char *buf, const Offs &vo) {
        const auto rsrc = __builtin_amdgcn_make_buffer_rsrc((void *)base, 0, nrec, RSRC_FLAGS);
        lds_void *dst = (lds_void *)(buf + w * Gm::RW * ROWB);
        static_for([&](auto i) {
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, dst, 16, vo.v[i.value], 0, i.value * 1024, 0);
        }, std::make_integer_sequence<int, Gm::NI>{});
    };
    auto offs_k = [&](int t) { Offs o;
#pragma unroll
        for (int i = 0; i < Gm::NI; i++) o.v[i] = t < TP ? vk_p[i] : vk_s[i];
        return o; };
    auto offs_v = [&](int t) { Offs o;
#pragma unroll
        for (int i = 0; i < Gm::NI; i++) o.v[i] = t < TP ? vv_p[i] : vv_s[i];
        return o; };

    // ---- running state --------------------------------------------------------------------
    f32x16 O[Gm::DB];
#pragma unroll
    for (int db = 0; db < Gm::DB; db++)
#pragma unroll
        for (int r = 0; r < 16; r++) O[db][r] = 0.f;
    // negM: -M in every register of an MFMA accumulator, M being the reference (log2 units) the
    // scores are taken relative to; l_part: this lane's share of the row sum; lb: the same for the
    // block whose probabilities were formed last (not yet added to l_part: it is the overflow probe)
    float l_part = 0.f, lb = 0.f;
    bool redo = false;                                     // wave-uniform: some lane's lb is out of range
    f32x16 negM;
#pragma unroll
    for (int r = 0; r < 16; r++) negM[r] = 0.f;

    // ---- per-lane LDS operand offsets (the swizzle makes them lane- and chunk-specific) ---
    // K operand (kb, dc): row 32*kb + li, chunk 2*dc + lh
    int k_off[Gm::DC];
#pragma unroll
    for (int dc = 0; dc < Gm::DC; dc++) k_off[dc] = li * ROWB + (((2 * dc + lh) ^ Gm::swz_k(li)) << 4);
    // V operand (kb, u, db): rows 32*kb + 16*u + 4*lh + (l&15)/4 (+8), 8 bytes at
    // d = 16*db + (D/2)*((l>>4)&1) + 4*(l&3): MFMA rows 0-15 take d in [16db, 16db+16),
    // rows 16-31 take d in D/2 + [16db, 16db+16)
    int v_off_l[Gm::DB];
    {
        const int vrow = 4 * lh + ((l & 15) >> 2);
#pragma unroll
        for (int db = 0; db < Gm::DB; db++) {
            const int d0 = 16 * db + (D / 2) * ((l >> 4) & 1) + 4 * (l & 3);
            v_off_l[db] = vrow * ROWB + ((((d0 >> 3)) ^ Gm::swz_v(vrow)) << 4) + ((d0 & 4) << 1);
        }
    }
    auto k_operand = [&](const char *kbuf, int kb, int dc) {
        return *(const bf16x8 *)(kbuf + k_off[dc] + kb * 32 * ROWB);
    };
    auto v_operand = [&](const char *vbuf, int kb, int s) {     // s = (u, db)
        const int u = s / Gm::DB, db = s % Gm::DB;
        const char *vp = vbuf + v_off_l[db] + (32 * kb + 16 * u) * ROWB;
        const bf16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4 *)vp);
        const bf16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4 *)(vp + 8 * ROWB));
        return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    };
    // Block kb of tile t holds prefix keys 64t + 32kb .. (valid below the prefix end) or suffix
    // tokens 64(t-TP) + 32kb .. (valid up to the row's own token); also true of the blocks past
    // the last tile, which the pipeline touches while it drains.  needs_mask is wave-uniform.
    auto needs_mask = [&](int t, int kb) {
        return t < TP ? t * BN + 32 * kb + 32 > td.prefix_len : (t - TP) * BN + 32 * kb + 31 > wave_min_tok;
    };
    auto mask_block = [&](f32x16 &S, int t, int kb) {
        const int lim = t < TP ? td.prefix_len - 1 - t * BN : my_tokc - (t - TP) * BN;
        const int rel = lim - 4 * lh - 32 * kb;
#pragma unroll
        for (int r = 0; r < 16; r++)
            if (8 * (r >> 2) + (r & 3) > rel) S[r] = -INFINITY;
    };

    // ---- prologue: K(0) into LDS ---------------------------------------------------------------
    Src prev = tile_src(0);
    issue_loads(prev.k, prev.nrec, sK0, offs_k(0));
    // while that fetch is in flight, zero the V buffers once: rows past the last key are never
    // loaded, and 0 * stale bits must not be able to produce a NaN in the PV product
    for (int i = tid; i < Gm::TILEB / 16; i += NT) {
        *(uint4 *)(sV0 + i * 16) = make_uint4(0, 0, 0, 0);
        *(uint4 *)(sV1 + i * 16) = make_uint4(0, 0, 0, 0);
    }
    __builtin_amdgcn_s_waitcnt(0x0F70);                   // vmcnt(0): the loads have landed in LDS
    __syncthreads();                                      // ... and the V buffers are zero

    if constexpr (PROBE) {
        // valid rows of tile t (0 outside the tile range)
        auto valid_rows = [&](int t) {
            const int v = t < TP ? td.prefix_len - t * BN : tok_end - (t - TP) * BN;
            return t < 0 ? 0 : (v < 0 ? 0 : (v > BN ? BN : v));
        };
        unsigned acc = 0;
        auto fold = [&](const char *buf, int rows) {          // the rows this wave loaded
            const int lrow = l / Gm::CPR;
#pragma unroll
            for (int i = 0; i < Gm::NI; i++) {
                const uint4 v = *(const uint4 *)(buf + (w * Gm::RW + i * Gm::RPI) * ROWB + l * 16);
                if (w * Gm::RW + i * Gm::RPI + lrow < rows) acc ^= v.x ^ v.y ^ v.z ^ v.w;
            }
        };
        auto pstep = [&](int j, char *kcur, char *knext, char *vprev, char *vcur) __attribute__((always_inline)) {
            const Src next = tile_src(j + 1);
            issue_loads(next.k, next.nrec, knext, offs_k(j + 1));
            issue_loads(prev.v, prev.nrec, vcur, offs_v(j));
            prev = next;
            fold(kcur, valid_rows(j));
            fold(vprev, valid_rows(j - 1));
            __builtin_amdgcn_s_waitcnt(0x0F70);
            __syncthreads();
        };
        for (int j = 0; j <= n_tiles; j += 2) {
            pstep(j, sK0, sK1, sV1, sV0);
            if (j + 1 <= n_tiles) pstep(j + 1, sK1, sK0, sV0, sV1);
        }
#pragma unroll
        for (int m = 32; m >= 1; m >>= 1) acc ^= __shfl_xor(acc, m, 64);
        unsigned *red = (unsigned *)sK0;                      // every wave is past its last read of sK0
        if (l == 0) red[w] = acc;
        __syncthreads();
        if (tid == 0) {
            unsigned x = 0;
            for (int i = 0; i < NW; i++) x ^= red[i];
            ((unsigned *)p.out)[((int64_t)td.pad * nsplit + split) * p.Hkv + kvh] = x;
        }
        return;
    } else {

    // pending t of the even / odd blocks, and their probabilities (B operands of PV: [u] = keys 16u..16u+15)
    f32x16 T0, T1;
    bf16x8 P0[2], P1[2];
#pragma unroll
    for (int r = 0; r < 16; r++) { T0[r] = -INFINITY; T1[r] = -INFINITY; }
#pragma unroll
    for (int u = 0; u < 2; u++)
#pragma unroll
        for (int e = 0; e < 8; e++) { P0[u][e] = (__bf16)0.f; P1[u][e] = (__bf16)0.f; }
    bf16x2 ones;
    ones[0] = (__bf16)1.0f;
    ones[1] = (__bf16)1.0f;

    // The common path never computes a row maximum.  The probabilities of the previous block were
    // formed under the current reference M; their lane sum lb tells whether that was safe: a sum
    // above 2^12 (or inf) means some score ran far ahead of M.  Then -- rarely -- the block is redone:
    // its scores are still in Tn (the score product of the iteration has not overwritten them yet), M
    // moves up to their row maximum, O and the row sum (which hold exactly the blocks before it) are
    // rescaled, and its probabilities are formed again.  The first block is always redone, which sets
    // M to its row maximum whatever the magnitude of the scores (key 0 is visible to every row, so
    // that maximum is finite).
    auto redo_block = [&](f32x16 &Tc, f32x16 &Tn, bf16x8 (&Pp)[2], bool first_check) __attribute__((always_inline)) {
        float mxp = Tn[0];
#pragma unroll
        for (int r = 1; r < 16; r++) mxp = fmaxf(mxp, Tn[r]);
        mxp = xmax32(mxp);
        const float d = first_check ? mxp : fmaxf(mxp, 0.f);      // later moves never lower the reference
        const float alpha = first_check ? 1.f : __builtin_amdgcn_exp2f(-d);
        l_part *= alpha;
        // whole-vector updates: the 16-register accumulator tuples stay where they are
#pragma unroll
        for (int db = 0; db < Gm::DB; db++) O[db] *= alpha;
        Tn -= d;
        Tc -= d;
        negM -= d;
        lb = 0.f;
#pragma unroll
        for (int r = 0; r < 16; r += 2) {
            f32x2 pv;
            pv[0] = __builtin_amdgcn_exp2f(Tn[r]);
            pv[1] = __builtin_amdgcn_exp2f(Tn[r + 1]);
            const bf16x2 pk = __builtin_convertvector(pv, bf16x2);
            Pp[r / 8][r % 8] = pk[0];
            Pp[r / 8][r % 8 + 1] = pk[1];
            lb = __builtin_amdgcn_fdot2_f32_bf16(pk, ones, lb, false);
        }
        // (a block that still overflows after its own maximum became the reference cannot exist)
    };

    // ---- tile step j = iterations 2j-1 and 2j: K(j) and V(j-1) are read, K(j+1) and V(j) are fetched.
    // The pipeline is filled by a step of its own (scores of tile 0 only: there is nothing to
    // exponentiate or multiply yet) and drained by another (probabilities of the last block and the
    // products of the last tile only: there are no further scores); the n_tiles - 1 steps between
    // them are the full step below.
    //
    // The 4H MFMAs of a step take their LDS operands (K rows for the score halves, transposed V
    // for the product halves) from ONE stream that runs PF MFMAs ahead, across the half and
    // iteration boundaries, so only the start of a step exposes LDS latency.
    //
    auto step = [&](int j, char *kcur, char *knext, char *vprev, char *vcur) __attribute__((always_inline)) {
        constexpr int NM = 4 * H;                          // MFMAs per step
        constexpr int LD_SP = H / (2 * Gm::NI);            // MFMAs between two tile loads
        static_assert(LD_SP >= 1, "the tile loads of a step fit its first half iteration");
        // sources: K(j+1) now, V(j) from what the previous step found for tile j
        const Src next = tile_src(j + 1);
        const Offs ok = offs_k(j + 1), ov = offs_v(j);
        const bool masked = j >= TPF;                      // tile j is not a full prefix tile
        const auto rsrc_k = __builtin_amdgcn_make_buffer_rsrc((void *)next.k, 0, next.nrec, RSRC_FLAGS);
        const auto rsrc_v = __builtin_amdgcn_make_buffer_rsrc((void *)prev.v, 0, prev.nrec, RSRC_FLAGS);
        lds_void *dst_k = (lds_void *)(knext + w * Gm::RW * ROWB);
        lds_void *dst_v = (lds_void *)(vcur + w * Gm::RW * ROWB);
        prev = next;

        // operand stream: entry m feeds MFMA m of the step
        bf16x8 op[PF + 1];
        auto operand = [&](auto mc) {
            constexpr int m = decltype(mc)::value;
            constexpr int i = m / (2 * H), half = (m / H) & 1, s2 = m % H;
            if constexpr (half == 0) return k_operand(kcur, i, s2);
            else return v_operand(vprev, i, s2);
        };
        static_for([&](auto mc) { op[mc.value % (PF + 1)] = operand(mc); }, std::make_integer_sequence<int, PF>{});

        auto iteration = [&](auto ic, f32x16 &Tc, f32x16 &Tn, bf16x8 (&Pc)[2], bf16x8 (&Pp)[2], bool first_check) __attribute__((always_inline)) {
            constexpr int i = decltype(ic)::value;
            constexpr int m0 = i * 2 * H;
            if (__builtin_expect(first_check || redo, 0)) redo_block(Tc, Tn, Pp, first_check);
            l_part += lb;
            lb = 0.f;
            auto exp_pair = [&](int r) {                  // scores r, r+1 of the pending block
                f32x2 pv;
                pv[0] = __builtin_amdgcn_exp2f(Tc[r]);
                pv[1] = __builtin_amdgcn_exp2f(Tc[r + 1]);
                const bf16x2 pk = __builtin_convertvector(pv, bf16x2);
                Pc[r / 8][r % 8] = pk[0];
                Pc[r / 8][r % 8 + 1] = pk[1];
            };
            __builtin_amdgcn_sched_barrier(0);

            // ---- first half: t(b+1) = K Q^T - M  ||  probabilities of keys 0-15 of block b; tile loads ----
            // (statements appear in issue order; the group barriers below pin that interleaving)
            static_for([&](auto sc) {
                constexpr int s2 = decltype(sc)::value, m = m0 + s2;
                if constexpr (m + PF < NM) op[(m + PF) % (PF + 1)] = operand(IntC<m + PF>{});
                MFMA_PRIO(1);
                Tn = __builtin_amdgcn_mfma_f32_32x32x16_bf16(op[m % (PF + 1)], qreg[s2], s2 == 0 ? negM : Tn, 0, 0, 0);
                MFMA_PRIO(0);
                // all tile loads of the step go out in its first half iteration, K and V rows
                // alternating, one every LD_SP MFMAs: they have the rest of the step to land
                if constexpr (i == 0 && s2 % LD_SP == 0) {
                    constexpr int q = s2 / LD_SP, li2 = q / 2;
                    if constexpr (q % 2 == 0) __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc_k, dst_k, 16, ok.v[li2], 0, li2 * 1024, 0);
                    else __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc_v, dst_v, 16, ov.v[li2], 0, li2 * 1024, 0);
                }
                // four score pairs over H steps
                if constexpr (H == 8) { if constexpr (s2 % 2 == 0) exp_pair(s2); }
                else exp_pair(2 * s2);
            }, std::make_integer_sequence<int, H>{});
            static_for([&](auto sc) {
                constexpr int s2 = decltype(sc)::value, m = m0 + s2;
                if constexpr (m == 0) __builtin_amdgcn_sched_group_barrier(SG_DSRD, PF, 0);
                __builtin_amdgcn_sched_group_barrier(SG_MFMA, 1, 0);
                if constexpr (i == 0 && s2 % LD_SP == 0) __builtin_amdgcn_sched_group_barrier(SG_VMRD, 1, 0);
                __builtin_amdgcn_sched_group_barrier(SG_VALU, 16 / H, 0);
                if constexpr (m + PF < NM) __builtin_amdgcn_sched_group_barrier(SG_DSRD, ((m + PF) / H) & 1 ? 2 : 1, 0);
            }, std::make_integer_sequence<int, H>{});
            // the probabilities are only consumed an iteration later; keep their computation here,
            // in the MFMA shadow
            PIN_V(Pc[0]);
            PIN_V(lb);
            __builtin_amdgcn_sched_barrier(0);
            if (__builtin_expect(masked, 0)) {
                if (needs_mask(j, i)) mask_block(Tn, j, i);
            }
            __builtin_amdgcn_sched_barrier(0);

            // ---- second half: O += V^T P of block b-1  ||  probabilities of keys 16-31 of block b ----
            static_for([&](auto sc) {
                constexpr int s2 = decltype(sc)::value, m = m0 + H + s2;
                if constexpr (m + PF < NM) op[(m + PF) % (PF + 1)] = operand(IntC<m + PF>{});
                MFMA_PRIO(1);
                O[s2 % Gm::DB] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(op[m % (PF + 1)], Pp[s2 / Gm::DB], O[s2 % Gm::DB], 0, 0, 0);
                MFMA_PRIO(0);
                if constexpr (H == 8) { if constexpr (s2 % 2 == 0) exp_pair(8 + s2); }
                else exp_pair(8 + 2 * s2);
                // the row sum of the block (of what PV will use: the rounded probabilities), all eight
                // dot2 in one run behind the last MFMA, and the overflow probe on it, so that the next
                // iteration starts with a branch on a scalar that is already there
                if constexpr (s2 == H - 1) {
#pragma unroll
                    for (int r = 0; r < 16; r += 2) {
                        bf16x2 pk;
                        pk[0] = Pc[r / 8][r % 8];
                        pk[1] = Pc[r / 8][r % 8 + 1];
                        lb = __builtin_amdgcn_fdot2_f32_bf16(pk, ones, lb, false);
                    }
                    redo = __any(!(lb <= RESCALE_SUM));
                }
            }, std::make_integer_sequence<int, H>{});
            static_for([&](auto sc) {
                constexpr int s2 = decltype(sc)::value, m = m0 + H + s2;
                __builtin_amdgcn_sched_group_barrier(SG_MFMA, 1, 1);
                __builtin_amdgcn_sched_group_barrier(SG_VALU, s2 == H - 1 ? 12 : 16 / H, 1);
                if constexpr (m + PF < NM) __builtin_amdgcn_sched_group_barrier(SG_DSRD, ((m + PF) / H) & 1 ? 2 : 1, 1);
            }, std::make_integer_sequence<int, H>{});
            PIN_V(Pc[1]);
            PIN_V(lb);
            __builtin_amdgcn_sched_barrier(0);
        };
        iteration(IntC<0>{}, T1, T0, P1, P0, j == 1);      // block 0 is redone before its PV product
        iteration(IntC<1>{}, T0, T1, P0, P1, false);
        __builtin_amdgcn_s_waitcnt(0x0F70);               // vmcnt(0): K(j+1), V(j) are in LDS
        __syncthreads();                                  // ... and every wave is done with K(j), V(j-1)
    };
    // fill: scores of the two blocks of tile 0 (from the reference 0; the first full or drain step
    // moves the reference to block 0's row maximum before anything is exponentiated); K(1), V(0) fetched
    {
        const Src next = tile_src(1);
        issue_loads(next.k, next.nrec, sK1, offs_k(1));
        issue_loads(prev.v, prev.nrec, sV0, offs_v(0));
        prev = next;
        static_for([&](auto dc) {
            T0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(k_operand(sK0, 0, dc.value), qreg[dc.value], dc.value == 0 ? negM : T0, 0, 0, 0);
        }, std::make_integer_sequence<int, Gm::DC>{});
        static_for([&](auto dc) {
            T1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(k_operand(sK0, 1, dc.value), qreg[dc.value], dc.value == 0 ? negM : T1, 0, 0, 0);
        }, std::make_integer_sequence<int, Gm::DC>{});
        if (0 >= TPF) {
            if (needs_mask(0, 0)) mask_block(T0, 0, 0);
            if (needs_mask(0, 1)) mask_block(T1, 0, 1);
        }
        __builtin_amdgcn_s_waitcnt(0x0F70);
        __syncthreads();
    }
    // full steps 1 .. n_tiles - 1, in pairs so that the LDS buffers are compile-time constants
    for (int j = 1; j < n_tiles; j += 2) {
        step(j, sK1, sK0, sV0, sV1);
        if (j + 1 < n_tiles) step(j + 1, sK0, sK1, sV1, sV0);
    }
    // drain: probabilities of the last block, products of tile n_tiles - 1 (its V rows were fetched
    // by the step before and are in the buffer that step wrote)
    {
        const char *vlast = (n_tiles - 1) & 1 ? sV1 : sV0;
        auto exp_all = [&](f32x16 &Tc, bf16x8 (&Pc)[2]) __attribute__((always_inline)) {
#pragma unroll
            for (int r = 0; r < 16; r += 2) {
                f32x2 pv;
                pv[0] = __builtin_amdgcn_exp2f(Tc[r]);
                pv[1] = __builtin_amdgcn_exp2f(Tc[r + 1]);
                const bf16x2 pk = __builtin_convertvector(pv, bf16x2);
                Pc[r / 8][r % 8] = pk[0];
                Pc[r / 8][r % 8 + 1] = pk[1];
                lb = __builtin_amdgcn_fdot2_f32_bf16(pk, ones, lb, false);
            }
        };
        auto product = [&](int kb, bf16x8 (&Pp)[2]) __attribute__((always_inline)) {
            static_for([&](auto sc) {
                constexpr int s2 = decltype(sc)::value;
                O[s2 % Gm::DB] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(v_operand(vlast, kb, s2), Pp[s2 / Gm::DB], O[s2 % Gm::DB], 0, 0, 0);
            }, std::make_integer_sequence<int, H>{});
        };
        if (n_tiles == 1 || redo) redo_block(T1, T0, P0, n_tiles == 1);
        l_part += lb;
        lb = 0.f;
        exp_all(T1, P1);
        product(0, P0);
        if (__any(!(lb <= RESCALE_SUM))) redo_block(T0, T1, P1, false);
        l_part += lb;
        lb = 0.f;
        product(1, P1);
    }

    // ---- epilogue: normalise, round once to bf16, store -----------------------------------
    // register r of O[db] is MFMA row 8*(r/4) + 4*lh + r%4; rows 0-15 are d = 16*db + row,
    // rows 16-31 are d = D/2 + 16*db + (row - 16)
    const float inv = 1.0f / xsum32(l_part);
    if (my_tok < td.new_len) {
        __bf16 *op = (__bf16 *)p.out + ((td.row0 + my_tok) * p.Hq + head) * D + 4 * lh;
#pragma unroll
        for (int db = 0; db < Gm::DB; db++)
#pragma unroll
            for (int b4 = 0; b4 < 4; b4++) {
                bf16x4 v;
#pragma unroll
                for (int cc = 0; cc < 4; cc++) v[cc] = (__bf16)(O[db][4 * b4 + cc] * inv);
                *(bf16x4 *)(op + 16 * db + 8 * (b4 & 1) + (D / 2) * (b4 >> 1)) = v;
            }
    }
    }   // !PROBE
#endif
}

// ================================================================================================
// The 64-token-per-wave form of the same kernel: four waves per work-group, ONE per SIMD, each
// serving one query head of the GQA group over 64 suffix tokens as two 32-token sub-tiles.  Every
// K / V^T operand read from LDS feeds two MFMAs (one per sub-tile), so the LDS reads, the barrier
// participants and the scalar bookkeeping per useful FLOP are half of the eight-wave form's, with
// the same MFMA / vector-ALU mix per SIMD.  A wave needs about 400 registers for the state of two
// sub-tiles; a wave alone on its SIMD may use 512, but only 256 of them can be operands of vector
// instructions.  The compiler allots MFMA accumulators either all to the vector or all to the
// accumulation registers of a function, so the matrix instructions are written in assembly with
// the classes given by hand: the output accumulators O live in accumulation registers (only MFMAs
// touch them on the common path), the scores, probabilities, references and Q operands in vector
// registers.  Assembly statements get no hazard handling from the compiler; the pipeline keeps
// every producer at least a half iteration (16 MFMAs) ahead of its consumer, and the three places
// where that is not so (masking right after a score chain, the rare reference move, the epilogue)
// wait explicitly.
// A wave alone on its SIMD issues in order with nothing to cover for it, so the place of every
// instruction counts: the exponentials and packs of the common path are assembly statements too
// (plain intrinsics carry no ordering against the MFMA statements and were all gathered in front
// of the first MFMA of a half iteration, a quarter of the kernel's time with an idle matrix
// pipe), and the sixteen row-sum dot2 of an iteration, which run in the matrix pipe's order,
// stand together at its start.
typedef __attribute__((ext_vector_type(4))) int i32x4;

[[maybe_unused]] static __device__ __forceinline__ i32x4 as_i(const bf16x8 &v) { return __builtin_bit_cast(i32x4, v); }

#if defined(__HIP_DEVICE_COMPILE__)
// d = a b + c, scores: everything in vector registers except the Q operand b
static __device__ __forceinline__ void mfma_s_first(f32x16 &d, const i32x4 &a, const i32x4 &b, const f32x16 &c) {
    asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %3" : "=&v"(d) : "v"(a), "v"(b), "v"(c));
}
static __device__ __forceinline__ void mfma_s_acc(f32x16 &d, const i32x4 &a, const i32x4 &b) {
    asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(d) : "v"(a), "v"(b));
}
// d += a b, outputs: accumulator in accumulation registers, operands in vector registers
static __device__ __forceinline__ void mfma_o_acc(f32x16 &d, const i32x4 &a, const i32x4 &b) {
    asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+a"(d) : "v"(a), "v"(b));
}
// "whatever wrote these registers has finished": 36 idle cycles tied to the values by operands
#define SETTLE_V2(x, y) asm volatile("s_nop 15\n\ts_nop 15\n\ts_nop 3" : "+v"(x), "+v"(y))
#define SETTLE_A2(x, y) asm volatile("s_nop 15\n\ts_nop 15\n\ts_nop 3" : "+a"(x), "+a"(y))
#endif

template <int D>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, 1)))
void attn_bf16_w64_kernel(AttnParams p, int G, int Gw) {
#if defined(__HIP_DEVICE_COMPILE__)
    constexpr int NW = 4;
    using Gm = Geom<D, NW>;
    constexpr int H = Gm::H;
    constexpr int NT = 64 * NW;
    constexpr int ROWB = Gm::ROWB;
    constexpr int PFW = 3;                                 // LDS operand prefetch distance, in operand fetches (PFW + 1 divides 4H)

    __shared__ __attribute__((aligned(1024))) char sK0[Gm::TILEB];
    __shared__ __attribute__((aligned(1024))) char sK1[Gm::TILEB];
    __shared__ __attribute__((aligned(1024))) char sV0[Gm::TILEB];
    __shared__ __attribute__((aligned(1024))) char sV1[Gm::TILEB];

    const int tid = threadIdx.x, l = tid & 63, li = l & 31, lh = l >> 5;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int kvh = blockIdx.x % p.Hkv;
    const int rest = blockIdx.x / p.Hkv;
    const int nsplit = G / Gw;
    const int split = rest % nsplit;
    const TileDesc td = p.tiles[rest / nsplit];
    if (p.mirror != nullptr && kvh == 0 && split == 0 && tid == 0) p.mirror[rest / nsplit] = td;
    const int head = kvh * G + split * Gw + (w % Gw);
    const int tile_tok = 64 * (NW / Gw);
    const int tok_base = td.tok0 + (w / Gw) * 64;          // sub-tile s holds tokens tok_base + 32 s + li
    const int tok_end = min(td.tok0 + tile_tok, td.new_len);
    const int TP = (td.prefix_len + BN - 1) / BN;
    const int TPF = td.prefix_len / BN;
    const int n_tiles = TP + (tok_end + BN - 1) / BN;
    int my_tok[2], my_tokc[2], wave_min_tok[2];
#pragma unroll
    for (int s = 0; s < 2; s++) {
        my_tok[s] = tok_base + 32 * s + li;
        my_tokc[s] = min(my_tok[s], td.new_len - 1);
        wave_min_tok[s] = min(tok_base + 32 * s, td.new_len - 1);
    }

    // ---- Q^T operands of both sub-tiles, pre-scaled by log2(e)/sqrt(D) and rounded once to bf16 ----
    const float c = 1.4426950408889634f * rsqrtf((float)D);
    i32x4 qreg[2][Gm::DC];
#pragma unroll
    for (int s = 0; s < 2; s++) {
        const __bf16 *qp = (const __bf16 *)p.q + ((td.row0 + my_tokc[s]) * p.Hq + head) * D + 8 * lh;
#pragma unroll
        for (int dc = 0; dc < Gm::DC; dc++) {
            const bf16x8 raw = *(const bf16x8 *)(qp + dc * 16);
            bf16x8 sc;
#pragma unroll
            for (int e = 0; e < 8; e++) sc[e] = (__bf16)((float)raw[e] * c);
            qreg[s][dc] = as_i(sc);
        }
    }

    // ---- tile sources (as in the kernel above; a wave's 16 rows of a tile are one page) ----
    constexpr int PPT = BN / 16;
    const int pw = (w * Gm::RW) >> 4;
    const int slot0 = (w * Gm::RW) & 15;
    const int32_t *bt = p.block_table + (int64_t)td.req * p.max_pages;
    const int n_prefix_pages = (td.prefix_len + 15) >> 4;
    // A wave alone on its SIMD pays for every scalar instruction, so the page ids are held as page
    // offsets in units of 256 bytes (a page is a multiple of that, and a pool of less than 1 TiB
    // keeps them in 32 bits; the host checks it): a tile's K address is one lane read, one shift and
    // one 64-bit add.
    const int row_pitch = p.Hkv * ROWB;
    const int64_t page_bytes = 2 * (int64_t)p.Hkv * 16 * ROWB;
    const unsigned page_units = (unsigned)(page_bytes >> 8);
    auto load_id_block = [&](int blk) {
        const int lp = blk * 64 + l;
        int pg = lp < n_prefix_pages ? bt[lp] : 0;
        pg = pg < 0 ? 0 : (pg >= p.num_pages ? p.num_pages - 1 : pg);
        return (int)((unsigned)pg * page_units);
    };
    int ids_cur = load_id_block(0), ids_next = load_id_block(1);
    struct Src { const char *k, *v; int nrec; };
    const int64_t v_in_page = (int64_t)p.Hkv * 16 * ROWB;
    const char *pool_k = (const char *)p.kv_pool + (int64_t)kvh * 16 * ROWB;
    const char *kn_h = (const char *)p.k_new + (int64_t)kvh * ROWB;
    const char *vn_h = (const char *)p.v_new + (int64_t)kvh * ROWB;
    // rows of this wave's page of the last prefix tile (the only one that can be partly filled or unused)
    const int last_nrec = min(max(td.prefix_len - ((TP - 1) * PPT + pw) * 16, 0), 16) * ROWB;
    auto tile_src = [&](int t) {
        Src s;
        if (t < TP) {
            if (__builtin_expect((t & 15) == 0 && t > 0, 0)) {
                ids_cur = ids_next;
                ids_next = load_id_block((t >> 4) + 1);
            }
            const unsigned units = (unsigned)__builtin_amdgcn_readlane(ids_cur, (t & 15) * PPT + pw);
            s.k = pool_k + ((uint64_t)units << 8);
            s.v = s.k + v_in_page;
            s.nrec = t < TP - 1 ? 16 * ROWB : last_nrec;
        } else {
            const int s0 = (t - TP) * BN + w * Gm::RW;
            const int srows = min(tok_end - s0, Gm::RW);
            const int64_t off = (td.row0 + s0) * (int64_t)row_pitch;
            s.k = kn_h + off;
            s.v = vn_h + off;
            s.nrec = srows > 0 ? (srows - 1) * row_pitch + ROWB : 0;
        }
        return s;
    };
    int vk_p[Gm::NI], vk_s[Gm::NI], vv_p[Gm::NI], vv_s[Gm::NI];
    {
        const int lrow = l / Gm::CPR, cpos = l % Gm::CPR;
#pragma unroll
        for (int i = 0; i < Gm::NI; i++) {
            const int row = w * Gm::RW + i * Gm::RPI + lrow;
            const int ck = (cpos ^ Gm::swz_k(row)) << 4, cv = (cpos ^ Gm::swz_v(row)) << 4;
            vk_p[i] = (slot0 + i * Gm::RPI + lrow) * ROWB - i * 1024 + ck;
            vv_p[i] = (slot0 + i * Gm::RPI + lrow) * ROWB - i * 1024 + cv;
            vk_s[i] = (i * Gm::RPI + lrow) * row_pitch - i * 1024 + ck;
            vv_s[i] = (i * Gm::RPI + lrow) * row_pitch - i * 1024 + cv;
        }
    }
    constexpr int RSRC_FLAGS = 0x00020000;
    struct Offs { int v[Gm::NI]; };
    auto issue_loads = [&](const char *base, int nrec, char *buf, const Offs &vo) {
        const auto rsrc = __builtin_amdgcn_make_buffer_rsrc((void *)base, 0, nrec, RSRC_FLAGS);
        lds_void *dst = (lds_void *)(buf + w * Gm::RW * ROWB);
        static_for([&](auto i) {
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, dst, 16, vo.v[i.value], 0, i.value * 1024, 0);
        }, std::make_integer_sequence<int, Gm::NI>{});
    };
    auto offs_k = [&](int t) { Offs o;
#pragma unroll
        for (int i = 0; i < Gm::NI; i++) o.v[i] = t < TP ? vk_p[i] : vk_s[i];
        return o; };
    auto offs_v = [&](int t) { Offs o;
#pragma unroll
        for (int i = 0; i < Gm::NI; i++) o.v[i] = t < TP ? vv_p[i] : vv_s[i];
        return o; };

    // ---- running state of the two sub-tiles ----
    f32x16 O[2][Gm::DB];
#pragma unroll
    for (int s = 0; s < 2; s++)
#pragma unroll
        for (int db = 0; db < Gm::DB; db++)
#pragma unroll
            for (int r = 0; r < 16; r++) O[s][db][r] = 0.f;
    float l_part[2] = {0.f, 0.f}, lb[2] = {0.f, 0.f};
    f32x16 negM[2];
#pragma unroll
    for (int s = 0; s < 2; s++)
#pragma unroll
        for (int r = 0; r < 16; r++) negM[s][r] = 0.f;

    int k_off[Gm::DC];
#pragma unroll
    for (int dc = 0; dc < Gm::DC; dc++) k_off[dc] = li * ROWB + (((2 * dc + lh) ^ Gm::swz_k(li)) << 4);
    int v_off_l[Gm::DB];
    {
        const int vrow = 4 * lh + ((l & 15) >> 2);
#pragma unroll
        for (int db = 0; db < Gm::DB; db++) {
            const int d0 = 16 * db + (D / 2) * ((l >> 4) & 1) + 4 * (l & 3);
            v_off_l[db] = vrow * ROWB + ((((d0 >> 3)) ^ Gm::swz_v(vrow)) << 4) + ((d0 & 4) << 1);
        }
    }
    auto k_operand = [&](const char *kbuf, int kb, int dc) {
        return as_i(*(const bf16x8 *)(kbuf + k_off[dc] + kb * 32 * ROWB));
    };
    auto v_operand = [&](const char *vbuf, int kb, int s) {
        const int u = s / Gm::DB, db = s % Gm::DB;
        const char *vp = vbuf + v_off_l[db] + (32 * kb + 16 * u) * ROWB;
        const bf16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4 *)vp);
        const bf16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4 *)(vp + 8 * ROWB));
        return as_i(__builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
    };
    auto needs_mask = [&](int t, int kb, int s) {
        return t < TP ? t * BN + 32 * kb + 32 > td.prefix_len : (t - TP) * BN + 32 * kb + 31 > wave_min_tok[s];
    };
    auto mask_block = [&](f32x16 &S, int t, int kb, int s) {
        const int lim = t < TP ? td.prefix_len - 1 - t * BN : my_tokc[s] - (t - TP) * BN;
        const int rel = lim - 4 * lh - 32 * kb;
#pragma unroll
        for (int r = 0; r < 16; r++)
            if (8 * (r >> 2) + (r & 3) > rel) S[r] = -INFINITY;
    };

    // ---- prologue ----
    Src prev = tile_src(0);
    issue_loads(prev.k, prev.nrec, sK0, offs_k(0));
    for (int i = tid; i < Gm::TILEB / 16; i += NT) {
        *(uint4 *)(sV0 + i * 16) = make_uint4(0, 0, 0, 0);
        *(uint4 *)(sV1 + i * 16) = make_uint4(0, 0, 0, 0);
    }
    __builtin_amdgcn_s_waitcnt(0x0F70);
    __syncthreads();

    f32x16 T0[2], T1[2];
    bf16x8 P0[2][2], P1[2][2];
#pragma unroll
    for (int s = 0; s < 2; s++) {
#pragma unroll
        for (int r = 0; r < 16; r++) { T0[s][r] = -INFINITY; T1[s][r] = -INFINITY; }
#pragma unroll
        for (int u = 0; u < 2; u++)
#pragma unroll
            for (int e = 0; e < 8; e++) { P0[s][u][e] = (__bf16)0.f; P1[s][u][e] = (__bf16)0.f; }
    }
    bf16x2 ones;
    ones[0] = (__bf16)1.0f;
    ones[1] = (__bf16)1.0f;

    auto exp_pair = [&](const f32x16 &Tc, bf16x8 (&Pc)[2], float &lbs, int r) __attribute__((always_inline)) {
        f32x2 pv;
        pv[0] = __builtin_amdgcn_exp2f(Tc[r]);
        pv[1] = __builtin_amdgcn_exp2f(Tc[r + 1]);
        const bf16x2 pk = __builtin_convertvector(pv, bf16x2);
        Pc[r / 8][r % 8] = pk[0];
        Pc[r / 8][r % 8 + 1] = pk[1];
        lbs = __builtin_amdgcn_fdot2_f32_bf16(pk, ones, lbs, false);
    };
    // The common path's form of it, in two halves, so that the wave's one instruction stream has an MFMA
    // between the exponentials and the pack that depends on them; assembly statements, because they
    // must stay where they are written (plain intrinsics carry no ordering against the MFMA statements).
    // The row sums are not formed here: see block_sums.
    auto exp_pair_a = [&](const f32x16 &Tc, int r) __attribute__((always_inline)) {
        f32x2 pv;
        float a, b;
        asm volatile("v_exp_f32 %0, %1" : "=v"(a) : "v"(Tc[r]));
        asm volatile("v_exp_f32 %0, %1" : "=v"(b) : "v"(Tc[r + 1]));
        pv[0] = a;
        pv[1] = b;
        return pv;
    };
    auto exp_pair_b = [&](const f32x2 &pv, bf16x8 (&Pc)[2], int r) __attribute__((always_inline)) {
        int bits;
        asm volatile("v_cvt_pk_bf16_f32 %0, %1, %2" : "=v"(bits) : "v"(pv[0]), "v"(pv[1]));
        i32x4 t = __builtin_bit_cast(i32x4, Pc[r / 8]);
        t[(r % 8) / 2] = bits;
        Pc[r / 8] = __builtin_bit_cast(bf16x8, t);
    };
    // Row sums of a finished block of both sub-tiles, from its packed (rounded) probabilities, in
    // score order: the same dot2 chain as the other forms of the kernel run.  A dot2 goes through the
    // matrix pipe in order with the MFMAs, so the sixteen stand together, at the start of the
    // iteration that multiplies the block with V, where the overflow test needs them.
    auto block_sums = [&](const bf16x8 (&Pp)[2][2]) __attribute__((always_inline)) {
#pragma unroll
        for (int s = 0; s < 2; s++) {
            lb[s] = 0.f;
#pragma unroll
            for (int r = 0; r < 16; r += 2) {
                bf16x2 pk;
                pk[0] = Pp[s][r / 8][r % 8];
                pk[1] = Pp[s][r / 8][r % 8 + 1];
                lb[s] = __builtin_amdgcn_fdot2_f32_bf16(pk, ones, lb[s], false);
            }
        }
    };
    // the reference move of one sub-tile (see the kernel above); its scores and outputs have settled
    auto redo_block = [&](int s, f32x16 &Tc, f32x16 &Tn, bf16x8 (&Pp)[2], bool first_check) __attribute__((always_inline)) {
        float mxp = Tn[0];
#pragma unroll
        for (int r = 1; r < 16; r++) mxp = fmaxf(mxp, Tn[r]);
        mxp = xmax32(mxp);
        const float d = first_check ? mxp : fmaxf(mxp, 0.f);
        const float alpha = first_check ? 1.f : __builtin_amdgcn_exp2f(-d);
        l_part[s] *= alpha;
#pragma unroll
        for (int db = 0; db < Gm::DB; db++) O[s][db] *= alpha;
        Tn -= d;
        Tc -= d;
        negM[s] -= d;
        lb[s] = 0.f;
#pragma unroll
        for (int r = 0; r < 16; r += 2) exp_pair(Tn, Pp, lb[s], r);
    };
    auto redo_both = [&](f32x16 (&Tc)[2], f32x16 (&Tn)[2], bf16x8 (&Pp)[2][2], bool first_check) __attribute__((always_inline)) {
        SETTLE_V2(Tn[0], Tn[1]);
        SETTLE_V2(Tc[0], Tc[1]);
#pragma unroll
        for (int db = 0; db < Gm::DB; db++) SETTLE_A2(O[0][db], O[1][db]);
        // each sub-tile moves its reference exactly when a wave serving it alone would
        const bool r0 = __any(!(lb[0] <= RESCALE_SUM)), r1 = __any(!(lb[1] <= RESCALE_SUM));
        if (first_check || r0) redo_block(0, Tc[0], Tn[0], Pp[0], first_check);
        if (first_check || r1) redo_block(1, Tc[1], Tn[1], Pp[1], first_check);
        SETTLE_V2(negM[0], negM[1]);
#pragma unroll
        for (int db = 0; db < Gm::DB; db++) SETTLE_A2(O[0][db], O[1][db]);
    };

    // ---- full tile step: 4H operand fetches, each feeding the two sub-tiles' MFMAs ----
    // A wave is alone on its SIMD, so nothing covers for it while it waits: the stream of LDS
    // operands therefore runs on across the step boundary (the waves meet PFW fetches before the end
    // of a step, once every read of the step's tiles has returned, and the first K operands of the
    // next step are fetched while the last products of this one run), and the source of the tile the
    // next step will fetch is worked out in the middle of this one.
    i32x4 op[PFW + 1];
    Src pre = prev;                                        // source of tile j + 1 while step j runs
    auto step = [&](int j, char *kcur, char *knext, char *vprev, char *vcur) __attribute__((always_inline)) {
        constexpr int NM = 4 * H;
        constexpr int NL = 2 * Gm::NI;                     // tile loads of the step, one per group of its first half
        static_assert(NL <= H, "the tile loads of a step fit its first half iteration");
        static_assert(NM % (PFW + 1) == 0 && PFW <= H, "the operand ring closes at the step boundary");
        const Src next = pre;
        const Offs ok = offs_k(j + 1), ov = offs_v(j);
        const bool masked = j >= TPF;
        const auto rsrc_k = __builtin_amdgcn_make_buffer_rsrc((void *)next.k, 0, next.nrec, RSRC_FLAGS);
        const auto rsrc_v = __builtin_amdgcn_make_buffer_rsrc((void *)prev.v, 0, prev.nrec, RSRC_FLAGS);
        lds_void *dst_k = (lds_void *)(knext + w * Gm::RW * ROWB);
        lds_void *dst_v = (lds_void *)(vcur + w * Gm::RW * ROWB);
        prev = next;

        auto operand = [&](auto mc) {
            constexpr int m = decltype(mc)::value;
            if constexpr (m >= NM) return k_operand(knext, 0, m - NM);       // first operands of the next step
            else {
                constexpr int i = m / (2 * H), half = (m / H) & 1, s2 = m % H;
                if constexpr (half == 0) return k_operand(kcur, i, s2);
                else return v_operand(vprev, i, s2);
            }
        };
        auto fetch = [&](auto mc) __attribute__((always_inline)) {
            constexpr int m = decltype(mc)::value;
            if constexpr (m + PFW == NM) {
                // every LDS read of this step's tiles has been issued; once they have returned and this
                // wave's part of the fetched tiles has landed, the waves meet
                __builtin_amdgcn_s_waitcnt(0x0070);           // vmcnt(0) lgkmcnt(0)
                __syncthreads();
            }
            op[(m + PFW) % (PFW + 1)] = operand(IntC<m + PFW>{});
        };

        auto iteration = [&](auto ic, f32x16 (&Tc)[2], f32x16 (&Tn)[2], bf16x8 (&Pc)[2][2], bf16x8 (&Pp)[2][2], bool first_check) __attribute__((always_inline)) {
            constexpr int i = decltype(ic)::value;
            constexpr int m0 = i * 2 * H;
            constexpr int PPG = 8 / H;                     // score pairs exponentiated beside one operand's two MFMAs
            block_sums(Pp);
            if (__builtin_expect(first_check || __any(!(lb[0] <= RESCALE_SUM) || !(lb[1] <= RESCALE_SUM)), 0)) redo_both(Tc, Tn, Pp, first_check);
            l_part[0] += lb[0];
            l_part[1] += lb[1];
            lb[0] = 0.f;
            lb[1] = 0.f;
            __builtin_amdgcn_sched_barrier(0);
            // first half: t(b+1) = K Q^T - M for both sub-tiles  ||  probabilities of sub-tile 0's block b; tile loads.
            // Order inside a group: MFMA, exponentials, MFMA, tile load, pack -- a wave issues in order, so two
            // MFMAs back to back would hold the vector work behind the second one's wait for the matrix pipe
            static_for([&](auto sc) {
                constexpr int s2 = decltype(sc)::value, m = m0 + s2;
                fetch(IntC<m>{});
                f32x2 pv[PPG];
                if constexpr (s2 == 0) mfma_s_first(Tn[0], op[m % (PFW + 1)], qreg[0][s2], negM[0]);
                else mfma_s_acc(Tn[0], op[m % (PFW + 1)], qreg[0][s2]);
                __builtin_amdgcn_sched_barrier(0);
                static_for([&](auto pc) { pv[pc.value] = exp_pair_a(Tc[0], 2 * (PPG * s2 + pc.value)); }, std::make_integer_sequence<int, PPG>{});
                __builtin_amdgcn_sched_barrier(0);
                if constexpr (s2 == 0) mfma_s_first(Tn[1], op[m % (PFW + 1)], qreg[1][s2], negM[1]);
                else mfma_s_acc(Tn[1], op[m % (PFW + 1)], qreg[1][s2]);
                __builtin_amdgcn_sched_barrier(0);
                if constexpr (i == 0 && s2 < NL) {
                    constexpr int li2 = s2 / 2;
                    if constexpr (s2 % 2 == 0) __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc_k, dst_k, 16, ok.v[li2], 0, li2 * 1024, 0);
                    else __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc_v, dst_v, 16, ov.v[li2], 0, li2 * 1024, 0);
                }
                static_for([&](auto pc) { exp_pair_b(pv[pc.value], Pc[0], 2 * (PPG * s2 + pc.value)); }, std::make_integer_sequence<int, PPG>{});
                __builtin_amdgcn_sched_barrier(0);
            }, std::make_integer_sequence<int, H>{});
            if (__builtin_expect(masked, 0)) {
                const bool m0k = needs_mask(j, i, 0), m1k = needs_mask(j, i, 1);
                if (m0k || m1k) {
                    SETTLE_V2(Tn[0], Tn[1]);
                    if (m0k) mask_block(Tn[0], j, i, 0);
                    if (m1k) mask_block(Tn[1], j, i, 1);
                }
            }
            if constexpr (i == 0) pre = tile_src(j + 2);   // in the shadow of the MFMAs in flight
            __builtin_amdgcn_sched_barrier(0);
            // second half: O += V^T P of block b-1 for both sub-tiles  ||  probabilities of sub-tile 1's block b
            static_for([&](auto sc) {
                constexpr int s2 = decltype(sc)::value, m = m0 + H + s2;
                fetch(IntC<m>{});
                f32x2 pv[PPG];
                mfma_o_acc(O[0][s2 % Gm::DB], op[m % (PFW + 1)], as_i(Pp[0][s2 / Gm::DB]));
                __builtin_amdgcn_sched_barrier(0);
                static_for([&](auto pc) { pv[pc.value] = exp_pair_a(Tc[1], 2 * (PPG * s2 + pc.value)); }, std::make_integer_sequence<int, PPG>{});
                __builtin_amdgcn_sched_barrier(0);
                mfma_o_acc(O[1][s2 % Gm::DB], op[m % (PFW + 1)], as_i(Pp[1][s2 / Gm::DB]));
                __builtin_amdgcn_sched_barrier(0);
                static_for([&](auto pc) { exp_pair_b(pv[pc.value], Pc[1], 2 * (PPG * s2 + pc.value)); }, std::make_integer_sequence<int, PPG>{});
                __builtin_amdgcn_sched_barrier(0);
            }, std::make_integer_sequence<int, H>{});
        };
        iteration(IntC<0>{}, T1, T0, P1, P0, j == 1);
        iteration(IntC<1>{}, T0, T1, P0, P1, false);
    };
    // fill: scores of tile 0 for both sub-tiles; K(1), V(0) fetched
    {
        const Src next = tile_src(1);
        issue_loads(next.k, next.nrec, sK1, offs_k(1));
        issue_loads(prev.v, prev.nrec, sV0, offs_v(0));
        prev = next;
        pre = tile_src(2);
        static_for([&](auto dc) {
            const i32x4 a0 = k_operand(sK0, 0, dc.value), a1 = k_operand(sK0, 1, dc.value);
            if constexpr (dc.value == 0) {
                mfma_s_first(T0[0], a0, qreg[0][0], negM[0]);
                mfma_s_first(T0[1], a0, qreg[1][0], negM[1]);
                mfma_s_first(T1[0], a1, qreg[0][0], negM[0]);
                mfma_s_first(T1[1], a1, qreg[1][0], negM[1]);
            } else {
                mfma_s_acc(T0[0], a0, qreg[0][dc.value]);
                mfma_s_acc(T0[1], a0, qreg[1][dc.value]);
                mfma_s_acc(T1[0], a1, qreg[0][dc.value]);
                mfma_s_acc(T1[1], a1, qreg[1][dc.value]);
            }
        }, std::make_integer_sequence<int, Gm::DC>{});
        SETTLE_V2(T0[0], T0[1]);
        SETTLE_V2(T1[0], T1[1]);
        if (0 >= TPF) {
#pragma unroll
            for (int s = 0; s < 2; s++) {
                if (needs_mask(0, 0, s)) mask_block(T0[s], 0, 0, s);
                if (needs_mask(0, 1, s)) mask_block(T1[s], 0, 1, s);
            }
        }
        __builtin_amdgcn_s_waitcnt(0x0F70);
        __syncthreads();
        static_for([&](auto mc) { op[mc.value] = k_operand(sK1, 0, mc.value); }, std::make_integer_sequence<int, PFW>{});
    }
    for (int j = 1; j < n_tiles; j += 2) {
        step(j, sK1, sK0, sV0, sV1);
        if (j + 1 < n_tiles) step(j + 1, sK0, sK1, sV1, sV0);
    }
    // drain: probabilities of the last block, products of tile n_tiles - 1
    {
        const char *vlast = (n_tiles - 1) & 1 ? sV1 : sV0;
        auto exp_all = [&](int s, f32x16 &Tc, bf16x8 (&Pc)[2]) __attribute__((always_inline)) {
#pragma unroll
            for (int r = 0; r < 16; r += 2) exp_pair(Tc, Pc, lb[s], r);
        };
        auto product = [&](int kb, bf16x8 (&Pp)[2][2]) __attribute__((always_inline)) {
            static_for([&](auto sc) {
                constexpr int s2 = decltype(sc)::value;
                const i32x4 a = v_operand(vlast, kb, s2);
                mfma_o_acc(O[0][s2 % Gm::DB], a, as_i(Pp[0][s2 / Gm::DB]));
                mfma_o_acc(O[1][s2 % Gm::DB], a, as_i(Pp[1][s2 / Gm::DB]));
            }, std::make_integer_sequence<int, H>{});
        };
        block_sums(P0);
        if (n_tiles == 1 || __any(!(lb[0] <= RESCALE_SUM) || !(lb[1] <= RESCALE_SUM))) redo_both(T1, T0, P0, n_tiles == 1);
        l_part[0] += lb[0];
        l_part[1] += lb[1];
        lb[0] = 0.f;
        lb[1] = 0.f;
        SETTLE_V2(T1[0], T1[1]);
        exp_all(0, T1[0], P1[0]);
        exp_all(1, T1[1], P1[1]);
        product(0, P0);
        if (__any(!(lb[0] <= RESCALE_SUM) || !(lb[1] <= RESCALE_SUM))) redo_both(T0, T1, P1, false);
        l_part[0] += lb[0];
        l_part[1] += lb[1];
        product(1, P1);
#pragma unroll
        for (int db = 0; db < Gm::DB; db++) SETTLE_A2(O[0][db], O[1][db]);
    }
    // ---- epilogue ----
#pragma unroll
    for (int s = 0; s < 2; s++) {
        const float inv = 1.0f / xsum32(l_part[s]);
        if (my_tok[s] < td.new_len) {
            __bf16 *opp = (__bf16 *)p.out + ((td.row0 + my_tok[s]) * p.Hq + head) * D + 4 * lh;
#pragma unroll
            for (int db = 0; db < Gm::DB; db++)
#pragma unroll
                for (int b4 = 0; b4 < 4; b4++) {
                    bf16x4 v;
#pragma unroll
                    for (int cc = 0; cc < 4; cc++) v[cc] = (__bf16)(O[s][db][4 * b4 + cc] * inv);
                    *(bf16x4 *)(opp + 16 * db + 8 * (b4 & 1) + (D / 2) * (b4 >> 1)) = v;
                }
        }
    }
#endif
}

template <int D>
static hipError_t launch_w64(const AttnParams &p, int G, int Gw, hipStream_t s) {
    const unsigned grid = (unsigned)p.n_tiles * (G / Gw) * p.Hkv;
    hipLaunchKernelGGL((attn_bf16_w64_kernel<D>), dim3(grid), dim3(256), 0, s, p, G, Gw);
    return hipGetLastError();
}

template <int D, int NW, bool PROBE>
static hipError_t launch_one(const AttnParams &p, int G, int Gw, hipStream_t s) {
    const unsigned grid = (unsigned)p.n_tiles * (G / Gw) * p.Hkv;
    hipLaunchKernelGGL((attn_bf16_kernel<D, NW, PROBE>), dim3(grid), dim3(64 * NW), 0, s, p, G, Gw);
    return hipGetLastError();
}


hipError_t launch_attn_bf16(const AttnParams &p0, int head_dim, hipStream_t s) {
    AttnParams p = p0;
    if (p.n_tiles == 0) return hipSuccess;
    const int G = p.Hq / p.Hkv;
    const int Gw = G < 4 ? G : 4;
    if (p.waves == 4) return head_dim == 128 ? launch_one<128, 4, false>(p, G, Gw, s) : launch_one<64, 4, false>(p, G, Gw, s);
    if (p.waves == 64) return head_dim == 128 ? launch_w64<128>(p, G, Gw, s) : launch_w64<64>(p, G, Gw, s);
    return head_dim == 128 ? launch_one<128, 8, false>(p, G, Gw, s) : launch_one<64, 8, false>(p, G, Gw, s);
}

int attn_bf16_units_per_tile(int num_kv_heads, int group) {
    const int gw = group < 4 ? group : 4;
    return (group / gw) * num_kv_heads;
}

hipError_t launch_gather_probe(const AttnParams &p, int head_dim, hipStream_t s) {
    if (p.n_tiles == 0) return hipSuccess;
    const int G = p.Hq / p.Hkv;
    const int Gw = G < 4 ? G : 4;
    if (p.waves == 4) return head_dim == 128 ? launch_one<128, 4, true>(p, G, Gw, s) : launch_one<64, 4, true>(p, G, Gw, s);
    // (the 64-row form cuts the work and stages the tiles as the eight-wave form does: one probe serves both)
    return head_dim == 128 ? launch_one<128, 8, true>(p, G, Gw, s) : launch_one<64, 8, true>(p, G, Gw, s);
}

}  // namespace pbkv
