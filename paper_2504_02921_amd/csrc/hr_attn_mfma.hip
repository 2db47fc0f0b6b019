// Paged grouped-query prefix attention on MFMA (gfx950): the KV-streaming kernel of the scoring pass.
//
// One work item per (pair, kv head), or per (group of pairs that share a document, kv head).  Its query
// rows are the g * q_len rows (token i, head a of the group) of every pair in it that share this kv
// head, cut into 32-row blocks (a pair starts a new block); wave w owns blocks w, w + NW, ...  The document's pages are
// streamed HBM -> LDS in 32 KiB stages (double buffered, every page is one contiguous burst and is
// copied verbatim: the pool already holds the LDS-friendly arrangement), all keys of the document are
// visible to every row; then each pair's own query keys, which the QKV projection wrote as pages of the
// same arrangement, follow in the same stream and are processed with the causal mask by the blocks of
// that pair.  Softmax is the online form in fp32.  A row's arithmetic does not depend on which block or
// work item carries it: grouped and ungrouped runs give the same bits.
//
// MFMA orientation (v_mfma_f32_32x32x16_f16): scores are computed transposed, S^T = K * Q^T, so a
// lane owns ONE query row (column lane & 31) and 16 of the 32 keys of a sub-tile.  Row maxima and
// sums are then in-lane reductions plus a single exchange with lane ^ 32, the probabilities are
// already in B-operand order for O^T += V^T * P^T, and the rescale factor of a row is a per-lane
// scalar.  The 8 keys a lane holds per MFMA are {4h..4h+3, 8+4h..8+4h+3} of a 16-key page, which is
// why pages store V transposed in exactly that grouping.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <atomic>
#include <cstdlib>
#include <type_traits>

#include "hr_device_types.h"
#include "hr_kernels.h"
#include "hr_layout.h"

namespace hr {

typedef __attribute__((ext_vector_type(8))) _Float16 halfx8;
typedef __attribute__((ext_vector_type(4))) _Float16 halfx4;
typedef __attribute__((ext_vector_type(2))) _Float16 halfx2;
typedef __attribute__((ext_vector_type(16))) float floatx16;
typedef __attribute__((ext_vector_type(2))) float floatx2;
typedef __attribute__((address_space(3))) void* lds_ptr_t;
typedef const __attribute__((address_space(1))) void* gbl_ptr_t;

namespace {

// LDS stage: 32 KiB of half pages; an fp8 pool streams the same number of keys per stage in 16 KiB and spends the
// other 32 KiB on the expanded copy of the current stage, so both kinds fit two workgroups per CU.
constexpr int kStageBytesHalf = 32768;
constexpr int stage_bytes(bool fp8) { return fp8 ? kStageBytesHalf / 2 : kStageBytesHalf; }
constexpr int kMaxRowsPerWg = 512;
constexpr float kLazyMax = 8.0f;

template <int HD, bool FP8, int kStageBytes>
struct Geo {
    static constexpr int ESZ = FP8 ? 1 : 2;
    static constexpr int BLOCK_BYTES = kPageTokens * HD * ESZ;   // one K (or V) block
    static constexpr int PAGE_BYTES = 2 * BLOCK_BYTES;
    static constexpr int PPS = kStageBytes / PAGE_BYTES;         // pages per stage
    static constexpr int TK = kPageTokens * PPS;                 // keys per stage
};

// 8 consecutive fp8 codes (one 64-bit LDS word) -> 8 halves, times a power of two.
// An E4M3 code s.eeee.mmm placed at bits 15, 13..7 of a half (sign kept, exponent and mantissa fields shifted down
// by one) reads as (-1)^s 2^(e-15) (1 + m/8), or (-1)^s 2^-14 (m/8) when e = 0: in both cases the E4M3 value
// (bias 7, subnormals m/8 * 2^-6) divided by 2^8.  So the conversion is a byte shuffle, two masks, a shift and one
// packed half multiplication by 2^8 * 2^k, exact while the product is a half.  (The hardware's scaled conversion
// instruction gives the same values but measured ~88 cycles per wavefront instruction, against 4 for these.)
// The two NaN codes (0x7f, 0xff) read as +-480; a pool never holds them.
__device__ __forceinline__ halfx8 fp8x8_to_half(uint2 w, halfx2 pow2) {
    auto pair = [&](unsigned x, unsigned sel) {
        const unsigned t = __builtin_amdgcn_perm(x, 0u, sel);                    // code bytes to the high byte of each 16-bit half
        const unsigned h = (t & 0x80008000u) | ((t & 0x7F007F00u) >> 1);
        halfx2 v;
        __builtin_memcpy(&v, &h, 4);
        return v * pow2;
    };
    const halfx2 a = pair(w.x, 0x050c040cu), b = pair(w.x, 0x070c060cu), c = pair(w.y, 0x050c040cu), d = pair(w.y, 0x070c060cu);
    halfx8 r;
    r[0] = a[0]; r[1] = a[1]; r[2] = b[0]; r[3] = b[1]; r[4] = c[0]; r[5] = c[1]; r[6] = d[0]; r[7] = d[1];
    return r;
}

// Reductions over lanes l and l ^ 32 (the two lanes that share a query row) through the VALU lane-swap instruction instead of an
// LDS round trip: v_permlane32_swap exchanges the upper half of its first operand with the lower half of its second, so
// with the same value in both the first result holds lanes 0..31 twice and the second lanes 32..63 twice.
__device__ __forceinline__ float row_max2(float x) {       // max over the two lanes of a row, in both
    const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float row_sum2(float x) {       // sum over the two lanes of a row, in both (same bits in both)
    const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

// 2^8 times the power of two of a positive scale, as a pair of halves (clamped to the normal range of half)
__device__ __forceinline__ halfx2 fp8_expand_factor(float scale) {
    int e = (int)((__float_as_uint(scale) >> 23) & 0xFFu) - 127 + 8;
    e = e < -14 ? -14 : (e > 15 ? 15 : e);
    const _Float16 f = (_Float16)__uint_as_float((unsigned)(e + 127) << 23);
    return halfx2{f, f};
}

// What a workgroup needs to know about one work item = (pair or group of pairs with one document, kv head)
struct ItemCtx {
    int p0, h, D, n_pages, n_tiles;
    int blk0, n_blk;              // 32-row blocks (grouped: a range of the plan's block arrays)
    int sub0, n_sub, n_new_tiles; // 32-key sub-tiles of the pairs' own keys, and the stages they fill
    const int32_t* pt;        // page-table row
    const char* layer_base;   // pool address of page 0 for this (layer, kv head)
};

// PREC: the 22-bit form of the first layers (split operands).  q and o are [T][hi n_q d | lo n_q d] halves (value = hi + lo),
// the new tokens' K/V pages have a second buffer of lo pages (kv_new_lo, same arrangement), and the probabilities are
// split in registers; every product that carries a hi x lo term is an extra MFMA chain into the same accumulator:
//   S = K q_hi + K q_lo (+ K_lo q_hi for the pair's own keys),  O = V p_hi + V p_lo (+ V_lo p_hi likewise).
// Document K/V from the pool are exact as stored.  One wave per SIMD (the extra fragments need the registers).
template <int HD, int NW, int R, bool FP8, bool PREC>
__global__ void __launch_bounds__(NW * 64) __attribute__((amdgpu_waves_per_eu(PREC ? 1 : ((HD == 64 && R == 1 && NW == 8) ? 4 : (HD * R <= 128 ? 2 : 1)), 8))) attn_mfma_kernel(const half_t* __restrict__ q, const char* __restrict__ kv_new,
                                                           const char* __restrict__ kv_new_lo,
                                                           half_t* __restrict__ o, MetaView mv, PoolView pv, int layer, int n_q,
                                                           const int32_t* __restrict__ m_cu, const int32_t* __restrict__ m_prefix,
                                                           const int32_t* __restrict__ m_pt, const int32_t* __restrict__ m_new_cu,
                                                           const float* __restrict__ p_scales, int last_only, int n_groups,
                                                           const int32_t* __restrict__ g_p0, const int32_t* __restrict__ g_blk_cu,
                                                           const int32_t* __restrict__ g_sub_cu, const int32_t* __restrict__ g_blk_seq,
                                                           const int32_t* __restrict__ g_blk_row0, const int32_t* __restrict__ g_sub_page,
                                                           const int32_t* __restrict__ g_sub_seq, const int32_t* __restrict__ g_sub_key0) {
    // The metadata arrays come as separate read-only, non-aliased parameters so that the per-item lookups (uniform
    // over the workgroup) compile to scalar loads: a vector load that is used right away makes the wave wait for
    // everything it has in flight, including the stage it requested a moment earlier, because vector memory
    // operations complete in order.
    constexpr int kStageBytes = stage_bytes(FP8);
    using G = Geo<HD, FP8, kStageBytes>;
    using GN = Geo<HD, false, kStageBytes>;          // the pair's own keys are always half
    constexpr int NT = NW * 64;
    constexpr int NPASS = kStageBytes / (NT * 16);   // 16-byte loads per thread and stage
    constexpr int KC = HD / 16;                      // MFMA k-steps over head_dim
    constexpr int MB = HD / 32;                      // 32-channel blocks of the output
    extern __shared__ __attribute__((aligned(16))) char smem[];      // [2][kStageBytes] + scales + (fp8) expanded stage
    float* s_scale = (float*)(smem + 2 * kStageBytes);              // [2][PPS][2]  (fp8 only)
    char* hbuf = smem + 2 * kStageBytes + 2 * G::PPS * 2 * sizeof(float);   // fp8 only: the current stage as half pages
    char* lobuf = hbuf + (FP8 ? 2 * kStageBytes : 0);                       // PREC only: [2][kStageBytes] lo pages of the pair's own keys
    const int q_ld = (PREC ? 2 : 1) * n_q * HD;                             // row stride of q and o; lo halves n_q * HD further

    const int n_kv = pv.n_kv;
    const int g = n_q / n_kv;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int ln = lane & 31, hh = lane >> 5;
    const int wave_u = __builtin_amdgcn_readfirstlane(wave);
    const float c_log2 = 1.4426950408889634f / sqrtf((float)HD);
    const size_t page_stride = (size_t)n_kv * G::PAGE_BYTES;                         // between consecutive page ids
    const bool grouped = n_groups > 0;
    const int n_items = (grouped ? n_groups : mv.n_seq) * n_kv;
    constexpr int SUBS = GN::TK / 32;                // sub-tiles of the pairs' own keys per stage

    auto load_ctx = [&](int item) {
        ItemCtx c;
        const int gi = item / n_kv;
        c.h = item - gi * n_kv;
        if (grouped) {
            c.p0 = g_p0[gi];
            c.blk0 = g_blk_cu[gi];
            c.n_blk = g_blk_cu[gi + 1] - c.blk0;
            c.sub0 = g_sub_cu[gi];
            c.n_sub = g_sub_cu[gi + 1] - c.sub0;
        } else {
            c.p0 = gi;
            const int qn = m_cu[gi + 1] - m_cu[gi];
            c.blk0 = 0;
            c.n_blk = ((last_only ? g : qn * g) + 31) / 32;
            c.sub0 = 0;
            c.n_sub = (qn + 31) / 32;
        }
        c.D = m_prefix[c.p0];
        c.n_pages = (c.D + kPageTokens - 1) / kPageTokens;
        c.n_tiles = (c.n_pages + G::PPS - 1) / G::PPS;
        c.n_new_tiles = (c.n_sub + SUBS - 1) / SUBS;
        c.pt = m_pt + (size_t)c.p0 * mv.pt_stride;
        c.layer_base = pv.data + ((size_t)layer * pv.num_pages * n_kv + c.h) * G::PAGE_BYTES;
        return c;
    };
    // block b of an item: whose rows, and which of them (uniform over the wave)
    auto blk_lookup = [&](const ItemCtx& c, int b, int& seq, int& row0) {
        if (grouped) {
            seq = g_blk_seq[c.blk0 + b];
            row0 = g_blk_row0[c.blk0 + b];
        } else {
            seq = c.p0;
            row0 = b * 32;
        }
    };
    // sub-tile s of an item's own keys: first of its two pages in the new-KV buffer, the pair, its first key
    auto sub_lookup = [&](const ItemCtx& c, int s, int& page, int& seq, int& key0) {
        if (grouped) {
            page = g_sub_page[c.sub0 + s];
            seq = g_sub_seq[c.sub0 + s];
            key0 = g_sub_key0[c.sub0 + s];
        } else {
            page = (m_new_cu[c.p0] >> 4) + 2 * s;
            seq = c.p0;
            key0 = 32 * s;
        }
    };

    // ---- KV stream: the document's pages, then the pair's own (causal) keys, which the QKV projection has already
    // written as half pages in the same arrangement.  HBM -> LDS directly (global_load_lds_dwordx4: lane l of a
    // wave writes LDS bytes [base + 16 l, +16)), two stages, pages land verbatim.
    float stg_scale = 0.f;
    // Page ids (and fp8 scales' page) travel one step ahead of the data: ids_load(c, t) requests the ids of document
    // tile t into registers, dma_doc(c, t, buf) consumes them.  The page-table latency is thus never on the path
    // between two stages.
    int pgid[NPASS];
    int pgid_scale = 0;
    auto ids_load = [&](const ItemCtx& c, int tile) {
#pragma unroll
        for (int ps = 0; ps < NPASS; ++ps) {
            const int slot = (ps * NT * 16 + tid * 16) / G::PAGE_BYTES;
            int pgi = tile * G::PPS + slot;
            pgi = pgi < c.n_pages ? pgi : c.n_pages - 1;       // past the end: re-read the last page (finite data, masked)
            pgid[ps] = c.pt[pgi];
        }
        if constexpr (FP8) {      // every thread asks (threads past 2 * PPS repeat an earlier one): no branch, no copy that waits
            int pgi = tile * G::PPS + ((tid >> 1) % G::PPS);
            pgi = pgi < c.n_pages ? pgi : c.n_pages - 1;
            pgid_scale = c.pt[pgi];
        }
    };
    auto dma_doc = [&](const ItemCtx& c, int buf) {
        char* dst = smem + buf * kStageBytes + wave_u * 1024;
#pragma unroll
        for (int ps = 0; ps < NPASS; ++ps) {
            const int off = ps * NT * 16 + tid * 16;
            const int within = off % G::PAGE_BYTES;
            const char* src = c.layer_base + (size_t)pgid[ps] * page_stride + within;
            // non-temporal: a document's pages are read once per work item (a pure stream of random 4-8 KiB bursts
            // measured 6.7 TB/s with the hint against 6.1 without)
            __builtin_amdgcn_global_load_lds((gbl_ptr_t)src, (lds_ptr_t)(dst + ps * NT * 16), 16, 0, 2);
        }
        if constexpr (FP8) stg_scale = p_scales[(((size_t)layer * pv.num_pages + pgid_scale) * n_kv + c.h) * 2 + (tid & 1)];
    };
    auto dma_new = [&](const ItemCtx& c, int nt, int buf) {
        char* dst = smem + buf * kStageBytes + wave_u * 1024;
#pragma unroll
        for (int ps = 0; ps < NPASS; ++ps) {
            const int off = ps * NT * 16 + wave_u * 1024;      // whole waves stay inside one page
            const int slot = off / GN::PAGE_BYTES, within = off - slot * GN::PAGE_BYTES + lane * 16;
            const int s = nt * SUBS + (slot >> 1);
            if (s < c.n_sub) {                                 // wave-uniform
                int page, seq, key0;
                sub_lookup(c, s, page, seq, key0);
                const size_t src_off = ((size_t)(page + (slot & 1)) * n_kv + c.h) * GN::PAGE_BYTES + within;
                __builtin_amdgcn_global_load_lds((gbl_ptr_t)(kv_new + src_off), (lds_ptr_t)(dst + ps * NT * 16), 16, 0, 0);
                if constexpr (PREC)
                    __builtin_amdgcn_global_load_lds((gbl_ptr_t)(kv_new_lo + src_off),
                                                     (lds_ptr_t)(lobuf + buf * kStageBytes + wave_u * 1024 + ps * NT * 16), 16, 0, 0);
            }
        }
    };
    auto dma_first = [&](const ItemCtx& c, int buf) {          // first stage of a work item (ids already requested)
        if (c.n_tiles > 0) dma_doc(c, buf);
        else dma_new(c, 0, buf);                               // there is always at least one query key
    };
    // Invariant: pgid holds the ids of the next document tile in stream order after the last requested one.  Called
    // right after the stage of document tile `tile` of item `c_item` has been requested (documents of length 0 have
    // no tiles and are skipped; normally the scan takes one step).
    auto ids_after = [&](const ItemCtx& c, int tile, int c_item) {
        if (tile + 1 < c.n_tiles) {
            ids_load(c, tile + 1);
            return;
        }
        for (int it = c_item + (int)gridDim.x; it < n_items; it += (int)gridDim.x) {
            const ItemCtx n = load_ctx(it);
            if (n.n_tiles > 0) {
                ids_load(n, 0);
                return;
            }
        }
    };
    auto scale_store = [&](int buf) {
        if constexpr (FP8) {
            if (tid < G::PPS * 2) s_scale[buf * G::PPS * 2 + tid] = stg_scale;
        }
    };

    halfx8 qf[R][KC];      // Q^T fragments (B operand), loaded once the first stage is on its way
    halfx8 qf_lo[PREC ? R : 1][PREC ? KC : 1];      // PREC: their lo halves
    int row_i[R];          // query token index of the lane's row in block rb
    size_t row_off[R];     // element offset of that row in q / o
    bool row_ok[R];
    floatx16 oacc[R][MB];
    float m_run[R], l_run[R];
    bool blk_on[R];        // the wave's block rb exists in the current work item   (these three: uniform over the wave)
    int blk_seq[R];        // ... and belongs to this pair
    int blk_qn[R];         // ... which has this many query tokens
    int blk_row0[R];       // ... first row of the block within the pair
    int blk_t0[R];         // ... first token row of the pair

    // fp8 pools: the stage that has just landed is expanded to half pages once, by all threads together (8 codes
    // per step and thread), instead of by every wave for its own fragments: the conversions are the largest
    // VALU item of the fp8 path and every wave of the workgroup needs every key.
    auto expand_stage = [&](const char* sb, const float* sc) {
        constexpr int UPP = G::PAGE_BYTES / 8;               // 8-byte words per fp8 page
        constexpr int KU = G::BLOCK_BYTES / 8;               // ... of which the K block
#pragma unroll
        for (int u0 = 0; u0 < kStageBytes / 8; u0 += NT) {
            const int u = u0 + tid;
            const int page = u / UPP, w = u - page * UPP;    // whole waves stay inside one block of one page
            const uint2 src = *(const uint2*)(sb + (size_t)u * 8);
            char* dpage = hbuf + page * GN::PAGE_BYTES;
            if (w < KU) {
                const int t = w / (HD / 8), c8 = (w % (HD / 8)) ^ k_swizzle(t, HD, 1);
                *(halfx8*)(dpage + (t * HD + ((c8 ^ k_swizzle(t, HD, 2)) << 3)) * 2) = fp8x8_to_half(src, fp8_expand_factor(1.0f));
            } else {
                *(halfx8*)(dpage + GN::BLOCK_BYTES + (w - KU) * 16) = fp8x8_to_half(src, fp8_expand_factor(sc[page * 2 + 1]));
            }
        }
    };

    // ---- one 32-key sub-tile held in LDS (two pages) against every row block of this wave.
    // Order: K fragments -> S = K Q^T for all row blocks -> V^T fragments (K registers are dead by then, the
    // LDS latency hides under the softmax) -> softmax -> O^T += V^T P^T.
    // `sb` holds half pages; scaled_tag: they were expanded from fp8 codes and `sc` carries the pages' scales.
    // on[rb]: the wave's block rb takes part; nv[rb]: keys of the sub-tile that exist for it.
    auto process = [&](auto scaled_tag, auto causal_tag, const char* sb, int st, const bool (&on)[R], const int (&nv)[R], const float* sc,
                       const char* sb_lo) {
        constexpr bool KV8 = decltype(scaled_tag)::value;
        constexpr bool CAUSAL = decltype(causal_tag)::value;
        using GG = GN;
        floatx16 s[R];
        {
            // K fragments (A operand): lane = key row ln of the sub-tile, channels chunk (2 kk + hh)
            halfx8 kf[KC];
            const int t = ln & 15;
            const char* kb = sb + (st * 2 + (ln >> 4)) * GG::PAGE_BYTES;
#pragma unroll
            for (int kk = 0; kk < KC; ++kk) {
                const int e = t * HD + (((2 * kk + hh) ^ k_swizzle(t, HD, GG::ESZ)) << 3);
                kf[kk] = *(const halfx8*)(kb + e * 2);
            }
#pragma unroll
            for (int rb = 0; rb < R; ++rb) {
#pragma unroll
                for (int r = 0; r < 16; ++r) s[rb][r] = 0.f;
                if (!on[rb]) continue;                             // wave-uniform
#pragma unroll
                for (int kk = 0; kk < KC; ++kk) s[rb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(kf[kk], qf[rb][kk], s[rb], 0, 0, 0);
                if constexpr (R == 1 && !PREC) {
                    // one row block per wave: left alone, the scheduler reads each K fragment right before the MFMA that
                    // uses it and the wave sits out one LDS round trip per MFMA; all reads first, then the chain
                    __builtin_amdgcn_sched_group_barrier(0x100, KC, 0);
                    __builtin_amdgcn_sched_group_barrier(0x008, KC, 0);
                }
                if constexpr (PREC) {
#pragma unroll
                    for (int kk = 0; kk < KC; ++kk) s[rb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(kf[kk], qf_lo[rb][kk], s[rb], 0, 0, 0);
                }
            }
            if constexpr (PREC && CAUSAL) {
                // the pair's own keys carry lo pages: K_lo q_hi
                const char* kbl = sb_lo + (st * 2 + (ln >> 4)) * GG::PAGE_BYTES;
#pragma unroll
                for (int kk = 0; kk < KC; ++kk) {
                    const int e = t * HD + (((2 * kk + hh) ^ k_swizzle(t, HD, GG::ESZ)) << 3);
                    kf[kk] = *(const halfx8*)(kbl + e * 2);
                }
#pragma unroll
                for (int rb = 0; rb < R; ++rb) {
                    if (!on[rb]) continue;
#pragma unroll
                    for (int kk = 0; kk < KC; ++kk) s[rb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(kf[kk], qf[rb][kk], s[rb], 0, 0, 0);
                }
            }
        }
        // fp8 pages: K scale goes into the softmax exponent (fp32).  The V scale is split into its power of two,
        // applied exactly while the codes were expanded, and its mantissa in [1, 2), applied to the probabilities:
        // folding the whole scale (~1e-2) into P would push probabilities into the subnormal range of half.
        float cs0 = c_log2, cs1 = c_log2, vs0 = 1.f, vs1 = 1.f;
        if constexpr (KV8) {
            cs0 *= sc[(st * 2) * 2];
            cs1 *= sc[(st * 2 + 1) * 2];
            vs0 = __uint_as_float((__float_as_uint(sc[(st * 2) * 2 + 1]) & 0x007FFFFFu) | 0x3F800000u);
            vs1 = __uint_as_float((__float_as_uint(sc[(st * 2 + 1) * 2 + 1]) & 0x007FFFFFu) | 0x3F800000u);
        }
        // V^T fragments (A operand): lane = channel mb*32 + ln, 8 keys of key group hh of page s2
        halfx8 vf[MB][2];
#pragma unroll
        for (int s2 = 0; s2 < 2; ++s2) {
            const char* vb = sb + (st * 2 + s2) * GG::PAGE_BYTES + GG::BLOCK_BYTES;
#pragma unroll
            for (int mb = 0; mb < MB; ++mb) {
                const int e = (hh * HD + mb * 32 + ln) * 8;
                vf[mb][s2] = *(const halfx8*)(vb + e * 2);
            }
        }
#pragma unroll
        for (int rb = 0; rb < R; ++rb) {
            if (!on[rb]) continue;                             // wave-uniform
            floatx16& sr = s[rb];
            // lane holds keys 8*(r>>2) + 4*hh + (r&3) of the sub-tile for query row ln
            const int limit = CAUSAL ? min(nv[rb], row_i[rb] + 1) : nv[rb];       // keys [0, limit) visible (sub-tile relative)
            if (limit < 32) {
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int key = 8 * (r >> 2) + 4 * hh + (r & 3);
                    sr[r] = key < limit ? sr[r] : -INFINITY;
                }
            }
            // row maximum of the scaled logits: the two pages of a sub-tile may carry different (positive) K scales
            float mx0 = sr[0], mx1 = sr[8];
#pragma unroll
            for (int r = 1; r < 8; ++r) {
                mx0 = fmaxf(mx0, sr[r]);
                mx1 = fmaxf(mx1, sr[8 + r]);
            }
            float mx = fmaxf(mx0 * cs0, mx1 * cs1);
            mx = row_max2(mx);
            // The running maximum only follows the scores when they exceed it by more than kLazyMax (log2 units): below
            // that the probabilities of this sub-tile are at most 2^kLazyMax (no overflow in half, and the final division
            // by the row sum cancels the factor), and the rescale of O and of the row sum, 32-64 multiplications
            // per block, is skipped for the whole wavefront unless one of its rows moves.  Decided per row, so a row's
            // arithmetic does not depend on its neighbours.
            const float m_cand = fmaxf(m_run[rb], mx);
            const bool move = m_cand > m_run[rb] + kLazyMax;       // false while everything so far is masked (-inf)
            const float m_new = move ? m_cand : m_run[rb];
            const float alpha = !move ? 1.0f : (m_run[rb] == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(m_run[rb] - m_new));
            const float m_use = m_new == -INFINITY ? 0.f : m_new;   // a row with nothing visible yet keeps p = 0
            float lsum = 0.f;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const float pr = __builtin_amdgcn_exp2f(fmaf(sr[r], r < 8 ? cs0 : cs1, -m_use));
                lsum += pr;
                sr[r] = pr;
            }
            l_run[rb] = l_run[rb] * alpha + lsum;
            m_run[rb] = m_new;
            if (__any(alpha != 1.0f)) {
#pragma unroll
                for (int mb = 0; mb < MB; ++mb)
#pragma unroll
                    for (int r = 0; r < 16; ++r) oacc[rb][mb][r] *= alpha;
            }
            halfx8 pf[2];
            halfx8 pl[PREC ? 2 : 1];          // PREC: what the rounding of P to half left out
#pragma unroll
            for (int j = 0; j < 8; j += 2) {
                const floatx2 a = {KV8 ? sr[j] * vs0 : sr[j], KV8 ? sr[j + 1] * vs0 : sr[j + 1]};
                const floatx2 b = {KV8 ? sr[8 + j] * vs1 : sr[8 + j], KV8 ? sr[9 + j] * vs1 : sr[9 + j]};
                const halfx2 ha = __builtin_convertvector(a, halfx2), hb2 = __builtin_convertvector(b, halfx2);
                pf[0][j] = ha[0]; pf[0][j + 1] = ha[1];
                pf[1][j] = hb2[0]; pf[1][j + 1] = hb2[1];
                if constexpr (PREC) {
                    const floatx2 ra = a - __builtin_convertvector(ha, floatx2), rb2 = b - __builtin_convertvector(hb2, floatx2);
                    const halfx2 la = __builtin_convertvector(ra, halfx2), lb = __builtin_convertvector(rb2, halfx2);
                    pl[0][j] = la[0]; pl[0][j + 1] = la[1];
                    pl[1][j] = lb[0]; pl[1][j + 1] = lb[1];
                }
            }
#pragma unroll
            for (int mb = 0; mb < MB; ++mb) {
                oacc[rb][mb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(vf[mb][0], pf[0], oacc[rb][mb], 0, 0, 0);
                oacc[rb][mb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(vf[mb][1], pf[1], oacc[rb][mb], 0, 0, 0);
                if constexpr (PREC) {
                    oacc[rb][mb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(vf[mb][0], pl[0], oacc[rb][mb], 0, 0, 0);
                    oacc[rb][mb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(vf[mb][1], pl[1], oacc[rb][mb], 0, 0, 0);
                }
            }
            if constexpr (PREC && CAUSAL) {
                // V_lo p_hi for the pair's own keys (fragments read per block: this path is rare and short)
#pragma unroll
                for (int s2 = 0; s2 < 2; ++s2) {
                    const char* vbl = sb_lo + (st * 2 + s2) * GG::PAGE_BYTES + GG::BLOCK_BYTES;
#pragma unroll
                    for (int mb = 0; mb < MB; ++mb) {
                        const halfx8 vl = *(const halfx8*)(vbl + ((hh * HD + mb * 32 + ln) * 8) * 2);
                        oacc[rb][mb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(vl, pf[s2], oacc[rb][mb], 0, 0, 0);
                    }
                }
            }
        }
    };

    // ---- persistent loop over work items.  The first stage of the next item is requested while the last stage of
    // the current one is consumed, and its Q fragments are fetched before the current item's output is stored, so
    // only the very first item of a workgroup pays the start-up latency.
    // last_only: only the last query token of every pair is computed (g rows per item, all of the pair's own keys
    // visible) and its output goes to row `pair` of a compact [n_pairs][n_q][d] buffer: what the last layer needs.
    auto setup_rows = [&](const ItemCtx& c) {
#pragma unroll
        for (int rb = 0; rb < R; ++rb) {
            const int b = wave_u + rb * NW;
            blk_on[rb] = b < c.n_blk;
            int seq = c.p0, row0 = 0;
            if (blk_on[rb]) blk_lookup(c, b, seq, row0);
            const int t0 = m_cu[seq], qn = m_cu[seq + 1] - t0;
            blk_seq[rb] = seq;
            blk_qn[rb] = qn;
            blk_row0[rb] = row0;
            blk_t0[rb] = t0;
            const int M = last_only ? g : qn * g;                  // rows of this pair
            const int row = row0 + ln;
            row_ok[rb] = blk_on[rb] && row < M;
            const int rc = row < M ? row : M - 1;
            const int i = last_only ? qn - 1 : rc / g, a = last_only ? rc : rc - i * g;
            row_i[rb] = i;
            row_off[rb] = (size_t)(t0 + i) * q_ld + (size_t)(c.h * g + a) * HD;
#pragma unroll
            for (int kk = 0; kk < KC; ++kk) qf[rb][kk] = *(const halfx8*)(q + row_off[rb] + (2 * kk + hh) * 8);
            if constexpr (PREC) {
#pragma unroll
                for (int kk = 0; kk < KC; ++kk) qf_lo[rb][kk] = *(const halfx8*)(q + row_off[rb] + (size_t)n_q * HD + (2 * kk + hh) * 8);
            }
        }
    };

    // The previous item's output waits, packed, in registers and is stored behind the next item's first barrier (the
    // split-operand variant stores at once).
    constexpr bool DEFER = !PREC;
    // In the accumulator layout a lane holds 8 bytes of each of 4 x MB places of one row, and a store instruction
    // touches 32 rows with 16 bytes each (measured: the 16 such stores per block cost ~8 k cycles per work item, queued in
    // front of the next stage's loads).  The output is therefore turned through LDS, 32 channels at a time, into whole
    // 64-byte row segments: chunk c = lane + 64 j (j = 0, 1) is 16 bytes, piece c & 3 of row c >> 2 of the block.
    typedef __attribute__((ext_vector_type(4))) unsigned ochunk_t;
    ochunk_t opk[DEFER ? R : 1][DEFER ? MB : 1][2];
    size_t out_off[R][2];
    bool out_ok[R][2];
    bool out_pending = false;
    auto flush_out = [&]() {
        if (!out_pending) return;
#pragma unroll
        for (int rb = 0; rb < R; ++rb)
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                if (!out_ok[rb][j]) continue;
                half_t* dst = o + out_off[rb][j] + (lane & 3) * 8;
#pragma unroll
                for (int mb = 0; mb < MB; ++mb) *(ochunk_t*)(dst + mb * 32) = opk[rb][mb][j];
            }
        out_pending = false;
    };

    int stage = 0;                                  // LDS stage that holds (or will hold) the current item's next tile
    ItemCtx cur = load_ctx(blockIdx.x);
    if (cur.n_tiles > 0) ids_load(cur, 0);
    dma_first(cur, 0);
    ids_after(cur, 0, (int)blockIdx.x);
    setup_rows(cur);
    for (int item = blockIdx.x; item < n_items; item += gridDim.x) {
        const int next_item = item + gridDim.x;
        const bool has_next = next_item < n_items;
        const ItemCtx nxt = has_next ? load_ctx(next_item) : cur;
#pragma unroll
        for (int rb = 0; rb < R; ++rb) {
            m_run[rb] = -INFINITY;
            l_run[rb] = 0.f;
#pragma unroll
            for (int mb = 0; mb < MB; ++mb)
#pragma unroll
                for (int r = 0; r < 16; ++r) oacc[rb][mb][r] = 0.f;
        }
        if (cur.n_tiles > 0) scale_store(stage);
        __builtin_amdgcn_s_waitcnt(0x0F70);       // vmcnt(0): this wave's part of the stage has landed
        __syncthreads();                          // ... and everyone is past the previous item's last stage
        flush_out();                              // previous item's output: completes under this item's first stage

        for (int tile = 0; tile < cur.n_tiles; ++tile) {
            const char* sb = smem + stage * kStageBytes;
            const float* sc = s_scale + stage * G::PPS * 2;
            if constexpr (FP8) {
                // Before the next stage is requested: LDS accesses that follow a direct-to-LDS load in program order
                // can be made to wait for it, and these would wait for a load that has just been issued.
                expand_stage(sb, sc);
                __syncthreads();
                sb = hbuf;
            }
            // every wave is past its reads of the other stage (barrier at the end of the previous iteration)
            if (tile + 1 < cur.n_tiles) {
                dma_doc(cur, stage ^ 1);
                ids_after(cur, tile + 1, item);
            } else {
                dma_new(cur, 0, stage ^ 1);
            }
#pragma unroll 1
            for (int st = 0; st < G::TK / 32; ++st) {
                const int key0 = tile * G::TK + st * 32;
                if (key0 >= cur.D) break;
                int nv[R];
#pragma unroll
                for (int rb = 0; rb < R; ++rb) nv[rb] = cur.D - key0;
                process(std::integral_constant<bool, FP8>{}, std::false_type{}, sb, st, blk_on, nv, sc, nullptr);
            }
            if (tile + 1 < cur.n_tiles) scale_store(stage ^ 1);
            __builtin_amdgcn_s_waitcnt(0x0F70);
            __syncthreads();
            stage ^= 1;
        }
        for (int nt = 0; nt < cur.n_new_tiles; ++nt) {
            const bool last = nt + 1 == cur.n_new_tiles;
            if (!last) dma_new(cur, nt + 1, stage ^ 1);
            else if (has_next) {
                dma_first(nxt, stage ^ 1);
                if (nxt.n_tiles > 0) ids_after(nxt, 0, next_item);
            }
            const char* sb = smem + stage * kStageBytes;
#pragma unroll 1
            for (int st = 0; st < SUBS; ++st) {
                const int s = nt * SUBS + st;
                if (s >= cur.n_sub) break;
                int page, seq, key0;
                sub_lookup(cur, s, page, seq, key0);
                // only the blocks of the pair these keys belong to; row i sees new keys 0..i: the sub-tile relative
                // limit is i + 1 - key0
                bool on[R], any = false;
                int nv[R];
#pragma unroll
                for (int rb = 0; rb < R; ++rb) {
                    on[rb] = blk_on[rb] && blk_seq[rb] == seq;
                    nv[rb] = blk_qn[rb] - key0;
                    any = any || on[rb];
                }
                if (!any) continue;                                // wave-uniform
#pragma unroll
                for (int rb = 0; rb < R; ++rb) row_i[rb] -= key0;
                process(std::false_type{}, std::true_type{}, sb, st, on, nv, nullptr, lobuf + stage * kStageBytes);
#pragma unroll
                for (int rb = 0; rb < R; ++rb) row_i[rb] += key0;
            }
            if (!last) {
                __builtin_amdgcn_s_waitcnt(0x0F70);
                __syncthreads();
            }
            stage ^= 1;
        }

        // ---- normalise; the output is packed to half and kept in registers: the stores are issued after the next
        // item's first barrier (flush_out), so neither their issue nor their completion sits in front of a vmcnt wait.
        // The next item's Q fragments are requested now so their latency hides as well.
        if constexpr (DEFER) {
            // every wave is past its reads of the stage the last own-key tile sat in; that stage is free until the next
            // item's second tile is requested (behind the next barrier), and 2 KiB of it per wave turn the output
            asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
        }
        char* tbuf = smem + (stage ^ 1) * kStageBytes + wave_u * (kStageBytes / NW);
#pragma unroll
        for (int rb = 0; rb < R; ++rb) {
            const float l = row_sum2(l_run[rb]);
            const float inv = 1.0f / l;
            if constexpr (PREC) {
                // [hi | lo] halves of the output row, stored right away (this variant does not defer its stores)
                if (row_ok[rb]) {
                    half_t* dst = o + row_off[rb];
#pragma unroll
                    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
                        for (int r4 = 0; r4 < 4; ++r4) {
                            halfx4 hi, lo;
#pragma unroll
                            for (int e = 0; e < 4; ++e) {
                                const float v = oacc[rb][mb][r4 * 4 + e] * inv;
                                hi[e] = from_float<half_t>(v);
                                lo[e] = from_float<half_t>(v - (float)hi[e]);
                            }
                            *(halfx4*)(dst + mb * 32 + 8 * r4 + 4 * hh) = hi;
                            *(halfx4*)(dst + (size_t)n_q * HD + mb * 32 + 8 * r4 + 4 * hh) = lo;
                        }
                }
            } else {
                // where the two chunk rows of this lane go (same row arithmetic as setup_rows)
                const int M = last_only ? g : blk_qn[rb] * g;
#pragma unroll
                for (int j = 0; j < 2; ++j) {
                    const int row = blk_row0[rb] + (lane >> 2) + 16 * j;
                    out_ok[rb][j] = blk_on[rb] && row < M;
                    const int rc = row < M ? row : M - 1;
                    const int i = last_only ? 0 : rc / g, a = last_only ? rc : rc - i * g;
                    out_off[rb][j] = last_only ? ((size_t)blk_seq[rb] * n_q + cur.h * g + a) * HD
                                               : (size_t)(blk_t0[rb] + i) * q_ld + (size_t)(cur.h * g + a) * HD;
                }
                // as many 32-channel units (2 KiB each) per round trip as the wave's share of the stage holds
                constexpr int UPR = (kStageBytes / NW / 2048) < MB ? (kStageBytes / NW / 2048) : MB;
                static_assert(UPR >= 1 && MB % UPR == 0, "units per round");
#pragma unroll
                for (int mb0 = 0; mb0 < MB; mb0 += UPR) {
#pragma unroll
                    for (int u = 0; u < UPR; ++u)
#pragma unroll
                        for (int r4 = 0; r4 < 4; ++r4) {
                            halfx4 w;
#pragma unroll
                            for (int e = 0; e < 4; ++e) w[e] = from_float<half_t>(oacc[rb][mb0 + u][r4 * 4 + e] * inv);
                            *(halfx4*)(tbuf + u * 2048 + ln * 64 + r4 * 16 + hh * 8) = w;
                        }
                    __builtin_amdgcn_wave_barrier();       // LDS accesses of one wave execute in order: written, then read back
#pragma unroll
                    for (int u = 0; u < UPR; ++u)
#pragma unroll
                        for (int j = 0; j < 2; ++j) opk[rb][mb0 + u][j] = *(const ochunk_t*)(tbuf + u * 2048 + (lane + 64 * j) * 16);
                    __builtin_amdgcn_wave_barrier();
                }
            }
        }
        out_pending = DEFER;
        if (has_next) setup_rows(nxt);
        cur = nxt;
    }
    flush_out();
}

template <int HD, int NW, int R, bool FP8, bool PREC>
hipError_t launch_one(const half_t* q, const char* kv_new, const char* kv_new_lo, half_t* o, const MetaView& mv, const PoolView& pv,
                      int layer, int n_q, int last_only, const GroupView& gv, hipStream_t st) {
    constexpr int SB = stage_bytes(FP8);
    const size_t lds = 2 * SB + 2 * Geo<HD, FP8, SB>::PPS * 2 * sizeof(float) + (FP8 ? 2 * SB : 0) + (PREC ? 2 * SB : 0);
    // once per kernel instantiation and device (a host thread may drive any device): the LDS attribute, and the size of
    // the persistent grid = as many workgroups as can be resident (LDS: two per CU), each looping over work items
    constexpr int kMaxDevices = 64;
    static std::atomic<int> max_wgs_dev[kMaxDevices];
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return hipErrorUnknown;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    int max_wgs = max_wgs_dev[dev].load(std::memory_order_acquire);
    if (max_wgs == 0) {
        hipError_t e = hipFuncSetAttribute((const void*)attn_mfma_kernel<HD, NW, R, FP8, PREC>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                           (int)lds);
        if (e != hipSuccess) return e;
        int per_cu = 0, cus = 0;
        if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0) return hipErrorUnknown;
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, attn_mfma_kernel<HD, NW, R, FP8, PREC>, NW * 64, lds) != hipSuccess || per_cu < 1)
            per_cu = 1;
        max_wgs = cus * per_cu;
        max_wgs_dev[dev].store(max_wgs, std::memory_order_release);
    }
    const int n_items = (gv.n_groups > 0 ? gv.n_groups : mv.n_seq) * pv.n_kv;
    const int grid = std::min(n_items, max_wgs);
    attn_mfma_kernel<HD, NW, R, FP8, PREC><<<dim3((unsigned)grid), NW * 64, lds, st>>>(q, kv_new, kv_new_lo, o, mv, pv, layer, n_q, mv.cu, mv.prefix_len,
                                                                                   mv.page_table, mv.new_cu, pv.scales, last_only, gv.n_groups, gv.p0,
                                                                                   gv.blk_cu, gv.sub_cu, gv.blk_seq, gv.blk_row0, gv.sub_page,
                                                                                   gv.sub_seq, gv.sub_key0);
    return hipGetLastError();
}

}  // namespace

// rows per workgroup = (n_q / n_kv) * max_q_len must fit NW * R blocks of 32 (the pair's own keys may take any number of
// stages: they are streamed like document pages)
bool attn_mfma_supported(const hr_model_cfg& c, int kv_dtype, int max_q_len) {
    if (c.dtype != HR_BF16) return false;
    if (kv_dtype != HR_BF16 && kv_dtype != HR_FP8_E4M3) return false;
    if (c.head_dim != 64 && c.head_dim != 128) return false;
    const int g = c.n_q_heads / c.n_kv_heads;
    if ((int64_t)g * max_q_len > kMaxRowsPerWg) return false;
    return true;
}

// The same for a call that travels with a group plan: the row blocks of a long query are spread over work items of at most
// 16 blocks (8 at 128-wide heads), up to kMaxPiecesPerSeq of them.
bool attn_mfma_supported_cut(const hr_model_cfg& c, int kv_dtype, int max_q_len) {
    if (attn_mfma_supported(c, kv_dtype, max_q_len)) return true;
    if (!attn_mfma_supported(c, kv_dtype, 1)) return false;
    const int64_t blocks = ((int64_t)(c.n_q_heads / c.n_kv_heads) * max_q_len + 31) / 32;
    const int cap = c.head_dim == 64 ? 16 : 8;
    return (blocks + cap - 1) / cap <= kMaxPiecesPerSeq;
}

hipError_t launch_attn_mfma(const void* q, const void* kv_new_pages, void* o, const MetaView& mv, const PoolView& pv, int layer,
                            int n_q, int max_q_len, hipStream_t st, bool last_only, const GroupView* groups, const void* kv_new_lo_pages) {
    if (mv.n_seq == 0) return hipSuccess;
    const GroupView gv = groups && !last_only ? *groups : GroupView{};
    const int rows = gv.n_groups > 0 ? gv.max_blocks * 32 : n_q / pv.n_kv * (last_only ? 1 : max_q_len);
    if (rows > kMaxRowsPerWg) return hipErrorInvalidValue;
    const half_t* qh = (const half_t*)q;
    const char* kvn = (const char*)kv_new_pages;
    const char* kvl = (const char*)kv_new_lo_pages;
    half_t* oh = (half_t*)o;
    const bool fp8 = pv.kv_dtype == HR_FP8_E4M3;
    if (kvl) {
        // the 22-bit form: split q / o and lo pages of the new keys (see the kernel); one wave per SIMD, 8 waves
        if (last_only) return hipErrorInvalidValue;
#define HR_ATTN_PREC(HD, R)                                                                                 \
    return fp8 ? launch_one<HD, 8, R, true, true>(qh, kvn, kvl, oh, mv, pv, layer, n_q, 0, gv, st)             \
               : launch_one<HD, 8, R, false, true>(qh, kvn, kvl, oh, mv, pv, layer, n_q, 0, gv, st)
        if (pv.d == 64) {
            if (rows <= 256) { HR_ATTN_PREC(64, 1); }
            HR_ATTN_PREC(64, 2);
        } else {
            if (rows <= 256) { HR_ATTN_PREC(128, 1); }
            HR_ATTN_PREC(128, 2);
        }
#undef HR_ATTN_PREC
    }
#define HR_ATTN_CASE(HD, NW, R)                                                                                   \
    return fp8 ? launch_one<HD, NW, R, true, false>(qh, kvn, nullptr, oh, mv, pv, layer, n_q, last_only ? 1 : 0, gv, st)   \
               : launch_one<HD, NW, R, false, false>(qh, kvn, nullptr, oh, mv, pv, layer, n_q, last_only ? 1 : 0, gv, st)
    if (pv.d == 64) {
        if (rows <= 128) { HR_ATTN_CASE(64, 4, 1); }
        if (rows <= 256) { HR_ATTN_CASE(64, 4, 2); }
        HR_ATTN_CASE(64, 8, 2);
    } else {
        if (rows <= 128) { HR_ATTN_CASE(128, 4, 1); }
        if (rows <= 256) {
            // two row blocks per wave at d = 128 need more registers than two waves per SIMD leave (measured at 256 rows,
            // fp8 pool: 2.1 ms with 4 waves x 2 blocks, 1.3 ms with 8 waves x 1 block)
            HR_ATTN_CASE(128, 8, 1);
        }
        HR_ATTN_CASE(128, 8, 2);
    }
#undef HR_ATTN_CASE
}

}  // namespace hr
