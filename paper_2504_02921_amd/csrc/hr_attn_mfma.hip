// Paged grouped-query prefix attention on MFMA (gfx950): the KV-streaming kernel of the scoring pass.
//
// One workgroup per (pair, kv head).  Its query rows are the g * q_len rows (token i, head a of the
// group) that share this kv head; wave w owns 32-row blocks w, w + NW, ...  The document's pages are
// streamed HBM -> LDS in 32 KiB stages (double buffered, every page is one contiguous burst and is
// copied verbatim: the pool already holds the LDS-friendly arrangement), all keys of the document are
// visible to every row; then the pair's own query keys are staged once and processed with the causal
// mask.  Softmax is the online form in fp32.
//
// MFMA orientation (v_mfma_f32_32x32x16_f16): scores are computed transposed, S^T = K * Q^T, so a
// lane owns ONE query row (column lane & 31) and 16 of the 32 keys of a sub-tile.  Row maxima and
// sums are then in-lane reductions plus a single exchange with lane ^ 32, the probabilities are
// already in B-operand order for O^T += V^T * P^T, and the rescale factor of a row is a per-lane
// scalar.  The 8 keys a lane holds per MFMA are {4h..4h+3, 8+4h..8+4h+3} of a 16-key page, which is
// why pages store V transposed in exactly that grouping.
#include <hip/hip_runtime.h>

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

namespace {

constexpr int kStageBytes = 32768;
constexpr int kMaxRowsPerWg = 512;

template <int HD, bool FP8>
struct Geo {
    static constexpr int ESZ = FP8 ? 1 : 2;
    static constexpr int BLOCK_BYTES = kPageTokens * HD * ESZ;   // one K (or V) block
    static constexpr int PAGE_BYTES = 2 * BLOCK_BYTES;
    static constexpr int PPS = kStageBytes / PAGE_BYTES;         // pages per stage
    static constexpr int TK = kPageTokens * PPS;                 // keys per stage
};

// 8 consecutive fp8 codes (one 64-bit LDS word) -> 8 halves, exact (every E4M3 value is a half)
__device__ __forceinline__ halfx8 fp8x8_to_half(uint2 w) {
    halfx2 a = __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(w.x, 1.0f, false);
    halfx2 b = __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(w.x, 1.0f, true);
    halfx2 c = __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(w.y, 1.0f, false);
    halfx2 d = __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(w.y, 1.0f, true);
    halfx8 r;
    r[0] = a[0]; r[1] = a[1]; r[2] = b[0]; r[3] = b[1]; r[4] = c[0]; r[5] = c[1]; r[6] = d[0]; r[7] = d[1];
    return r;
}

template <int HD, int NW, int R, bool FP8>
__global__ void __launch_bounds__(NW * 64) attn_mfma_kernel(const half_t* __restrict__ q, const half_t* __restrict__ k_new,
                                                           const half_t* __restrict__ v_new, half_t* __restrict__ o,
                                                           MetaView mv, PoolView pv, int layer, int n_q) {
    using G = Geo<HD, FP8>;
    using GN = Geo<HD, false>;                       // the pair's own keys are always half
    constexpr int NT = NW * 64;
    constexpr int NPASS = kStageBytes / (NT * 16);   // 16-byte loads per thread and stage
    constexpr int KC = HD / 16;                      // MFMA k-steps over head_dim
    constexpr int MB = HD / 32;                      // 32-channel blocks of the output
    extern __shared__ __attribute__((aligned(16))) char smem[];      // [2][kStageBytes] + scales
    float* s_scale = (float*)(smem + 2 * kStageBytes);              // [2][PPS][2]  (fp8 only)

    const int n_kv = pv.n_kv;
    const int p = blockIdx.x / n_kv, h = blockIdx.x - p * n_kv;
    const int t0 = mv.cu[p];
    const int qn = mv.cu[p + 1] - t0;
    const int D = mv.prefix_len[p];
    const int g = n_q / n_kv;
    const int M = qn * g;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int ln = lane & 31, hh = lane >> 5;
    const float c_log2 = 1.4426950408889634f / sqrtf((float)HD);

    // ---- this lane's query rows and Q^T fragments (B operand: 8 consecutive channels of one row)
    halfx8 qf[R][KC];
    int row_i[R];          // query token index of the lane's row in block rb
    size_t row_off[R];     // element offset of that row in q / o
    bool row_ok[R];
#pragma unroll
    for (int rb = 0; rb < R; ++rb) {
        int row = (wave + rb * NW) * 32 + ln;
        row_ok[rb] = row < M;
        int rc = row < M ? row : M - 1;
        int i = rc / g, a = rc - i * g;
        row_i[rb] = i;
        row_off[rb] = ((size_t)(t0 + i) * n_q + h * g + a) * HD;
#pragma unroll
        for (int kk = 0; kk < KC; ++kk) qf[rb][kk] = *(const halfx8*)(q + row_off[rb] + (2 * kk + hh) * 8);
    }

    floatx16 oacc[R][MB];
    float m_run[R], l_run[R];
#pragma unroll
    for (int rb = 0; rb < R; ++rb) {
        m_run[rb] = -INFINITY;
        l_run[rb] = 0.f;
#pragma unroll
        for (int mb = 0; mb < MB; ++mb)
#pragma unroll
            for (int r = 0; r < 16; ++r) oacc[rb][mb][r] = 0.f;
    }

    // ---- one 32-key sub-tile held in LDS (two pages) against every row block of this wave
    auto process = [&](auto kv8_tag, auto causal_tag, const char* sb, int st, int key0, int n_valid, const float* sc) {
        constexpr bool KV8 = decltype(kv8_tag)::value;
        constexpr bool CAUSAL = decltype(causal_tag)::value;
        using GG = Geo<HD, KV8>;
        // K fragments (A operand): lane = key row ln of the sub-tile, channels chunk (2 kk + hh)
        halfx8 kf[KC];
        {
            const int t = ln & 15;
            const char* kb = sb + (st * 2 + (ln >> 4)) * GG::PAGE_BYTES;
#pragma unroll
            for (int kk = 0; kk < KC; ++kk) {
                const int e = t * HD + (((2 * kk + hh) ^ k_swizzle(t, HD, GG::ESZ)) << 3);
                if constexpr (KV8) kf[kk] = fp8x8_to_half(*(const uint2*)(kb + e));
                else kf[kk] = *(const halfx8*)(kb + e * 2);
            }
        }
        // V^T fragments (A operand): lane = channel mb*32 + ln, 8 keys of key group hh of page s
        halfx8 vf[MB][2];
#pragma unroll
        for (int s = 0; s < 2; ++s) {
            const char* vb = sb + (st * 2 + s) * GG::PAGE_BYTES + GG::BLOCK_BYTES;
#pragma unroll
            for (int mb = 0; mb < MB; ++mb) {
                const int e = (hh * HD + mb * 32 + ln) * 8;
                if constexpr (KV8) vf[mb][s] = fp8x8_to_half(*(const uint2*)(vb + e));
                else vf[mb][s] = *(const halfx8*)(vb + e * 2);
            }
        }
        float cs0 = c_log2, cs1 = c_log2, vs0 = 1.f, vs1 = 1.f;
        if constexpr (KV8) {
            cs0 *= sc[(st * 2) * 2];
            vs0 = sc[(st * 2) * 2 + 1];
            cs1 *= sc[(st * 2 + 1) * 2];
            vs1 = sc[(st * 2 + 1) * 2 + 1];
        }
#pragma unroll
        for (int rb = 0; rb < R; ++rb) {
            if ((wave + rb * NW) * 32 >= M) continue;          // wave-uniform
            floatx16 s;
#pragma unroll
            for (int r = 0; r < 16; ++r) s[r] = 0.f;
#pragma unroll
            for (int kk = 0; kk < KC; ++kk) s = __builtin_amdgcn_mfma_f32_32x32x16_f16(kf[kk], qf[rb][kk], s, 0, 0, 0);
            // lane holds keys key0 + 8*(r>>2) + 4*hh + (r&3) of query row ln
            const int limit = CAUSAL ? min(n_valid, row_i[rb] + 1) : n_valid;     // keys [0, limit) visible (sub-tile relative)
            const bool need_mask = limit < 32;
            float mx = -INFINITY;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                float v = s[r] * (r < 8 ? cs0 : cs1);
                if (need_mask) {
                    const int key = 8 * (r >> 2) + 4 * hh + (r & 3);
                    v = key < limit ? v : -INFINITY;
                }
                s[r] = v;
                mx = fmaxf(mx, v);
            }
            mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
            const float m_new = fmaxf(m_run[rb], mx);
            const float alpha = m_run[rb] == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(m_run[rb] - m_new);
            const float m_use = m_new == -INFINITY ? 0.f : m_new;   // a row with nothing visible yet keeps p = 0
            float lsum = 0.f;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                float pr = __builtin_amdgcn_exp2f(s[r] - m_use);
                lsum += pr;
                s[r] = pr;
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
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                pf[0][j] = (half_t)(KV8 ? s[j] * vs0 : s[j]);
                pf[1][j] = (half_t)(KV8 ? s[8 + j] * vs1 : s[8 + j]);
            }
#pragma unroll
            for (int mb = 0; mb < MB; ++mb) {
                oacc[rb][mb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(vf[mb][0], pf[0], oacc[rb][mb], 0, 0, 0);
                oacc[rb][mb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(vf[mb][1], pf[1], oacc[rb][mb], 0, 0, 0);
            }
        }
    };

    // ---- document pages: HBM -> registers -> LDS, double buffered
    const int n_pages = (D + kPageTokens - 1) / kPageTokens;
    const int n_tiles = (n_pages + G::PPS - 1) / G::PPS;
    const int32_t* pt = mv.page_table + (size_t)p * mv.pt_stride;
    const char* pool = pv.data;
    const size_t page_stride = (size_t)n_kv * G::PAGE_BYTES;                         // between consecutive page ids
    const char* layer_base = pool + ((size_t)layer * pv.num_pages * n_kv + h) * G::PAGE_BYTES;
    uint4 stg[NPASS];
    float stg_scale = 0.f;
    auto gload = [&](int tile) {
#pragma unroll
        for (int ps = 0; ps < NPASS; ++ps) {
            const int off = ps * NT * 16 + tid * 16;
            const int slot = off / G::PAGE_BYTES, within = off - slot * G::PAGE_BYTES;
            int pgi = tile * G::PPS + slot;
            pgi = pgi < n_pages ? pgi : n_pages - 1;           // past the end: re-read the last page (finite data, masked)
            stg[ps] = *(const uint4*)(layer_base + (size_t)pt[pgi] * page_stride + within);
        }
        if constexpr (FP8) {
            if (tid < G::PPS * 2) {
                int pgi = tile * G::PPS + (tid >> 1);
                pgi = pgi < n_pages ? pgi : n_pages - 1;
                stg_scale = pv.scales[(((size_t)layer * pv.num_pages + pt[pgi]) * n_kv + h) * 2 + (tid & 1)];
            }
        }
    };
    auto lstore = [&](int buf) {
#pragma unroll
        for (int ps = 0; ps < NPASS; ++ps) *(uint4*)(smem + buf * kStageBytes + ps * NT * 16 + tid * 16) = stg[ps];
        if constexpr (FP8) {
            if (tid < G::PPS * 2) s_scale[buf * G::PPS * 2 + tid] = stg_scale;
        }
    };

    if (n_tiles > 0) {
        gload(0);
        lstore(0);
    }
    __syncthreads();
    for (int tile = 0; tile < n_tiles; ++tile) {
        const int cur = tile & 1;
        if (tile + 1 < n_tiles) gload(tile + 1);
        const char* sb = smem + cur * kStageBytes;
        const float* sc = s_scale + cur * G::PPS * 2;
#pragma unroll 1
        for (int st = 0; st < G::TK / 32; ++st) {
            const int key0 = tile * G::TK + st * 32;
            if (key0 >= D) break;
            process(std::integral_constant<bool, FP8>{}, std::false_type{}, sb, st, key0, D - key0, sc);
        }
        if (tile + 1 < n_tiles) lstore(cur ^ 1);
        __syncthreads();
    }

    // ---- the pair's own query keys (causal), staged once as half pseudo-pages in the same arrangement
    {
        const int nq_pages = ((qn + 31) / 32) * 2;                   // whole 32-key sub-tiles
        const int chunks = nq_pages * kPageTokens * (HD / 8);       // 16-byte chunks of K (and of V)
        for (int idx = tid; idx < chunks; idx += NT) {
            const int j = idx / (HD / 8), ch = idx - j * (HD / 8);   // key j, channel chunk ch
            const int pg = j >> 4, t = j & 15;
            halfx8 kv = {0, 0, 0, 0, 0, 0, 0, 0}, vv = {0, 0, 0, 0, 0, 0, 0, 0};
            if (j < qn) {
                const size_t src = ((size_t)(t0 + j) * n_kv + h) * HD + ch * 8;
                kv = *(const halfx8*)(k_new + src);
                vv = *(const halfx8*)(v_new + src);
            }
            char* pb = smem + pg * GN::PAGE_BYTES;
            *(halfx8*)(pb + (t * HD + ((ch ^ k_swizzle(t, HD, 2)) << 3)) * 2) = kv;
            half_t* vb = (half_t*)(pb + GN::BLOCK_BYTES);
#pragma unroll
            for (int e = 0; e < 8; ++e) vb[v_elem(t, ch * 8 + e, HD)] = vv[e];
        }
        __syncthreads();
        for (int st = 0; st < nq_pages / 2; ++st) {
            const int key0 = st * 32;
            // row i sees new keys 0..i: sub-tile relative limit is i + 1 - key0
#pragma unroll
            for (int rb = 0; rb < R; ++rb) row_i[rb] -= key0;
            process(std::false_type{}, std::true_type{}, smem, st, key0, qn - key0, nullptr);
#pragma unroll
            for (int rb = 0; rb < R; ++rb) row_i[rb] += key0;
        }
    }

    // ---- normalise and store: lane owns query row ln of each block, channels mb*32 + 8*(r>>2) + 4*hh + (r&3)
#pragma unroll
    for (int rb = 0; rb < R; ++rb) {
        const float l = l_run[rb] + __shfl_xor(l_run[rb], 32, 64);
        if (!row_ok[rb]) continue;
        const float inv = 1.0f / l;
        half_t* dst = o + row_off[rb];
#pragma unroll
        for (int mb = 0; mb < MB; ++mb)
#pragma unroll
            for (int r4 = 0; r4 < 4; ++r4) {
                halfx4 w;
#pragma unroll
                for (int e = 0; e < 4; ++e) w[e] = from_float<half_t>(oacc[rb][mb][r4 * 4 + e] * inv);
                *(halfx4*)(dst + mb * 32 + 8 * r4 + 4 * hh) = w;
            }
    }
}

template <int HD, int NW, int R, bool FP8>
hipError_t launch_one(const half_t* q, const half_t* k, const half_t* v, half_t* o, const MetaView& mv, const PoolView& pv,
                      int layer, int n_q, hipStream_t st) {
    const size_t lds = 2 * kStageBytes + 2 * Geo<HD, FP8>::PPS * 2 * sizeof(float);
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute((const void*)attn_mfma_kernel<HD, NW, R, FP8>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                           (int)lds);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    attn_mfma_kernel<HD, NW, R, FP8><<<dim3((unsigned)(mv.n_seq * pv.n_kv)), NW * 64, lds, st>>>(q, k, v, o, mv, pv, layer, n_q);
    return hipGetLastError();
}

}  // namespace

// rows per workgroup = (n_q / n_kv) * max_q_len must fit NW * R blocks of 32; the pair's own keys must fit the
// two LDS stages as half pseudo-pages
bool attn_mfma_supported(const hr_model_cfg& c, int kv_dtype, int max_q_len) {
    if (c.dtype != HR_BF16) return false;
    if (kv_dtype != HR_BF16 && kv_dtype != HR_FP8_E4M3) return false;
    if (c.head_dim != 64 && c.head_dim != 128) return false;
    const int g = c.n_q_heads / c.n_kv_heads;
    if ((int64_t)g * max_q_len > kMaxRowsPerWg) return false;
    const int q_keys = (max_q_len + 31) / 32 * 32;
    if ((int64_t)q_keys * c.head_dim * 4 > 2 * kStageBytes) return false;
    return true;
}

hipError_t launch_attn_mfma(const void* q, const void* k_new, const void* v_new, void* o, const MetaView& mv, const PoolView& pv,
                            int layer, int n_q, int max_q_len, hipStream_t st) {
    if (mv.n_seq == 0) return hipSuccess;
    const int rows = n_q / pv.n_kv * max_q_len;
    const half_t* qh = (const half_t*)q;
    const half_t* kh = (const half_t*)k_new;
    const half_t* vh = (const half_t*)v_new;
    half_t* oh = (half_t*)o;
    const bool fp8 = pv.kv_dtype == HR_FP8_E4M3;
#define HR_ATTN_CASE(HD, NW, R)                                                                       \
    return fp8 ? launch_one<HD, NW, R, true>(qh, kh, vh, oh, mv, pv, layer, n_q, st)                   \
               : launch_one<HD, NW, R, false>(qh, kh, vh, oh, mv, pv, layer, n_q, st)
    static int var = -1;
    if (var < 0) {
        const char* e = getenv("HR_ATTN_VARIANT");
        var = e ? atoi(e) : 1;
    }
    if (pv.d == 64) {
        if (rows <= 128) { HR_ATTN_CASE(64, 4, 1); }
        if (rows <= 256) {
            if (var == 1) { HR_ATTN_CASE(64, 8, 1); }
            HR_ATTN_CASE(64, 4, 2);
        }
        HR_ATTN_CASE(64, 8, 2);
    } else {
        if (rows <= 128) { HR_ATTN_CASE(128, 4, 1); }
        if (rows <= 256) {
            if (var == 1) { HR_ATTN_CASE(128, 8, 1); }
            HR_ATTN_CASE(128, 4, 2);
        }
        HR_ATTN_CASE(128, 8, 2);
    }
#undef HR_ATTN_CASE
}

}  // namespace hr
