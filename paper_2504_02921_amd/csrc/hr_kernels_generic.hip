// Shape-agnostic kernels of the scoring pass: fp32 VALU arithmetic, storage type templated.
// They are the whole path for fp32 models and the fallback for shapes the MFMA kernels do not
// cover; the elementwise ones (embedding gather, RMSNorm, RoPE table, scoring head, pool scatter,
// weight packing) serve every path.
#include <hip/hip_runtime.h>

#include <algorithm>

#include "hr_device_types.h"
#include "hr_kernels.h"
#include "hr_layout.h"

namespace hr {

// ------------------------------------------------------------------------------------------------
// embedding gather: x[t][:] = E[token[t]][:]   (fp32 residual stream)
// ------------------------------------------------------------------------------------------------
template <typename T>
__global__ void embed_kernel(const T* __restrict__ E, const int32_t* __restrict__ tok_id, float* __restrict__ x, int H) {
    size_t t = blockIdx.x;
    const T* src = E + (size_t)tok_id[t] * H;
    float* dst = x + t * H;
    for (int c = threadIdx.x; c < H; c += blockDim.x) dst[c] = to_float(src[c]);
}

// ------------------------------------------------------------------------------------------------
// RoPE table: tab[t][j] = (cos, sin)(pos[t] * base^(-2j/d)), angles in fp64, once per call
// ------------------------------------------------------------------------------------------------
__global__ void rope_table_kernel(const int32_t* __restrict__ tok_pos, float2* __restrict__ tab, int64_t T, int half,
                                  double base) {
    int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= T * half) return;
    int64_t t = idx / half;
    int j = (int)(idx - t * half);
    double inv_freq = pow(base, -(double)j / (double)half);
    double ang = (double)tok_pos[t] * inv_freq;
    double s, c;
    sincos(ang, &s, &c);
    tab[idx] = make_float2((float)c, (float)s);
}

// ------------------------------------------------------------------------------------------------
// RMSNorm: y = x * rsqrt(mean(x^2) + eps) * gain ; one 256-thread block per row
// ------------------------------------------------------------------------------------------------
__device__ __forceinline__ float block_sum_256(float v, float* red) {
    v = wave_sum(v);
    int w = threadIdx.x >> 6;
    if ((threadIdx.x & 63) == 0) red[w] = v;
    __syncthreads();
    float r = red[0] + red[1] + red[2] + red[3];
    __syncthreads();
    return r;
}

__device__ __forceinline__ float block_max_256(float v, float* red) {
    v = wave_max(v);
    int w = threadIdx.x >> 6;
    if ((threadIdx.x & 63) == 0) red[w] = v;
    __syncthreads();
    float r = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
    __syncthreads();
    return r;
}

// rows: optional gather, y row t <- x row rows[t]
template <typename T>
__global__ void __launch_bounds__(256) rmsnorm_kernel(const float* __restrict__ x, const float* __restrict__ gain,
                                                      T* __restrict__ y, int H, float eps, const int32_t* __restrict__ rows) {
    __shared__ float red[4];
    size_t t = blockIdx.x;
    const float* xr = x + (rows ? (size_t)rows[t] : t) * H;
    float ss = 0.f;
    for (int c = threadIdx.x; c < H; c += 256) { float v = xr[c]; ss += v * v; }
    ss = block_sum_256(ss, red);
    float rs = 1.0f / sqrtf(ss / (float)H + eps);
    T* yr = y + t * H;
    for (int c = threadIdx.x; c < H; c += 256) yr[c] = from_float<T>(xr[c] * rs * gain[c]);
}

// Same, for 16-bit outputs and H a multiple of 4 up to 4 * 256 * VPT: the row stays in registers between the
// reduction and the scaling (one pass over HBM), 16-byte loads, 8-byte stores.
template <int VPT>
__global__ void __launch_bounds__(256) rmsnorm_vec_kernel(const float* __restrict__ x, const float* __restrict__ gain,
                                                          half_t* __restrict__ y, int H, float eps, const int32_t* __restrict__ rows) {
    __shared__ float red[4];
    const size_t t = blockIdx.x;
    const float4* xr = (const float4*)(x + (rows ? (size_t)rows[t] : t) * H);
    const float4* gr = (const float4*)gain;
    const int n4 = H >> 2;
    float4 v[VPT];
    float ss = 0.f;
#pragma unroll
    for (int i = 0; i < VPT; ++i) {
        const int c = threadIdx.x + i * 256;
        v[i] = c < n4 ? xr[c] : make_float4(0.f, 0.f, 0.f, 0.f);
        ss += v[i].x * v[i].x + v[i].y * v[i].y + v[i].z * v[i].z + v[i].w * v[i].w;
    }
    ss = block_sum_256(ss, red);
    const float rs = 1.0f / sqrtf(ss / (float)H + eps);
    typedef __attribute__((ext_vector_type(4))) _Float16 h4;
    h4* yr = (h4*)(y + t * H);
#pragma unroll
    for (int i = 0; i < VPT; ++i) {
        const int c = threadIdx.x + i * 256;
        if (c < n4) {
            const float4 g = gr[c];
            h4 o;
            o[0] = from_float<half_t>(v[i].x * rs * g.x);
            o[1] = from_float<half_t>(v[i].y * rs * g.y);
            o[2] = from_float<half_t>(v[i].z * rs * g.z);
            o[3] = from_float<half_t>(v[i].w * rs * g.w);
            yr[c] = o;
        }
    }
}

// Split form for the layers that run with 22-bit operands: y = hi + lo, written as [T][hi H | lo H] halves.
__global__ void __launch_bounds__(256) rmsnorm_split_kernel(const float* __restrict__ x, const float* __restrict__ gain,
                                                            half_t* __restrict__ y, int H, float eps, const int32_t* __restrict__ rows) {
    __shared__ float red[4];
    const size_t t = blockIdx.x;
    const float* xr = x + (rows ? (size_t)rows[t] : t) * H;
    float ss = 0.f;
    for (int c = threadIdx.x; c < H; c += 256) { const float v = xr[c]; ss += v * v; }
    ss = block_sum_256(ss, red);
    const float rs = 1.0f / sqrtf(ss / (float)H + eps);
    half_t* yr = y + t * 2 * H;
    for (int c = threadIdx.x; c < H; c += 256) {
        const float v = xr[c] * rs * gain[c];
        const half_t hi = from_float<half_t>(v);
        yr[c] = hi;
        yr[H + c] = from_float<half_t>(v - (float)hi);
    }
}

// ------------------------------------------------------------------------------------------------
// generic GEMM: C[M][N] (+)= A[M][K] W[N][K]^T, 64x64 tile, 256 threads x (4x4), fp32 FMA
// ------------------------------------------------------------------------------------------------
template <typename T>
__global__ void __launch_bounds__(256) gemm_generic_kernel(const T* __restrict__ A, const T* __restrict__ W,
                                                           float* __restrict__ C, int64_t M, int N, int K, int accumulate) {
    constexpr int BM = 64, BN = 64, BK = 16;
    __shared__ float sA[BK][BM + 4];
    __shared__ float sW[BK][BN + 4];
    int64_t m0 = (int64_t)blockIdx.x * BM;
    int n0 = blockIdx.y * BN;
    int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
    float acc[4][4] = {};
    int lr = threadIdx.x >> 2;         // 0..63 tile row loaded by this thread
    int lc = (threadIdx.x & 3) * 4;    // 0,4,8,12 first of 4 k's
    for (int k0 = 0; k0 < K; k0 += BK) {
        for (int u = 0; u < 4; ++u) {
            int kk = k0 + lc + u;
            int64_t am = m0 + lr;
            int wn = n0 + lr;
            sA[lc + u][lr] = (am < M && kk < K) ? to_float(A[am * K + kk]) : 0.f;
            sW[lc + u][lr] = (wn < N && kk < K) ? to_float(W[(size_t)wn * K + kk]) : 0.f;
        }
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < BK; ++kk) {
            float a[4], w[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) { a[i] = sA[kk][ty * 4 + i]; w[i] = sW[kk][tx * 4 + i]; }
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], w[j], acc[i][j]);
        }
        __syncthreads();
    }
    for (int i = 0; i < 4; ++i) {
        int64_t m = m0 + ty * 4 + i;
        if (m >= M) continue;
        for (int j = 0; j < 4; ++j) {
            int n = n0 + tx * 4 + j;
            if (n >= N) continue;
            float* c = C + m * N + n;
            *c = accumulate ? (*c + acc[i][j]) : acc[i][j];
        }
    }
}

// ------------------------------------------------------------------------------------------------
// RoPE + split of the fused projection: qkv fp32 [T][(n_q + 2 n_kv) d] -> q, k (rotated), v
// rotate-half pairing (j, j + d/2); one block per token
// ------------------------------------------------------------------------------------------------
template <typename T>
__global__ void rope_split_kernel(const float* __restrict__ qkv, const float2* __restrict__ tab, T* __restrict__ q,
                                  T* __restrict__ k, T* __restrict__ v, int n_q, int n_kv, int d) {
    size_t t = blockIdx.x;
    int half = d / 2;
    int nqkv = (n_q + 2 * n_kv) * d;
    const float* row = qkv + t * nqkv;
    const float2* tr = tab + t * half;
    int rot_heads = n_q + n_kv;
    for (int idx = threadIdx.x; idx < rot_heads * half; idx += blockDim.x) {
        int hd = idx / half, j = idx - hd * half;
        float x1 = row[hd * d + j], x2 = row[hd * d + j + half];
        float2 cs = tr[j];
        float o1 = x1 * cs.x - x2 * cs.y;
        float o2 = x2 * cs.x + x1 * cs.y;
        T* dst = hd < n_q ? q + (t * n_q + hd) * d : k + (t * n_kv + (hd - n_q)) * d;
        dst[j] = from_float<T>(o1);
        dst[j + half] = from_float<T>(o2);
    }
    const float* vr = row + (size_t)rot_heads * d;
    for (int idx = threadIdx.x; idx < n_kv * d; idx += blockDim.x) v[t * n_kv * d + idx] = from_float<T>(vr[idx]);
}

// The same step behind an MFMA projection that left fp32 rows, with the new tokens' K and V written as 16-slot pages in
// the pool arrangement (token t at slot new_slot[t]).  Used where the projection's fused epilogue cannot be:
//   SPLIT   the layers that run with 22-bit operands: q goes out as [T][hi n_q d | lo n_q d] halves, and K / V twice
//           over: the values rounded to half in kv_hi, what the rounding left out in kv_lo;
//   tok_src the first layer when several sequences carry the same token string: token t takes row tok_src[t] of a
//           projection that was computed once per distinct string (its own position's rotation still applies).
template <bool SPLIT>
__global__ void rope_pages_kernel(const float* __restrict__ qkv, const float2* __restrict__ tab, half_t* __restrict__ q,
                                  half_t* __restrict__ kv_hi, half_t* __restrict__ kv_lo, const int32_t* __restrict__ new_slot,
                                  const int32_t* __restrict__ tok_src, int n_q, int n_kv, int d) {
    const size_t t = blockIdx.x;
    const int half = d / 2;
    const int nqkv = (n_q + 2 * n_kv) * d;
    const float* row = qkv + (tok_src ? (size_t)tok_src[t] : t) * nqkv;
    const float2* tr = tab + t * half;
    const int slot = new_slot[t];
    const size_t page_elems = (size_t)2 * kPageTokens * d;          // K block | V block of one (page, kv head)
    const int ts = slot & 15;
    const int rot_heads = n_q + n_kv;
    const size_t q_ld = (size_t)(SPLIT ? 2 : 1) * n_q * d;
    for (int idx = threadIdx.x; idx < rot_heads * half; idx += blockDim.x) {
        const int hd = idx / half, j = idx - hd * half;
        const float x1 = row[hd * d + j], x2 = row[hd * d + j + half];
        const float2 cs = tr[j];
        const float o1 = rope_lo(x1, x2, cs.x, cs.y);
        const float o2 = rope_hi(x1, x2, cs.x, cs.y);
        const half_t h1 = from_float<half_t>(o1), h2 = from_float<half_t>(o2);
        if (hd < n_q) {
            half_t* dst = q + t * q_ld + (size_t)hd * d;
            dst[j] = h1;
            dst[j + half] = h2;
            if constexpr (SPLIT) {
                dst[(size_t)n_q * d + j] = from_float<half_t>(o1 - (float)h1);
                dst[(size_t)n_q * d + j + half] = from_float<half_t>(o2 - (float)h2);
            }
        } else {
            const size_t blk = ((size_t)(slot >> 4) * n_kv + (hd - n_q)) * page_elems;
            kv_hi[blk + k_elem(ts, j, d, 2)] = h1;
            kv_hi[blk + k_elem(ts, j + half, d, 2)] = h2;
            if constexpr (SPLIT) {
                kv_lo[blk + k_elem(ts, j, d, 2)] = from_float<half_t>(o1 - (float)h1);
                kv_lo[blk + k_elem(ts, j + half, d, 2)] = from_float<half_t>(o2 - (float)h2);
            }
        }
    }
    const float* vr = row + (size_t)rot_heads * d;
    for (int idx = threadIdx.x; idx < n_kv * d; idx += blockDim.x) {
        const int h = idx / d, c = idx - h * d;
        const float v = vr[idx];
        const half_t hi = from_float<half_t>(v);
        const size_t blk = ((size_t)(slot >> 4) * n_kv + h) * page_elems + (size_t)kPageTokens * d;
        kv_hi[blk + v_elem(ts, c, d)] = hi;
        if constexpr (SPLIT) kv_lo[blk + v_elem(ts, c, d)] = from_float<half_t>(v - (float)hi);
    }
}

// ------------------------------------------------------------------------------------------------
// SwiGLU on the fused gate/up projection (rows interleaved in blocks of `ib`)
// ------------------------------------------------------------------------------------------------
template <typename T>
__global__ void swiglu_kernel(const float* __restrict__ gu, T* __restrict__ m, int F, int ib) {
    size_t t = blockIdx.x;
    const float* row = gu + t * 2 * F;
    for (int f = threadIdx.x; f < F; f += blockDim.x) {
        int base = (f / ib) * 2 * ib + f % ib;
        float g = row[base], u = row[base + ib];
        m[t * F + f] = from_float<T>(g / (1.0f + expf(-g)) * u);
    }
}

// ------------------------------------------------------------------------------------------------
// generic prefix + causal attention: one wave per (new token, q head)
//   pass 1: lanes split the keys, scores to LDS; pass 2: lanes split head_dim
// ------------------------------------------------------------------------------------------------
template <typename KVT>
__device__ __forceinline__ float kv_load(const KVT* p, size_t i) { return to_float(p[i]); }
template <>
__device__ __forceinline__ float kv_load<uint8_t>(const uint8_t* p, size_t i) { return e4m3_to_float(p[i]); }

template <typename T, typename KVT>
__global__ void __launch_bounds__(64) attn_generic_kernel(const T* __restrict__ q, const T* __restrict__ k_new,
                                                         const T* __restrict__ v_new, T* __restrict__ o, MetaView mv,
                                                         PoolView pv, int layer, int n_q) {
    extern __shared__ float sm[];
    const int d = pv.d, n_kv = pv.n_kv, g = n_q / n_kv;
    float* sq = sm;
    float* ss = sm + d;
    const int lane = threadIdx.x;
    const size_t t = blockIdx.x;
    const int a = blockIdx.y, h = a / g;
    const int p = mv.tok_seq[t];
    const int t0 = mv.cu[p];
    const int i = (int)t - t0;
    const int D = mv.prefix_len[p];
    const int nkeys = D + i + 1;
    const float scale = 1.0f / sqrtf((float)d);
    const int32_t* pt = mv.page_table + (size_t)p * mv.pt_stride;
    const KVT* pool = (const KVT*)pv.data;
    const size_t blk = (size_t)kPageTokens * d;

    for (int c = lane; c < d; c += 64) sq[c] = to_float(q[(t * n_q + a) * d + c]);
    __syncthreads();

    float mx = -INFINITY;
    for (int j = lane; j < nkeys; j += 64) {
        float s = 0.f;
        if (j < D) {
            int page = pt[j >> 4], slot = j & 15;
            size_t bi = ((((size_t)layer * pv.num_pages + page) * n_kv + h) * 2 + 0);
            const KVT* kr = pool + bi * blk;
            for (int c = 0; c < d; ++c) s = fmaf(sq[c], kv_load<KVT>(kr, k_elem(slot, c, d, (int)sizeof(KVT))), s);
            if (pv.scales) s *= pv.scales[bi];
        } else {
            const T* kr = k_new + ((size_t)(t0 + j - D) * n_kv + h) * d;
            for (int c = 0; c < d; ++c) s = fmaf(sq[c], to_float(kr[c]), s);
        }
        s *= scale;
        ss[j] = s;
        mx = fmaxf(mx, s);
    }
    mx = wave_max(mx);
    float sum = 0.f;
    for (int j = lane; j < nkeys; j += 64) {
        float e = expf(ss[j] - mx);
        ss[j] = e;
        sum += e;
    }
    sum = wave_sum(sum);
    __syncthreads();
    const float inv = 1.0f / sum;
    const int n_pages = (D + kPageTokens - 1) / kPageTokens;
    for (int c = lane; c < d; c += 64) {
        float acc = 0.f;
        for (int pg = 0; pg < n_pages; ++pg) {
            int page = pt[pg];
            size_t bi = ((((size_t)layer * pv.num_pages + page) * n_kv + h) * 2 + 1);
            const KVT* vb = pool + bi * blk;
            float part = 0.f;
            int lim = min(kPageTokens, D - pg * kPageTokens);
            for (int tk = 0; tk < lim; ++tk) part = fmaf(ss[pg * kPageTokens + tk], kv_load<KVT>(vb, v_elem(tk, c, d)), part);
            acc += pv.scales ? part * pv.scales[bi] : part;
        }
        for (int j = 0; j <= i; ++j) acc = fmaf(ss[D + j], to_float(v_new[((size_t)(t0 + j) * n_kv + h) * d + c]), acc);
        o[(t * n_q + a) * d + c] = from_float<T>(acc * inv);
    }
}

// ------------------------------------------------------------------------------------------------
// scoring head: final RMSNorm on each sequence's last token, then <y, E[yes]> - <y, E[no]>
// ------------------------------------------------------------------------------------------------
template <typename T>
__global__ void __launch_bounds__(256) score_head_kernel(const float* __restrict__ x, const float* __restrict__ gain,
                                                         const T* __restrict__ E, const int32_t* __restrict__ out_row,
                                                         float* __restrict__ scores, int H, float eps, int yes_id, int no_id) {
    __shared__ float red[4];
    int p = blockIdx.x;
    const float* xr = x + (size_t)(out_row ? out_row[p] : p) * H;     // no table: row p
    float ssq = 0.f;
    for (int c = threadIdx.x; c < H; c += 256) { float v = xr[c]; ssq += v * v; }
    ssq = block_sum_256(ssq, red);
    float rs = 1.0f / sqrtf(ssq / (float)H + eps);
    const T* ey = E + (size_t)yes_id * H;
    const T* en = E + (size_t)no_id * H;
    float acc = 0.f;
    for (int c = threadIdx.x; c < H; c += 256) acc += xr[c] * rs * gain[c] * (to_float(ey[c]) - to_float(en[c]));
    acc = block_sum_256(acc, red);
    if (threadIdx.x == 0) scores[p] = acc;
}

// ------------------------------------------------------------------------------------------------
struct PageIdChunk { int32_t ids[256]; };   // page ids travel as kernel arguments: no device staging

// pool write: logical [L][D][n_kv][d] -> pages in the private arrangement (see hr_layout.h), tail zeroed
// grid: (n_pages, n_layers * n_kv); 256 threads
// ------------------------------------------------------------------------------------------------
template <typename SRC, typename DST> __device__ __forceinline__ DST kv_convert(SRC v) { return (DST)v; }
// 16-bit pools: the caller's bf16 values are stored as half (exact for |x| in [2^-14, 65504]; smaller
// magnitudes keep an absolute error below 2^-25, larger ones become infinity; both are counted)
template <> __device__ __forceinline__ half_t kv_convert<bf16_t, half_t>(bf16_t v) { return from_float<half_t>((float)v); }

__device__ __forceinline__ void flush_range_counts(long long* counters, int over, int under, int nonfinite, int nan_code, int bad_scale) {
    if (!counters) return;
    if (over) atomicAdd((unsigned long long*)(counters + RC_OVERFLOW), (unsigned long long)over);
    if (under) atomicAdd((unsigned long long*)(counters + RC_UNDERFLOW), (unsigned long long)under);
    if (nonfinite) atomicAdd((unsigned long long*)(counters + RC_NONFINITE_IN), (unsigned long long)nonfinite);
    if (nan_code) atomicAdd((unsigned long long*)(counters + RC_FP8_NAN_CODE), (unsigned long long)nan_code);
    if (bad_scale) atomicAdd((unsigned long long*)(counters + RC_FP8_BAD_SCALE), (unsigned long long)bad_scale);
}

template <typename KVT, typename KVS>
__global__ void __launch_bounds__(256) kv_scatter_kernel(KVT* __restrict__ pool, float* __restrict__ scales,
                                                         PageIdChunk page_ids, int pg0, int doc_len, int n_pages,
                                                         const KVS* __restrict__ k, const KVS* __restrict__ v,
                                                         const float* __restrict__ ks, const float* __restrict__ vs,
                                                         int num_pages, int n_kv, int d, long long* __restrict__ counters) {
    int pg = pg0 + blockIdx.x;
    int layer = blockIdx.y / n_kv, h = blockIdx.y % n_kv;
    int page = page_ids.ids[blockIdx.x];
    size_t blk = (size_t)kPageTokens * d;
    size_t bi = (((size_t)layer * num_pages + page) * n_kv + h) * 2;
    KVT* kb = pool + bi * blk;
    KVT* vb = kb + blk;
    int over = 0, under = 0, nonfinite = 0, nan_code = 0, bad_scale = 0;
    for (int e = threadIdx.x; e < (int)blk; e += 256) {
        int tk = e / d, c = e - tk * d;
        int tok = pg * kPageTokens + tk;
        KVT kvl = KVT(0.0f), vvl = KVT(0.0f);
        if (tok < doc_len) {
            size_t src = (((size_t)layer * doc_len + tok) * n_kv + h) * d + c;
            kvl = kv_convert<KVS, KVT>(k[src]);
            vvl = kv_convert<KVS, KVT>(v[src]);
            if constexpr (sizeof(KVT) == 2) {
                count_half_range((float)k[src], over, under, nonfinite);
                count_half_range((float)v[src], over, under, nonfinite);
            } else if constexpr (sizeof(KVT) == 1) {          // E4M3 has two NaN codes and no infinity
                nan_code += ((unsigned)k[src] & 0x7Fu) == 0x7Fu;
                nan_code += ((unsigned)v[src] & 0x7Fu) == 0x7Fu;
            }
        }
        kb[k_elem(tk, c, d, (int)sizeof(KVT))] = kvl;
        vb[v_elem(tk, c, d)] = vvl;
    }
    if (scales && threadIdx.x == 0) {
        size_t si = ((size_t)layer * n_pages + pg) * n_kv + h;
        const float sk = ks[si], sv = vs[si];
        scales[bi] = sk;
        scales[bi + 1] = sv;
        // a scale must be positive and finite; the V scale's power of two is applied while the codes are expanded to
        // half, which covers 2^-22 <= scale < 2^8
        bad_scale += !(sk > 0.0f && sk <= 3.0e38f);
        bad_scale += !(sv >= 2.384185791015625e-07f && sv < 256.0f);
    }
    flush_range_counts(counters, over, under, nonfinite, nan_code, bad_scale);
}

template <typename S, typename D>
__global__ void pack_rows_kernel(const S* __restrict__ src, D* __restrict__ dst, int rows, int cols, int ib, int mul, int sel,
                                 long long* __restrict__ counters) {
    int r = blockIdx.x;
    if (r >= rows) return;
    size_t drow = ((size_t)(r / ib) * mul + sel) * ib + r % ib;
    int over = 0, under = 0, nonfinite = 0;
    for (int c = threadIdx.x; c < cols; c += blockDim.x) {
        const float v = to_float<S>(src[(size_t)r * cols + c]);
        if constexpr (sizeof(D) == 2) count_half_range(v, over, under, nonfinite);
        dst[drow * cols + c] = from_float<D>(v);
    }
    flush_range_counts(counters, over, under, nonfinite, 0, 0);
}

__global__ void fill_zero_kernel(uint4* dst, size_t n16) {
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (; i < n16; i += stride) dst[i] = make_uint4(0, 0, 0, 0);
}

__global__ void pages_to_pool_kernel(const uint4* __restrict__ src, uint4* __restrict__ dst, const int32_t* __restrict__ src_page,
                                     const int32_t* __restrict__ dst_page, int n16) {
    const uint4* s = src + (size_t)src_page[blockIdx.x] * n16;
    uint4* d = dst + (size_t)dst_page[blockIdx.x] * n16;
    for (int i = threadIdx.x; i < n16; i += blockDim.x) d[i] = s[i];
}

// Round to the nearest E4M3 value, ties to the even code, saturating at +-448 (bias 7, subnormals m/8 * 2^-6, no
// infinities).  fp64 in, so that a quotient computed in fp64 is rounded once.
__device__ __forceinline__ uint8_t e4m3_encode_rne(double q) {
    const double a = fmin(fabs(q), 448.0);
    int e;
    frexp(a, &e);                                   // a = f * 2^e, f in [0.5, 1): floor(log2 a) = e - 1 (a = 0: e = 0)
    int eb = (a > 0.0 ? e - 1 : -6);
    eb = eb < -6 ? -6 : eb;                         // the subnormal range shares the spacing of the first binade
    const double n = rint(ldexp(a, 3 - eb));       // multiples of the spacing 2^(eb - 3); rint = ties to even; 0 .. 16
    int code;
    if (n < 8.0) code = (int)n;                     // subnormal (only when eb = -6)
    else if (n < 16.0) code = ((eb + 7) << 3) | ((int)n - 8);
    else code = (eb + 8) << 3;                      // rounded up into the next binade (never past 448: a <= 448 = 1.75 * 2^8)
    return (uint8_t)(code | (q < 0.0 || (q == 0.0 && signbit(q)) ? 0x80 : 0));
}

// fp8 pools, document prefill: half pages of this pass -> quantised pool pages.  One workgroup per (page, kv head):
// amax over the page's K block and over its V block (slots past the document's end hold zeros), scale = amax / 448
// (1 when amax = 0) in fp32, code = encode(x / scale) with the quotient in fp64.
__global__ void __launch_bounds__(256) pages_to_pool_fp8_kernel(const half_t* __restrict__ src, uint8_t* __restrict__ dst,
                                                               float* __restrict__ scales, const int32_t* __restrict__ src_page,
                                                               const int32_t* __restrict__ dst_page, int n_kv, int d) {
    __shared__ float red[4];
    const int h = blockIdx.y;
    const int blk = kPageTokens * d;
    const half_t* sp = src + ((size_t)src_page[blockIdx.x] * n_kv + h) * (2 * blk);
    const size_t dpage = (size_t)dst_page[blockIdx.x] * n_kv + h;
    uint8_t* dp = dst + dpage * (2 * blk);
    float amax[2];
    for (int part = 0; part < 2; ++part) {
        float m = 0.f;
        for (int e = threadIdx.x; e < blk; e += 256) m = fmaxf(m, fabsf((float)sp[part * blk + e]));
        amax[part] = block_max_256(m, red);
    }
    const float sk = amax[0] > 0.f ? amax[0] / 448.0f : 1.0f, sv = amax[1] > 0.f ? amax[1] / 448.0f : 1.0f;
    for (int e = threadIdx.x; e < blk; e += 256) {
        const int t = e / d, c = e - t * d;
        dp[k_elem(t, c, d, 1)] = e4m3_encode_rne((double)(float)sp[k_elem(t, c, d, 2)] / (double)sk);
        dp[blk + v_elem(t, c, d)] = e4m3_encode_rne((double)(float)sp[blk + v_elem(t, c, d)] / (double)sv);
    }
    if (threadIdx.x == 0) {
        scales[dpage * 2] = sk;
        scales[dpage * 2 + 1] = sv;
    }
}

// pool read-back: pages in the private arrangement -> logical [L][D][n_kv][d] in the pool's own element type
// grid: (n_pages, n_layers * n_kv); 256 threads
template <typename KVT>
__global__ void __launch_bounds__(256) kv_gather_kernel(const KVT* __restrict__ pool, const float* __restrict__ scales, PageIdChunk page_ids,
                                                        int pg0, int doc_len, int n_pages, KVT* __restrict__ k, KVT* __restrict__ v,
                                                        float* __restrict__ ks, float* __restrict__ vs, int num_pages, int n_kv, int d) {
    const int pg = pg0 + blockIdx.x;
    const int layer = blockIdx.y / n_kv, h = blockIdx.y % n_kv;
    const int page = page_ids.ids[blockIdx.x];
    const size_t blk = (size_t)kPageTokens * d;
    const size_t bi = (((size_t)layer * num_pages + page) * n_kv + h) * 2;
    const KVT* kb = pool + bi * blk;
    const KVT* vb = kb + blk;
    for (int e = threadIdx.x; e < (int)blk; e += 256) {
        const int tk = e / d, c = e - tk * d;
        const int tok = pg * kPageTokens + tk;
        if (tok >= doc_len) continue;
        const size_t o = (((size_t)layer * doc_len + tok) * n_kv + h) * d + c;
        k[o] = kb[k_elem(tk, c, d, (int)sizeof(KVT))];
        v[o] = vb[v_elem(tk, c, d)];
    }
    if (scales && threadIdx.x == 0) {
        const size_t si = ((size_t)layer * n_pages + pg) * n_kv + h;
        ks[si] = scales[bi];
        vs[si] = scales[bi + 1];
    }
}

// ------------------------------------------------------------------------------------------------
// launchers
// ------------------------------------------------------------------------------------------------
hipError_t launch_pages_to_pool_fp8(const char* kv_new, char* pool_layer_base, float* scales_layer_base, const int32_t* src_page,
                                    const int32_t* dst_page, int n_pages, int n_kv, int d, hipStream_t st) {
    if (n_pages == 0) return hipSuccess;
    pages_to_pool_fp8_kernel<<<dim3((unsigned)n_pages, (unsigned)n_kv), 256, 0, st>>>((const half_t*)kv_new, (uint8_t*)pool_layer_base,
                                                                                     scales_layer_base, src_page, dst_page, n_kv, d);
    return hipGetLastError();
}

hipError_t launch_kv_gather(const PoolLayout& lay, const char* pool_base, const int32_t* page_ids_host, int doc_len, void* k, void* v,
                            float* ks, float* vs, hipStream_t st) {
    const int n_pages = (doc_len + kPageTokens - 1) / kPageTokens;
    const float* scales = lay.kv_dtype == HR_FP8_E4M3 ? (const float*)(pool_base + lay.data_bytes) : nullptr;
    for (int pg0 = 0; pg0 < n_pages; pg0 += 256) {
        const int n = n_pages - pg0 < 256 ? n_pages - pg0 : 256;
        PageIdChunk ids;
        for (int i = 0; i < 256; ++i) ids.ids[i] = i < n ? page_ids_host[pg0 + i] : 0;
        const dim3 grid((unsigned)n, (unsigned)(lay.n_layers * lay.n_kv));
        if (lay.kv_dtype == HR_F32)
            kv_gather_kernel<float><<<grid, 256, 0, st>>>((const float*)pool_base, nullptr, ids, pg0, doc_len, n_pages, (float*)k, (float*)v,
                                                          nullptr, nullptr, lay.num_pages, lay.n_kv, lay.d);
        else if (lay.kv_dtype == HR_BF16)
            kv_gather_kernel<half_t><<<grid, 256, 0, st>>>((const half_t*)pool_base, nullptr, ids, pg0, doc_len, n_pages, (half_t*)k,
                                                           (half_t*)v, nullptr, nullptr, lay.num_pages, lay.n_kv, lay.d);
        else
            kv_gather_kernel<uint8_t><<<grid, 256, 0, st>>>((const uint8_t*)pool_base, scales, ids, pg0, doc_len, n_pages, (uint8_t*)k,
                                                            (uint8_t*)v, ks, vs, lay.num_pages, lay.n_kv, lay.d);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

hipError_t launch_pages_to_pool(const char* kv_new, char* pool_layer_base, const int32_t* src_page, const int32_t* dst_page,
                                int n_pages, int page_bytes_all_heads, hipStream_t st) {
    if (n_pages == 0) return hipSuccess;
    pages_to_pool_kernel<<<dim3((unsigned)n_pages), 256, 0, st>>>((const uint4*)kv_new, (uint4*)pool_layer_base, src_page, dst_page,
                                                                  page_bytes_all_heads / 16);
    return hipGetLastError();
}

hipError_t launch_fill_zero(void* dst, size_t bytes, hipStream_t st) {     // bytes: multiple of 16
    if (bytes == 0) return hipSuccess;
    const size_t n16 = bytes / 16;
    const unsigned blocks = (unsigned)std::min<size_t>((n16 + 255) / 256, 4096);
    fill_zero_kernel<<<dim3(blocks), 256, 0, st>>>((uint4*)dst, n16);
    return hipGetLastError();
}

#define HR_DISPATCH_ACT(dtype, ...)                                   \
    do {                                                              \
        if ((dtype) == HR_F32) { using AT = float; __VA_ARGS__; }      \
        else { using AT = half_t; __VA_ARGS__; }                        \
    } while (0)

#define HR_DISPATCH_EMB(dtype, ...)                                   \
    do {                                                              \
        if ((dtype) == HR_F32) { using AT = float; __VA_ARGS__; }     \
        else { using AT = bf16_t; __VA_ARGS__; }                      \
    } while (0)

hipError_t launch_embed(int dtype, const void* E, const MetaView& mv, float* x, int H, hipStream_t st) {
    if (mv.T == 0) return hipSuccess;
    HR_DISPATCH_EMB(dtype, embed_kernel<AT><<<dim3((unsigned)mv.T), 256, 0, st>>>((const AT*)E, mv.tok_id, x, H));
    return hipGetLastError();
}

hipError_t launch_rope_table(const MetaView& mv, float2* tab, int head_dim, float base, hipStream_t st) {
    if (mv.T == 0) return hipSuccess;
    int half = head_dim / 2;
    int64_t n = mv.T * half;
    rope_table_kernel<<<dim3((unsigned)((n + 255) / 256)), 256, 0, st>>>(mv.tok_pos, tab, mv.T, half, (double)base);
    return hipGetLastError();
}

hipError_t launch_rmsnorm(int dtype, const float* x, const float* gain, void* y, int64_t T, int H, float eps, hipStream_t st,
                          const int32_t* rows) {
    if (T == 0) return hipSuccess;
    if (dtype != HR_F32 && H % 4 == 0 && H <= 4096) {
        if (H <= 1024) rmsnorm_vec_kernel<1><<<dim3((unsigned)T), 256, 0, st>>>(x, gain, (half_t*)y, H, eps, rows);
        else if (H <= 2048) rmsnorm_vec_kernel<2><<<dim3((unsigned)T), 256, 0, st>>>(x, gain, (half_t*)y, H, eps, rows);
        else rmsnorm_vec_kernel<4><<<dim3((unsigned)T), 256, 0, st>>>(x, gain, (half_t*)y, H, eps, rows);
        return hipGetLastError();
    }
    HR_DISPATCH_ACT(dtype, rmsnorm_kernel<AT><<<dim3((unsigned)T), 256, 0, st>>>(x, gain, (AT*)y, H, eps, rows));
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
// Yardstick for the memory side: a read-only pass over a buffer.  Plain form: 16-byte loads into registers, eight in
// flight per lane, XOR-folded so that nothing can be dropped.  LDS form: the direct-to-LDS loads the attention kernel
// streams with (16 bytes per lane, a ring of 16 one-KiB slots per wave, at most 16 loads in flight per wave).
// ------------------------------------------------------------------------------------------------
typedef __attribute__((address_space(3))) void* probe_lds_ptr_t;
typedef const __attribute__((address_space(1))) void* probe_gbl_ptr_t;

typedef __attribute__((ext_vector_type(4))) unsigned probe_u4;

__global__ void __launch_bounds__(256) probe_read_kernel(const probe_u4* __restrict__ src, size_t n16, unsigned* __restrict__ sink,
                                                         unsigned sink_mask) {
    // grid-stride, eight non-temporal 16-byte loads in flight per lane (measured on a 4 GiB buffer: 6.7 TB/s with 32
    // workgroups per CU; 6.0 without the non-temporal hint, 5.5 with 8 workgroups per CU and four loads)
    constexpr int U = 8;
    const size_t stride = (size_t)gridDim.x * 256;
    size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    probe_u4 acc = {0, 0, 0, 0};
    for (; i + (U - 1) * stride < n16; i += U * stride) {
        probe_u4 v[U];
#pragma unroll
        for (int u = 0; u < U; ++u) v[u] = __builtin_nontemporal_load(src + i + u * stride);
#pragma unroll
        for (int u = 0; u < U; ++u) acc ^= v[u];
    }
    for (; i < n16; i += stride) acc ^= __builtin_nontemporal_load(src + i);
    sink[((size_t)blockIdx.x * 256 + threadIdx.x) & sink_mask] = acc.x ^ acc.y ^ acc.z ^ acc.w;
}

__global__ void __launch_bounds__(256) probe_read_lds_kernel(const char* __restrict__ src, size_t n_kib, unsigned* __restrict__ sink,
                                                             unsigned sink_mask) {
    __shared__ __attribute__((aligned(16))) char ring[4 * 16 * 1024];       // 4 waves x 16 slots x 1 KiB
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const size_t n_waves = (size_t)gridDim.x * 4;
    char* mine = ring + wave * 16 * 1024;
    int slot = 0;
    for (size_t k = (size_t)blockIdx.x * 4 + wave; k < n_kib; k += n_waves) {
        __builtin_amdgcn_global_load_lds((probe_gbl_ptr_t)(src + k * 1024 + lane * 16), (probe_lds_ptr_t)(mine + slot * 1024), 16, 0, 0);
        slot = (slot + 1) & 15;
        __builtin_amdgcn_s_waitcnt(0x0F7F);       // vmcnt(15): the slot about to be reused has landed
    }
    __builtin_amdgcn_s_waitcnt(0x0F70);
    sink[((size_t)blockIdx.x * 256 + threadIdx.x) & sink_mask] = *(const unsigned*)(mine + lane * 16);
}

hipError_t launch_probe_read(const void* src, size_t bytes, void* sink, size_t sink_bytes, bool to_lds, int cus, hipStream_t st) {
    if (bytes < 1024 || sink_bytes < 4) return hipSuccess;
    unsigned mask = 1;
    while ((size_t)(mask << 1) * 4 <= sink_bytes && mask < (1u << 20)) mask <<= 1;     // largest power of two of words that fits
    const unsigned cu = (unsigned)std::max(1, cus);
    if (to_lds) probe_read_lds_kernel<<<dim3(cu * 8), 256, 0, st>>>((const char*)src, bytes / 1024, (unsigned*)sink, mask - 1);
    else probe_read_kernel<<<dim3(cu * 32), 256, 0, st>>>((const probe_u4*)src, bytes / 16, (unsigned*)sink, mask - 1);
    return hipGetLastError();
}

hipError_t launch_rmsnorm_split(const float* x, const float* gain, void* y, int64_t T, int H, float eps, hipStream_t st,
                                const int32_t* rows) {
    if (T == 0) return hipSuccess;
    rmsnorm_split_kernel<<<dim3((unsigned)T), 256, 0, st>>>(x, gain, (half_t*)y, H, eps, rows);
    return hipGetLastError();
}

hipError_t launch_rope_pages(const float* qkv, const float2* tab, void* q, void* kv_hi, void* kv_lo, const int32_t* new_slot,
                             const int32_t* tok_src, int64_t T, int n_q, int n_kv, int d, hipStream_t st) {
    if (T == 0) return hipSuccess;
    if (kv_lo)
        rope_pages_kernel<true><<<dim3((unsigned)T), 256, 0, st>>>(qkv, tab, (half_t*)q, (half_t*)kv_hi, (half_t*)kv_lo, new_slot, tok_src,
                                                                   n_q, n_kv, d);
    else
        rope_pages_kernel<false><<<dim3((unsigned)T), 256, 0, st>>>(qkv, tab, (half_t*)q, (half_t*)kv_hi, nullptr, new_slot, tok_src, n_q,
                                                                    n_kv, d);
    return hipGetLastError();
}

hipError_t launch_gemm_generic(int dtype, const void* A, const void* W, float* C, int64_t M, int N, int K, bool accumulate,
                               hipStream_t st) {
    if (M == 0) return hipSuccess;
    dim3 grid((unsigned)((M + 63) / 64), (unsigned)((N + 63) / 64));
    HR_DISPATCH_ACT(dtype, gemm_generic_kernel<AT><<<grid, 256, 0, st>>>((const AT*)A, (const AT*)W, C, M, N, K, accumulate ? 1 : 0));
    return hipGetLastError();
}

hipError_t launch_rope_split(int dtype, const float* qkv, const float2* tab, void* q, void* k, void* v, int64_t T, int n_q,
                             int n_kv, int d, hipStream_t st) {
    if (T == 0) return hipSuccess;
    HR_DISPATCH_ACT(dtype, rope_split_kernel<AT><<<dim3((unsigned)T), 256, 0, st>>>(qkv, tab, (AT*)q, (AT*)k, (AT*)v, n_q, n_kv, d));
    return hipGetLastError();
}

hipError_t launch_swiglu(int dtype, const float* gu, void* m, int64_t T, int F, int interleave, hipStream_t st) {
    if (T == 0) return hipSuccess;
    HR_DISPATCH_ACT(dtype, swiglu_kernel<AT><<<dim3((unsigned)T), 256, 0, st>>>(gu, (AT*)m, F, interleave));
    return hipGetLastError();
}

hipError_t launch_attn_generic(int dtype, const void* q, const void* k_new, const void* v_new, void* o, const MetaView& mv,
                               const PoolView& pv, int layer, int n_q, int max_keys, hipStream_t st) {
    if (mv.T == 0) return hipSuccess;
    dim3 grid((unsigned)mv.T, (unsigned)n_q);
    size_t lds = (size_t)(pv.d + max_keys) * sizeof(float);
    if (dtype == HR_F32) {
        attn_generic_kernel<float, float><<<grid, 64, lds, st>>>((const float*)q, (const float*)k_new, (const float*)v_new,
                                                                 (float*)o, mv, pv, layer, n_q);
    } else if (pv.kv_dtype == HR_FP8_E4M3) {
        attn_generic_kernel<half_t, uint8_t><<<grid, 64, lds, st>>>((const half_t*)q, (const half_t*)k_new,
                                                                    (const half_t*)v_new, (half_t*)o, mv, pv, layer, n_q);
    } else {
        attn_generic_kernel<half_t, half_t><<<grid, 64, lds, st>>>((const half_t*)q, (const half_t*)k_new,
                                                                   (const half_t*)v_new, (half_t*)o, mv, pv, layer, n_q);
    }
    return hipGetLastError();
}

hipError_t launch_score_head(int dtype, const float* x, const float* gain, const void* E, const MetaView& mv, float* scores,
                             int H, float eps, int yes_id, int no_id, hipStream_t st) {
    if (mv.n_out == 0) return hipSuccess;
    HR_DISPATCH_EMB(dtype, score_head_kernel<AT><<<dim3((unsigned)mv.n_out), 256, 0, st>>>(x, gain, (const AT*)E, mv.out_row, scores, H,
                                                                                        eps, yes_id, no_id));
    return hipGetLastError();
}

hipError_t launch_kv_scatter(const PoolLayout& lay, char* pool_base, const int32_t* page_ids_host, int doc_len, const void* k,
                             const void* v, const float* ks, const float* vs, long long* counters, hipStream_t st) {
    int n_pages = (doc_len + kPageTokens - 1) / kPageTokens;
    float* scales = lay.kv_dtype == HR_FP8_E4M3 ? (float*)(pool_base + lay.data_bytes) : nullptr;
    for (int pg0 = 0; pg0 < n_pages; pg0 += 256) {
        int n = n_pages - pg0 < 256 ? n_pages - pg0 : 256;
        PageIdChunk ids;
        for (int i = 0; i < 256; ++i) ids.ids[i] = i < n ? page_ids_host[pg0 + i] : 0;
        dim3 grid((unsigned)n, (unsigned)(lay.n_layers * lay.n_kv));
        if (lay.kv_dtype == HR_F32)
            kv_scatter_kernel<float, float><<<grid, 256, 0, st>>>((float*)pool_base, nullptr, ids, pg0, doc_len, n_pages,
                                                           (const float*)k, (const float*)v, nullptr, nullptr, lay.num_pages,
                                                           lay.n_kv, lay.d, counters);
        else if (lay.kv_dtype == HR_BF16)
            kv_scatter_kernel<half_t, bf16_t><<<grid, 256, 0, st>>>((half_t*)pool_base, nullptr, ids, pg0, doc_len, n_pages,
                                                              (const bf16_t*)k, (const bf16_t*)v, nullptr, nullptr,
                                                              lay.num_pages, lay.n_kv, lay.d, counters);
        else
            kv_scatter_kernel<uint8_t, uint8_t><<<grid, 256, 0, st>>>((uint8_t*)pool_base, scales, ids, pg0, doc_len, n_pages,
                                                             (const uint8_t*)k, (const uint8_t*)v, ks, vs, lay.num_pages,
                                                             lay.n_kv, lay.d, counters);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

hipError_t launch_pack_rows(int dtype, const void* src, void* dst, int rows, int cols, int ib, int mul, int sel,
                            long long* counters, hipStream_t st) {
    if (dtype == HR_F32)
        pack_rows_kernel<float, float><<<dim3((unsigned)rows), 256, 0, st>>>((const float*)src, (float*)dst, rows, cols, ib, mul, sel, counters);
    else   // the caller's bf16 weights become half operands (same rule as kv_convert)
        pack_rows_kernel<bf16_t, half_t><<<dim3((unsigned)rows), 256, 0, st>>>((const bf16_t*)src, (half_t*)dst, rows, cols, ib,
                                                                              mul, sel, counters);
    return hipGetLastError();
}


// ---- host tier: whole pages between the pool and page records; a (page, layer) unit is n_kv * (K block + V block)
// bytes, contiguous on both sides, moved as 16-byte words.
// Out of the pool: one workgroup per unit; the first 2 * n_kv threads also move the layer's fp8 scales.
// Into the pool: a fixed, small number of workgroups walk the chunk's records word by word in record order, eight
// 16-byte loads in flight per thread.  The records may be pinned host memory behind the bus, and a page-in usually runs
// next to a scoring call that fills the compute units: a few long-lived workgroups hold on to the slots they have won
// and keep ~1 MB of reads outstanding, where thousands of short ones wait for a slot each (measured at the 0.5B shape
// next to scoring: 53 against 44 GB/s sustained over a batch; alone both reach the bus rate).
namespace {
constexpr int kPageInWalkers = 64;    // measured: 16 too few (40 GB/s), 32..64 the bus rate, 96 and more lose again
constexpr int kPageIn4Walkers = 128;  // 4-bit records (one unit in flight ahead per workgroup): 32 too few, 96..128 best

__global__ void __launch_bounds__(256) pages_out_kernel(const char* __restrict__ pool, const float* __restrict__ scales,
                                                        PageIdChunk page_ids, char* __restrict__ records, size_t record_bytes,
                                                        int layer_bytes, int n_layers, int num_pages, int n_kv) {
    const int page = page_ids.ids[blockIdx.x], layer = blockIdx.y;
    char* rec = records + (size_t)blockIdx.x * record_bytes;
    const uint4* src = (const uint4*)(pool + ((size_t)layer * num_pages + page) * layer_bytes);
    uint4* dst = (uint4*)(rec + (size_t)layer * layer_bytes);
    const int n = layer_bytes / 16;
    for (int i0 = threadIdx.x; i0 < n; i0 += 4 * 256) {
        uint4 v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u)
            if (i0 + u * 256 < n) v[u] = src[i0 + u * 256];
#pragma unroll
        for (int u = 0; u < 4; ++u)
            if (i0 + u * 256 < n) dst[i0 + u * 256] = v[u];
    }
    if (scales && (int)threadIdx.x < 2 * n_kv)
        ((float*)(rec + (size_t)n_layers * layer_bytes))[(size_t)layer * n_kv * 2 + threadIdx.x] =
            scales[((size_t)layer * num_pages + page) * n_kv * 2 + threadIdx.x];
}

__global__ void __launch_bounds__(256) pages_in_kernel(char* __restrict__ pool, float* __restrict__ scales, PageIdChunk page_ids,
                                                       const char* __restrict__ records, size_t record_bytes, int layer_bytes,
                                                       int n_layers, int num_pages, int n_kv, int n_chunk_pages) {
    const int n = layer_bytes / 16;                            // words of one unit
    const long long words = (long long)n_chunk_pages * n_layers * n;
    for (long long w0 = (long long)blockIdx.x * 2048 + threadIdx.x; w0 < words; w0 += (long long)gridDim.x * 2048) {
        uint4 v[8];
        uint4* dst[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const long long w = w0 + u * 256;
            dst[u] = nullptr;
            if (w < words) {
                const int unit = (int)(w / n), off = (int)(w - (long long)unit * n);
                const int pi = unit / n_layers, layer = unit - pi * n_layers;
                v[u] = ((const uint4*)(records + (size_t)pi * record_bytes + (size_t)layer * layer_bytes))[off];
                dst[u] = (uint4*)(pool + ((size_t)layer * num_pages + page_ids.ids[pi]) * layer_bytes) + off;
            }
        }
#pragma unroll
        for (int u = 0; u < 8; ++u)
            if (dst[u]) *dst[u] = v[u];
    }
    if (scales) {
        const int per_page = n_layers * n_kv * 2;
        for (int s = blockIdx.x * 256 + threadIdx.x; s < n_chunk_pages * per_page; s += gridDim.x * 256) {
            const int pi = s / per_page, r = s - pi * per_page, layer = r / (n_kv * 2), j = r - layer * (n_kv * 2);
            scales[((size_t)layer * num_pages + page_ids.ids[pi]) * n_kv * 2 + j] =
                ((const float*)(records + (size_t)pi * record_bytes + (size_t)n_layers * layer_bytes))[r];
        }
    }
}
}  // namespace

hipError_t launch_pages_move(const PoolLayout& lay, char* pool_base, const int32_t* page_ids_host, int64_t n_pages, char* records,
                             bool to_pool, hipStream_t st) {
    float* scales = lay.kv_dtype == HR_FP8_E4M3 ? (float*)(pool_base + lay.data_bytes) : nullptr;
    const size_t rec = page_record_bytes(lay);
    const int layer_bytes = (int)((size_t)lay.n_kv * 2 * lay.block_elems * lay.esz);
    for (int64_t pg0 = 0; pg0 < n_pages; pg0 += 256) {
        const int n = (int)(n_pages - pg0 < 256 ? n_pages - pg0 : 256);
        PageIdChunk ids;
        for (int i = 0; i < 256; ++i) ids.ids[i] = i < n ? page_ids_host[pg0 + i] : 0;
        char* r = records + (size_t)pg0 * rec;
        if (to_pool) {
            const long long passes = ((long long)n * lay.n_layers * (layer_bytes / 16) + 2047) / 2048;
            const unsigned grid = (unsigned)(passes < kPageInWalkers ? passes : kPageInWalkers);
            pages_in_kernel<<<grid, 256, 0, st>>>(pool_base, scales, ids, r, rec, layer_bytes, lay.n_layers, lay.num_pages, lay.n_kv, n);
        } else {
            pages_out_kernel<<<dim3((unsigned)n, (unsigned)lay.n_layers), 256, 0, st>>>(pool_base, scales, ids, r, rec, layer_bytes,
                                                                                        lay.n_layers, lay.num_pages, lay.n_kv);
        }
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

// ---- host tier, 4-bit records of a 16-bit pool.  A unit is a (page, layer, kv head); one thread per group of 32
// channels of one token of K or V: 2 * 16 * d / 32 = d threads.  Out of the pool one workgroup per unit, into the pool
// kPageIn4Walkers workgroups that walk the units (see above).  Out: gather the group from the page (K: four 16-byte
// chunks of the token's row, V: 32 keys-major elements), scale = amax / 7, codes by round-to-nearest-even of the exact
// quotient.  In: codes * scale, rounded to half, back to the page positions.
namespace {
__device__ __forceinline__ size_t kv4_group_elem(bool is_v, int t, int c, int d) {
    return is_v ? (size_t)kPageTokens * d + v_elem(t, c, d) : (size_t)k_elem(t, c, d, 2);
}

template <bool TO_POOL>
__global__ void pages_move4_kernel(half_t* __restrict__ pool, PageIdChunk page_ids, char* __restrict__ records, size_t record_bytes,
                                   int num_pages, int n_kv, int d, int units_per_page, int n_units) {
    // The page (4 or 8 KiB) passes through LDS so that the pool side is read and written in whole 16-byte words; the
    // groups' element order (strided in the V block) is an LDS access pattern only.  A workgroup walks the units
    // (page, layer, kv head) in record order with the grid's stride; on the way in, the next unit's codes and scale are
    // requested before the current one is expanded, so that every workgroup keeps a read on the bus.
    __shared__ __attribute__((aligned(16))) half_t page_lds[2 * kPageTokens * 128];
    const int gpt = d / 32;                                   // groups per token
    const int tid = threadIdx.x;                              // 0 .. d - 1
    const bool is_v = tid >= kPageTokens * gpt;
    const int r = is_v ? tid - kPageTokens * gpt : tid;
    const int t = r / gpt, gi = r - t * gpt;
    uint4* lds16 = (uint4*)page_lds;
    constexpr int WPT = 2 * kPageTokens * 2 / 16;             // 16-byte words of the page per thread: 4 (page = 64 d bytes)
    const size_t code_off = (size_t)(is_v ? kPageTokens * d / 2 : 0) + t * (d / 2) + gi * 16;
    const size_t scale_off = (size_t)kPageTokens * d + 4 * ((is_v ? kPageTokens * gpt : 0) + t * gpt + gi);
    auto unit_rec = [&](int u) { return records + (size_t)(u / units_per_page) * record_bytes + (size_t)(u % units_per_page) * (20 * d); };
    auto unit_page = [&](int u) {
        const int y = u % units_per_page, layer = y / n_kv, h = y - layer * n_kv;
        return (uint4*)(pool + (((size_t)layer * num_pages + page_ids.ids[u / units_per_page]) * n_kv + h) * (2 * kPageTokens * d));
    };
    int u = blockIdx.x;
    if (u >= n_units) return;
    uint4 cw = make_uint4(0u, 0u, 0u, 0u);
    float sc = 0.f;
    if constexpr (TO_POOL) {
        cw = *(const uint4*)(unit_rec(u) + code_off);
        sc = *(const float*)(unit_rec(u) + scale_off);
    }
    for (; u < n_units; u += gridDim.x) {
        uint4* pg = unit_page(u);
        if constexpr (!TO_POOL) {
            char* rec = unit_rec(u);
#pragma unroll
            for (int i = 0; i < WPT; ++i) lds16[i * d + tid] = pg[i * d + tid];
            __syncthreads();
            float x[32];
            float amax = 0.f;
#pragma unroll
            for (int i = 0; i < 32; ++i) {
                x[i] = (float)page_lds[kv4_group_elem(is_v, t, gi * 32 + i, d)];
                amax = fmaxf(amax, fabsf(x[i]));
            }
            const float s1 = amax > 0.f ? amax / 7.0f : 1.0f;
            uint32_t w[4] = {0u, 0u, 0u, 0u};
#pragma unroll
            for (int i = 0; i < 32; ++i) {
                double q = rint((double)x[i] / (double)s1);   // the default rounding mode: ties to even
                q = q < -7.0 ? -7.0 : (q > 7.0 ? 7.0 : q);
                w[i >> 3] |= ((uint32_t)(int)q & 0xFu) << ((i & 7) * 4);
            }
            *(uint4*)(rec + code_off) = make_uint4(w[0], w[1], w[2], w[3]);
            *(float*)(rec + scale_off) = s1;
            __syncthreads();                                  // the page in LDS is read out before the next one lands
        } else {
            const uint4 cur = cw;
            const float cur_sc = sc;
            const int un = u + (int)gridDim.x;
            if (un < n_units) {
                cw = *(const uint4*)(unit_rec(un) + code_off);
                sc = *(const float*)(unit_rec(un) + scale_off);
            }
            const uint32_t w[4] = {cur.x, cur.y, cur.z, cur.w};
#pragma unroll
            for (int i = 0; i < 32; ++i) {
                const int code = ((int)(w[i >> 3] << (28 - (i & 7) * 4))) >> 28;      // sign-extended nibble
                page_lds[kv4_group_elem(is_v, t, gi * 32 + i, d)] = from_float<half_t>((float)code * cur_sc);
            }
            __syncthreads();
#pragma unroll
            for (int i = 0; i < WPT; ++i) pg[i * d + tid] = lds16[i * d + tid];
            __syncthreads();
        }
    }
}
}  // namespace

hipError_t launch_pages_move4(const PoolLayout& lay, char* pool_base, const int32_t* page_ids_host, int64_t n_pages, char* records,
                              bool to_pool, hipStream_t st) {
    const size_t rec = page_record4_bytes(lay);
    if (rec == 0) return hipErrorInvalidValue;
    for (int64_t pg0 = 0; pg0 < n_pages; pg0 += 256) {
        const int n = (int)(n_pages - pg0 < 256 ? n_pages - pg0 : 256);
        PageIdChunk ids;
        for (int i = 0; i < 256; ++i) ids.ids[i] = i < n ? page_ids_host[pg0 + i] : 0;
        const int upp = lay.n_layers * lay.n_kv, units = n * upp;
        const unsigned grid = (unsigned)(to_pool && kPageIn4Walkers < units ? kPageIn4Walkers : units);
        char* r = records + (size_t)pg0 * rec;
        if (to_pool) pages_move4_kernel<true><<<grid, lay.d, 0, st>>>((half_t*)pool_base, ids, r, rec, lay.num_pages, lay.n_kv, lay.d, upp, units);
        else pages_move4_kernel<false><<<grid, lay.d, 0, st>>>((half_t*)pool_base, ids, r, rec, lay.num_pages, lay.n_kv, lay.d, upp, units);
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

// ---- dst[i][:] = src[rows[i]][:]: the rows of the last query tokens, for the last layer's shortened tail
namespace {
__global__ void __launch_bounds__(256) gather_rows_f32_kernel(const float* __restrict__ src, const int32_t* __restrict__ rows,
                                                              float* __restrict__ dst, int cols) {
    const float4* s = (const float4*)(src + (size_t)rows[blockIdx.x] * cols);
    float4* d = (float4*)(dst + (size_t)blockIdx.x * cols);
    for (int c = threadIdx.x; c < cols / 4; c += 256) d[c] = s[c];
}
}  // namespace

hipError_t launch_gather_rows_f32(const float* src, const int32_t* rows, float* dst, int n, int cols, hipStream_t st) {
    if (n == 0) return hipSuccess;
    if (cols % 4 != 0) return hipErrorInvalidValue;
    gather_rows_f32_kernel<<<dim3((unsigned)n), 256, 0, st>>>(src, rows, dst, cols);
    return hipGetLastError();
}

// ---- per-query top-k.  One workgroup per query; the candidates' keys sit in LDS and every candidate counts the
// candidates that beat it (higher score, or equal score and lower index), which is its rank: O(n^2) compares for
// n <= 4096 candidates, no sorting network, and the order is total, so the result does not depend on scheduling.
namespace {
constexpr int kTopkThreads = 256;
constexpr int kTopkMaxCands = 4096;

__global__ void __launch_bounds__(kTopkThreads) segment_topk_kernel(const float* __restrict__ scores, const int32_t* __restrict__ seg,
                                                                     int max_cands, int k, int32_t* __restrict__ idx,
                                                                     float* __restrict__ out_scores) {
    __shared__ float key[kTopkMaxCands];
    const int q = blockIdx.x;
    const int begin = seg[q];
    int n = seg[q + 1] - begin;
    n = n < 0 ? 0 : (n > max_cands ? max_cands : n);
    for (int i = threadIdx.x; i < k; i += kTopkThreads) {
        idx[(size_t)q * k + i] = -1;
        if (out_scores) out_scores[(size_t)q * k + i] = 0.f;
    }
    for (int i = threadIdx.x; i < n; i += kTopkThreads) {
        const float s = scores[begin + i];
        key[i] = s != s ? -INFINITY : s;            // NaN ranks below every number (ties with -inf go by index)
    }
    __syncthreads();                                // also orders the -1 fill before the winners' stores below
    for (int i = threadIdx.x; i < n; i += kTopkThreads) {
        const float si = key[i];
        int rank = 0;
        for (int j = 0; j < n; ++j) {
            const float sj = key[j];
            rank += (sj > si || (sj == si && j < i)) ? 1 : 0;
        }
        if (rank < k) {
            idx[(size_t)q * k + rank] = i;
            if (out_scores) out_scores[(size_t)q * k + rank] = scores[begin + i];
        }
    }
}
}  // namespace

hipError_t launch_segment_topk(const float* scores, const int32_t* seg, int n_seg, int max_cands, int k, int32_t* idx, float* out_scores,
                               hipStream_t st) {
    if (n_seg == 0) return hipSuccess;
    if (max_cands < 1 || max_cands > kTopkMaxCands || k < 1 || k > max_cands) return hipErrorInvalidValue;
    segment_topk_kernel<<<dim3((unsigned)n_seg), kTopkThreads, 0, st>>>(scores, seg, max_cands, k, idx, out_scores);
    return hipGetLastError();
}

}  // namespace hr
