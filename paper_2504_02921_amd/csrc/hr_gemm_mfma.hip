// 16-bit MFMA GEMM family for the projections of the scoring pass (gfx950).  Operands are half
// (the caller's bf16 weights are converted once when they are packed; activations are produced as half):
//   C[M][N] = A[M][K] * W[N][K]^T with fp32 accumulation and a fused epilogue
//     EPI_QKV_ROPE  : split into q / k / v, rotate-half RoPE on q and k, store bf16
//     EPI_RESID_ADD : x[M][N] += C   (fp32 residual stream)
//     EPI_SWIGLU    : gate/up rows interleaved in blocks of 32 -> m = silu(g) * u, store bf16
// Both operands are K-contiguous, which is exactly the MFMA operand order (a lane holds 8
// consecutive k of one row / column), so tiles go global -> LDS -> registers without transposes.
//
// Tiling: 256 x BN x 64 macro tile per 256-thread workgroup (4 wavefronts as 2 x 2, each wave
// 128 x BN/2 = 4 x (BN/64) blocks of v_mfma_f32_32x32x16_f16), LDS double-buffered, rows of 64
// k (128 B) with the 16-byte chunk index XOR-swizzled by (row & 7) so that both the ds_write_b128
// of the loader and the ds_read_b128 of the fragment reads are bank-conflict free.
// Workgroup ids are remapped so that each XCD (ids are dealt round-robin over 8 XCDs) works on a
// contiguous run of tiles, grouped 8 tiles tall, keeping its private L2 on few A/W panels.
#include <hip/hip_runtime.h>

#include "hr_device_types.h"
#include "hr_kernels.h"

namespace hr {

typedef __attribute__((ext_vector_type(8))) _Float16 halfx8;
typedef __attribute__((ext_vector_type(16))) float floatx16;

namespace {

constexpr int BM = 256, BK = 64;
constexpr int kXcds = 8, kGroupM = 8;

struct TileCoord { int tm, tn; bool valid; };

__device__ __forceinline__ TileCoord map_tile(int pid, int tiles_m, int tiles_n) {
    int n_tiles = tiles_m * tiles_n;
    int per_xcd = (n_tiles + kXcds - 1) / kXcds;
    int tile = (pid % kXcds) * per_xcd + pid / kXcds;
    TileCoord c;
    c.valid = tile < n_tiles && pid / kXcds < per_xcd;
    int width = kGroupM * tiles_n;
    int group = tile / width;
    int first_m = group * kGroupM;
    int gsz = min(tiles_m - first_m, kGroupM);
    int in = tile - group * width;
    c.tm = first_m + in % gsz;
    c.tn = in / gsz;
    return c;
}

template <int EPI, int BN, int HB>
__global__ void __launch_bounds__(256) gemm_mfma_kernel(GemmArgs a) {
    constexpr int WNB = BN / 64;             // 32-wide column blocks per wave
    constexpr int WN = BN / 2;               // wave tile width
    constexpr int PA = BM / 32, PB = BN / 32;  // loader passes (32 rows per pass)
    extern __shared__ __attribute__((aligned(16))) char smem[];
    half_t* sA = (half_t*)smem;                         // [2][BM][BK]
    half_t* sB = sA + 2 * BM * BK;                      // [2][BN][BK]

    const int tiles_m = (int)((a.M + BM - 1) / BM), tiles_n = (a.N + BN - 1) / BN;
    TileCoord tc = map_tile(blockIdx.x, tiles_m, tiles_n);
    if (!tc.valid) return;
    const int64_t m0 = (int64_t)tc.tm * BM;
    const int n0 = tc.tn * BN;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int K = a.K;
    const half_t* A = (const half_t*)a.A;
    const half_t* W = (const half_t*)a.W;

    // loader: thread -> (row within a 32-row pass, 16-byte chunk of the 128-byte k row)
    const int lrow = tid >> 3, lchunk = tid & 7;
    const half_t* pa[PA];
    const half_t* pb[PB];
#pragma unroll
    for (int p = 0; p < PA; ++p) {
        int64_t r = m0 + p * 32 + lrow;
        r = r < a.M ? r : a.M - 1;
        pa[p] = A + r * K + lchunk * 8;
    }
#pragma unroll
    for (int p = 0; p < PB; ++p) {
        int r = n0 + p * 32 + lrow;
        r = r < a.N ? r : a.N - 1;
        pb[p] = W + (size_t)r * K + lchunk * 8;
    }
    const int lds_off = lrow * BK + ((lchunk ^ (lrow & 7)) * 8);   // (p*32 + lrow) & 7 == lrow & 7

    halfx8 ga[PA], gb[PB];
    auto gload = [&](int kt) {
#pragma unroll
        for (int p = 0; p < PA; ++p) ga[p] = *(const halfx8*)(pa[p] + kt * BK);
#pragma unroll
        for (int p = 0; p < PB; ++p) gb[p] = *(const halfx8*)(pb[p] + kt * BK);
    };
    auto lstore = [&](int buf) {
        half_t* da = sA + buf * BM * BK + lds_off;
        half_t* db = sB + buf * BN * BK + lds_off;
#pragma unroll
        for (int p = 0; p < PA; ++p) *(halfx8*)(da + p * 32 * BK) = ga[p];
#pragma unroll
        for (int p = 0; p < PB; ++p) *(halfx8*)(db + p * 32 * BK) = gb[p];
    };

    floatx16 acc[4][WNB];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < WNB; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    const int frow = lane & 31, fh = lane >> 5;
    const int a_row0 = wm * 128 + frow;
    const int b_row0 = wn * WN + frow;
    const int sw = frow & 7;                  // (row0 + 32 * i) & 7 == frow & 7

    const int nk = K / BK;
    gload(0);
    lstore(0);
    __syncthreads();
    for (int kt = 0; kt < nk; ++kt) {
        const int cur = kt & 1;
        if (kt + 1 < nk) gload(kt + 1);
        const half_t* cA = sA + cur * BM * BK;
        const half_t* cB = sB + cur * BN * BK;
#pragma unroll
        for (int kk = 0; kk < BK / 16; ++kk) {
            const int pch = ((kk * 2 + fh) ^ sw) * 8;
            halfx8 af[4], bfr[WNB];
#pragma unroll
            for (int i = 0; i < 4; ++i) af[i] = *(const halfx8*)(cA + (a_row0 + i * 32) * BK + pch);
#pragma unroll
            for (int j = 0; j < WNB; ++j) bfr[j] = *(const halfx8*)(cB + (b_row0 + j * 32) * BK + pch);
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < WNB; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(af[i], bfr[j], acc[i][j], 0, 0, 0);
        }
        if (kt + 1 < nk) lstore(cur ^ 1);
        __syncthreads();
    }

    // ---- epilogue: lane holds column (lane & 31) of each 32x32 block, rows 8*(r/4) + 4*(lane>>5) + r%4
    const int64_t row_base = m0 + wm * 128 + 4 * fh;
    const int col_base = n0 + wn * WN + frow;
    if constexpr (EPI == EPI_RESID_ADD) {
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < WNB; ++j) {
                const int col = col_base + j * 32;
                if (col >= a.N) continue;
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int64_t row = row_base + i * 32 + 8 * (r >> 2) + (r & 3);
                    if (row < a.M) {
                        float* px = a.x + row * a.N + col;
                        *px += acc[i][j][r];
                    }
                }
            }
    } else if constexpr (EPI == EPI_SWIGLU) {
        half_t* out = (half_t*)a.out0;
        const int F = a.N / 2;
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < WNB; j += 2) {
                const int col = (n0 + wn * WN) / 2 + (j / 2) * 32 + frow;
                if (col >= F) continue;
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int64_t row = row_base + i * 32 + 8 * (r >> 2) + (r & 3);
                    if (row < a.M) {
                        float g = acc[i][j][r], u = acc[i][j + 1][r];
                        out[row * F + col] = from_float<half_t>(g / (1.0f + __expf(-g)) * u);
                    }
                }
            }
    } else {   // EPI_QKV_ROPE
        constexpr int hb = HB;                                  // 32-wide blocks per half head
        const int d = a.d, half = d / 2;
        const int nq = a.n_q * d, nkv = a.n_kv * d;
        half_t* q = (half_t*)a.out0;
        half_t* k = (half_t*)a.out1;
        half_t* v = (half_t*)a.out2;
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < WNB; ++j) {
                const int col = col_base + j * 32;
                if (col >= a.N) continue;
                const int blk = j % (2 * hb);                 // block index inside its head
                const bool lo = blk < hb;
                const int jj = (lo ? blk : blk - hb) * 32 + frow;   // rotary index
                const int jp = lo ? j + hb : j - hb;           // partner block (same lane, same register)
                half_t* dst;
                int ld;
                bool rot = true;
                if (col < nq) { dst = q + col; ld = nq; }
                else if (col < nq + nkv) { dst = k + (col - nq); ld = nkv; }
                else { dst = v + (col - nq - nkv); ld = nkv; rot = false; }
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int64_t row = row_base + i * 32 + 8 * (r >> 2) + (r & 3);
                    if (row >= a.M) continue;
                    float val = acc[i][j][r];
                    if (rot) {
                        const float2 cs = a.rope[row * half + jj];
                        const float other = acc[i][jp][r];
                        val = lo ? val * cs.x - other * cs.y : val * cs.x + other * cs.y;
                    }
                    dst[row * ld] = from_float<half_t>(val);
                }
            }
    }
}

template <int EPI, int BN, int HB>
hipError_t launch_tile(const GemmArgs& a, hipStream_t st) {
    const int tiles_m = (int)((a.M + BM - 1) / BM), tiles_n = (a.N + BN - 1) / BN;
    const int n_tiles = tiles_m * tiles_n;
    const int per_xcd = (n_tiles + kXcds - 1) / kXcds;
    const size_t lds = (size_t)2 * (BM + BN) * BK * sizeof(half_t);
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute((const void*)gemm_mfma_kernel<EPI, BN, HB>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    gemm_mfma_kernel<EPI, BN, HB><<<dim3((unsigned)(per_xcd * kXcds)), 256, lds, st>>>(a);
    return hipGetLastError();
}

}  // namespace

bool gemm_mfma_supported(const hr_model_cfg& c) {
    if (c.dtype != HR_BF16) return false;
    if (c.head_dim != 64 && c.head_dim != 128) return false;
    const int nq = c.n_q_heads * c.head_dim;
    if (c.hidden % BK != 0 || c.ffn % BK != 0 || nq % BK != 0) return false;   // every K is a multiple of 64
    if (c.ffn % 32 != 0) return false;                                         // gate/up interleave of 32
    return true;
}

hipError_t launch_gemm_mfma(GemmEpilogue epi, const GemmArgs& a, hipStream_t st) {
    if (a.M == 0) return hipSuccess;
    if (a.K % BK != 0) return hipErrorInvalidValue;
    switch (epi) {
        case EPI_QKV_ROPE:
            return a.d == 64 ? launch_tile<EPI_QKV_ROPE, 256, 1>(a, st) : launch_tile<EPI_QKV_ROPE, 256, 2>(a, st);
        case EPI_RESID_ADD: return launch_tile<EPI_RESID_ADD, 256, 1>(a, st);
        case EPI_SWIGLU: return launch_tile<EPI_SWIGLU, 256, 1>(a, st);
    }
    return hipErrorInvalidValue;
}

}  // namespace hr
