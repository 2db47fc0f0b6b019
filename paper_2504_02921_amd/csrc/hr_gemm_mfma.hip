// 16-bit MFMA GEMM family for the projections of the scoring pass (gfx950).  Operands are half
// (the caller's bf16 weights are converted once when they are packed; activations are produced as half):
//   C[M][N] = A[M][K] * W[N][K]^T with fp32 accumulation and a fused epilogue
//     EPI_QKV_ROPE  : split into q / k / v, rotate-half RoPE on q and k, store half (K and V as pool-format pages)
//     EPI_RESID_ADD : x[M][N] += C   (fp32 residual stream)
//     EPI_SWIGLU    : gate/up rows interleaved in blocks of 32 -> m = silu(g) * u, store half
// Both operands are K-contiguous, which is exactly the MFMA operand order (a lane holds 8
// consecutive k of one row / column), so tiles go global -> LDS -> registers without transposes.
//
// Tiling: BM x BN x 64 macro tiles of 32 x 32 blocks of v_mfma_f32_32x32x16_f16: 256 x 256 with 8 wavefronts
// (one workgroup per CU), 320 x 256 with 8 for residual-add and long-K gate/up launches where it saves rounds of the chip,
// 128 x 128 with 4 (two per CU), wider-than-tall shapes for 128-wide heads, and ring variants with 3-5 LDS stages for
// launches of few rows; the launcher picks per call.  LDS rows are 64 k
// (128 B) with the 16-byte chunk index XOR-swizzled by the row pair ((row >> 1) & 7): LDS serves
// 256 bytes per cycle to 16 lanes of a ds_read_b128, i.e. two 128-byte rows side by side, so 16
// consecutive rows must use 8 different chunk positions per row parity (measured: 217 B/clk/CU with
// this pattern against 119 with a (row & 7) swizzle and 32 unswizzled).
// Workgroup ids are remapped so that each XCD (ids are dealt round-robin over 8 XCDs) works on a
// contiguous run of tiles, grouped 8 tiles tall, keeping its private L2 on few A/W panels (groups 4 or 16 tall
// measured the same).
#include <hip/hip_runtime.h>

#include <atomic>
#include <cstdlib>
#include <type_traits>

#include "hr_device_types.h"
#include "hr_internal.h"
#include "hr_kernels.h"
#include "hr_layout.h"

namespace hr {

typedef __attribute__((ext_vector_type(8))) _Float16 halfx8;
typedef __attribute__((ext_vector_type(4))) _Float16 halfx4;
typedef __attribute__((ext_vector_type(16))) float floatx16;
typedef __attribute__((ext_vector_type(4))) unsigned uint4v;

namespace {

constexpr int BK = 64;
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

typedef __attribute__((address_space(3))) void* lds_ptr_t;
typedef const __attribute__((address_space(1))) void* gbl_ptr_t;

// Epilogues on transposed accumulators: a lane owns output row (lane & 31) of each 32 x 32 block, register r holds
// column 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3).  `smem` is the kernel's LDS (two stages of A, then two of W), free
// behind the main loop's last barrier except that, in a persistent launch, stage 0 may be receiving the next tile.
template <int EPI, int BM, int BN, int WM, int WN, int HB>
__device__ __forceinline__ void gemm_epilogue(floatx16 (&acc)[BM / WM / 32][BN / WN / 32], const GemmArgs& a, char* smem,
                                              int64_t tile_m0, int tile_n0) {
    constexpr int NT = WM * WN * 64;
    constexpr int TM = BM / WM, TN = BN / WN;
    constexpr int MI = TM / 32, NI = TN / 32;
    half_t* sA = (half_t*)smem;
    half_t* sB = sA + 2 * BM * BK;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / WN, wn = wave % WN;
    const int frow = lane & 31, fh = lane >> 5;
    const int64_t row_base = tile_m0 + wm * TM + frow;
    const int col_base = tile_n0 + wn * TN + 4 * fh;
    (void)sA; (void)sB; (void)row_base; (void)col_base; (void)NT; (void)MI; (void)NI;
    if constexpr (EPI == EPI_RESID_ADD) {
        // x += C through LDS.  In the accumulator layout a lane holds 16 bytes of one row, so a direct update touches
        // 32 rows per instruction; staged as an fp32 [BM][CW] tile (16-byte chunks XOR-swizzled by the row against
        // bank conflicts of the column-wise writes) the update reads and writes whole 512-byte row segments.  The
        // stages hold BM x CW floats, so the tile goes in PASSES column slabs; each wave tile lies in one slab.
        constexpr int LDS_BYTES = 2 * (BM + BN) * BK * (int)sizeof(half_t);
        constexpr int PASSES_MIN = (BM * BN * 4 + LDS_BYTES - 1) / LDS_BYTES;
        constexpr int PASSES = PASSES_MIN <= 2 ? PASSES_MIN : (PASSES_MIN <= 4 ? 4 : 8);     // a divisor of BN
        constexpr int CW = BN / PASSES;                 // slab width in columns
        constexpr int CPRW = CW / 4;                    // 16-byte chunks per slab row
        constexpr int ITER = BM * CPRW / NT;
        constexpr int NG = ITER % 4 == 0 ? 4 : 5;       // register groups of the x update (320-row tiles: 10 = 5 x 2)
        static_assert(EPI != EPI_RESID_ADD || (CW % TN == 0 && CPRW % 16 == 0 && (BM * CPRW) % (NG * NT) == 0 && BM * CW * 4 <= LDS_BYTES),
                      "slab shape");
        float* stage = (float*)smem;
#pragma unroll
        for (int p = 0; p < PASSES; ++p) {
            // x in NG groups of G chunks per lane (registers): the first is requested before the stage is written, so
            // its latency hides behind the write and the barrier.  Every address is clamped into the matrix, only
            // valid chunks are written back.
            constexpr int G = ITER / NG;
            float4 xv[G];
            auto load_x = [&](int first) {
#pragma unroll
                for (int it = 0; it < G; ++it) {
                    const int L = (first + it) * NT + tid;
                    const int row = L / CPRW, pch = L % CPRW;
                    int col = tile_n0 + p * CW + ((pch ^ (row & 15)) << 2);
                    int64_t grow = tile_m0 + row;
                    grow = grow < a.M ? grow : a.M - 1;
                    col = col < a.N ? col : a.N - 4;
                    xv[it] = *(const float4*)(a.x + grow * a.N + col);
                }
            };
            auto update_x = [&](int first) {
#pragma unroll
                for (int it = 0; it < G; ++it) {
                    const int L = (first + it) * NT + tid;
                    const int row = L / CPRW, pch = L % CPRW;
                    const int col = tile_n0 + p * CW + ((pch ^ (row & 15)) << 2);
                    const int64_t grow = tile_m0 + row;
                    if (grow >= a.M || col >= a.N) continue;        // N is a multiple of 8: whole chunks
                    const float4 c = *(const float4*)(stage + row * CW + (pch << 2));
                    float4 v = xv[it];
                    v.x += c.x;
                    v.y += c.y;
                    v.z += c.z;
                    v.w += c.w;
                    *(float4*)(a.x + grow * a.N + col) = v;
                }
            };
            load_x(0);
            if (p > 0) __syncthreads();                 // the previous slab has been read
            if ((wn * TN) / CW == p) {
                const int c_off = wn * TN - p * CW + 4 * fh;
#pragma unroll
                for (int i = 0; i < MI; ++i) {
                    const int lr = wm * TM + i * 32 + frow;
#pragma unroll
                    for (int j = 0; j < NI; ++j)
#pragma unroll
                        for (int r4 = 0; r4 < 4; ++r4) {
                            const int ch = (c_off + j * 32 + 8 * r4) >> 2;
                            float4 v;
                            v.x = acc[i][j][r4 * 4 + 0];
                            v.y = acc[i][j][r4 * 4 + 1];
                            v.z = acc[i][j][r4 * 4 + 2];
                            v.w = acc[i][j][r4 * 4 + 3];
                            *(float4*)(stage + lr * CW + ((ch ^ (lr & 15)) << 2)) = v;
                        }
                }
            }
            __syncthreads();
            update_x(0);
#pragma unroll
            for (int g = 1; g < NG; ++g) {
                load_x(g * G);
                update_x(g * G);
            }
        }
    } else if constexpr (EPI == EPI_SWIGLU) {
        static_assert(EPI != EPI_SWIGLU || NI % 2 == 0, "gate/up block pairs");
        // m = silu(g) * u goes through LDS as a half [BM][BN / 2] tile (16-byte chunks XOR-swizzled by the row) and
        // leaves in whole row segments, like the residual update above.
        constexpr int OW = BN / 2;                      // output columns of the tile
        constexpr int CPRO = OW / 8;                    // 16-byte chunks per tile row: 16 (256-byte rows) or 8 (128-byte rows)
        constexpr int ITER = BM * CPRO / NT;
        static_assert(EPI != EPI_SWIGLU || ((CPRO == 16 || CPRO == 8) && (BM * CPRO) % NT == 0), "output tile shape");
        auto swz = [](int r) { return CPRO == 16 ? (r & 15) : ((r >> 1) & 7); };
        // staged in the second stages of A and W: the first ones may already be receiving the next tile.  The tall tile's
        // output does not fit there; its launch is not persistent and stages from the start of the LDS.
        constexpr bool WHOLE = BM > 256;
        constexpr int R1 = BM * BK / OW;                 // tile rows that fit the A stage
        static_assert(EPI != EPI_SWIGLU || (WHOLE ? BM * OW <= 2 * (BM + BN) * BK : (R1 <= BM && (BM - R1) * OW <= BN * BK)),
                      "staging fits the stages");
        auto stage_row = [&](int r) {
            if constexpr (WHOLE) return (half_t*)smem + r * OW;
            else return r < R1 ? sA + BM * BK + r * OW : sB + BN * BK + (r - R1) * OW;
        };
        half_t* out = (half_t*)a.out0;
        const int F = a.N / 2;
        // split output (the layers that run with 22-bit operands): m = hi + lo is written as [M][hi F | lo F], one half
        // after the other through the same stage
        const int parts = a.split_out ? 2 : 1;
        const int ldo = parts * F;
        for (int part = 0; part < parts; ++part) {
            if (part) asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");     // the hi tile has been read out of the stage
#pragma unroll
            for (int i = 0; i < MI; ++i) {
                const int lr = wm * TM + i * 32 + frow;
#pragma unroll
                for (int j = 0; j < NI; j += 2)
#pragma unroll
                    for (int r4 = 0; r4 < 4; ++r4) {
                        const int ch = ((wn * TN) / 2 + (j / 2) * 32) / 8 + r4;
                        halfx4 w;
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            const float g = acc[i][j][r4 * 4 + e], u = acc[i][j + 1][r4 * 4 + e];
                            const float sg = __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(-1.4426950408889634f * g));
                            const float v = g * sg * u;
                            const half_t hi = from_float<half_t>(v);
                            w[e] = part ? from_float<half_t>(v - (float)hi) : hi;
                        }
                        *(halfx4*)(stage_row(lr) + ((ch ^ swz(lr)) << 3) + 4 * fh) = w;
                    }
            }
            // LDS-only barrier: __syncthreads() would also wait for the next tile's loads, which were just requested
            asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
#pragma unroll
            for (int it = 0; it < ITER; ++it) {
                const int L = it * NT + tid;
                const int row = L / CPRO, pch = L % CPRO;
                const int col = tile_n0 / 2 + ((pch ^ swz(row)) << 3);
                const int64_t grow = tile_m0 + row;
                if (grow >= a.M || col >= F) continue;          // F is a multiple of 32: whole chunks
                *(uint4v*)(out + grow * ldo + part * F + col) = *(const uint4v*)(stage_row(row) + (pch << 3));
            }
        }
    } else {   // EPI_QKV_ROPE
        constexpr int hb = HB;                                  // 32-wide blocks per half head: head_dim = 64 * HB
        static_assert(EPI != EPI_QKV_ROPE || NI % (2 * HB) == 0, "a wave must hold whole heads");
        constexpr int d = 64 * HB, half = d / 2;
        const int nq = a.n_q * d, nkv = a.n_kv * d;
        // The (cos, sin) rows of this tile's tokens go to LDS first (the stages are free: nobody reads them behind
        // the last barrier of the main loop).  A lane owns one token row and would otherwise fetch its 16-byte
        // pieces of the table from 32 different cache lines per load instruction.  Chunks of 16 bytes are
        // XOR-swizzled by the row so that the 16 rows read together hit 16 different bank groups.
        constexpr int CPR = d / 4;                               // chunks per table row (d / 2 pairs of 8 bytes)
        static_assert(EPI != EPI_QKV_ROPE || (BM * CPR) % NT == 0, "table loader shape");
        static_assert(EPI != EPI_QKV_ROPE || BM * CPR * 16 <= 2 * (BM + BN) * BK * (int)sizeof(half_t), "table fits the stages");
        {
            const char* rope_bytes = (const char*)a.rope;
#pragma unroll
            for (int base = 0; base < BM * CPR; base += NT) {
                const int L = base + tid;
                const int row = L / CPR, pc = L % CPR;
                int64_t gr = tile_m0 + row;
                gr = gr < a.M ? gr : a.M - 1;
                const char* g = rope_bytes + (gr * half) * (int64_t)sizeof(float2) + ((pc ^ (row & 15)) << 4);
                __builtin_amdgcn_global_load_lds((gbl_ptr_t)g, (lds_ptr_t)(smem + (size_t)(base + wave * 64) * 16), 16, 0, 0);
            }
        }
        int slot_i[MI];
#pragma unroll
        for (int i = 0; i < MI; ++i) {
            const int64_t row = row_base + i * 32;
            slot_i[i] = (a.kv_pages && row < a.M) ? a.new_slot[row] : 0;
        }
        __builtin_amdgcn_s_waitcnt(0x0F70);
        __syncthreads();
        // q and K quads are kept (rotated and rounded) until the table is no longer needed, then staged in LDS as a
        // half [BM][BN] tile and stored in whole row segments; V quads go straight to their pages: a lane's 32 tokens
        // fall into two pages, where each channel's keys are adjacent, which is as coalesced as V gets.
        halfx4 res[MI][NI][4];
        auto store_v_quad = [&](int i, int64_t row, int col, halfx4 w) {
            const int c_all = col - nq - nkv;
            if (!a.kv_pages) {
                *(halfx4*)((half_t*)a.out2 + row * nkv + c_all) = w;
                return;
            }
            // 16-slot pages in the pool arrangement: [page][kv head][K block | V block]
            const int kv_head = c_all / d, kv_c = c_all - kv_head * d;
            const int slot = slot_i[i];
            half_t* vb = (half_t*)a.kv_pages + ((size_t)(slot >> 4) * a.n_kv + kv_head) * (2 * kPageTokens * d) + kPageTokens * d;
            const int t = slot & 15;
#pragma unroll
            for (int e = 0; e < 4; ++e) vb[v_elem(t, kv_c + e, d)] = w[e];
        };
#pragma unroll
        for (int i = 0; i < MI; ++i) {
            const int64_t row = row_base + i * 32;
            const bool row_ok = row < a.M;
            const int lrow = wm * TM + i * 32 + frow;              // row inside the tile
            const char* trow = smem + (size_t)lrow * (CPR * 16);
#pragma unroll
            for (int hbi = 0; hbi < hb; ++hbi)
#pragma unroll
                for (int r4 = 0; r4 < 4; ++r4) {
                    // rotary indices hbi * 32 + 8 * r4 + 4 * fh + {0..3}: two chunks of two (cos, sin) pairs
                    const int c0 = hbi * 16 + 4 * r4 + 2 * fh;
                    const float4 cs01 = *(const float4*)(trow + ((c0 ^ (lrow & 15)) << 4));
                    const float4 cs23 = *(const float4*)(trow + (((c0 + 1) ^ (lrow & 15)) << 4));
                    const float cs_c[4] = {cs01.x, cs01.z, cs23.x, cs23.z}, cs_s[4] = {cs01.y, cs01.w, cs23.y, cs23.w};
#pragma unroll
                    for (int hd = 0; hd < NI / (2 * hb); ++hd) {
                        const int jl = hd * 2 * hb + hbi, jh = jl + hb;       // low / high half of the head: same lane, same register
                        const int col_l = col_base + jl * 32 + 8 * r4, col_h = col_base + jh * 32 + 8 * r4;
                        const bool rot = col_l < nq + nkv;                      // q and k rotate, v does not
                        halfx4 wl, wh;
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            const float lo = acc[i][jl][r4 * 4 + e], hi = acc[i][jh][r4 * 4 + e];
                            wl[e] = from_float<half_t>(rot ? rope_lo(lo, hi, cs_c[e], cs_s[e]) : lo);
                            wh[e] = from_float<half_t>(rot ? rope_hi(lo, hi, cs_c[e], cs_s[e]) : hi);
                        }
                        res[i][jl][r4] = wl;
                        res[i][jh][r4] = wh;
                        if (!rot && row_ok && col_l < a.N) {                  // N is a multiple of the head size
                            store_v_quad(i, row, col_l, wl);
                            store_v_quad(i, row, col_h, wh);
                        }
                    }
                }
        }
        __syncthreads();                                            // every lane is done with the table
        constexpr int CPT = BN / 8;                                 // 16-byte chunks per tile row (16 or 32)
        static_assert(EPI != EPI_QKV_ROPE || (CPT % 16 == 0 && (BM * CPT) % NT == 0), "output tile shape");
        half_t* stage = (half_t*)smem;
#pragma unroll
        for (int i = 0; i < MI; ++i) {
            const int lr = wm * TM + i * 32 + frow;
#pragma unroll
            for (int j = 0; j < NI; ++j)
#pragma unroll
                for (int r4 = 0; r4 < 4; ++r4) {
                    const int ch = (wn * TN + j * 32) / 8 + r4;
                    *(halfx4*)(stage + lr * BN + ((ch ^ (lr & 15)) << 3) + 4 * fh) = res[i][j][r4];
                }
        }
        __syncthreads();
#pragma unroll
        for (int it = 0; it < BM * CPT / NT; ++it) {
            const int L = it * NT + tid;
            const int row = L / CPT, pch = L % CPT;
            const int col = tile_n0 + ((pch ^ (row & 15)) << 3);
            const int64_t grow = tile_m0 + row;
            if (grow >= a.M || col >= nq + nkv) continue;           // past the matrix, or V (stored above)
            const uint4v w = *(const uint4v*)(stage + row * BN + (pch << 3));
            if (col < nq) {
                *(uint4v*)((half_t*)a.out0 + grow * nq + col) = w;
            } else if (!a.kv_pages) {
                *(uint4v*)((half_t*)a.out1 + grow * nkv + (col - nq)) = w;
            } else {
                const int c_all = col - nq, kv_head = c_all / d, kv_c = c_all - kv_head * d;
                const int slot = a.new_slot[grow];
                half_t* blk0 = (half_t*)a.kv_pages + ((size_t)(slot >> 4) * a.n_kv + kv_head) * (2 * kPageTokens * d);
                *(uint4v*)(blk0 + k_elem(slot & 15, kv_c, d, 2)) = w;   // 8 channels = one swizzled 16-byte chunk
            }
        }
    }
}

// BM x BN x 64 macro tile, WM x WN wavefronts, each wave (BM/WM) x (BN/WN) = MI x NI blocks of 32 x 32.
//
// Data path: global_load_lds_dwordx4 (HBM/L2 -> LDS without passing through VGPRs; lane l of a wave
// writes LDS bytes [base + 16 l, base + 16 l + 16)), two LDS stages.  The loads of k-tile kt + 1 are
// issued at the top of iteration kt and waited for just before the last k-step of the iteration,
// where the only workgroup barrier of the iteration sits; the fragments of the next k-step are read
// one step ahead and the scheduler is pinned to alternate one ds_read with one MFMA.
// Accumulation is transposed (D = W_frag * A_frag^T): a lane owns ONE output row (lane & 31) and
// 4 consecutive columns per register quad, so the epilogues address one row pointer per block and
// store 8 / 16 bytes at a time.
template <int EPI, int BM, int BN, int WM, int WN, int HB>
__global__ void __launch_bounds__(WM * WN * 64) gemm_mfma_kernel(GemmArgs a) {
    constexpr int NT = WM * WN * 64;
    constexpr int TM = BM / WM, TN = BN / WN;      // wave tile
    constexpr int MI = TM / 32, NI = TN / 32;
    constexpr int RPP = NT / 8;                     // rows per loader pass (8 lanes cover one 128-byte k row)
    constexpr int PA = BM / RPP, PB = BN / RPP;
    constexpr int KS = BK / 16;
    static_assert(RPP % 16 == 0 && BM % RPP == 0 && BN % RPP == 0, "loader shape");
    extern __shared__ __attribute__((aligned(16))) char smem[];
    half_t* sA = (half_t*)smem;                         // [2][BM][BK]
    half_t* sB = sA + 2 * BM * BK;                      // [2][BN][BK]

    // The gate/up launch is persistent: a workgroup walks tiles blockIdx.x, blockIdx.x + gridDim.x, ... (the same
    // XCD-chunked order) and requests the first k-tile of its next tile before it starts the epilogue of the current
    // one, so only a workgroup's first tile pays the start-up round trip (3.4k of a 50k-cycle tile at K = 896).  Its
    // epilogue has no loads that would queue behind that request.  The other launches run one tile per workgroup.
    constexpr bool PERSIST = EPI == EPI_SWIGLU && BM <= 256;
    const int tiles_m = (int)((a.M + BM - 1) / BM), tiles_n = (a.N + BN - 1) / BN;
    int vpid = blockIdx.x;
    TileCoord tc = map_tile(vpid, tiles_m, tiles_n);
    if (!tc.valid) return;
    int64_t m0;
    int n0;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / WN, wn = wave % WN;
    const int K = a.K;
    const int Kw = a.Kw > 0 ? a.Kw : K;         // columns of W: K, or K / 2 when A carries [hi | lo] halves of a split operand
    const int nkw = Kw / BK;
    const half_t* A = (const half_t*)a.A;
    const half_t* W = (const half_t*)a.W;

    // loader: lane -> LDS chunk (row lrow of the pass, physical 16-byte chunk tid & 7); it fetches the logical
    // chunk that the row-pair swizzle maps there
    const int lrow = tid >> 3;
    const int lchunk = (tid & 7) ^ ((lrow >> 1) & 7);
    const half_t* pa[PA];
    const half_t* pb[PB];
    auto set_tile = [&](const TileCoord& t) {
        m0 = (int64_t)t.tm * BM;
        n0 = t.tn * BN;
#pragma unroll
        for (int p = 0; p < PA; ++p) {
            int64_t r = m0 + p * RPP + lrow;
            r = r < a.M ? r : a.M - 1;
            pa[p] = A + r * K + lchunk * 8;
        }
#pragma unroll
        for (int p = 0; p < PB; ++p) {
            int r = n0 + p * RPP + lrow;
            r = r < a.N ? r : a.N - 1;
            pb[p] = W + (size_t)r * Kw + lchunk * 8;
        }
    };
    set_tile(tc);
    auto dma = [&](int kt, int buf) {
        half_t* da = sA + buf * BM * BK + wave * 64 * 8;      // wave-uniform: the hardware adds 16 bytes per lane
        half_t* db = sB + buf * BN * BK + wave * 64 * 8;
        const int ktw = kt < nkw ? kt : kt - nkw;             // the lo half of a split A meets the same W columns again
#pragma unroll
        for (int p = 0; p < PA; ++p)
            __builtin_amdgcn_global_load_lds((gbl_ptr_t)(pa[p] + kt * BK), (lds_ptr_t)(da + p * NT * 8), 16, 0, 0);
#pragma unroll
        for (int p = 0; p < PB; ++p)
            __builtin_amdgcn_global_load_lds((gbl_ptr_t)(pb[p] + ktw * BK), (lds_ptr_t)(db + p * NT * 8), 16, 0, 0);
    };

    floatx16 acc[MI][NI];

    const int frow = lane & 31, fh = lane >> 5;
    const int a_row0 = wm * TM + frow;
    const int b_row0 = wn * TN + frow;
    const int sw = (frow >> 1) & 7;           // row pair index: rows are 128 bytes, the bank window 256

    halfx8 af[2][MI], bfr[2][NI];             // fragment double buffer
    auto fload = [&](int slot, const half_t* cA, const half_t* cB, int kk) {
        const int pch = ((kk * 2 + fh) ^ sw) * 8;
#pragma unroll
        for (int i = 0; i < MI; ++i) af[slot][i] = *(const halfx8*)(cA + (a_row0 + i * 32) * BK + pch);
#pragma unroll
        for (int j = 0; j < NI; ++j) bfr[slot][j] = *(const halfx8*)(cB + (b_row0 + j * 32) * BK + pch);
    };
    auto mfmas = [&](int slot) {
#pragma unroll
        for (int i = 0; i < MI; ++i)
#pragma unroll
            for (int j = 0; j < NI; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(bfr[slot][j], af[slot][i], acc[i][j], 0, 0, 0);
    };

    const int nk = K / BK;
    dma(0, 0);
    for (;;) {                                // one tile per pass; a single pass unless PERSIST
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NI; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
    // k-tile 0 has landed; every wave is done with the previous tile's staging reads (PERSIST)
    __builtin_amdgcn_s_waitcnt(0x0F70);       // vmcnt(0)
    __syncthreads();
    fload(0, sA, sB, 0);
    for (int kt = 0; kt < nk; ++kt) {
        const int cur = kt & 1;
        const bool more = kt + 1 < nk;
        if (more) dma(kt + 1, cur ^ 1);
        const half_t* cA = sA + cur * BM * BK;
        const half_t* cB = sB + cur * BN * BK;
#pragma unroll
        for (int kk = 0; kk < KS - 1; ++kk) {
            fload((kk + 1) & 1, cA, cB, kk + 1);
            mfmas(kk & 1);
#pragma unroll
            for (int n = 0; n < MI + NI; ++n) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);   // one MFMA
                __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);   // one LDS read
            }
            __builtin_amdgcn_sched_group_barrier(0x008, MI * NI - (MI + NI), 0);
        }
        // the next k-tile has landed (own loads) and every wave is past its last read of the other stage
        __builtin_amdgcn_s_waitcnt(0x0F70);
        __syncthreads();
        if (more) fload(KS & 1, sA + (cur ^ 1) * BM * BK, sB + (cur ^ 1) * BN * BK, 0);
        mfmas((KS - 1) & 1);
        static_assert(KS % 2 == 0, "slot parity of the first fragment of a tile");
    }

    // ---- epilogue: lane owns output row (lane & 31) of each block; register r holds column 8*(r>>2) + 4*(lane>>5) + (r&3)
    const int64_t tile_m0 = m0;               // the epilogue's tile; m0 / n0 move on to the next one below
    const int tile_n0 = n0;
    bool has_next = false;
    if constexpr (PERSIST) {
        vpid += (int)gridDim.x;
        const TileCoord nx = map_tile(vpid, tiles_m, tiles_n);
        has_next = nx.valid;
        if (has_next) {
            set_tile(nx);
            dma(0, 0);                        // stage 0 of A and W: nobody reads LDS behind the loop's last barrier
        }
    }
    gemm_epilogue<EPI, BM, BN, WM, WN, HB>(acc, a, smem, tile_m0, tile_n0);
    if (!has_next) break;
    }
}

// Small-M variant: the same tile arithmetic with a ring of NS LDS stages.  With fewer tiles than CUs a tile has its
// CU to itself and the two-stage loop above is bound by latency (one load round trip, ~1 us, per k-tile: the down
// projection's 76 k-tiles alone are 77 us for 640 rows); with NS - 1 k-tiles in flight the loop runs at the rate the
// direct-to-LDS path delivers.  Vector memory operations complete in order, so "k-tile kt has landed" is a wait
// until at most the loads of the NS - 2 younger k-tiles are outstanding; the one barrier per k-tile also tells that
// every wave is done with the stage of k-tile kt - 1, which is where k-tile kt + NS - 1 goes.  Same operand order and
// same k order as the kernel above: an output element gets the same bits from either.
template <int EPI, int BM, int BN, int WM, int WN, int HB, int NS>
__global__ void __launch_bounds__(WM * WN * 64) gemm_ring_kernel(GemmArgs a) {
    constexpr int NT = WM * WN * 64;
    constexpr int TM = BM / WM, TN = BN / WN;
    constexpr int MI = TM / 32, NI = TN / 32;
    constexpr int RPP = NT / 8;
    constexpr int PA = BM / RPP, PB = BN / RPP;
    constexpr int KS = BK / 16;
    constexpr int LPT = PA + PB;                    // loads per thread and k-tile
    constexpr int AHEAD = (NS - 2) * LPT;           // loads that may still be outstanding when a k-tile is consumed
    static_assert(RPP % 16 == 0 && BM % RPP == 0 && BN % RPP == 0, "loader shape");
    static_assert(NS >= 3 && AHEAD < 64, "the load counter has six bits");
    constexpr int kWaitAhead = (AHEAD & 15) | ((AHEAD >> 4) << 14) | 0x0F70;     // s_waitcnt vmcnt(AHEAD) only
    extern __shared__ __attribute__((aligned(16))) char smem[];
    half_t* sA = (half_t*)smem;                         // [NS][BM][BK]
    half_t* sB = sA + NS * BM * BK;                     // [NS][BN][BK]

    const int tiles_m = (int)((a.M + BM - 1) / BM), tiles_n = (a.N + BN - 1) / BN;
    const TileCoord tc = map_tile(blockIdx.x, tiles_m, tiles_n);
    if (!tc.valid) return;
    const int64_t m0 = (int64_t)tc.tm * BM;
    const int n0 = tc.tn * BN;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / WN, wn = wave % WN;
    const int K = a.K;
    const int Kw = a.Kw > 0 ? a.Kw : K;
    const int nkw = Kw / BK;
    const half_t* A = (const half_t*)a.A;
    const half_t* W = (const half_t*)a.W;

    const int lrow = tid >> 3;
    const int lchunk = (tid & 7) ^ ((lrow >> 1) & 7);
    const half_t* pa[PA];
    const half_t* pb[PB];
#pragma unroll
    for (int p = 0; p < PA; ++p) {
        int64_t r = m0 + p * RPP + lrow;
        r = r < a.M ? r : a.M - 1;
        pa[p] = A + r * K + lchunk * 8;
    }
#pragma unroll
    for (int p = 0; p < PB; ++p) {
        int r = n0 + p * RPP + lrow;
        r = r < a.N ? r : a.N - 1;
        pb[p] = W + (size_t)r * Kw + lchunk * 8;
    }
    auto dma = [&](int kt, int buf) {
        half_t* da = sA + buf * BM * BK + wave * 64 * 8;
        half_t* db = sB + buf * BN * BK + wave * 64 * 8;
        const int ktw = kt < nkw ? kt : kt - nkw;
#pragma unroll
        for (int p = 0; p < PA; ++p)
            __builtin_amdgcn_global_load_lds((gbl_ptr_t)(pa[p] + kt * BK), (lds_ptr_t)(da + p * NT * 8), 16, 0, 0);
#pragma unroll
        for (int p = 0; p < PB; ++p)
            __builtin_amdgcn_global_load_lds((gbl_ptr_t)(pb[p] + ktw * BK), (lds_ptr_t)(db + p * NT * 8), 16, 0, 0);
    };

    floatx16 acc[MI][NI];
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NI; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
    const int frow = lane & 31, fh = lane >> 5;
    const int a_row0 = wm * TM + frow;
    const int b_row0 = wn * TN + frow;
    const int sw = (frow >> 1) & 7;
    halfx8 af[2][MI], bfr[2][NI];
    auto fload = [&](int slot, const half_t* cA, const half_t* cB, int kk) {
        const int pch = ((kk * 2 + fh) ^ sw) * 8;
#pragma unroll
        for (int i = 0; i < MI; ++i) af[slot][i] = *(const halfx8*)(cA + (a_row0 + i * 32) * BK + pch);
#pragma unroll
        for (int j = 0; j < NI; ++j) bfr[slot][j] = *(const halfx8*)(cB + (b_row0 + j * 32) * BK + pch);
    };
    auto mfmas = [&](int slot) {
#pragma unroll
        for (int i = 0; i < MI; ++i)
#pragma unroll
            for (int j = 0; j < NI; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(bfr[slot][j], af[slot][i], acc[i][j], 0, 0, 0);
    };

    const int nk = K / BK;
#pragma unroll
    for (int s = 0; s < NS - 1; ++s)
        if (s < nk) dma(s, s);
    int cur = 0;                                   // stage of k-tile kt
    for (int kt = 0; kt < nk; ++kt) {
        // own loads of k-tile kt have landed: in the steady state the NS - 2 younger k-tiles may be outstanding; once no
        // new loads are issued everything is simply waited for
        if (kt + NS - 2 < nk) __builtin_amdgcn_s_waitcnt(kWaitAhead);
        else __builtin_amdgcn_s_waitcnt(0x0F70);
        // LDS-only barrier (a __syncthreads() would wait for the loads in flight as well)
        asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
        const int nxt = kt + NS - 1;
        if (nxt < nk) dma(nxt, cur == 0 ? NS - 1 : cur - 1);       // the stage k-tile kt - 1 was read from
        const half_t* cA = sA + cur * BM * BK;
        const half_t* cB = sB + cur * BN * BK;
        fload(0, cA, cB, 0);
#pragma unroll
        for (int kk = 0; kk < KS; ++kk) {
            if (kk + 1 < KS) fload((kk + 1) & 1, cA, cB, kk + 1);
            mfmas(kk & 1);
        }
        cur = cur + 1 == NS ? 0 : cur + 1;
    }
    __syncthreads();                               // every wave is done reading the stages before the epilogue reuses them
    gemm_epilogue<EPI, BM, BN, WM, WN, HB>(acc, a, smem, m0, n0);
}

int cu_count();

// Per-device "done once" flags and cached values: a host thread may drive any device, and different model handles may
// be used from different threads.
constexpr int kMaxDevices = 64;
inline int current_device() {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return 0;
    return dev;
}
// hipFuncSetAttribute(max dynamic LDS) once per kernel instantiation and device
template <typename K>
hipError_t allow_dynamic_lds(K kernel, size_t lds, std::atomic<uint64_t>& done) {
    const uint64_t bit = (uint64_t)1 << current_device();
    if (done.load(std::memory_order_acquire) & bit) return hipSuccess;
    hipError_t e = hipFuncSetAttribute((const void*)kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e == hipSuccess) done.fetch_or(bit, std::memory_order_release);
    return e;
}

template <int EPI, int BM, int BN, int WM, int WN, int HB>
hipError_t launch_tile(const GemmArgs& a, hipStream_t st) {
    const int tiles_m = (int)((a.M + BM - 1) / BM), tiles_n = (a.N + BN - 1) / BN;
    const int n_tiles = tiles_m * tiles_n;
    const int per_xcd = (n_tiles + kXcds - 1) / kXcds;
    int grid = per_xcd * kXcds;
    if (EPI == EPI_SWIGLU && BM <= 256) {
        // persistent launch: as many workgroups as are resident at once (one big or two small tiles per CU), a multiple
        // of the XCD count so that the walk blockIdx.x + k * gridDim.x stays on its XCD
        const int resident = cu_count() * (BM >= 256 ? 1 : 2) / kXcds * kXcds;
        if (resident >= kXcds && grid > resident) grid = resident;
    }
    const size_t lds = (size_t)2 * (BM + BN) * BK * sizeof(half_t);
    static std::atomic<uint64_t> attr_done{0};
    if (hipError_t e = allow_dynamic_lds(gemm_mfma_kernel<EPI, BM, BN, WM, WN, HB>, lds, attr_done); e != hipSuccess) return e;
    gemm_mfma_kernel<EPI, BM, BN, WM, WN, HB><<<dim3((unsigned)grid), WM * WN * 64, lds, st>>>(a);
    return hipGetLastError();
}

template <int EPI, int BM, int BN, int WM, int WN, int HB, int NS>
hipError_t launch_ring(const GemmArgs& a, hipStream_t st) {
    const int tiles_m = (int)((a.M + BM - 1) / BM), tiles_n = (a.N + BN - 1) / BN;
    const int grid = (tiles_m * tiles_n + kXcds - 1) / kXcds * kXcds;
    const size_t lds = (size_t)NS * (BM + BN) * BK * sizeof(half_t);
    static std::atomic<uint64_t> attr_done{0};
    if (hipError_t e = allow_dynamic_lds(gemm_ring_kernel<EPI, BM, BN, WM, WN, HB, NS>, lds, attr_done); e != hipSuccess) return e;
    gemm_ring_kernel<EPI, BM, BN, WM, WN, HB, NS><<<dim3((unsigned)grid), WM * WN * 64, lds, st>>>(a);
    return hipGetLastError();
}

int cu_count() {
    static std::atomic<int> cache[kMaxDevices];
    const int dev = current_device();
    int n = cache[dev].load(std::memory_order_relaxed);
    if (n == 0) {
        if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) n = 256;
        cache[dev].store(n, std::memory_order_relaxed);
    }
    return n;
}

}  // namespace

int device_cu_count() { return cu_count(); }

double gemm_resid_fill(int64_t M, int N) { return gemm_tile_fill(M, N, cu_count()); }

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
    if (a.Kw > 0 && (a.Kw % BK != 0 || (a.K != a.Kw && a.K != 2 * a.Kw))) return hipErrorInvalidValue;
    const bool wide_head = epi == EPI_QKV_ROPE && a.d == 128;       // a wave must span a whole 128-wide head
    // Few rows: when even 128 x 128 tiles do not give every CU one, the ring variants take over.  64-row tiles double
    // the tile count; they pay when that still fits one round of the chip (a ring workgroup has its CU to itself),
    // otherwise 128-row tiles with fewer, larger k-steps do (modelled as rounds x bytes per k-tile).
    const int64_t tiles128 = ((a.M + 127) / 128) * ((a.N + (wide_head ? 255 : 127)) / (wide_head ? 256 : 128));
    if (tiles128 < cu_count()) {
        const int64_t cus = cu_count();
        const int64_t t64 = ((a.M + 63) / 64) * ((a.N + (wide_head ? 255 : 127)) / (wide_head ? 256 : 128));
        if (wide_head) return launch_ring<EPI_QKV_ROPE, 64, 256, 2, 2, 2, 3>(a, st);
        const int64_t cost64 = ((t64 + cus - 1) / cus) * (64 + 128), cost128 = ((tiles128 + cus - 1) / cus) * (128 + 128);
        const bool r64 = cost64 <= cost128;
        // residual-add launches with so few rows that even 64 x 64 tiles fit one round: four times the workgroups of the
        // 128 x 128 shape, each with eight k-tiles in flight (nine stages of 16 KiB)
        const int64_t t6464 = ((a.M + 63) / 64) * ((a.N + 63) / 64);
        if (epi == EPI_RESID_ADD && t6464 <= cus) return launch_ring<EPI_RESID_ADD, 64, 64, 2, 2, 1, 9>(a, st);
        switch (epi) {
            case EPI_QKV_ROPE:
                return r64 ? launch_ring<EPI_QKV_ROPE, 64, 128, 2, 2, 1, 5>(a, st) : launch_ring<EPI_QKV_ROPE, 128, 128, 2, 2, 1, 4>(a, st);
            case EPI_RESID_ADD:
                return r64 ? launch_ring<EPI_RESID_ADD, 64, 128, 2, 2, 1, 5>(a, st) : launch_ring<EPI_RESID_ADD, 128, 128, 2, 2, 1, 4>(a, st);
            case EPI_SWIGLU:
                return r64 ? launch_ring<EPI_SWIGLU, 64, 128, 2, 2, 1, 5>(a, st) : launch_ring<EPI_SWIGLU, 128, 128, 2, 2, 1, 4>(a, st);
        }
    }
    // the tall tile: residual-add launches, and gate/up launches with a long k loop (not persistent: at K = 896 the
    // start-up round trip per tile costs more than the shape saves: 8.8 against 8.0 ms per step at the 0.5B shape)
    const bool tall_ok = epi == EPI_RESID_ADD || (epi == EPI_SWIGLU && a.K >= 2048);
    const TileChoice tile = choose_gemm_tile(a.M, a.N, wide_head ? 256 : 128, tall_ok, cu_count());
    if (tile == TILE_TALL)
        return epi == EPI_RESID_ADD ? launch_tile<EPI_RESID_ADD, 320, 256, 2, 4, 1>(a, st) : launch_tile<EPI_SWIGLU, 320, 256, 2, 4, 1>(a, st);
    const bool big = tile == TILE_BIG;
    switch (epi) {
        case EPI_QKV_ROPE:
            if (!wide_head) {
                return big ? launch_tile<EPI_QKV_ROPE, 256, 256, 2, 4, 1>(a, st) : launch_tile<EPI_QKV_ROPE, 128, 128, 2, 2, 1>(a, st);
            }
            return big ? launch_tile<EPI_QKV_ROPE, 256, 256, 4, 2, 2>(a, st) : launch_tile<EPI_QKV_ROPE, 128, 256, 2, 2, 2>(a, st);
        case EPI_RESID_ADD:
            return big ? launch_tile<EPI_RESID_ADD, 256, 256, 2, 4, 1>(a, st) : launch_tile<EPI_RESID_ADD, 128, 128, 2, 2, 1>(a, st);
        case EPI_SWIGLU:
            return big ? launch_tile<EPI_SWIGLU, 256, 256, 2, 4, 1>(a, st) : launch_tile<EPI_SWIGLU, 128, 128, 2, 2, 1>(a, st);
    }
    return hipErrorInvalidValue;
}

}  // namespace hr
