// Launchers of the HIP kernels (gfx950).  Every launcher enqueues on `st` and returns the HIP status
// of the launch; none of them synchronises.
#pragma once

#include <hip/hip_runtime.h>

#include "hr_internal.h"

namespace hr {

// Per-layer view of the document-KV pool handed to attention kernels.
struct PoolView {
    const char* data;      // pool base
    const float* scales;   // fp8 only, else nullptr
    int num_pages, n_kv, d, kv_dtype;
    size_t esz;
};

// Device-side view of the per-call metadata.
struct MetaView {
    const int32_t* cu;          // [n_seq + 1] start of each sequence's new tokens
    const int32_t* tok_id;      // [T]
    const int32_t* tok_pos;     // [T] RoPE position
    const int32_t* tok_seq;     // [T] sequence of each token
    const int32_t* prefix_len;  // [n_seq] cached-document length
    const int32_t* page_table;  // [n_seq][pt_stride]
    const int32_t* new_slot;    // [T] slot of each new token in the paged new-KV buffer
    const int32_t* new_cu;      // [n_seq + 1] first slot of each sequence (multiples of 32)
    const int32_t* out_row;     // [n_out] token row whose score is read
    // sequences with identical token strings (set when at most half of the token rows are distinct): token t's first-layer
    // projection is row tok_src[t] of n_uniq shared rows, and rep_row[u] is a token row that carries shared row u's token
    const int32_t* tok_src;
    const int32_t* rep_row;
    int32_t n_uniq;
    int32_t n_out;
    int32_t pt_stride;
    int32_t n_seq;
    int64_t T;
};

// ---- generic (any shape, VALU arithmetic in fp32) ----
hipError_t launch_embed(int dtype, const void* E, const MetaView& mv, float* x, int H, hipStream_t st);
hipError_t launch_rope_table(const MetaView& mv, float2* tab, int head_dim, float base, hipStream_t st);
// rows: optional gather (device array of T row indices into x): y row t <- x row rows[t]
hipError_t launch_rmsnorm(int dtype, const float* x, const float* gain, void* y, int64_t T, int H, float eps, hipStream_t st,
                          const int32_t* rows = nullptr);
// 22-bit operand form (16-bit models): y as [T][hi H | lo H] halves
hipError_t launch_rmsnorm_split(const float* x, const float* gain, void* y, int64_t T, int H, float eps, hipStream_t st,
                                const int32_t* rows = nullptr);
// fp32 qkv rows -> RoPE -> q and the new tokens' K/V as pages.  kv_lo != nullptr: the split form (q as [T][hi | lo] halves,
// the rounding residue of K/V in kv_lo).  tok_src != nullptr: token t reads qkv row tok_src[t] instead of row t.
hipError_t launch_rope_pages(const float* qkv, const float2* tab, void* q, void* kv_hi, void* kv_lo, const int32_t* new_slot,
                             const int32_t* tok_src, int64_t T, int n_q, int n_kv, int d, hipStream_t st);
// C[M][N] (+)= A[M][K] * W[N][K]^T, C fp32
hipError_t launch_gemm_generic(int dtype, const void* A, const void* W, float* C, int64_t M, int N, int K,
                               bool accumulate, hipStream_t st);
hipError_t launch_rope_split(int dtype, const float* qkv, const float2* tab, void* q, void* k, void* v, int64_t T,
                             int n_q, int n_kv, int d, hipStream_t st);
hipError_t launch_swiglu(int dtype, const float* gu, void* m, int64_t T, int F, int interleave, hipStream_t st);
hipError_t launch_attn_generic(int dtype, const void* q, const void* k_new, const void* v_new, void* o,
                               const MetaView& mv, const PoolView& pv, int layer, int n_q, int max_keys, hipStream_t st);
hipError_t launch_score_head(int dtype, const float* x, const float* gain, const void* E, const MetaView& mv,
                             float* scores, int H, float eps, int yes_id, int no_id, hipStream_t st);
// counters: 8 int64 in device memory (RangeCounter indices), or nullptr
hipError_t launch_kv_scatter(const PoolLayout& lay, char* pool_base, const int32_t* page_ids_host, int doc_len,
                             const void* k, const void* v, const float* ks, const float* vs, long long* counters, hipStream_t st);
// dst row ((r / ib) * mul + sel) * ib + r % ib  <-  src row r   (rows of `cols` elements)
hipError_t launch_pack_rows(int dtype, const void* src, void* dst, int rows, int cols, int ib, int mul, int sel,
                            long long* counters, hipStream_t st);

// ---- MFMA paths (bf16) ----
bool gemm_mfma_supported(const hr_model_cfg& c);
int device_cu_count();      // compute units of the current device (256 if it cannot be asked)
// Share of the workgroup slots that the tiles of an M x N residual GEMM fill in the rounds they take (tile shape as the
// launcher would choose it): 1.0 = every round full.
double gemm_resid_fill(int64_t M, int N);
enum GemmEpilogue { EPI_QKV_ROPE = 0, EPI_RESID_ADD = 1, EPI_SWIGLU = 2 };
struct GemmArgs {
    const void* A;      // [M][K] bf16
    const void* W;      // [N][K] bf16 (packed)
    int64_t M;
    int N, K;
    // Split A operand: 0 (or K) = plain; K / 2 = A is [M][K] holding [hi | lo] halves of a K/2-wide activation (the value
    // is hi + lo, 22 significant bits) and W has K / 2 columns, met by both halves: C = hi W^T + lo W^T
    int Kw;
    // EPI_SWIGLU: m is written as [M][2 * N/2] = [hi | lo]; EPI_QKV_ROPE: q is written as [M][2 * n_q * d] = [hi | lo]
    int split_out;
    // epilogue operands
    float* x;           // EPI_RESID_ADD: fp32 [M][N], x += acc
    void* out0;         // EPI_QKV_ROPE: q ; EPI_SWIGLU: m [M][N/2]
    void* out1;         // EPI_QKV_ROPE: k
    void* out2;         // EPI_QKV_ROPE: v
    const float2* rope; // [M][d/2]
    int n_q, n_kv, d;
    // EPI_QKV_ROPE, optional: K and V of the new tokens go to 16-slot pages (pool arrangement) at kv_pages,
    // token t at slot new_slot[t]; out1 / out2 are ignored then
    void* kv_pages;
    const int32_t* new_slot;
};
hipError_t launch_gemm_mfma(GemmEpilogue epi, const GemmArgs& a, hipStream_t st);

bool attn_mfma_supported(const hr_model_cfg& c, int kv_dtype, int max_q_len);          // one work item per (sequence, kv head)
bool attn_mfma_supported_cut(const hr_model_cfg& c, int kv_dtype, int max_q_len);      // ... or several, by a group plan
// Device-side view of a group plan (GroupPlan): sequences that share a cached document are one work item per kv head.
struct GroupView {
    int32_t n_groups = 0, max_blocks = 0;
    const int32_t *p0 = nullptr, *blk_cu = nullptr, *sub_cu = nullptr, *blk_seq = nullptr, *blk_row0 = nullptr, *sub_page = nullptr,
                  *sub_seq = nullptr, *sub_key0 = nullptr;
};
// kv_new_pages: the new tokens' K/V as pages (see GemmArgs::kv_pages).  groups: nullptr = every sequence on its own.
// kv_new_lo_pages: if set, the 22-bit form: q and o are [T][hi | lo] halves, and this buffer (same arrangement as
// kv_new_pages) holds what the rounding of the new tokens' K/V to half left out.
hipError_t launch_attn_mfma(const void* q, const void* kv_new_pages, void* o, const MetaView& mv,
                            const PoolView& pv, int layer, int n_q, int max_q_len, hipStream_t st, bool last_only = false,
                            const GroupView* groups = nullptr, const void* kv_new_lo_pages = nullptr);
// fp8 pools: quantising copy of whole pages (amax -> scale -> E4M3 codes per page and kv head) from the half new-KV buffer
hipError_t launch_pages_to_pool_fp8(const char* kv_new, char* pool_layer_base, float* scales_layer_base, const int32_t* src_page,
                                    const int32_t* dst_page, int n_pages, int n_kv, int d, hipStream_t st);
// inverse of launch_kv_scatter: pages -> logical [L][D][n_kv][d] in the pool's element type (+ scales for fp8)
hipError_t launch_kv_gather(const PoolLayout& lay, const char* pool_base, const int32_t* page_ids_host, int doc_len, void* k, void* v,
                            float* ks, float* vs, hipStream_t st);
// whole pages between the pool and page records ([layer][kv head][K | V], then the fp8 scales): to_pool picks the direction
hipError_t launch_pages_move(const PoolLayout& lay, char* pool_base, const int32_t* page_ids_host, int64_t n_pages, char* records,
                             bool to_pool, hipStream_t st);
// the same with 4-bit records (16-bit pools; quantised on the way out, expanded on the way in)
hipError_t launch_pages_move4(const PoolLayout& lay, char* pool_base, const int32_t* page_ids_host, int64_t n_pages, char* records,
                              bool to_pool, hipStream_t st);
hipError_t launch_fill_zero(void* dst, size_t bytes, hipStream_t st);
// read-only pass over `bytes` of src (whole KiB), folding what it reads into sink (>= 4 bytes); to_lds: direct-to-LDS loads
hipError_t launch_probe_read(const void* src, size_t bytes, void* sink, size_t sink_bytes, bool to_lds, int cus, hipStream_t st);
// dst[i][:] = src[rows[i]][:] for n rows of `cols` floats (device arrays)
hipError_t launch_gather_rows_f32(const float* src, const int32_t* rows, float* dst, int n, int cols, hipStream_t st);
// per-segment top-k by rank counting: idx [n_seg][k] (-1 padded), optional scores [n_seg][k]
hipError_t launch_segment_topk(const float* scores, const int32_t* seg, int n_seg, int max_cands, int k, int32_t* idx, float* out_scores,
                               hipStream_t st);
// copy whole pages (all kv heads) from the new-KV page buffer to pool pages of one layer:
// pool page dst_table[i] <- new page src_first[doc(i)] + i  (16-bit pools: same arrangement on both sides)
hipError_t launch_pages_to_pool(const char* kv_new, char* pool_layer_base, const int32_t* src_page, const int32_t* dst_page,
                                int n_pages, int page_bytes_all_heads, hipStream_t st);

}  // namespace hr
