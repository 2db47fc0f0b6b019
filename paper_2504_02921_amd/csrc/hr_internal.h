// Internal definitions shared by the host logic and the HIP engine of libhyperrerank.
#pragma once

#include <cstddef>
#include <cstdint>
#include <vector>

#include "hyperrerank.h"

namespace hr {

constexpr int kPageTokens = HR_PAGE_TOKENS;
constexpr size_t kAlign = 256;
constexpr size_t kRangeCounterBytes = 256;     // room for 8 int64 counters of what the one-time conversions of caller data met
// ... (weights, document K/V), indexed by
enum RangeCounter { RC_OVERFLOW = 0, RC_UNDERFLOW = 1, RC_NONFINITE_IN = 2, RC_FP8_NAN_CODE = 3, RC_FP8_BAD_SCALE = 4 };

inline size_t align_up(size_t x, size_t a = kAlign) { return (x + a - 1) / a * a; }
inline size_t dtype_size(int dt) { return dt == HR_F32 ? 4 : dt == HR_BF16 ? 2 : dt == HR_FP8_E4M3 ? 1 : 0; }

enum PageState : uint8_t { PAGE_FREE = 0, PAGE_RESERVED = 1, PAGE_USED = 2 };

// Physical arrangement of the pool (private to the library):
//   data:   [layer][page][kv_head][K | V] blocks of 16 * head_dim elements.
//           Element order inside the K and V blocks: see hr_layout.h.
//   scales: fp8 pools only, after the data: [layer][page][kv_head][2] fp32 (K scale, V scale).
struct PoolLayout {
    int n_layers = 0, n_kv = 0, d = 0, num_pages = 0, kv_dtype = 0;
    size_t esz = 0;          // bytes per element
    size_t block_elems = 0;  // 16 * d
    size_t data_bytes = 0;   // aligned
    size_t scale_bytes = 0;  // aligned, 0 unless fp8
    size_t counter_off = 0;  // 8 int64 range counters (kRangeCounterBytes) behind data and scales
    size_t total_bytes = 0;

    size_t block_index(int layer, int page, int kvh, int which) const {
        return ((((size_t)layer * num_pages + page) * n_kv + kvh) * 2 + which);
    }
    size_t scale_index(int layer, int page, int kvh, int which) const { return block_index(layer, page, kvh, which); }
};

bool pool_cfg_valid(const hr_pool_cfg* cfg);
bool model_cfg_valid(const hr_model_cfg* cfg);
PoolLayout make_layout(const hr_pool_cfg& cfg);

// Packed weights of one layer (element offsets into the pack buffer).
struct PackLayout {
    size_t wqkv = 0, wo = 0, wgu = 0, wd = 0;   // element offsets within one layer's slab
    size_t layer_elems = 0;
    size_t counter_off = 0;  // bytes: range counters behind the last layer's slab
    size_t total_bytes = 0;
    int gu_interleave = 1;   // rows of gate / up alternate in blocks of this many
};
PackLayout make_pack_layout(const hr_model_cfg& cfg);

// Workspace carving for one call over `n_seq` sequences and `T` new tokens.
struct Workspace {
    size_t meta_ints = 0;      // int32 count of the metadata block
    size_t off_meta = 0, off_rope = 0, off_x = 0, off_y = 0, off_q = 0, off_k = 0, off_v = 0, off_kvlo = 0, off_o = 0,
           off_m = 0, off_f32 = 0;
    size_t total = 0;
};
// full_path: sequences carry their own document tokens (no page table).
// split_ops: room for the layers that run with split (hi + lo) operands
Workspace make_workspace(const hr_model_cfg& cfg, int64_t n_seq, int64_t T, int64_t pt_stride, bool need_f32_scratch,
                         int64_t n_out = -1, int64_t dst_ints = 0, int64_t grp_ints = 0, bool split_ops = false, bool share = false);

// Metadata block layout (int32 offsets inside the block), uploaded once per call.
// new_slot[t] / new_cu[p]: where the K/V of new token t goes when the new keys are kept as 16-token
// pages per sequence (each sequence starts on a 32-slot boundary so that MFMA sub-tiles are whole).
struct MetaLayout {
    size_t cu = 0, tok_id = 0, tok_pos = 0, tok_seq = 0, prefix_len = 0, page_table = 0, new_slot = 0, new_cu = 0, out_row = 0,
           dst_table = 0, tok_src = 0, rep_row = 0, grp = 0, total = 0;
};
// n_out: rows whose score is read (one per pair); dst_ints: extra table for the prefill target pages; grp_ints: room
// for a group plan (group_plan_ints_bound)
// share: room for the tables of sequences with identical token strings (tok_src [T], rep_row [T / 2 + 1])
MetaLayout make_meta_layout(int64_t n_seq, int64_t T, int64_t pt_stride, int64_t n_out = -1, int64_t dst_ints = 0,
                            int64_t grp_ints = 0, bool share = false);

}  // namespace hr

struct hr_pool {
    hr_pool_cfg cfg;
    hr::PoolLayout lay;
    char* base = nullptr;
    std::vector<uint8_t> state;
    int64_t n_free = 0;
    bool counters_zeroed = false;   // the range counters are cleared on the stream of the first write
};

// Host-side validation / bookkeeping (no HIP calls), used by the engine and testable on a CPU.
namespace hr {
int pool_check_write(const hr_pool* pool, int32_t doc_len, const int32_t* page_ids);
int pool_check_read(const hr_pool* pool, int32_t doc_len, const int32_t* page_ids);
void pool_mark(hr_pool* pool, const int32_t* page_ids, int n, PageState st);
// n pages by id: all in range, and all holding a document (want_used) or all distinct and not holding one
int pool_check_pages(const hr_pool* pool, int64_t n, const int32_t* page_ids, bool want_used);
size_t page_record_bytes(const PoolLayout& lay);
size_t page_record4_bytes(const PoolLayout& lay);      // 4-bit records of a 16-bit pool; 0 for other pools
int score_check_args(const hr_model_cfg& mc, const hr_pool* pool, int32_t n_pairs, const int32_t* page_table,
                     int32_t pt_stride, const int32_t* doc_lens, const int32_t* query_tokens,
                     const int32_t* query_lens, int64_t max_keys, int64_t* total_q_out);
// Fills the metadata block for a call.  new_lens[p] tokens at positions prefix_lens[p]..; tokens flat.
// out_rows / n_out: rows whose score is read; nullptr = the last new token of every sequence (then the layout must
// have been made with n_out == n_seq)
void fill_meta(int32_t* meta, const MetaLayout& ml, int64_t n_seq, const int32_t* prefix_lens,
               const int32_t* new_lens, const int32_t* tokens, const int32_t* page_table, int64_t pt_stride,
               const int32_t* out_rows = nullptr, int64_t n_out = 0);

// Sequences with identical new-token strings (the same query scored against several documents: Section 3.3, pairwise
// independence) have identical embeddings and, in the first layer, identical normalised rows and pre-RoPE q / k / v: those
// are computed once per distinct string.  rep_row[u] = a token row in [0, T) that carries unique row u's token;
// tok_src[t] = the unique row of token t.
struct QueryShare {
    std::vector<int32_t> rep_row, tok_src;
    int64_t n_uniq = 0;
};
QueryShare make_query_share(int64_t n_seq, const int32_t* new_lens, const int32_t* tokens);

// A long sequence run as chunks of at most `chunk` tokens: chunk c of a sequence is a pseudo-sequence whose
// prefix is the sequence's own earlier tokens, found as pages of the call's new-token K/V buffer.  Used by the
// no-reuse pass and by the document prefill (the scoring kernels are reused unchanged).
struct ChunkPlan {
    std::vector<int32_t> prefix_lens, new_lens;   // per pseudo-sequence
    std::vector<int32_t> page_table;              // [n_chunks][pt_stride] pages of the new-KV buffer
    std::vector<int32_t> out_row;                 // per original sequence: row of its last token
    std::vector<int32_t> first_page;              // per original sequence: first page in the new-KV buffer
    int64_t pt_stride = 0, n_chunks = 0, T = 0;
};
ChunkPlan make_chunk_plan(int64_t n_seq, const int32_t* lens, int chunk);

// Sequences that attend to the same cached document (same prefix length, identical page-table rows) share one
// pass over its pages: a group is one work item per kv head of the MFMA attention.  Its query rows are cut into
// blocks of 32 (the rows of a sequence are token-major, g heads per token; every sequence starts a new block), its
// own keys into sub-tiles of 32 (one sequence per sub-tile).  All arrays are int32 and go to the device as they are.
struct GroupPlan {
    std::vector<int32_t> p0;                 // [n_groups] a sequence of the group (its page-table row is followed)
    std::vector<int32_t> blk_cu, sub_cu;     // [n_groups + 1] ranges into blk_* / sub_*
    std::vector<int32_t> blk_seq, blk_row0;  // per block: sequence, first row of the block within the sequence
    std::vector<int32_t> sub_page, sub_seq, sub_key0;   // per sub-tile: first of its two pages in the new-KV buffer,
                                                         // sequence, first new-key index
    int32_t n_groups = 0, max_blocks = 0;
    bool shared = false;                     // some group holds more than one sequence
    bool uneven = false;                     // the groups differ in work: the heaviest-first order is worth having
    bool cut = false;                        // some sequence's blocks are spread over several groups
    size_t ints() const {
        return p0.size() + blk_cu.size() + sub_cu.size() + 2 * blk_seq.size() + 3 * sub_page.size();
    }
};
// g: query heads per kv head; cap_blocks: most blocks a group may hold.  A sequence with more blocks is a group of its
// own, or, with cut_long (calls of at most kGroupCutMaxSeqs sequences, where work items are scarce), is cut into several
// groups that each stream the document and the sequence's own keys for their share of its rows.
// Groups come in order of decreasing work (document keys x blocks), so that a round-robin walk starts the long ones
// first.
constexpr int64_t kGroupCutMaxSeqs = 128;      // more sequences than this always give every other CU a work item
constexpr int kMaxPiecesPerSeq = 8;            // a sequence's row blocks are spread over at most this many work items
GroupPlan make_group_plan(int64_t n_seq, const int32_t* prefix_lens, const int32_t* new_lens, const int32_t* page_table,
                          int64_t pt_stride, int g, int cap_blocks, bool cut_long = false);
size_t group_plan_ints_bound(int64_t n_seq, int64_t T, int g);

// ---- tile shape of an M x N MFMA GEMM launch on a device of `cus` compute units.  "big" = 256 x 256 with 8 waves (one
// workgroup per CU, the highest rate per output), "tall" = 320 x 256 with 8 waves (where the caller allows it: 12.5 % more
// operand bytes per k-tile for 25 % more rows, and 20 % fewer tiles) and "small" = 128 x small_bn with 4 waves (two
// workgroups per CU, ~14 % more time per output but four times finer tiles).  With M x N outputs spread over the CUs the
// last round of tiles is what decides (e.g. M = 20480, N = 896 on 256 CUs: 320 big tiles are two rounds, 256 tall tiles
// one), so the cost of a shape is modelled as rounds x resident workgroups x tile area x relative cost per output,
// from measured rates.
enum TileChoice { TILE_SMALL, TILE_BIG, TILE_TALL };
TileChoice choose_gemm_tile(int64_t M, int N, int small_bn, bool tall_ok, int cus);
// Share of the workgroup slots that the tiles of an M x N residual GEMM fill in the rounds they take, in the shape
// choose_gemm_tile picks for it (tall allowed): 1.0 = every round full.
double gemm_tile_fill(int64_t M, int N, int cus);
// Writes the plan at dst (>= plan.ints() entries) in the order p0, blk_cu, sub_cu, blk_seq, blk_row0, sub_page, sub_seq,
// sub_key0.
void store_group_plan(const GroupPlan& plan, int32_t* dst);
}  // namespace hr
