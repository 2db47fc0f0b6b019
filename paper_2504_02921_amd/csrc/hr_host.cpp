// Host-only part of libhyperrerank: configuration checks, pool layout and page bookkeeping,
// argument validation of the scoring call and the per-call metadata (schedule) builder.
// No HIP calls here, so every error path can be exercised on a machine without a GPU.
#include <algorithm>
#include <cstring>
#include <initializer_list>
#include <new>

#include "hr_internal.h"

namespace hr {

bool pool_cfg_valid(const hr_pool_cfg* c) {
    if (!c) return false;
    if (c->n_layers <= 0 || c->n_kv_heads <= 0 || c->num_pages <= 0) return false;
    if (c->head_dim <= 0 || c->head_dim % 16 != 0 || c->head_dim > 256) return false;
    if (c->page_tokens != kPageTokens) return false;
    if (c->kv_dtype != HR_F32 && c->kv_dtype != HR_BF16 && c->kv_dtype != HR_FP8_E4M3) return false;
    return true;
}

bool model_cfg_valid(const hr_model_cfg* c) {
    if (!c) return false;
    if (c->n_layers <= 0 || c->hidden <= 0 || c->n_q_heads <= 0 || c->n_kv_heads <= 0) return false;
    if (c->n_q_heads % c->n_kv_heads != 0) return false;
    if (c->head_dim <= 0 || c->head_dim % 16 != 0 || c->head_dim > 256) return false;
    if (c->ffn <= 0 || c->vocab <= 0) return false;
    if (c->hidden % 8 != 0 || c->ffn % 8 != 0) return false;
    if (c->yes_id < 0 || c->yes_id >= c->vocab || c->no_id < 0 || c->no_id >= c->vocab) return false;
    if (c->dtype != HR_F32 && c->dtype != HR_BF16) return false;
    if (!(c->rope_base > 1.0f) || !(c->rms_eps >= 0.0f)) return false;
    return true;
}

PoolLayout make_layout(const hr_pool_cfg& c) {
    PoolLayout l;
    l.n_layers = c.n_layers; l.n_kv = c.n_kv_heads; l.d = c.head_dim; l.num_pages = c.num_pages; l.kv_dtype = c.kv_dtype;
    l.esz = dtype_size(c.kv_dtype);
    l.block_elems = (size_t)kPageTokens * c.head_dim;
    size_t blocks = (size_t)c.n_layers * c.num_pages * c.n_kv_heads * 2;
    l.data_bytes = align_up(blocks * l.block_elems * l.esz);
    l.scale_bytes = c.kv_dtype == HR_FP8_E4M3 ? align_up(blocks * sizeof(float)) : 0;
    l.counter_off = l.data_bytes + l.scale_bytes;
    l.total_bytes = l.counter_off + kRangeCounterBytes;
    return l;
}

PackLayout make_pack_layout(const hr_model_cfg& c) {
    PackLayout p;
    size_t H = c.hidden, d = c.head_dim, F = c.ffn;
    size_t nqkv = (size_t)(c.n_q_heads + 2 * c.n_kv_heads) * d;
    // every slab starts on a 256-byte boundary for either element size
    auto up = [](size_t e) { return (e + 127) / 128 * 128; };
    p.wqkv = 0;
    p.wo = up(p.wqkv + nqkv * H);
    p.wgu = up(p.wo + H * (size_t)c.n_q_heads * d);
    p.wd = up(p.wgu + 2 * F * H);
    p.layer_elems = up(p.wd + H * F);
    p.counter_off = align_up(p.layer_elems * (size_t)c.n_layers * dtype_size(c.dtype));
    p.total_bytes = p.counter_off + kRangeCounterBytes;
    p.gu_interleave = (c.ffn % 32 == 0) ? 32 : 1;
    return p;
}

MetaLayout make_meta_layout(int64_t n_seq, int64_t T, int64_t pt_stride, int64_t n_out, int64_t dst_ints, int64_t grp_ints, bool share) {
    if (n_out < 0) n_out = n_seq;
    MetaLayout m;
    auto up = [](size_t e) { return (e + 63) / 64 * 64; };
    size_t o = 0;
    m.cu = o;          o = up(o + (size_t)n_seq + 1);
    m.tok_id = o;      o = up(o + (size_t)T);
    m.tok_pos = o;     o = up(o + (size_t)T);
    m.tok_seq = o;     o = up(o + (size_t)T);
    m.prefix_len = o;  o = up(o + (size_t)n_seq);
    m.page_table = o;  o = up(o + (size_t)n_seq * (size_t)pt_stride);
    m.new_slot = o;    o = up(o + (size_t)T);
    m.new_cu = o;      o = up(o + (size_t)n_seq + 1);
    m.out_row = o;     o = up(o + (size_t)n_out);
    m.dst_table = o;   o = up(o + (size_t)dst_ints);
    m.tok_src = o;     o = up(o + (share ? (size_t)T : 0));
    m.rep_row = o;     o = up(o + (share ? (size_t)T / 2 + 1 : 0));
    m.grp = o;         o = up(o + (size_t)grp_ints);
    m.total = o;
    return m;
}

Workspace make_workspace(const hr_model_cfg& c, int64_t n_seq, int64_t T, int64_t pt_stride, bool need_f32_scratch,
                         int64_t n_out, int64_t dst_ints, int64_t grp_ints, bool split_ops, bool share) {
    Workspace w;
    size_t asz = dtype_size(c.dtype);
    size_t H = c.hidden, d = c.head_dim, F = c.ffn;
    size_t nq = (size_t)c.n_q_heads * d, nkv = (size_t)c.n_kv_heads * d;
    size_t t = (size_t)T;
    // split_ops: some layers run with 22-bit operands, i.e. activations as [hi | lo] pairs of halves: y, q, o and m take
    // twice the room, the new tokens' K/V pages get a second buffer for their rounding residue, and the QKV projection of
    // those layers leaves fp32 rows for a RoPE kernel of its own
    const size_t sp = split_ops ? 2 : 1;
    MetaLayout ml = make_meta_layout(n_seq, T, pt_stride, n_out, dst_ints, grp_ints, share);
    w.meta_ints = ml.total;
    size_t o = 0;
    w.off_meta = o; o = align_up(o + ml.total * sizeof(int32_t));
    w.off_rope = o; o = align_up(o + t * (d / 2) * 2 * sizeof(float));
    w.off_x = o;    o = align_up(o + t * H * sizeof(float));
    w.off_y = o;    o = align_up(o + sp * t * H * asz);
    w.off_q = o;    o = align_up(o + sp * t * nq * asz);
    // new-token K and V: either [T][n_kv][d] each, or pages of 16 slots (32-slot aligned per sequence), K|V blocks
    // interleaved like the pool; one region of 2 * (T + 32 n_seq) token slots serves both forms
    const size_t kv_slots = t + 32 * (size_t)n_seq;
    w.off_k = o;    o = align_up(o + kv_slots * nkv * asz);
    w.off_v = o;    o = align_up(o + kv_slots * nkv * asz);
    w.off_kvlo = o;
    if (split_ops) o = align_up(o + 2 * kv_slots * nkv * asz);      // between K/V and o: cleared together with them
    w.off_o = o;    o = align_up(o + sp * t * nq * asz);
    w.off_m = o;    o = align_up(o + sp * t * F * asz);
    w.off_f32 = o;
    if (need_f32_scratch) o = align_up(o + t * std::max(nq + 2 * nkv, 2 * F) * sizeof(float));
    else if (split_ops) o = align_up(o + t * (nq + 2 * nkv) * sizeof(float));
    else if (share) o = align_up(o + (t / 2 + 1) * (nq + 2 * nkv) * sizeof(float));     // shared first-layer rows: at most T / 2
    w.total = o;
    return w;
}

int pool_check_read(const hr_pool* pool, int32_t doc_len, const int32_t* page_ids) {
    if (!pool || !page_ids) return HR_ERR_INVALID_ARG;
    if (doc_len <= 0) return HR_ERR_LEN_RANGE;
    int64_t n = ((int64_t)doc_len + kPageTokens - 1) / kPageTokens;
    if (n > pool->cfg.num_pages) return HR_ERR_LEN_RANGE;
    for (int64_t i = 0; i < n; ++i) {
        int32_t p = page_ids[i];
        if (p < 0 || p >= pool->cfg.num_pages) return HR_ERR_PAGE_RANGE;
    }
    for (int64_t i = 0; i < n; ++i)
        if (pool->state[page_ids[i]] != PAGE_USED) return HR_ERR_TABLE_SHORT;
    return HR_OK;
}

size_t page_record4_bytes(const PoolLayout& lay) {
    if (lay.kv_dtype != HR_BF16 || lay.d % 32 != 0) return 0;
    return (size_t)lay.n_layers * lay.n_kv * 20 * lay.d;      // per (layer, kv head): 16 d bytes of codes + 4 d of scales
}

int pool_check_write(const hr_pool* pool, int32_t doc_len, const int32_t* page_ids) {
    if (!pool || !page_ids) return HR_ERR_INVALID_ARG;
    if (doc_len <= 0) return HR_ERR_LEN_RANGE;
    int64_t n = ((int64_t)doc_len + kPageTokens - 1) / kPageTokens;
    if (n > pool->cfg.num_pages) return HR_ERR_LEN_RANGE;
    for (int64_t i = 0; i < n; ++i) {
        int32_t p = page_ids[i];
        if (p < 0 || p >= pool->cfg.num_pages) return HR_ERR_PAGE_RANGE;
    }
    for (int64_t i = 0; i < n; ++i)
        if (pool->state[page_ids[i]] == PAGE_USED) return HR_ERR_PAGE_IN_USE;
    // duplicates: sort a copy (documents have at most a few thousand pages)
    std::vector<int32_t> s(page_ids, page_ids + n);
    std::sort(s.begin(), s.end());
    if (std::adjacent_find(s.begin(), s.end()) != s.end()) return HR_ERR_PAGE_DUP;
    return HR_OK;
}

int pool_check_pages(const hr_pool* pool, int64_t n, const int32_t* page_ids, bool want_used) {
    if (!pool || n < 0 || (n > 0 && !page_ids)) return HR_ERR_INVALID_ARG;
    if (!want_used && n > pool->cfg.num_pages) return HR_ERR_PAGE_DUP;      // more ids than pages: some id repeats
    for (int64_t i = 0; i < n; ++i)
        if (page_ids[i] < 0 || page_ids[i] >= pool->cfg.num_pages) return HR_ERR_PAGE_RANGE;
    if (want_used) {
        for (int64_t i = 0; i < n; ++i)
            if (pool->state[page_ids[i]] != PAGE_USED) return HR_ERR_TABLE_SHORT;
        return HR_OK;
    }
    for (int64_t i = 0; i < n; ++i)
        if (pool->state[page_ids[i]] == PAGE_USED) return HR_ERR_PAGE_IN_USE;
    std::vector<int32_t> s(page_ids, page_ids + n);
    std::sort(s.begin(), s.end());
    if (std::adjacent_find(s.begin(), s.end()) != s.end()) return HR_ERR_PAGE_DUP;
    return HR_OK;
}

size_t page_record_bytes(const PoolLayout& lay) {
    const size_t data = (size_t)lay.n_layers * lay.n_kv * 2 * lay.block_elems * lay.esz;
    const size_t scales = lay.kv_dtype == HR_FP8_E4M3 ? (size_t)lay.n_layers * lay.n_kv * 2 * sizeof(float) : 0;
    return (data + scales + 15) / 16 * 16;
}

void pool_mark(hr_pool* pool, const int32_t* page_ids, int n, PageState st) {
    for (int i = 0; i < n; ++i) {
        uint8_t& cur = pool->state[page_ids[i]];
        if (cur == PAGE_FREE && st != PAGE_FREE) pool->n_free--;
        if (cur != PAGE_FREE && st == PAGE_FREE) pool->n_free++;
        cur = st;
    }
}

int score_check_args(const hr_model_cfg& mc, const hr_pool* pool, int32_t n_pairs, const int32_t* page_table,
                     int32_t pt_stride, const int32_t* doc_lens, const int32_t* query_tokens,
                     const int32_t* query_lens, int64_t max_keys, int64_t* total_q_out) {
    if (!pool || n_pairs < 0 || pt_stride < 0) return HR_ERR_INVALID_ARG;
    if (n_pairs > 0 && (!doc_lens || !query_lens || !query_tokens)) return HR_ERR_INVALID_ARG;
    if (pool->cfg.n_layers != mc.n_layers || pool->cfg.n_kv_heads != mc.n_kv_heads || pool->cfg.head_dim != mc.head_dim)
        return HR_ERR_MISMATCH;
    if (mc.dtype == HR_F32 && pool->cfg.kv_dtype != HR_F32) return HR_ERR_MISMATCH;
    if (mc.dtype == HR_BF16 && pool->cfg.kv_dtype == HR_F32) return HR_ERR_MISMATCH;
    int64_t T = 0;
    for (int32_t p = 0; p < n_pairs; ++p) {
        int32_t D = doc_lens[p], q = query_lens[p];
        if (D < 0 || q <= 0) return HR_ERR_LEN_RANGE;
        if ((int64_t)D + q > max_keys) return HR_ERR_LEN_RANGE;
        int64_t np = ((int64_t)D + kPageTokens - 1) / kPageTokens;
        if (np > pt_stride) return HR_ERR_TABLE_SHORT;
        if (np > 0 && !page_table) return HR_ERR_INVALID_ARG;
        const int32_t* row = page_table + (size_t)p * pt_stride;
        for (int64_t i = 0; i < np; ++i) {
            int32_t pg = row[i];
            if (pg == -1) return HR_ERR_TABLE_SHORT;
            if (pg < 0 || pg >= pool->cfg.num_pages) return HR_ERR_PAGE_RANGE;
            if (pool->state[pg] != PAGE_USED) return HR_ERR_TABLE_SHORT;
        }
        T += q;
    }
    if (T > (int64_t)1 << 30) return HR_ERR_LEN_RANGE;
    for (int64_t t = 0; t < T; ++t)
        if (query_tokens[t] < 0 || query_tokens[t] >= mc.vocab) return HR_ERR_TOKEN_RANGE;
    if (total_q_out) *total_q_out = T;
    return HR_OK;
}

void fill_meta(int32_t* meta, const MetaLayout& ml, int64_t n_seq, const int32_t* prefix_lens,
               const int32_t* new_lens, const int32_t* tokens, const int32_t* page_table, int64_t pt_stride,
               const int32_t* out_rows, int64_t n_out) {
    int32_t* cu = meta + ml.cu;
    int32_t* tok_id = meta + ml.tok_id;
    int32_t* tok_pos = meta + ml.tok_pos;
    int32_t* tok_seq = meta + ml.tok_seq;
    int32_t* pre = meta + ml.prefix_len;
    int32_t* new_slot = meta + ml.new_slot;
    int32_t* new_cu = meta + ml.new_cu;
    int64_t t = 0;
    int64_t slot0 = 0;
    cu[0] = 0;
    for (int64_t p = 0; p < n_seq; ++p) {
        int32_t D = prefix_lens ? prefix_lens[p] : 0;
        pre[p] = D;
        for (int32_t i = 0; i < new_lens[p]; ++i, ++t) {
            tok_id[t] = tokens[t];
            tok_pos[t] = D + i;       // positions continue right after the document
            tok_seq[t] = (int32_t)p;
            new_slot[t] = (int32_t)(slot0 + i);
        }
        cu[p + 1] = (int32_t)t;
        new_cu[p] = (int32_t)slot0;
        slot0 += ((int64_t)new_lens[p] + 31) / 32 * 32;
    }
    new_cu[n_seq] = (int32_t)slot0;
    int32_t* out_row = meta + ml.out_row;
    if (out_rows) {
        std::memcpy(out_row, out_rows, sizeof(int32_t) * (size_t)n_out);
    } else {                                           // default: the last new token of every sequence
        for (int64_t p = 0; p < n_seq; ++p) out_row[p] = cu[p + 1] - 1;
    }
    if (page_table && pt_stride > 0)
        std::memcpy(meta + ml.page_table, page_table, sizeof(int32_t) * (size_t)n_seq * (size_t)pt_stride);
}

QueryShare make_query_share(int64_t n_seq, const int32_t* new_lens, const int32_t* tokens) {
    QueryShare qs;
    std::vector<int64_t> start((size_t)n_seq + 1, 0);
    for (int64_t p = 0; p < n_seq; ++p) start[p + 1] = start[p] + new_lens[p];
    qs.tok_src.resize((size_t)start[n_seq]);
    // sequences in the order (length, hash of the string, index); equal strings end up next to each other and are told
    // apart from mere hash collisions by comparing the tokens
    std::vector<uint64_t> hash((size_t)n_seq);
    for (int64_t p = 0; p < n_seq; ++p) {
        uint64_t h = 1469598103934665603ull;
        for (int64_t t = start[p]; t < start[p + 1]; ++t) h = (h ^ (uint32_t)tokens[t]) * 1099511628211ull;
        hash[p] = h;
    }
    std::vector<int32_t> order((size_t)n_seq);
    for (int64_t p = 0; p < n_seq; ++p) order[p] = (int32_t)p;
    std::sort(order.begin(), order.end(), [&](int32_t a, int32_t b) {
        if (new_lens[a] != new_lens[b]) return new_lens[a] < new_lens[b];
        if (hash[a] != hash[b]) return hash[a] < hash[b];
        return a < b;
    });
    std::vector<int32_t> leader((size_t)n_seq, -1);          // first sequence (lowest index) with the same string
    for (int64_t i = 0; i < n_seq;) {
        int64_t j = i;
        while (j < n_seq && new_lens[order[j]] == new_lens[order[i]] && hash[order[j]] == hash[order[i]]) ++j;
        for (int64_t a = i; a < j; ++a) {
            if (leader[order[a]] >= 0) continue;
            leader[order[a]] = order[a];
            for (int64_t b = a + 1; b < j; ++b)
                if (leader[order[b]] < 0 && std::memcmp(tokens + start[order[a]], tokens + start[order[b]],
                                                        sizeof(int32_t) * (size_t)new_lens[order[a]]) == 0)
                    leader[order[b]] = order[a];
        }
        i = j;
    }
    std::vector<int64_t> first_row((size_t)n_seq, -1);       // unique row of a leader's first token
    for (int64_t p = 0; p < n_seq; ++p) {
        const int32_t ld = leader[p];
        if (ld == p) {
            first_row[p] = qs.n_uniq;
            for (int64_t t = start[p]; t < start[p + 1]; ++t) qs.rep_row.push_back((int32_t)t);
            qs.n_uniq += new_lens[p];
        }
        for (int64_t i = 0; i < new_lens[p]; ++i) qs.tok_src[start[p] + i] = (int32_t)(first_row[ld] + i);
    }
    return qs;
}

ChunkPlan make_chunk_plan(int64_t n_seq, const int32_t* lens, int chunk) {
    ChunkPlan cp;
    int64_t slot = 0, row = 0;
    for (int64_t s = 0; s < n_seq; ++s) {
        const int64_t n_ch = ((int64_t)lens[s] + chunk - 1) / chunk;
        cp.pt_stride = std::max<int64_t>(cp.pt_stride, (n_ch - 1) * chunk / kPageTokens);
        cp.n_chunks += n_ch;
    }
    cp.page_table.assign((size_t)cp.n_chunks * (size_t)std::max<int64_t>(cp.pt_stride, 1), -1);
    const int64_t stride = std::max<int64_t>(cp.pt_stride, 1);
    cp.pt_stride = stride;
    int64_t ci = 0;
    for (int64_t s = 0; s < n_seq; ++s) {
        const int64_t first_page = slot / kPageTokens;
        cp.first_page.push_back((int32_t)first_page);
        for (int64_t off = 0; off < lens[s]; off += chunk, ++ci) {
            const int32_t n = (int32_t)std::min<int64_t>(chunk, lens[s] - off);
            cp.prefix_lens.push_back((int32_t)off);
            cp.new_lens.push_back(n);
            for (int64_t pg = 0; pg < off / kPageTokens; ++pg) cp.page_table[ci * stride + pg] = (int32_t)(first_page + pg);
            slot += (n + 31) / 32 * 32;          // same rule as fill_meta: full chunks keep a sequence's slots contiguous
            row += n;
        }
        cp.out_row.push_back((int32_t)(row - 1));
    }
    cp.T = row;
    return cp;
}

size_t group_plan_ints_bound(int64_t n_seq, int64_t T, int g) {
    // every sequence adds at most one partial block and one partial sub-tile; a sequence may be cut into up to
    // kMaxPiecesPerSeq work items (few sequences: pieces of 4 blocks; long queries: pieces of 8 or 16), each of which
    // lists the sequence's sub-tiles
    const size_t cut = kMaxPiecesPerSeq;
    const size_t nb = (size_t)(T * g / 32 + n_seq), ns = (size_t)(T / 32 + n_seq) * cut, ng = (size_t)n_seq * cut;
    return ng + 2 * (ng + 1) + 2 * nb + 3 * ns;
}

GroupPlan make_group_plan(int64_t n_seq, const int32_t* prefix_lens, const int32_t* new_lens, const int32_t* page_table,
                          int64_t pt_stride, int g, int cap_blocks, bool cut_long) {
    GroupPlan gp;
    auto blocks_of = [&](int64_t p) { return (int)(((int64_t)new_lens[p] * g + 31) / 32); };
    auto pages_of = [&](int64_t p) { return ((int64_t)prefix_lens[p] + kPageTokens - 1) / kPageTokens; };
    const int32_t* pt = page_table;
    // sequences with the same document next to each other: by first page, then length, then index
    std::vector<int32_t> order((size_t)n_seq);
    for (int64_t p = 0; p < n_seq; ++p) order[p] = (int32_t)p;
    auto first_page = [&](int32_t p) { return prefix_lens[p] > 0 && pt ? pt[(int64_t)p * pt_stride] : -1; };
    std::sort(order.begin(), order.end(), [&](int32_t a, int32_t b) {
        const int32_t fa = first_page(a), fb = first_page(b);
        if (fa != fb) return fa < fb;
        if (prefix_lens[a] != prefix_lens[b]) return prefix_lens[a] < prefix_lens[b];
        return a < b;
    });
    struct Piece { int32_t seq; int b0, nb; };               // blocks b0 .. b0 + nb - 1 of a sequence
    struct Grp { std::vector<Piece> pieces; int blocks; int64_t cost; };
    std::vector<Grp> groups;
    for (int64_t i = 0; i < n_seq;) {
        // run of sequences whose rows equal the first one's (a sequence without a document is a run of its own)
        const int32_t lead = order[i];
        int64_t j = i + 1;
        if (prefix_lens[lead] > 0 && pt)                   // without a page table every sequence is taken to have its own document
            while (j < n_seq && first_page(order[j]) == first_page(lead) && prefix_lens[order[j]] == prefix_lens[lead] &&
                   std::memcmp(pt + (int64_t)order[j] * pt_stride, pt + (int64_t)lead * pt_stride,
                               sizeof(int32_t) * (size_t)pages_of(lead)) == 0)
                ++j;
        // first fit over the run's groups, sequences in index order; a sequence with more blocks than a group holds is a
        // group of its own, or (cut_long) is cut into pieces of at most cap_blocks
        const size_t run_first = groups.size();
        for (int64_t k = i; k < j; ++k) {
            const int32_t p = order[k];
            const int nb_all = blocks_of(p);
            const int step = cut_long ? cap_blocks : nb_all;
            for (int b0 = 0; b0 < nb_all; b0 += step) {
                const int nb = std::min(step, nb_all - b0);
                size_t gi = run_first;
                while (gi < groups.size() && groups[gi].blocks + nb > cap_blocks) ++gi;
                if (gi == groups.size()) groups.push_back(Grp{{}, 0, 0});
                groups[gi].pieces.push_back(Piece{p, b0, nb});
                groups[gi].blocks += nb;
                gp.cut = gp.cut || nb < nb_all;
            }
        }
        for (size_t gi = run_first; gi < groups.size(); ++gi)
            groups[gi].cost = ((int64_t)prefix_lens[lead] + 64) * groups[gi].blocks;
        i = j;
    }
    for (const Grp& gr : groups) gp.uneven = gp.uneven || gr.cost != groups[0].cost;
    std::stable_sort(groups.begin(), groups.end(), [](const Grp& a, const Grp& b) { return a.cost > b.cost; });

    // start of every sequence's pages in the new-KV buffer: each sequence begins on a 32-slot boundary (fill_meta)
    std::vector<int64_t> new_page((size_t)n_seq);
    int64_t slot0 = 0;
    for (int64_t p = 0; p < n_seq; ++p) {
        new_page[p] = slot0 / kPageTokens;
        slot0 += ((int64_t)new_lens[p] + 31) / 32 * 32;
    }
    gp.n_groups = (int32_t)groups.size();
    gp.blk_cu.push_back(0);
    gp.sub_cu.push_back(0);
    for (const Grp& gr : groups) {
        gp.p0.push_back(gr.pieces[0].seq);
        gp.max_blocks = std::max(gp.max_blocks, gr.blocks);
        for (size_t pi = 0; pi < gr.pieces.size(); ++pi) {
            const Piece& pc = gr.pieces[pi];
            for (int b = pc.b0; b < pc.b0 + pc.nb; ++b) {
                gp.blk_seq.push_back(pc.seq);
                gp.blk_row0.push_back(b * 32);
            }
            bool listed = false;                             // the sequence's own keys once per group
            for (size_t pj = 0; pj < pi; ++pj) listed = listed || gr.pieces[pj].seq == pc.seq;
            if (listed) continue;
            gp.shared = gp.shared || pi > 0;
            for (int32_t k0 = 0; k0 < new_lens[pc.seq]; k0 += 32) {
                gp.sub_page.push_back((int32_t)(new_page[pc.seq] + k0 / kPageTokens));
                gp.sub_seq.push_back(pc.seq);
                gp.sub_key0.push_back(k0);
            }
        }
        gp.blk_cu.push_back((int32_t)gp.blk_seq.size());
        gp.sub_cu.push_back((int32_t)gp.sub_page.size());
    }
    return gp;
}

void store_group_plan(const GroupPlan& gp, int32_t* dst) {
    for (const std::vector<int32_t>* v : {&gp.p0, &gp.blk_cu, &gp.sub_cu, &gp.blk_seq, &gp.blk_row0, &gp.sub_page, &gp.sub_seq,
                                          &gp.sub_key0}) {
        std::memcpy(dst, v->data(), sizeof(int32_t) * v->size());
        dst += v->size();
    }
}

TileChoice choose_gemm_tile(int64_t M, int N, int small_bn, bool tall_ok, int cus_) {
    const int64_t cus = cus_ > 0 ? cus_ : 1;
    const int64_t big_tiles = ((M + 255) / 256) * ((N + 255) / 256);
    const int64_t tall_tiles = ((M + 319) / 320) * ((N + 255) / 256);
    const int64_t small_tiles = ((M + 127) / 128) * ((N + small_bn - 1) / small_bn);
    const double big = (double)((big_tiles + cus - 1) / cus) * 256.0 * 256.0 * 1.0;
    const double tall = (double)((tall_tiles + cus - 1) / cus) * 320.0 * 256.0 * 0.9;
    const double small = (double)((small_tiles + 2 * cus - 1) / (2 * cus)) * 2.0 * 128.0 * small_bn * 1.14;
    if (tall_ok && tall < big && tall <= small) return TILE_TALL;
    return big <= small ? TILE_BIG : TILE_SMALL;
}

double gemm_tile_fill(int64_t M, int N, int cus_) {
    const int64_t cus = cus_ > 0 ? cus_ : 1;
    int64_t tiles = 0, slots = cus;
    switch (choose_gemm_tile(M, N, 128, true, (int)cus)) {
        case TILE_TALL: tiles = ((M + 319) / 320) * ((N + 255) / 256); break;
        case TILE_BIG: tiles = ((M + 255) / 256) * ((N + 255) / 256); break;
        case TILE_SMALL: tiles = ((M + 127) / 128) * ((N + 127) / 128); slots = 2 * cus; break;
    }
    if (tiles <= 0) return 1.0;
    return (double)tiles / (double)(((tiles + slots - 1) / slots) * slots);
}

}  // namespace hr

// ------------------------------------------------------------------------------------------------
// C ABI: the calls that need no device work
// ------------------------------------------------------------------------------------------------
extern "C" {

const char* hr_status_str(int s) {
    switch (s) {
        case HR_OK: return "ok";
        case HR_ERR_INVALID_ARG: return "invalid argument";
        case HR_ERR_POOL_TOO_SMALL: return "pool buffer too small";
        case HR_ERR_PAGE_RANGE: return "page id out of range";
        case HR_ERR_PAGE_IN_USE: return "page already in use";
        case HR_ERR_PAGE_DUP: return "duplicate page id";
        case HR_ERR_LEN_RANGE: return "length out of range";
        case HR_ERR_TABLE_SHORT: return "page table row too short or names an unwritten page";
        case HR_ERR_TOKEN_RANGE: return "token id out of range";
        case HR_ERR_WORKSPACE_SMALL: return "workspace too small";
        case HR_ERR_UNSUPPORTED_SHAPE: return "unsupported shape";
        case HR_ERR_DEVICE: return "device error";
        case HR_ERR_POOL_FULL: return "not enough free pages";
        case HR_ERR_MISMATCH: return "pool and model do not match";
        default: return "unknown status";
    }
}

size_t hr_kv_page_record_bytes(const hr_pool* pool) { return pool ? hr::page_record_bytes(pool->lay) : 0; }
size_t hr_kv_page_record4_bytes(const hr_pool* pool) { return pool ? hr::page_record4_bytes(pool->lay) : 0; }

size_t hr_kv_pool_bytes(const hr_pool_cfg* cfg) {
    if (!hr::pool_cfg_valid(cfg)) return 0;
    return hr::make_layout(*cfg).total_bytes;
}

int hr_kv_pool_create(const hr_pool_cfg* cfg, void* dev_mem, size_t bytes, hr_pool** out) {
    if (!out) return HR_ERR_INVALID_ARG;
    *out = nullptr;
    if (!hr::pool_cfg_valid(cfg) || !dev_mem) return HR_ERR_INVALID_ARG;
    if ((uintptr_t)dev_mem % hr::kAlign != 0) return HR_ERR_INVALID_ARG;
    hr::PoolLayout lay = hr::make_layout(*cfg);
    if (bytes < lay.total_bytes) return HR_ERR_POOL_TOO_SMALL;
    hr_pool* p = new (std::nothrow) hr_pool();
    if (!p) return HR_ERR_INVALID_ARG;
    p->cfg = *cfg;
    p->lay = lay;
    p->base = (char*)dev_mem;
    p->state.assign((size_t)cfg->num_pages, hr::PAGE_FREE);
    p->n_free = cfg->num_pages;
    *out = p;
    return HR_OK;
}

void hr_kv_pool_destroy(hr_pool* pool) { delete pool; }

int64_t hr_kv_pool_free_pages(const hr_pool* pool) {
    if (!pool) return HR_ERR_INVALID_ARG;
    return pool->n_free;
}

int hr_kv_pool_alloc_pages(hr_pool* pool, int32_t n, int32_t* out) {
    if (!pool || !out || n <= 0) return HR_ERR_INVALID_ARG;
    if (n > pool->n_free) return HR_ERR_POOL_FULL;
    int32_t got = 0;
    for (int32_t pg = 0; pg < pool->cfg.num_pages && got < n; ++pg)
        if (pool->state[pg] == hr::PAGE_FREE) out[got++] = pg;
    hr::pool_mark(pool, out, n, hr::PAGE_RESERVED);
    return HR_OK;
}

int hr_doc_kv_free(hr_pool* pool, const int32_t* page_ids, int32_t n) {
    if (!pool || n < 0 || (n > 0 && !page_ids)) return HR_ERR_INVALID_ARG;
    for (int32_t i = 0; i < n; ++i)
        if (page_ids[i] < 0 || page_ids[i] >= pool->cfg.num_pages) return HR_ERR_PAGE_RANGE;
    hr::pool_mark(pool, page_ids, n, hr::PAGE_FREE);
    return HR_OK;
}

size_t hr_weights_pack_bytes(const hr_model_cfg* cfg) {
    if (!hr::model_cfg_valid(cfg)) return 0;
    return hr::make_pack_layout(*cfg).total_bytes;
}

}  // extern "C"
