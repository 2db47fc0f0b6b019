// Device-facing entry points of libhyperrerank: weight packing, pool writes and reads, the host tier's page moves, and
// the layer loop shared by the scoring pass (query suffix over cached document KV; large calls as two halves on two
// streams), the no-reuse reference pass and the document prefill.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <new>
#include <vector>

#include "hr_internal.h"
#include "hr_kernels.h"

struct hr_model {
    hr_model_cfg cfg;
    hr::PackLayout pack;
    const char* pack_base = nullptr;
    const void* embedding = nullptr;
    const float* final_norm = nullptr;
    std::vector<const float*> norm1, norm2;
    bool mfma_gemm = false;
    bool force_generic = false;
    // optional per-kernel timing with HIP events (benchmarks)
    bool prof_on = false;
    bool no_last_short = false;           // HR_NO_LAST_SHORTCUT=1: run the last layer on every token (A/B runs)
    bool no_doc_groups = false;           // HR_NO_DOC_GROUPS=1: pairs that share a document are not batched (A/B runs)
    bool no_query_share = false;          // HR_NO_QUERY_SHARING=1: the first layer's projections are computed per pair (A/B runs)
    int n_streams = 2;                    // a large scoring call runs as two halves on two streams (hr_rerank_set_streams)
    hipStream_t aux_stream = nullptr;     // the second one, created on first use
    hipEvent_t fork_ev = nullptr, join_ev = nullptr;
    uint32_t prof_mask = 0xFFFFFFFFu;     // kernel classes that are timed while prof_on
    std::vector<hipEvent_t> prof_events;          // pool, two per timed launch
    std::vector<int> prof_class;                  // class of each recorded launch
    size_t prof_used = 0;                         // events in use
    // pinned staging for the per-call metadata upload
    int32_t* stage = nullptr;
    size_t stage_ints = 0;
    hipEvent_t stage_ev = nullptr;
    bool stage_pending = false;
    int device = -1;                      // the HIP device that was current when the weights were loaded
    int n_precise = 0;                    // leading layers of a scoring pass that run with split (hi + lo) operands
};

// Scratch of hr_rerank_score_static: the workspace of a scoring call as a file-scope device array, for callers that
// cannot hand over (or allocate) a workspace.  Every GPU the library runs on holds its own copy until the process ends.
// In host code the array's name is only a stand-in for the symbol: the device address comes from hipGetSymbolAddress,
// once per device, and that pointer is what kernels, copies and fills get.
constexpr size_t kStaticScratchBytes = (size_t)128 << 20;
static __device__ __align__(256) unsigned char g_static_scratch[kStaticScratchBytes];

namespace {

using namespace hr;

constexpr int64_t kGenericMaxKeys = 15000;     // scores of one row live in LDS in the generic attention
constexpr int64_t kMfmaMaxKeys = 1 << 20;
constexpr int64_t kChunkedMaxKeys = 1 << 15;   // longest sequence of the chunked passes (no-reuse pass, document prefill): bounds
                                               // the self page table, which has one row per 32- or 64-token chunk
constexpr int64_t kSplitMinTokens = 8192;      // query tokens from which a scoring call is cut in two halves
constexpr double kSplitMaxFill = 0.85;         // ... when the N = hidden GEMMs' tiles fill less than this share of their rounds
constexpr size_t kSplitSlackBytes = (size_t)1 << 20;   // what two carvings of a workspace may need beyond one (alignment gaps,
                                                       // the larger group-plan room of calls with few pairs)

thread_local char g_last_error[256] = "";

void note_hip_error(hipError_t e, const char* what) {
    snprintf(g_last_error, sizeof(g_last_error), "%s: %s", what, hipGetErrorString(e));
}

#define HR_HIP(expr)                                   \
    do {                                               \
        hipError_t e__ = (expr);                       \
        if (e__ != hipSuccess) {                       \
            note_hip_error(e__, #expr);                \
            return HR_ERR_DEVICE;                      \
        }                                              \
    } while (0)

// The MFMA attention reads the new tokens' K/V as pool-format pages, which only the MFMA QKV projection's epilogue
// writes: the two kernel families are chosen together.
// may_cut: the call can spread a sequence's row blocks over several work items (a group plan travels with it), so more
// rows per kv head than one work item holds are fine as long as kMaxPiecesPerSeq items of the largest size take them.
bool use_mfma_attn(const hr_model* m, int kv_dtype, int max_new_len, bool may_cut = false) {
    if (m->force_generic || !m->mfma_gemm) return false;
    if (may_cut && !m->no_doc_groups) return attn_mfma_supported_cut(m->cfg, kv_dtype, max_new_len);
    return attn_mfma_supported(m->cfg, kv_dtype, max_new_len);
}

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mu;
char* g_scratch_ptr[kMaxDevices] = {};      // device address of g_static_scratch, per HIP device

// Address of the static scratch on the current device (looked up on first use per device, with that device current).
int static_scratch_ptr(char** out, int* dev_out = nullptr) {
    int dev = -1;
    HR_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return HR_ERR_DEVICE;
    std::lock_guard<std::mutex> lock(g_scratch_mu);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        HR_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(g_static_scratch)));
        if (!p || (uintptr_t)p % kAlign != 0) return HR_ERR_DEVICE;
        g_scratch_ptr[dev] = (char*)p;
    }
    *out = g_scratch_ptr[dev];
    if (dev_out) *dev_out = dev;
    return HR_OK;
}

// How many leading layers of a scoring pass run with split (hi + lo) operands unless the caller says otherwise.
// Measured on random-initialised models against the float64 definition: 16-bit operands leave a score error of rms
// 0.002 at 24 layers x 896 hidden and 0.007 at 32 layers x 4096 hidden (scores ~ N(0, 1.8^2)), of which the first
// layer's roundings alone account for 80 % and the first two for 94 % at the larger shape.  Two split layers bring that
// shape to rms 0.002 for 1/16 more projection work; the smaller shape is left as it is.
int default_precise_layers(const hr_model_cfg& c, bool mfma) {
    if (!mfma) return 0;
    return (int64_t)c.n_layers * c.hidden >= 65536 ? std::min(2, c.n_layers) : 0;
}

const void* layer_w(const hr_model* m, int l, size_t off) {
    size_t esz = dtype_size(m->cfg.dtype);
    return m->pack_base + ((size_t)l * m->pack.layer_elems + off) * esz;
}

constexpr size_t kStageMinInts = (size_t)1 << 18;      // staging a model handle starts with (1 MiB of pinned host memory)

int stage_reserve(hr_model* m, size_t ints, bool may_grow = true) {
    if (m->stage_pending) {
        HR_HIP(hipEventSynchronize(m->stage_ev));
        m->stage_pending = false;
    }
    if (ints > m->stage_ints) {
        if (!may_grow) {
            snprintf(g_last_error, sizeof(g_last_error), "metadata of this call (%zu bytes) exceeds the handle's staging buffer (%zu bytes)",
                     ints * sizeof(int32_t), m->stage_ints * sizeof(int32_t));
            return HR_ERR_WORKSPACE_SMALL;
        }
        if (m->stage) (void)hipHostFree(m->stage);
        m->stage = nullptr;
        m->stage_ints = 0;
        size_t want = std::max(ints, kStageMinInts);
        HR_HIP(hipHostMalloc((void**)&m->stage, want * sizeof(int32_t), hipHostMallocDefault));
        m->stage_ints = want;
    }
    if (!m->stage_ev) HR_HIP(hipEventCreateWithFlags(&m->stage_ev, hipEventDisableTiming));
    return HR_OK;
}

enum ProfClass { PC_EMBED = 0, PC_RMSNORM, PC_GEMM_QKV, PC_ATTENTION, PC_GEMM_O, PC_GEMM_GATE_UP, PC_GEMM_DOWN, PC_SCORE_HEAD,
                 PC_ELEMENTWISE, PC_COUNT };
const char* const kProfNames[PC_COUNT] = {"embed_rope_table", "rmsnorm", "gemm_qkv", "attention", "gemm_o", "gemm_gate_up",
                                          "gemm_down", "score_head", "elementwise"};

struct ProfScope {
    hr_model* m;
    hipStream_t st;
    bool on;
    ProfScope(hr_model* m_, int cls, hipStream_t st_) : m(m_), st(st_), on(m_->prof_on && ((m_->prof_mask >> cls) & 1u)) {
        if (!on) return;
        if (m->prof_used + 2 > m->prof_events.size()) {
            for (int i = 0; i < 64; ++i) {
                hipEvent_t e;
                if (hipEventCreate(&e) != hipSuccess) { on = false; return; }
                m->prof_events.push_back(e);
            }
        }
        m->prof_class.push_back(cls);
        (void)hipEventRecord(m->prof_events[m->prof_used], st);
    }
    ~ProfScope() {
        if (!on) return;
        (void)hipEventRecord(m->prof_events[m->prof_used + 1], st);
        m->prof_used += 2;
    }
};
#define HR_TIMED(cls, expr)              \
    do {                                 \
        ProfScope scope__(m, cls, st);   \
        HR_HIP(expr);                    \
    } while (0)

// One pass of all layers over the T new tokens described by `mv`, scores for every sequence.
// Where a prefill pass stores each layer's K/V: pool page dst_page[i] <- new-KV page src_page[i] (device arrays)
struct PrefillTarget {
    hr_pool* pool;
    const int32_t* src_page;
    const int32_t* dst_page;
    int n_pages;
};

// One pass of all layers over the T new tokens described by `mv`.
//   pool         cached-document pool (scoring pass), or nullptr
//   self_prefix  the sequences are chunks of longer sequences whose earlier tokens are found as pages of this call's
//                own new-KV buffer (no-reuse pass, document prefill)
//   fill         if set, every layer's K/V pages are copied into that pool and the pass stops after the last
//                layer's K/V (no scores)
//   groups       if set, the attention work items are these groups of sequences with one shared document
//   after_qkv0   if set, recorded on `st` behind the first layer's QKV projection
int run_layers(hr_model* m, const hr_pool* pool, bool self_prefix, const MetaView& mv, const Workspace& ws, char* wsb,
               int max_keys, int max_new_len, float* scores, hipStream_t st, const PrefillTarget* fill = nullptr,
               const GroupView* groups = nullptr, hipEvent_t after_qkv0 = nullptr, int n_precise = 0) {
    const hr_model_cfg& c = m->cfg;
    const int dt = c.dtype;
    const int H = c.hidden, d = c.head_dim, F = c.ffn;
    const int nq = c.n_q_heads * d, nkv = c.n_kv_heads * d, nqkv = nq + 2 * nkv;
    float* x = (float*)(wsb + ws.off_x);
    void* y = wsb + ws.off_y;
    void* q = wsb + ws.off_q;
    void* k = wsb + ws.off_k;
    void* v = wsb + ws.off_v;
    void* o = wsb + ws.off_o;
    void* mm = wsb + ws.off_m;
    float* f32 = (float*)(wsb + ws.off_f32);
    float2* rope = (float2*)(wsb + ws.off_rope);
    const int64_t T = mv.T;

    PoolView pv{};
    pv.n_kv = c.n_kv_heads;
    pv.d = d;
    if (pool) {
        pv.data = pool->base;
        pv.scales = pool->cfg.kv_dtype == HR_FP8_E4M3 ? (const float*)(pool->base + pool->lay.data_bytes) : nullptr;
        pv.num_pages = pool->cfg.num_pages;
        pv.kv_dtype = pool->cfg.kv_dtype;
        pv.esz = pool->lay.esz;
    } else {
        pv.kv_dtype = dt;
        pv.esz = dtype_size(dt);
        pv.num_pages = 1;
        if (self_prefix) pv.data = (const char*)k;     // layer index 0 of a one-layer "pool" = the new-KV page buffer
    }
    const bool mfma_attn = use_mfma_attn(m, pv.kv_dtype, max_new_len, groups && groups->n_groups > 0);
    if (self_prefix && !mfma_attn) return HR_ERR_UNSUPPORTED_SHAPE;
    if (!mfma_attn && max_keys > kGenericMaxKeys) return HR_ERR_UNSUPPORTED_SHAPE;     // the generic attention keeps a row's scores in LDS
    // the shortened last layer needs one output row per sequence, the MFMA kernels, something to save (T > P), and
    // room for P fp32 rows in the q buffer
    // Layers l < n_prec run with 22-bit operands: every activation that feeds an MFMA (the normalised rows, q, the new
    // tokens' K/V, the probabilities, the attention output, the SwiGLU output) is carried as a pair of halves hi + lo and
    // each product with a lo term is one more MFMA chain into the same fp32 accumulator; weights and cached document K/V
    // are exact as stored.  A 16-bit operand's rounding in the first layers is what dominates the score error of a
    // deep, wide model (the residual stream is still small there, and everything downstream amplifies it).
    const int n_prec = (mfma_attn && m->mfma_gemm && pool && !fill && !self_prefix) ? std::min(n_precise, c.n_layers) : 0;
    void* kvlo = wsb + ws.off_kvlo;
    const bool share0 = mfma_attn && m->mfma_gemm && pool && !fill && !self_prefix && mv.tok_src && mv.n_uniq > 0;
    const bool last_short = !m->no_last_short && mfma_attn && m->mfma_gemm && !fill && !self_prefix && mv.n_out == mv.n_seq &&
                            T > mv.n_seq && (size_t)T * nq * dtype_size(dt) >= (size_t)mv.n_seq * H * sizeof(float) && H % 4 == 0 &&
                            n_prec < c.n_layers;

    // with the MFMA attention the new tokens' K/V are written straight into 16-slot pages (k and v regions together);
    // slots past a sequence's end are never written by any layer, so one clear per call keeps them finite
    const size_t kv_region = ws.off_o - ws.off_k;
    if (mfma_attn) HR_TIMED(PC_EMBED, launch_fill_zero(k, kv_region, st));
    HR_TIMED(PC_EMBED, launch_embed(dt, m->embedding, mv, x, H, st));
    HR_TIMED(PC_EMBED, launch_rope_table(mv, rope, d, c.rope_base, st));
    for (int l = 0; l < c.n_layers; ++l) {
        // First layer, several sequences with the same token string (one query against its candidates): the normalised
        // rows and the pre-RoPE q / k / v of equal strings are equal, so they are computed on the distinct rows only and
        // every token takes its row, rotated for its own position (exact: same bits as computing every row).
        const bool shared0 = l == 0 && share0;
        const int64_t Tq = shared0 ? mv.n_uniq : T;                   // rows of this layer's first norm and QKV projection
        const int32_t* rows0 = shared0 ? mv.rep_row : nullptr;
        const int32_t* src0 = shared0 ? mv.tok_src : nullptr;
        if (l < n_prec) {
            HR_TIMED(PC_RMSNORM, launch_rmsnorm_split(x, m->norm1[l], y, Tq, H, c.rms_eps, st, rows0));
            // the projection leaves fp32 rows (x += C on a cleared buffer); RoPE, the hi / lo split and the page scatter
            // are a kernel of their own
            HR_TIMED(PC_ELEMENTWISE, launch_fill_zero(f32, (size_t)Tq * nqkv * sizeof(float), st));
            GemmArgs a{};
            a.A = y; a.W = layer_w(m, l, m->pack.wqkv); a.M = Tq; a.N = nqkv; a.K = 2 * H; a.Kw = H; a.x = f32;
            HR_TIMED(PC_GEMM_QKV, launch_gemm_mfma(EPI_RESID_ADD, a, st));
            HR_TIMED(PC_ELEMENTWISE, launch_rope_pages(f32, rope, q, k, kvlo, mv.new_slot, src0, T, c.n_q_heads, c.n_kv_heads, d, st));
            if (l == 0 && after_qkv0) HR_HIP(hipEventRecord(after_qkv0, st));
            HR_TIMED(PC_ATTENTION, launch_attn_mfma(q, k, o, mv, pv, l, c.n_q_heads, max_new_len, st, false, groups, kvlo));
            GemmArgs b{};
            b.A = o; b.W = layer_w(m, l, m->pack.wo); b.M = T; b.N = H; b.K = 2 * nq; b.Kw = nq; b.x = x;
            HR_TIMED(PC_GEMM_O, launch_gemm_mfma(EPI_RESID_ADD, b, st));
            HR_TIMED(PC_RMSNORM, launch_rmsnorm_split(x, m->norm2[l], y, T, H, c.rms_eps, st));
            GemmArgs gu{};
            gu.A = y; gu.W = layer_w(m, l, m->pack.wgu); gu.M = T; gu.N = 2 * F; gu.K = 2 * H; gu.Kw = H; gu.out0 = mm; gu.split_out = 1;
            HR_TIMED(PC_GEMM_GATE_UP, launch_gemm_mfma(EPI_SWIGLU, gu, st));
            GemmArgs dn{};
            dn.A = mm; dn.W = layer_w(m, l, m->pack.wd); dn.M = T; dn.N = H; dn.K = 2 * F; dn.Kw = F; dn.x = x;
            HR_TIMED(PC_GEMM_DOWN, launch_gemm_mfma(EPI_RESID_ADD, dn, st));
            continue;
        }
        HR_TIMED(PC_RMSNORM, launch_rmsnorm(dt, x, m->norm1[l], y, Tq, H, c.rms_eps, st, rows0));
        if (shared0) {
            HR_TIMED(PC_ELEMENTWISE, launch_fill_zero(f32, (size_t)Tq * nqkv * sizeof(float), st));
            GemmArgs a{};
            a.A = y; a.W = layer_w(m, l, m->pack.wqkv); a.M = Tq; a.N = nqkv; a.K = H; a.x = f32;
            HR_TIMED(PC_GEMM_QKV, launch_gemm_mfma(EPI_RESID_ADD, a, st));
            HR_TIMED(PC_ELEMENTWISE, launch_rope_pages(f32, rope, q, k, nullptr, mv.new_slot, src0, T, c.n_q_heads, c.n_kv_heads, d, st));
        } else if (m->mfma_gemm) {
            GemmArgs a{};
            a.A = y; a.W = layer_w(m, l, m->pack.wqkv); a.M = T; a.N = nqkv; a.K = H;
            a.out0 = q; a.out1 = k; a.out2 = v; a.rope = rope; a.n_q = c.n_q_heads; a.n_kv = c.n_kv_heads; a.d = d;
            if (mfma_attn) { a.kv_pages = k; a.new_slot = mv.new_slot; }
            HR_TIMED(PC_GEMM_QKV, launch_gemm_mfma(EPI_QKV_ROPE, a, st));
        } else {
            HR_TIMED(PC_GEMM_QKV, launch_gemm_generic(dt, y, layer_w(m, l, m->pack.wqkv), f32, T, nqkv, H, false, st));
            HR_TIMED(PC_ELEMENTWISE, launch_rope_split(dt, f32, rope, q, k, v, T, c.n_q_heads, c.n_kv_heads, d, st));
        }
        if (l == 0 && after_qkv0) HR_HIP(hipEventRecord(after_qkv0, st));
        if (fill) {
            // this layer's K/V pages are final: store them, and stop once the last layer's are in
            const hr_pool* fp = fill->pool;
            const size_t pages_all_heads = (size_t)l * fp->cfg.num_pages * c.n_kv_heads;
            if (fp->cfg.kv_dtype == HR_FP8_E4M3) {
                float* scales = (float*)(fp->base + fp->lay.data_bytes) + pages_all_heads * 2;
                HR_TIMED(PC_ELEMENTWISE, launch_pages_to_pool_fp8((const char*)k, fp->base + pages_all_heads * 2 * kPageTokens * d, scales,
                                                                  fill->src_page, fill->dst_page, fill->n_pages, c.n_kv_heads, d, st));
            } else {
                HR_TIMED(PC_ELEMENTWISE, launch_pages_to_pool((const char*)k, fp->base + pages_all_heads * 2 * kPageTokens * d * 2,
                                                              fill->src_page, fill->dst_page, fill->n_pages,
                                                              c.n_kv_heads * 2 * kPageTokens * d * 2, st));
            }
            if (l + 1 == c.n_layers) return HR_OK;
        }
        if (last_short && l + 1 == c.n_layers) {
            // Last layer, scoring pass: only each pair's last token feeds the score, so attention runs g rows per
            // (pair, kv head) into a compact [P][n_q][d] buffer and the rest of the layer runs on P rows instead
            // of T (exact: the other rows' outputs of this layer are never read).
            const int64_t P = mv.n_seq;
            float* x_last = (float*)q;                      // q is dead once attention has run
            HR_TIMED(PC_ATTENTION, launch_attn_mfma(q, k, o, mv, pv, l, c.n_q_heads, max_new_len, st, true));
            HR_TIMED(PC_ELEMENTWISE, launch_gather_rows_f32(x, mv.out_row, x_last, (int)P, H, st));
            GemmArgs a{};
            a.A = o; a.W = layer_w(m, l, m->pack.wo); a.M = P; a.N = H; a.K = nq; a.x = x_last;
            HR_TIMED(PC_GEMM_O, launch_gemm_mfma(EPI_RESID_ADD, a, st));
            HR_TIMED(PC_RMSNORM, launch_rmsnorm(dt, x_last, m->norm2[l], y, P, H, c.rms_eps, st));
            GemmArgs gu{};
            gu.A = y; gu.W = layer_w(m, l, m->pack.wgu); gu.M = P; gu.N = 2 * F; gu.K = H; gu.out0 = mm;
            HR_TIMED(PC_GEMM_GATE_UP, launch_gemm_mfma(EPI_SWIGLU, gu, st));
            GemmArgs b{};
            b.A = mm; b.W = layer_w(m, l, m->pack.wd); b.M = P; b.N = H; b.K = F; b.x = x_last;
            HR_TIMED(PC_GEMM_DOWN, launch_gemm_mfma(EPI_RESID_ADD, b, st));
            MetaView compact = mv;
            compact.out_row = nullptr;                      // row p of x_last belongs to pair p
            HR_TIMED(PC_SCORE_HEAD, launch_score_head(dt, x_last, m->final_norm, m->embedding, compact, scores, H, c.rms_eps, c.yes_id,
                                                      c.no_id, st));
            return HR_OK;
        }
        if (mfma_attn) {
            HR_TIMED(PC_ATTENTION, launch_attn_mfma(q, k, o, mv, pv, self_prefix ? 0 : l, c.n_q_heads, max_new_len, st, false, groups));
        } else {
            HR_TIMED(PC_ATTENTION, launch_attn_generic(dt, q, k, v, o, mv, pv, l, c.n_q_heads, max_keys, st));
        }
        if (m->mfma_gemm) {
            GemmArgs a{};
            a.A = o; a.W = layer_w(m, l, m->pack.wo); a.M = T; a.N = H; a.K = nq; a.x = x;
            HR_TIMED(PC_GEMM_O, launch_gemm_mfma(EPI_RESID_ADD, a, st));
        } else {
            HR_TIMED(PC_GEMM_O, launch_gemm_generic(dt, o, layer_w(m, l, m->pack.wo), x, T, H, nq, true, st));
        }
        HR_TIMED(PC_RMSNORM, launch_rmsnorm(dt, x, m->norm2[l], y, T, H, c.rms_eps, st));
        if (m->mfma_gemm) {
            GemmArgs a{};
            a.A = y; a.W = layer_w(m, l, m->pack.wgu); a.M = T; a.N = 2 * F; a.K = H; a.out0 = mm;
            HR_TIMED(PC_GEMM_GATE_UP, launch_gemm_mfma(EPI_SWIGLU, a, st));
            GemmArgs b{};
            b.A = mm; b.W = layer_w(m, l, m->pack.wd); b.M = T; b.N = H; b.K = F; b.x = x;
            HR_TIMED(PC_GEMM_DOWN, launch_gemm_mfma(EPI_RESID_ADD, b, st));
        } else {
            HR_TIMED(PC_GEMM_GATE_UP, launch_gemm_generic(dt, y, layer_w(m, l, m->pack.wgu), f32, T, 2 * F, H, false, st));
            HR_TIMED(PC_ELEMENTWISE, launch_swiglu(dt, f32, mm, T, F, m->pack.gu_interleave, st));
            HR_TIMED(PC_GEMM_DOWN, launch_gemm_generic(dt, mm, layer_w(m, l, m->pack.wd), x, T, H, F, true, st));
        }
    }
    HR_TIMED(PC_SCORE_HEAD, launch_score_head(dt, x, m->final_norm, m->embedding, mv, scores, H, c.rms_eps, c.yes_id, c.no_id, st));
    return HR_OK;
}

MetaView make_meta_view(const int32_t* dev_meta, const MetaLayout& ml, int64_t n_seq, int64_t T, int64_t pt_stride) {
    MetaView mv{};
    mv.cu = dev_meta + ml.cu;
    mv.tok_id = dev_meta + ml.tok_id;
    mv.tok_pos = dev_meta + ml.tok_pos;
    mv.tok_seq = dev_meta + ml.tok_seq;
    mv.prefix_len = dev_meta + ml.prefix_len;
    mv.page_table = dev_meta + ml.page_table;
    mv.new_slot = dev_meta + ml.new_slot;
    mv.new_cu = dev_meta + ml.new_cu;
    mv.out_row = dev_meta + ml.out_row;
    mv.n_out = (int32_t)n_seq;
    mv.pt_stride = (int32_t)pt_stride;
    mv.n_seq = (int32_t)n_seq;
    mv.T = T;
    return mv;
}

// chunk length of the self-prefix passes: as many query rows per kv head as the attention kernel takes
int full_chunk(const hr_model* m) {
    const int g = m->cfg.n_q_heads / m->cfg.n_kv_heads;
    return g * 64 <= 512 ? 64 : 32;
}

bool chunked_ok(const hr_model* m) {
    return !m->force_generic && m->mfma_gemm && hr::attn_mfma_supported(m->cfg, HR_BF16, full_chunk(m));
}

}  // namespace

extern "C" {

int hr_weights_load(const hr_model_cfg* cfg, const hr_weight_ptrs* w, void* pack_dev, size_t pack_bytes, void* stream,
                    hr_model** out) {
    if (!out) return HR_ERR_INVALID_ARG;
    *out = nullptr;
    if (!hr::model_cfg_valid(cfg) || !w || !pack_dev) return HR_ERR_INVALID_ARG;
    if ((uintptr_t)pack_dev % hr::kAlign != 0) return HR_ERR_INVALID_ARG;
    if (!w->embedding || !w->final_norm || !w->wq || !w->wk || !w->wv || !w->wo || !w->wg || !w->wu || !w->wd || !w->norm1 ||
        !w->norm2)
        return HR_ERR_INVALID_ARG;
    for (int l = 0; l < cfg->n_layers; ++l)
        if (!w->wq[l] || !w->wk[l] || !w->wv[l] || !w->wo[l] || !w->wg[l] || !w->wu[l] || !w->wd[l] || !w->norm1[l] ||
            !w->norm2[l])
            return HR_ERR_INVALID_ARG;
    hr::PackLayout pl = hr::make_pack_layout(*cfg);
    if (pack_bytes < pl.total_bytes) return HR_ERR_WORKSPACE_SMALL;

    hr_model* m = new (std::nothrow) hr_model();
    if (!m) return HR_ERR_INVALID_ARG;
    m->cfg = *cfg;
    m->pack = pl;
    m->pack_base = (const char*)pack_dev;
    m->embedding = w->embedding;
    m->final_norm = w->final_norm;
    m->norm1.assign(w->norm1, w->norm1 + cfg->n_layers);
    m->norm2.assign(w->norm2, w->norm2 + cfg->n_layers);
    const char* force = getenv("HR_FORCE_GENERIC");      // A/B switch for tests and benchmarks
    m->force_generic = force && force[0] == '1';
    m->mfma_gemm = !m->force_generic && hr::gemm_mfma_supported(*cfg);
    const char* nls = getenv("HR_NO_LAST_SHORTCUT");
    m->no_last_short = nls && nls[0] == '1';
    const char* ndg = getenv("HR_NO_DOC_GROUPS");
    m->no_doc_groups = ndg && ndg[0] == '1';
    const char* nqs = getenv("HR_NO_QUERY_SHARING");
    m->no_query_share = nqs && nqs[0] == '1';
    const char* ns = getenv("HR_STREAMS");               // "1": scoring calls stay on the caller's stream (profiling runs)
    if (ns && ns[0] == '1') m->n_streams = 1;
    m->n_precise = default_precise_layers(*cfg, m->mfma_gemm);
    const char* npl = getenv("HR_PRECISE_LAYERS");       // A/B runs: overrides the default number of split-operand layers
    if (npl && npl[0] >= '0' && npl[0] <= '9' && m->mfma_gemm) m->n_precise = std::min(atoi(npl), cfg->n_layers);

    // set-up that later calls must not have to do: the address of the static scratch on this device, the pinned
    // staging buffer for per-call metadata and its event
    {
        char* scratch = nullptr;
        int rc = static_scratch_ptr(&scratch, &m->device);
        if (rc == HR_OK) rc = stage_reserve(m, kStageMinInts);
        if (rc != HR_OK) {
            hr_model_destroy(m);
            return rc;
        }
    }

    hipStream_t st = (hipStream_t)stream;
    const int dt = cfg->dtype;
    const size_t esz = hr::dtype_size(dt);
    const int H = cfg->hidden, d = cfg->head_dim, F = cfg->ffn;
    const int nq = cfg->n_q_heads * d, nkv = cfg->n_kv_heads * d;
    long long* rc = (long long*)((char*)pack_dev + pl.counter_off);      // what the conversion to half meets (hr_model_range_report)
    {
        hipError_t e = hr::launch_fill_zero(rc, hr::kRangeCounterBytes, st);
        if (e != hipSuccess) {
            note_hip_error(e, "counter fill kernel");
            hr_model_destroy(m);
            return HR_ERR_DEVICE;
        }
    }
    for (int l = 0; l < cfg->n_layers; ++l) {
        char* slab = (char*)pack_dev + (size_t)l * pl.layer_elems * esz;
        char* wqkv = slab + pl.wqkv * esz;
        hipError_t e = hr::launch_pack_rows(dt, w->wq[l], wqkv, nq, H, nq, 1, 0, rc, st);
        if (e == hipSuccess) e = hr::launch_pack_rows(dt, w->wk[l], wqkv + (size_t)nq * H * esz, nkv, H, nkv, 1, 0, rc, st);
        if (e == hipSuccess) e = hr::launch_pack_rows(dt, w->wv[l], wqkv + (size_t)(nq + nkv) * H * esz, nkv, H, nkv, 1, 0, rc, st);
        if (e == hipSuccess) e = hr::launch_pack_rows(dt, w->wo[l], slab + pl.wo * esz, H, nq, H, 1, 0, rc, st);
        if (e == hipSuccess) e = hr::launch_pack_rows(dt, w->wg[l], slab + pl.wgu * esz, F, H, pl.gu_interleave, 2, 0, rc, st);
        if (e == hipSuccess) e = hr::launch_pack_rows(dt, w->wu[l], slab + pl.wgu * esz, F, H, pl.gu_interleave, 2, 1, rc, st);
        if (e == hipSuccess) e = hr::launch_pack_rows(dt, w->wd[l], slab + pl.wd * esz, H, F, H, 1, 0, rc, st);
        if (e != hipSuccess) {
            note_hip_error(e, "weight packing kernels");
            hr_model_destroy(m);
            return HR_ERR_DEVICE;
        }
    }
    *out = m;
    return HR_OK;
}

void hr_model_destroy(hr_model* m) {
    if (!m) return;
    if (m->stage_pending) (void)hipEventSynchronize(m->stage_ev);
    if (m->stage_ev) (void)hipEventDestroy(m->stage_ev);
    if (m->aux_stream) {
        (void)hipStreamSynchronize(m->aux_stream);
        (void)hipStreamDestroy(m->aux_stream);
    }
    if (m->fork_ev) (void)hipEventDestroy(m->fork_ev);
    if (m->join_ev) (void)hipEventDestroy(m->join_ev);
    if (m->stage) (void)hipHostFree(m->stage);
    for (hipEvent_t e : m->prof_events) (void)hipEventDestroy(e);
    delete m;
}

int hr_doc_kv_write(hr_pool* pool, int32_t doc_len, const int32_t* page_ids, const void* k_dev, const void* v_dev,
                    const float* ks, const float* vs, void* stream) {
    int rc = hr::pool_check_write(pool, doc_len, page_ids);
    if (rc != HR_OK) return rc;
    if (!k_dev || !v_dev) return HR_ERR_INVALID_ARG;
    bool fp8 = pool->cfg.kv_dtype == HR_FP8_E4M3;
    if (fp8 && (!ks || !vs)) return HR_ERR_INVALID_ARG;
    long long* counters = (long long*)(pool->base + pool->lay.counter_off);
    hipError_t e = hipSuccess;
    if (!pool->counters_zeroed) {
        e = hr::launch_fill_zero(counters, hr::kRangeCounterBytes, (hipStream_t)stream);
        pool->counters_zeroed = e == hipSuccess;
    }
    if (e == hipSuccess)
        e = hr::launch_kv_scatter(pool->lay, pool->base, page_ids, doc_len, k_dev, v_dev, ks, vs, counters, (hipStream_t)stream);
    if (e != hipSuccess) {
        note_hip_error(e, "pool scatter kernel");
        return HR_ERR_DEVICE;
    }
    hr::pool_mark(pool, page_ids, (doc_len + hr::kPageTokens - 1) / hr::kPageTokens, hr::PAGE_USED);
    return HR_OK;
}

int hr_doc_kv_read(const hr_pool* pool, int32_t doc_len, const int32_t* page_ids, void* k_dev, void* v_dev, float* ks, float* vs,
                   void* stream) {
    int rc = hr::pool_check_read(pool, doc_len, page_ids);
    if (rc != HR_OK) return rc;
    if (!k_dev || !v_dev) return HR_ERR_INVALID_ARG;
    if (pool->cfg.kv_dtype == HR_FP8_E4M3 && (!ks || !vs)) return HR_ERR_INVALID_ARG;
    hipError_t e = hr::launch_kv_gather(pool->lay, pool->base, page_ids, doc_len, k_dev, v_dev, ks, vs, (hipStream_t)stream);
    if (e != hipSuccess) {
        note_hip_error(e, "pool gather kernel");
        return HR_ERR_DEVICE;
    }
    return HR_OK;
}

// Address the GPU uses for caller memory that must be device memory or host memory pinned by the runtime; nullptr for
// anything else (pageable host memory would fault in a kernel).
static char* device_view(const void* p) {
    hipPointerAttribute_t attr;
    if (hipPointerGetAttributes(&attr, p) != hipSuccess) {
        (void)hipGetLastError();
        return nullptr;
    }
    if (attr.type != hipMemoryTypeDevice && attr.type != hipMemoryTypeHost) return nullptr;
    return (char*)attr.devicePointer;
}

static int pages_move(hr_pool* pool, int32_t n_pages, const int32_t* page_ids, const void* records, bool to_pool, void* stream,
                      bool four_bit = false) {
    int rc = hr::pool_check_pages(pool, n_pages, page_ids, !to_pool);
    if (rc != HR_OK) return rc;
    if (four_bit && hr::page_record4_bytes(pool->lay) == 0) return HR_ERR_UNSUPPORTED_SHAPE;
    if (n_pages == 0) return HR_OK;
    if (!records || (uintptr_t)records % 16 != 0) return HR_ERR_INVALID_ARG;
    char* rec = device_view(records);
    if (!rec || (uintptr_t)rec % 16 != 0) {
        snprintf(g_last_error, sizeof(g_last_error), "page records must be device memory or host memory pinned by the HIP runtime");
        return HR_ERR_INVALID_ARG;
    }
    hipError_t e = four_bit ? hr::launch_pages_move4(pool->lay, pool->base, page_ids, n_pages, rec, to_pool, (hipStream_t)stream)
                            : hr::launch_pages_move(pool->lay, pool->base, page_ids, n_pages, rec, to_pool, (hipStream_t)stream);
    if (e != hipSuccess) {
        note_hip_error(e, "page move kernel");
        return HR_ERR_DEVICE;
    }
    if (to_pool) hr::pool_mark(pool, page_ids, n_pages, hr::PAGE_USED);
    return HR_OK;
}

int hr_kv_pages_out(const hr_pool* pool, int32_t n_pages, const int32_t* page_ids, void* dst, void* stream) {
    return pages_move(const_cast<hr_pool*>(pool), n_pages, page_ids, dst, false, stream);
}

int hr_kv_pages_in(hr_pool* pool, int32_t n_pages, const int32_t* page_ids, const void* src, void* stream) {
    return pages_move(pool, n_pages, page_ids, src, true, stream);
}

int hr_kv_pages_out4(const hr_pool* pool, int32_t n_pages, const int32_t* page_ids, void* dst, void* stream) {
    return pages_move(const_cast<hr_pool*>(pool), n_pages, page_ids, dst, false, stream, true);
}

int hr_kv_pages_in4(hr_pool* pool, int32_t n_pages, const int32_t* page_ids, const void* src, void* stream) {
    return pages_move(pool, n_pages, page_ids, src, true, stream, true);
}

size_t hr_rerank_workspace_bytes(const hr_model* m, int32_t n_pairs, int64_t total_q_tokens, int32_t pt_stride) {
    if (!m || n_pairs < 0 || total_q_tokens < 0 || pt_stride < 0) return 0;
    // + room for the per-part alignment when the call runs as two halves (each with its own carving)
    return hr::make_workspace(m->cfg, n_pairs, total_q_tokens, pt_stride, !m->mfma_gemm, -1, 0,
                              (int64_t)hr::group_plan_ints_bound(n_pairs, total_q_tokens, m->cfg.n_q_heads / m->cfg.n_kv_heads),
                              m->n_precise > 0, m->mfma_gemm)
               .total + (m->mfma_gemm ? kSplitSlackBytes : 0);
}

// Whether a scoring call of T query tokens is cut in two halves (given the MFMA attention and at least two pairs): when
// the tiles of the N = hidden GEMMs would leave more than 15 % of the workgroup slots of their rounds empty.
static bool split_wanted(const hr_model* m, int64_t T) {
    return m->n_streams >= 2 && m->mfma_gemm && T >= kSplitMinTokens && hr::gemm_resid_fill(T, m->cfg.hidden) < kSplitMaxFill;
}

// One contiguous part of a scoring call.  prepare: its metadata (already validated) is built at `stage` and its upload to the
// head of `wsb` is enqueued on `st`; run: the layers are enqueued (on any stream ordered behind the upload).  ws / ml are
// the part's own carving.
struct ScorePart {
    hr::MetaView mv{};
    hr::GroupView gv{};
    int max_keys = 0;
};

// Builds a part's metadata (already validated) at `stage`: the token / position / slot tables, the page table, and the
// two content-dependent plans: pairs that share a document (one attention work item per kv head) and pairs that share
// a query string (first-layer rows computed once).  content_plans = false leaves both out, so that the layout of the
// work depends on the lengths alone (fixed-shape plans, whose launches are recorded once and replayed with other
// tokens and pages).  *upload_ints = how much of the block the device needs.
static void build_score_part(hr_model* m, int32_t n_pairs, const int32_t* page_table, int32_t pt_stride, const int32_t* doc_lens,
                             const int32_t* query_tokens, const int32_t* query_lens, int64_t T, bool mfma_attn, const hr::Workspace& ws,
                             const hr::MetaLayout& ml, int64_t grp_ints, int32_t* stage, char* wsb, bool content_plans, ScorePart* out,
                             size_t* upload_ints) {
    hr::fill_meta(stage, ml, n_pairs, doc_lens, query_lens, query_tokens, page_table, pt_stride);
    // Pairs that share a document become one attention work item per kv head (up to 16 row blocks at 64-wide heads,
    // 8 at 128-wide heads, where two blocks per wave do not fit the register file at two waves per SIMD).
    const int g = m->cfg.n_q_heads / m->cfg.n_kv_heads;
    hr::GroupView& gv = out->gv;
    size_t plan_ints = 0;                                    // of the room reserved for a plan, what this call uses
    int max_q = 0;
    for (int32_t p = 0; p < n_pairs; ++p) max_q = std::max(max_q, query_lens[p]);
    const int64_t blocks_max = ((int64_t)g * max_q + 31) / 32;           // row blocks of the longest query, per kv head
    const int cap_full = m->cfg.head_dim == 64 ? 16 : 8;                 // what one work item holds
    if (mfma_attn && !m->no_doc_groups && (pt_stride > 0 || blocks_max > cap_full)) {
        // few work items (less than half the CUs would get one): a pair's row blocks are spread over several work items
        // of at most four, one per wave of the smallest kernel, each streaming the document for its share of the rows
        const bool scarce = n_pairs <= hr::kGroupCutMaxSeqs && (int64_t)n_pairs * m->cfg.n_kv_heads * 2 <= hr::device_cu_count() &&
                            blocks_max <= 4 * hr::kMaxPiecesPerSeq;
        const int cap = scarce ? 4 : cap_full;
        // 128-wide heads: a pair with more than 8 row blocks is cut in two work items as well.  Two blocks per wave do not
        // fit the registers there (the kernel for 9-16 blocks spills), and two items that each stream the document run
        // the 512-row shape 1.8 times faster (measured at the 8B shape, 128-token queries; same bits).
        // Queries of more rows than any work item holds are cut the same way (use_mfma_attn has checked that
        // kMaxPiecesPerSeq pieces are enough, and the room reserved for a plan covers that many).
        const bool cut_long = scarce || m->cfg.head_dim == 128 || blocks_max > cap_full;
        const hr::GroupPlan plan = hr::make_group_plan(n_pairs, doc_lens, query_lens, content_plans ? page_table : nullptr, pt_stride, g,
                                                       cap, cut_long);
        // also without a shared document when the pairs differ in length: the plan's heaviest-first order keeps the
        // persistent workgroups' last items short
        if ((plan.shared || plan.uneven || plan.cut) && plan.ints() <= (size_t)grp_ints) {
            hr::store_group_plan(plan, stage + ml.grp);
            plan_ints = plan.ints();
            const int32_t* dv = (const int32_t*)(wsb + ws.off_meta) + ml.grp;
            gv.n_groups = plan.n_groups;
            gv.max_blocks = plan.max_blocks;
            gv.p0 = dv;                              dv += plan.p0.size();
            gv.blk_cu = dv;                          dv += plan.blk_cu.size();
            gv.sub_cu = dv;                          dv += plan.sub_cu.size();
            gv.blk_seq = dv;                         dv += plan.blk_seq.size();
            gv.blk_row0 = dv;                        dv += plan.blk_row0.size();
            gv.sub_page = dv;                        dv += plan.sub_page.size();
            gv.sub_seq = dv;                         dv += plan.sub_seq.size();
            gv.sub_key0 = dv;
        }
    }
    // sequences with the same token string share the first layer's normalised rows and projections, where that at least
    // halves the rows (the shared rows take the y and fp32 buffers)
    int64_t n_uniq = 0;
    if (content_plans && mfma_attn && !m->no_query_share && ml.rep_row > ml.tok_src && n_pairs >= 2) {
        const hr::QueryShare qs = hr::make_query_share(n_pairs, query_lens, query_tokens);
        if (qs.n_uniq * 2 <= T) {
            std::memcpy(stage + ml.tok_src, qs.tok_src.data(), sizeof(int32_t) * qs.tok_src.size());
            std::memcpy(stage + ml.rep_row, qs.rep_row.data(), sizeof(int32_t) * qs.rep_row.size());
            n_uniq = qs.n_uniq;
        }
    }
    out->max_keys = 0;
    for (int32_t p = 0; p < n_pairs; ++p) out->max_keys = std::max(out->max_keys, doc_lens[p] + query_lens[p]);
    out->mv = make_meta_view((const int32_t*)(wsb + ws.off_meta), ml, n_pairs, T, pt_stride);
    if (n_uniq > 0) {
        out->mv.tok_src = (const int32_t*)(wsb + ws.off_meta) + ml.tok_src;
        out->mv.rep_row = (const int32_t*)(wsb + ws.off_meta) + ml.rep_row;
        out->mv.n_uniq = (int32_t)n_uniq;
    }
    *upload_ints = ml.grp + plan_ints;
}

static int prepare_score_part(hr_model* m, int32_t n_pairs, const int32_t* page_table, int32_t pt_stride, const int32_t* doc_lens,
                              const int32_t* query_tokens, const int32_t* query_lens, int64_t T, bool mfma_attn, const hr::Workspace& ws,
                              const hr::MetaLayout& ml, int64_t grp_ints, int32_t* stage, char* wsb, hipStream_t st, ScorePart* out) {
    size_t upload_ints = 0;
    build_score_part(m, n_pairs, page_table, pt_stride, doc_lens, query_tokens, query_lens, T, mfma_attn, ws, ml, grp_ints, stage, wsb, true,
                     out, &upload_ints);
    HR_HIP(hipMemcpyAsync(wsb + ws.off_meta, stage, upload_ints * sizeof(int32_t), hipMemcpyHostToDevice, st));
    return HR_OK;
}

static int run_score_part(hr_model* m, const hr_pool* pool, const ScorePart& part, const hr::Workspace& ws, char* wsb, int max_q,
                          float* scores_dev, hipStream_t st, hipEvent_t after_qkv0 = nullptr) {
    return run_layers(m, pool, false, part.mv, ws, wsb, part.max_keys, max_q, scores_dev, st, nullptr,
                      part.gv.n_groups > 0 ? &part.gv : nullptr, after_qkv0, m->n_precise);
}

// A scoring call (already validated) in one piece on `st`, with the workspace at `wsb`.
static int score_one_piece(hr_model* m, const hr_pool* pool, int32_t n_pairs, const int32_t* page_table, int32_t pt_stride,
                           const int32_t* doc_lens, const int32_t* query_tokens, const int32_t* query_lens, int64_t T, bool mfma_attn,
                           int max_q, const hr::Workspace& ws, int64_t grp_ints, char* wsb, float* scores_dev, hipStream_t st,
                           bool staging_may_grow) {
    const hr::MetaLayout ml = hr::make_meta_layout(n_pairs, T, pt_stride, -1, 0, grp_ints, m->mfma_gemm);
    int rc = stage_reserve(m, ml.total, staging_may_grow);
    if (rc != HR_OK) return rc;
    ScorePart part;
    rc = prepare_score_part(m, n_pairs, page_table, pt_stride, doc_lens, query_tokens, query_lens, T, mfma_attn, ws, ml, grp_ints,
                            m->stage, wsb, st, &part);
    HR_HIP(hipEventRecord(m->stage_ev, st));
    m->stage_pending = true;
    if (rc != HR_OK) return rc;
    return run_score_part(m, pool, part, ws, wsb, max_q, scores_dev, st);
}

int hr_rerank_score(hr_model* m, const hr_pool* pool, int32_t n_pairs, const int32_t* page_table, int32_t pt_stride,
                    const int32_t* doc_lens, const int32_t* query_tokens, const int32_t* query_lens, void* workspace_dev,
                    size_t workspace_bytes, float* scores_dev, void* stream) {
    if (!m || !pool) return HR_ERR_INVALID_ARG;
    int max_q = 0;
    if (n_pairs > 0 && query_lens)
        for (int32_t p = 0; p < n_pairs; ++p) max_q = std::max(max_q, query_lens[p]);
    const bool mfma_attn = use_mfma_attn(m, pool->cfg.kv_dtype, max_q, true);
    int64_t T = 0;
    int rc = hr::score_check_args(m->cfg, pool, n_pairs, page_table, pt_stride, doc_lens, query_tokens, query_lens,
                                  mfma_attn ? kMfmaMaxKeys : kGenericMaxKeys, &T);
    if (rc != HR_OK) return rc;
    if (n_pairs == 0) return HR_OK;
    if (!workspace_dev || !scores_dev) return HR_ERR_INVALID_ARG;
    if ((uintptr_t)workspace_dev % hr::kAlign != 0) return HR_ERR_INVALID_ARG;
    const int g = m->cfg.n_q_heads / m->cfg.n_kv_heads;
    const int64_t grp_ints = (int64_t)hr::group_plan_ints_bound(n_pairs, T, g);
    const hr::Workspace ws = hr::make_workspace(m->cfg, n_pairs, T, pt_stride, !m->mfma_gemm, -1, 0, grp_ints, m->n_precise > 0, m->mfma_gemm);
    if (workspace_bytes < ws.total) return HR_ERR_WORKSPACE_SMALL;
    hipStream_t st = (hipStream_t)stream;
    char* wsb = (char*)workspace_dev;

    // Two halves on two streams.  A GEMM whose tiles do not divide into full rounds of the chip ends with a round that
    // fills only part of it, and the next kernel of the same stream cannot start before it is over; with the pairs cut in
    // two halves that run on two streams, one half's kernels start on the CUs the other half's last round leaves idle.
    // A pair's arithmetic does not depend on the batch around it, so the scores are bit for bit the same.  Only on the
    // MFMA path, and only when the narrowest GEMMs of a layer (O and down projection, N = hidden) leave a sizeable
    // share of their rounds empty: two kernels that share the chip cost each other a few percent, which the halves
    // must first win back.
    int32_t n_a = n_pairs;
    int64_t T_a = T;
    // Measured, two streams against one, by the fill of those rounds: 0.5B shape 62 % -> -11 %, 78 % -> -5 %, 94 % ->
    // +9 % and -3 %, 100 % -> -0.7 %, -2 %, +2 %; 8B shape 83 % -> -1.5 %, 87 % -> 0, 92 % -> +5.4 %, 94 % -> -1.2 %,
    // +3.8 %, +1 %, 98 % -> +3 %, 100 % -> 0, +3.5 %.
    if (mfma_attn && n_pairs >= 2 && split_wanted(m, T)) {
        int64_t t = 0;
        int32_t p = 0;
        while (p < n_pairs - 1 && t < T / 2) t += query_lens[p++];
        if (p >= 1 && t >= kSplitMinTokens / 4 && T - t >= kSplitMinTokens / 4) {
            n_a = p;
            T_a = t;
        }
    }
    if (n_a < n_pairs) {
        const int32_t n_b = n_pairs - n_a;
        const int64_t T_b = T - T_a;
        const int64_t gi_a = (int64_t)hr::group_plan_ints_bound(n_a, T_a, g), gi_b = (int64_t)hr::group_plan_ints_bound(n_b, T_b, g);
        const hr::Workspace ws_a = hr::make_workspace(m->cfg, n_a, T_a, pt_stride, false, -1, 0, gi_a, m->n_precise > 0, true);
        const hr::Workspace ws_b = hr::make_workspace(m->cfg, n_b, T_b, pt_stride, false, -1, 0, gi_b, m->n_precise > 0, true);
        if (ws_a.total + ws_b.total <= workspace_bytes) {
            const hr::MetaLayout ml_a = hr::make_meta_layout(n_a, T_a, pt_stride, -1, 0, gi_a, true);
            const hr::MetaLayout ml_b = hr::make_meta_layout(n_b, T_b, pt_stride, -1, 0, gi_b, true);
            rc = stage_reserve(m, ml_a.total + ml_b.total);
            if (rc != HR_OK) return rc;
            if (!m->aux_stream) {
                HR_HIP(hipStreamCreateWithFlags(&m->aux_stream, hipStreamNonBlocking));
                HR_HIP(hipEventCreateWithFlags(&m->fork_ev, hipEventDisableTiming));
                HR_HIP(hipEventCreateWithFlags(&m->join_ev, hipEventDisableTiming));
            }
            // Both parts' metadata go up on the caller's stream (the host may then reuse the staging buffer and run ahead
            // of the device).  The second stream starts behind the first half's first QKV projection, so that the halves
            // run one kernel apart, each kernel starting on the CUs the other half's kernel is leaving, rather than as
            // twin kernels side by side whose last rounds coincide; the caller's stream ends behind the second half.
            ScorePart pa, pb;
            char* wsb_b = wsb + ws_a.total;
            rc = prepare_score_part(m, n_a, page_table, pt_stride, doc_lens, query_tokens, query_lens, T_a, mfma_attn, ws_a, ml_a, gi_a,
                                    m->stage, wsb, st, &pa);
            if (rc == HR_OK)
                rc = prepare_score_part(m, n_b, page_table ? page_table + (size_t)n_a * pt_stride : nullptr, pt_stride, doc_lens + n_a,
                                        query_tokens + T_a, query_lens + n_a, T_b, mfma_attn, ws_b, ml_b, gi_b, m->stage + ml_a.total,
                                        wsb_b, st, &pb);
            HR_HIP(hipEventRecord(m->stage_ev, st));
            m->stage_pending = true;
            if (rc != HR_OK) return rc;
            const int rc_a = run_score_part(m, pool, pa, ws_a, wsb, max_q, scores_dev, st, m->fork_ev);
            if (rc_a != HR_OK) return rc_a;
            HR_HIP(hipStreamWaitEvent(m->aux_stream, m->fork_ev, 0));
            const int rc_b = run_score_part(m, pool, pb, ws_b, wsb_b, max_q, scores_dev + n_a, m->aux_stream);
            HR_HIP(hipEventRecord(m->join_ev, m->aux_stream));
            HR_HIP(hipStreamWaitEvent(st, m->join_ev, 0));
            return rc_a != HR_OK ? rc_a : rc_b;
        }
    }
    return score_one_piece(m, pool, n_pairs, page_table, pt_stride, doc_lens, query_tokens, query_lens, T, mfma_attn, max_q, ws, grp_ints,
                           wsb, scores_dev, st, true);
}

size_t hr_rerank_static_scratch_bytes(void) { return kStaticScratchBytes; }

int hr_rerank_score_static(hr_model* m, const hr_pool* pool, int32_t n_pairs, const int32_t* page_table, int32_t pt_stride,
                           const int32_t* doc_lens, const int32_t* query_tokens, const int32_t* query_lens, float* scores_dev,
                           void* stream) {
    if (!m || !pool) return HR_ERR_INVALID_ARG;
    int max_q = 0;
    if (n_pairs > 0 && query_lens)
        for (int32_t p = 0; p < n_pairs; ++p) max_q = std::max(max_q, query_lens[p]);
    const bool mfma_attn = use_mfma_attn(m, pool->cfg.kv_dtype, max_q, true);
    int64_t T = 0;
    int rc = hr::score_check_args(m->cfg, pool, n_pairs, page_table, pt_stride, doc_lens, query_tokens, query_lens,
                                  mfma_attn ? kMfmaMaxKeys : kGenericMaxKeys, &T);
    if (rc != HR_OK) return rc;
    if (n_pairs == 0) return HR_OK;
    if (!scores_dev) return HR_ERR_INVALID_ARG;
    const int g = m->cfg.n_q_heads / m->cfg.n_kv_heads;
    const int64_t grp_ints = (int64_t)hr::group_plan_ints_bound(n_pairs, T, g);
    const hr::Workspace ws = hr::make_workspace(m->cfg, n_pairs, T, pt_stride, !m->mfma_gemm, -1, 0, grp_ints, m->n_precise > 0, m->mfma_gemm);
    if (ws.total > kStaticScratchBytes) {
        snprintf(g_last_error, sizeof(g_last_error), "hr_rerank_score_static: this call needs %zu bytes of scratch, the static array holds %zu",
                 ws.total, kStaticScratchBytes);
        return HR_ERR_WORKSPACE_SMALL;
    }
    char* scratch = nullptr;                    // this device's copy of the array (a table lookup after the first call)
    rc = static_scratch_ptr(&scratch);
    if (rc != HR_OK) return rc;
    // one piece on the caller's stream, no timing events (their pool grows on demand), staging as it was set up at load
    const bool prof = m->prof_on;
    m->prof_on = false;
    rc = score_one_piece(m, pool, n_pairs, page_table, pt_stride, doc_lens, query_tokens, query_lens, T, mfma_attn, max_q, ws, grp_ints,
                         scratch, scores_dev, (hipStream_t)stream, false);
    m->prof_on = prof;
    return rc;
}

// ---- fixed-shape scoring plans -----------------------------------------------------------------------------------
struct hr_plan {
    hr_model* m = nullptr;
    const hr_pool* pool = nullptr;
    int32_t n_pairs = 0, pt_stride = 0;
    int64_t T = 0, grp_ints = 0;
    int max_q = 0;
    bool mfma_attn = false, inputs_set = false;
    int n_precise = 0;                               // as the model was set when the plan was made (the workspace is carved for it)
    std::vector<int32_t> doc_lens, query_lens;
    hr::Workspace ws;
    hr::MetaLayout ml;
    char* wsb = nullptr;
    int32_t* stage = nullptr;                        // pinned, ml.total ints, owned by the plan
    size_t upload_ints = 0;
    ScorePart part;
};

int hr_rerank_plan_create(hr_model* m, const hr_pool* pool, int32_t n_pairs, const int32_t* doc_lens, const int32_t* query_lens,
                          int32_t pt_stride, void* workspace_dev, size_t workspace_bytes, hr_plan** out) {
    if (!out) return HR_ERR_INVALID_ARG;
    *out = nullptr;
    if (!m || !pool || n_pairs <= 0 || pt_stride < 0 || !doc_lens || !query_lens || !workspace_dev) return HR_ERR_INVALID_ARG;
    if ((uintptr_t)workspace_dev % hr::kAlign != 0) return HR_ERR_INVALID_ARG;
    const hr_model_cfg& mc = m->cfg;
    if (pool->cfg.n_layers != mc.n_layers || pool->cfg.n_kv_heads != mc.n_kv_heads || pool->cfg.head_dim != mc.head_dim) return HR_ERR_MISMATCH;
    if ((mc.dtype == HR_F32) != (pool->cfg.kv_dtype == HR_F32)) return HR_ERR_MISMATCH;
    int max_q = 0;
    for (int32_t p = 0; p < n_pairs; ++p) max_q = std::max(max_q, query_lens[p]);
    const bool mfma_attn = use_mfma_attn(m, pool->cfg.kv_dtype, max_q, true);
    int64_t T = 0;
    for (int32_t p = 0; p < n_pairs; ++p) {
        if (doc_lens[p] < 0 || query_lens[p] <= 0) return HR_ERR_LEN_RANGE;
        if ((int64_t)doc_lens[p] + query_lens[p] > (mfma_attn ? kMfmaMaxKeys : kGenericMaxKeys)) return HR_ERR_LEN_RANGE;
        if (((int64_t)doc_lens[p] + hr::kPageTokens - 1) / hr::kPageTokens > pt_stride) return HR_ERR_TABLE_SHORT;
        T += query_lens[p];
    }
    if (T > (int64_t)1 << 30) return HR_ERR_LEN_RANGE;
    hr_plan* pl = new (std::nothrow) hr_plan();
    if (!pl) return HR_ERR_INVALID_ARG;
    pl->m = m; pl->pool = pool; pl->n_pairs = n_pairs; pl->pt_stride = pt_stride; pl->T = T; pl->max_q = max_q;
    pl->mfma_attn = mfma_attn; pl->n_precise = m->n_precise;
    pl->doc_lens.assign(doc_lens, doc_lens + n_pairs);
    pl->query_lens.assign(query_lens, query_lens + n_pairs);
    pl->grp_ints = (int64_t)hr::group_plan_ints_bound(n_pairs, T, mc.n_q_heads / mc.n_kv_heads);
    pl->ws = hr::make_workspace(mc, n_pairs, T, pt_stride, !m->mfma_gemm, -1, 0, pl->grp_ints, m->n_precise > 0, m->mfma_gemm);
    pl->ml = hr::make_meta_layout(n_pairs, T, pt_stride, -1, 0, pl->grp_ints, m->mfma_gemm);
    pl->wsb = (char*)workspace_dev;
    if (workspace_bytes < pl->ws.total) {
        delete pl;
        return HR_ERR_WORKSPACE_SMALL;
    }
    hipError_t e = hipHostMalloc((void**)&pl->stage, std::max<size_t>(pl->ml.total, 64) * sizeof(int32_t), hipHostMallocDefault);
    if (e != hipSuccess) {
        note_hip_error(e, "hipHostMalloc (plan metadata)");
        delete pl;
        return HR_ERR_DEVICE;
    }
    std::memset(pl->stage, 0, pl->ml.total * sizeof(int32_t));
    *out = pl;
    return HR_OK;
}

int hr_rerank_plan_set_inputs(hr_plan* pl, const int32_t* page_table, const int32_t* query_tokens) {
    if (!pl || !query_tokens) return HR_ERR_INVALID_ARG;
    int64_t T = 0;
    int rc = hr::score_check_args(pl->m->cfg, pl->pool, pl->n_pairs, page_table, pl->pt_stride, pl->doc_lens.data(), query_tokens,
                                  pl->query_lens.data(), pl->mfma_attn ? kMfmaMaxKeys : kGenericMaxKeys, &T);
    if (rc != HR_OK) return rc;
    build_score_part(pl->m, pl->n_pairs, page_table, pl->pt_stride, pl->doc_lens.data(), query_tokens, pl->query_lens.data(), pl->T,
                     pl->mfma_attn, pl->ws, pl->ml, pl->grp_ints, pl->stage, pl->wsb, false, &pl->part, &pl->upload_ints);
    pl->inputs_set = true;
    return HR_OK;
}

int hr_rerank_plan_run(hr_plan* pl, float* scores_dev, void* stream) {
    if (!pl || !scores_dev) return HR_ERR_INVALID_ARG;
    if (!pl->inputs_set) {
        snprintf(g_last_error, sizeof(g_last_error), "hr_rerank_plan_run: no inputs set (hr_rerank_plan_set_inputs)");
        return HR_ERR_INVALID_ARG;
    }
    hr_model* m = pl->m;
    hipStream_t st = (hipStream_t)stream;
    // everything below is stream work only: one copy from the plan's own pinned block and the kernels.  No host wait, no
    // allocation, no event, no second stream, no timing.
    HR_HIP(hipMemcpyAsync(pl->wsb + pl->ws.off_meta, pl->stage, pl->upload_ints * sizeof(int32_t), hipMemcpyHostToDevice, st));
    const bool prof = m->prof_on;
    m->prof_on = false;
    const int rc = run_layers(m, pl->pool, false, pl->part.mv, pl->ws, pl->wsb, pl->part.max_keys, pl->max_q, scores_dev, st, nullptr,
                              pl->part.gv.n_groups > 0 ? &pl->part.gv : nullptr, nullptr, pl->n_precise);
    m->prof_on = prof;
    return rc;
}

void hr_rerank_plan_destroy(hr_plan* pl) {
    if (!pl) return;
    if (pl->stage) (void)hipHostFree(pl->stage);
    delete pl;
}

int hr_model_set_precise_layers(hr_model* m, int n_layers) {
    if (!m || n_layers < -1 || n_layers > m->cfg.n_layers) return HR_ERR_INVALID_ARG;
    if (n_layers > 0 && !m->mfma_gemm) return HR_ERR_UNSUPPORTED_SHAPE;
    m->n_precise = n_layers < 0 ? default_precise_layers(m->cfg, m->mfma_gemm) : n_layers;
    return HR_OK;
}

int hr_model_precise_layers(const hr_model* m) { return m ? m->n_precise : HR_ERR_INVALID_ARG; }

int hr_rerank_parts(const hr_model* m, int64_t total_q_tokens) {
    if (!m || total_q_tokens < 0) return HR_ERR_INVALID_ARG;
    return split_wanted(m, total_q_tokens) ? 2 : 1;
}

int hr_rerank_set_streams(hr_model* m, int n_streams) {
    if (!m || n_streams < 1 || n_streams > 2) return HR_ERR_INVALID_ARG;
    m->n_streams = n_streams;
    return HR_OK;
}

int hr_rerank_validate(const hr_model_cfg* cfg, const hr_pool* pool, int32_t n_pairs, const int32_t* page_table,
                       int32_t pt_stride, const int32_t* doc_lens, const int32_t* query_tokens, const int32_t* query_lens) {
    if (!hr::model_cfg_valid(cfg) || !pool) return HR_ERR_INVALID_ARG;
    int max_q = 0;
    if (n_pairs > 0 && query_lens)
        for (int32_t p = 0; p < n_pairs; ++p) max_q = std::max(max_q, query_lens[p]);
    const bool mfma_attn = hr::gemm_mfma_supported(*cfg) && hr::attn_mfma_supported_cut(*cfg, pool->cfg.kv_dtype, max_q);
    return hr::score_check_args(*cfg, pool, n_pairs, page_table, pt_stride, doc_lens, query_tokens, query_lens,
                                mfma_attn ? kMfmaMaxKeys : kGenericMaxKeys, nullptr);
}

size_t hr_rerank_full_workspace_bytes(const hr_model* m, int32_t n_pairs, int64_t total_tokens) {
    if (!m || n_pairs < 0 || total_tokens < 0) return 0;
    if (chunked_ok(m)) {
        // upper bounds without the lengths: every pair adds at most one partial chunk; a row of the self page table
        // is at most as long as the longest sequence, itself at most total_tokens
        const int ch = full_chunk(m);
        const int64_t n_chunks = total_tokens / ch + n_pairs;
        const int64_t stride = std::max<int64_t>(1, std::min<int64_t>(total_tokens, kChunkedMaxKeys) / hr::kPageTokens);
        return hr::make_workspace(m->cfg, n_chunks, total_tokens, stride, false, n_pairs, 0).total;
    }
    return hr::make_workspace(m->cfg, n_pairs, total_tokens, 0, !m->mfma_gemm).total;
}

int hr_rerank_score_full(hr_model* m, int32_t n_pairs, const int32_t* doc_tokens, const int32_t* doc_lens,
                         const int32_t* query_tokens, const int32_t* query_lens, void* workspace_dev, size_t workspace_bytes,
                         float* scores_dev, void* stream) {
    if (!m || n_pairs < 0) return HR_ERR_INVALID_ARG;
    if (n_pairs == 0) return HR_OK;
    if (!doc_lens || !query_lens || !query_tokens || !workspace_dev || !scores_dev) return HR_ERR_INVALID_ARG;
    if ((uintptr_t)workspace_dev % hr::kAlign != 0) return HR_ERR_INVALID_ARG;
    int64_t T = 0, Td = 0;
    int max_len = 0;
    for (int32_t p = 0; p < n_pairs; ++p) {
        if (doc_lens[p] < 0 || query_lens[p] <= 0) return HR_ERR_LEN_RANGE;
        int64_t n = (int64_t)doc_lens[p] + query_lens[p];
        if (n > (chunked_ok(m) ? kChunkedMaxKeys : kGenericMaxKeys)) return HR_ERR_LEN_RANGE;
        max_len = std::max(max_len, (int)n);
        T += n;
        Td += doc_lens[p];
    }
    if (T > (int64_t)1 << 30) return HR_ERR_LEN_RANGE;
    if (Td > 0 && !doc_tokens) return HR_ERR_INVALID_ARG;
    // concatenated [doc ; query] token stream and its lengths
    std::vector<int32_t> toks((size_t)T), lens((size_t)n_pairs);
    {
        int64_t t = 0, td = 0, tq = 0;
        for (int32_t p = 0; p < n_pairs; ++p) {
            for (int32_t i = 0; i < doc_lens[p]; ++i) toks[t++] = doc_tokens[td++];
            for (int32_t i = 0; i < query_lens[p]; ++i) toks[t++] = query_tokens[tq++];
            lens[p] = doc_lens[p] + query_lens[p];
        }
    }
    for (int64_t t = 0; t < T; ++t)
        if (toks[t] < 0 || toks[t] >= m->cfg.vocab) return HR_ERR_TOKEN_RANGE;

    hipStream_t st = (hipStream_t)stream;
    char* wsb = (char*)workspace_dev;
    if (chunked_ok(m)) {
        const int ch = full_chunk(m);
        hr::ChunkPlan cp = hr::make_chunk_plan(n_pairs, lens.data(), ch);
        hr::Workspace ws = hr::make_workspace(m->cfg, cp.n_chunks, T, cp.pt_stride, false, n_pairs, 0);
        if (workspace_bytes < ws.total) return HR_ERR_WORKSPACE_SMALL;
        hr::MetaLayout ml = hr::make_meta_layout(cp.n_chunks, T, cp.pt_stride, n_pairs, 0);
        int rc = stage_reserve(m, ml.total);
        if (rc != HR_OK) return rc;
        hr::fill_meta(m->stage, ml, cp.n_chunks, cp.prefix_lens.data(), cp.new_lens.data(), toks.data(), cp.page_table.data(),
                      cp.pt_stride, cp.out_row.data(), n_pairs);
        HR_HIP(hipMemcpyAsync(wsb + ws.off_meta, m->stage, ml.total * sizeof(int32_t), hipMemcpyHostToDevice, st));
        HR_HIP(hipEventRecord(m->stage_ev, st));
        m->stage_pending = true;
        hr::MetaView mv = make_meta_view((const int32_t*)(wsb + ws.off_meta), ml, cp.n_chunks, T, cp.pt_stride);
        mv.n_out = n_pairs;
        return run_layers(m, nullptr, true, mv, ws, wsb, max_len, ch, scores_dev, st);
    }
    hr::Workspace ws = hr::make_workspace(m->cfg, n_pairs, T, 0, !m->mfma_gemm);
    if (workspace_bytes < ws.total) return HR_ERR_WORKSPACE_SMALL;
    hr::MetaLayout ml = hr::make_meta_layout(n_pairs, T, 0);
    int rc = stage_reserve(m, ml.total);
    if (rc != HR_OK) return rc;
    hr::fill_meta(m->stage, ml, n_pairs, nullptr, lens.data(), toks.data(), nullptr, 0);
    HR_HIP(hipMemcpyAsync(wsb + ws.off_meta, m->stage, ml.total * sizeof(int32_t), hipMemcpyHostToDevice, st));
    HR_HIP(hipEventRecord(m->stage_ev, st));
    m->stage_pending = true;
    hr::MetaView mv = make_meta_view((const int32_t*)(wsb + ws.off_meta), ml, n_pairs, T, 0);
    return run_layers(m, nullptr, false, mv, ws, wsb, max_len, max_len, scores_dev, st);
}

size_t hr_doc_prefill_workspace_bytes(const hr_model* m, int32_t n_docs, int64_t total_tokens) {
    if (!m || n_docs < 0 || total_tokens < 0 || !chunked_ok(m)) return 0;
    const int ch = full_chunk(m);
    const int64_t n_chunks = total_tokens / ch + n_docs;
    const int64_t stride = std::max<int64_t>(1, std::min<int64_t>(total_tokens, kChunkedMaxKeys) / hr::kPageTokens);
    const int64_t pages = total_tokens / hr::kPageTokens + n_docs;
    return hr::make_workspace(m->cfg, n_chunks, total_tokens, stride, false, n_docs, 2 * pages).total;
}

int hr_doc_prefill(hr_model* m, hr_pool* pool, int32_t n_docs, const int32_t* doc_tokens, const int32_t* doc_lens,
                   const int32_t* page_table, int32_t pt_stride, void* workspace_dev, size_t workspace_bytes, void* stream) {
    if (!m || !pool || n_docs < 0 || pt_stride < 0) return HR_ERR_INVALID_ARG;
    if (n_docs == 0) return HR_OK;
    if (!doc_tokens || !doc_lens || !page_table || !workspace_dev) return HR_ERR_INVALID_ARG;
    if ((uintptr_t)workspace_dev % hr::kAlign != 0) return HR_ERR_INVALID_ARG;
    const hr_model_cfg& c = m->cfg;
    if (pool->cfg.n_layers != c.n_layers || pool->cfg.n_kv_heads != c.n_kv_heads || pool->cfg.head_dim != c.head_dim)
        return HR_ERR_MISMATCH;
    if ((pool->cfg.kv_dtype != HR_BF16 && pool->cfg.kv_dtype != HR_FP8_E4M3) || !chunked_ok(m)) return HR_ERR_UNSUPPORTED_SHAPE;
    int64_t T = 0;
    int max_len = 0;
    std::vector<int32_t> dst;          // flat list of target pages, document after document
    for (int32_t d = 0; d < n_docs; ++d) {
        if (doc_lens[d] <= 0 || doc_lens[d] > kChunkedMaxKeys) return HR_ERR_LEN_RANGE;
        const int64_t np = ((int64_t)doc_lens[d] + hr::kPageTokens - 1) / hr::kPageTokens;
        if (np > pt_stride) return HR_ERR_TABLE_SHORT;
        int rc = hr::pool_check_write(pool, doc_lens[d], page_table + (size_t)d * pt_stride);
        if (rc != HR_OK) return rc;
        for (int64_t i = 0; i < np; ++i) dst.push_back(page_table[(size_t)d * pt_stride + i]);
        max_len = std::max(max_len, doc_lens[d]);
        T += doc_lens[d];
    }
    {   // the same page must not be given to two documents of this call
        std::vector<int32_t> sorted(dst);
        std::sort(sorted.begin(), sorted.end());
        if (std::adjacent_find(sorted.begin(), sorted.end()) != sorted.end()) return HR_ERR_PAGE_DUP;
    }
    for (int64_t t = 0; t < T; ++t)
        if (doc_tokens[t] < 0 || doc_tokens[t] >= c.vocab) return HR_ERR_TOKEN_RANGE;

    const int ch = full_chunk(m);
    hr::ChunkPlan cp = hr::make_chunk_plan(n_docs, doc_lens, ch);
    const int64_t n_pages = (int64_t)dst.size();
    hr::Workspace ws = hr::make_workspace(c, cp.n_chunks, T, cp.pt_stride, false, n_docs, 2 * n_pages);
    if (workspace_bytes < ws.total) return HR_ERR_WORKSPACE_SMALL;
    hr::MetaLayout ml = hr::make_meta_layout(cp.n_chunks, T, cp.pt_stride, n_docs, 2 * n_pages);
    int rc = stage_reserve(m, ml.total);
    if (rc != HR_OK) return rc;
    hr::fill_meta(m->stage, ml, cp.n_chunks, cp.prefix_lens.data(), cp.new_lens.data(), doc_tokens, cp.page_table.data(), cp.pt_stride,
                  cp.out_row.data(), n_docs);
    {
        int32_t* src = m->stage + ml.dst_table;
        int32_t* dstp = src + n_pages;
        int64_t i = 0;
        for (int32_t d = 0; d < n_docs; ++d) {
            const int64_t np = ((int64_t)doc_lens[d] + hr::kPageTokens - 1) / hr::kPageTokens;
            for (int64_t pg = 0; pg < np; ++pg, ++i) {
                src[i] = cp.first_page[d] + (int32_t)pg;
                dstp[i] = dst[i];
            }
        }
    }
    hipStream_t st = (hipStream_t)stream;
    char* wsb = (char*)workspace_dev;
    HR_HIP(hipMemcpyAsync(wsb + ws.off_meta, m->stage, ml.total * sizeof(int32_t), hipMemcpyHostToDevice, st));
    HR_HIP(hipEventRecord(m->stage_ev, st));
    m->stage_pending = true;
    hr::MetaView mv = make_meta_view((const int32_t*)(wsb + ws.off_meta), ml, cp.n_chunks, T, cp.pt_stride);
    mv.n_out = n_docs;
    PrefillTarget pf{pool, (const int32_t*)(wsb + ws.off_meta) + ml.dst_table, (const int32_t*)(wsb + ws.off_meta) + ml.dst_table + n_pages,
                     (int)n_pages};
    rc = run_layers(m, nullptr, true, mv, ws, wsb, max_len, ch, nullptr, st, &pf);
    if (rc != HR_OK) return rc;
    for (int32_t d = 0; d < n_docs; ++d)
        hr::pool_mark(pool, page_table + (size_t)d * pt_stride, (doc_lens[d] + hr::kPageTokens - 1) / hr::kPageTokens, hr::PAGE_USED);
    return HR_OK;
}

int hr_rerank_topk(const float* scores_dev, const int32_t* seg_dev, int32_t n_queries, int32_t max_cands, int32_t k,
                   int32_t* topk_idx_dev, float* topk_scores_dev, void* stream) {
    if (n_queries == 0) return HR_OK;
    if (!scores_dev || !seg_dev || !topk_idx_dev || n_queries < 0 || max_cands < 1 || max_cands > 4096 || k < 1 || k > max_cands) {
        snprintf(g_last_error, sizeof(g_last_error), "hr_rerank_topk: null pointer, or n_queries / max_cands (1..4096) / k (1..max_cands) out of range");
        return HR_ERR_INVALID_ARG;
    }
    HR_HIP(launch_segment_topk(scores_dev, seg_dev, n_queries, max_cands, k, topk_idx_dev, topk_scores_dev, (hipStream_t)stream));
    return HR_OK;
}

int hr_profile_enable(hr_model* m, int enable) {
    if (!m) return HR_ERR_INVALID_ARG;
    m->prof_on = enable != 0;
    return HR_OK;
}

int hr_profile_select(hr_model* m, uint32_t class_mask) {
    if (!m) return HR_ERR_INVALID_ARG;
    m->prof_mask = class_mask;
    return HR_OK;
}

int hr_profile_count(void) { return PC_COUNT; }

const char* hr_profile_name(int idx) { return idx >= 0 && idx < PC_COUNT ? kProfNames[idx] : ""; }

int hr_profile_read(hr_model* m, double* ms_out, int64_t* launches_out) {
    if (!m || !ms_out || !launches_out) return HR_ERR_INVALID_ARG;
    for (int i = 0; i < PC_COUNT; ++i) { ms_out[i] = 0.0; launches_out[i] = 0; }
    for (size_t i = 0; i + 1 < m->prof_used; i += 2) {
        HR_HIP(hipEventSynchronize(m->prof_events[i + 1]));
        float ms = 0.f;
        HR_HIP(hipEventElapsedTime(&ms, m->prof_events[i], m->prof_events[i + 1]));
        int cls = m->prof_class[i / 2];
        ms_out[cls] += ms;
        launches_out[cls] += 1;
    }
    m->prof_used = 0;
    m->prof_class.clear();
    return HR_OK;
}

static int read_range_counters(const void* dev, hr_range_report* out) {
    long long c[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    HR_HIP(hipMemcpy(c, dev, sizeof(c), hipMemcpyDeviceToHost));        // waits for the work enqueued so far
    out->overflow = c[hr::RC_OVERFLOW];
    out->underflow = c[hr::RC_UNDERFLOW];
    out->nonfinite_inputs = c[hr::RC_NONFINITE_IN];
    out->fp8_nan_codes = c[hr::RC_FP8_NAN_CODE];
    out->fp8_bad_scales = c[hr::RC_FP8_BAD_SCALE];
    return HR_OK;
}

int hr_model_range_report(const hr_model* m, hr_range_report* out) {
    if (!m || !out) return HR_ERR_INVALID_ARG;
    *out = hr_range_report{};
    return read_range_counters(m->pack_base + m->pack.counter_off, out);
}

int hr_kv_pool_range_report(const hr_pool* pool, hr_range_report* out) {
    if (!pool || !out) return HR_ERR_INVALID_ARG;
    *out = hr_range_report{};
    if (!pool->counters_zeroed) return HR_OK;                          // nothing has been written through hr_doc_kv_write yet
    return read_range_counters(pool->base + pool->lay.counter_off, out);
}

int hr_probe_read_bandwidth(const void* src_dev, size_t bytes, void* sink_dev, size_t sink_bytes, int to_lds, void* stream) {
    if (!src_dev || !sink_dev || bytes < 1024 || sink_bytes < 4 || (uintptr_t)src_dev % 16 != 0 || (uintptr_t)sink_dev % 4 != 0)
        return HR_ERR_INVALID_ARG;
    HR_HIP(launch_probe_read(src_dev, bytes, sink_dev, sink_bytes, to_lds != 0, hr::device_cu_count(), (hipStream_t)stream));
    return HR_OK;
}

const char* hr_last_error(void) { return g_last_error; }

const char* hr_attention_path(const hr_model* m, const hr_pool* pool) {
    if (!m || !pool) return "none";
    return use_mfma_attn(m, pool->cfg.kv_dtype, 1) ? "mfma" : "generic";
}

const char* hr_gemm_path(const hr_model* m) {
    if (!m) return "none";
    return m->mfma_gemm ? "mfma" : "generic";
}

}  // extern "C"
