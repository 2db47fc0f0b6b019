/*
 * hyperrerank - C ABI of the MI355X reranker scoring library.
 *
 * The method (HyperRAG, Section 3.3 Property 1 and Section 4.2): a decoder-only
 * reranker scores a (document, query) pair on the sequence [document ; query].
 * Because attention is lower-triangular and the document always starts the
 * sequence, every layer's K/V of the document can be computed once, stored, and
 * reused for any query; scoring then runs only the short query suffix through
 * the layers while attending to the stored document K/V ("static document
 * prefix | query suffix" KV layout).  This library keeps the stored K/V in a
 * paged pool in HBM and implements that scoring pass for a batch of pairs.
 *
 * Conventions
 *   - "host" pointers are ordinary CPU memory, read during the call only.
 *   - "device" pointers are HBM addresses on the current HIP device.  The
 *     library never allocates or frees device memory: pools, packed weights,
 *     workspaces and outputs are all caller-owned.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Calls that take a stream enqueue work and return without waiting.
 *   - A model handle carries per-call host state (a pinned staging buffer, an event, a second stream): calls on
 *     one handle must not overlap in host time; different handles, and pools, are independent.  The library
 *     allocates no device memory, but it owns that small pinned host buffer (1 MiB from hr_weights_load on, grown
 *     when a call's metadata needs more) and, once a scoring call has been cut in two halves, one stream and three
 *     events per model handle (released by hr_model_destroy).
 *   - Calls that upload per-call metadata (scoring, prefill) wait on the host for the previous upload of the same
 *     handle and copy from its staging buffer: they are not meant to be recorded into a HIP graph.  hr_rerank_plan_run
 *     is the form that is.
 *   - Every call returns HR_OK (0) or a negative hr_status.  Every argument check happens before anything is enqueued
 *     or any library state changes; only HR_ERR_DEVICE (a HIP call failed mid-way) can leave part of a call's work on the
 *     stream, and the outputs of that call are then undefined.  Nothing throws or aborts.
 *   - All matrices are row-major [out][in]; activations use the model dtype
 *     (HR_F32 or HR_BF16); norm gains and scores are fp32.
 *   - A page holds 16 consecutive tokens of one document for one (layer,
 *     kv head): K as [16][head_dim] and V transposed; the in-pool arrangement
 *     is private to the library (use hr_doc_kv_write to fill it).
 */
#ifndef HYPERRERANK_H
#define HYPERRERANK_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define HR_PAGE_TOKENS 16

typedef enum hr_status {
    HR_OK = 0,
    HR_ERR_INVALID_ARG = -1,       /* null pointer, non-positive count, bad enum                    */
    HR_ERR_POOL_TOO_SMALL = -2,    /* device buffer smaller than hr_kv_pool_bytes                    */
    HR_ERR_PAGE_RANGE = -3,        /* page id < 0 or >= num_pages                                     */
    HR_ERR_PAGE_IN_USE = -4,       /* writing a page that already holds a document                    */
    HR_ERR_PAGE_DUP = -5,          /* the same page id twice in one document                          */
    HR_ERR_LEN_RANGE = -6,         /* document / query length <= 0 or above the supported maximum    */
    HR_ERR_TABLE_SHORT = -7,       /* page-table row too short, or -1 / unwritten page inside it     */
    HR_ERR_TOKEN_RANGE = -8,       /* token id < 0 or >= vocab                                        */
    HR_ERR_WORKSPACE_SMALL = -9,   /* workspace smaller than hr_rerank_workspace_bytes                */
    HR_ERR_UNSUPPORTED_SHAPE = -10,/* model / pool shape the kernels do not cover                     */
    HR_ERR_DEVICE = -11,           /* a HIP runtime call failed (no device, launch error)            */
    HR_ERR_POOL_FULL = -12,        /* hr_kv_pool_alloc_pages: not enough free pages                   */
    HR_ERR_MISMATCH = -13          /* pool and model disagree (layers, kv heads, head_dim, dtype)    */
} hr_status;

typedef enum hr_dtype { HR_F32 = 0, HR_BF16 = 1, HR_FP8_E4M3 = 2 } hr_dtype;

/* Paged document-KV pool.  kv_dtype: HR_F32, HR_BF16, or HR_FP8_E4M3 (OCP E4M3, one fp32 scale
 * per (layer, page, kv head) for K and one for V; value = decode(code) * scale).  The 8-bit form
 * follows Section 4.1 "KV-cache Quantization" / Appendix B (KV8, expanded after loading). */
typedef struct hr_pool_cfg {
    int32_t n_layers;
    int32_t n_kv_heads;
    int32_t head_dim;      /* multiple of 16, at most 256 */
    int32_t page_tokens;   /* must be HR_PAGE_TOKENS */
    int32_t num_pages;
    int32_t kv_dtype;      /* hr_dtype */
} hr_pool_cfg;

/* Reranker: pre-norm decoder blocks with RMSNorm, rotate-half RoPE, grouped-query attention,
 * SwiGLU, no biases; score = logit[yes_id] - logit[no_id] at the last query token with the
 * embedding matrix as the (tied) head, after the final RMSNorm. */
typedef struct hr_model_cfg {
    int32_t n_layers;
    int32_t hidden;
    int32_t n_q_heads;
    int32_t n_kv_heads;    /* divides n_q_heads */
    int32_t head_dim;
    int32_t ffn;
    int32_t vocab;
    int32_t yes_id;
    int32_t no_id;
    int32_t dtype;         /* HR_F32 or HR_BF16: weights and activations */
    float rope_base;
    float rms_eps;
} hr_model_cfg;

/* Device pointers to the caller's weights.  The per-layer members are HOST arrays of n_layers
 * DEVICE pointers.  Matrices are in the model dtype; norm gains are fp32. */
typedef struct hr_weight_ptrs {
    const void* embedding;        /* device [vocab][hidden] */
    const float* final_norm;      /* device [hidden] */
    const void* const* wq;        /* [n_q_heads*head_dim][hidden] */
    const void* const* wk;        /* [n_kv_heads*head_dim][hidden] */
    const void* const* wv;        /* [n_kv_heads*head_dim][hidden] */
    const void* const* wo;        /* [hidden][n_q_heads*head_dim] */
    const void* const* wg;        /* [ffn][hidden] */
    const void* const* wu;        /* [ffn][hidden] */
    const void* const* wd;        /* [hidden][ffn] */
    const float* const* norm1;    /* [hidden] pre-attention gain */
    const float* const* norm2;    /* [hidden] pre-MLP gain */
} hr_weight_ptrs;

typedef struct hr_pool hr_pool;     /* host-side handle: layout + page bookkeeping */
typedef struct hr_model hr_model;   /* host-side handle: config + packed-weight pointers */

const char* hr_status_str(int status);

/* Text of the HIP error behind the calling thread's most recent HR_ERR_DEVICE ("" if none). */
const char* hr_last_error(void);

/* ---- document-KV pool (the stored per-document KV of Section 3.3 / 4.2, kept resident in HBM) ---- */

/* Bytes of device memory a pool of this shape needs; 0 if cfg is invalid. */
size_t hr_kv_pool_bytes(const hr_pool_cfg* cfg);

/* Bind a pool to caller-owned device memory `dev_mem` (>= hr_kv_pool_bytes, 256-byte aligned).
 * Pure host work: nothing is enqueued; all pages start free.  *out is freed by hr_kv_pool_destroy
 * (which does not touch dev_mem). */
int hr_kv_pool_create(const hr_pool_cfg* cfg, void* dev_mem, size_t bytes, hr_pool** out);
void hr_kv_pool_destroy(hr_pool* pool);

/* Number of free pages, or a negative status. */
int64_t hr_kv_pool_free_pages(const hr_pool* pool);

/* Reserve the n lowest-numbered free pages and return their ids in page_ids_out (host).  Reserved
 * pages can be written once with hr_doc_kv_write and are released with hr_doc_kv_free. */
int hr_kv_pool_alloc_pages(hr_pool* pool, int32_t n, int32_t* page_ids_out);

/* Store one document's K/V (stage one of the two-stage inference) into the pages the caller names.
 *   page_ids      host, ceil(doc_len/16) distinct ids, each free or reserved
 *   k_dev, v_dev  device, logical layout [n_layers][doc_len][n_kv_heads][head_dim] in kv_dtype
 *                 (fp8: E4M3 codes, one byte each); K is post-RoPE at positions 0..doc_len-1
 *   k_scales_dev, v_scales_dev   fp8 only: device fp32 [n_layers][n_pages][n_kv_heads]; else NULL
 * One HBM->HBM scatter kernel is enqueued on `stream`; the tail of a short last page is zeroed.
 * The source buffers must stay valid until that kernel has run. */
int hr_doc_kv_write(hr_pool* pool, int32_t doc_len, const int32_t* page_ids,
                    const void* k_dev, const void* v_dev,
                    const float* k_scales_dev, const float* v_scales_dev, void* stream);

/* Read one document's K/V back from its pages (the inverse of hr_doc_kv_write): what a storage tier would take
 * from the pool (Section 4.1 keeps the cached KV outside GPU memory), and what makes the pages a prefill wrote
 * checkable value by value.
 *   page_ids      host, ceil(doc_len/16) ids of pages that hold a document (written or prefilled)
 *   k_dev, v_dev  device, logical layout [n_layers][doc_len][n_kv_heads][head_dim] in the pool's own element type:
 *                 fp32 for HR_F32 pools, IEEE half for HR_BF16 pools (the pool keeps the caller's bf16 values as
 *                 halves: exactly for magnitudes in [2^-14, 65504], see hr_kv_pool_range_report for the rest; prefilled
 *                 pages are halves in the first place), E4M3 codes for fp8 pools
 *   k_scales_dev, v_scales_dev   fp8 only: device fp32 [n_layers][n_pages][n_kv_heads]; else NULL
 * One gather kernel is enqueued on `stream`.  HR_ERR_PAGE_RANGE for an id out of range, HR_ERR_TABLE_SHORT for a page
 * that holds nothing, HR_ERR_LEN_RANGE for doc_len <= 0. */
int hr_doc_kv_read(const hr_pool* pool, int32_t doc_len, const int32_t* page_ids,
                   void* k_dev, void* v_dev, float* k_scales_dev, float* v_scales_dev, void* stream);

/* Mark pages free again (contents are left as they are). */
int hr_doc_kv_free(hr_pool* pool, const int32_t* page_ids, int32_t n);

/* ---- host tier (Sections 4.1 and 4.3: the documents' KV lives in a storage backend behind the GPU and is loaded for
 * the retrieved candidates; here the backend is the caller's memory, normally pinned host memory, and a page moves
 * as one record) ---- */

/* Bytes of one page record: the page's K and V blocks of every layer and kv head in the pool's own arrangement
 * ([n_layers][n_kv_heads][K block | V block]), followed for fp8 pools by its scales ([n_layers][n_kv_heads][K, V] fp32).
 * A multiple of 16; 0 if pool is NULL.  Records are opaque: only a pool of the same configuration reads them. */
size_t hr_kv_page_record_bytes(const hr_pool* pool);

/* Copy n_pages pages out of the pool: record i at dst + i * hr_kv_page_record_bytes is page page_ids[i].
 *   page_ids  host, ids of pages that hold a document (HR_ERR_PAGE_RANGE / HR_ERR_TABLE_SHORT otherwise)
 *   dst       n_pages records of memory the GPU can address: device memory, or host memory pinned by the HIP runtime
 *             (hipHostMalloc); 16-byte aligned.  Pageable host memory is refused with HR_ERR_INVALID_ARG.
 * Copy kernels are enqueued on `stream` (they write pinned host memory over the bus directly: no staging buffer);
 * dst is complete when the stream has drained.  The pool is unchanged. */
int hr_kv_pages_out(const hr_pool* pool, int32_t n_pages, const int32_t* page_ids, void* dst, void* stream);

/* The inverse: page page_ids[i] <- record i of src (same kinds of memory as dst above).  The pages must be distinct
 * and free or reserved (HR_ERR_PAGE_DUP / HR_ERR_PAGE_IN_USE) and are marked used on success; they may be scored as
 * soon as work enqueued after this call on the same stream runs, or after an event recorded behind it.  Issued on
 * a second stream it overlaps with hr_rerank_score calls that read other pages of the same pool. */
int hr_kv_pages_in(hr_pool* pool, int32_t n_pages, const int32_t* page_ids, const void* src, void* stream);

/* The same with 4-bit records (Section 4.1 names a 4-bit KV cache, KV4W16A16, and Appendix B expands quantised KV
 * to 16 bits after it is loaded; the paper gives no format, this is the library's): the pool stays 16-bit, a page
 * is quantised as it leaves and expanded as it arrives.  16-bit pools only (HR_ERR_UNSUPPORTED_SHAPE otherwise).
 * Per token and per 32 consecutive channels of one (layer, kv head), separately for K and V: scale = amax / 7 in
 * fp32 (1 if all zero), code = x / scale rounded to the nearest integer (ties to even) in [-7, 7]; a loaded page
 * holds code * scale rounded to half.  Record of one page, for every (layer, kv head) in that order:
 *   K codes [16 tokens][head_dim / 2] bytes (channel 2i in the low nibble, 2i + 1 in the high one, two's complement),
 *   V codes likewise, K scales [16][head_dim / 32] fp32, V scales [16][head_dim / 32] fp32
 * = 20 * head_dim bytes per (layer, kv head), 3.2 times smaller than the 16-bit record.  Arguments, memory kinds,
 * page states and errors as for hr_kv_pages_out / hr_kv_pages_in. */
size_t hr_kv_page_record4_bytes(const hr_pool* pool);
int hr_kv_pages_out4(const hr_pool* pool, int32_t n_pages, const int32_t* page_ids, void* dst, void* stream);
int hr_kv_pages_in4(hr_pool* pool, int32_t n_pages, const int32_t* page_ids, const void* src, void* stream);

/* ---- what the 16-bit operand format met ----
 * A 16-bit model computes on IEEE halves: the caller's bf16 weights and bf16 document K/V are converted once, when the
 * weights are packed and when a document is written.  bf16 has the range of fp32, half does not: a magnitude of 65520 or
 * more becomes infinity, and below 2^-14 half is subnormal (a bf16 value below 2^-17 loses bits, below 2^-25 it becomes
 * zero).  The conversions count what they meet, and for fp8 pools the write also counts what the format cannot express:
 *   overflow          values that became infinity (scores that depend on them come out non-finite)
 *   underflow         values that half does not hold exactly (absolute error below 2^-25; random-initialised weights
 *                     always have a few per ten thousand of these)
 *   nonfinite_inputs  NaN or infinity in the caller's data
 *   fp8_nan_codes     E4M3 codes 0x7f / 0xff (NaN; the kernels read them as +-480)
 *   fp8_bad_scales    K or V scales that are not positive and finite, and V scales outside [2^-22, 2^8) (the power of
 *                     two of a V scale is applied while the codes are expanded to half, which covers that range)
 * Activations are not counted: one that exceeds the half range becomes infinity and makes the pair's score non-finite.
 * The report calls copy 64 bytes from the device and wait for the work enqueued so far (not for use in a hot loop).
 * Pages that arrive through hr_kv_pages_in / hr_doc_prefill are not counted (they were halves or codes already). */
typedef struct hr_range_report {
    int64_t overflow, underflow, nonfinite_inputs, fp8_nan_codes, fp8_bad_scales;
    int64_t reserved[3];
} hr_range_report;
int hr_model_range_report(const hr_model* model, hr_range_report* out);      /* since hr_weights_load */
int hr_kv_pool_range_report(const hr_pool* pool, hr_range_report* out);      /* over every hr_doc_kv_write so far */

/* ---- weights ---- */

/* Bytes of device memory for the library's packed copy of the layer weights
 * (fused QKV rows, interleaved gate/up rows); 0 if cfg is invalid. */
size_t hr_weights_pack_bytes(const hr_model_cfg* cfg);

/* Build the packed copy inside caller-owned `pack_dev` (copy kernels on `stream`) and return a
 * handle.  The embedding and the norm gains are borrowed (must outlive the handle); the per-layer
 * matrices may be released once `stream` has drained. */
int hr_weights_load(const hr_model_cfg* cfg, const hr_weight_ptrs* weights,
                    void* pack_dev, size_t pack_bytes, void* stream, hr_model** out);
void hr_model_destroy(hr_model* model);

/* ---- scoring (stage two: only the query suffix is computed) ---- */

/* Workspace bytes for one hr_rerank_score call of this size; 0 on invalid arguments. */
size_t hr_rerank_workspace_bytes(const hr_model* model, int32_t n_pairs, int64_t total_q_tokens,
                                 int32_t pt_stride);

/* scores[p] for p < n_pairs.  For pair p the query tokens sit at positions doc_lens[p] + 0,1,..,
 * attend to all doc_lens[p] cached document keys (found through page_table row p) and causally to
 * the query keys before them; the score is read at the last query token.
 *   page_table    host int32 [n_pairs][pt_stride]; row p lists ceil(doc_lens[p]/16) written pages,
 *                 the rest of the row is ignored (-1 by convention)
 *   doc_lens      host int32 [n_pairs], each >= 0 (0: no cached document, plain causal pass)
 *   query_tokens  host int32, the pairs' query token ids back to back (sum of query_lens entries)
 *   query_lens    host int32 [n_pairs], each >= 1
 *   workspace_dev device scratch, >= hr_rerank_workspace_bytes, 256-byte aligned, private to this
 *                 call until `stream` has drained
 *   scores_dev    device fp32 [n_pairs]
 * The pool is only read.  Host arrays may be reused as soon as the call returns.
 * Pairs of one call whose doc_lens and page-table rows are identical (the same cached document: Section 3.3,
 * pairwise independence makes a document's KV reusable for every query) share one pass over its pages in the
 * attention kernels; the scores are bit for bit those of the pairs scored alone.
 * Pairs of one call with identical query token strings (the same query against several candidates) share the first
 * layer's normalised rows and pre-RoPE q / k / v projections, which are equal for equal strings; each pair's rotation for
 * its own positions doc_lens[p] + i is applied afterwards.  Same bits again.
 * A call with at least 8192 query tokens on the MFMA path whose O / down projection tiles would leave more than 15 % of
 * the device's workgroup slots empty in the rounds they take runs as two halves of the pairs, the first on `stream`,
 * the second on a stream of the library's own that starts behind the work already enqueued on `stream` and that
 * `stream` waits for before anything enqueued after the call (see hr_rerank_set_streams); to the caller the call
 * is ordered on `stream` as if it were one piece of work. */
int hr_rerank_score(hr_model* model, const hr_pool* pool, int32_t n_pairs,
                    const int32_t* page_table, int32_t pt_stride, const int32_t* doc_lens,
                    const int32_t* query_tokens, const int32_t* query_lens,
                    void* workspace_dev, size_t workspace_bytes, float* scores_dev, void* stream);

/* ---- fixed-shape plans: a scoring call whose launches can be recorded once and replayed (Section 4.2: the static
 * [document prefix | query suffix] layout exists so that the reranker's execution can be captured ahead of time) ----
 * A plan fixes the shape of a call: the number of pairs and every pair's document and query length.  Which pages and
 * which query tokens it scores can change between runs.  hr_rerank_plan_run enqueues one host-to-device copy from a
 * pinned block the plan owns, and the kernels; it never waits on the host, allocates nothing and uses `stream` only,
 * so it may be recorded into a HIP graph (stream capture) and replayed.  The work of a plan depends on the lengths
 * alone: pairs are not regrouped by shared documents or shared query strings as hr_rerank_score does, which changes no
 * score bit.
 *   hr_rerank_plan_create      host: checks the lengths, carves `workspace_dev` (>= hr_rerank_workspace_bytes for these
 *                              sizes, private to the plan while it lives) and allocates the pinned metadata block (the one
 *                              allocation of a plan's life).  Uses the model's split-operand setting at this moment.
 *   hr_rerank_plan_set_inputs  host: validates page_table [n_pairs][pt_stride] and query_tokens (flat, pair after pair)
 *                              like hr_rerank_score and writes them into the pinned block.  The copy in a run or replay
 *                              reads that block when it executes: do not call this while a run or replay that has not
 *                              finished could still read the block.
 *   hr_rerank_plan_run         stream work only (see above); scores_dev fp32 [n_pairs].  HR_ERR_INVALID_ARG before the
 *                              first set_inputs.  Run it once outside capture first: the first launch of a kernel sets
 *                              its function attributes.
 * Plans of one model share its kernels but no state; a plan must not outlive its model, pool or workspace. */
typedef struct hr_plan hr_plan;
int hr_rerank_plan_create(hr_model* model, const hr_pool* pool, int32_t n_pairs, const int32_t* doc_lens,
                          const int32_t* query_lens, int32_t pt_stride, void* workspace_dev, size_t workspace_bytes,
                          hr_plan** out);
int hr_rerank_plan_set_inputs(hr_plan* plan, const int32_t* page_table, const int32_t* query_tokens);
int hr_rerank_plan_run(hr_plan* plan, float* scores_dev, void* stream);
void hr_rerank_plan_destroy(hr_plan* plan);

/* hr_rerank_score for callers that cannot allocate or hand over a workspace: code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc.  Same arguments, validation, kernels and scores (bit for bit) as
 * hr_rerank_score, except that the workspace is a file-scope device array inside the library
 * (hr_rerank_static_scratch_bytes() = 128 MiB; every GPU the library runs on holds its own copy until the process ends)
 * and the per-call metadata goes through the pinned staging buffer the model handle got at hr_weights_load (1 MiB).
 * The call allocates nothing: no device or pinned memory, no streams, no events; it always runs in one piece on `stream`,
 * and per-kernel timing (hr_profile_enable) is off for its duration.
 *   HR_ERR_WORKSPACE_SMALL  the call would need more scratch than the array holds, or more metadata than the staging
 *                           buffer holds (hr_last_error says which and how much); nothing is enqueued.  One query with
 *                           20 candidates of 32 query tokens needs about 13 MiB at the 0.5B shape and 85 MiB at the 8B shape.
 * The array is shared by every static call on that GPU, whatever the model handle, and keeps the last call's contents
 * (what must start at zero is cleared by the call itself): static calls that overlap in time on one GPU race with each
 * other, also when issued on different streams.  Order them on one stream or with events. */
size_t hr_rerank_static_scratch_bytes(void);
int hr_rerank_score_static(hr_model* model, const hr_pool* pool, int32_t n_pairs,
                           const int32_t* page_table, int32_t pt_stride, const int32_t* doc_lens,
                           const int32_t* query_tokens, const int32_t* query_lens,
                           float* scores_dev, void* stream);

/* Precision of the scoring pass on the MFMA kernels (16-bit models).  Operands of the matrix instructions are IEEE halves
 * (11 significant bits): weights and cached document K/V are exact as halves, but every activation that feeds an MFMA is
 * rounded once per layer, and a deep, wide network amplifies the first layers' roundings most (Section 3.3 calls the
 * cached pass lossless; the arithmetic's own rounding is what is left).  The first `n_layers` layers of hr_rerank_score
 * therefore can run with split operands: each such activation is carried as a pair of halves hi + lo (22 bits) and every
 * product with a lo term is one more MFMA chain into the same fp32 accumulator, about twice the work of those layers.
 *   n_layers   0 .. model layers, or -1 for the default: 2 when layers x hidden >= 65536 (the 8B shape), else 0
 * Changes hr_rerank_workspace_bytes (ask again after setting it).  hr_rerank_score_full and hr_doc_prefill always run
 * with plain 16-bit operands.  HR_ERR_UNSUPPORTED_SHAPE if n_layers > 0 on a model that runs the generic kernels
 * (those compute in fp32 throughout). */
int hr_model_set_precise_layers(hr_model* model, int n_layers);
int hr_model_precise_layers(const hr_model* model);

/* 1: scoring calls use the caller's stream only; 2 (the default): large calls are cut in two halves that run on
 * two streams, so that one half's kernels fill the compute units that the last, partly filled round of the other
 * half's GEMM tiles leaves idle (pairs are independent, Section 3.3: the scores do not change by a bit).
 * HR_ERR_INVALID_ARG for other values. */
int hr_rerank_set_streams(hr_model* model, int n_streams);

/* In how many parts (1 or 2) a scoring call with this many query tokens runs on the current device, given at least two
 * pairs and a model / pool combination on the MFMA kernels; a negative status on invalid arguments.  For reporting. */
int hr_rerank_parts(const hr_model* model, int64_t total_q_tokens);

/* The host-side checks hr_rerank_score performs before it enqueues anything, on their own: no
 * device work, no model handle needed.  Returns HR_OK or the status hr_rerank_score would return
 * for these arguments (lengths, page-table rows, page states, token ids, pool/model agreement). */
int hr_rerank_validate(const hr_model_cfg* cfg, const hr_pool* pool, int32_t n_pairs,
                       const int32_t* page_table, int32_t pt_stride, const int32_t* doc_lens,
                       const int32_t* query_tokens, const int32_t* query_lens);

/* ---- same-GPU reference without reuse: full prefill of [document ; query] per pair ---- */
/* (Section 3.3 "Potential 1": what the scoring pass is compared with.) */
size_t hr_rerank_full_workspace_bytes(const hr_model* model, int32_t n_pairs, int64_t total_tokens);

/* scores[p] from one causal pass over the concatenation of doc_tokens and query_tokens of pair p;
 * no pool is involved.  doc_tokens / query_tokens are flat host int32 arrays, pair after pair.
 * A sequence may hold up to 32768 tokens on the MFMA kernels (15000 on the generic ones): HR_ERR_LEN_RANGE beyond. */
int hr_rerank_score_full(hr_model* model, int32_t n_pairs,
                         const int32_t* doc_tokens, const int32_t* doc_lens,
                         const int32_t* query_tokens, const int32_t* query_lens,
                         void* workspace_dev, size_t workspace_bytes, float* scores_dev, void* stream);

/* ---- document prefill (stage one of the two-stage inference, Section 3.3 Property 1) ---- */

/* Workspace bytes for hr_doc_prefill; 0 if the model / shape is not covered (see hr_doc_prefill). */
size_t hr_doc_prefill_workspace_bytes(const hr_model* model, int32_t n_docs, int64_t total_tokens);

/* Run n_docs documents alone through the layers (positions 0..len-1, causal) and store every layer's post-RoPE
 * K and V in the pool pages the caller names, ready for hr_rerank_score.  Same kernels as the scoring pass: a
 * document is processed as chunks of 64 tokens whose prefix is the document's own earlier pages.
 *   doc_tokens  host int32, the documents' token ids back to back
 *   doc_lens    host int32 [n_docs], each 1 .. 32768
 *   page_table  host int32 [n_docs][pt_stride]; row d names ceil(doc_lens[d]/16) distinct free (or reserved) pages
 * 16-bit and fp8 pools, MFMA-covered models only (HR_ERR_UNSUPPORTED_SHAPE otherwise).  For an fp8 pool every page
 * is quantised as it is stored: per (layer, page, kv head) and separately for K and V, scale = amax / 448 over the page
 * (1 if amax = 0) in fp32, code = the E4M3 value nearest to x / scale (ties to the even code).  Pages are marked used on
 * success.  Work is enqueued on `stream`. */
int hr_doc_prefill(hr_model* model, hr_pool* pool, int32_t n_docs, const int32_t* doc_tokens, const int32_t* doc_lens,
                   const int32_t* page_table, int32_t pt_stride, void* workspace_dev, size_t workspace_bytes, void* stream);

/* ---- per-query selection (what the pipeline does with the scores: Section 3.1, "select top-k"; Table 1 reranks
 * 5 / 10 / 20 candidates down to the best one) ---- */

/* For each query the k best of its candidates, best first: score descending, candidate index ascending among equal
 * scores (-0 equals +0; NaN ranks below every number).
 *   scores_dev   device fp32, the scores of all pairs (what hr_rerank_score wrote)
 *   seg_dev      device int32 [n_queries + 1], ascending: query i owns pairs seg[i] .. seg[i+1]-1
 *   max_cands    host int, an upper bound of seg[i+1] - seg[i] (1 .. 4096); a longer segment is cut to its first
 *                max_cands candidates
 *   k            1 .. max_cands
 *   topk_idx_dev device int32 [n_queries][k]: candidate index inside the query's segment, -1 where the query has
 *                fewer than k candidates
 *   topk_scores_dev  optional (may be NULL) device fp32 [n_queries][k], 0 where the index is -1
 * Nothing is allocated; work is enqueued on `stream`; n_queries = 0 is a no-op.  HR_ERR_INVALID_ARG on null
 * pointers or sizes out of range. */
int hr_rerank_topk(const float* scores_dev, const int32_t* seg_dev, int32_t n_queries, int32_t max_cands, int32_t k,
                   int32_t* topk_idx_dev, float* topk_scores_dev, void* stream);

/* ---- introspection for benchmarks ---- */

/* Per-kernel timing for benchmarks.  While enabled, every kernel launch of a scoring call is
 * bracketed by two HIP events on the call's stream, tagged with a kernel class (hr_profile_name:
 * "gemm_gate_up", "attention", ...; hr_profile_count classes).  hr_profile_read waits for the
 * recorded events, returns per class the summed duration in ms and the number of launches
 * (arrays of hr_profile_count entries, host) and clears the record. */
int hr_profile_enable(hr_model* model, int enable);
/* Restrict the timing to the classes whose bit (1 << class index) is set; the default is all classes.  Two
 * event records cost a few microseconds of stream time per launch, which adds up over ~170 launches per call,
 * so a benchmark times only the classes it reports while it measures the whole call. */
int hr_profile_select(hr_model* model, uint32_t class_mask);
int hr_profile_count(void);
const char* hr_profile_name(int idx);
int hr_profile_read(hr_model* model, double* ms_out, int64_t* launches_out);

/* A yardstick for the roofline of the KV-streaming attention (which is bound by reading HBM): one read-only pass over
 * `bytes` (whole KiB are read) of device memory at src_dev (16-byte aligned) with a kernel of the library's own, enqueued
 * on `stream`; time it from outside.  to_lds = 0: 16-byte loads into registers; 1: the direct-to-LDS loads the attention
 * kernel streams pages with.  sink_dev: >= 4 bytes of device memory that receive a fold of what was read (so that no load
 * can be dropped).  HR_ERR_INVALID_ARG on null or misaligned pointers or bytes < 1024. */
int hr_probe_read_bandwidth(const void* src_dev, size_t bytes, void* sink_dev, size_t sink_bytes, int to_lds, void* stream);

/* Name of the kernel family a model / pool combination runs: "mfma" or "generic" ("none" for a null handle); never
 * NULL.  The MFMA attention is only chosen together with the MFMA projections.  hr_attention_path answers for short
 * queries.  One attention work item holds 512 rows (query tokens x query heads per kv head) at 64-wide heads and 256 at
 * 128-wide heads; a scoring call spreads a longer query's rows over up to eight work items (each streams the document),
 * and beyond that (or with HR_NO_DOC_GROUPS=1, which switches the plan off that does the spreading) runs its attention on
 * the generic kernel next to the MFMA projections: same results within the tolerance of the model's dtype, and a
 * document plus query of at most 15000 tokens. */
const char* hr_attention_path(const hr_model* model, const hr_pool* pool);
const char* hr_gemm_path(const hr_model* model);

/* Environment switches, read once per model handle at hr_weights_load.  They exist for A/B runs of the tests and
 * benchmarks (each pair of settings must give the same score bits) and change no result:
 *   HR_FORCE_GENERIC=1      every step on the generic fp32-arithmetic kernels
 *   HR_NO_LAST_SHORTCUT=1   the last layer runs on every token instead of each pair's last one
 *   HR_NO_DOC_GROUPS=1      pairs that share a document are not batched into one attention work item
 *   HR_NO_QUERY_SHARING=1   the first layer's projections are computed for every pair instead of once per distinct query
 *   HR_STREAMS=1            the initial value of hr_rerank_set_streams is 1
 * and one that does change results (within the tolerance): HR_PRECISE_LAYERS=n, the initial value of
 * hr_model_set_precise_layers. */

#ifdef __cplusplus
}
#endif
#endif /* HYPERRERANK_H */
