"""End-to-end walk through the library on one GPU: prefill a few documents into a paged pool, score every (query,
document) pair with only the query tokens run through the layers, pick each query's best candidates, move a document
to pinned host memory and back (16-bit records, then 4-bit ones).  Random weights and token ids; run as `python -m paper_2504_02921_amd.demo`."""

import numpy as np


def main(n_queries: int = 3, n_docs: int = 6, doc_len: int = 200, query_len: int = 24, top_k: int = 2, verbose: bool = True):
    import torch

    from . import binding as hb
    from . import workloads as wlmod

    dev = "cuda:0"
    cfg = wlmod.ModelCfg("demo", 4, 512, 8, 2, 64, 1408, 4096, 1e6, 1e-6, dtype="bf16")     # a small Qwen2-shaped decoder
    weights = wlmod.SeededWeights(cfg, seed=1, std=0.05)
    model = hb.Model(cfg, weights, dev)
    rng = np.random.default_rng(0)

    # stage one: every document's K/V of every layer, computed once and kept in pool pages
    pages_per_doc = (doc_len + hb.PAGE_TOKENS - 1) // hb.PAGE_TOKENS
    pool = hb.KVPool(cfg.n_layers, cfg.n_kv_heads, cfg.head_dim, n_docs * pages_per_doc + 8, "bf16", dev)
    docs = [rng.integers(0, cfg.vocab, doc_len).astype(np.int32) for _ in range(n_docs)]
    doc_pages = [pool.alloc(pages_per_doc) for _ in range(n_docs)]
    model.doc_prefill(pool, docs, doc_pages)

    # stage two: each query against every document; only the query tokens go through the layers
    queries = [rng.integers(0, cfg.vocab, query_len).astype(np.int32) for _ in range(n_queries)]
    page_table = np.stack([doc_pages[d] for _ in range(n_queries) for d in range(n_docs)]).astype(np.int32)
    doc_lens = np.full(n_queries * n_docs, doc_len, np.int32)
    q_tokens = np.concatenate([queries[q] for q in range(n_queries) for _ in range(n_docs)])
    q_lens = np.full(n_queries * n_docs, query_len, np.int32)
    scores = model.score(pool, page_table, doc_lens, q_tokens, q_lens)
    seg = np.arange(0, n_queries * n_docs + 1, n_docs)
    best = hb.rerank_topk(scores, seg, top_k)
    torch.cuda.synchronize()

    # the same scores without reuse: the full [document ; query] sequence per pair
    full = model.score_full([docs[d] for _ in range(n_queries) for d in range(n_docs)],
                            [queries[q] for q in range(n_queries) for _ in range(n_docs)])
    torch.cuda.synchronize()
    gap = float((scores - full).abs().max())

    # host tier: evict document 0 to pinned host memory, free its pages, bring it back at other pages
    rec = torch.empty(pages_per_doc * pool.page_record_bytes, dtype=torch.uint8, pin_memory=True)
    pool.pages_out(doc_pages[0], rec)
    torch.cuda.synchronize()
    pool.free(doc_pages[0])
    spare = pool.alloc(8)                      # the lowest free pages: the spare ones are not among them any more
    new_pages = pool.alloc(pages_per_doc)
    pool.free(spare)
    pool.pages_in(new_pages, rec)
    page_table2 = page_table.copy()
    page_table2[0::n_docs] = new_pages
    again = model.score(pool, page_table2, doc_lens, q_tokens, q_lens)
    torch.cuda.synchronize()
    same = bool(torch.equal(scores, again))

    # the same through 4-bit records: a third of the bytes over the bus, scores change by the quantisation
    rec4 = torch.empty(pages_per_doc * pool.page_record4_bytes, dtype=torch.uint8, pin_memory=True)
    pool.pages_out4(new_pages, rec4)
    torch.cuda.synchronize()
    pool.free(new_pages)
    pool.pages_in4(new_pages, rec4)
    lossy = model.score(pool, page_table2, doc_lens, q_tokens, q_lens)
    torch.cuda.synchronize()
    change4 = float((lossy - scores).abs().max())

    if verbose:
        for q in range(n_queries):
            print(f"query {q}: best documents {best[q].tolist()}  scores {[round(float(scores[q * n_docs + int(d)]), 4) for d in best[q]]}")
        print(f"max |reuse - full recompute| = {gap:.2e}; scores after the host-tier round trip identical: {same}; "
              f"after a round trip of one document in 4 bits they move by at most {change4:.2e}")
    model.close()
    pool.close()
    return scores.cpu().numpy(), best.cpu().numpy(), gap, same


if __name__ == "__main__":
    main()
