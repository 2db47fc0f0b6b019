"""Glue used by the GPU parity tests: fills the oracle's paged store and the library's HBM pool
with the same bytes and runs both sides on the same seeded inputs."""

from __future__ import annotations

from typing import List, Optional, Sequence

import numpy as np

from oracle import fp8 as ofp8
from oracle import reranker as orr
from paper_2504_02921_amd import workloads as wlmod

TOL = {"f32": 1e-4, "bf16": 2e-2}     # absolute score tolerance per model dtype (spec bar)


def torch_dtype(name: str):
    import torch
    return {"f32": torch.float32, "bf16": torch.bfloat16}[name]


def round_kv(k64: np.ndarray, kv_dtype: str):
    """float64 [L][D][n_kv][d] -> (torch CPU tensor in the pool dtype, float64 numpy of the same values)."""
    import torch
    t = torch.from_numpy(np.ascontiguousarray(k64)).to(torch_dtype(kv_dtype))
    return t, t.to(torch.float64).numpy()


class Case:
    """One workload instantiated on both sides."""

    def __init__(self, wl: wlmod.Workload, weights, device="cuda:0"):
        from paper_2504_02921_amd import binding as hb
        self.hb = hb
        self.wl, self.w, self.device = wl, weights, device
        m = wl.cfg.model
        self.model = hb.Model(m, weights, device)
        self.pool = hb.KVPool(m.n_layers, m.n_kv_heads, m.head_dim, wl.num_pages, wl.cfg.kv_dtype, device)
        self.opool = orr.PagedKV(m.n_layers, m.n_kv_heads, m.head_dim, 16, wl.cfg.kv_dtype)
        self.oracle_docs = set()

    # -- document KV from the oracle's own stage-one pass (small shapes) --------------------------
    def fill_from_prefill(self, doc_ids: Optional[Sequence[int]] = None):
        wl, m = self.wl, self.wl.cfg.model
        doc_ids = sorted(set(int(d) for d in (wl.pair_doc if doc_ids is None else doc_ids)))
        kvs = orr.doc_prefill(self.w, m, [wl.doc_tokens(d) for d in doc_ids])
        import torch
        for d, (k, v) in zip(doc_ids, kvs):
            pages = wl.pool_doc_pages[d]
            if wl.cfg.kv_dtype == "fp8":
                kc, ks = ofp8.quantize_doc_kv(k)
                vc, vs = ofp8.quantize_doc_kv(v)
                self.opool.write(pages, kc, vc, ks, vs)
                self.pool.write(k.shape[1], pages, torch.from_numpy(kc).to(self.device), torch.from_numpy(vc).to(self.device),
                                torch.from_numpy(ks).to(self.device), torch.from_numpy(vs).to(self.device))
            else:
                kt, k64 = round_kv(k, wl.cfg.kv_dtype)
                vt, v64 = round_kv(v, wl.cfg.kv_dtype)
                self.opool.write(pages, k64, v64)
                self.pool.write(k.shape[1], pages, kt.to(self.device), vt.to(self.device))
            self.oracle_docs.add(d)
        torch.cuda.synchronize()

    # -- opaque synthetic KV (large shapes): GPU pool gets every doc, the oracle only what it scores ----
    def fill_synthetic(self, oracle_doc_ids: Sequence[int], all_docs: bool = True):
        import torch
        wl = self.wl
        want = set(int(d) for d in oracle_doc_ids)
        docs = range(wl.n_docs) if all_docs else sorted(want)
        for d in docs:
            kv = wlmod.synthetic_doc_kv(wl, d, self.device)
            D = int(wl.pool_doc_lens[d])
            pages = wl.pool_doc_pages[d]
            if wl.cfg.kv_dtype == "fp8":
                self.pool.write(D, pages, kv["k"], kv["v"], kv["k_scale"], kv["v_scale"])
            else:
                self.pool.write(D, pages, kv["k"], kv["v"])
            if d in want:
                if wl.cfg.kv_dtype == "fp8":
                    self.opool.write(pages, kv["k"].cpu().numpy(), kv["v"].cpu().numpy(),
                                     kv["k_scale"].cpu().numpy(), kv["v_scale"].cpu().numpy())
                else:
                    self.opool.write(pages, kv["k"].to(torch.float64).cpu().numpy(), kv["v"].to(torch.float64).cpu().numpy())
                self.oracle_docs.add(d)
            torch.cuda.synchronize()      # the source tensors are dropped at the end of each iteration

    def gpu_scores(self, wl: Optional[wlmod.Workload] = None) -> np.ndarray:
        import torch
        wl = self.wl if wl is None else wl
        s = self.model.score(self.pool, wl.page_table, wl.doc_lens, wl.query_tokens, wl.query_lens)
        torch.cuda.synchronize()
        return s.cpu().numpy().astype(np.float64)

    def oracle_scores(self, wl: Optional[wlmod.Workload] = None) -> np.ndarray:
        wl = self.wl if wl is None else wl
        assert all(int(d) in self.oracle_docs or wl.pool_doc_lens[int(d)] == 0 for d in wl.pair_doc)
        return orr.score_cached(self.w, wl.cfg.model, self.opool, wl.page_table, wl.doc_lens, wl.query_tokens, wl.query_lens)

    def close(self):
        self.model.close()
        self.pool.close()


def assert_scores_close(got: np.ndarray, want: np.ndarray, tol: float, what: str = ""):
    assert got.shape == want.shape
    assert np.all(np.isfinite(got)), f"{what}: non-finite scores"
    err = np.abs(got - want)
    assert err.max() <= tol, f"{what}: max |err| {err.max():.3e} > {tol:g} (at pair {int(err.argmax())}; scores ~{np.abs(want).mean():.3f})"


def assert_same_topk_up_to_ties(got: np.ndarray, want: np.ndarray, n_queries: int, n_cands: int, tol: float):
    """Per-query ranking must agree unless every discordant pair is a tie within 2 * tol in the oracle."""
    og, ow = orr.topk_order(got, n_queries, n_cands), orr.topk_order(want, n_queries, n_cands)
    w = want.reshape(n_queries, n_cands)
    for q in range(n_queries):
        if np.array_equal(og[q], ow[q]):
            continue
        rank_g = np.argsort(og[q])
        rank_w = np.argsort(ow[q])
        for i in range(n_cands):
            for j in range(i + 1, n_cands):
                if (rank_g[i] < rank_g[j]) != (rank_w[i] < rank_w[j]):
                    assert abs(w[q, i] - w[q, j]) <= 2 * tol, f"query {q}: candidates {i},{j} swapped beyond tolerance"


def sample_pairs(wl: wlmod.Workload, n: int, seed: int = 0) -> np.ndarray:
    """Seeded sample of pairs that always includes the extreme document / query lengths."""
    rng = np.random.default_rng(seed)
    must = {int(np.argmin(wl.doc_lens)), int(np.argmax(wl.doc_lens)), int(np.argmin(wl.query_lens)), int(np.argmax(wl.query_lens))}
    rest = [i for i in rng.permutation(wl.n_pairs) if i not in must]
    return np.array(sorted(list(must) + rest[: max(0, n - len(must))]), dtype=np.int64)
