"""TEST INFRASTRUCTURE - plain CPU oracle of the reranker scoring pass (float64 numpy).

What it computes
----------------
The paper's Property 1 (Section 3.3): because a decoder-only reranker uses a
lower-triangular attention mask and its input is ordered [document ; query]
(Appendix C), scoring the concatenation in one pass gives exactly the result
of (i) running the document alone and keeping every layer's K/V, then
(ii) running only the query tokens, at positions continuing after the
document, with attention over the cached document K/V plus the causal part of
the query.  The pair structure (each document scored against the query on its
own, document at the start of the sequence) is what makes the cache reusable
across queries.

Two routes are written out here:
  * `score_full`   - the definition: one causal forward over [doc ; query].
  * `score_cached` - the two-stage form the GPU library implements: document
    K/V kept in a paged store (Section 4.2's static "document prefix | query
    suffix" KV layout, with the prefix held in 16-token pages), query pass on
    top of it.
The model maths (pre-norm blocks, RMSNorm, rotate-half RoPE, grouped-query
attention with 1/sqrt(d) scaling, SwiGLU, tied yes/no head) is not spelled out
by the paper; it is the standard decoder block of the model families the
workloads are shaped after.

Everything is float64; stored KV may carry the rounding of the pool's dtype
(f32 / bf16 values, or fp8 codes with scales) because those bytes are inputs.
No blocking, fusion or reordering: linear maps are single matmuls over the
stacked token rows, attention is an explicit masked softmax per head.

Only tests, the smoke check and the benchmark's CPU-baseline leg may import
this file.  It imports nothing from the GPU package.
"""

from __future__ import annotations

from typing import Callable, Dict, List, Optional, Sequence, Tuple

import numpy as np

from . import fp8 as _fp8

F64 = np.float64


# --------------------------------------------------------------------------- #
# building blocks
# --------------------------------------------------------------------------- #
def rmsnorm(x: np.ndarray, gain: np.ndarray, eps: float) -> np.ndarray:
    """y = x / sqrt(mean(x^2) + eps) * gain, over the last axis."""
    x = np.asarray(x, F64)
    ms = np.mean(x * x, axis=-1, keepdims=True)
    return x / np.sqrt(ms + eps) * np.asarray(gain, F64)


def rope(x: np.ndarray, pos: np.ndarray, base: float) -> np.ndarray:
    """Rotary embedding, rotate-half pairing: element j pairs with j + d/2.

    x [n][heads][d], pos [n].  angle[n][j] = pos[n] * base^(-2j/d), j < d/2.
    out[j] = x[j] cos - x[j+d/2] sin ; out[j+d/2] = x[j+d/2] cos + x[j] sin.
    """
    x = np.asarray(x, F64)
    d = x.shape[-1]
    half = d // 2
    inv_freq = F64(base) ** (-2.0 * np.arange(half, dtype=F64) / d)
    ang = np.asarray(pos, F64)[:, None] * inv_freq[None, :]          # [n][half]
    c, s = np.cos(ang)[:, None, :], np.sin(ang)[:, None, :]
    x1, x2 = x[..., :half], x[..., half:]
    return np.concatenate([x1 * c - x2 * s, x2 * c + x1 * s], axis=-1)


def softmax_masked(s: np.ndarray, visible: np.ndarray) -> np.ndarray:
    """Row softmax over the visible entries only (max-subtracted)."""
    s = np.where(visible, s, -np.inf)
    m = s.max(axis=-1, keepdims=True)
    e = np.where(visible, np.exp(s - m), 0.0)
    return e / e.sum(axis=-1, keepdims=True)


def prefix_causal_attention(q: np.ndarray, k_pre: np.ndarray, v_pre: np.ndarray,
                            k_new: np.ndarray, v_new: np.ndarray) -> np.ndarray:
    """Grouped-query attention of n new tokens over [prefix ; new tokens].

    q [n][n_q][d]; k_pre, v_pre [D][n_kv][d] (every prefix key visible to every row);
    k_new, v_new [n][n_kv][d] (row i sees new keys 0..i).  Query head a uses kv head
    a // (n_q / n_kv).  Returns [n][n_q][d].
    """
    n, n_q, d = q.shape
    D, n_kv = k_pre.shape[0], k_new.shape[1]
    g = n_q // n_kv
    keys = np.concatenate([k_pre, k_new], axis=0)        # [D+n][n_kv][d]
    vals = np.concatenate([v_pre, v_new], axis=0)
    visible = np.concatenate([np.ones((n, D), bool), np.tril(np.ones((n, n), bool))], axis=1)
    out = np.empty((n, n_q, d), F64)
    for a in range(n_q):
        h = a // g
        s = (q[:, a, :] @ keys[:, h, :].T) / np.sqrt(F64(d))
        p = softmax_masked(s, visible)
        out[:, a, :] = p @ vals[:, h, :]
    return out


def silu(x: np.ndarray) -> np.ndarray:
    return x / (1.0 + np.exp(-x))


# --------------------------------------------------------------------------- #
# paged document-KV store (the oracle's own, sparse, logical layout)
# --------------------------------------------------------------------------- #
class PagedKV:
    """Document K/V kept in fixed-size pages addressed by physical page id.

    Pages hold `page_tokens` tokens of one document for all layers and kv heads.
    kv_dtype "f32"/"bf16": pages store the given values (already rounded by the
    caller).  "fp8": pages store E4M3 codes plus one K and one V scale per
    (layer, kv head); reads return decode(code) * scale.  A short last page is
    zero-filled; readers cut it with the document length.
    """

    def __init__(self, n_layers: int, n_kv_heads: int, head_dim: int, page_tokens: int = 16, kv_dtype: str = "f32"):
        self.L, self.n_kv, self.d, self.pt, self.kv_dtype = n_layers, n_kv_heads, head_dim, page_tokens, kv_dtype
        self.pages: Dict[int, dict] = {}

    def write(self, page_ids: Sequence[int], k: np.ndarray, v: np.ndarray,
              k_scale: Optional[np.ndarray] = None, v_scale: Optional[np.ndarray] = None) -> None:
        """k, v [L][D][n_kv][d] (values, or uint8 codes for fp8 with scales [L][n_pages][n_kv])."""
        L, D = k.shape[0], k.shape[1]
        n_pages = (D + self.pt - 1) // self.pt
        assert L == self.L and len(page_ids) == n_pages and len(set(int(p) for p in page_ids)) == n_pages
        store_t = np.uint8 if self.kv_dtype == "fp8" else F64
        for i, pid in enumerate(page_ids):
            pid = int(pid)
            assert pid >= 0 and pid not in self.pages, "page already in use"
            t0, t1 = i * self.pt, min(D, (i + 1) * self.pt)
            pk = np.zeros((L, self.pt, self.n_kv, self.d), store_t)
            pv = np.zeros((L, self.pt, self.n_kv, self.d), store_t)
            pk[:, : t1 - t0] = k[:, t0:t1]
            pv[:, : t1 - t0] = v[:, t0:t1]
            page = {"k": pk, "v": pv}
            if self.kv_dtype == "fp8":
                page["ks"] = np.asarray(k_scale[:, i, :], F64).copy()      # [L][n_kv]
                page["vs"] = np.asarray(v_scale[:, i, :], F64).copy()
            self.pages[pid] = page

    def gather(self, layer: int, page_row: np.ndarray, doc_len: int) -> Tuple[np.ndarray, np.ndarray]:
        """K, V [doc_len][n_kv][d] float64 of one document at one layer, through its page-table row."""
        n_pages = (doc_len + self.pt - 1) // self.pt
        ks, vs = [], []
        for i in range(n_pages):
            page = self.pages[int(page_row[i])]
            pk, pv = page["k"][layer], page["v"][layer]
            if self.kv_dtype == "fp8":
                pk = _fp8.e4m3_decode(pk) * page["ks"][layer][None, :, None]
                pv = _fp8.e4m3_decode(pv) * page["vs"][layer][None, :, None]
            ks.append(np.asarray(pk, F64))
            vs.append(np.asarray(pv, F64))
        if not ks:
            z = np.zeros((0, self.n_kv, self.d), F64)
            return z, z.copy()
        return np.concatenate(ks, axis=0)[:doc_len], np.concatenate(vs, axis=0)[:doc_len]


# --------------------------------------------------------------------------- #
# decoder forward
# --------------------------------------------------------------------------- #
PrefixFn = Callable[[int, int], Tuple[np.ndarray, np.ndarray]]   # (layer, seq index) -> (K, V) [D][n_kv][d]


def decoder_forward(weights, cfg, seqs: List[np.ndarray], prefix_lens: Optional[Sequence[int]] = None,
                    prefix_kv: Optional[PrefixFn] = None, keep_kv: bool = False):
    """Run token sequences through all layers.

    weights: object with .get(kind, layer) -> array ([out][in] matrices: "wq","wk","wv","wo",
             "wg","wu","wd"; gains "norm1","norm2"; "embedding" [V][H]; "final_norm").
    cfg:     object with n_layers, hidden, n_q_heads, n_kv_heads, head_dim, rope_base, rms_eps.
    seqs[i]: the new token ids of sequence i; they sit at positions prefix_lens[i] + 0,1,...
             and attend to prefix_kv(layer, i) (all visible) plus themselves causally.
    Returns (final hidden states per sequence [n_i][H], kv) where kv[i] = (K, V)
    [L][n_i][n_kv][d] post-RoPE if keep_kv.
    """
    n_seq = len(seqs)
    prefix_lens = [0] * n_seq if prefix_lens is None else [int(p) for p in prefix_lens]
    lens = [len(s) for s in seqs]
    bounds = np.concatenate([[0], np.cumsum(lens)]).astype(int)
    tokens = np.concatenate([np.asarray(s, np.int64) for s in seqs]) if n_seq else np.zeros(0, np.int64)
    pos = np.concatenate([prefix_lens[i] + np.arange(lens[i]) for i in range(n_seq)]) if n_seq else np.zeros(0)
    emb = weights.get("embedding", -1)
    x = np.asarray(emb[tokens], F64)                                   # [T][H]
    n_q, n_kv, d = cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim
    kv_out = [(np.empty((cfg.n_layers, n, n_kv, d), F64), np.empty((cfg.n_layers, n, n_kv, d), F64)) for n in lens] \
        if keep_kv else None
    empty = np.zeros((0, n_kv, d), F64)

    for l in range(cfg.n_layers):
        w = {k: np.asarray(weights.get(k, l), F64) for k in ("wq", "wk", "wv", "wo", "wg", "wu", "wd", "norm1", "norm2")}
        h = rmsnorm(x, w["norm1"], cfg.rms_eps)
        q = (h @ w["wq"].T).reshape(-1, n_q, d)
        k = (h @ w["wk"].T).reshape(-1, n_kv, d)
        v = (h @ w["wv"].T).reshape(-1, n_kv, d)
        q = rope(q, pos, cfg.rope_base)
        k = rope(k, pos, cfg.rope_base)
        attn = np.empty_like(q)
        for i in range(n_seq):
            a, b = bounds[i], bounds[i + 1]
            kp, vp = prefix_kv(l, i) if (prefix_kv is not None and prefix_lens[i] > 0) else (empty, empty)
            assert kp.shape[0] == prefix_lens[i]
            attn[a:b] = prefix_causal_attention(q[a:b], kp, vp, k[a:b], v[a:b])
            if keep_kv:
                kv_out[i][0][l] = k[a:b]
                kv_out[i][1][l] = v[a:b]
        x = x + attn.reshape(-1, n_q * d) @ w["wo"].T
        h2 = rmsnorm(x, w["norm2"], cfg.rms_eps)
        x = x + (silu(h2 @ w["wg"].T) * (h2 @ w["wu"].T)) @ w["wd"].T
    hidden = [x[bounds[i]:bounds[i + 1]] for i in range(n_seq)]
    return hidden, kv_out


def yes_no_score(weights, cfg, last_hidden: np.ndarray) -> np.ndarray:
    """Final RMSNorm, then logit[yes] - logit[no] with the tied embedding rows as the head."""
    emb = weights.get("embedding", -1)
    y = rmsnorm(last_hidden, weights.get("final_norm", -1), cfg.rms_eps)
    return y @ np.asarray(emb[cfg.yes_id], F64) - y @ np.asarray(emb[cfg.no_id], F64)


def score_full(weights, cfg, doc_tokens: List[np.ndarray], query_tokens: List[np.ndarray]) -> np.ndarray:
    """Definition: causal forward over [doc ; query] per pair, score at the last position."""
    seqs = [np.concatenate([np.asarray(dt), np.asarray(qt)]) for dt, qt in zip(doc_tokens, query_tokens)]
    hidden, _ = decoder_forward(weights, cfg, seqs)
    last = np.stack([h[-1] for h in hidden]) if hidden else np.zeros((0, cfg.hidden))
    return yes_no_score(weights, cfg, last)


def doc_prefill(weights, cfg, doc_tokens: List[np.ndarray]):
    """Stage one: documents alone at positions 0.., returning per doc (K, V) [L][D][n_kv][d] post-RoPE."""
    _, kv = decoder_forward(weights, cfg, [np.asarray(t) for t in doc_tokens], keep_kv=True)
    return kv


def score_cached(weights, cfg, pool: PagedKV, page_table: np.ndarray, doc_lens: np.ndarray,
                 query_tokens: np.ndarray, query_lens: np.ndarray) -> np.ndarray:
    """Stage two: only the query tokens are computed; document K/V come from the paged store.

    page_table [P][stride] physical page ids (-1 padded), doc_lens [P], query_tokens flat [sum q],
    query_lens [P].  Returns scores [P] (float64).
    """
    P = len(doc_lens)
    starts = np.concatenate([[0], np.cumsum(query_lens)]).astype(int)
    seqs = [np.asarray(query_tokens[starts[p]:starts[p + 1]]) for p in range(P)]

    def prefix(layer: int, p: int):
        return pool.gather(layer, page_table[p], int(doc_lens[p]))

    hidden, _ = decoder_forward(weights, cfg, seqs, prefix_lens=doc_lens, prefix_kv=prefix)
    last = np.stack([h[-1] for h in hidden]) if hidden else np.zeros((0, cfg.hidden))
    return yes_no_score(weights, cfg, last)


def topk(scores: np.ndarray, seg_offsets: Sequence[int], k: int) -> np.ndarray:
    """Per-query selection (Section 3.1: the reranker's scores pick the top-k candidates): for query i over pairs
    seg_offsets[i] .. seg_offsets[i+1]-1, the indices (inside the segment) of the k best, best first; score descending,
    index ascending among equal scores, NaN below every number, -1 where the query has fewer than k candidates."""
    s = np.asarray(scores, F64)
    out = np.full((len(seg_offsets) - 1, k), -1, dtype=np.int64)
    for i in range(len(seg_offsets) - 1):
        row = s[seg_offsets[i]:seg_offsets[i + 1]]
        key = np.where(np.isnan(row), -np.inf, row) + 0.0          # + 0.0 turns -0 into +0
        order = np.argsort(-key, kind="stable")                      # stable: equal keys keep ascending index
        out[i, :min(k, len(row))] = order[:k]
    return out


def topk_order(scores: np.ndarray, n_queries: int, n_cands: int) -> np.ndarray:
    """Per-query candidate ranking: score descending, candidate index ascending on ties."""
    s = np.asarray(scores, F64).reshape(n_queries, n_cands)
    return np.stack([np.lexsort((np.arange(n_cands), -row)) for row in s])
