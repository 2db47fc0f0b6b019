"""Seeded synthetic inputs for the reranker scoring pass.

This module only *draws* data: model shapes, random-init weights, token ids,
document / query lengths, candidate lists, the physical placement of KV pages
and opaque synthetic document KV.  It contains none of the reranker's
arithmetic (no norm, no RoPE, no attention, no quantiser): the CPU oracle and
the HIP library each implement that on their own and both consume the arrays
produced here.  Dtype casts (fp32 -> bf16, fp32 -> fp8) are plain library
conversions applied once so both sides receive identical bytes.

The shapes follow the paper's reranking workloads (Section 3.3, Properties 2
and 3; Section 5 set-up): fixed-size document chunks of a few hundred tokens,
a much shorter query suffix, 5-100 candidates per query, many queries batched.
The corpora themselves are not available; token ids are uniform random.
"""

from __future__ import annotations

import dataclasses
import math
from dataclasses import dataclass
from typing import Dict, List, Optional, Tuple, Union

import numpy as np

PAGE_TOKENS = 16

_LAYER_KINDS = ("wq", "wk", "wv", "wo", "wg", "wu", "wd", "norm1", "norm2")
_KIND_INDEX = {k: i for i, k in enumerate(("embedding", "final_norm") + _LAYER_KINDS)}


# --------------------------------------------------------------------------- #
# configs
# --------------------------------------------------------------------------- #
@dataclass(frozen=True)
class ModelCfg:
    """Decoder-only reranker dimensions (pre-norm, RMSNorm, RoPE, GQA, SwiGLU, tied head)."""

    name: str
    n_layers: int
    hidden: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    ffn: int
    vocab: int
    rope_base: float
    rms_eps: float
    yes_id: int = 1
    no_id: int = 2
    dtype: str = "bf16"  # "f32" | "bf16": storage type of weights and activations

    @property
    def group(self) -> int:
        return self.n_q_heads // self.n_kv_heads

    @property
    def qkv_out(self) -> int:
        return (self.n_q_heads + 2 * self.n_kv_heads) * self.head_dim

    def shape(self, kind: str) -> Tuple[int, ...]:
        h, d = self.hidden, self.head_dim
        return {
            "embedding": (self.vocab, h),
            "final_norm": (h,),
            "wq": (self.n_q_heads * d, h),
            "wk": (self.n_kv_heads * d, h),
            "wv": (self.n_kv_heads * d, h),
            "wo": (h, self.n_q_heads * d),
            "wg": (self.ffn, h),
            "wu": (self.ffn, h),
            "wd": (h, self.ffn),
            "norm1": (h,),
            "norm2": (h,),
        }[kind]

    def gemm_flop_per_token(self) -> float:
        h, d = self.hidden, self.head_dim
        per_layer = h * self.qkv_out + self.n_q_heads * d * h + 3 * h * self.ffn
        return 2.0 * self.n_layers * per_layer

    def kv_bytes_per_token(self, kv_dtype: str) -> int:
        size = {"f32": 4, "bf16": 2, "fp8": 1}[kv_dtype]
        return self.n_layers * 2 * self.n_kv_heads * self.head_dim * size


MODELS: Dict[str, ModelCfg] = {
    "tiny": ModelCfg("tiny", 2, 256, 4, 4, 64, 688, 1000, 10000.0, 1e-6, dtype="f32"),
    "qwen2_0p5b": ModelCfg("qwen2_0p5b", 24, 896, 14, 2, 64, 4864, 32000, 1.0e6, 1e-6),
    "llama3_8b": ModelCfg("llama3_8b", 32, 4096, 32, 8, 128, 14336, 128256, 500000.0, 1e-5),
}

LenSpec = Union[int, Tuple[int, int]]


@dataclass(frozen=True)
class WorkloadCfg:
    name: str
    model: ModelCfg
    n_queries: int
    n_cands: int
    doc_len: LenSpec          # fixed, or inclusive (lo, hi) drawn per pool document
    query_len: LenSpec        # fixed, or inclusive (lo, hi) drawn per query
    kv_dtype: str             # "f32" | "bf16" | "fp8"
    pool_docs: Optional[int] = None   # None: one distinct doc per pair
    zipf_a: Optional[float] = None    # candidate popularity exponent when pool_docs is set
    seed: int = 0

    @property
    def n_pairs(self) -> int:
        return self.n_queries * self.n_cands


CONFIGS: Dict[str, WorkloadCfg] = {
    "c1_tiny": WorkloadCfg("c1_tiny", MODELS["tiny"], 1, 8, 128, 16, "f32"),
    "c2_qwen0p5b": WorkloadCfg("c2_qwen0p5b", MODELS["qwen2_0p5b"], 32, 20, 512, 32, "bf16"),
    "c3_llama8b": WorkloadCfg("c3_llama8b", MODELS["llama3_8b"], 8, 50, 256, 32, "bf16"),
    "c4_ragged": WorkloadCfg("c4_ragged", MODELS["qwen2_0p5b"], 256, 100, (64, 1024), (8, 64), "bf16",
                             pool_docs=8192, zipf_a=1.1),
    "c5_long_fp8": WorkloadCfg("c5_long_fp8", MODELS["llama3_8b"], 4, 100, 2048, 64, "fp8"),
}


def scaled(cfg: WorkloadCfg, **changes) -> WorkloadCfg:
    """Copy of a workload with some fields replaced (model fields via model_<field>=...)."""
    model_changes = {k[6:]: v for k, v in changes.items() if k.startswith("model_")}
    rest = {k: v for k, v in changes.items() if not k.startswith("model_")}
    model = dataclasses.replace(cfg.model, **model_changes) if model_changes else cfg.model
    return dataclasses.replace(cfg, model=model, **rest)


# --------------------------------------------------------------------------- #
# dtype casts (library conversions only)
# --------------------------------------------------------------------------- #
def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even fp32 -> bf16, returned as the uint16 bit pattern."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + bias) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def round_to(a: np.ndarray, dtype: str) -> np.ndarray:
    """fp32 array holding values exactly representable in `dtype` ("f32" | "bf16")."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    if dtype == "f32":
        return a
    if dtype == "bf16":
        return bf16_bits_to_f32(f32_to_bf16_bits(a))
    raise ValueError(dtype)


# --------------------------------------------------------------------------- #
# weights
# --------------------------------------------------------------------------- #
def _n_workers() -> int:
    import os
    try:
        n = len(os.sched_getaffinity(0))
    except AttributeError:
        n = os.cpu_count() or 1
    return max(1, min(16, n))


class SeededWeights:
    """Random-init weights: every matrix ~ N(0, 0.02^2), norm gains 1 (+ optional jitter).

    Tensors are generated on demand from (seed, layer, kind) so an 8B-shaped
    model never has to sit in host memory at once.  Matrices are row-major
    [out][in]; bf16 models get values rounded once to bf16 (returned as fp32
    arrays that hold exactly those values); norm gains are always fp32.
    """

    def __init__(self, model: ModelCfg, seed: int = 0, std: float = 0.02, gain_jitter: float = 0.0):
        self.model = model
        self.seed = seed
        self.std = std
        self.gain_jitter = gain_jitter
        self._embedding = None

    _CHUNK = 1 << 22      # elements per independently seeded block (blocks are drawn in parallel)

    def _rng(self, kind: str, layer: int, block: int = 0) -> np.random.Generator:
        return np.random.Generator(np.random.PCG64(np.random.SeedSequence([self.seed, layer + 1, _KIND_INDEX[kind], block])))

    def _fill_block(self, flat: np.ndarray, kind: str, layer: int, block: int) -> None:
        lo = block * self._CHUNK
        hi = min(flat.shape[0], lo + self._CHUNK)
        part = self._rng(kind, layer, block).standard_normal(hi - lo, dtype=np.float32)
        part *= np.float32(self.std)
        flat[lo:hi] = round_to(part, self.model.dtype)

    def get(self, kind: str, layer: int = -1) -> np.ndarray:
        if kind == "embedding" and self._embedding is not None:
            return self._embedding
        shape = self.model.shape(kind)
        if kind in ("final_norm", "norm1", "norm2"):
            g = np.ones(shape, dtype=np.float32)
            if self.gain_jitter:
                g += (self.gain_jitter * self._rng(kind, layer).standard_normal(shape, dtype=np.float32)).astype(np.float32)
            return g
        n = int(np.prod(shape))
        flat = np.empty(n, dtype=np.float32)
        blocks = (n + self._CHUNK - 1) // self._CHUNK
        if blocks <= 1:
            self._fill_block(flat, kind, layer, 0)
        else:
            from concurrent.futures import ThreadPoolExecutor
            with ThreadPoolExecutor(max_workers=min(blocks, _n_workers())) as ex:
                list(ex.map(lambda b: self._fill_block(flat, kind, layer, b), range(blocks)))
        w = flat.reshape(shape)
        if kind == "embedding":
            self._embedding = w
        return w

    def layer(self, l: int) -> Dict[str, np.ndarray]:
        return {k: self.get(k, l) for k in _LAYER_KINDS}

    def embedding_rows(self, ids: np.ndarray) -> np.ndarray:
        return self.get("embedding")[np.asarray(ids)]


# --------------------------------------------------------------------------- #
# workload: lengths, tokens, candidates, page placement
# --------------------------------------------------------------------------- #
def _draw_len(rng: np.random.Generator, spec: LenSpec, n: int) -> np.ndarray:
    if isinstance(spec, tuple):
        return rng.integers(spec[0], spec[1] + 1, size=n).astype(np.int32)
    return np.full(n, spec, dtype=np.int32)


@dataclass
class Workload:
    cfg: WorkloadCfg
    n_docs: int
    pool_doc_lens: np.ndarray        # [n_docs] int32
    pool_doc_pages: List[np.ndarray]  # per doc: physical page ids int32
    num_pages: int
    query_lens_per_query: np.ndarray  # [n_queries]
    query_tokens_per_query: List[np.ndarray]
    pair_query: np.ndarray           # [P] int32
    pair_doc: np.ndarray             # [P] int32
    # flat per-pair inputs of the scoring call
    page_table: np.ndarray           # [P][pt_stride] int32, -1 padded
    doc_lens: np.ndarray             # [P] int32
    query_lens: np.ndarray           # [P] int32
    query_tokens: np.ndarray         # [T] int32, pair-major

    @property
    def n_pairs(self) -> int:
        return int(self.pair_doc.shape[0])

    @property
    def total_q_tokens(self) -> int:
        return int(self.query_tokens.shape[0])

    def doc_tokens(self, doc_id: int) -> np.ndarray:
        rng = np.random.default_rng(np.random.SeedSequence([self.cfg.seed, 7001, int(doc_id)]))
        return rng.integers(0, self.cfg.model.vocab, size=int(self.pool_doc_lens[doc_id])).astype(np.int32)

    def kv_stream_bytes(self) -> int:
        """Algorithmic document-KV bytes one scoring call must read (all layers)."""
        per_tok = self.cfg.model.kv_bytes_per_token(self.cfg.kv_dtype)
        total = int(self.doc_lens.astype(np.int64).sum()) * per_tok
        if self.cfg.kv_dtype == "fp8":
            pages = int(((self.doc_lens.astype(np.int64) + PAGE_TOKENS - 1) // PAGE_TOKENS).sum())
            total += pages * self.cfg.model.n_layers * self.cfg.model.n_kv_heads * 2 * 4
        return total

    def gemm_flop(self) -> float:
        return self.cfg.model.gemm_flop_per_token() * self.total_q_tokens

    def subset(self, pair_idx) -> "Workload":
        """The same workload restricted to some pairs (pairs are scored independently)."""
        pair_idx = np.asarray(pair_idx, dtype=np.int64)
        starts = np.concatenate([[0], np.cumsum(self.query_lens)])[:-1]
        toks = [self.query_tokens[starts[i]:starts[i] + self.query_lens[i]] for i in pair_idx]
        return dataclasses.replace(
            self,
            pair_query=self.pair_query[pair_idx], pair_doc=self.pair_doc[pair_idx],
            page_table=np.ascontiguousarray(self.page_table[pair_idx]),
            doc_lens=self.doc_lens[pair_idx], query_lens=self.query_lens[pair_idx],
            query_tokens=(np.concatenate(toks).astype(np.int32) if len(toks) else np.zeros(0, np.int32)),
        )


def make_workload(cfg: WorkloadCfg, spare_pages: int = 0) -> Workload:
    """Draw every integer input of one scoring call from cfg.seed."""
    ss = np.random.SeedSequence([cfg.seed, 4242])
    r_len, r_perm, r_q, r_cand = (np.random.default_rng(s) for s in ss.spawn(4))
    n_docs = cfg.pool_docs if cfg.pool_docs is not None else cfg.n_pairs
    pool_doc_lens = _draw_len(r_len, cfg.doc_len, n_docs)
    pages_per_doc = (pool_doc_lens + PAGE_TOKENS - 1) // PAGE_TOKENS
    num_pages = int(pages_per_doc.sum()) + spare_pages
    perm = r_perm.permutation(num_pages).astype(np.int32)      # shuffled physical placement
    offs = np.concatenate([[0], np.cumsum(pages_per_doc)])
    pool_doc_pages = [perm[offs[i]:offs[i + 1]].copy() for i in range(n_docs)]

    qlens = _draw_len(r_q, cfg.query_len, cfg.n_queries)
    qtoks = [r_q.integers(0, cfg.model.vocab, size=int(n)).astype(np.int32) for n in qlens]

    pair_query = np.repeat(np.arange(cfg.n_queries, dtype=np.int32), cfg.n_cands)
    if cfg.pool_docs is None:
        pair_doc = np.arange(cfg.n_pairs, dtype=np.int32)
    else:
        ranks = np.arange(1, n_docs + 1, dtype=np.float64)
        p = ranks ** (-(cfg.zipf_a if cfg.zipf_a is not None else 0.0))
        p /= p.sum()
        pair_doc = np.concatenate([
            r_cand.choice(n_docs, size=cfg.n_cands, replace=False, p=p) for _ in range(cfg.n_queries)
        ]).astype(np.int32)

    doc_lens = pool_doc_lens[pair_doc]
    query_lens = qlens[pair_query]
    pt_stride = int(pages_per_doc.max()) if n_docs else 0
    page_table = np.full((cfg.n_pairs, pt_stride), -1, dtype=np.int32)
    for i, dix in enumerate(pair_doc):
        pg = pool_doc_pages[dix]
        page_table[i, :len(pg)] = pg
    query_tokens = np.concatenate([qtoks[q] for q in pair_query]).astype(np.int32) if cfg.n_pairs else np.zeros(0, np.int32)
    return Workload(cfg, n_docs, pool_doc_lens, pool_doc_pages, num_pages, qlens, qtoks,
                    pair_query, pair_doc, page_table, doc_lens.astype(np.int32),
                    query_lens.astype(np.int32), query_tokens)


# --------------------------------------------------------------------------- #
# opaque synthetic document KV (for shapes whose document prefill is too costly on a CPU)
# --------------------------------------------------------------------------- #
def synthetic_kv_sigma(model: ModelCfg) -> float:
    """Std of a K/V element when RMS-1 activations meet N(0, 0.02^2) projections."""
    return 0.02 * math.sqrt(model.hidden)


_M31 = (1 << 31) - 1


def _hash31(x):
    """Integer mixer on int64 tensors whose values lie in [0, 2^31): multiply / xor-shift rounds kept below 2^31,
    with multipliers below 2^32, so that no product reaches 2^63 (no reliance on wrap-around).  Pure integer
    arithmetic: the same bits on every device."""
    x = (x * 0x9E3779B1) & _M31
    x = ((x ^ (x >> 15)) * 0x45D9F3B) & _M31
    x = ((x ^ (x >> 13)) * 0x2C1B3C6D) & _M31
    x = ((x ^ (x >> 16)) * 0x297A2D39) & _M31
    return x ^ (x >> 15)


def _stream_key(seed: int, doc_id: int, which: int) -> int:
    return int(np.random.SeedSequence([seed, 9001, int(doc_id), which]).generate_state(1)[0]) & _M31


_IH_MEAN = 6 * 1023 / 2.0                                  # six uniform 10-bit fields
_IH_STD = math.sqrt(6 * (1024.0 ** 2 - 1.0) / 12.0)


def _bell_int(n: int, key_a: int, key_b: int, device):
    """n seeded bell-shaped integers (sum of six uniform 10-bit fields of two counter hashes), as an int64 tensor:
    mean _IH_MEAN, std _IH_STD, support within 4.24 std of the mean."""
    import torch
    idx = torch.arange(n, dtype=torch.int64, device=device)
    h1 = _hash31(idx ^ key_a)
    h2 = _hash31((idx + 0x3C6EF35) & _M31 ^ key_b)
    s = (h1 & 1023) + ((h1 >> 10) & 1023) + ((h1 >> 20) & 1023)
    s += (h2 & 1023) + ((h2 >> 10) & 1023) + ((h2 >> 20) & 1023)
    return s


def synthetic_doc_kv(wl: Workload, doc_id: int, device: str = "cpu"):
    """Seeded stand-in for one document's cached KV, logical layout [L][D][n_kv][d].

    Returns a dict of torch tensors on `device`:
      f32 / bf16 pools: {"k", "v"} in that dtype, bell-shaped with std synthetic_kv_sigma.
      fp8 pools: {"k", "v"} as uint8 E4M3 codes, {"k_scale", "v_scale"} fp32
      [L][n_pages][n_kv]; the coded values are bell-shaped with std 96 and the
      scales are drawn directly (log-uniform within a factor sqrt(2) of sigma/96),
      so no quantiser is involved: the scoring pass treats document KV as an opaque input.
    Counter-based: every element is an integer hash of (seed, document, tensor, element index) turned into a value
    by exact float operations (integer -> fp32, one multiplication, one library cast), so the bytes do not depend
    on the device that draws them: the CPU oracle's inputs can be produced without a GPU and the GPU pool filled
    on the device.
    """
    import torch

    m = wl.cfg.model
    D = int(wl.pool_doc_lens[doc_id])
    shape = (m.n_layers, D, m.n_kv_heads, m.head_dim)
    n = m.n_layers * D * m.n_kv_heads * m.head_dim
    assert n < (1 << 31)
    sigma = synthetic_kv_sigma(m)
    seed = wl.cfg.seed
    out = {}
    if wl.cfg.kv_dtype in ("f32", "bf16"):
        dt = torch.float32 if wl.cfg.kv_dtype == "f32" else torch.bfloat16
        unit = float(np.float32(sigma / _IH_STD))
        for w, name in enumerate(("k", "v")):
            s = _bell_int(n, _stream_key(seed, doc_id, 2 * w), _stream_key(seed, doc_id, 2 * w + 1), device)
            x = (s * 2 - int(2 * _IH_MEAN)).to(torch.float32) * (0.5 * unit)
            out[name] = x.to(dt).reshape(shape)
        return out
    if wl.cfg.kv_dtype == "fp8":
        n_pages = (D + PAGE_TOKENS - 1) // PAGE_TOKENS
        unit = float(np.float32(96.0 / _IH_STD))
        table = torch.from_numpy(((sigma / 96.0) * np.exp2(np.arange(256, dtype=np.float64) / 256.0 - 0.5)).astype(np.float32)).to(device)
        ns = m.n_layers * n_pages * m.n_kv_heads
        for w, name in enumerate(("k", "v")):
            s = _bell_int(n, _stream_key(seed, doc_id, 2 * w), _stream_key(seed, doc_id, 2 * w + 1), device)
            x = (s * 2 - int(2 * _IH_MEAN)).to(torch.float32) * (0.5 * unit)
            out[name] = x.clamp_(-448.0, 448.0).to(torch.float8_e4m3fn).view(torch.uint8).reshape(shape)
            pick = _hash31(torch.arange(ns, dtype=torch.int64, device=device) ^ _stream_key(seed, doc_id, 4 + w)) & 255
            out[name + "_scale"] = table[pick].reshape(m.n_layers, n_pages, m.n_kv_heads)
        return out
    raise ValueError(wl.cfg.kv_dtype)
