"""Pins for the CPU oracle: what the paper and the mathematics fix, not the oracle itself.

 * Section 3.3 Property 1 (lossless two-stage inference): cached-document scoring equals
   one causal pass over [doc ; query].
 * Pair independence (same section): a pair's score does not depend on its batch.
 * Library / textbook reductions: a stock Llama implementation run in float64, torch's
   scaled-dot-product attention, explicit per-row brute force, closed forms.
"""

import dataclasses
import os

import numpy as np
import pytest

from oracle import fp8 as ofp8
from oracle import reranker as orr
from paper_2504_02921_amd import workloads as wlmod

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def small_model(n_layers=2, hidden=64, n_q=4, n_kv=2, d=16, ffn=96, vocab=50, base=10000.0, eps=1e-6, dtype="f32"):
    return wlmod.ModelCfg("small", n_layers, hidden, n_q, n_kv, d, ffn, vocab, base, eps, dtype=dtype)


def build_pool(model, weights, doc_tokens, page_lists, kv_dtype="f32"):
    pool = orr.PagedKV(model.n_layers, model.n_kv_heads, model.head_dim, 16, kv_dtype)
    kvs = orr.doc_prefill(weights, model, doc_tokens)
    for (k, v), pages in zip(kvs, page_lists):
        if kv_dtype == "fp8":
            kc, ks = ofp8.quantize_doc_kv(k)
            vc, vs = ofp8.quantize_doc_kv(v)
            pool.write(pages, kc, vc, ks, vs)
        else:
            pool.write(pages, k, v)
    return pool, kvs


def random_case(model, doc_lens, query_lens, seed=0):
    rng = np.random.default_rng(seed)
    docs = [rng.integers(0, model.vocab, size=n) for n in doc_lens]
    qs = [rng.integers(0, model.vocab, size=n) for n in query_lens]
    n_pages = [(n + 15) // 16 for n in doc_lens]
    perm = rng.permutation(sum(n_pages) + 3)
    offs = np.concatenate([[0], np.cumsum(n_pages)])
    page_lists = [perm[offs[i]:offs[i + 1]] for i in range(len(docs))]
    stride = max(n_pages)
    table = np.full((len(docs), stride), -1, np.int32)
    for i, pg in enumerate(page_lists):
        table[i, :len(pg)] = pg
    return docs, qs, page_lists, table


# ----------------------------------------------------------------------------- Property 1
@pytest.mark.parametrize("n_q,n_kv,doc_lens,query_lens", [
    (4, 2, [32, 16, 48], [5, 1, 8]),          # page-aligned docs, q = 1 included
    (4, 4, [17, 1, 31], [3, 7, 1]),           # ragged tails, one-token doc
    (8, 2, [40, 23], [9, 2]),                 # group of 4
    (6, 2, [20], [4]),                        # group of 3
])
def test_cached_equals_full_recompute(n_q, n_kv, doc_lens, query_lens):
    model = small_model(n_q=n_q, n_kv=n_kv, hidden=16 * n_q)
    w = wlmod.SeededWeights(model, seed=3, std=0.2, gain_jitter=0.2)
    docs, qs, page_lists, table = random_case(model, doc_lens, query_lens, seed=11)
    pool, _ = build_pool(model, w, docs, page_lists)
    cached = orr.score_cached(w, model, pool, table, np.array(doc_lens), np.concatenate(qs), np.array(query_lens))
    full = orr.score_full(w, model, docs, qs)
    assert np.abs(full).max() > 1e-3
    np.testing.assert_allclose(cached, full, rtol=0, atol=1e-10)


def test_cached_equals_full_on_config1_shape():
    cfg = wlmod.scaled(wlmod.CONFIGS["c1_tiny"], n_cands=2)
    wl = wlmod.make_workload(cfg)
    model = cfg.model
    w = wlmod.SeededWeights(model, seed=0)
    docs = [wl.doc_tokens(d) for d in wl.pair_doc]
    pool, _ = build_pool(model, w, docs, [wl.pool_doc_pages[d] for d in wl.pair_doc])
    cached = orr.score_cached(w, model, pool, wl.page_table, wl.doc_lens, wl.query_tokens, wl.query_lens)
    qs = [wl.query_tokens_per_query[q] for q in wl.pair_query]
    full = orr.score_full(w, model, docs, qs)
    np.testing.assert_allclose(cached, full, rtol=0, atol=1e-10)


def test_scores_invariant_to_physical_page_order():
    model = small_model()
    w = wlmod.SeededWeights(model, seed=5, std=0.2, gain_jitter=0.1)
    doc_lens, query_lens = [37, 64, 5], [6, 3, 4]
    docs, qs, pages_a, table_a = random_case(model, doc_lens, query_lens, seed=1)
    _, _, pages_b, table_b = random_case(model, doc_lens, query_lens, seed=2)
    assert any((a != b).any() for a, b in zip(pages_a, pages_b))
    pool_a, _ = build_pool(model, w, docs, pages_a)
    pool_b, _ = build_pool(model, w, docs, pages_b)
    args = (np.array(doc_lens), np.concatenate(qs), np.array(query_lens))
    sa = orr.score_cached(w, model, pool_a, table_a, *args)
    sb = orr.score_cached(w, model, pool_b, table_b, *args)
    assert np.array_equal(sa, sb)          # bit-identical: placement must not enter the arithmetic


def test_pair_independence():
    model = small_model()
    w = wlmod.SeededWeights(model, seed=9, std=0.2)
    doc_lens, query_lens = [33, 18, 50, 16], [4, 9, 2, 5]
    docs, qs, pages, table = random_case(model, doc_lens, query_lens, seed=4)
    pool, _ = build_pool(model, w, docs, pages)
    batch = orr.score_cached(w, model, pool, table, np.array(doc_lens), np.concatenate(qs), np.array(query_lens))
    for p in (2, 0, 3):
        alone = orr.score_cached(w, model, pool, table[p:p + 1], np.array(doc_lens[p:p + 1]), qs[p], np.array(query_lens[p:p + 1]))
        np.testing.assert_allclose(alone[0], batch[p], rtol=0, atol=1e-12)
    order = [3, 1, 0, 2]
    shuffled = orr.score_cached(w, model, pool, table[order], np.array(doc_lens)[order],
                                np.concatenate([qs[i] for i in order]), np.array(query_lens)[order])
    np.testing.assert_allclose(shuffled, batch[order], rtol=0, atol=1e-12)


# ----------------------------------------------------------------------------- attention core
def brute_force_attention(q, k_all, v_all, n_prefix, group):
    """Materialise the full (D+n) x (D+n) lower-triangular mask and loop row by row."""
    total = k_all.shape[0]
    n = total - n_prefix
    mask = np.tril(np.ones((total, total), bool))
    out = np.zeros_like(q)
    d = q.shape[-1]
    for i in range(n):
        row = n_prefix + i
        for a in range(q.shape[1]):
            h = a // group
            logits = np.array([np.dot(q[i, a], k_all[j, h]) / np.sqrt(d) if mask[row, j] else -np.inf
                               for j in range(total)])
            wts = np.exp(logits - logits[np.isfinite(logits)].max())
            wts /= wts.sum()
            out[i, a] = sum(wts[j] * v_all[j, h] for j in range(total))
    return out


@pytest.mark.parametrize("D,n,n_q,n_kv", [(0, 5, 2, 1), (7, 1, 4, 4), (19, 6, 6, 2), (16, 3, 2, 2)])
def test_prefix_attention_matches_brute_force(D, n, n_q, n_kv):
    rng = np.random.default_rng(D * 31 + n)
    d = 8
    q = rng.standard_normal((n, n_q, d))
    k_all = rng.standard_normal((D + n, n_kv, d))
    v_all = rng.standard_normal((D + n, n_kv, d))
    got = orr.prefix_causal_attention(q, k_all[:D], v_all[:D], k_all[D:], v_all[D:])
    want = brute_force_attention(q, k_all, v_all, D, n_q // n_kv)
    np.testing.assert_allclose(got, want, rtol=0, atol=1e-12)


def test_attention_equal_keys_gives_running_mean_of_values():
    rng = np.random.default_rng(0)
    D, n, d = 5, 4, 8
    q = rng.standard_normal((n, 2, d))
    key = rng.standard_normal(d)
    k_all = np.broadcast_to(key, (D + n, 1, d)).copy()
    v_all = rng.standard_normal((D + n, 1, d))
    out = orr.prefix_causal_attention(q, k_all[:D], v_all[:D], k_all[D:], v_all[D:])
    for i in range(n):
        want = v_all[: D + i + 1, 0].mean(axis=0)
        np.testing.assert_allclose(out[i, 0], want, atol=1e-12)
        np.testing.assert_allclose(out[i, 1], want, atol=1e-12)


def test_attention_matches_torch_sdpa_causal():
    import torch
    import torch.nn.functional as F
    rng = np.random.default_rng(2)
    n, n_q, n_kv, d = 11, 6, 2, 16
    q = rng.standard_normal((n, n_q, d))
    k = rng.standard_normal((n, n_kv, d))
    v = rng.standard_normal((n, n_kv, d))
    z = np.zeros((0, n_kv, d))
    got = orr.prefix_causal_attention(q, z, z, k, v)
    tq, tk, tv = (torch.from_numpy(a).permute(1, 0, 2)[None] for a in (q, k, v))
    want = F.scaled_dot_product_attention(tq, tk, tv, is_causal=True, enable_gqa=True)[0].permute(1, 0, 2).numpy()
    np.testing.assert_allclose(got, want, atol=1e-12)
    # splitting the same sequence into a prefix and a suffix changes nothing for the suffix rows
    split = 4
    got2 = orr.prefix_causal_attention(q[split:], k[:split], v[:split], k[split:], v[split:])
    np.testing.assert_allclose(got2, want[split:], atol=1e-12)


def test_gqa_equals_mha_with_repeated_kv_heads():
    rng = np.random.default_rng(3)
    D, n, n_q, n_kv, d = 9, 4, 6, 2, 8
    q = rng.standard_normal((n, n_q, d))
    k = rng.standard_normal((D + n, n_kv, d))
    v = rng.standard_normal((D + n, n_kv, d))
    g = n_q // n_kv
    k_rep, v_rep = np.repeat(k, g, axis=1), np.repeat(v, g, axis=1)
    a = orr.prefix_causal_attention(q, k[:D], v[:D], k[D:], v[D:])
    b = orr.prefix_causal_attention(q, k_rep[:D], v_rep[:D], k_rep[D:], v_rep[D:])
    np.testing.assert_allclose(a, b, atol=1e-13)


# ----------------------------------------------------------------------------- RoPE / RMSNorm / SiLU
def test_rope_known_rotation_and_invariants():
    # d = 2: a single pair, frequency base^0 = 1 -> rotation by pos radians, counter-clockwise
    x = np.array([[[1.0, 0.0]], [[0.0, 1.0]]])
    out = orr.rope(x, np.array([0.5, 0.5]), 10000.0)
    np.testing.assert_allclose(out[0, 0], [np.cos(0.5), np.sin(0.5)], atol=1e-15)
    np.testing.assert_allclose(out[1, 0], [-np.sin(0.5), np.cos(0.5)], atol=1e-15)
    # d = 4, base 100: pair (0,2) rotates by pos, pair (1,3) by pos / 10
    x = np.array([[[1.0, 1.0, 0.0, 0.0]]])
    out = orr.rope(x, np.array([2.0]), 100.0)
    np.testing.assert_allclose(out[0, 0], [np.cos(2.0), np.cos(0.2), np.sin(2.0), np.sin(0.2)], atol=1e-15)
    rng = np.random.default_rng(0)
    q = rng.standard_normal((1, 3, 16))
    k = rng.standard_normal((1, 3, 16))
    np.testing.assert_allclose(orr.rope(q, np.array([0]), 1e4), q, atol=0)           # position 0 is the identity
    for m, n_, s in [(5, 2, 100), (40, 47, 3)]:
        a = (orr.rope(q, np.array([m]), 1e4) * orr.rope(k, np.array([n_]), 1e4)).sum(-1)
        b = (orr.rope(q, np.array([m + s]), 1e4) * orr.rope(k, np.array([n_ + s]), 1e4)).sum(-1)
        np.testing.assert_allclose(a, b, atol=1e-12)                                   # depends on m - n only
        np.testing.assert_allclose(np.linalg.norm(orr.rope(q, np.array([m]), 1e4), axis=-1),
                                   np.linalg.norm(q, axis=-1), atol=1e-12)


def test_rmsnorm_known_values():
    np.testing.assert_allclose(orr.rmsnorm(np.array([[3.0, 4.0]]), np.array([1.0, 2.0]), 0.0),
                               [[3 / np.sqrt(12.5), 8 / np.sqrt(12.5)]], atol=1e-15)
    np.testing.assert_allclose(orr.rmsnorm(np.array([[1.0, 1.0, 1.0, 1.0]]), np.ones(4), 3.0), [[0.5] * 4], atol=1e-15)
    x = np.random.default_rng(1).standard_normal((5, 32))
    y = orr.rmsnorm(x, np.ones(32), 0.0)
    np.testing.assert_allclose(np.sqrt((y * y).mean(-1)), 1.0, atol=1e-12)
    import torch
    import torch.nn.functional as F
    g = np.random.default_rng(2).standard_normal(32)
    want = F.rms_norm(torch.from_numpy(x), (32,), torch.from_numpy(g), 1e-5).numpy()
    np.testing.assert_allclose(orr.rmsnorm(x, g, 1e-5), want, atol=1e-13)


def test_silu_known_values():
    np.testing.assert_allclose(orr.silu(np.array([0.0, 1.0, -1.0])),
                               [0.0, 1 / (1 + np.exp(-1.0)), -1 / (1 + np.exp(1.0))], atol=1e-15)


# ----------------------------------------------------------------------------- whole forward
class ZeroOut:
    """Weights view whose attention-output and down projections are zero."""

    def __init__(self, base):
        self.base = base

    def get(self, kind, layer=-1):
        a = self.base.get(kind, layer)
        return np.zeros_like(a) if kind in ("wo", "wd") else a


def test_zero_output_projections_give_embedding_closed_form():
    model = small_model()
    w = ZeroOut(wlmod.SeededWeights(model, seed=2, std=0.3, gain_jitter=0.3))
    docs, qs, pages, table = random_case(model, [20, 33], [4, 6], seed=8)
    pool, _ = build_pool(model, w, docs, pages)
    got = orr.score_cached(w, model, pool, table, np.array([20, 33]), np.concatenate(qs), np.array([4, 6]))
    E = w.get("embedding").astype(np.float64)
    gain = w.get("final_norm").astype(np.float64)
    for p, qtok in enumerate(qs):
        e = E[qtok[-1]]
        y = e / np.sqrt((e * e).mean() + model.rms_eps) * gain
        want = float(y @ (E[model.yes_id] - E[model.no_id]))
        assert abs(got[p] - want) < 1e-12


def hf_llama(model, w):
    import torch
    from transformers import LlamaConfig, LlamaForCausalLM
    kwargs = dict(vocab_size=model.vocab, hidden_size=model.hidden, intermediate_size=model.ffn,
                  num_hidden_layers=model.n_layers, num_attention_heads=model.n_q_heads,
                  num_key_value_heads=model.n_kv_heads, head_dim=model.head_dim, rms_norm_eps=model.rms_eps,
                  tie_word_embeddings=True, attention_bias=False, mlp_bias=False, max_position_embeddings=4096)
    try:
        c = LlamaConfig(rope_parameters={"rope_type": "default", "rope_theta": float(model.rope_base)}, **kwargs)
    except TypeError:
        c = LlamaConfig(rope_theta=float(model.rope_base), **kwargs)
    c._attn_implementation = "eager"
    net = LlamaForCausalLM(c).double().eval()
    sd = {"model.embed_tokens.weight": w.get("embedding"), "model.norm.weight": w.get("final_norm"),
          "lm_head.weight": w.get("embedding")}
    names = {"wq": "self_attn.q_proj", "wk": "self_attn.k_proj", "wv": "self_attn.v_proj", "wo": "self_attn.o_proj",
             "wg": "mlp.gate_proj", "wu": "mlp.up_proj", "wd": "mlp.down_proj",
             "norm1": "input_layernorm", "norm2": "post_attention_layernorm"}
    for l in range(model.n_layers):
        for k, n in names.items():
            sd[f"model.layers.{l}.{n}.weight"] = w.get(k, l)
    missing = net.load_state_dict({k: torch.from_numpy(np.asarray(v, np.float64)) for k, v in sd.items()}, strict=False)
    assert not [m for m in missing.missing_keys if "rotary" not in m and "lm_head" not in m], missing
    return net


@pytest.mark.parametrize("base", [10000.0, 500000.0])
def test_full_and_cached_match_stock_llama_implementation(base):
    """The decoder block is the Llama-family block: a stock implementation in float64 must agree."""
    import torch
    model = small_model(n_layers=3, hidden=64, n_q=4, n_kv=2, d=16, ffn=112, vocab=60, base=base, eps=1e-5)
    w = wlmod.SeededWeights(model, seed=21, std=0.25, gain_jitter=0.2)
    net = hf_llama(model, w)
    assert abs(float(net.model.rotary_emb.inv_freq[1]) - base ** (-2.0 / model.head_dim)) < 1e-6
    doc_lens, query_lens = [29, 48], [7, 3]
    docs, qs, pages, table = random_case(model, doc_lens, query_lens, seed=5)
    want = []
    with torch.no_grad():
        for dt, qt in zip(docs, qs):
            ids = torch.from_numpy(np.concatenate([dt, qt]))[None]
            logits = net(ids).logits[0, -1]
            want.append(float(logits[model.yes_id] - logits[model.no_id]))
    want = np.array(want)
    full = orr.score_full(w, model, docs, qs)
    pool, _ = build_pool(model, w, docs, pages)
    cached = orr.score_cached(w, model, pool, table, np.array(doc_lens), np.concatenate(qs), np.array(query_lens))
    assert np.abs(want).max() > 1e-2
    # the stock rotary table is built in fp32, hence not 1e-12
    np.testing.assert_allclose(full, want, rtol=0, atol=2e-5)
    np.testing.assert_allclose(cached, want, rtol=0, atol=2e-5)


# ----------------------------------------------------------------------------- paged store
def test_paged_store_roundtrip_and_tail():
    rng = np.random.default_rng(0)
    L, D, n_kv, d = 2, 37, 2, 8
    k = rng.standard_normal((L, D, n_kv, d))
    v = rng.standard_normal((L, D, n_kv, d))
    pool = orr.PagedKV(L, n_kv, d)
    pool.write([9, 2, 5], k, v)
    row = np.array([9, 2, 5, -1, -1])
    for l in range(L):
        gk, gv = pool.gather(l, row, D)
        assert np.array_equal(gk, k[l]) and np.array_equal(gv, v[l])
    gk, _ = pool.gather(0, row, 20)
    assert gk.shape[0] == 20 and np.array_equal(gk, k[0, :20])
    assert np.all(pool.pages[5]["k"][:, 5:] == 0)            # zero-filled tail of the last page
    with pytest.raises(AssertionError):
        pool.write([2], k[:, :16], v[:, :16])                # page already in use


# ----------------------------------------------------------------------------- fp8
def test_e4m3_table_against_format_definition_fixture():
    table = ofp8.e4m3_decode_table()
    with open(os.path.join(GOLDEN, "ocp_e4m3_named_values.txt")) as f:
        rows = [ln.split() for ln in f if ln.strip() and not ln.startswith("#")]
    assert len(rows) >= 8
    for code, value in rows:
        assert table[int(code, 16)] == float(value), (code, value)
    assert np.isnan(table[0x7F]) and np.isnan(table[0xFF]) and np.isnan(table).sum() == 2
    assert np.all(np.diff(table[:0x7F]) > 0)
    assert np.array_equal(table[0x80:0xFF], -table[0x00:0x7F])


def test_e4m3_table_against_torch_dtype():
    import torch
    codes = torch.arange(256, dtype=torch.uint8)
    want = codes.view(torch.float8_e4m3fn).to(torch.float64).numpy()
    got = ofp8.e4m3_decode_table()
    ok = ~np.isnan(want)
    assert np.array_equal(np.isnan(got), np.isnan(want))
    assert np.array_equal(got[ok], want[ok])


def test_e4m3_encode_rounding():
    table = ofp8.e4m3_decode_table()
    finite = np.array([c for c in range(256) if not np.isnan(table[c]) and c != 0x80], dtype=np.uint8)
    assert np.array_equal(ofp8.e4m3_encode(table[finite]), finite)                    # exact values map to themselves
    assert ofp8.e4m3_encode(np.array([1.0625]))[0] == 0x38                            # tie 1.0 | 1.125 -> even (1.0)
    assert ofp8.e4m3_encode(np.array([1.1875]))[0] == 0x3A                            # tie 1.125 | 1.25 -> even (1.25)
    assert ofp8.e4m3_encode(np.array([1.07]))[0] == 0x39
    assert ofp8.e4m3_encode(np.array([-1.07]))[0] == 0xB9
    assert ofp8.e4m3_encode(np.array([1000.0]))[0] == 0x7E and ofp8.e4m3_encode(np.array([-1e9]))[0] == 0xFE
    assert ofp8.e4m3_encode(np.array([2.0 ** -11]))[0] in (0x00,)                      # below half the smallest subnormal
    assert ofp8.e4m3_encode(np.array([2.0 ** -10]))[0] == 0x00                         # tie 0 | 2^-9 -> even (0)
    assert ofp8.e4m3_encode(np.array([1.5 * 2.0 ** -9]))[0] == 0x02                    # tie 1|2 subnormal steps -> even
    import torch
    x = np.random.default_rng(0).standard_normal(20000) * 60
    x = np.clip(x, -448, 448)
    want = torch.from_numpy(x).to(torch.float32).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    got = ofp8.e4m3_encode(x.astype(np.float32))
    assert np.array_equal(got & 0x7F, want & 0x7F) and np.array_equal(got[x != 0] >> 7, want[x != 0] >> 7)


def test_quantize_doc_kv_scales_and_error_bound():
    rng = np.random.default_rng(0)
    L, D, n_kv, d = 2, 40, 2, 8
    x = rng.standard_normal((L, D, n_kv, d)) * np.array([0.1, 5.0])[None, None, :, None]
    x[1, 16:32, 0] = 0.0                                                    # an all-zero (layer, page, head)
    codes, scales = ofp8.quantize_doc_kv(x)
    assert scales.shape == (L, 3, n_kv) and scales.dtype == np.float32
    assert scales[1, 1, 0] == 1.0 and np.all(codes[1, 16:32, 0] == 0)
    amax_last = np.abs(x[0, 32:40, 1]).max()
    assert abs(scales[0, 2, 1] - amax_last / 448.0) < 1e-6 * amax_last        # tail page: valid tokens only
    deq = ofp8.dequantize_doc_kv(codes, scales)
    per_tok_scale = np.repeat(scales.astype(np.float64), 16, axis=1)[:, :D][..., None]
    # relative step of a 3-bit mantissa is 2^-3; half of it, plus the subnormal floor
    assert np.all(np.abs(deq - x) <= np.abs(x) * 2.0 ** -4 + per_tok_scale * 2.0 ** -10 + 1e-12)
    assert (codes & 0x7F).max() == 0x7E                                       # amax maps to the largest code


def test_fp8_pool_scores_close_to_unquantised_and_cached_path_consistent():
    model = small_model()
    w = wlmod.SeededWeights(model, seed=6, std=0.2)
    doc_lens, query_lens = [40, 21], [5, 3]
    docs, qs, pages, table = random_case(model, doc_lens, query_lens, seed=3)
    pool8, kvs = build_pool(model, w, docs, pages, kv_dtype="fp8")
    pool, _ = build_pool(model, w, docs, pages)
    args = (np.array(doc_lens), np.concatenate(qs), np.array(query_lens))
    s8 = orr.score_cached(w, model, pool8, table, *args)
    s = orr.score_cached(w, model, pool, table, *args)
    assert 0 < np.abs(s8 - s).max() < 0.1 * np.abs(s).max() + 0.05
    # gather returns exactly decode(code) * scale
    kc, ks = ofp8.quantize_doc_kv(kvs[0][0])
    gk, _ = pool8.gather(1, table[0], doc_lens[0])
    np.testing.assert_array_equal(gk, ofp8.dequantize_doc_kv(kc, ks)[1])


def test_kv4_known_values_and_properties():
    """The 4-bit transfer format against hand-computed cases and the properties any symmetric 15-level quantiser with
    scale amax / 7 must have: the extreme element is exact, errors are at most half a step, codes of a group hit +-7,
    zero groups stay zero, ties go to the even code, and storing twice changes nothing more."""
    from oracle import kv4
    x = np.zeros((2, 64))
    x[0, :8] = [7.0, -7.0, 3.5, 2.5, 0.5, -0.5, 1.0, 6.49]           # scale 1: ties 3.5 -> 4, 2.5 -> 2, +-0.5 -> 0
    x[0, 32:36] = [0.875, 0.4375, -0.0625, 0.0]                       # scale 0.125 exactly: ties 3.5 -> 4, -0.5 -> 0
    codes, scale = kv4.quantize(x)
    assert codes.dtype == np.int8 and scale.dtype == np.float32 and scale.shape == (2, 2)
    assert codes[0, :8].tolist() == [7, -7, 4, 2, 0, 0, 1, 6]
    assert scale[0, 0] == np.float32(1.0) and scale[0, 1] == np.float32(0.125)
    assert codes[0, 32:36].tolist() == [7, 4, 0, 0]
    assert np.all(codes[1] == 0) and np.all(scale[1] == 1.0)
    y = kv4.dequantize(codes, scale)
    assert y[0, 0] == 7.0 and y[0, 3] == 2.0 and y[0, 32] == 0.875 and y[0, 33] == 0.5 and y[0, 34] == 0.0
    rng = np.random.default_rng(0)
    z = rng.standard_normal((3, 5, 2, 128)).astype(np.float16).astype(np.float64) * 3
    c, sc = kv4.quantize(z)
    g = z.reshape(3, 5, 2, 4, 32)
    assert np.array_equal(np.abs(c).reshape(3, 5, 2, 4, 32).max(-1), np.full((3, 5, 2, 4), 7))
    back = kv4.dequantize(c, sc).reshape(3, 5, 2, 4, 32)
    step = sc.astype(np.float64)[..., None]
    assert np.all(np.abs(back - g) <= step / 2 + np.abs(g) * 2.0 ** -10)     # half a step, plus the rounding to half
    again = kv4.round_trip(back.reshape(z.shape))
    assert np.abs(again - back.reshape(z.shape)).max() <= np.abs(back).max() * 2.0 ** -9   # a second pass is (nearly) idempotent


def test_topk_order_ties_break_by_index():
    s = np.array([0.5, 2.0, 2.0, -1.0, 3.0, 3.0, 3.0, 0.0])
    order = orr.topk_order(s, 2, 4)
    assert order.tolist() == [[1, 2, 0, 3], [0, 1, 2, 3]]


def test_topk_against_brute_force_selection():
    """Per-query selection: compared with repeatedly taking the best remaining candidate (score, then lower
    index), on quantised scores so that ties are common; NaN below everything, -0 equal to +0, short queries padded."""
    rng = np.random.default_rng(5)
    for trial in range(20):
        lens = rng.integers(0, 12, size=rng.integers(1, 6))
        seg = np.concatenate([[0], np.cumsum(lens)])
        s = np.round(rng.normal(size=seg[-1]) * 2) / 2
        s[rng.random(len(s)) < 0.1] = np.nan
        s[rng.random(len(s)) < 0.1] = -0.0
        k = int(rng.integers(1, 8))
        got = orr.topk(s, seg, k)
        for q in range(len(lens)):
            row = list(s[seg[q]:seg[q + 1]])
            key = [(-np.inf if np.isnan(v) else float(v)) for v in row]
            left = list(range(len(row)))
            want = []
            while left and len(want) < k:
                best = left[0]
                for i in left[1:]:
                    if key[i] > key[best]:          # strictly better only: the earlier index keeps equal scores
                        best = i
                want.append(best)
                left.remove(best)
            want += [-1] * (k - len(want))
            assert got[q].tolist() == want, (trial, q)
    # worked example: ties by index, NaN last
    assert orr.topk(np.array([1.0, 3.0, 3.0, np.nan, 2.0]), [0, 5], 4).tolist() == [[1, 2, 4, 0]]
    assert orr.topk(np.array([np.nan, -np.inf]), [0, 2], 3).tolist() == [[0, 1, -1]]


# ----------------------------------------------------------------------------- generators
def test_generator_casts_and_workload_shapes():
    a = np.array([1.0, 1.00390625, 1.01171875, -3.0e-40, 65504.0], np.float32)
    import torch
    want = torch.from_numpy(a).to(torch.bfloat16).view(torch.uint16).numpy()
    assert np.array_equal(wlmod.f32_to_bf16_bits(a), want)
    wl = wlmod.make_workload(wlmod.scaled(wlmod.CONFIGS["c4_ragged"], n_queries=6, n_cands=10, pool_docs=64))
    assert wl.n_pairs == 60 and wl.page_table.shape[0] == 60
    assert wl.doc_lens.min() >= 64 and wl.doc_lens.max() <= 1024 and wl.query_lens.min() >= 8 and wl.query_lens.max() <= 64
    for q in range(6):
        assert len(set(wl.pair_doc[q * 10:(q + 1) * 10].tolist())) == 10             # de-duplicated within a query
    used = np.concatenate(wl.pool_doc_pages)
    assert len(set(used.tolist())) == len(used) == wl.num_pages                      # a permutation of the pool
    for p in range(wl.n_pairs):
        n = (wl.doc_lens[p] + 15) // 16
        assert np.all(wl.page_table[p, :n] >= 0) and np.all(wl.page_table[p, n:] == -1)
    c2 = wlmod.make_workload(wlmod.CONFIGS["c2_qwen0p5b"])
    assert c2.n_pairs == 640 and c2.total_q_tokens == 20480 and c2.kv_stream_bytes() == 640 * 512 * 12288
    assert abs(c2.gemm_flop() - 14.7e12) < 0.1e12


@pytest.mark.timeout(600)
@pytest.mark.parametrize("name,picks", [("c2_qwen0p5b", [0, 333]), ("c4_ragged", [0, 1, -1])])
def test_stored_scores_are_what_the_oracle_computes_today(name, picks):
    """tests/golden/<config>_scores.json (what the GPU suite compares against at the full sizes) against a fresh oracle
    run on a few of their pairs: same seeded inputs, same float64 arithmetic, so the same numbers to rounding order."""
    import json
    import os
    import sys
    golden = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")
    if golden not in sys.path:
        sys.path.insert(0, golden)
    import make_golden
    with open(os.path.join(golden, f"{name}_scores.json")) as f:
        g = json.load(f)
    cfg = wlmod.CONFIGS[name]
    wl = wlmod.make_workload(cfg)
    pairs = np.array(g["pairs"], dtype=np.int64)
    assert np.array_equal(pairs, make_golden.golden_pairs(wl))
    assert g["inputs_sha256"] == make_golden.inputs_digest(wl, pairs)
    stored = np.array([float(x) for x in g["scores"]])
    sel = np.array([pairs[i] for i in picks])
    w = wlmod.SeededWeights(cfg.model, seed=cfg.seed)
    opool = orr.PagedKV(cfg.model.n_layers, cfg.model.n_kv_heads, cfg.model.head_dim, 16, cfg.kv_dtype)
    for d in sorted(set(int(wl.pair_doc[p]) for p in sel)):
        make_golden.write_doc(opool, wl, d)
    sub = wl.subset(sel)
    got = orr.score_cached(w, cfg.model, opool, sub.page_table, sub.doc_lens, sub.query_tokens, sub.query_lens)
    want = np.array([stored[np.searchsorted(pairs, p)] for p in sel])
    np.testing.assert_allclose(got, want, rtol=0, atol=1e-9)
