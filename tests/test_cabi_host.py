"""Host-side behaviour of the C ABI: symbols, layout sizes, page bookkeeping, every error code
that validation can raise before any device work.  No compute call needs a GPU here."""

import ctypes as C
import os
import re

import numpy as np
import pytest

from paper_2504_02921_amd import binding as hb
from paper_2504_02921_amd import workloads as wlmod

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FAKE_DEV = 0x7F0000000000      # 256-aligned, never dereferenced on the host


def i32p(a):
    return a.ctypes.data_as(C.POINTER(C.c_int32))


def test_library_exports_every_declared_symbol():
    text = open(os.path.join(ROOT, "include", "hyperrerank.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    declared = set(re.findall(r"\b(hr_[a-z0-9_]+)\s*\(", text))
    assert declared, "header parse failed"
    for name in declared:
        assert hasattr(hb.lib, name), f"{name} declared but not exported"
    assert declared == set(hb.EXPORTS)


def test_status_strings_are_distinct():
    seen = {hb.lib.hr_status_str(code).decode() for code in hb.STATUS}
    assert len(seen) == len(hb.STATUS)
    assert hb.lib.hr_status_str(-999).decode() == "unknown status"


def test_pool_bytes_and_cfg_validation():
    cfg = hb.make_pool_cfg(24, 2, 64, 20480, "bf16")
    # [layer][page][kv head][K|V][16][d] bf16, then 256 bytes of range counters
    assert hb.hr_kv_pool_bytes(cfg) == 24 * 20480 * 2 * 2 * 16 * 64 * 2 + 256
    cfg8 = hb.make_pool_cfg(32, 8, 128, 100, "fp8")
    data = 32 * 100 * 8 * 2 * 16 * 128
    assert hb.hr_kv_pool_bytes(cfg8) == data + 32 * 100 * 8 * 2 * 4 + 256
    for bad in (dict(head_dim=60), dict(head_dim=0), dict(num_pages=0), dict(n_layers=0), dict(kv_dtype=7), dict(page_tokens=32)):
        c = hb.make_pool_cfg(2, 2, 64, 8, "f32")
        for k, v in bad.items():
            setattr(c, k, v)
        assert hb.hr_kv_pool_bytes(c) == 0
        st, h = hb.hr_kv_pool_create(c, FAKE_DEV, 1 << 30)
        assert st == hb.HR_ERR_INVALID_ARG and not h


def make_pool(num_pages=8, kv="f32", layers=2, n_kv=2, d=64):
    cfg = hb.make_pool_cfg(layers, n_kv, d, num_pages, kv)
    st, h = hb.hr_kv_pool_create(cfg, FAKE_DEV, hb.hr_kv_pool_bytes(cfg))
    assert st == hb.HR_OK
    return cfg, h


def test_pool_create_errors():
    cfg = hb.make_pool_cfg(2, 2, 64, 8, "f32")
    need = hb.hr_kv_pool_bytes(cfg)
    st, _ = hb.hr_kv_pool_create(cfg, FAKE_DEV, need - 1)
    assert st == hb.HR_ERR_POOL_TOO_SMALL
    st, _ = hb.hr_kv_pool_create(cfg, 0, need)
    assert st == hb.HR_ERR_INVALID_ARG
    st, _ = hb.hr_kv_pool_create(cfg, FAKE_DEV + 8, need)
    assert st == hb.HR_ERR_INVALID_ARG
    assert hb.lib.hr_kv_pool_create(C.byref(cfg), C.c_void_p(FAKE_DEV), need, None) == hb.HR_ERR_INVALID_ARG


def test_page_bookkeeping_alloc_free():
    _, h = make_pool(num_pages=8)
    assert hb.lib.hr_kv_pool_free_pages(h) == 8
    out = np.zeros(3, np.int32)
    assert hb.lib.hr_kv_pool_alloc_pages(h, 3, i32p(out)) == hb.HR_OK
    assert out.tolist() == [0, 1, 2] and hb.lib.hr_kv_pool_free_pages(h) == 5
    big = np.zeros(6, np.int32)
    assert hb.lib.hr_kv_pool_alloc_pages(h, 6, i32p(big)) == hb.HR_ERR_POOL_FULL
    assert hb.lib.hr_kv_pool_free_pages(h) == 5
    assert hb.lib.hr_doc_kv_free(h, i32p(np.array([1], np.int32)), 1) == hb.HR_OK
    out2 = np.zeros(2, np.int32)
    assert hb.lib.hr_kv_pool_alloc_pages(h, 2, i32p(out2)) == hb.HR_OK
    assert out2.tolist() == [1, 3]                      # lowest free first
    assert hb.lib.hr_doc_kv_free(h, i32p(np.array([99], np.int32)), 1) == hb.HR_ERR_PAGE_RANGE
    assert hb.lib.hr_kv_pool_alloc_pages(h, 0, i32p(out2)) == hb.HR_ERR_INVALID_ARG
    assert hb.lib.hr_kv_pool_free_pages(None) == hb.HR_ERR_INVALID_ARG
    hb.lib.hr_kv_pool_destroy(h)


def write(h, doc_len, ids, k=FAKE_DEV, v=FAKE_DEV, ks=None, vs=None):
    ids = np.asarray(ids, np.int32)
    return hb.lib.hr_doc_kv_write(h, doc_len, i32p(ids), C.c_void_p(k), C.c_void_p(v), ks, vs, None)


def test_doc_kv_write_validation_leaves_pool_unchanged():
    _, h = make_pool(num_pages=8)
    assert write(h, 0, [0]) == hb.HR_ERR_LEN_RANGE
    assert write(h, -5, [0]) == hb.HR_ERR_LEN_RANGE
    assert write(h, 16 * 9, list(range(9))) == hb.HR_ERR_LEN_RANGE          # more pages than the pool has
    assert write(h, 20, [0, 8]) == hb.HR_ERR_PAGE_RANGE
    assert write(h, 20, [-1, 1]) == hb.HR_ERR_PAGE_RANGE
    assert write(h, 40, [2, 5, 2]) == hb.HR_ERR_PAGE_DUP
    assert hb.lib.hr_doc_kv_write(h, 16, None, C.c_void_p(FAKE_DEV), C.c_void_p(FAKE_DEV), None, None, None) == hb.HR_ERR_INVALID_ARG
    assert write(h, 16, [0], k=0) == hb.HR_ERR_INVALID_ARG
    assert hb.lib.hr_kv_pool_free_pages(h) == 8
    hb.lib.hr_kv_pool_destroy(h)
    _, h8 = make_pool(num_pages=4, kv="fp8")
    assert write(h8, 16, [0]) == hb.HR_ERR_INVALID_ARG                       # fp8 needs both scale arrays
    hb.lib.hr_kv_pool_destroy(h8)


def test_doc_kv_read_validation():
    _, h = make_pool(num_pages=8)
    fake = C.c_void_p(FAKE_DEV)
    ids = (C.c_int32 * 2)(0, 1)

    def read(doc_len, pages, k=fake):
        arr = (C.c_int32 * len(pages))(*pages)
        return hb.lib.hr_doc_kv_read(h, doc_len, arr, k, fake, None, None, None)

    assert hb.lib.hr_doc_kv_read(None, 16, ids, fake, fake, None, None, None) == hb.HR_ERR_INVALID_ARG
    assert hb.lib.hr_doc_kv_read(h, 16, None, fake, fake, None, None, None) == hb.HR_ERR_INVALID_ARG
    assert read(0, [0]) == hb.HR_ERR_LEN_RANGE
    assert read(20, [0, 8]) == hb.HR_ERR_PAGE_RANGE
    assert read(20, [0, 1]) == hb.HR_ERR_TABLE_SHORT                        # nothing has been written there
    got = (C.c_int32 * 2)()
    assert hb.lib.hr_kv_pool_alloc_pages(h, 2, got) == hb.HR_OK
    assert read(20, list(got)) == hb.HR_ERR_TABLE_SHORT                     # reserved is not written
    hb.lib.hr_kv_pool_destroy(h)


def test_page_record_size_and_host_tier_validation():
    """Record size is the page's blocks over all layers and kv heads (+ fp8 scales); every argument error of the page
    move calls is reported before any device work (the record pointer itself is only examined after these)."""
    cfg, h = make_pool(num_pages=8)
    rec = hb.lib.hr_kv_page_record_bytes(h)
    esz = {hb.HR_F32: 4, hb.HR_BF16: 2, hb.HR_FP8_E4M3: 1}[cfg.kv_dtype]
    want = cfg.n_layers * cfg.n_kv_heads * 2 * 16 * cfg.head_dim * esz
    if cfg.kv_dtype == hb.HR_FP8_E4M3:
        want += cfg.n_layers * cfg.n_kv_heads * 2 * 4
    assert rec == (want + 15) // 16 * 16
    assert hb.lib.hr_kv_page_record_bytes(None) == 0
    fake = C.c_void_p(FAKE_DEV)

    def move(fn, pages, pool=h):
        arr = (C.c_int32 * max(len(pages), 1))(*pages)
        return fn(pool, len(pages), arr, fake, None)

    for fn in (hb.lib.hr_kv_pages_out, hb.lib.hr_kv_pages_in):
        assert move(fn, [0], pool=None) == hb.HR_ERR_INVALID_ARG
        assert fn(h, 1, None, fake, None) == hb.HR_ERR_INVALID_ARG
        assert fn(h, -1, (C.c_int32 * 1)(0), fake, None) == hb.HR_ERR_INVALID_ARG
        assert move(fn, [0, 8]) == hb.HR_ERR_PAGE_RANGE
        assert move(fn, [-1]) == hb.HR_ERR_PAGE_RANGE
        assert move(fn, []) == hb.HR_OK                                       # nothing to move
    assert move(hb.lib.hr_kv_pages_out, [0, 1]) == hb.HR_ERR_TABLE_SHORT      # nothing has been written there
    assert move(hb.lib.hr_kv_pages_in, [2, 5, 2]) == hb.HR_ERR_PAGE_DUP
    assert move(hb.lib.hr_kv_pages_in, list(range(8)) + [0]) == hb.HR_ERR_PAGE_DUP
    assert hb.lib.hr_kv_pages_in(h, 1, (C.c_int32 * 1)(3), None, None) == hb.HR_ERR_INVALID_ARG
    assert hb.lib.hr_kv_pages_in(h, 1, (C.c_int32 * 1)(3), C.c_void_p(FAKE_DEV + 4), None) == hb.HR_ERR_INVALID_ARG   # alignment
    assert hb.lib.hr_kv_pool_free_pages(h) == 8                               # nothing was marked by the refused calls
    # 4-bit records exist for 16-bit pools only: 20 bytes per channel of every (layer, kv head)
    assert hb.lib.hr_kv_page_record4_bytes(h) == 0 and hb.lib.hr_kv_page_record4_bytes(None) == 0
    assert move(hb.lib.hr_kv_pages_in4, [3]) == hb.HR_ERR_UNSUPPORTED_SHAPE   # this one is an fp32 pool
    hb.lib.hr_kv_pool_destroy(h)
    cfg16, h16 = make_pool(num_pages=8, kv="bf16", layers=3, n_kv=2, d=128)
    assert hb.lib.hr_kv_page_record4_bytes(h16) == 3 * 2 * 20 * 128
    assert hb.lib.hr_kv_page_record_bytes(h16) == 3 * 2 * 2 * 16 * 128 * 2
    for fn in (hb.lib.hr_kv_pages_out4, hb.lib.hr_kv_pages_in4):
        assert move(fn, [0, 8], pool=h16) == hb.HR_ERR_PAGE_RANGE
        assert move(fn, [], pool=h16) == hb.HR_OK
    assert move(hb.lib.hr_kv_pages_out4, [0], pool=h16) == hb.HR_ERR_TABLE_SHORT
    assert move(hb.lib.hr_kv_pages_in4, [1, 1], pool=h16) == hb.HR_ERR_PAGE_DUP
    hb.lib.hr_kv_pool_destroy(h16)


def test_weights_pack_bytes_and_model_cfg_validation():
    m = wlmod.MODELS["qwen2_0p5b"]
    cfg = hb.make_model_cfg(m)
    layer = (m.qkv_out * m.hidden + m.hidden * m.n_q_heads * m.head_dim + 3 * m.hidden * m.ffn)
    assert hb.hr_weights_pack_bytes(cfg) >= layer * m.n_layers * 2
    assert hb.hr_weights_pack_bytes(cfg) < layer * m.n_layers * 2 * 1.01
    for bad in (dict(n_kv_heads=3), dict(head_dim=48 + 4), dict(yes_id=m.vocab), dict(no_id=-1), dict(dtype=2),
                dict(rope_base=1.0), dict(hidden=0), dict(ffn=0)):
        c = hb.make_model_cfg(m)
        for k, v in bad.items():
            setattr(c, k, v)
        assert hb.hr_weights_pack_bytes(c) == 0, bad
        out = C.c_void_p()
        ptrs = hb.hr_weight_ptrs()
        st = hb.lib.hr_weights_load(C.byref(c), C.byref(ptrs), C.c_void_p(FAKE_DEV), 1 << 40, None, C.byref(out))
        assert st == hb.HR_ERR_INVALID_ARG and not out
    out = C.c_void_p()
    st = hb.lib.hr_weights_load(C.byref(cfg), None, C.c_void_p(FAKE_DEV), 1 << 40, None, C.byref(out))
    assert st == hb.HR_ERR_INVALID_ARG
    ptrs = hb.hr_weight_ptrs()                           # all-null pointers
    st = hb.lib.hr_weights_load(C.byref(cfg), C.byref(ptrs), C.c_void_p(FAKE_DEV), 1 << 40, None, C.byref(out))
    assert st == hb.HR_ERR_INVALID_ARG


def test_null_handles_are_rejected_everywhere():
    assert hb.lib.hr_rerank_workspace_bytes(None, 1, 1, 1) == 0
    assert hb.lib.hr_rerank_full_workspace_bytes(None, 1, 1) == 0
    st = hb.lib.hr_rerank_score(None, None, 1, None, 0, None, None, None, None, 0, None, None)
    assert st == hb.HR_ERR_INVALID_ARG
    st = hb.lib.hr_rerank_score_full(None, 1, None, None, None, None, None, 0, None, None)
    assert st == hb.HR_ERR_INVALID_ARG
    st = hb.lib.hr_rerank_topk(None, None, 1, 4, 1, None, None, None)
    assert st == hb.HR_ERR_INVALID_ARG
    fake = C.c_void_p(FAKE_DEV)
    for n_q, max_c, k in [(-1, 4, 1), (1, 0, 1), (1, 4097, 1), (1, 4, 0), (1, 4, 5)]:      # sizes out of range: rejected before any launch
        assert hb.lib.hr_rerank_topk(fake, fake, n_q, max_c, k, fake, None, None) == hb.HR_ERR_INVALID_ARG
    assert hb.lib.hr_attention_path(None, None).decode() == "none"
    assert hb.lib.hr_gemm_path(None).decode() == "none"
    hb.lib.hr_model_destroy(None)
    hb.lib.hr_kv_pool_destroy(None)


def validate(mcfg, h, table, doc_lens, qtok, qlens, stride=None):
    table = np.ascontiguousarray(table, np.int32)
    dl, qt, ql = (np.ascontiguousarray(a, np.int32) for a in (doc_lens, qtok, qlens))
    stride = table.shape[1] if stride is None else stride
    return hb.lib.hr_rerank_validate(C.byref(mcfg), h, len(dl), i32p(table), stride, i32p(dl), i32p(qt), i32p(ql))


def test_score_argument_validation_on_host():
    m = wlmod.MODELS["tiny"]
    mcfg = hb.make_model_cfg(m)
    _, h = make_pool(num_pages=8, kv="f32", layers=m.n_layers, n_kv=m.n_kv_heads, d=m.head_dim)
    table = np.full((2, 2), -1, np.int32)
    ok_tok = np.array([1, 2, 3, 4, 5], np.int32)
    # documents of length 0 need no pages: the whole argument set is valid without any written page
    assert validate(mcfg, h, table, [0, 0], ok_tok, [2, 3]) == hb.HR_OK
    assert validate(mcfg, h, table, [0, 0], np.array([1, 2, m.vocab, 4, 5]), [2, 3]) == hb.HR_ERR_TOKEN_RANGE
    assert validate(mcfg, h, table, [0, 0], np.array([1, -2, 3, 4, 5]), [2, 3]) == hb.HR_ERR_TOKEN_RANGE
    assert validate(mcfg, h, table, [0, 0], ok_tok, [0, 5]) == hb.HR_ERR_LEN_RANGE
    assert validate(mcfg, h, table, [-1, 0], ok_tok, [2, 3]) == hb.HR_ERR_LEN_RANGE
    assert validate(mcfg, h, table, [0, 20000], ok_tok, [2, 3], stride=4000) in (hb.HR_ERR_LEN_RANGE, hb.HR_ERR_TABLE_SHORT)
    assert validate(mcfg, h, table, [40, 0], ok_tok, [2, 3]) == hb.HR_ERR_TABLE_SHORT           # needs 3 pages, stride 2
    assert validate(mcfg, h, table, [20, 0], ok_tok, [2, 3]) == hb.HR_ERR_TABLE_SHORT           # -1 inside the row
    t2 = table.copy(); t2[0] = [3, 9]
    assert validate(mcfg, h, t2, [20, 0], ok_tok, [2, 3]) == hb.HR_ERR_TABLE_SHORT              # page 3 never written
    t2[0] = [9, 3]
    assert validate(mcfg, h, t2, [20, 0], ok_tok, [2, 3]) == hb.HR_ERR_PAGE_RANGE
    assert hb.lib.hr_rerank_validate(C.byref(mcfg), h, -1, None, 0, None, None, None) == hb.HR_ERR_INVALID_ARG
    assert hb.lib.hr_rerank_validate(C.byref(mcfg), h, 2, None, 0, None, None, None) == hb.HR_ERR_INVALID_ARG
    assert hb.lib.hr_rerank_validate(C.byref(mcfg), h, 0, None, 0, None, None, None) == hb.HR_OK   # empty batch
    hb.lib.hr_kv_pool_destroy(h)
    # pool / model disagreement
    for kw in (dict(layers=m.n_layers + 1), dict(n_kv=2), dict(d=128), dict(kv="bf16")):
        args = dict(layers=m.n_layers, n_kv=m.n_kv_heads, d=m.head_dim, kv="f32")
        args.update(kw)
        _, hp = make_pool(num_pages=4, **args)
        assert validate(mcfg, hp, table, [0, 0], ok_tok, [2, 3]) == hb.HR_ERR_MISMATCH, kw
        hb.lib.hr_kv_pool_destroy(hp)


def test_write_without_device_reports_device_error_and_changes_nothing():
    import torch
    if torch.cuda.is_available():
        pytest.skip("needs a machine without a GPU")
    _, h = make_pool(num_pages=4)
    assert write(h, 20, [1, 2]) == hb.HR_ERR_DEVICE
    assert hb.lib.hr_kv_pool_free_pages(h) == 4
    hb.lib.hr_kv_pool_destroy(h)
