"""hr_rerank_score_static (the entry point that allocates nothing: its workspace is a static device array inside
the library) against hr_rerank_score on the same inputs, through the C ABI: same kernels, so the same bits; and
both against the CPU oracle.  Two calls in a row, the second with a smaller input, because the array keeps the
previous call's contents."""

import ctypes as C

import numpy as np
import pytest

from paper_2504_02921_amd import workloads as wlmod

import helpers as H

pytestmark = pytest.mark.gpu


def _static_scores(case, wl, out):
    import torch
    s = case.model.score_static(case.pool, wl.page_table, wl.doc_lens, wl.query_tokens, wl.query_lens, out)
    torch.cuda.synchronize()
    return s.cpu().numpy().astype(np.float64)


@pytest.mark.parametrize("dtype,d,n_q,n_kv,kv,tol", [("bf16", 64, 8, 2, "bf16", 2e-2), ("bf16", 128, 4, 1, "fp8", 2e-2),
                                                     ("f32", 32, 4, 2, "f32", 1e-4)])
def test_static_scratch_entry_point_matches_the_workspace_one(dtype, d, n_q, n_kv, kv, tol):
    import torch
    hb = __import__("paper_2504_02921_amd.binding", fromlist=["x"])
    model = wlmod.ModelCfg("static", 2, 256, n_q, n_kv, d, 320, 500, 10000.0, 1e-6, dtype=dtype)
    cfg = wlmod.WorkloadCfg("static", model, 4, 5, (20, 150), (3, 40), kv, pool_docs=9, zipf_a=0.4, seed=d + n_q)
    w = wlmod.SeededWeights(model, seed=21, std=0.05, gain_jitter=0.1)
    wl = wlmod.make_workload(cfg, spare_pages=3)
    case = H.Case(wl, w)
    try:
        case.fill_from_prefill()
        assert int(hb.lib.hr_rerank_static_scratch_bytes()) == 128 << 20
        out = torch.full((wl.n_pairs,), float("nan"), dtype=torch.float32, device="cuda:0")
        want_all = case.gpu_scores()                                   # hr_rerank_score, caller's workspace
        oracle_all = case.oracle_scores()
        H.assert_scores_close(want_all, oracle_all, tol, "workspace entry point")
        # first call: the whole batch
        got_all = _static_scores(case, wl, out)
        np.testing.assert_array_equal(got_all, want_all)
        # second call, smaller input (other pairs, fewer tokens): the array still holds the first call's data
        sub = wl.subset(np.array([7, 2, 11]))
        want_sub = case.gpu_scores(sub)
        free_before = torch.cuda.mem_get_info()[0]
        out.fill_(float("nan"))
        torch.cuda.synchronize()
        got_sub = _static_scores(case, sub, out)
        assert torch.cuda.mem_get_info()[0] == free_before             # no device memory was taken
        np.testing.assert_array_equal(got_sub, want_sub)
        H.assert_scores_close(got_sub, oracle_all[[7, 2, 11]], tol, "static entry point, second call")
        assert np.all(np.isnan(out[3:].cpu().numpy()))                 # nothing written past the call's pairs
        # and the big one again after the small one
        np.testing.assert_array_equal(_static_scores(case, wl, out), want_all)
    finally:
        case.close()


def test_static_scratch_entry_point_rejects_what_does_not_fit():
    import torch
    hb = __import__("paper_2504_02921_amd.binding", fromlist=["x"])
    model = wlmod.ModelCfg("static_big", 1, 1024, 16, 4, 64, 4096, 500, 10000.0, 1e-6, dtype="bf16")
    cfg = wlmod.WorkloadCfg("static_big", model, 1, 2, 16, 32, "bf16", seed=3)
    w = wlmod.SeededWeights(model, seed=22)
    wl = wlmod.make_workload(cfg)
    case = H.Case(wl, w)
    try:
        case.fill_synthetic(oracle_doc_ids=[])
        out = torch.zeros(4096, dtype=torch.float32, device="cuda:0")
        # the same two pairs repeated until the workspace passes 128 MiB (2048 pairs x 32 tokens: x alone is 256 MiB)
        reps = 1024
        pt = np.tile(wl.page_table, (reps, 1))
        dl, ql = np.tile(wl.doc_lens, reps), np.tile(wl.query_lens, reps)
        qt = np.tile(wl.query_tokens, reps)
        with pytest.raises(hb.HrError) as e:
            case.model.score_static(case.pool, pt, dl, qt, ql, out)
        assert e.value.status == hb.HR_ERR_WORKSPACE_SMALL
        torch.cuda.synchronize()
        assert float(out.abs().sum()) == 0.0                           # nothing was enqueued
        # the workspace entry point takes the same call
        got = case.model.score(case.pool, pt, dl, qt, ql)
        torch.cuda.synchronize()
        g = got.cpu().numpy()
        assert np.all(np.isfinite(g)) and np.array_equal(g[:2], g[2:4])
        # and a call that fits still works afterwards
        s = case.model.score_static(case.pool, wl.page_table, wl.doc_lens, wl.query_tokens, wl.query_lens, out)
        torch.cuda.synchronize()
        np.testing.assert_array_equal(s.cpu().numpy(), g[:2])
    finally:
        case.close()
