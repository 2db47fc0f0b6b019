"""Fixed-shape scoring plans (hr_rerank_plan_*): the same scores as hr_rerank_score, bit for bit, from a call that is
stream work only, recorded into a HIP graph and replayed with other pages and query tokens of the same shape
(Section 4.2: the static document-prefix | query-suffix layout is what makes the reranker's execution capturable)."""

import numpy as np
import pytest

from paper_2504_02921_amd import workloads as wlmod

import helpers as H

pytestmark = pytest.mark.gpu


def _same_shape_other_inputs(wl, seed):
    """Other documents (a permutation of the pairs' page-table rows: every document has the same length here) and other
    query tokens for the same lengths."""
    rng = np.random.default_rng(seed)
    perm = rng.permutation(wl.n_pairs)
    toks = rng.integers(0, wl.cfg.model.vocab, size=wl.total_q_tokens).astype(np.int32)
    return np.ascontiguousarray(wl.page_table[perm]), toks, perm


@pytest.mark.parametrize("dtype,d,n_q,n_kv,kv,n_split,tol,qlen", [
    ("bf16", 64, 14, 2, "bf16", 0, 2e-2, (3, 40)), ("bf16", 128, 8, 2, "fp8", 1, 2e-2, (3, 40)), ("f32", 32, 4, 2, "f32", 0, 1e-4, (3, 40)),
    ("bf16", 64, 16, 2, "bf16", 0, 2e-2, (70, 100)),     # up to 800 rows per kv head: the plan spreads a pair over two work items
])
def test_plan_runs_and_graph_replays_give_the_bits_of_the_plain_call(dtype, d, n_q, n_kv, kv, n_split, tol, qlen):
    import torch
    model = wlmod.ModelCfg("plan", 3, 256, n_q, n_kv, d, 320, 500, 10000.0, 1e-6, dtype=dtype)
    cfg = wlmod.WorkloadCfg("plan", model, 2, 5, 70, qlen, kv, seed=d + n_q)
    w = wlmod.SeededWeights(model, seed=23, std=0.05, gain_jitter=0.1)
    wl = wlmod.make_workload(cfg, spare_pages=3)
    case = H.Case(wl, w)
    plan = None
    try:
        case.fill_from_prefill()
        if n_split:
            case.model.set_precise_layers(n_split)
        hb = case.hb
        want = case.gpu_scores()                                        # hr_rerank_score
        H.assert_scores_close(want, case.oracle_scores(), tol, "plain call")
        plan = hb.Plan(case.model, case.pool, wl.doc_lens, wl.query_lens, wl.page_table.shape[1])
        out = torch.full((wl.n_pairs,), float("nan"), dtype=torch.float32, device="cuda:0")
        with pytest.raises(hb.HrError):
            plan.run(out)                                               # no inputs yet
        plan.set_inputs(wl.page_table, wl.query_tokens)
        plan.run(out)                                                   # eager, also the first launch of every kernel
        torch.cuda.synchronize()
        np.testing.assert_array_equal(out.cpu().numpy().astype(np.float64), want)

        graph = torch.cuda.CUDAGraph()
        out.fill_(float("nan"))
        torch.cuda.synchronize()
        with torch.cuda.graph(graph):
            plan.run(out)
        torch.cuda.synchronize()
        for rep in range(3):
            out.fill_(float("nan"))
            # eager work of the same library between the replays, on the same model handle and pool
            other = case.gpu_scores(wl.subset(np.array([rep, rep + 1])))
            np.testing.assert_array_equal(other, want[[rep, rep + 1]])
            graph.replay()
            torch.cuda.synchronize()
            np.testing.assert_array_equal(out.cpu().numpy().astype(np.float64), want)

        # other pages and tokens of the same shape: the recorded launches are replayed as they are
        for seed in (1, 2):
            pt2, toks2, perm = _same_shape_other_inputs(wl, seed)
            import dataclasses
            wl2 = dataclasses.replace(wl, page_table=pt2, query_tokens=toks2, pair_doc=wl.pair_doc[perm])
            want2 = case.gpu_scores(wl2)
            torch.cuda.synchronize()
            plan.set_inputs(pt2, toks2)
            out.fill_(float("nan"))
            graph.replay()
            torch.cuda.synchronize()
            np.testing.assert_array_equal(out.cpu().numpy().astype(np.float64), want2)
            assert np.abs(want2 - want).max() > 1e-3
        # rejected inputs leave the plan as it was
        bad = wl.page_table.copy()
        bad[0, 0] = wl.num_pages + 5
        with pytest.raises(hb.HrError) as e:
            plan.set_inputs(bad, wl.query_tokens)
        assert e.value.status == hb.HR_ERR_PAGE_RANGE
        graph.replay()
        torch.cuda.synchronize()
        np.testing.assert_array_equal(out.cpu().numpy().astype(np.float64), want2)
        del graph
    finally:
        if plan is not None:
            plan.close()
        case.close()


def test_plan_rejects_shapes_and_workspaces_that_do_not_fit():
    import ctypes as C
    import torch
    model = wlmod.ModelCfg("plan", 2, 256, 4, 2, 64, 320, 500, 10000.0, 1e-6, dtype="bf16")
    cfg = wlmod.WorkloadCfg("plan", model, 1, 3, 40, 8, "bf16", seed=2)
    w = wlmod.SeededWeights(model, seed=24, std=0.05)
    wl = wlmod.make_workload(cfg)
    case = H.Case(wl, w)
    try:
        hb = case.hb
        ws = torch.empty(1 << 20, dtype=torch.uint8, device="cuda:0")
        dl, ql = hb._i32(wl.doc_lens), hb._i32(wl.query_lens)
        out = C.c_void_p()

        def create(n, dlens, qlens, stride, nbytes):
            return hb.lib.hr_rerank_plan_create(case.model.handle, case.pool.handle, n, hb._i32p(dlens), hb._i32p(qlens), stride,
                                                C.c_void_p(ws.data_ptr()), nbytes, C.byref(out))
        assert create(3, dl, ql, 3, 1024) == hb.HR_ERR_WORKSPACE_SMALL
        assert create(3, dl, ql, 2, ws.numel()) == hb.HR_ERR_TABLE_SHORT          # 40 tokens need 3 pages
        assert create(0, dl, ql, 3, ws.numel()) == hb.HR_ERR_INVALID_ARG
        assert create(3, dl, hb._i32([8, 0, 8]), 3, ws.numel()) == hb.HR_ERR_LEN_RANGE
        assert out.value is None
    finally:
        case.close()
