#!/usr/bin/env python3
"""Benchmark of the reranker scoring pass (query suffix over cached document KV) on one MI355X.

One "step" = one hr_rerank_score call over the whole workload (all pairs, all layers), inputs
(weights, document-KV pool) resident in HBM before the timed region.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload c2_qwen0p5b]

The timed steps run the way the library runs them: in one piece, or (where the library chooses so for
the size of the call) as two halves on two streams; config.streams says which.
Besides the headline pairs/s the line carries
  roofline            the kernel class with the largest share of the step (per-kernel HIP events,
                      recorded by the library on the stream it launches on), measured in K more steps
                      with the second stream switched off, where the kernel has the chip to itself
  one_stream          the rate of those steps
  roofline_attention  the KV-streaming attention kernel against HBM peak
  ceilings            yardsticks on the same device from plain library calls (a copy-like kernel, the
                      vendor GEMM on a large square and on this workload's projection shapes)
  cpu_baseline        the CPU oracle timed on a bounded sample of the same pairs
  no_reuse            the same GPU running the full [doc ; query] prefill on a few pairs
  doc_prefill         stage one on the device: documents prefilled into pool pages (ingest rate)
  host_tier           the same batch when every document's pages first come from pinned host memory
                      (bus-inclusive rate, page-in overlapped with scoring; never `value`)
  host_tier_4bit      the same with 4-bit records in the tier (16-bit pools)
"""

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import numpy as np

HBM_PEAK_GBS = 8000.0
MFMA_BF16_PEAK_TFLOPS = 2500.0
FP32_VECTOR_PEAK_TFLOPS = 157.3


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="c2_qwen0p5b")
    ap.add_argument("--cpu-pairs", type=int, default=0, help="pairs for the CPU-oracle leg (0 = pick for ~15 s)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-reuse-pairs", type=int, default=256, help="pairs for the no-reuse reference (0 = skip)")
    ap.add_argument("--no-events", action="store_true", help="do not record per-kernel events during the timed steps")
    ap.add_argument("--prefill-docs", type=int, default=128, help="documents for the document-prefill (ingest) leg (0 = skip)")
    ap.add_argument("--host-tier-batches", type=int, default=6,
                    help="batches of the paged leg: every batch's documents come from pinned host memory (0 = skip)")
    ap.add_argument("--no-ceilings", action="store_true", help="skip the vendor-library yardsticks (copy kernel, library GEMM)")
    ap.add_argument("--calibration-copy-mib", type=int, default=0,
                    help="also run a plain device copy of this many MiB (known traffic, for scaling rocprofv3 byte counters)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        log("bench.py: this build measures ONE GPU only (pairs are independent, so they shard over GPUs with no collective). "
            "Run with --gpus 1.")
        sys.exit(2)

    import torch
    from paper_2504_02921_amd import binding as hb
    from paper_2504_02921_amd import workloads as wlmod

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = "cuda:0"
    cfg = wlmod.CONFIGS[args.workload]
    m = cfg.model
    t0 = time.time()
    wl = wlmod.make_workload(cfg)
    weights = wlmod.SeededWeights(m, seed=cfg.seed)
    model = hb.Model(m, weights, dev)
    pool = hb.KVPool(m.n_layers, m.n_kv_heads, m.head_dim, wl.num_pages, cfg.kv_dtype, dev)
    for d in range(wl.n_docs):
        kv = wlmod.synthetic_doc_kv(wl, d, dev)
        if cfg.kv_dtype == "fp8":
            pool.write(int(wl.pool_doc_lens[d]), wl.pool_doc_pages[d], kv["k"], kv["v"], kv["k_scale"], kv["v_scale"])
        else:
            pool.write(int(wl.pool_doc_lens[d]), wl.pool_doc_pages[d], kv["k"], kv["v"])
        torch.cuda.synchronize()
    log(f"setup {time.time() - t0:.1f}s: {wl.n_pairs} pairs, {wl.total_q_tokens} query tokens, pool {pool.mem.numel() / 1e9:.2f} GB, "
        f"gemm={model.gemm_path()} attention={model.attention_path(pool)}")

    scores = torch.empty(wl.n_pairs, dtype=torch.float32, device=dev)
    if args.calibration_copy_mib > 0:
        src = torch.ones(args.calibration_copy_mib << 20, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        for _ in range(3):
            torch.bitwise_not(src, out=dst)     # a plain elementwise kernel with a name of its own: reads N, writes N
        torch.cuda.synchronize()
        del src, dst

    def step():
        model.score(pool, wl.page_table, wl.doc_lens, wl.query_tokens, wl.query_lens, out=scores)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    # The library may run a large call as two halves on two streams (one half's kernels fill the CUs that the other half's
    # last round of GEMM tiles leaves idle).  The timed region measures what it chooses for this size.  A kernel's own duration is then
    # no longer a statement about the kernel: it includes waiting for CUs the other half's kernel holds.  So the
    # per-kernel figures come from steps with the second stream switched off, where every kernel has the chip to itself:
    # two survey steps before the timed region time every kernel class (the breakdown, and which class is dominant);
    # K more such steps after it bracket only the dominant class and attention (two event records cost a few
    # microseconds of stream time per launch, ~6 % of a step when all ~170 launches are bracketed) and give the
    # rooflines.  The timed region itself records no events (on two streams they cost more than they tell).
    streams = 1 if os.environ.get("HR_STREAMS", "") == "1" else 2
    model.set_streams(streams)
    parts = model.parts(wl.total_q_tokens) if model.attention_path(pool) == "mfma" else 1     # what the library does at this size
    survey = {}
    if not args.no_events:
        model.set_streams(1)
        model.profile_select(None)
        model.profile_enable(True)
        for _ in range(2):
            step()
        torch.cuda.synchronize()
        survey = model.profile_read()
        dominant = max(survey, key=lambda k: survey[k]["ms"])
        if dominant != "attention" and dominant not in ("gemm_qkv", "gemm_o", "gemm_gate_up", "gemm_down"):
            dominant = "gemm_gate_up"
        model.profile_enable(False)
        model.set_streams(streams)
        step()
        torch.cuda.synchronize()
    # no collector pause inside a timed region (a full collection over the workload's arrays takes ~45 ms, two steps)
    import gc
    gc.collect()
    gc.disable()
    t1 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t1
    ms_per_step = dt / args.steps * 1e3
    pairs_per_s = wl.n_pairs / (dt / args.steps)
    assert bool(torch.isfinite(scores).all()), "non-finite scores"
    scores_timed = scores.clone()
    prof = {}
    single = None
    if not args.no_events:
        model.set_streams(1)
        model.profile_select(sorted({dominant, "attention"}))
        model.profile_enable(True)
        step()
        torch.cuda.synchronize()
        model.profile_read()
        t2 = time.perf_counter()
        for _ in range(args.steps):
            step()
        torch.cuda.synchronize()
        dt1 = time.perf_counter() - t2
        prof = model.profile_read()
        single = {"ms_per_step": round(dt1 / args.steps * 1e3, 4), "value": round(wl.n_pairs / (dt1 / args.steps), 2), "unit": "pairs/s",
                  "note": "the same steps on the caller's stream only (hr_rerank_set_streams(1)); the rooflines are measured here"}
        assert torch.equal(scores, scores_timed), "one-stream and two-stream scores differ"
        model.set_streams(streams)
    model.profile_enable(False)
    model.profile_select(None)
    gc.enable()

    # HBM bytes per launch measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (recorded summary, see profiles/)
    traffic = {}
    try:
        with open(os.path.join(ROOT, "profiles", "hbm_traffic.json")) as f:
            traffic = json.load(f).get(cfg.name, {})
    except (OSError, ValueError):
        pass

    # ---- rooflines from the per-kernel events ------------------------------------------------
    T = wl.total_q_tokens
    H, d, F = m.hidden, m.head_dim, m.ffn
    nq = m.n_q_heads * d
    # In the last layer only each pair's last token goes through the O, gate/up and down projections (P rows instead
    # of T; the library does this whenever the MFMA kernels run, and a test checks the scores are bit-identical), so the
    # algorithmic flop of an average launch of those classes is ((L - 1) T + P) / (L T) of a full-size launch.
    P, L = wl.n_pairs, m.n_layers
    shortened = (model.gemm_path() == "mfma" and model.attention_path(pool) == "mfma" and T > P
                 and os.environ.get("HR_NO_LAST_SHORTCUT", "0") != "1")
    tail = ((L - 1) * T + P) / (L * T) if shortened else 1.0
    flop_per_launch = {
        "gemm_qkv": 2.0 * T * H * m.qkv_out, "gemm_o": 2.0 * T * nq * H * tail,
        "gemm_gate_up": 2.0 * T * H * 2 * F * tail, "gemm_down": 2.0 * T * F * H * tail,
    }
    kv_bytes_per_launch = wl.kv_stream_bytes() / m.n_layers
    roofline = None
    roof_attn = None
    breakdown = {}
    if prof:
        total_ms = sum(v["ms"] for v in survey.values()) or 1.0
        for name, v in survey.items():                  # from the survey steps (all classes timed), not the timed region
            if v["launches"]:
                breakdown[name] = {"ms_per_step": round(v["ms"] / 2, 4), "launches_per_step": v["launches"] // 2,
                                   "share": round(v["ms"] / total_ms, 4)}

        def gemm_roof(name):
            avg_s = prof[name]["ms"] / prof[name]["launches"] * 1e-3
            if model.gemm_path() == "mfma":
                ach = flop_per_launch[name] / avg_s / 1e12
                return {"kernel": name, "bound": "mfma", "achieved": round(ach, 2), "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                        "frac": round(ach / MFMA_BF16_PEAK_TFLOPS, 4), "traffic": traffic.get(name), "avg_launch_ms": round(avg_s * 1e3, 4),
                        "algorithmic_flop_per_launch": flop_per_launch[name],
                        "launches_measured": prof[name]["launches"]}
            ach = flop_per_launch[name] / avg_s / 1e12
            return {"kernel": name, "bound": "alu", "achieved": round(ach, 3), "peak": FP32_VECTOR_PEAK_TFLOPS, "unit": "TFLOP/s",
                    "frac": round(ach / FP32_VECTOR_PEAK_TFLOPS, 4), "traffic": None, "avg_launch_ms": round(avg_s * 1e3, 4)}

        def attn_roof():
            avg_s = prof["attention"]["ms"] / prof["attention"]["launches"] * 1e-3
            ach = kv_bytes_per_launch / avg_s / 1e9
            return {"kernel": "attention", "bound": "hbm", "achieved": round(ach, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                    "frac": round(ach / HBM_PEAK_GBS, 4), "traffic": traffic.get("attention"), "avg_launch_ms": round(avg_s * 1e3, 4),
                    "algorithmic_bytes_per_launch": int(kv_bytes_per_launch)}

        roof_attn = attn_roof()
        roofline = roof_attn if dominant == "attention" else gemm_roof(dominant)
        gemm_ms = sum(survey[k]["ms"] for k in flop_per_launch)
        gemm_all = {"achieved_tflops": round(sum(flop_per_launch.values()) * L * 2 / (gemm_ms * 1e-3) / 1e12, 2),
                    "note": "all four projections, from the survey steps"}
    else:
        gemm_all = None

    # ---- what this device gives to plain library calls (yardsticks, not part of the scoring path): a 1 GiB copy-like
    # kernel for the memory side, the vendor GEMM on a large square and on the dominant projection's own shape
    ceilings = None
    if not args.no_ceilings and model.gemm_path() == "mfma":
        def timed(fn, n):
            for _ in range(3):
                fn()
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(n):
                fn()
            e1.record()
            torch.cuda.synchronize()
            return e0.elapsed_time(e1) / n * 1e-3
        src = torch.zeros(1 << 28, dtype=torch.int32, device=dev)
        dst = torch.empty_like(src)
        t_copy = timed(lambda: torch.bitwise_not(src, out=dst), 10)
        del src, dst
        ceilings = {"hbm_copy_GBps": round(2 * (1 << 30) / t_copy / 1e9, 1),
                    "note": "torch.bitwise_not over 1 GiB (read + write); torch.matmul in half precision (the vendor library), without the "
                            "fused epilogues of this path"}
        shapes = {"square_8192": (8192, 8192, 8192)}
        if T >= 1024:
            shapes["gate_up_shape"] = (T, 2 * m.ffn, m.hidden)
            shapes["down_shape"] = (T, m.hidden, m.ffn)
        for key, (mm, nn, kk) in shapes.items():
            a_ = torch.randn(mm, kk, device=dev, dtype=torch.float16) * 0.1
            b_ = torch.randn(nn, kk, device=dev, dtype=torch.float16) * 0.1
            c_ = torch.empty(mm, nn, device=dev, dtype=torch.float16)
            t_mm = timed(lambda: torch.matmul(a_, b_.t(), out=c_), 10)
            ceilings["matmul_" + key] = {"M": mm, "N": nn, "K": kk, "ms": round(t_mm * 1e3, 4), "TFLOPs": round(2.0 * mm * nn * kk / t_mm / 1e12, 1)}
            del a_, b_, c_
        if roofline and roofline.get("bound") == "mfma":
            roofline["frac_of_library_square_gemm"] = round(roofline["achieved"] / ceilings["matmul_square_8192"]["TFLOPs"], 4)
        if roof_attn:
            roof_attn["frac_of_copy_kernel"] = round(roof_attn["achieved"] / ceilings["hbm_copy_GBps"], 4)

    # ---- same-GPU no-reuse reference on a few pairs ------------------------------------------
    no_reuse = None
    if args.no_reuse_pairs > 0:
        n = min(args.no_reuse_pairs, wl.n_pairs)
        docs = [wl.doc_tokens(int(dd)) for dd in wl.pair_doc[:n]]
        qs = [wl.query_tokens_per_query[int(q)] for q in wl.pair_query[:n]]
        try:
            model.score_full(docs, qs)
            torch.cuda.synchronize()
            tt = time.perf_counter()
            model.score_full(docs, qs)
            torch.cuda.synchronize()
            el = time.perf_counter() - tt
            no_reuse = {"value": round(n / el, 2), "unit": "pairs/s", "pairs": n,
                        "note": "full [doc ; query] prefill per pair on the same GPU, random doc tokens of the same lengths"}
        except hb.HrError as e:
            no_reuse = {"value": None, "note": str(e)}

    # ---- stage one on the device: documents prefilled straight into pool pages (ingest rate) ---------
    doc_prefill = None
    if args.prefill_docs > 0:
        nd = min(args.prefill_docs, wl.n_docs)
        toks = [wl.doc_tokens(d) for d in range(nd)]
        pages = [wl.pool_doc_pages[d] for d in range(nd)]
        n_tok = int(sum(len(t) for t in toks))
        try:
            pool_p = hb.KVPool(m.n_layers, m.n_kv_heads, m.head_dim, wl.num_pages, cfg.kv_dtype, dev)
            best = None
            for _ in range(2):
                torch.cuda.synchronize()
                tt = time.perf_counter()
                model.doc_prefill(pool_p, toks, pages)
                torch.cuda.synchronize()
                el = time.perf_counter() - tt
                best = el if best is None else min(best, el)
                pool_p.free(np.concatenate(pages))
            doc_prefill = {"value": round(n_tok / best, 1), "unit": "document tokens/s", "docs": nd, "docs_per_s": round(nd / best, 1),
                           "note": "hr_doc_prefill: random document tokens of the workload's lengths, K/V of every layer written to pool pages"
                                   + (" (quantised to fp8 as stored)" if cfg.kv_dtype == "fp8" else "")}
            pool_p.close()
            del pool_p
        except hb.HrError as e:
            doc_prefill = {"value": None, "note": str(e)}

    # ---- host tier: every batch's document pages are paged in from pinned host memory ----------------
    # Two pools alternate: while one batch is scored from one of them, the next batch's pages arrive in the other on a
    # second stream.  The rate includes the bus (it is not `value`): with every document cold it is the bus that
    # bounds it.
    host_tier = None
    host_tier4 = None
    if args.host_tier_batches > 0:
        all_pages = np.concatenate([wl.pool_doc_pages[d] for d in range(wl.n_docs)]).astype(np.int32)

        def tier_leg(rec, out_fn, in_fn, exact):
            tier_bytes = len(all_pages) * rec
            if tier_bytes > 16e9:
                return {"value": None, "note": f"skipped: {tier_bytes / 1e9:.1f} GB of page records (leg capped at 16 GB of pinned memory)"}
            tier = torch.empty(tier_bytes, dtype=torch.uint8, pin_memory=True)
            pool_b = hb.KVPool(m.n_layers, m.n_kv_heads, m.head_dim, wl.num_pages, cfg.kv_dtype, dev)
            torch.cuda.synchronize()
            tt = time.perf_counter()
            out_fn(pool, all_pages, tier)
            torch.cuda.synchronize()
            out_s = time.perf_counter() - tt
            tt = time.perf_counter()
            in_fn(pool_b, all_pages, tier)
            torch.cuda.synchronize()
            in_s = time.perf_counter() - tt
            scores_b = torch.empty_like(scores)
            pools = [pool, pool_b]
            B = args.host_tier_batches
            side, main_s = torch.cuda.Stream(), torch.cuda.current_stream()
            ev_sc = []
            torch.cuda.synchronize()
            tt = time.perf_counter()
            for b in range(B):
                pl = pools[b % 2]
                if b >= 2:
                    side.wait_event(ev_sc[b - 2])                  # this pool's previous batch has been scored
                pl.free(all_pages)
                with torch.cuda.stream(side):
                    in_fn(pl, all_pages, tier)
                    ev_in = torch.cuda.Event()
                    ev_in.record()
                main_s.wait_event(ev_in)
                model.score(pl, wl.page_table, wl.doc_lens, wl.query_tokens, wl.query_lens, out=scores_b)
                ev = torch.cuda.Event()
                ev.record()
                ev_sc.append(ev)
            torch.cuda.synchronize()
            el = time.perf_counter() - tt
            diff = float((scores - scores_b).abs().max())
            if exact:
                assert diff == 0.0, "scores from paged-in documents differ"
            res = {"value": round(B * wl.n_pairs / el, 2), "unit": "pairs/s", "batches": B,
                   "bytes_per_batch": int(tier_bytes), "page_record_bytes": int(rec),
                   "page_in_GBps": round(tier_bytes / in_s / 1e9, 2), "page_out_GBps": round(tier_bytes / out_s / 1e9, 2),
                   "max_abs_score_change": diff}
            del tier, pool_b
            return res

        host_tier = tier_leg(pool.page_record_bytes, lambda p, ids, t: p.pages_out(ids, t), lambda p, ids, t: p.pages_in(ids, t), True)
        if host_tier.get("value") is not None:
            host_tier["note"] = ("every document of every batch paged in from pinned host memory (hr_kv_pages_in on a second stream, "
                                 "two pools alternating); includes the first batch's unoverlapped page-in")
        if cfg.kv_dtype == "bf16":
            # after the 16-bit leg both pools hold the original pages again, so the 4-bit records are made from those
            host_tier4 = tier_leg(pool.page_record4_bytes, lambda p, ids, t: p.pages_out4(ids, t), lambda p, ids, t: p.pages_in4(ids, t), False)
            if host_tier4.get("value") is not None:
                host_tier4["note"] = ("the same with 4-bit records (hr_kv_pages_in4: quantised in the tier, expanded to 16 bits as they arrive); "
                                      "max_abs_score_change is against the scores from the unquantised documents")
            # the leg leaves quantised documents in the pool: put the originals back for what follows
            for d in range(wl.n_docs):
                kv = wlmod.synthetic_doc_kv(wl, d, dev)
                pool.free(wl.pool_doc_pages[d])
                pool.write(int(wl.pool_doc_lens[d]), wl.pool_doc_pages[d], kv["k"], kv["v"])
                torch.cuda.synchronize()

    # ---- CPU oracle on a bounded sample ---------------------------------------------------------
    cpu = None
    if not args.no_cpu_baseline:
        from oracle import reranker as orr
        try:
            from threadpoolctl import threadpool_info
            cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
        except Exception:
            cores = len(os.sched_getaffinity(0))
        opool = orr.PagedKV(m.n_layers, m.n_kv_heads, m.head_dim, 16, cfg.kv_dtype)

        def load_doc(dd):
            kv = wlmod.synthetic_doc_kv(wl, dd, dev)
            if cfg.kv_dtype == "fp8":
                opool.write(wl.pool_doc_pages[dd], kv["k"].cpu().numpy(), kv["v"].cpu().numpy(),
                            kv["k_scale"].cpu().numpy(), kv["v_scale"].cpu().numpy())
            else:
                opool.write(wl.pool_doc_pages[dd], kv["k"].double().cpu().numpy(), kv["v"].double().cpu().numpy())

        rng = np.random.default_rng(0)
        order = rng.permutation(wl.n_pairs)

        class Cached:                        # keep small models' tensors so the timing is the oracle's arithmetic
            def __init__(self, base, keep):
                self.base, self.keep, self.store = base, keep, {}

            def get(self, kind, layer=-1):
                if not self.keep:
                    return self.base.get(kind, layer)
                if (kind, layer) not in self.store:
                    self.store[(kind, layer)] = self.base.get(kind, layer)
                return self.store[(kind, layer)]

        n_params = m.gemm_flop_per_token() / 2
        oweights = Cached(weights, keep=n_params < 1.5e9)

        def run_oracle(idx):
            sub = wl.subset(idx)
            for dd in set(int(x) for x in sub.pair_doc):
                if int(wl.pool_doc_pages[dd][0]) not in opool.pages:
                    load_doc(dd)
            t = time.perf_counter()
            s = orr.score_cached(oweights, m, opool, sub.page_table, sub.doc_lens, sub.query_tokens, sub.query_lens)
            return time.perf_counter() - t, s, sub

        n_cpu = args.cpu_pairs
        if n_cpu <= 0:
            run_oracle(order[:1])                              # warms the BLAS threads and the weight cache
            el2, _, _ = run_oracle(order[:2])
            n_cpu = int(max(2, min(wl.n_pairs, 256, round(15.0 / max(el2 / 2, 1e-3)))))
        el, s_cpu, sub = run_oracle(order[:n_cpu])
        while el < 8.0 and n_cpu < min(wl.n_pairs, 1024) and args.cpu_pairs <= 0:   # aim for 10-30 s of oracle time
            n_cpu = int(min(wl.n_pairs, 1024, max(n_cpu + 1, round(n_cpu * 15.0 / max(el, 1e-3)))))
            el, s_cpu, sub = run_oracle(order[:n_cpu])
        s_gpu = scores[torch.from_numpy(order[:n_cpu].copy()).to(dev)].cpu().numpy()
        cpu = {"value": round(n_cpu / el, 4), "unit": "pairs/s", "cores": int(cores), "kind": "oracle",
               "sample": f"{n_cpu} seeded pairs of {wl.n_pairs} ({el:.1f} s, float64 numpy" + ("" if oweights.keep else "; weight generation inside the timed call") + f")",
               "max_abs_err_vs_gpu": float(np.abs(s_cpu - s_gpu).max())}

    line = {
        "metric": "rerank_pairs_per_sec", "value": round(pairs_per_s, 2), "unit": "pairs/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": ("f32" if m.dtype == "f32" else "f16") + ("+fp8kv" if cfg.kv_dtype == "fp8" else ""), "data": "synthetic",
        "config": {"workload": cfg.name, "model_shape": m.name, "pairs": wl.n_pairs, "query_tokens": T,
                   "doc_len": cfg.doc_len, "query_len": cfg.query_len, "kv_dtype": cfg.kv_dtype,
                   "gemm_path": model.gemm_path(), "attention_path": model.attention_path(pool),
                   "last_layer": "last token of each pair only" if shortened else "all tokens",
                   "streams": parts,
                   "roofline_region": (f"{args.steps} one-stream steps right after the timed region (kernel alone on the chip); breakdown from 2 one-stream "
                                       "survey steps before it" if not args.no_events else "none"),
                   "events_in_timed_region": "none"},
        "roofline": roofline, "roofline_attention": roof_attn, "gemm_overall": gemm_all, "one_stream": single,
        "kernel_breakdown": breakdown, "ceilings": ceilings, "cpu_baseline": cpu, "no_reuse": no_reuse, "doc_prefill": doc_prefill, "host_tier": host_tier, "host_tier_4bit": host_tier4,
        "paper_context": "2-3x end-to-end service throughput from reranker KV reuse on 8x A100 (Table 1); not this metric",
    }
    print(json.dumps(line), flush=True)


if __name__ == "__main__":
    main()
