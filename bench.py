#!/usr/bin/env python3
"""Benchmark of the reranker scoring pass (query suffix over cached document KV) on one MI355X.

One "step" = one hr_rerank_score call over a whole workload (all pairs, all layers), inputs (weights,
document-KV pool) resident in HBM before the timed region.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload c2_qwen0p5b] [--also c3_llama8b,c5_long_fp8]

The headline (`value`, `roofline`, ...) is the workload named by --workload (default: the 0.5B-shaped config 2, the
configuration the metric is quoted on).  The metric names the 0.5B and the 8B shapes, so a default run also measures
the 8B-shaped workloads and reports them under `other_workloads` with their own rates and rooflines: config 3
(with the CPU oracle timed on a few of its pairs) and config 5 (fp8 KV, long documents, with the same GPU's no-reuse
pass timed as the reference the reuse is compared with).  --also none skips them.

The timed steps run the way the library runs them: in one piece, or (where the library chooses so for the size of
the call) as two halves on two streams; config.streams says which.  Per workload the line carries
  roofline            the kernel class with the largest share of the step (per-kernel HIP events, recorded by the
                      library on the stream it launches on), measured in K more steps with the second stream
                      switched off, where the kernel has the chip to itself
  one_stream          the rate of those steps
  roofline_attention  the KV-streaming attention kernel against HBM peak
  gemm_rooflines      each of the four projection classes against the MFMA peak (survey steps)
and for the headline workload also
  ceilings            yardsticks on the same device: the library's own read-only streaming kernel, a copy-like kernel,
                      the vendor GEMM on a large square and on this workload's projection shapes
  cpu_baseline        the CPU oracle timed on a bounded sample of the same pairs
  no_reuse            the same GPU running the full [doc ; query] prefill on a few pairs
  doc_prefill         stage one on the device: documents prefilled into pool pages (ingest rate)
  host_tier           the same batch when every document's pages first come from pinned host memory
                      (bus-inclusive rate, page-in overlapped with scoring; never `value`)
  host_tier_4bit      the same with 4-bit records in the tier (16-bit pools)
  small_request       one query with 20 candidates: latency of a plain call, of a fixed-shape plan, of its graph replay
"""

import argparse
import gc
import hashlib
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
GEMM_CLASSES = ("gemm_qkv", "gemm_o", "gemm_gate_up", "gemm_down")


def log(*a):
    print(*a, file=sys.stderr, flush=True)


class CachedWeights:
    """Keeps the generated tensors (fp32 numpy) so that the device upload and the CPU oracle share one generation."""

    def __init__(self, base, keep=True):
        self.base, self.keep, self.store = base, keep, {}

    def get(self, kind, layer=-1):
        if not self.keep:
            return self.base.get(kind, layer)
        if (kind, layer) not in self.store:
            self.store[(kind, layer)] = self.base.get(kind, layer)
        return self.store[(kind, layer)]


def kernel_sources_sha():
    h = hashlib.sha256()
    for f in ("hr_gemm_mfma.hip", "hr_attn_mfma.hip", "hr_kernels_generic.hip"):
        with open(os.path.join(ROOT, "paper_2504_02921_amd", "csrc", f), "rb") as fh:
            h.update(fh.read())
    return h.hexdigest()[:16]


def recorded_traffic(name):
    """HBM-side bytes per launch from rocprofv3 --pmc runs recorded under profiles/ (FETCH_SIZE + WRITE_SIZE, scaled
    by a copy kernel of known size).  They are replayed here, not measured in this run: the record carries the date and
    the hash of the kernel sources it was taken with, and is dropped when the sources have changed since."""
    try:
        with open(os.path.join(ROOT, "profiles", "hbm_traffic.json")) as f:
            rec = json.load(f)
    except (OSError, ValueError):
        return {}, None
    entry = rec.get(name)
    if not entry:
        return {}, None
    meta = rec.get("_recorded", {})
    src = {"from": "profiles/hbm_traffic.json (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, replayed, not measured in this run)",
           "recorded": meta.get("date"), "kernel_sources_sha": meta.get("kernel_sources_sha")}
    if meta.get("kernel_sources_sha") != kernel_sources_sha():
        src["stale"] = "the kernel sources have changed since the record was taken: figures dropped"
        return {}, src
    return entry, src


def get_model(shared, m, seed, dev, hb, wlmod):
    key = (m.name, seed)
    if key not in shared["models"]:
        t0 = time.time()
        weights = CachedWeights(wlmod.SeededWeights(m, seed=seed), keep=True)
        model = hb.Model(m, weights, dev)
        shared["models"][key] = (model, weights)
        log(f"model {m.name}: weights generated, uploaded and packed in {time.time() - t0:.1f}s; split-operand layers {model.precise_layers()}")
    return shared["models"][key]


def measure(name, args, shared, legs, dev="cuda:0"):
    import torch
    from paper_2504_02921_amd import binding as hb
    from paper_2504_02921_amd import workloads as wlmod

    cfg = wlmod.CONFIGS[name]
    m = cfg.model
    t0 = time.time()
    wl = wlmod.make_workload(cfg)
    model, weights = get_model(shared, m, cfg.seed, dev, hb, wlmod)
    pool = hb.KVPool(m.n_layers, m.n_kv_heads, m.head_dim, wl.num_pages, cfg.kv_dtype, dev)
    for d in range(wl.n_docs):
        kv = wlmod.synthetic_doc_kv(wl, d, dev)
        if cfg.kv_dtype == "fp8":
            pool.write(int(wl.pool_doc_lens[d]), wl.pool_doc_pages[d], kv["k"], kv["v"], kv["k_scale"], kv["v_scale"])
        else:
            pool.write(int(wl.pool_doc_lens[d]), wl.pool_doc_pages[d], kv["k"], kv["v"])
        torch.cuda.synchronize()
    log(f"[{name}] setup {time.time() - t0:.1f}s: {wl.n_pairs} pairs, {wl.total_q_tokens} query tokens, pool {pool.mem.numel() / 1e9:.2f} GB, "
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
    # last round of GEMM tiles leaves idle).  The timed region measures what it chooses for this size.  A kernel's own
    # duration is then no longer a statement about the kernel: it includes waiting for CUs the other half's kernel holds.
    # So the per-kernel figures come from steps with the second stream switched off, where every kernel has the chip to
    # itself: two survey steps before the timed region time every kernel class (the breakdown, and which class is
    # dominant); K more such steps after it bracket only the dominant class and attention (two event records cost a few
    # microseconds of stream time per launch, ~6 % of a step when all ~170 launches are bracketed) and give the
    # rooflines.  The timed region itself records no events (on two streams they cost more than they tell).
    streams = 1 if os.environ.get("HR_STREAMS", "") == "1" else 2
    model.set_streams(streams)
    parts = model.parts(wl.total_q_tokens) if model.attention_path(pool) == "mfma" else 1     # what the library does at this size
    survey = {}
    dominant = "gemm_gate_up"
    if not args.no_events:
        model.set_streams(1)
        model.profile_select(None)
        model.profile_enable(True)
        for _ in range(2):
            step()
        torch.cuda.synchronize()
        survey = model.profile_read()
        dominant = max(survey, key=lambda k: survey[k]["ms"])
        if dominant != "attention" and dominant not in GEMM_CLASSES:
            dominant = "gemm_gate_up"
        model.profile_enable(False)
        model.set_streams(streams)
        step()
        torch.cuda.synchronize()
    # no collector pause inside a timed region (a full collection over the workload's arrays takes ~45 ms)
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

    traffic, traffic_src = recorded_traffic(cfg.name)

    # ---- rooflines from the per-kernel events ------------------------------------------------
    T = wl.total_q_tokens
    H, d, F = m.hidden, m.head_dim, m.ffn
    nq = m.n_q_heads * d
    P, L = wl.n_pairs, m.n_layers
    n_split = model.precise_layers() if model.gemm_path() == "mfma" and model.attention_path(pool) == "mfma" else 0
    # In the last layer only each pair's last token goes through the O, gate/up and down projections (P rows instead
    # of T; the library does this whenever the MFMA kernels run, and a test checks the scores are bit-identical), so the
    # algorithmic flop of an average launch of those classes is ((L - 1) T + P) / (L T) of a full-size launch.  The
    # split-operand layers run twice the MFMA work of a plain layer; the algorithmic flop stays that of the plain
    # projection, so their extra time counts against the achieved rate.
    shortened = (model.gemm_path() == "mfma" and model.attention_path(pool) == "mfma" and T > P
                 and os.environ.get("HR_NO_LAST_SHORTCUT", "0") != "1" and n_split < L)
    tail = ((L - 1) * T + P) / (L * T) if shortened else 1.0
    flop_per_launch = {
        "gemm_qkv": 2.0 * T * H * m.qkv_out, "gemm_o": 2.0 * T * nq * H * tail,
        "gemm_gate_up": 2.0 * T * H * 2 * F * tail, "gemm_down": 2.0 * T * F * H * tail,
    }
    kv_bytes_per_launch = wl.kv_stream_bytes() / m.n_layers
    # pairs that share a document are one attention work item: the document is streamed once for all of them
    seen = {}
    for p in range(P):
        seen.setdefault(int(wl.pair_doc[p]), int(wl.doc_lens[p]))
    per_tok = m.kv_bytes_per_token(cfg.kv_dtype) / m.n_layers
    distinct_doc_bytes = sum(seen.values()) * per_tok
    roofline = None
    roof_attn = None
    gemm_roofs = None
    breakdown = {}
    gemm_all = None
    if prof:
        total_ms = sum(v["ms"] for v in survey.values()) or 1.0
        for kname, v in survey.items():                  # from the survey steps (all classes timed), not the timed region
            if v["launches"]:
                breakdown[kname] = {"ms_per_step": round(v["ms"] / 2, 4), "launches_per_step": v["launches"] // 2,
                                    "share": round(v["ms"] / total_ms, 4)}

        def gemm_roof(kname, src):
            avg_s = src[kname]["ms"] / src[kname]["launches"] * 1e-3
            ach = flop_per_launch[kname] / avg_s / 1e12
            if model.gemm_path() == "mfma":
                return {"kernel": kname, "bound": "mfma", "achieved": round(ach, 2), "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                        "frac": round(ach / MFMA_BF16_PEAK_TFLOPS, 4), "traffic": traffic.get(kname), "traffic_source": traffic_src,
                        "avg_launch_ms": round(avg_s * 1e3, 4), "algorithmic_flop_per_launch": flop_per_launch[kname],
                        "launches_measured": src[kname]["launches"]}
            return {"kernel": kname, "bound": "alu", "achieved": round(ach, 3), "peak": FP32_VECTOR_PEAK_TFLOPS, "unit": "TFLOP/s",
                    "frac": round(ach / FP32_VECTOR_PEAK_TFLOPS, 4), "traffic": None, "avg_launch_ms": round(avg_s * 1e3, 4)}

        avg_s = prof["attention"]["ms"] / prof["attention"]["launches"] * 1e-3
        ach = kv_bytes_per_launch / avg_s / 1e9
        roof_attn = {"kernel": "attention", "bound": "hbm", "achieved": round(ach, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(ach / HBM_PEAK_GBS, 4), "traffic": traffic.get("attention"), "traffic_source": traffic_src,
                     "avg_launch_ms": round(avg_s * 1e3, 4), "algorithmic_bytes_per_launch": int(kv_bytes_per_launch),
                     "algorithmic_bytes_are": "every pair's document K/V once per layer (per-pair equivalent)"}
        # The launch also has to read q and the new tokens' K/V pages and write o (16-bit each): at short documents that is
        # a third of what it moves, so the KV-stream figure alone understates how close the launch is to the memory system.
        other_bytes = 2 * T * nq * 2 + T * 2 * m.n_kv_heads * d * 2
        roof_attn["all_operand_bytes_per_launch"] = int(kv_bytes_per_launch + other_bytes)
        roof_attn["all_operand_GBps"] = round((kv_bytes_per_launch + other_bytes) / avg_s / 1e9, 1)
        roof_attn["frac_all_operands"] = round((kv_bytes_per_launch + other_bytes) / avg_s / 1e9 / HBM_PEAK_GBS, 4)
        roof_attn["all_operands_are"] = "KV stream + q read + the new tokens' K/V pages read + o written (plain layers' widths)"
        if distinct_doc_bytes < 0.999 * kv_bytes_per_launch:
            roof_attn["streamed_bytes_per_launch_lower_bound"] = int(distinct_doc_bytes)
            roof_attn["streamed_GBps_lower_bound"] = round(distinct_doc_bytes / avg_s / 1e9, 1)
            roof_attn["note"] = ("pairs that share a document are batched into one work item per kv head, so the kernel moves fewer bytes than "
                                 "the per-pair figure: between one pass per distinct document (the lower bound given here) and one per "
                                 "group of at most 16 row blocks")
        roofline = roof_attn if dominant == "attention" else gemm_roof(dominant, prof)
        gemm_ms = sum(survey[k]["ms"] for k in flop_per_launch)
        gemm_all = {"achieved_tflops": round(sum(flop_per_launch.values()) * L * 2 / (gemm_ms * 1e-3) / 1e12, 2),
                    "frac": round(sum(flop_per_launch.values()) * L * 2 / (gemm_ms * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS, 4),
                    "note": "all four projections, from the survey steps"}
        if model.gemm_path() == "mfma":
            gemm_roofs = {k: {kk: vv for kk, vv in gemm_roof(k, survey).items() if kk in ("achieved", "frac", "avg_launch_ms")}
                          for k in GEMM_CLASSES if survey.get(k, {}).get("launches")}

    res = {
        "value": round(pairs_per_s, 2), "unit": "pairs/s", "ms_per_step": round(ms_per_step, 4),
        "dtype": ("f32" if m.dtype == "f32" else "f16") + ("+fp8kv" if cfg.kv_dtype == "fp8" else ""),
        "config": {"workload": cfg.name, "model_shape": m.name, "pairs": wl.n_pairs, "query_tokens": T,
                   "doc_len": cfg.doc_len, "query_len": cfg.query_len, "kv_dtype": cfg.kv_dtype,
                   "gemm_path": model.gemm_path(), "attention_path": model.attention_path(pool),
                   "last_layer": "last token of each pair only" if shortened else "all tokens",
                   "split_operand_layers": n_split, "streams": parts,
                   "roofline_region": (f"{args.steps} one-stream steps right after the timed region (kernel alone on the chip); breakdown from 2 one-stream "
                                       "survey steps before it" if not args.no_events else "none"),
                   "events_in_timed_region": "none"},
        "roofline": roofline, "roofline_attention": roof_attn, "gemm_rooflines": gemm_roofs, "gemm_overall": gemm_all, "one_stream": single,
        "kernel_breakdown": breakdown,
    }

    # ---- what this device gives to plain streaming and library calls (yardsticks, not part of the scoring path) ------
    if "ceilings" in legs and model.gemm_path() == "mfma":
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
        sink = torch.zeros(1 << 16, dtype=torch.int32, device=dev)
        big = torch.zeros(1 << 30, dtype=torch.int32, device=dev)        # 4 GiB: larger than the 256 MB last-level cache
        t_read = timed(lambda: hb.probe_read_bandwidth(big, sink), 10)
        t_read_lds = timed(lambda: hb.probe_read_bandwidth(big, sink, to_lds=True), 10)
        del src, dst, big
        ceilings = {"hbm_read_GBps": round(4 * (1 << 30) / t_read / 1e9, 1),
                    "hbm_read_to_lds_GBps": round(4 * (1 << 30) / t_read_lds / 1e9, 1),
                    "hbm_copy_GBps": round(2 * (1 << 30) / t_copy / 1e9, 1),
                    "note": "hbm_read: the library's own read-only streaming kernel over 4 GiB (hr_probe_read_bandwidth: 16-byte loads into "
                            "registers; ..._to_lds: the direct-to-LDS loads the attention kernel streams with); hbm_copy: torch.bitwise_not over "
                            "1 GiB (read + write); torch.matmul in half precision (the vendor library), without the fused epilogues of this path"}
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
            roof_attn["frac_of_read_only_kernel"] = round(roof_attn["achieved"] / ceilings["hbm_read_GBps"], 4)
        res["ceilings"] = ceilings
        shared["ceilings"] = ceilings
    elif roof_attn and shared.get("ceilings"):
        roof_attn["frac_of_read_only_kernel"] = round(roof_attn["achieved"] / shared["ceilings"]["hbm_read_GBps"], 4)

    # ---- one request: one query with its candidates (latency, not throughput) ---------------------------------
    if "small_request" in legs:
        n_small = min(cfg.n_cands, 20)
        sub = wl.subset(np.arange(n_small))
        out_small = torch.empty(n_small, dtype=torch.float32, device=dev)

        def timed_calls(fn, n=30):
            for _ in range(5):
                fn()
            torch.cuda.synchronize()
            t = time.perf_counter()
            for _ in range(n):
                fn()
            torch.cuda.synchronize()
            return (time.perf_counter() - t) / n * 1e3

        ms_call = timed_calls(lambda: model.score(pool, sub.page_table, sub.doc_lens, sub.query_tokens, sub.query_lens, out=out_small))
        ref_small = out_small.clone()
        small = {"pairs": n_small, "query_tokens": sub.total_q_tokens, "hr_rerank_score_ms": round(ms_call, 4)}
        try:
            plan = hb.Plan(model, pool, sub.doc_lens, sub.query_lens, sub.page_table.shape[1])
            plan.set_inputs(sub.page_table, sub.query_tokens)
            small["plan_run_ms"] = round(timed_calls(lambda: plan.run(out_small)), 4)
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph):
                plan.run(out_small)
            small["graph_replay_ms"] = round(timed_calls(graph.replay), 4)
            assert torch.equal(out_small, ref_small), "plan / graph replay scores differ from hr_rerank_score"
            small["note"] = ("one query with its first candidates, documents resident: hr_rerank_score (host builds and uploads the metadata "
                             "every call), hr_rerank_plan_run (fixed shape, stream work only), and the plan recorded once into a HIP graph "
                             "and replayed; same score bits in all three")
            del graph
            plan.close()
        except hb.HrError as e:
            small["note"] = str(e)
        res["small_request"] = small

    # ---- same-GPU no-reuse reference on a few pairs ------------------------------------------
    if "no_reuse" in legs and args.no_reuse_pairs > 0:
        # sized so that the leg stays at a few seconds: ~0.5 M tokens of [doc ; query] at the 0.5B shape, ~70 k at the 8B shape
        per_pair = int(wl.doc_lens[0]) + int(wl.query_lens[0])
        budget = 600_000 if m.hidden < 2048 else 70_000
        n = max(2, min(args.no_reuse_pairs, wl.n_pairs, budget // max(per_pair, 1)))
        docs = [wl.doc_tokens(int(dd)) for dd in wl.pair_doc[:n]]
        qs = [wl.query_tokens_per_query[int(q)] for q in wl.pair_query[:n]]
        try:
            model.score_full(docs, qs)
            torch.cuda.synchronize()
            tt = time.perf_counter()
            model.score_full(docs, qs)
            torch.cuda.synchronize()
            el = time.perf_counter() - tt
            res["no_reuse"] = {"value": round(n / el, 2), "unit": "pairs/s", "pairs": n, "tokens_per_pair": per_pair,
                               "reuse_speedup": round(pairs_per_s / (n / el), 2),
                               "note": "hr_rerank_score_full: full [doc ; query] prefill per pair on the same GPU in 16-bit, random doc tokens "
                                       "of the same lengths; reuse_speedup = this workload's pairs/s with cached document KV over this rate"}
        except hb.HrError as e:
            res["no_reuse"] = {"value": None, "note": str(e)}

    # ---- stage one on the device: documents prefilled straight into pool pages (ingest rate) ---------
    if "prefill" in legs and args.prefill_docs > 0:
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
            res["doc_prefill"] = {"value": round(n_tok / best, 1), "unit": "document tokens/s", "docs": nd, "docs_per_s": round(nd / best, 1),
                                  "note": "hr_doc_prefill: random document tokens of the workload's lengths, K/V of every layer written to pool pages"
                                          + (" (quantised to fp8 as stored)" if cfg.kv_dtype == "fp8" else "")}
            pool_p.close()
            del pool_p
        except hb.HrError as e:
            res["doc_prefill"] = {"value": None, "note": str(e)}

    # ---- host tier: every batch's document pages are paged in from pinned host memory ----------------
    # Two pools alternate: while one batch is scored from one of them, the next batch's pages arrive in the other on a
    # second stream.  The rate includes the bus (it is not `value`): with every document cold it is the bus that
    # bounds it.
    if "host_tier" in legs and args.host_tier_batches > 0:
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
            out = {"value": round(B * wl.n_pairs / el, 2), "unit": "pairs/s", "batches": B,
                   "bytes_per_batch": int(tier_bytes), "page_record_bytes": int(rec),
                   "page_in_GBps": round(tier_bytes / in_s / 1e9, 2), "page_out_GBps": round(tier_bytes / out_s / 1e9, 2),
                   "max_abs_score_change": diff}
            del tier, pool_b
            return out

        host_tier = tier_leg(pool.page_record_bytes, lambda p, ids, t: p.pages_out(ids, t), lambda p, ids, t: p.pages_in(ids, t), True)
        if host_tier.get("value") is not None:
            host_tier["note"] = ("every document of every batch paged in from pinned host memory (hr_kv_pages_in on a second stream, "
                                 "two pools alternating); includes the first batch's unoverlapped page-in")
        res["host_tier"] = host_tier
        if cfg.kv_dtype == "bf16":
            # after the 16-bit leg both pools hold the original pages again, so the 4-bit records are made from those
            host_tier4 = tier_leg(pool.page_record4_bytes, lambda p, ids, t: p.pages_out4(ids, t), lambda p, ids, t: p.pages_in4(ids, t), False)
            if host_tier4.get("value") is not None:
                host_tier4["note"] = ("the same with 4-bit records (hr_kv_pages_in4: quantised in the tier, expanded to 16 bits as they arrive); "
                                      "max_abs_score_change is against the scores from the unquantised documents")
            res["host_tier_4bit"] = host_tier4
            # the leg leaves quantised documents in the pool: put the originals back for what follows
            for d in range(wl.n_docs):
                kv = wlmod.synthetic_doc_kv(wl, d, dev)
                pool.free(wl.pool_doc_pages[d])
                pool.write(int(wl.pool_doc_lens[d]), wl.pool_doc_pages[d], kv["k"], kv["v"])
                torch.cuda.synchronize()

    # ---- CPU oracle on a bounded sample ---------------------------------------------------------
    if "cpu" in legs and not args.no_cpu_baseline:
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

        def run_oracle(idx):
            sub = wl.subset(idx)
            for dd in set(int(x) for x in sub.pair_doc):
                if int(wl.pool_doc_pages[dd][0]) not in opool.pages:
                    load_doc(dd)
            t = time.perf_counter()
            s = orr.score_cached(weights, m, opool, sub.page_table, sub.doc_lens, sub.query_tokens, sub.query_lens)
            return time.perf_counter() - t, s, sub

        big = m.gemm_flop_per_token() / 2 > 1.5e9
        n_cpu = args.cpu_pairs
        if n_cpu <= 0 and big:
            # one call: every call converts all layers' weights to float64 (half a minute at the 8B shape), so the sample is
            # fixed rather than grown
            n_cpu = 4
        elif n_cpu <= 0:
            run_oracle(order[:1])                              # warms the BLAS threads
            el2, _, _ = run_oracle(order[:2])
            n_cpu = int(max(2, min(wl.n_pairs, 256, round(15.0 / max(el2 / 2, 1e-3)))))
        el, s_cpu, sub = run_oracle(order[:n_cpu])
        while el < 8.0 and n_cpu < min(wl.n_pairs, 1024) and args.cpu_pairs <= 0 and not big:   # aim for 10-30 s of oracle time
            n_cpu = int(min(wl.n_pairs, 1024, max(n_cpu + 1, round(n_cpu * 15.0 / max(el, 1e-3)))))
            el, s_cpu, sub = run_oracle(order[:n_cpu])
        s_gpu = scores[torch.from_numpy(order[:n_cpu].copy()).to(dev)].cpu().numpy()
        res["cpu_baseline"] = {"value": round(n_cpu / el, 4), "unit": "pairs/s", "cores": int(cores), "kind": "oracle",
                               "sample": f"{n_cpu} seeded pairs of {wl.n_pairs} ({el:.1f} s, float64 numpy, weights already generated"
                                         + (", their conversion to float64 inside the timed call" if big else "") + ")",
                               "max_abs_err_vs_gpu": float(np.abs(s_cpu - s_gpu).max())}
        del opool

    pool.close()
    del pool, scores
    torch.cuda.empty_cache()
    return res


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="c2_qwen0p5b")
    ap.add_argument("--also", default=None,
                    help="comma-separated workloads measured after the headline one and reported under other_workloads "
                         "(default: c3_llama8b,c5_long_fp8 when the headline is the default; 'none' to skip)")
    ap.add_argument("--cpu-pairs", type=int, default=0, help="pairs for the CPU-oracle leg (0 = pick for ~15 s)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-reuse-pairs", type=int, default=256, help="most pairs for the no-reuse reference (0 = skip)")
    ap.add_argument("--no-events", action="store_true", help="do not record per-kernel events")
    ap.add_argument("--prefill-docs", type=int, default=128, help="documents for the document-prefill (ingest) leg (0 = skip)")
    ap.add_argument("--host-tier-batches", type=int, default=6,
                    help="batches of the paged leg: every batch's documents come from pinned host memory (0 = skip)")
    ap.add_argument("--no-ceilings", action="store_true", help="skip the yardsticks (streaming kernels, library GEMM)")
    ap.add_argument("--no-small-request", action="store_true", help="skip the one-query latency leg")
    ap.add_argument("--calibration-copy-mib", type=int, default=0,
                    help="also run a plain device copy of this many MiB (known traffic, for scaling rocprofv3 byte counters)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        log("bench.py: this build measures ONE GPU only (pairs are independent, so they shard over GPUs with no collective). "
            "Run with --gpus 1.")
        sys.exit(2)

    import torch
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    also = args.also
    if also is None:
        also = "c3_llama8b,c5_long_fp8" if args.workload == "c2_qwen0p5b" else "none"
    others = [x for x in also.split(",") if x and x != "none" and x != args.workload]

    shared = {"models": {}}
    legs = {"cpu", "no_reuse", "prefill", "host_tier"} | (set() if args.no_ceilings else {"ceilings"}) | (set() if args.no_small_request else {"small_request"})
    t_start = time.time()
    main_res = measure(args.workload, args, shared, legs)
    other_res = {}
    for name in others:
        # free the previous shape's model before the next one is built
        from paper_2504_02921_amd import workloads as wlmod
        want = (wlmod.CONFIGS[name].model.name, wlmod.CONFIGS[name].seed)
        for key in [k for k in shared["models"] if k != want]:
            shared["models"].pop(key)[0].close()
        gc.collect()
        torch.cuda.empty_cache()
        extra = {"c3_llama8b": {"cpu"} | (set() if args.no_small_request else {"small_request"}), "c5_long_fp8": {"no_reuse"}}.get(name, set())
        other_res[name] = measure(name, args, shared, extra)
        log(f"[{name}] done at {time.time() - t_start:.0f}s: {other_res[name]['value']} pairs/s")

    line = {
        "metric": "rerank_pairs_per_sec", "value": main_res.pop("value"), "unit": main_res.pop("unit"),
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": main_res.pop("ms_per_step"),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": main_res.pop("dtype"), "data": "synthetic",
    }
    line.update(main_res)
    for k in ("ceilings", "cpu_baseline", "no_reuse", "doc_prefill", "host_tier", "host_tier_4bit", "small_request"):
        line.setdefault(k, None)
    line["other_workloads"] = other_res or None
    line["paper_context"] = "2-3x end-to-end service throughput from reranker KV reuse on 8x A100 (Table 1); not this metric"
    print(json.dumps(line), flush=True)


if __name__ == "__main__":
    main()
