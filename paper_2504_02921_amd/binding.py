"""ctypes binding of libhyperrerank.so: the same entry points as include/hyperrerank.h.

Only argument marshalling happens here.  PyTorch provides device memory and
streams; every step of the scoring pass runs inside the library's HIP kernels.
There is no fallback: if the shared library is missing, importing this module
raises.
"""

from __future__ import annotations

import ctypes as C
import os
from typing import Dict, List, Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libhyperrerank.so")

HR_F32, HR_BF16, HR_FP8_E4M3 = 0, 1, 2
DTYPE_CODE = {"f32": HR_F32, "bf16": HR_BF16, "fp8": HR_FP8_E4M3}
PAGE_TOKENS = 16

STATUS = {
    0: "HR_OK", -1: "HR_ERR_INVALID_ARG", -2: "HR_ERR_POOL_TOO_SMALL", -3: "HR_ERR_PAGE_RANGE",
    -4: "HR_ERR_PAGE_IN_USE", -5: "HR_ERR_PAGE_DUP", -6: "HR_ERR_LEN_RANGE", -7: "HR_ERR_TABLE_SHORT",
    -8: "HR_ERR_TOKEN_RANGE", -9: "HR_ERR_WORKSPACE_SMALL", -10: "HR_ERR_UNSUPPORTED_SHAPE",
    -11: "HR_ERR_DEVICE", -12: "HR_ERR_POOL_FULL", -13: "HR_ERR_MISMATCH",
}
HR_OK = 0
for _code, _name in STATUS.items():
    globals()[_name] = _code


class hr_pool_cfg(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32),
                ("page_tokens", C.c_int32), ("num_pages", C.c_int32), ("kv_dtype", C.c_int32)]


class hr_model_cfg(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("hidden", C.c_int32), ("n_q_heads", C.c_int32),
                ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32), ("ffn", C.c_int32), ("vocab", C.c_int32),
                ("yes_id", C.c_int32), ("no_id", C.c_int32), ("dtype", C.c_int32),
                ("rope_base", C.c_float), ("rms_eps", C.c_float)]


class hr_range_report(C.Structure):
    _fields_ = [("overflow", C.c_int64), ("underflow", C.c_int64), ("nonfinite_inputs", C.c_int64),
                ("fp8_nan_codes", C.c_int64), ("fp8_bad_scales", C.c_int64), ("reserved", C.c_int64 * 3)]

    def as_dict(self):
        return {k: int(getattr(self, k)) for k in ("overflow", "underflow", "nonfinite_inputs", "fp8_nan_codes", "fp8_bad_scales")}


_PP = C.POINTER(C.c_void_p)


class hr_weight_ptrs(C.Structure):
    _fields_ = [("embedding", C.c_void_p), ("final_norm", C.c_void_p),
                ("wq", _PP), ("wk", _PP), ("wv", _PP), ("wo", _PP), ("wg", _PP), ("wu", _PP), ("wd", _PP),
                ("norm1", _PP), ("norm2", _PP)]


EXPORTS = [
    "hr_status_str", "hr_last_error", "hr_kv_pool_bytes", "hr_kv_pool_create", "hr_kv_pool_destroy", "hr_kv_pool_free_pages",
    "hr_kv_pool_alloc_pages", "hr_doc_kv_write", "hr_doc_kv_read", "hr_doc_kv_free", "hr_kv_page_record_bytes", "hr_kv_pages_out",
    "hr_kv_pages_in", "hr_kv_page_record4_bytes", "hr_kv_pages_out4", "hr_kv_pages_in4", "hr_weights_pack_bytes", "hr_weights_load",
    "hr_model_destroy", "hr_rerank_workspace_bytes", "hr_rerank_score", "hr_rerank_static_scratch_bytes",
    "hr_rerank_score_static", "hr_rerank_plan_create", "hr_rerank_plan_set_inputs", "hr_rerank_plan_run",
    "hr_rerank_plan_destroy", "hr_model_set_precise_layers", "hr_model_precise_layers", "hr_rerank_set_streams", "hr_rerank_parts", "hr_rerank_validate",
    "hr_rerank_full_workspace_bytes", "hr_rerank_score_full", "hr_doc_prefill_workspace_bytes", "hr_doc_prefill", "hr_attention_path", "hr_gemm_path",
    "hr_rerank_topk", "hr_model_range_report", "hr_kv_pool_range_report", "hr_probe_read_bandwidth", "hr_profile_enable", "hr_profile_select", "hr_profile_count", "hr_profile_name", "hr_profile_read",
]


def _load() -> C.CDLL:
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: build it first (python -m paper_2504_02921_amd.build "
                          "or __graft_entry__.build()); there is no CPU fallback")
    # PyTorch ships its own HIP runtime; it must be the one this library binds to, or streams and
    # allocations made by torch would belong to a different runtime instance.  Loading torch first
    # puts its libamdhip64 (same soname) in the process before ours is resolved.
    import torch  # noqa: F401
    bundled = os.path.join(os.path.dirname(torch.__file__), "lib", "libamdhip64.so")
    if os.path.exists(bundled):
        C.CDLL(bundled, mode=C.RTLD_GLOBAL)
    lib = C.CDLL(LIB_PATH)
    i32p = C.POINTER(C.c_int32)
    sig = {
        "hr_status_str": (C.c_char_p, [C.c_int]),
        "hr_last_error": (C.c_char_p, []),
        "hr_kv_pool_bytes": (C.c_size_t, [C.POINTER(hr_pool_cfg)]),
        "hr_kv_pool_create": (C.c_int, [C.POINTER(hr_pool_cfg), C.c_void_p, C.c_size_t, C.POINTER(C.c_void_p)]),
        "hr_kv_pool_destroy": (None, [C.c_void_p]),
        "hr_kv_pool_free_pages": (C.c_int64, [C.c_void_p]),
        "hr_kv_pool_alloc_pages": (C.c_int, [C.c_void_p, C.c_int32, i32p]),
        "hr_doc_kv_write": (C.c_int, [C.c_void_p, C.c_int32, i32p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]),
        "hr_doc_kv_read": (C.c_int, [C.c_void_p, C.c_int32, i32p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]),
        "hr_doc_kv_free": (C.c_int, [C.c_void_p, i32p, C.c_int32]),
        "hr_kv_page_record_bytes": (C.c_size_t, [C.c_void_p]),
        "hr_kv_pages_out": (C.c_int, [C.c_void_p, C.c_int32, i32p, C.c_void_p, C.c_void_p]),
        "hr_kv_pages_in": (C.c_int, [C.c_void_p, C.c_int32, i32p, C.c_void_p, C.c_void_p]),
        "hr_kv_page_record4_bytes": (C.c_size_t, [C.c_void_p]),
        "hr_kv_pages_out4": (C.c_int, [C.c_void_p, C.c_int32, i32p, C.c_void_p, C.c_void_p]),
        "hr_kv_pages_in4": (C.c_int, [C.c_void_p, C.c_int32, i32p, C.c_void_p, C.c_void_p]),
        "hr_weights_pack_bytes": (C.c_size_t, [C.POINTER(hr_model_cfg)]),
        "hr_weights_load": (C.c_int, [C.POINTER(hr_model_cfg), C.POINTER(hr_weight_ptrs), C.c_void_p, C.c_size_t,
                                      C.c_void_p, C.POINTER(C.c_void_p)]),
        "hr_model_destroy": (None, [C.c_void_p]),
        "hr_rerank_workspace_bytes": (C.c_size_t, [C.c_void_p, C.c_int32, C.c_int64, C.c_int32]),
        "hr_rerank_score": (C.c_int, [C.c_void_p, C.c_void_p, C.c_int32, i32p, C.c_int32, i32p, i32p, i32p,
                                      C.c_void_p, C.c_size_t, C.c_void_p, C.c_void_p]),
        "hr_rerank_static_scratch_bytes": (C.c_size_t, []),
        "hr_rerank_score_static": (C.c_int, [C.c_void_p, C.c_void_p, C.c_int32, i32p, C.c_int32, i32p, i32p, i32p,
                                             C.c_void_p, C.c_void_p]),
        "hr_rerank_plan_create": (C.c_int, [C.c_void_p, C.c_void_p, C.c_int32, i32p, i32p, C.c_int32, C.c_void_p, C.c_size_t,
                                            C.POINTER(C.c_void_p)]),
        "hr_rerank_plan_set_inputs": (C.c_int, [C.c_void_p, i32p, i32p]),
        "hr_rerank_plan_run": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p]),
        "hr_rerank_plan_destroy": (None, [C.c_void_p]),
        "hr_model_set_precise_layers": (C.c_int, [C.c_void_p, C.c_int]),
        "hr_model_precise_layers": (C.c_int, [C.c_void_p]),
        "hr_rerank_set_streams": (C.c_int, [C.c_void_p, C.c_int]),
        "hr_rerank_parts": (C.c_int, [C.c_void_p, C.c_int64]),
        "hr_rerank_validate": (C.c_int, [C.POINTER(hr_model_cfg), C.c_void_p, C.c_int32, i32p, C.c_int32, i32p, i32p, i32p]),
        "hr_rerank_full_workspace_bytes": (C.c_size_t, [C.c_void_p, C.c_int32, C.c_int64]),
        "hr_rerank_score_full": (C.c_int, [C.c_void_p, C.c_int32, i32p, i32p, i32p, i32p, C.c_void_p, C.c_size_t,
                                           C.c_void_p, C.c_void_p]),
        "hr_doc_prefill_workspace_bytes": (C.c_size_t, [C.c_void_p, C.c_int32, C.c_int64]),
        "hr_doc_prefill": (C.c_int, [C.c_void_p, C.c_void_p, C.c_int32, i32p, i32p, i32p, C.c_int32, C.c_void_p, C.c_size_t, C.c_void_p]),
        "hr_attention_path": (C.c_char_p, [C.c_void_p, C.c_void_p]),
        "hr_gemm_path": (C.c_char_p, [C.c_void_p]),
        "hr_rerank_topk": (C.c_int, [C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p]),
        "hr_model_range_report": (C.c_int, [C.c_void_p, C.POINTER(hr_range_report)]),
        "hr_kv_pool_range_report": (C.c_int, [C.c_void_p, C.POINTER(hr_range_report)]),
        "hr_probe_read_bandwidth": (C.c_int, [C.c_void_p, C.c_size_t, C.c_void_p, C.c_size_t, C.c_int, C.c_void_p]),
        "hr_profile_enable": (C.c_int, [C.c_void_p, C.c_int]),
        "hr_profile_select": (C.c_int, [C.c_void_p, C.c_uint32]),
        "hr_profile_count": (C.c_int, []),
        "hr_profile_name": (C.c_char_p, [C.c_int]),
        "hr_profile_read": (C.c_int, [C.c_void_p, C.POINTER(C.c_double), C.POINTER(C.c_int64)]),
    }
    for name, (res, args) in sig.items():
        fn = getattr(lib, name)
        fn.restype = res
        fn.argtypes = args
    return lib


lib = _load()


class HrError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        detail = lib.hr_last_error().decode() if status == -11 else ""
        super().__init__(f"{where}: {STATUS.get(status, status)} ({lib.hr_status_str(status).decode()}) {detail}")


def check(status: int, where: str) -> None:
    if status != HR_OK:
        raise HrError(status, where)


def _i32(a) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(a), dtype=np.int32)


def _i32p(a: Optional[np.ndarray]):
    if a is None:
        return None
    return a.ctypes.data_as(C.POINTER(C.c_int32))


def _stream_ptr(stream=None) -> C.c_void_p:
    import torch
    s = stream if stream is not None else torch.cuda.current_stream()
    return C.c_void_p(s.cuda_stream)


# ----------------------------------------------------------------------------------------------
# thin, same-named wrappers (raw pointers in, status out)
# ----------------------------------------------------------------------------------------------
def make_pool_cfg(n_layers, n_kv_heads, head_dim, num_pages, kv_dtype) -> hr_pool_cfg:
    return hr_pool_cfg(n_layers, n_kv_heads, head_dim, PAGE_TOKENS, num_pages, DTYPE_CODE.get(kv_dtype, kv_dtype))


def make_model_cfg(m) -> hr_model_cfg:
    """m: any object with the ModelCfg fields of the workload generators."""
    return hr_model_cfg(m.n_layers, m.hidden, m.n_q_heads, m.n_kv_heads, m.head_dim, m.ffn, m.vocab,
                        m.yes_id, m.no_id, DTYPE_CODE[m.dtype], float(m.rope_base), float(m.rms_eps))


def hr_kv_pool_bytes(cfg: hr_pool_cfg) -> int:
    return int(lib.hr_kv_pool_bytes(C.byref(cfg)))


def hr_kv_pool_create(cfg: hr_pool_cfg, dev_ptr: int, nbytes: int):
    out = C.c_void_p()
    st = lib.hr_kv_pool_create(C.byref(cfg), C.c_void_p(dev_ptr), nbytes, C.byref(out))
    return st, out


def hr_weights_pack_bytes(cfg: hr_model_cfg) -> int:
    return int(lib.hr_weights_pack_bytes(C.byref(cfg)))


# ----------------------------------------------------------------------------------------------
# convenience holders: own the torch tensors behind the handles
# ----------------------------------------------------------------------------------------------
def rerank_topk(scores, seg_offsets, k: int, with_scores: bool = False, stream=None):
    """Per-query top-k of device scores: seg_offsets (host ints, [n_queries + 1]) delimits each query's pairs.
    Returns an int32 device tensor [n_queries][k] of candidate indices inside each segment (-1 padded), and the
    matching scores when asked."""
    import torch
    seg = _i32(seg_offsets)
    n_q = len(seg) - 1
    max_c = max(int((seg[1:] - seg[:-1]).max()) if n_q > 0 else 1, k, 1)      # an upper bound is all the library needs
    seg_dev = torch.from_numpy(seg).to(scores.device)
    idx = torch.empty((max(n_q, 0), k), dtype=torch.int32, device=scores.device)
    sc = torch.empty((max(n_q, 0), k), dtype=torch.float32, device=scores.device) if with_scores else None
    check(lib.hr_rerank_topk(C.c_void_p(scores.data_ptr()), C.c_void_p(seg_dev.data_ptr()), n_q, max_c, k,
                             C.c_void_p(idx.data_ptr()), C.c_void_p(sc.data_ptr()) if with_scores else None, _stream_ptr(stream)),
          "hr_rerank_topk")
    idx._hr_seg = seg_dev          # keep the offsets alive until the result is dropped (the kernel may still be queued)
    return (idx, sc) if with_scores else idx


def probe_read_bandwidth(src, sink, to_lds: bool = False, stream=None) -> None:
    """One read-only pass of the library's streaming yardstick kernel over the device tensor `src`."""
    check(lib.hr_probe_read_bandwidth(C.c_void_p(src.data_ptr()), src.numel() * src.element_size(), C.c_void_p(sink.data_ptr()),
                                      sink.numel() * sink.element_size(), 1 if to_lds else 0, _stream_ptr(stream)),
          "hr_probe_read_bandwidth")


class KVPool:
    """Device buffer + library handle of one paged document-KV pool."""

    def __init__(self, n_layers: int, n_kv_heads: int, head_dim: int, num_pages: int, kv_dtype: str, device="cuda:0"):
        import torch
        self.cfg = make_pool_cfg(n_layers, n_kv_heads, head_dim, num_pages, kv_dtype)
        self.kv_dtype = kv_dtype
        nbytes = hr_kv_pool_bytes(self.cfg)
        if nbytes == 0:
            raise HrError(HR_ERR_INVALID_ARG, "hr_kv_pool_bytes")
        self.mem = torch.zeros(nbytes, dtype=torch.uint8, device=device)
        st, self.handle = hr_kv_pool_create(self.cfg, self.mem.data_ptr(), nbytes)
        check(st, "hr_kv_pool_create")

    def write(self, doc_len: int, page_ids, k, v, k_scale=None, v_scale=None, stream=None) -> None:
        """k, v: device tensors [L][doc_len][n_kv][d] in the pool dtype (uint8 codes for fp8)."""
        ids = _i32(page_ids)
        assert k.is_contiguous() and v.is_contiguous() and k.is_cuda and v.is_cuda
        ks = C.c_void_p(k_scale.data_ptr()) if k_scale is not None else None
        vs = C.c_void_p(v_scale.data_ptr()) if v_scale is not None else None
        st = lib.hr_doc_kv_write(self.handle, int(doc_len), _i32p(ids), C.c_void_p(k.data_ptr()), C.c_void_p(v.data_ptr()),
                                 ks, vs, _stream_ptr(stream))
        check(st, "hr_doc_kv_write")

    def read(self, doc_len: int, page_ids, stream=None):
        """The document's K/V back from its pages: device tensors [L][doc_len][n_kv][d] in the pool's element type
        (float32, float16 for 16-bit pools, uint8 codes for fp8), plus K / V scales [L][n_pages][n_kv] for fp8."""
        import torch
        ids = _i32(page_ids)
        L, n_kv, d = self.cfg.n_layers, self.cfg.n_kv_heads, self.cfg.head_dim
        dt = {HR_F32: torch.float32, HR_BF16: torch.float16, HR_FP8_E4M3: torch.uint8}[self.cfg.kv_dtype]
        k = torch.empty((L, int(doc_len), n_kv, d), dtype=dt, device=self.mem.device)
        v = torch.empty_like(k)
        ks = vs = None
        if self.cfg.kv_dtype == HR_FP8_E4M3:
            ks = torch.empty((L, len(ids), n_kv), dtype=torch.float32, device=self.mem.device)
            vs = torch.empty_like(ks)
        check(lib.hr_doc_kv_read(self.handle, int(doc_len), _i32p(ids), C.c_void_p(k.data_ptr()), C.c_void_p(v.data_ptr()),
                                 C.c_void_p(ks.data_ptr()) if ks is not None else None,
                                 C.c_void_p(vs.data_ptr()) if vs is not None else None, _stream_ptr(stream)), "hr_doc_kv_read")
        return (k, v, ks, vs) if ks is not None else (k, v)

    def free(self, page_ids) -> None:
        ids = _i32(page_ids)
        check(lib.hr_doc_kv_free(self.handle, _i32p(ids), len(ids)), "hr_doc_kv_free")

    def range_report(self) -> dict:
        r = hr_range_report()
        check(lib.hr_kv_pool_range_report(self.handle, C.byref(r)), "hr_kv_pool_range_report")
        return r.as_dict()

    @property
    def page_record_bytes(self) -> int:
        return int(lib.hr_kv_page_record_bytes(self.handle))

    @property
    def page_record4_bytes(self) -> int:
        return int(lib.hr_kv_page_record4_bytes(self.handle))

    def pages_out4(self, page_ids, records, stream=None) -> None:
        """4-bit records (16-bit pools): quantised as the pages leave."""
        ids = _i32(page_ids)
        assert records.numel() * records.element_size() >= len(ids) * self.page_record4_bytes
        check(lib.hr_kv_pages_out4(self.handle, len(ids), _i32p(ids), C.c_void_p(records.data_ptr()), _stream_ptr(stream)),
              "hr_kv_pages_out4")

    def pages_in4(self, page_ids, records, stream=None) -> None:
        ids = _i32(page_ids)
        assert records.numel() * records.element_size() >= len(ids) * self.page_record4_bytes
        check(lib.hr_kv_pages_in4(self.handle, len(ids), _i32p(ids), C.c_void_p(records.data_ptr()), _stream_ptr(stream)),
              "hr_kv_pages_in4")

    def pages_out(self, page_ids, records, stream=None) -> None:
        """records: uint8 tensor of len(page_ids) * page_record_bytes, on the device or in pinned host memory."""
        ids = _i32(page_ids)
        assert records.numel() * records.element_size() >= len(ids) * self.page_record_bytes
        check(lib.hr_kv_pages_out(self.handle, len(ids), _i32p(ids), C.c_void_p(records.data_ptr()), _stream_ptr(stream)),
              "hr_kv_pages_out")

    def pages_in(self, page_ids, records, stream=None) -> None:
        ids = _i32(page_ids)
        assert records.numel() * records.element_size() >= len(ids) * self.page_record_bytes
        check(lib.hr_kv_pages_in(self.handle, len(ids), _i32p(ids), C.c_void_p(records.data_ptr()), _stream_ptr(stream)),
              "hr_kv_pages_in")

    def alloc(self, n: int) -> np.ndarray:
        out = np.zeros(n, np.int32)
        check(lib.hr_kv_pool_alloc_pages(self.handle, n, _i32p(out)), "hr_kv_pool_alloc_pages")
        return out

    @property
    def free_pages(self) -> int:
        return int(lib.hr_kv_pool_free_pages(self.handle))

    def close(self):
        if getattr(self, "handle", None):
            lib.hr_kv_pool_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


_LAYER_KINDS = ("wq", "wk", "wv", "wo", "wg", "wu", "wd", "norm1", "norm2")


class Plan:
    """A fixed-shape scoring plan (hr_rerank_plan_*): owns its workspace tensor; run() is stream work only."""

    def __init__(self, model: "Model", pool: KVPool, doc_lens, query_lens, pt_stride: int):
        import torch
        self.model, self.pool = model, pool
        dl, ql = _i32(doc_lens), _i32(query_lens)
        self.n_pairs, self.pt_stride = len(dl), int(pt_stride)
        nbytes = int(lib.hr_rerank_workspace_bytes(model.handle, self.n_pairs, int(ql.sum()), self.pt_stride))
        self.ws = torch.empty(max(nbytes, 256), dtype=torch.uint8, device=model.device)
        out = C.c_void_p()
        check(lib.hr_rerank_plan_create(model.handle, pool.handle, self.n_pairs, _i32p(dl), _i32p(ql), self.pt_stride,
                                        C.c_void_p(self.ws.data_ptr()), self.ws.numel(), C.byref(out)), "hr_rerank_plan_create")
        self.handle = out

    def set_inputs(self, page_table, query_tokens) -> None:
        pt, qt = _i32(page_table), _i32(query_tokens)
        check(lib.hr_rerank_plan_set_inputs(self.handle, _i32p(pt), _i32p(qt)), "hr_rerank_plan_set_inputs")

    def run(self, out, stream=None):
        check(lib.hr_rerank_plan_run(self.handle, C.c_void_p(out.data_ptr()), _stream_ptr(stream)), "hr_rerank_plan_run")
        return out[:self.n_pairs]

    def close(self):
        if getattr(self, "handle", None):
            lib.hr_rerank_plan_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class Model:
    """Uploads weights (numpy fp32 arrays holding values of the model dtype), packs them, keeps the handle."""

    def __init__(self, model_cfg, weights, device="cuda:0"):
        import torch
        self.m = model_cfg
        self.device = device
        self.cfg = make_model_cfg(model_cfg)
        tdt = torch.float32 if model_cfg.dtype == "f32" else torch.bfloat16

        def up(a, dt):
            return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(device=device, dtype=dt)

        self.embedding = up(weights.get("embedding", -1), tdt)
        self.final_norm = up(weights.get("final_norm", -1), torch.float32)
        L = model_cfg.n_layers
        per_layer: Dict[str, List] = {k: [] for k in _LAYER_KINDS}
        for l in range(L):
            for k in _LAYER_KINDS:
                per_layer[k].append(up(weights.get(k, l), torch.float32 if k.startswith("norm") else tdt))
        self.norm1, self.norm2 = per_layer["norm1"], per_layer["norm2"]
        arrays = {k: (C.c_void_p * L)(*[t.data_ptr() for t in per_layer[k]]) for k in _LAYER_KINDS}
        ptrs = hr_weight_ptrs(self.embedding.data_ptr(), self.final_norm.data_ptr(),
                              *[C.cast(arrays[k], _PP) for k in _LAYER_KINDS])
        nbytes = hr_weights_pack_bytes(self.cfg)
        if nbytes == 0:
            raise HrError(HR_ERR_INVALID_ARG, "hr_weights_pack_bytes")
        self.pack = torch.empty(nbytes, dtype=torch.uint8, device=device)
        out = C.c_void_p()
        st = lib.hr_weights_load(C.byref(self.cfg), C.byref(ptrs), C.c_void_p(self.pack.data_ptr()), nbytes,
                                 _stream_ptr(), C.byref(out))
        check(st, "hr_weights_load")
        self.handle = out
        torch.cuda.synchronize()
        del per_layer, arrays          # the matrices now live in the packed copy
        self._ws = None

    def _workspace(self, nbytes: int):
        import torch
        if self._ws is None or self._ws.numel() < nbytes:
            self._ws = None
            self._ws = torch.empty(nbytes, dtype=torch.uint8, device=self.device)
        return self._ws

    def range_report(self) -> dict:
        r = hr_range_report()
        check(lib.hr_model_range_report(self.handle, C.byref(r)), "hr_model_range_report")
        return r.as_dict()

    def gemm_path(self) -> str:
        return lib.hr_gemm_path(self.handle).decode()

    def attention_path(self, pool: KVPool) -> str:
        return lib.hr_attention_path(self.handle, pool.handle).decode()

    def profile_enable(self, on: bool) -> None:
        check(lib.hr_profile_enable(self.handle, 1 if on else 0), "hr_profile_enable")

    def profile_select(self, names=None) -> None:
        """Time only the named kernel classes (None: all)."""
        n = lib.hr_profile_count()
        all_names = [lib.hr_profile_name(i).decode() for i in range(n)]
        mask = 0xFFFFFFFF if names is None else sum(1 << all_names.index(x) for x in names)
        check(lib.hr_profile_select(self.handle, mask), "hr_profile_select")

    def profile_read(self) -> Dict[str, Dict[str, float]]:
        n = lib.hr_profile_count()
        ms = (C.c_double * n)()
        cnt = (C.c_int64 * n)()
        check(lib.hr_profile_read(self.handle, ms, cnt), "hr_profile_read")
        return {lib.hr_profile_name(i).decode(): {"ms": float(ms[i]), "launches": int(cnt[i])} for i in range(n)}

    def score(self, pool: KVPool, page_table, doc_lens, query_tokens, query_lens, out=None, stream=None):
        import torch
        pt = _i32(page_table)
        if pt.ndim == 1:
            pt = pt.reshape(len(doc_lens), -1)
        dl, qt, ql = _i32(doc_lens), _i32(query_tokens), _i32(query_lens)
        P = len(dl)
        stride = pt.shape[1] if pt.ndim == 2 else 0
        nbytes = int(lib.hr_rerank_workspace_bytes(self.handle, P, int(ql.sum()), stride))
        ws = self._workspace(max(nbytes, 256))
        scores = out if out is not None else torch.empty(max(P, 1), dtype=torch.float32, device=self.device)
        st = lib.hr_rerank_score(self.handle, pool.handle, P, _i32p(pt), stride, _i32p(dl), _i32p(qt), _i32p(ql),
                                 C.c_void_p(ws.data_ptr()), ws.numel(), C.c_void_p(scores.data_ptr()), _stream_ptr(stream))
        check(st, "hr_rerank_score")
        return scores[:P]

    def score_static(self, pool: KVPool, page_table, doc_lens, query_tokens, query_lens, out, stream=None):
        """hr_rerank_score_static: the workspace is the library's own static device array; `out` is the caller's
        fp32 device tensor of at least len(doc_lens) scores (nothing is allocated here either)."""
        pt = _i32(page_table)
        if pt.ndim == 1:
            pt = pt.reshape(len(doc_lens), -1)
        dl, qt, ql = _i32(doc_lens), _i32(query_tokens), _i32(query_lens)
        P = len(dl)
        stride = pt.shape[1] if pt.ndim == 2 else 0
        st = lib.hr_rerank_score_static(self.handle, pool.handle, P, _i32p(pt), stride, _i32p(dl), _i32p(qt), _i32p(ql),
                                        C.c_void_p(out.data_ptr()), _stream_ptr(stream))
        check(st, "hr_rerank_score_static")
        return out[:P]

    def parts(self, total_q_tokens: int) -> int:
        return int(lib.hr_rerank_parts(self.handle, int(total_q_tokens)))

    def set_precise_layers(self, n: int) -> None:
        check(lib.hr_model_set_precise_layers(self.handle, int(n)), "hr_model_set_precise_layers")

    def precise_layers(self) -> int:
        return int(lib.hr_model_precise_layers(self.handle))

    def set_streams(self, n: int) -> None:
        check(lib.hr_rerank_set_streams(self.handle, int(n)), "hr_rerank_set_streams")

    def score_full(self, doc_tokens: Sequence[np.ndarray], query_tokens: Sequence[np.ndarray], out=None, stream=None):
        import torch
        P = len(doc_tokens)
        dl = _i32([len(d) for d in doc_tokens])
        ql = _i32([len(q) for q in query_tokens])
        dt = _i32(np.concatenate(doc_tokens)) if P and dl.sum() else np.zeros(1, np.int32)
        qt = _i32(np.concatenate(query_tokens)) if P else np.zeros(1, np.int32)
        total = int(dl.sum() + ql.sum())
        nbytes = int(lib.hr_rerank_full_workspace_bytes(self.handle, P, total))
        ws = self._workspace(max(nbytes, 256))
        scores = out if out is not None else torch.empty(max(P, 1), dtype=torch.float32, device=self.device)
        st = lib.hr_rerank_score_full(self.handle, P, _i32p(dt), _i32p(dl), _i32p(qt), _i32p(ql),
                                      C.c_void_p(ws.data_ptr()), ws.numel(), C.c_void_p(scores.data_ptr()), _stream_ptr(stream))
        check(st, "hr_rerank_score_full")
        return scores[:P]

    def doc_prefill(self, pool: KVPool, doc_tokens: Sequence[np.ndarray], page_lists: Sequence[np.ndarray], stream=None) -> None:
        """Compute and store the documents' K/V on the device (stage one)."""
        n = len(doc_tokens)
        dl = _i32([len(d) for d in doc_tokens])
        stride = max(len(p) for p in page_lists)
        pt = np.full((n, stride), -1, np.int32)
        for i, pg in enumerate(page_lists):
            pt[i, :len(pg)] = pg
        toks = _i32(np.concatenate(doc_tokens))
        nbytes = int(lib.hr_doc_prefill_workspace_bytes(self.handle, n, int(dl.sum())))
        if nbytes == 0:
            raise HrError(HR_ERR_UNSUPPORTED_SHAPE, "hr_doc_prefill_workspace_bytes")
        ws = self._workspace(nbytes)
        st = lib.hr_doc_prefill(self.handle, pool.handle, n, _i32p(toks), _i32p(dl), _i32p(pt), stride,
                                C.c_void_p(ws.data_ptr()), ws.numel(), _stream_ptr(stream))
        check(st, "hr_doc_prefill")

    def close(self):
        if getattr(self, "handle", None):
            lib.hr_model_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
