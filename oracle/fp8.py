"""TEST INFRASTRUCTURE - CPU oracle, 8-bit KV format.

OCP FP8 E4M3 ("E4M3FN": 1 sign, 4 exponent bits with bias 7, 3 mantissa bits,
no infinities, the all-ones exponent+mantissa pattern is NaN, largest finite
448) with one fp32 scale per (layer, page, kv head), separately for K and V.
The paper only says the cached KV may be stored in 8 bits and is expanded to
16 bits after loading (Section 4.1 "KV-cache Quantization", Appendix B); the
concrete format is this build's reading.

Only tests, the smoke check and the benchmark's CPU-baseline leg may import
this file.  The GPU library shares nothing with it.
"""

from __future__ import annotations

import numpy as np

E4M3_MAX = 448.0


def e4m3_decode_table() -> np.ndarray:
    """All 256 codes decoded from the bit-field definition (float64, NaN for 0x7F / 0xFF)."""
    t = np.empty(256, dtype=np.float64)
    for code in range(256):
        sign = -1.0 if code & 0x80 else 1.0
        e = (code >> 3) & 0xF
        m = code & 0x7
        if e == 0xF and m == 0x7:
            t[code] = np.nan
        elif e == 0:
            t[code] = sign * (m / 8.0) * 2.0 ** (1 - 7)
        else:
            t[code] = sign * (1.0 + m / 8.0) * 2.0 ** (e - 7)
    return t


_TABLE = e4m3_decode_table()
_POS = _TABLE[:0x7F]          # 0 .. 448, strictly increasing, index == code


def e4m3_decode(codes: np.ndarray) -> np.ndarray:
    return _TABLE[np.asarray(codes, dtype=np.uint8)]


def e4m3_encode(x: np.ndarray) -> np.ndarray:
    """Round to nearest (ties to the even code), saturating at +-448.  NaN -> 0x7F."""
    x = np.asarray(x, dtype=np.float64)
    a = np.minimum(np.abs(x), E4M3_MAX)
    hi = np.clip(np.searchsorted(_POS, a, side="left"), 0, 0x7E)
    lo = np.maximum(hi - 1, 0)
    d_hi = _POS[hi] - a
    d_lo = a - _POS[lo]
    pick_lo = (d_lo < d_hi) | ((d_lo == d_hi) & (lo % 2 == 0))
    code = np.where(pick_lo, lo, hi).astype(np.uint8)
    code = np.where(np.signbit(x), code | 0x80, code).astype(np.uint8)
    return np.where(np.isnan(x), np.uint8(0x7F), code).astype(np.uint8)


def quantize_doc_kv(x: np.ndarray, page_tokens: int = 16):
    """Quantise one document's K (or V), logical layout [L][D][n_kv][d].

    scale[l][page][h] = amax over the page's valid tokens and all d / 448
    (1.0 when that amax is 0); code = encode(x / scale).
    Returns (codes uint8 like x, scales float32 [L][n_pages][n_kv]).
    """
    x = np.asarray(x, dtype=np.float64)
    L, D, n_kv, d = x.shape
    n_pages = (D + page_tokens - 1) // page_tokens
    codes = np.zeros(x.shape, dtype=np.uint8)
    scales = np.ones((L, n_pages, n_kv), dtype=np.float32)
    for p in range(n_pages):
        t0, t1 = p * page_tokens, min(D, (p + 1) * page_tokens)
        amax = np.abs(x[:, t0:t1]).max(axis=(1, 3))               # [L][n_kv]
        s = np.where(amax > 0, amax / E4M3_MAX, 1.0).astype(np.float32)
        scales[:, p, :] = s
        codes[:, t0:t1] = e4m3_encode(x[:, t0:t1] / s.astype(np.float64)[:, None, :, None])
    return codes, scales


def dequantize_doc_kv(codes: np.ndarray, scales: np.ndarray, page_tokens: int = 16) -> np.ndarray:
    """Inverse of quantize_doc_kv: decode(code) * scale, float64, layout [L][D][n_kv][d]."""
    L, D, n_kv, d = codes.shape
    per_tok = np.repeat(np.asarray(scales, dtype=np.float64), page_tokens, axis=1)[:, :D]   # [L][D][n_kv]
    return e4m3_decode(codes) * per_tok[..., None]
