"""TEST INFRASTRUCTURE - CPU oracle, 4-bit KV transfer format.

The paper names a 4-bit KV cache next to the 8-bit one (Section 4.1 "KV-cache Quantization": KV4W16A16) and says
the quantised KV is expanded to 16 bits after it is loaded, so that the softmax arithmetic is unchanged (Appendix B);
it gives no format and does not use it in its experiments.  This build's reading: 4 bits are the format in which a
document's K/V rests in the storage tier and crosses the bus; the pool in HBM stays 16-bit.  Per token and per 32
consecutive channels of one (layer, kv head), separately for K and V:

    scale = amax / 7 in fp32 (1 if the group is all zero)
    code  = x / scale rounded to the nearest integer, ties to even, clamped to [-7, 7]  (quotient exact: float64)
    x'    = code * scale in fp32, rounded to half: what the pool holds after the page has been loaded again

Only tests, the smoke check and the benchmark's CPU-baseline leg may import this file.  The GPU library shares
nothing with it.
"""

from __future__ import annotations

import numpy as np

GROUP = 32


def quantize(x: np.ndarray):
    """x [..., d] values that are exactly representable in half (d a multiple of 32).
    Returns codes int8 [..., d] in [-7, 7] and scales float32 [..., d / 32]."""
    x = np.asarray(x, dtype=np.float64)
    d = x.shape[-1]
    assert d % GROUP == 0
    g = x.reshape(x.shape[:-1] + (d // GROUP, GROUP))
    amax = np.abs(g).max(axis=-1).astype(np.float32)
    scale = np.where(amax > 0, amax / np.float32(7.0), np.float32(1.0)).astype(np.float32)
    q = g / scale[..., None].astype(np.float64)
    codes = np.clip(np.rint(q), -7, 7).astype(np.int8)          # numpy's rint rounds ties to even
    return codes.reshape(x.shape), scale


def dequantize(codes: np.ndarray, scale: np.ndarray) -> np.ndarray:
    """The half values a loaded page holds, as float64."""
    d = codes.shape[-1]
    c = codes.reshape(codes.shape[:-1] + (d // GROUP, GROUP)).astype(np.float32)
    v = (c * scale[..., None].astype(np.float32)).astype(np.float32)
    return v.astype(np.float16).astype(np.float64).reshape(codes.shape)


def round_trip(x: np.ndarray) -> np.ndarray:
    """What a document's K or V [L][D][n_kv][d] looks like after it has been stored in 4 bits and loaded again."""
    codes, scale = quantize(x)
    return dequantize(codes, scale)
