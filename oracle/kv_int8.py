"""Oracle for the INT8 KV cache.  TEST INFRASTRUCTURE ONLY.

The paper's appendix (quantization schemes): keys, queries and values are quantized dynamically
per head and per token, i.e. one range per row of D head elements -- the inner-product dimension
of the score product, which can then be taken in integer arithmetic.  Reading taken here (the paper gives the granularity, not the formula): symmetric
INT8 with the row's largest magnitude mapped to 127,

    amax = max_d |x_d|          (x: the bf16 row the model produced, exact in fp32)
    inv  = 127 / amax           (one fp32 division; amax = 0: inv = 0)
    code_d = rint(x_d * inv)    (one fp32 product, round half to even; in [-127, 127])
    s    = amax / 127           (one fp32 division): x_d is represented by code_d * s.

Every step is a single IEEE fp32 operation, so an implementation that takes the same steps gets
the same codes and scales bit for bit.  The attention over an INT8 cache is the plain ragged
attention over the represented values code * s of the queries (quantized per token and query
head), keys and values (oracle.verify_attention on fp32 inputs).
"""
from __future__ import annotations

import numpy as np


def quantize_rows(x_f32: np.ndarray):
    """[..., D] fp32 rows -> (int8 codes [..., D], fp32 scales [...])."""
    x = np.ascontiguousarray(x_f32, dtype=np.float32)
    amax = np.abs(x).max(axis=-1).astype(np.float32)
    safe = np.where(amax > 0, amax, np.float32(1)).astype(np.float32)
    inv = np.where(amax > 0, np.float32(127.0) / safe, np.float32(0)).astype(np.float32)
    prod = (x * inv[..., None]).astype(np.float32)
    codes = np.rint(prod).astype(np.int32)          # numpy rounds half to even
    assert codes.min(initial=0) >= -127 and codes.max(initial=0) <= 127
    scale = (amax / np.float32(127.0)).astype(np.float32)
    return codes.astype(np.int8), scale


def dequantize_rows(codes: np.ndarray, scale: np.ndarray) -> np.ndarray:
    """Represented values code * s as fp32 (the product is rounded once to fp32)."""
    return (codes.astype(np.float32) * scale[..., None].astype(np.float32)).astype(np.float32)
