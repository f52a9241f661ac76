"""Oracle (test infrastructure): 4-bit group-quantised weights (the paper's fastest setting runs the models
quantised to 4 bits; Sect. 5).  The paper takes the quantiser from the literature and does not fix a storage
format; the one used here is the common group-wise one, stated in full:

  * a weight matrix W [N][K] is stored as 4-bit codes q in 0..15, one bf16 scale s and one 4-bit zero point z
    per row and group of `group` consecutive k;  w = s * (q - z);
  * eight codes share a 32-bit word: code j (0..7) of word i of a row is k = 8 i + j and sits in bits 4j..4j+3;
  * the dequantised weight is a bf16 value: s * (q - z) is exact in fp32 (an 8-bit significand times an
    integer of at most 4 bits) and is rounded once to bf16, which is what enters the product.
"""
from __future__ import annotations

import numpy as np

from .model import round_bf16


def unpack_w4(qweight):
    """uint32 [N][K/8] -> codes uint8 [N][K]."""
    q = np.asarray(qweight, dtype=np.uint32)
    out = np.zeros((q.shape[0], q.shape[1] * 8), dtype=np.uint8)
    for j in range(8):
        out[:, j::8] = (q >> np.uint32(4 * j)) & np.uint32(15)
    return out


def dequantize_w4(qweight, scales, zeros, group):
    """Returns W as float64 [N][K] holding bf16 values.  scales: [N][K/group] (bf16 values), zeros: [N][K/group]
    integers 0..15."""
    q = unpack_w4(qweight).astype(np.float64)
    s = np.repeat(np.asarray(scales, dtype=np.float64), group, axis=1)
    z = np.repeat(np.asarray(zeros, dtype=np.float64), group, axis=1)
    return round_bf16(s * (q - z))


def gemm_w4a16(X, qweight, scales, zeros, group):
    """Y = X W^T with W dequantised as above; X [M][K] (bf16 values), fp64 accumulation."""
    X = X.detach().cpu().double().numpy() if hasattr(X, "detach") else np.asarray(X, dtype=np.float64)
    return X @ dequantize_w4(qweight, scales, zeros, group).T
