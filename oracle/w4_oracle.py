"""CPU oracle of the 4-bit expert-weight format (weights-only quantisation of the expert FFN).

TEST INFRASTRUCTURE ONLY: imported by tests, the smoke check and the benchmark's CPU-baseline leg; the
library's quantiser and kernels are written separately.

The paper runs its experts in 4 bits on the GPU (Marlin kernels, Section V) but does not define the
format.  The format here is the common group-wise symmetric one, written out so that both sides take
every rounding decision in the same precision:
  * a matrix W [N, K] (row = output feature) is cut along K into groups of 128;
  * scale of (row n, group g):  s = bf16( max_k |W[n, k]| / 7 ), the maximum and the division in fp32,
    the result rounded to bfloat16 (nearest even);
  * code of an element:  q = clamp( rint( W[n, k] / s ), -8, 7 ) + 8  in fp32 (rint = nearest even), an
    unsigned nibble; a group of zeros has s = 0 and all codes 8;
  * the value a code stands for is (q - 8) * s, and the quantised expert is the SwiGLU FFN of the layer
    equation with every weight replaced by that value.
"""
from __future__ import annotations

from typing import Tuple

import numpy as np

GROUP = 128


def _bf16_round(a: np.ndarray) -> np.ndarray:
    """fp32 -> nearest bfloat16 (ties to even), returned as fp32."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32).astype(np.uint64)
    u = (u + 0x7FFF + ((u >> 16) & 1)) >> 16 << 16
    return u.astype(np.uint32).view(np.float32)


def quantize_w4(w: np.ndarray) -> Tuple[np.ndarray, np.ndarray]:
    """w [N, K] float (values already representable in the storage dtype), K % 128 == 0.
    -> codes uint8 [N, K] in 0..15, scales fp32 [N, K/128] (each exactly a bfloat16 value)."""
    w = np.ascontiguousarray(w, dtype=np.float32)
    n, k = w.shape
    assert k % GROUP == 0
    g = w.reshape(n, k // GROUP, GROUP)
    scales = _bf16_round(np.abs(g).max(axis=2) / np.float32(7.0))
    safe = np.where(scales == 0, np.float32(1.0), scales)
    q = np.rint(g / safe[:, :, None]).astype(np.float32)          # fp32 division, nearest even
    q = np.clip(q, -8, 7) + 8
    q = np.where(scales[:, :, None] == 0, 8, q)
    return q.reshape(n, k).astype(np.uint8), scales


def dequantize_w4(codes: np.ndarray, scales: np.ndarray) -> np.ndarray:
    """-> float64 [N, K]: (q - 8) * s."""
    n, k = codes.shape
    v = (codes.astype(np.float64) - 8.0).reshape(n, k // GROUP, GROUP) * scales.astype(np.float64)[:, :, None]
    return v.reshape(n, k)
