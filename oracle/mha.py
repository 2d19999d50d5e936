"""CPU oracle for the scaled dot-product attention subgraph.  TEST INFRASTRUCTURE ONLY.

The paper's second workload (Section VII, Table I rows MHA-1..4) is the scaled dot-product part of
multi-head attention: a batch matmul of queries with transposed keys, a division by a scalar, the
addition of a mask, a softmax over the keys, and a batch matmul with the values.  This module
writes that definition out in numpy float64, one step per line, in that order; there is no
blocking, no running maximum, no fusion.

Two softmax forms (Section VII names a fast softmax that drops the max reduction):
  stable: exp(s - max_j s) / sum_j exp(s - max_j s)
  fast:   exp(s) / sum_j exp(s)
They are the same function wherever exp(s) does not overflow.

Only the tests, the smoke check and the cpu_baseline leg of the benchmark may import this module; it
imports nothing from the GPU package.
"""
from __future__ import annotations

from typing import Optional

import numpy as np

SOFTMAX_STABLE, SOFTMAX_FAST = 0, 1


def attention(q: np.ndarray, k: np.ndarray, v: np.ndarray, mask: Optional[np.ndarray], scale: float,
              softmax: int = SOFTMAX_STABLE) -> np.ndarray:
    """q, k, v: [B, H, S, d] (any float dtype, taken to float64).  mask: [B, S] additive, one value per key,
    the same for every head and every query of a batch entry (the padding mask of a BERT encoder), or
    None.  scale: the reciprocal of the divisor, taken as an fp32 value (the divide becomes a multiply by
    an fp32 constant, as for the requantize scale of the MLP path).  Returns [B, H, S, d] float64."""
    q64 = np.asarray(q, dtype=np.float64)
    k64 = np.asarray(k, dtype=np.float64)
    v64 = np.asarray(v, dtype=np.float64)
    assert q64.ndim == 4 and q64.shape == k64.shape == v64.shape
    s = np.matmul(q64, np.swapaxes(k64, -1, -2))          # [B,H,Sq,Sk]: s[i][j] = sum_c q[i][c] k[j][c]
    s = s * np.float64(np.float32(scale))
    if mask is not None:
        m64 = np.asarray(mask, dtype=np.float64)
        assert m64.shape == (q64.shape[0], q64.shape[2])
        s = s + m64[:, None, None, :]                     # one value per key j
    if softmax == SOFTMAX_STABLE:
        s = s - np.max(s, axis=-1, keepdims=True)
    elif softmax != SOFTMAX_FAST:
        raise ValueError("softmax must be SOFTMAX_STABLE or SOFTMAX_FAST")
    e = np.exp(s)
    p = e / np.sum(e, axis=-1, keepdims=True)
    return np.matmul(p, v64)                              # o[i][c] = sum_j p[i][j] v[j][c]
