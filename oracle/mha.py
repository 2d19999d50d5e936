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


def attention_i8(q: np.ndarray, k: np.ndarray, v: np.ndarray, mask: Optional[np.ndarray], scale: float, q_scale: float,
                 k_scale: float, v_scale: float, o_scale: float, return_weights: bool = False):
    """The Int8 rows of Table I.  The paper gives the scheme of its Int8 graphs only in general terms (Section V:
    low-precision conversion, Section VII: the quantization scheme) and not where the attention subgraph
    quantizes, so this is a reading, stated step by step (all tensors per batch entry and head):

      q, k, v   int8, symmetric (zero point 0: a batch matmul has no constant operand into which a zero point
                could be folded), real value = scale_of_tensor * integer
      S[i][j]   = sum_c q[i][c] k[j][c]                                   int32, exact
      s[i][j]   = S[i][j] * (q_scale * k_scale * scale) + mask[j]         dequantize, divide by the scalar, add the mask
      e[i][j]   = exp(s[i][j] - max_j s[i][j])                            softmax numerators, in (0, 1]
      P[i][j]   = rne(127 * e[i][j])                                      quantized to 7 bits unsigned (fits the signed
                                                                          int8 operand of the second matmul as it is)
      A[i][c]   = sum_j P[i][j] v[j][c],  L[i] = sum_j P[i][j]            int32, exact; L >= 127
      o[i][c]   = clamp(rne((float(A) / float(L)) * (v_scale / o_scale)), -128, 127)   fp32 operations, each rounded to
                                                                          nearest even: int->float, divide, multiply

    The normalisation by the sum of the QUANTIZED numerators comes after the integer product, so everything after P
    is exact integer arithmetic plus three fp32 operations that any implementation can reproduce bit for bit; only P
    itself depends on how an implementation evaluates exp (here: float64).
    q, k, v: [B, H, S, d] int8.  mask: [B, S] or None.  Returns o [B, H, S, d] int8 (and P as uint8 [B, H, S, S])."""
    q8, k8, v8 = (np.asarray(t) for t in (q, k, v))
    assert q8.dtype == k8.dtype == v8.dtype == np.int8 and q8.ndim == 4 and q8.shape == k8.shape == v8.shape
    s_int = np.matmul(q8.astype(np.int64), np.swapaxes(k8.astype(np.int64), -1, -2))
    c = np.float64(np.float32(q_scale)) * np.float64(np.float32(k_scale)) * np.float64(np.float32(scale))
    s = s_int.astype(np.float64) * c
    if mask is not None:
        m64 = np.asarray(mask, dtype=np.float64)
        assert m64.shape == (q8.shape[0], q8.shape[2])
        s = s + m64[:, None, None, :]
    e = np.exp(s - np.max(s, axis=-1, keepdims=True))
    p = np.rint(127.0 * e)                                   # numpy rounds halves to even
    assert p.min() >= 0 and p.max() == 127
    p_int = p.astype(np.int64)
    a = np.matmul(p_int, v8.astype(np.int64))
    l = p_int.sum(axis=-1, keepdims=True)
    r = np.float32(v_scale) / np.float32(o_scale)            # one fp32 division
    t = (a.astype(np.float32) / l.astype(np.float32)) * r    # fp32 divide, fp32 multiply
    o = np.clip(np.rint(t), -128, 127).astype(np.int8)
    return (o, p.astype(np.uint8)) if return_weights else o
