"""ctypes front end of the plain-C oracle (ogc_oracle.c).  TEST INFRASTRUCTURE ONLY.

The arithmetic lives in the C file; this module only compiles it, marshals numpy arrays and
walks a layer chain one layer at a time (each layer's output array is the next layer's input,
exactly as the definition says: no fusion, no buffer tricks).
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import List, Optional, Sequence

import numpy as np

ACT_NONE, ACT_RELU, ACT_GELU_TANH, ACT_SIGMOID = 0, 1, 2, 3

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "ogc_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (-O2 -fopenmp -ffp-contract=off, no fast-math)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.check_call(
            ["gcc", "-O2", "-fopenmp", "-ffp-contract=off", "-shared", "-fPIC", "-Wall", "-o", tmp, _SRC, "-lm"]
        )
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        c_int, c_float, c_void_p = ctypes.c_int, ctypes.c_float, ctypes.c_void_p
        lib.oracle_layer_f32.argtypes = [c_int] * 3 + [c_void_p, c_int, c_void_p, c_void_p, c_int, c_void_p, c_int,
                                                       c_void_p, c_int, c_int]
        lib.oracle_layer_f32.restype = c_int
        lib.oracle_layer_bf16.argtypes = lib.oracle_layer_f32.argtypes
        lib.oracle_layer_bf16.restype = c_int
        lib.oracle_layer_i8.argtypes = [c_int] * 3 + [c_void_p, c_int, c_void_p, c_void_p, c_void_p, c_float, c_int,
                                                      c_int, c_int, c_float, c_int, c_void_p, c_int]
        lib.oracle_layer_i8.restype = c_int
        lib.oracle_layer_i8_unfused.argtypes = [c_int] * 3 + [c_void_p, c_int, c_void_p, c_void_p, c_void_p, c_float,
                                                              c_int, c_int, c_float, c_int, c_void_p, c_int]
        lib.oracle_layer_i8_unfused.restype = c_int
        lib.oracle_layer_f8.argtypes = [c_int] * 3 + [c_void_p, c_int, c_void_p, c_void_p, c_void_p, c_float, c_int, c_int,
                                                      c_float, c_void_p, c_int, c_int]
        lib.oracle_layer_f8.restype = c_int
        lib.oracle_e4m3_to_f32.argtypes = [ctypes.c_uint8]
        lib.oracle_e4m3_to_f32.restype = c_float
        lib.oracle_f32_to_e4m3.argtypes = [c_float]
        lib.oracle_f32_to_e4m3.restype = ctypes.c_uint8
        lib.oracle_num_threads.restype = c_int
        lib.oracle_act_f64.argtypes = [ctypes.c_double, c_int]
        lib.oracle_act_f64.restype = ctypes.c_double
        lib.oracle_act_f32.argtypes = [c_float, c_int]
        lib.oracle_act_f32.restype = c_float
        _lib = lib
    return _lib


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def act_f64(y: float, act: int) -> float:
    return float(_load().oracle_act_f64(float(y), int(act)))


def act_f32(y: float, act: int) -> float:
    return float(_load().oracle_act_f32(float(y), int(act)))


def _ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _c(a: Optional[np.ndarray], dtype) -> Optional[np.ndarray]:
    if a is None:
        return None
    a = np.asarray(a)
    assert a.dtype == np.dtype(dtype), (a.dtype, dtype)
    assert a.ndim <= 2
    if a.ndim == 2:
        assert a.strides[1] == a.itemsize and a.strides[0] % a.itemsize == 0, "rows must be contiguous"
    return a


def _ld(a: np.ndarray) -> int:
    if a.ndim == 2 and a.shape[0] > 1:
        return a.strides[0] // a.itemsize
    return max(a.shape[-1], 1)


def _float_layer(fn, dt, x, w, bias, act, residual, accum_double):
    x, w = _c(x, dt), np.ascontiguousarray(_c(w, dt))
    bias = None if bias is None else np.ascontiguousarray(_c(bias, np.float32))
    residual = _c(residual, dt)
    m, k = x.shape
    k2, n = w.shape
    assert k == k2 and (bias is None or bias.shape == (n,))
    assert residual is None or residual.shape == (m, n)
    y = np.zeros((m, n), dtype=dt)
    rc = fn(m, k, n, _ptr(x), _ld(x), _ptr(w), _ptr(bias), int(act), _ptr(residual),
            _ld(residual) if residual is not None else 0, _ptr(y), n, int(bool(accum_double)))
    if rc != 0:
        raise RuntimeError("oracle layer failed: %d" % rc)
    return y


def layer_f32(x, w, bias=None, act=ACT_NONE, residual=None, accum_double=False) -> np.ndarray:
    """Y = act(X W + bias) (+ residual); fp32 arrays, W is [K, N]."""
    return _float_layer(_load().oracle_layer_f32, np.float32, x, w, bias, act, residual, accum_double)


def layer_bf16(x, w, bias=None, act=ACT_NONE, residual=None, accum_double=False) -> np.ndarray:
    """Same with bf16 bit patterns (uint16 arrays); bias fp32; output rounded to bf16 (RNE)."""
    return _float_layer(_load().oracle_layer_bf16, np.uint16, x, w, bias, act, residual, accum_double)


def layer_i8(xq, wq, w_scale, bias, a_s, a_z, act, c_s=1.0, c_z=0, out_f32=False) -> np.ndarray:
    """u8 activations x s8 per-channel weights -> u8 (requantized) or fp32 (out_f32)."""
    xq, wq = _c(xq, np.uint8), np.ascontiguousarray(_c(wq, np.int8))
    w_scale = np.ascontiguousarray(_c(w_scale, np.float32))
    bias = None if bias is None else np.ascontiguousarray(_c(bias, np.float32))
    m, k = xq.shape
    k2, n = wq.shape
    assert k == k2 and w_scale.shape == (n,) and (bias is None or bias.shape == (n,))
    y = np.zeros((m, n), dtype=np.float32 if out_f32 else np.uint8)
    rc = _load().oracle_layer_i8(m, k, n, _ptr(xq), _ld(xq), _ptr(wq), _ptr(w_scale), _ptr(bias), float(a_s), int(a_z),
                                 int(act), int(bool(out_f32)), float(c_s), int(c_z), _ptr(y), n)
    if rc != 0:
        raise RuntimeError("oracle int8 layer failed: %d" % rc)
    return y


def layer_i8_unfused(xq, wq, w_scale, bias, a_s, a_z, act, c_s, c_z) -> np.ndarray:
    """dequantize -> real matmul (fp64) -> bias -> act -> quantize with a true division."""
    xq, wq = _c(xq, np.uint8), np.ascontiguousarray(_c(wq, np.int8))
    w_scale = np.ascontiguousarray(_c(w_scale, np.float32))
    bias = None if bias is None else np.ascontiguousarray(_c(bias, np.float32))
    m, k = xq.shape
    n = wq.shape[1]
    y = np.zeros((m, n), dtype=np.uint8)
    rc = _load().oracle_layer_i8_unfused(m, k, n, _ptr(xq), _ld(xq), _ptr(wq), _ptr(w_scale), _ptr(bias), float(a_s),
                                         int(a_z), int(act), float(c_s), int(c_z), _ptr(y), n)
    if rc != 0:
        raise RuntimeError("oracle unfused int8 layer failed: %d" % rc)
    return y


def e4m3_to_f32(code: int) -> float:
    """Value of one E4M3 code (NaN for 0x7f / 0xff)."""
    return float(_load().oracle_e4m3_to_f32(int(code) & 0xFF))


def f32_to_e4m3(value: float) -> int:
    """fp32 -> E4M3 code, nearest-even, saturating at +-448."""
    return int(_load().oracle_f32_to_e4m3(float(np.float32(value))))


def layer_f8(x8, w8, w_scale, bias, a_s, act, c_s=1.0, out_f32=False, accum_double=True) -> np.ndarray:
    """E4M3 activations x E4M3 per-channel-scaled weights -> E4M3 (requantized) or fp32 (out_f32)."""
    x8, w8 = _c(x8, np.uint8), np.ascontiguousarray(_c(w8, np.uint8))
    w_scale = np.ascontiguousarray(_c(w_scale, np.float32))
    bias = None if bias is None else np.ascontiguousarray(_c(bias, np.float32))
    m, k = x8.shape
    k2, n = w8.shape
    assert k == k2 and w_scale.shape == (n,) and (bias is None or bias.shape == (n,))
    y = np.zeros((m, n), dtype=np.float32 if out_f32 else np.uint8)
    rc = _load().oracle_layer_f8(m, k, n, _ptr(x8), _ld(x8), _ptr(w8), _ptr(w_scale), _ptr(bias), float(a_s), int(act),
                                 int(bool(out_f32)), float(c_s), _ptr(y), n, int(bool(accum_double)))
    if rc != 0:
        raise RuntimeError("oracle fp8 layer failed: %d" % rc)
    return y


def mlp(wl, rows: Optional[slice] = None, accum_double: bool = False, keep: bool = False):
    """Run a whole chain described by a synthetic workload object (fields: dtype, layers, x, w,
    bias, w_scale, residual).  Returns the final output, or the list of every layer's output if
    keep is set.  rows selects a slice of the batch (rows are independent)."""
    x0 = wl.x if rows is None else wl.x[rows]
    outs: List[np.ndarray] = []
    cur = x0
    nl = len(wl.layers)
    for i, ly in enumerate(wl.layers):
        bias = wl.bias[i] if ly.has_bias else None
        res = x0 if (wl.residual and i == nl - 1) else None
        if wl.dtype == "f32":
            cur = layer_f32(cur, wl.w[i], bias, ly.act, res, accum_double)
        elif wl.dtype == "bf16":
            cur = layer_bf16(cur, wl.w[i], bias, ly.act, res, accum_double)
        elif wl.dtype == "i8":
            assert res is None
            cur = layer_i8(cur, wl.w[i], wl.w_scale[i], bias, ly.in_scale, ly.in_zp, ly.act, ly.out_scale, ly.out_zp,
                           ly.out_f32)
        elif wl.dtype == "f8":
            assert res is None
            # the fp64 sum is exact, so it is the reference whichever order the hardware adds in
            cur = layer_f8(cur, wl.w[i], wl.w_scale[i], bias, ly.in_scale, ly.act, ly.out_scale, ly.out_f32, accum_double=True)
        else:
            raise ValueError(wl.dtype)
        outs.append(cur)
    return outs if keep else cur
