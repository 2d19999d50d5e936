"""Thin ctypes binding of libogc_mlp.so (include/ogc_mlp.h): argument marshalling only.

Every step of the path runs in the library's HIP kernels.  PyTorch appears here only as the owner
of device memory and streams.  There is no CPU fallback: if the shared library is missing, loading
it raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import List, Optional, Sequence

OGC_F32, OGC_BF16, OGC_I8, OGC_F8 = 0, 1, 2, 3
OGC_ACT_NONE, OGC_ACT_RELU, OGC_ACT_GELU_TANH, OGC_ACT_SIGMOID = 0, 1, 2, 3
OGC_OUT_SAME, OGC_OUT_F32 = 0, 1
OGC_MODE_AUTO, OGC_MODE_PER_LAYER, OGC_MODE_FUSED, OGC_MODE_COOP = 0, 1, 2, 3
OGC_LAYOUT_PLAIN, OGC_LAYOUT_BLOCKED = 0, 1
OGC_SOFTMAX_STABLE, OGC_SOFTMAX_FAST = 0, 1
OGC_OK = 0
DTYPES = {"f32": OGC_F32, "bf16": OGC_BF16, "i8": OGC_I8, "f8": OGC_F8}

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libogc_mlp.so")

EXPORTS = [
    "ogc_mlp_plan", "ogc_mlp_packed_bytes", "ogc_mlp_workspace_bytes", "ogc_mlp_chosen_mode",
    "ogc_mlp_buffer_assignment", "ogc_mlp_prepack_weights", "ogc_mlp_run", "ogc_mlp_destroy",
    "ogc_status_string", "ogc_mlp_kernel_name", "ogc_mlp_num_launches", "ogc_mlp_run_profiled", "ogc_mlp_blocked_bytes", "ogc_mlp_estimated_us", "ogc_mlp_mode_estimates",
    "ogc_mlp_run_static", "ogc_mlp_static_workspace_limit", "ogc_mlp_plan_with_overrides", "ogc_mlp_check", "ogc_mlp_test_barrier", "ogc_mlp_cluster_layout",
    "ogc_mlp_run_clocked", "ogc_mlp_clock_words_per_launch",
    "ogc_quantize_e4m3", "ogc_dequantize_e4m3",
    "ogc_mha_validate", "ogc_mha_run", "ogc_mha_kernel_name", "ogc_mha_i8_validate", "ogc_mha_run_i8", "ogc_mha_i8_kernel_name",
]
OGC_ERR_TIMEOUT = -8


class ogc_layer_desc(ctypes.Structure):
    _fields_ = [("k", ctypes.c_int32), ("n", ctypes.c_int32), ("has_bias", ctypes.c_int32), ("act", ctypes.c_int32),
                ("in_scale", ctypes.c_float), ("in_zp", ctypes.c_int32), ("out_scale", ctypes.c_float),
                ("out_zp", ctypes.c_int32), ("out", ctypes.c_int32)]


class ogc_mlp_desc(ctypes.Structure):
    _fields_ = [("dtype", ctypes.c_int32), ("m", ctypes.c_int32), ("n_layers", ctypes.c_int32),
                ("layers", ctypes.POINTER(ogc_layer_desc)), ("ld_x", ctypes.c_int32), ("ld_y", ctypes.c_int32),
                ("residual", ctypes.c_int32), ("mode", ctypes.c_int32), ("x_layout", ctypes.c_int32),
                ("y_layout", ctypes.c_int32)]


class ogc_plan_overrides(ctypes.Structure):
    _fields_ = [("tile", ctypes.c_int32), ("ksplit_log2", ctypes.c_int32), ("cluster_split", ctypes.c_int32),
                ("cluster_ksplit", ctypes.c_int32), ("cluster_whole", ctypes.c_int32)]


class ogc_mha_desc(ctypes.Structure):
    _fields_ = [("dtype", ctypes.c_int32), ("batch", ctypes.c_int32), ("heads", ctypes.c_int32), ("seq", ctypes.c_int32),
                ("head_dim", ctypes.c_int32), ("softmax", ctypes.c_int32), ("scale", ctypes.c_float),
                ("q_stride", ctypes.c_int64 * 3), ("k_stride", ctypes.c_int64 * 3), ("v_stride", ctypes.c_int64 * 3),
                ("o_stride", ctypes.c_int64 * 3), ("query_groups", ctypes.c_int32)]


class ogc_mha_quant(ctypes.Structure):
    _fields_ = [("q_scale", ctypes.c_float), ("k_scale", ctypes.c_float), ("v_scale", ctypes.c_float), ("o_scale", ctypes.c_float)]


class OgcError(RuntimeError):
    def __init__(self, status: int, what: str):
        self.status = status
        super().__init__("%s: %s (%d)" % (what, status_string(status), status))


_lib = None


def lib():
    """Loads the shared library (fails loudly if it has not been built)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(
                "%s not found: build it with `python -m paper_2301_01333_amd.build` (there is no fallback path)" % LIB_PATH)
        l = ctypes.CDLL(LIB_PATH)
        vp, i32, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_size_t
        l.ogc_mlp_plan.argtypes = [ctypes.POINTER(ogc_mlp_desc), ctypes.POINTER(vp)]
        l.ogc_mlp_plan.restype = i32
        l.ogc_mlp_plan_with_overrides.argtypes = [ctypes.POINTER(ogc_mlp_desc), ctypes.POINTER(ogc_plan_overrides), ctypes.POINTER(vp)]
        l.ogc_mlp_plan_with_overrides.restype = i32
        l.ogc_mlp_check.argtypes = [vp, vp, vp]
        l.ogc_mlp_check.restype = i32
        l.ogc_mlp_test_barrier.argtypes = [vp, i32, i32]
        l.ogc_mlp_test_barrier.restype = i32
        l.ogc_mlp_cluster_layout.argtypes = [vp, ctypes.POINTER(i32), ctypes.POINTER(i32), ctypes.POINTER(ctypes.c_uint32), ctypes.POINTER(sz)]
        l.ogc_mlp_cluster_layout.restype = i32
        l.ogc_mlp_packed_bytes.argtypes = [vp, ctypes.POINTER(sz)]
        l.ogc_mlp_packed_bytes.restype = i32
        l.ogc_mlp_workspace_bytes.argtypes = [vp, ctypes.POINTER(sz)]
        l.ogc_mlp_workspace_bytes.restype = i32
        l.ogc_mlp_blocked_bytes.argtypes = [vp, i32, ctypes.POINTER(sz)]
        l.ogc_mlp_blocked_bytes.restype = i32
        l.ogc_mlp_chosen_mode.argtypes = [vp, ctypes.POINTER(i32)]
        l.ogc_mlp_chosen_mode.restype = i32
        l.ogc_mlp_buffer_assignment.argtypes = [vp, i32, ctypes.POINTER(i32), ctypes.POINTER(sz)]
        l.ogc_mlp_buffer_assignment.restype = i32
        l.ogc_mlp_prepack_weights.argtypes = [vp, ctypes.POINTER(vp), ctypes.POINTER(vp), ctypes.POINTER(vp), vp, vp]
        l.ogc_mlp_prepack_weights.restype = i32
        l.ogc_mlp_run.argtypes = [vp, vp, vp, vp, vp, vp]
        l.ogc_mlp_run.restype = i32
        l.ogc_mlp_run_static.argtypes = [vp, vp, vp, vp, vp]
        l.ogc_mlp_run_static.restype = i32
        l.ogc_mlp_static_workspace_limit.argtypes = []
        l.ogc_mlp_static_workspace_limit.restype = sz
        l.ogc_mlp_num_launches.argtypes = [vp, ctypes.POINTER(i32)]
        l.ogc_mlp_num_launches.restype = i32
        l.ogc_mlp_run_clocked.argtypes = [vp, vp, vp, vp, vp, vp, vp]
        l.ogc_mlp_run_clocked.restype = i32
        l.ogc_mlp_clock_words_per_launch.argtypes = []
        l.ogc_mlp_clock_words_per_launch.restype = ctypes.c_size_t
        l.ogc_mlp_run_profiled.argtypes = [vp, vp, vp, vp, vp, vp, ctypes.POINTER(ctypes.c_float)]
        l.ogc_mlp_run_profiled.restype = i32
        l.ogc_mlp_destroy.argtypes = [vp]
        l.ogc_mlp_destroy.restype = None
        l.ogc_status_string.argtypes = [i32]
        l.ogc_status_string.restype = ctypes.c_char_p
        l.ogc_mlp_kernel_name.argtypes = [vp, i32]
        l.ogc_mlp_kernel_name.restype = ctypes.c_char_p
        l.ogc_mlp_estimated_us.argtypes = [vp, i32, ctypes.POINTER(ctypes.c_float)]
        l.ogc_mlp_estimated_us.restype = i32
        l.ogc_mlp_mode_estimates.argtypes = [vp, ctypes.POINTER(ctypes.c_float)]
        l.ogc_mlp_mode_estimates.restype = i32
        l.ogc_quantize_e4m3.argtypes = [vp, vp, sz, ctypes.c_float, vp]
        l.ogc_quantize_e4m3.restype = i32
        l.ogc_dequantize_e4m3.argtypes = [vp, vp, sz, ctypes.c_float, vp]
        l.ogc_dequantize_e4m3.restype = i32
        l.ogc_mha_validate.argtypes = [ctypes.POINTER(ogc_mha_desc)]
        l.ogc_mha_validate.restype = i32
        l.ogc_mha_run.argtypes = [ctypes.POINTER(ogc_mha_desc), vp, vp, vp, vp, vp, vp]
        l.ogc_mha_run.restype = i32
        l.ogc_mha_kernel_name.argtypes = [ctypes.POINTER(ogc_mha_desc), i32]
        l.ogc_mha_kernel_name.restype = ctypes.c_char_p
        l.ogc_mha_i8_validate.argtypes = [ctypes.POINTER(ogc_mha_desc), ctypes.POINTER(ogc_mha_quant)]
        l.ogc_mha_i8_validate.restype = i32
        l.ogc_mha_run_i8.argtypes = [ctypes.POINTER(ogc_mha_desc), ctypes.POINTER(ogc_mha_quant), vp, vp, vp, vp, vp, vp]
        l.ogc_mha_run_i8.restype = i32
        l.ogc_mha_i8_kernel_name.argtypes = [ctypes.POINTER(ogc_mha_desc)]
        l.ogc_mha_i8_kernel_name.restype = ctypes.c_char_p
        _lib = l
    return _lib


def status_string(status: int) -> str:
    return lib().ogc_status_string(int(status)).decode()


def _check(status: int, what: str) -> None:
    if status != OGC_OK:
        raise OgcError(status, what)


# ---- one function per entry point, same names ---------------------------------------------------
def _desc(dtype, m, layers, ld_x, ld_y, residual, mode, x_layout, y_layout):
    arr = (ogc_layer_desc * max(len(layers), 1))()
    for i, ly in enumerate(layers):
        arr[i] = ogc_layer_desc(int(ly["k"]), int(ly["n"]), int(ly.get("has_bias", 0)), int(ly.get("act", 0)),
                                float(ly.get("in_scale", 0.0)), int(ly.get("in_zp", 0)), float(ly.get("out_scale", 0.0)),
                                int(ly.get("out_zp", 0)), int(ly.get("out", 0)))
    desc = ogc_mlp_desc(int(dtype), int(m), len(layers), arr, int(ld_x), int(ld_y), int(residual), int(mode), int(x_layout),
                        int(y_layout))
    return desc, arr


def ogc_mlp_plan(dtype: int, m: int, layers: Sequence[dict], ld_x: int, ld_y: int, residual: int = 0, mode: int = 0,
                 x_layout: int = 0, y_layout: int = 0) -> int:
    """layers: dicts with k, n, has_bias, act, in_scale, in_zp, out_scale, out_zp, out.  Returns the plan handle."""
    desc, _keep = _desc(dtype, m, layers, ld_x, ld_y, residual, mode, x_layout, y_layout)
    handle = ctypes.c_void_p()
    _check(lib().ogc_mlp_plan(ctypes.byref(desc), ctypes.byref(handle)), "ogc_mlp_plan")
    return handle.value


def ogc_mlp_plan_with_overrides(dtype: int, m: int, layers: Sequence[dict], ld_x: int, ld_y: int, residual: int = 0,
                                mode: int = 0, x_layout: int = 0, y_layout: int = 0, overrides: Optional[dict] = None) -> int:
    """overrides: dict with any of tile, ksplit_log2, cluster_split, cluster_ksplit, cluster_whole (missing or None = -1,
    the cost model's choice); None passes a NULL pointer."""
    desc, _keep = _desc(dtype, m, layers, ld_x, ld_y, residual, mode, x_layout, y_layout)
    ov = None
    if overrides is not None:
        unknown = set(overrides) - {f for f, _ in ogc_plan_overrides._fields_}
        if unknown:
            raise KeyError("unknown plan overrides: %s" % sorted(unknown))
        ov = ogc_plan_overrides(*[-1 if overrides.get(f) is None else int(overrides[f]) for f, _ in ogc_plan_overrides._fields_])
    handle = ctypes.c_void_p()
    _check(lib().ogc_mlp_plan_with_overrides(ctypes.byref(desc), ctypes.byref(ov) if ov is not None else None,
                                             ctypes.byref(handle)), "ogc_mlp_plan_with_overrides")
    return handle.value


def ogc_mlp_check(plan: int, packed_ptr: int, stream: int = 0) -> int:
    """Returns the status (OGC_OK or OGC_ERR_TIMEOUT); raises on any other error."""
    st = int(lib().ogc_mlp_check(plan, packed_ptr, stream))
    if st not in (OGC_OK, OGC_ERR_TIMEOUT):
        raise OgcError(st, "ogc_mlp_check")
    return st


def ogc_mlp_test_barrier(plan: int, budget: int, extra_target: int) -> None:
    _check(lib().ogc_mlp_test_barrier(plan, int(budget), int(extra_target)), "ogc_mlp_test_barrier")


def ogc_mlp_cluster_layout(plan: int):
    """(members per row tile, k-split variant?, whole-layer mask, tile stride in bytes)."""
    m, k, w, st = ctypes.c_int32(), ctypes.c_int32(), ctypes.c_uint32(), ctypes.c_size_t()
    _check(lib().ogc_mlp_cluster_layout(plan, ctypes.byref(m), ctypes.byref(k), ctypes.byref(w), ctypes.byref(st)),
           "ogc_mlp_cluster_layout")
    return m.value, k.value, w.value, st.value


def ogc_mlp_packed_bytes(plan: int) -> int:
    v = ctypes.c_size_t()
    _check(lib().ogc_mlp_packed_bytes(plan, ctypes.byref(v)), "ogc_mlp_packed_bytes")
    return v.value


def ogc_mlp_workspace_bytes(plan: int) -> int:
    v = ctypes.c_size_t()
    _check(lib().ogc_mlp_workspace_bytes(plan, ctypes.byref(v)), "ogc_mlp_workspace_bytes")
    return v.value


def ogc_mlp_blocked_bytes(plan: int, which: int) -> int:
    v = ctypes.c_size_t()
    _check(lib().ogc_mlp_blocked_bytes(plan, int(which), ctypes.byref(v)), "ogc_mlp_blocked_bytes")
    return v.value


def ogc_mlp_chosen_mode(plan: int) -> int:
    v = ctypes.c_int32()
    _check(lib().ogc_mlp_chosen_mode(plan, ctypes.byref(v)), "ogc_mlp_chosen_mode")
    return v.value


def ogc_mlp_buffer_assignment(plan: int, layer: int):
    s, o = ctypes.c_int32(), ctypes.c_size_t()
    _check(lib().ogc_mlp_buffer_assignment(plan, int(layer), ctypes.byref(s), ctypes.byref(o)), "ogc_mlp_buffer_assignment")
    return s.value, o.value


def _ptr_array(ptrs: Optional[Sequence[Optional[int]]], n: int):
    if ptrs is None:
        return None
    arr = (ctypes.c_void_p * max(n, 1))()
    for i in range(n):
        arr[i] = ptrs[i] if ptrs[i] else None
    return arr


def ogc_mlp_prepack_weights(plan: int, w_ptrs, bias_ptrs, w_scale_ptrs, packed_ptr: int, stream: int = 0) -> None:
    n = len(w_ptrs)
    _check(lib().ogc_mlp_prepack_weights(plan, _ptr_array(w_ptrs, n), _ptr_array(bias_ptrs, n), _ptr_array(w_scale_ptrs, n),
                                         packed_ptr, stream), "ogc_mlp_prepack_weights")


def ogc_mlp_run(plan: int, x_ptr: int, y_ptr: int, packed_ptr: int, workspace_ptr: int, stream: int = 0) -> None:
    _check(lib().ogc_mlp_run(plan, x_ptr, y_ptr, packed_ptr, workspace_ptr or None, stream), "ogc_mlp_run")


def ogc_mlp_run_static(plan: int, x_ptr: int, y_ptr: int, packed_ptr: int, stream: int = 0) -> None:
    _check(lib().ogc_mlp_run_static(plan, x_ptr, y_ptr, packed_ptr, stream), "ogc_mlp_run_static")


def ogc_quantize_e4m3(x: int, out: int, n: int, scale: float, stream: int = 0) -> None:
    _check(lib().ogc_quantize_e4m3(x, out, n, scale, stream), "ogc_quantize_e4m3")


def ogc_dequantize_e4m3(x: int, out: int, n: int, scale: float, stream: int = 0) -> None:
    _check(lib().ogc_dequantize_e4m3(x, out, n, scale, stream), "ogc_dequantize_e4m3")


def ogc_mlp_static_workspace_limit() -> int:
    return int(lib().ogc_mlp_static_workspace_limit())


def ogc_mlp_num_launches(plan: int) -> int:
    v = ctypes.c_int32()
    _check(lib().ogc_mlp_num_launches(plan, ctypes.byref(v)), "ogc_mlp_num_launches")
    return v.value


def ogc_mlp_run_clocked(plan: int, x_ptr: int, y_ptr: int, packed_ptr: int, workspace_ptr: int, clocks_ptr: int, stream: int = 0) -> None:
    _check(lib().ogc_mlp_run_clocked(plan, x_ptr, y_ptr, packed_ptr, workspace_ptr or None, stream, clocks_ptr), "ogc_mlp_run_clocked")


def ogc_mlp_clock_words_per_launch() -> int:
    return int(lib().ogc_mlp_clock_words_per_launch())


def ogc_mlp_run_profiled(plan: int, x_ptr: int, y_ptr: int, packed_ptr: int, workspace_ptr: int, stream: int = 0):
    """Returns the list of per-launch durations in milliseconds."""
    n = ogc_mlp_num_launches(plan)
    ms = (ctypes.c_float * n)()
    _check(lib().ogc_mlp_run_profiled(plan, x_ptr, y_ptr, packed_ptr, workspace_ptr or None, stream, ms), "ogc_mlp_run_profiled")
    return [float(v) for v in ms]


def ogc_mlp_estimated_us(plan: int, layer: int) -> float:
    v = ctypes.c_float()
    _check(lib().ogc_mlp_estimated_us(plan, int(layer), ctypes.byref(v)), "ogc_mlp_estimated_us")
    return v.value


def ogc_mlp_mode_estimates(plan: int):
    """(per layer, fused, cooperative) estimates of the whole chain in microseconds; -1 where not admissible."""
    v = (ctypes.c_float * 3)()
    _check(lib().ogc_mlp_mode_estimates(plan, v), "ogc_mlp_mode_estimates")
    return tuple(float(x) for x in v)


def ogc_mlp_destroy(plan: int) -> None:
    lib().ogc_mlp_destroy(plan)


def ogc_mlp_kernel_name(plan: int, layer: int) -> str:
    r = lib().ogc_mlp_kernel_name(plan, int(layer))
    return r.decode() if r else ""


def mha_desc(dtype: int, batch: int, heads: int, seq: int, head_dim: int, scale: float, softmax: int = OGC_SOFTMAX_STABLE,
             q_stride=None, k_stride=None, v_stride=None, o_stride=None, query_groups: int = 0) -> ogc_mha_desc:
    """Strides default to the [batch, seq, heads*head_dim] layout."""
    plain = (seq * heads * head_dim, head_dim, heads * head_dim)
    arrs = [(ctypes.c_int64 * 3)(*[int(v) for v in (st if st is not None else plain)])
            for st in (q_stride, k_stride, v_stride, o_stride)]
    return ogc_mha_desc(int(dtype), int(batch), int(heads), int(seq), int(head_dim), int(softmax), float(scale), *arrs,
                        int(query_groups))


def ogc_mha_validate(desc: ogc_mha_desc) -> int:
    return int(lib().ogc_mha_validate(ctypes.byref(desc)))


def ogc_mha_run(desc: ogc_mha_desc, q_ptr: int, k_ptr: int, v_ptr: int, mask_ptr: int, o_ptr: int, stream: int = 0) -> None:
    _check(lib().ogc_mha_run(ctypes.byref(desc), q_ptr or None, k_ptr or None, v_ptr or None, mask_ptr or None, o_ptr or None,
                             stream), "ogc_mha_run")


def ogc_mha_i8_validate(desc: ogc_mha_desc, quant: ogc_mha_quant) -> int:
    return int(lib().ogc_mha_i8_validate(ctypes.byref(desc), ctypes.byref(quant)))


def ogc_mha_run_i8(desc: ogc_mha_desc, quant: ogc_mha_quant, q_ptr: int, k_ptr: int, v_ptr: int, mask_ptr: int, o_ptr: int,
                   stream: int = 0) -> None:
    _check(lib().ogc_mha_run_i8(ctypes.byref(desc), ctypes.byref(quant), q_ptr or None, k_ptr or None, v_ptr or None,
                                mask_ptr or None, o_ptr or None, stream), "ogc_mha_run_i8")


def ogc_mha_i8_kernel_name(desc: ogc_mha_desc) -> str:
    r = lib().ogc_mha_i8_kernel_name(ctypes.byref(desc))
    return r.decode() if r else ""


def ogc_mha_kernel_name(desc: ogc_mha_desc, has_mask: bool = True) -> str:
    r = lib().ogc_mha_kernel_name(ctypes.byref(desc), int(bool(has_mask)))
    return r.decode() if r else ""


# ---- convenience wrapper: owns the torch tensors the library needs ---------------------------------
class FusedMLP:
    """plan + packed blob + workspace for one static MLP chain on the current CUDA/HIP device."""

    def __init__(self, dtype: str, m: int, layers: Sequence, ld_x: Optional[int] = None, ld_y: Optional[int] = None,
                 residual: bool = False, mode: int = OGC_MODE_AUTO, x_layout: int = OGC_LAYOUT_PLAIN,
                 y_layout: int = OGC_LAYOUT_PLAIN, overrides: Optional[dict] = None):
        import torch

        self.torch = torch
        self.dtype = dtype
        self.m = m
        self.layer_dicts = []
        for ly in layers:
            d = ly if isinstance(ly, dict) else dict(
                k=ly.k, n=ly.n, has_bias=int(ly.has_bias), act=ly.act, in_scale=ly.in_scale, in_zp=ly.in_zp,
                out_scale=ly.out_scale, out_zp=ly.out_zp, out=OGC_OUT_F32 if ly.out_f32 else OGC_OUT_SAME)
            self.layer_dicts.append(d)
        self.k0 = self.layer_dicts[0]["k"]
        self.n_last = self.layer_dicts[-1]["n"]
        self.ld_x = ld_x or self.k0
        self.ld_y = ld_y or self.n_last
        self.out_f32 = self.layer_dicts[-1].get("out", 0) == OGC_OUT_F32
        if overrides:
            self.plan = ogc_mlp_plan_with_overrides(DTYPES[dtype], m, self.layer_dicts, self.ld_x, self.ld_y, int(residual), mode,
                                                    x_layout, y_layout, overrides)
        else:
            self.plan = ogc_mlp_plan(DTYPES[dtype], m, self.layer_dicts, self.ld_x, self.ld_y, int(residual), mode, x_layout, y_layout)
        self.mode = ogc_mlp_chosen_mode(self.plan)
        self.packed_bytes = ogc_mlp_packed_bytes(self.plan)
        self.workspace_bytes = ogc_mlp_workspace_bytes(self.plan)
        self.packed = None
        self.workspace = None

    def close(self):
        if getattr(self, "plan", None):
            ogc_mlp_destroy(self.plan)
            self.plan = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _stream(self) -> int:
        return int(self.torch.cuda.current_stream().cuda_stream)

    def prepack(self, w: List, bias: Optional[List] = None, w_scale: Optional[List] = None) -> None:
        """w / bias / w_scale: lists of device tensors (bias and w_scale entries may be None)."""
        torch = self.torch
        dev = w[0].device
        self.packed = torch.empty(max(self.packed_bytes, 256), dtype=torch.uint8, device=dev)
        self.workspace = torch.empty(max(self.workspace_bytes, 256), dtype=torch.uint8, device=dev)
        wp = [t.data_ptr() for t in w]
        bp = None if bias is None else [None if t is None else t.data_ptr() for t in bias]
        sp = None if w_scale is None else [None if t is None else t.data_ptr() for t in w_scale]
        ogc_mlp_prepack_weights(self.plan, wp, bp, sp, self.packed.data_ptr(), self._stream())

    def run(self, x, y) -> None:
        ogc_mlp_run(self.plan, x.data_ptr(), y.data_ptr(), self.packed.data_ptr(),
                    self.workspace.data_ptr() if self.workspace_bytes else 0, self._stream())

    def check(self) -> int:
        """OGC_OK, or OGC_ERR_TIMEOUT if a barrier wait of the cooperative mode gave up since the last check."""
        return ogc_mlp_check(self.plan, self.packed.data_ptr(), self._stream())

    def run_clocked(self, x, y, clocks) -> None:
        ogc_mlp_run_clocked(self.plan, x.data_ptr(), y.data_ptr(), self.packed.data_ptr(),
                            self.workspace.data_ptr() if self.workspace_bytes else 0, clocks.data_ptr(), self._stream())

    def run_profiled(self, x, y):
        return ogc_mlp_run_profiled(self.plan, x.data_ptr(), y.data_ptr(), self.packed.data_ptr(),
                                    self.workspace.data_ptr() if self.workspace_bytes else 0, self._stream())
