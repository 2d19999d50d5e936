"""Glue between a synthetic workload (numpy arrays) and the GPU library: uploads the arrays as device
tensors, builds the plan, prepacks, runs, downloads.  Marshalling only; no arithmetic of the method."""
from __future__ import annotations

from typing import Optional

import numpy as np

from . import binding


def _to_device(torch, arr: np.ndarray):
    a = np.ascontiguousarray(arr)
    return torch.from_numpy(a.view(np.uint8).reshape(-1).copy()).cuda()


class DeviceMLP:
    """A workload resident on the GPU: plan, packed weights, input and output buffers."""

    def __init__(self, wl, mode: int = binding.OGC_MODE_AUTO, ld_y: Optional[int] = None, x_byte_offset: int = 0,
                 overrides: Optional[dict] = None):
        import torch

        self.torch = torch
        self.wl = wl
        xb = wl.x.base if wl.x.base is not None else wl.x
        if xb.ndim != 2 or xb.shape[0] != wl.x.shape[0]:
            xb = np.ascontiguousarray(wl.x)
        self.ld_x = xb.shape[1]
        last = wl.layers[-1]
        self.out_np_dtype = (np.float32 if (wl.dtype in ("i8", "f8") and last.out_f32)
                             else {"f32": np.float32, "bf16": np.uint16, "i8": np.uint8, "f8": np.uint8}[wl.dtype])
        self.ld_y = ld_y or last.n
        self.mlp = binding.FusedMLP(wl.dtype, wl.m, wl.layers, self.ld_x, self.ld_y, wl.residual, mode, overrides=overrides)
        self.w = [_to_device(torch, w) for w in wl.w]
        self.bias = [None if b is None else _to_device(torch, b) for b in wl.bias]
        self.w_scale = None if wl.dtype not in ("i8", "f8") else [_to_device(torch, s) for s in wl.w_scale]
        self.mlp.prepack(self.w, self.bias, self.w_scale)
        xbytes = np.ascontiguousarray(xb).view(np.uint8).reshape(-1)
        if x_byte_offset:
            xbytes = np.concatenate([np.zeros(x_byte_offset, np.uint8), xbytes])
        self.x_store = torch.from_numpy(xbytes.copy()).cuda()
        self.x = self.x_store[x_byte_offset:]
        ybytes = wl.m * self.ld_y * np.dtype(self.out_np_dtype).itemsize
        self.y = torch.full((ybytes,), 0xCD, dtype=torch.uint8, device="cuda")

    def run(self) -> None:
        self.mlp.run(self.x, self.y)

    def run_profiled(self):
        return self.mlp.run_profiled(self.x, self.y)

    def run_clocked(self):
        """One run with the stream kernel's workgroups recording their clocks; returns an int64 array
        [launch][workgroup][wall start, cycles start, wall end, cycles end] (zeros where nothing was recorded)."""
        words = binding.ogc_mlp_clock_words_per_launch()
        n = binding.ogc_mlp_num_launches(self.mlp.plan)
        buf = self.torch.zeros((n * words,), dtype=self.torch.int64, device="cuda")
        self.mlp.run_clocked(self.x, self.y, buf)
        self.torch.cuda.synchronize()
        return buf.cpu().numpy().reshape(n, words // 4, 4)

    def result(self) -> np.ndarray:
        self.torch.cuda.synchronize()
        full = self.y.cpu().numpy().view(self.out_np_dtype).reshape(self.wl.m, self.ld_y)
        return full

    def close(self):
        self.mlp.close()


class DeviceMHA:
    """An attention workload resident on the GPU (q, k, v, mask uploaded; o allocated and poisoned)."""

    def __init__(self, wl, softmax: int = binding.OGC_SOFTMAX_STABLE, use_mask: bool = True, query_groups: int = 0):
        import torch

        self.torch = torch
        self.wl = wl
        self.np_dtype = {"f32": np.float32, "bf16": np.uint16, "i8": np.int8}[wl.dtype]
        self.q, self.k, self.v = (_to_device(torch, t) for t in (wl.q, wl.k, wl.v))
        self.mask = _to_device(torch, wl.mask) if (use_mask and wl.mask is not None) else None
        self.o = torch.full((wl.q.nbytes,), 0xCD, dtype=torch.uint8, device="cuda")
        self.desc = binding.mha_desc(binding.DTYPES[wl.dtype], wl.batch, wl.heads, wl.seq, wl.head_dim, wl.scale, softmax,
                                     query_groups=query_groups)
        self.quant = binding.ogc_mha_quant(*[float(x) for x in wl.quant]) if wl.dtype == "i8" else None

    def run(self) -> None:
        stream = int(self.torch.cuda.current_stream().cuda_stream)
        if self.quant is not None:
            binding.ogc_mha_run_i8(self.desc, self.quant, self.q.data_ptr(), self.k.data_ptr(), self.v.data_ptr(),
                                   self.mask.data_ptr() if self.mask is not None else 0, self.o.data_ptr(), stream)
            return
        binding.ogc_mha_run(self.desc, self.q.data_ptr(), self.k.data_ptr(), self.v.data_ptr(),
                            self.mask.data_ptr() if self.mask is not None else 0, self.o.data_ptr(),
                            int(self.torch.cuda.current_stream().cuda_stream))

    def result(self) -> np.ndarray:
        """o as [batch, seq, heads*head_dim] in the workload's storage dtype."""
        self.torch.cuda.synchronize()
        return self.o.cpu().numpy().view(self.np_dtype).reshape(self.wl.batch, self.wl.seq, self.wl.hidden)
