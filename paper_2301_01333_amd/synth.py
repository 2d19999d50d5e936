"""Seeded synthetic workloads for the fused-MLP path.

This module only draws inputs; it holds none of the method's arithmetic (no matmul, no
quantize/dequantize of activations) and imports neither the CPU oracle nor the GPU library, so
both sides can be fed the very same arrays.

The paper's MLP workloads take their weight shapes from MLPerf DLRM (Section VII, Table I:
13x512x256x128 and 479x1024x1024x512x256x1, batch 32..512, FP32 and Int8 with u8 asymmetric
activations and s8 symmetric per-channel weights).  Neither model weights nor data are used
here: the tensors below are synthetic stand-ins with those shapes and that quantization scheme.

bf16 tensors are carried as uint16 bit patterns.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import List, Optional, Sequence

import numpy as np

ACT_NONE, ACT_RELU, ACT_GELU_TANH, ACT_SIGMOID = 0, 1, 2, 3
BASE_SEED = 23010133 * 10


def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """fp32 -> bf16 bit pattern, round to nearest even (finite inputs)."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32).astype(np.uint64)
    lsb = (u >> 16) & 1
    return ((u + 0x7FFF + lsb) >> 16).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32)


@dataclass
class Layer:
    k: int
    n: int
    has_bias: bool = True
    act: int = ACT_RELU
    in_scale: float = 0.0   # int8: a_s of this layer's input
    in_zp: int = 0          # int8: a_z
    out_scale: float = 0.0  # int8: c_s of this layer's output (unused if out_f32)
    out_zp: int = 0         # int8: c_z
    out_f32: bool = False   # int8: emit fp32 instead of requantizing (last layer only)


@dataclass
class Workload:
    name: str
    dtype: str              # "f32" | "bf16" | "i8" | "f8" (E4M3 codes in uint8 arrays)
    m: int
    layers: List[Layer]
    residual: bool
    x: np.ndarray
    w: List[np.ndarray]     # each [K, N] row-major
    bias: List[Optional[np.ndarray]]
    w_scale: List[Optional[np.ndarray]]
    seed: int = 0

    @property
    def dims(self) -> List[int]:
        return [self.layers[0].k] + [l.n for l in self.layers]

    @property
    def ops(self) -> int:
        """2 * M * sum_l K_l*N_l: useful multiply-adds only, padding never counted."""
        return 2 * self.m * sum(l.k * l.n for l in self.layers)

    @property
    def elt(self) -> int:
        return {"f32": 4, "bf16": 2, "i8": 1, "f8": 1}[self.dtype]

    @property
    def algorithmic_bytes(self) -> int:
        """Weights + per-channel parameters + input once + final output once.  Intermediate
        activations count zero: keeping them on chip is the method."""
        e = self.elt
        wbytes = sum(l.k * l.n for l in self.layers) * e
        if self.dtype == "i8":
            params = sum(l.n for l in self.layers) * 12  # scale, bias, compensation
        elif self.dtype == "f8":
            params = sum(l.n for l in self.layers) * 8   # scale, bias
        else:
            params = sum(l.n for l in self.layers if l.has_bias) * 4
        last = self.layers[-1]
        out_e = 4 if (self.dtype in ("i8", "f8") and last.out_f32) else e
        return wbytes + params + self.m * self.layers[0].k * e + self.m * last.n * out_e


def int8_output_scales(dims: Sequence[int], a_s: float, a_z: int, c_z: int, ws_lo: float, ws_hi: float) -> List[float]:
    """Closed-form static output scales c_s(l) for a ReLU chain, from the input distributions
    alone (no forward pass): the pre-activation of layer l is roughly N(0, sigma_l^2) with
    sigma_l^2 = K_l * E[x^2] * E[w^2]; post-ReLU inputs of the next layer have E[x^2] =
    sigma_l^2 / 2; the scale maps 3 sigma onto the top of the u8 range above the zero point."""
    e_ws2 = (ws_lo * ws_lo + ws_lo * ws_hi + ws_hi * ws_hi) / 3.0
    e_wq2 = 127.0 * 128.0 / 3.0                       # uniform integers in [-127, 127]
    e_w2 = e_ws2 * e_wq2
    e_x2 = a_s * a_s * ((256.0 * 256.0 - 1.0) / 12.0 + (127.5 - a_z) ** 2)  # uniform u8 about a_z
    scales = []
    for l in range(len(dims) - 1):
        var = dims[l] * e_x2 * e_w2
        sigma = math.sqrt(var)
        scales.append(float(np.float32(3.0 * sigma / max(255 - c_z, 1))))
        e_x2 = var / 2.0
    return scales


# The non-negative finite E4M3 values in code order (OCP 8-bit float: 4 exponent bits with bias 7, 3 mantissa bits,
# subnormals at exponent field 0, largest finite value 448 = code 0x7E).  Used only to draw input codes.
E4M3_VALUES = np.array([(m / 8.0) * 2.0 ** -6 if e == 0 else (1.0 + m / 8.0) * 2.0 ** (e - 7)
                        for e in range(16) for m in range(8)][:0x7F], dtype=np.float64)


def e4m3_nearest_codes(a: np.ndarray) -> np.ndarray:
    """Input drawing helper: the E4M3 code nearest to each value (values beyond +-448 take +-448; which neighbour an
    exact midpoint takes is immaterial here, any code is a valid input)."""
    a = np.asarray(a, dtype=np.float64)
    mag = np.minimum(np.abs(a), 448.0)
    hi = np.clip(np.searchsorted(E4M3_VALUES, mag), 1, len(E4M3_VALUES) - 1)
    lo = hi - 1
    code = np.where(mag - E4M3_VALUES[lo] <= E4M3_VALUES[hi] - mag, lo, hi).astype(np.uint8)
    return (code | (np.signbit(a).astype(np.uint8) << 7)).astype(np.uint8)


def f8_output_scales(dims: Sequence[int], acts: Sequence[int], x_var: float) -> List[float]:
    """Closed-form static output scales for an E4M3 chain with weights of variance 1/K: the pre-activation of
    layer l has variance E[x^2]; the scale maps 4 sigma onto the largest finite value 448.  After ReLU E[x^2]
    halves; any other activation is taken to keep it."""
    scales, e_x2 = [], x_var
    for l in range(len(dims) - 1):
        sigma = math.sqrt(e_x2)
        scales.append(float(np.float32(4.0 * sigma / 448.0)))
        e_x2 = e_x2 / 2.0 if acts[l] == ACT_RELU else e_x2
    return scales


def make_mlp(dtype: str, m: int, dims: Sequence[int], acts: Sequence[int], seed: int, *, has_bias: bool = True,
             residual: bool = False, name: str = "custom", x_scale: Optional[float] = None,
             w_std: Optional[Sequence[float]] = None, a_s: float = 0.05, a_z: int = 128, c_z: int = 128,
             ws_lo: float = 0.005, ws_hi: float = 0.02, last_f32: bool = False, ld_x: Optional[int] = None,
             wq_lo: int = -127) -> Workload:
    """Draw order: x, then per layer (W, bias, w_scale), all from one default_rng(seed) stream."""
    assert len(acts) == len(dims) - 1
    rng = np.random.default_rng(seed)
    nl = len(dims) - 1
    k0 = dims[0]
    ldx = k0 if ld_x is None else ld_x
    assert ldx >= k0
    layers, ws, bs, wss = [], [], [], []
    if dtype == "i8":
        xfull = rng.integers(0, 256, size=(m, ldx), dtype=np.uint8)
    elif dtype == "f8":
        f8_in_scale = float(np.float32(4.0 / 448.0))   # N(0,1) inputs, 4 sigma on the largest code
        xfull = e4m3_nearest_codes(rng.standard_normal((m, ldx)) / f8_in_scale)
        f8_cs = f8_output_scales(dims, acts, 1.0)
    else:
        xf = rng.standard_normal((m, ldx)).astype(np.float32)
        if x_scale is not None:
            xf = (xf * np.float32(x_scale)).astype(np.float32)
        xfull = xf if dtype == "f32" else f32_to_bf16_bits(xf)
    x = xfull[:, :k0]  # a view with row stride ldx when ld_x > k0
    cs = int8_output_scales(dims, a_s, a_z, c_z, ws_lo, ws_hi) if dtype == "i8" else None
    for l in range(nl):
        k, n = dims[l], dims[l + 1]
        if dtype == "i8":
            w = rng.integers(wq_lo, 128, size=(k, n), dtype=np.int8)
        elif dtype == "f8":
            wf = rng.standard_normal((k, n)) / math.sqrt(k)
            f8_ws = (np.abs(wf).max(axis=0) / 448.0).astype(np.float32)   # per output channel: its largest weight on 448
            w = e4m3_nearest_codes(wf / f8_ws.astype(np.float64))
        else:
            std = (w_std[l] if w_std is not None else 1.0 / math.sqrt(k))
            wf = (rng.standard_normal((k, n)) * std).astype(np.float32)
            w = wf if dtype == "f32" else f32_to_bf16_bits(wf)
        b = rng.uniform(-0.1, 0.1, size=(n,)).astype(np.float32) if has_bias else None
        if dtype == "i8":
            wsc = rng.uniform(ws_lo, ws_hi, size=(n,)).astype(np.float32)
            f32_out = bool(last_f32 and l == nl - 1)
            ly = Layer(k, n, has_bias, acts[l], in_scale=(a_s if l == 0 else cs[l - 1]), in_zp=(a_z if l == 0 else c_z),
                       out_scale=(1.0 if f32_out else cs[l]), out_zp=(0 if f32_out else c_z), out_f32=f32_out)
        elif dtype == "f8":
            wsc = f8_ws
            f32_out = bool(last_f32 and l == nl - 1)
            ly = Layer(k, n, has_bias, acts[l], in_scale=(f8_in_scale if l == 0 else f8_cs[l - 1]), in_zp=0,
                       out_scale=(1.0 if f32_out else f8_cs[l]), out_zp=0, out_f32=f32_out)
        else:
            wsc = None
            ly = Layer(k, n, has_bias, acts[l])
        layers.append(ly)
        ws.append(w)
        bs.append(b)
        wss.append(wsc)
    return Workload(name, dtype, m, layers, residual, x, ws, bs, wss, seed)


CONFIG_NAMES = {
    1: "cfg1 fp32 M=32 13-64-32-16 bias+ReLU",
    2: "cfg2 bf16 M=128 13-512-256-128-64 bias+ReLU",
    3: "cfg3 int8 M=256 479-1024-1024-512-256-1 ReLU+requant, fp32 sigmoid out",
    4: "cfg4 bf16 FFN M=4096 1024-4096(GELU tanh)-1024 +bias +residual",
    5: "cfg5 int8 M=32768 4x(1024-1024) ReLU+requant",
}


def make_config(idx: int, m: Optional[int] = None) -> Workload:
    """The five benchmark configurations (1-based).  m overrides the batch size (for reduced
    parity cases and for bounded CPU timing samples); everything else is as stated."""
    seed = BASE_SEED + idx
    if idx == 1:
        return make_mlp("f32", m or 32, [13, 64, 32, 16], [ACT_RELU] * 3, seed, x_scale=1.0 / math.sqrt(13.0),
                        name=CONFIG_NAMES[1])
    if idx == 2:
        return make_mlp("bf16", m or 128, [13, 512, 256, 128, 64], [ACT_RELU] * 4, seed, name=CONFIG_NAMES[2])
    if idx == 3:
        return make_mlp("i8", m or 256, [479, 1024, 1024, 512, 256, 1], [ACT_RELU] * 4 + [ACT_SIGMOID], seed,
                        last_f32=True, name=CONFIG_NAMES[3])
    if idx == 4:
        return make_mlp("bf16", m or 4096, [1024, 4096, 1024], [ACT_GELU_TANH, ACT_NONE], seed, residual=True,
                        w_std=[0.02, 0.02], name=CONFIG_NAMES[4])
    if idx == 5:
        return make_mlp("i8", m or 32768, [1024] * 5, [ACT_RELU] * 4, seed, has_bias=False, name=CONFIG_NAMES[5])
    raise ValueError("config index must be 1..5")


# ---- scaled dot-product attention (Section VII, Table I rows MHA-1..4) ----------------------------------------
# The paper takes sequence length, hidden size and head count from BERT models; no model or data is used here.
# q, k, v are N(0,1) tensors of shape [batch, seq, hidden] (hidden = heads * head_dim, the plain layout a
# projection layer leaves them in); the mask is a BERT-style padding mask: each batch entry has a valid length
# drawn uniformly from [seq/2, seq], keys beyond it get -10000.
MHA_TABLE1 = {  # name: (seq, hidden, heads)
    "MHA-1": (128, 768, 8),
    "MHA-2": (128, 768, 12),
    "MHA-3": (384, 1024, 8),
    "MHA-4": (512, 1024, 16),
}


@dataclass
class MhaWorkload:
    name: str
    dtype: str           # "f32" | "bf16" | "i8"
    batch: int
    seq: int
    heads: int
    head_dim: int
    q: np.ndarray        # [batch, seq, heads*head_dim]; fp32, bf16 bit patterns as uint16, or int8
    k: np.ndarray
    v: np.ndarray
    mask: Optional[np.ndarray]  # [batch, seq] fp32 additive, or None
    scale: float         # fp32 value of 1/sqrt(head_dim)
    seed: int = 0
    quant: Optional[tuple] = None   # "i8": (q_scale, k_scale, v_scale, o_scale), real value = scale * integer

    @property
    def hidden(self) -> int:
        return self.heads * self.head_dim

    @property
    def ops(self) -> int:
        """Two batch matmuls: 2 * (2 * B * H * S * S * d)."""
        return 4 * self.batch * self.heads * self.seq * self.seq * self.head_dim

    @property
    def algorithmic_bytes(self) -> int:
        """q, k, v read once, o written once, the mask once; the S x S scores count zero."""
        e = {"f32": 4, "bf16": 2, "i8": 1}[self.dtype]
        return 4 * self.batch * self.seq * self.hidden * e + (self.batch * self.seq * 4 if self.mask is not None else 0)


def make_mha(dtype: str, batch: int, seq: int, hidden: int, heads: int, seed: int, *, has_mask: bool = True,
             name: str = "custom", amplitude: float = 1.0) -> MhaWorkload:
    """Draw order: q, k, v, then the valid lengths, from one default_rng(seed) stream."""
    assert dtype in ("f32", "bf16", "i8") and hidden % heads == 0
    rng = np.random.default_rng(seed)
    d = hidden // heads
    ts = []
    quant = None
    if dtype == "i8":
        # static symmetric scales mapping 4 standard deviations of the N(0, amplitude^2) tensors onto 127; the
        # integers are drawn directly (round of a scaled normal, clipped)
        # (averages over the keys are much smaller than the values: the output step is a quarter of the input step,
        # which saturates the few outputs of very short sequences and exercises the clamp)
        step = float(np.float32(4.0 * amplitude / 127.0))
        quant = (step, step, step, float(np.float32(amplitude / 127.0)))
    for _ in range(3):
        t = (rng.standard_normal((batch, seq, hidden)) * amplitude).astype(np.float32)
        if dtype == "i8":
            ts.append(np.clip(np.rint(t / np.float32(quant[0])), -127, 127).astype(np.int8))
        else:
            ts.append(t if dtype == "f32" else f32_to_bf16_bits(t))
    mask = None
    if has_mask:
        lens = rng.integers(max(seq // 2, 1), seq + 1, size=(batch,))
        mask = np.where(np.arange(seq)[None, :] < lens[:, None], np.float32(0.0), np.float32(-10000.0)).astype(np.float32)
    return MhaWorkload(name, dtype, batch, seq, heads, d, ts[0], ts[1], ts[2], mask, float(np.float32(1.0 / math.sqrt(d))), seed, quant)


def make_mha_table1(row: str, dtype: str, batch: int) -> MhaWorkload:
    seq, hidden, heads = MHA_TABLE1[row]
    idx = sorted(MHA_TABLE1).index(row)
    return make_mha(dtype, batch, seq, hidden, heads, BASE_SEED + 100 + idx, name="%s %s batch %d" % (row, dtype, batch))
