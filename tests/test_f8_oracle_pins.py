"""Pins for the oracle's 8-bit-float (E4M3) layer: the encoding against hand-listed format facts and an independent
library implementation (torch's float8_e4m3fn on the CPU), the layer against a hand-worked case, exact rational
brute force, a library matmul and invariants.  CPU only."""
import math
import os
from fractions import Fraction

import numpy as np
import pytest
import torch

from paper_2301_01333_amd import synth

from test_oracle_pins import F, rne_f32

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "f8_hand_cases.txt")
RELU, NONE, GELU, SIGM = synth.ACT_RELU, synth.ACT_NONE, synth.ACT_GELU_TANH, synth.ACT_SIGMOID


def _golden():
    out = {"CODE": [], "ENC": []}
    for line in open(GOLDEN):
        line = line.split("#")[0].split()
        if not line:
            continue
        if line[0] in ("CODE", "ENC"):
            out[line[0]].append(line[1:])
        else:
            out[line[0]] = line[1:]
    return out


def _codes(tokens):
    return np.array([int(t, 16) for t in tokens], dtype=np.uint8)


def torch_decode(codes: np.ndarray) -> np.ndarray:
    return torch.from_numpy(np.ascontiguousarray(codes)).view(torch.float8_e4m3fn).to(torch.float64).numpy()


# ---------------------------------------------------------------------------------------------- the encoding
def test_decode_hand_listed_codes(oracle_mod):
    g = _golden()
    assert len(g["CODE"]) >= 15
    for code, value in g["CODE"]:
        got = oracle_mod.oracle.e4m3_to_f32(int(code, 16))
        assert got == float(value) and math.copysign(1.0, got) == math.copysign(1.0, float(value) if float(value) else 1.0), (code, got)
    assert math.isnan(oracle_mod.oracle.e4m3_to_f32(0x7F)) and math.isnan(oracle_mod.oracle.e4m3_to_f32(0xFF))
    assert math.copysign(1.0, oracle_mod.oracle.e4m3_to_f32(0x80)) == -1.0


def test_decode_all_codes_against_library(oracle_mod):
    codes = np.arange(256, dtype=np.uint8)
    lib = torch_decode(codes)
    got = np.array([oracle_mod.oracle.e4m3_to_f32(int(c)) for c in codes], dtype=np.float64)
    assert np.array_equal(np.isnan(got), np.isnan(lib)) and np.isnan(got).sum() == 2
    ok = ~np.isnan(lib)
    assert np.array_equal(got[ok], lib[ok]) and np.array_equal(np.signbit(got[ok]), np.signbit(lib[ok]))
    # the finite values are strictly increasing in the code within a sign, and symmetric
    assert (np.diff(got[:0x7F]) > 0).all() and np.array_equal(got[0x80:0xFF], -got[:0x7F])


def test_encode_hand_listed_values(oracle_mod):
    g = _golden()
    assert len(g["ENC"]) >= 15
    for value, code in g["ENC"]:
        assert oracle_mod.oracle.f32_to_e4m3(float(value)) == int(code, 16), (value, code)


def test_encode_against_library_below_saturation(oracle_mod):
    """torch rounds the same way (nearest, ties to even) but gives NaN above the range; below 464 the two must agree.
    The sample holds every representable value, every midpoint, their fp32 neighbours, and random values."""
    vals = torch_decode(np.arange(0x7F, dtype=np.uint8))
    mids = (vals[:-1] + vals[1:]) / 2
    pts = np.concatenate([vals, mids]).astype(np.float32)
    pts = np.concatenate([pts, np.nextafter(pts, np.float32(np.inf)), np.nextafter(pts, np.float32(-np.inf))])
    rng = np.random.default_rng(8)
    rnd = np.concatenate([rng.uniform(0, 464, 20000), np.exp(rng.uniform(math.log(2.0 ** -12), math.log(464.0), 20000))]).astype(np.float32)
    a = np.concatenate([pts, rnd])
    a = a[(a >= 0) & (a < 464.0)]
    a = np.concatenate([a, -a])
    lib = torch.from_numpy(a).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    got = np.array([oracle_mod.oracle.f32_to_e4m3(float(v)) for v in a], dtype=np.uint8)
    assert np.array_equal(got, lib), (a[got != lib][:5], got[got != lib][:5], lib[got != lib][:5])


def test_encode_decode_round_trip_and_monotone(oracle_mod):
    for c in list(range(0x7F)) + list(range(0x80, 0xFF)):
        assert oracle_mod.oracle.f32_to_e4m3(oracle_mod.oracle.e4m3_to_f32(c)) == c
    xs = np.linspace(-500, 500, 4001).astype(np.float32)
    dec = [oracle_mod.oracle.e4m3_to_f32(oracle_mod.oracle.f32_to_e4m3(float(x))) for x in xs]
    assert (np.diff(dec) >= 0).all() and max(dec) == 448.0 and min(dec) == -448.0


# ---------------------------------------------------------------------------------------------- the layer
def nearest_code_brute_force(t: Fraction, table) -> int:
    """Nearest finite E4M3 value by exhaustive search over the non-negative codes; a tie takes the even code (codes
    alternate in mantissa parity, so the even code is the even mantissa); beyond 448 saturates."""
    sign = 0x80 if t < 0 else 0
    a = -t if t < 0 else t
    best, best_d = None, None
    for c in range(0x7F):
        d = abs(table[c] - a)
        if best is None or d < best_d or (d == best_d and c % 2 == 0):
            best, best_d = c, d
    return sign | best


def exact_f8_output(xrow, wcol, table, a_s, b_s, bias, c_s, act, out_f32):
    val = lambda c: (-table[c & 0x7F] if c & 0x80 else table[c & 0x7F])
    acc = sum(val(int(x)) * val(int(w)) for x, w in zip(xrow, wcol))
    f = rne_f32(acc)
    s = rne_f32(F(a_s) * F(b_s))
    y = rne_f32(f * s + F(bias)) if bias is not None else rne_f32(f * s)
    if act == RELU and y < 0:
        y = Fraction(0)
    if out_f32:
        return y
    inv = rne_f32(1 / F(c_s))
    return nearest_code_brute_force(rne_f32(y * inv), table)


def test_layer_hand_case_and_chain(oracle_mod):
    g = _golden()
    x = _codes(g["LAYER_X"])[None, :]
    w = np.stack([_codes(g["LAYER_W0"]), _codes(g["LAYER_W1"])], axis=1)
    a_s, b0, b1, c_s = [float(v) for v in g["LAYER_SCALES"]]
    ws = np.array([b0, b1], dtype=np.float32)
    bias = np.array([float(v) for v in g["LAYER_BIAS"]], dtype=np.float32)
    lf = oracle_mod.oracle.layer_f8
    for exact in (True, False):
        assert lf(x, w, ws, bias, a_s, NONE, out_f32=True, accum_double=exact).tolist() == [[float(v) for v in g["LAYER_Y_F32"]]]
        assert lf(x, w, ws, bias, a_s, NONE, c_s, accum_double=exact).tolist() == [_codes(g["LAYER_Y_NONE"]).tolist()]
        assert lf(x, w, ws, bias, a_s, RELU, c_s, accum_double=exact).tolist() == [_codes(g["LAYER_Y_RELU"]).tolist()]
    # the chain: the first layer's codes and its output scale are the second layer's input
    w2 = np.ascontiguousarray(_codes(g["CHAIN_W"]).reshape(2, 1))
    layers = [synth.Layer(3, 2, True, NONE, in_scale=a_s, out_scale=c_s), synth.Layer(2, 1, False, NONE, in_scale=c_s, out_f32=True)]
    wl = synth.Workload("hand", "f8", 1, layers, False, x, [w, w2], [bias, None], [ws, np.ones(1, np.float32)], 0)
    outs = oracle_mod.mlp(wl, keep=True)
    assert outs[0].tolist() == [_codes(g["LAYER_Y_NONE"]).tolist()] and outs[1].tolist() == [[float(g["CHAIN_Y"][0])]]


def test_requantize_multiplies_by_the_reciprocal(oracle_mod):
    g = _golden()
    bias, c_s, code = float(g["RECIP"][0]), float(g["RECIP"][1]), int(g["RECIP"][2], 16)
    x = np.array([[0x38]], dtype=np.uint8)
    w = np.zeros((1, 1), dtype=np.uint8)
    got = oracle_mod.oracle.layer_f8(x, w, np.ones(1, np.float32), np.array([bias], np.float32), 1.0, NONE, c_s)
    assert got.tolist() == [[code]]


@pytest.mark.parametrize("seed", range(6))
def test_layer_brute_force_tiny(oracle_mod, seed):
    rng = np.random.default_rng(900 + seed)
    table = [Fraction(float(v)) for v in torch_decode(np.arange(0x7F, dtype=np.uint8))]
    m, k, n = 3, 5 + seed, 4
    finite = np.array([c for c in range(256) if c & 0x7F != 0x7F], dtype=np.uint8)
    x = rng.choice(finite[(finite & 0x7F) < 0x50], size=(m, k))   # |x| < 8
    w = rng.choice(finite[(finite & 0x7F) < 0x48], size=(k, n))   # |w| < 4
    ws = rng.uniform(0.01, 0.5, n).astype(np.float32)
    bias = rng.uniform(-1, 1, n).astype(np.float32) if seed % 2 == 0 else None
    a_s = float(np.float32(rng.uniform(0.05, 0.3)))
    c_s = float(np.float32(rng.uniform(0.0002, 0.002) if seed % 2 else rng.uniform(0.002, 0.05)))   # odd seeds: many outputs saturate
    act = RELU if seed % 3 == 0 else NONE
    got8 = oracle_mod.oracle.layer_f8(x, w, ws, bias, a_s, act, c_s)
    got32 = oracle_mod.oracle.layer_f8(x, w, ws, bias, a_s, act, out_f32=True)
    for i in range(m):
        for j in range(n):
            b = None if bias is None else bias[j]
            assert got8[i, j] == exact_f8_output(x[i], w[:, j], table, a_s, ws[j], b, c_s, act, False), (i, j)
            assert Fraction(float(got32[i, j])) == exact_f8_output(x[i], w[:, j], table, a_s, ws[j], b, c_s, act, True), (i, j)
    if seed % 2:
        sat = (got8 & 0x7F) == 0x7E
        print("saturated outputs:", int(sat.sum()), "of", sat.size)
        assert seed != 1 or (sat.any() and not sat.all()), "the case was meant to include saturated outputs"


def test_layer_matches_library_matmul(oracle_mod):
    """With fp32 output and no activation the layer is a plain matmul of the decoded operands (library decode and
    library matmul in fp64), scaled per channel."""
    rng = np.random.default_rng(77)
    m, k, n = 17, 300, 23
    x = rng.integers(0, 256, (m, k), dtype=np.uint8)
    w = rng.integers(0, 256, (k, n), dtype=np.uint8)
    x[(x & 0x7F) == 0x7F] = 0x38
    w[(w & 0x7F) == 0x7F] = 0xB8
    ws = rng.uniform(0.01, 0.02, n).astype(np.float32)
    bias = rng.uniform(-1, 1, n).astype(np.float32)
    a_s = 0.03125
    ref = torch_decode(x) @ torch_decode(w) * (np.float64(np.float32(a_s)) * ws.astype(np.float64)) + bias
    for exact in (True, False):
        got = oracle_mod.oracle.layer_f8(x, w, ws, bias, a_s, NONE, out_f32=True, accum_double=exact)
        scale = np.abs(torch_decode(x)) @ np.abs(torch_decode(w)) * (a_s * ws.astype(np.float64)) + 1.0
        assert (np.abs(got - ref) <= (3e-7 if exact else k * 6e-8) * scale).all()
    # operands transposed by mistake would not survive this: the matrix is far from symmetric
    assert not np.allclose(ref, (torch_decode(x) @ torch_decode(w[::-1])) * (a_s * ws) + bias)


def test_layer_invariants(oracle_mod):
    rng = np.random.default_rng(5)
    m, k, n = 9, 64, 12
    mag = rng.integers(0x10, 0x58, (m, k), dtype=np.uint8)            # normal values with headroom above and below
    x = (mag | (rng.integers(0, 2, (m, k), dtype=np.uint8) << 7)).astype(np.uint8)
    w = (rng.integers(0x10, 0x58, (k, n), dtype=np.uint8) | (rng.integers(0, 2, (k, n), dtype=np.uint8) << 7)).astype(np.uint8)
    ws = rng.uniform(0.01, 0.02, n).astype(np.float32)
    bias = rng.uniform(-1, 1, n).astype(np.float32)
    lf = oracle_mod.oracle.layer_f8
    base = lf(x, w, ws, bias, 0.25, RELU, 0.125)
    assert len(np.unique(base)) > 10
    # doubling every x (exponent field + 1) and halving the input scale changes nothing
    assert np.array_equal(lf((x + 8).astype(np.uint8), w, ws, bias, 0.125, RELU, 0.125), base)
    # the exact sum does not depend on the order along k
    p = rng.permutation(k)
    assert np.array_equal(lf(np.ascontiguousarray(x[:, p]), w[p], ws, bias, 0.25, RELU, 0.125), base)
    # flipping the signs of both operands changes nothing; of one operand and of the bias negates the result
    assert np.array_equal(lf(x ^ 0x80, w ^ 0x80, ws, bias, 0.25, RELU, 0.125), base)
    plain = lf(x, w, ws, bias, 0.25, NONE, 0.125)
    neg = lf(x ^ 0x80, w, ws, -bias, 0.25, NONE, 0.125)
    nz = (plain & 0x7F) != 0
    assert np.array_equal(neg[nz], plain[nz] ^ 0x80) and ((neg[~nz] & 0x7F) == 0).all()
    # zero weights: the output is the encoded activation of the bias alone
    z = lf(x, np.zeros_like(w), ws, bias, 0.25, RELU, 0.125)
    want = [oracle_mod.oracle.f32_to_e4m3(float(np.float32(max(b, 0.0)) * np.float32(8.0))) for b in bias]
    assert (z == np.array(want, dtype=np.uint8)[None, :]).all()
    # a power-of-two output scale shifts the exponent field only (away from saturation and subnormals)
    a, b2 = lf(x, w, ws, bias, 0.25, NONE, 0.125), lf(x, w, ws, bias, 0.25, NONE, 0.0625)
    mid = ((a & 0x7F) >= 0x10) & ((a & 0x7F) < 0x70)
    assert mid.sum() > 20 and np.array_equal(b2[mid], a[mid] + 8)


def test_fp32_running_sum_stays_within_its_bound_of_the_exact_sum(oracle_mod):
    rng = np.random.default_rng(6)
    m, k, n = 8, 2048, 8
    x = rng.integers(0, 0x70, (m, k), dtype=np.uint8) | (rng.integers(0, 2, (m, k), dtype=np.uint8) << 7).astype(np.uint8)
    w = rng.integers(0, 0x70, (k, n), dtype=np.uint8) | (rng.integers(0, 2, (k, n), dtype=np.uint8) << 7).astype(np.uint8)
    ws = np.ones(n, np.float32)
    e = oracle_mod.oracle.layer_f8(x, w, ws, None, 1.0, NONE, out_f32=True, accum_double=True)
    s = oracle_mod.oracle.layer_f8(x, w, ws, None, 1.0, NONE, out_f32=True, accum_double=False)
    bound = k * 2.0 ** -24 * (np.abs(torch_decode(x)) @ np.abs(torch_decode(w)))
    assert (np.abs(e.astype(np.float64) - s) <= bound).all() and not np.array_equal(e, s)
