"""Pins for the Int8 attention oracle (oracle.attention_i8): hand-computed fixtures, a scalar-loop brute force with
exact rational arithmetic after the quantized weights, and invariants, none of which re-types the oracle's code path.
No GPU needed."""
import math
import os
import re
from fractions import Fraction

import numpy as np
import pytest

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "mha_i8_hand_cases.txt")


def _num(tok: str) -> float:
    m = re.fullmatch(r"LN\((\d+)/(\d+)\)(?:/(\d+))?", tok)
    if m:
        return math.log(int(m.group(1)) / int(m.group(2))) / (int(m.group(3)) if m.group(3) else 1)
    return float(tok)


def _cases():
    cases, cur = [], None
    for line in open(GOLDEN):
        line = line.split("#")[0].strip()
        if not line:
            continue
        tag, *vals = line.split()
        if tag == "CASE":
            cur = {"S": int(vals[0]), "d": int(vals[1])}
            cases.append(cur)
        elif tag == "SCALES":
            cur["scales"] = [_num(v) for v in vals]
        elif tag == "M":
            cur["M"] = None if vals == ["-"] else [_num(v) for v in vals]
        else:
            cur[tag] = [int(v) for v in vals]
    return cases


def rne_f32(q: Fraction) -> Fraction:
    """Nearest binary32 value of an exact rational (normal range), ties to even."""
    if q == 0:
        return Fraction(0)
    sign, a = (-1, -q) if q < 0 else (1, q)
    e = a.numerator.bit_length() - a.denominator.bit_length()
    if Fraction(2) ** e > a:
        e -= 1
    elif Fraction(2) ** (e + 1) <= a:
        e += 1
    ulp = Fraction(2) ** (e - 23)
    n = a / ulp
    fl = n.numerator // n.denominator
    rem = n - fl
    if rem > Fraction(1, 2) or (rem == Fraction(1, 2) and fl % 2 == 1):
        fl += 1
    return sign * fl * ulp


def round_half_even(q: Fraction) -> int:
    fl = q.numerator // q.denominator
    rem = q - fl
    if rem > Fraction(1, 2) or (rem == Fraction(1, 2) and fl % 2 == 1):
        fl += 1
    return fl


def output_from_weights(p_row, v, v_scale, o_scale):
    """The part after P, in exact arithmetic with explicit fp32 roundings: int->float, divide, multiply, rne, clamp."""
    d = len(v[0])
    l = sum(int(x) for x in p_row)
    r = rne_f32(Fraction(float(np.float32(v_scale))) / Fraction(float(np.float32(o_scale))))
    out = []
    for c in range(d):
        a = sum(int(p_row[j]) * int(v[j][c]) for j in range(len(p_row)))
        t = rne_f32(rne_f32(rne_f32(Fraction(a)) / rne_f32(Fraction(l))) * r)
        out.append(max(-128, min(127, round_half_even(t))))
    return out


@pytest.mark.parametrize("case", _cases(), ids=lambda c: "S%d-d%d" % (c["S"], c["d"]))
def test_hand_cases(oracle_mod, case):
    s_, d = case["S"], case["d"]
    q = np.array(case["Q"], np.int8).reshape(1, 1, s_, d)
    k = np.array(case["K"], np.int8).reshape(1, 1, s_, d)
    v = np.array(case["V"], np.int8).reshape(1, 1, s_, d)
    mask = None if case["M"] is None else np.array(case["M"], np.float32).reshape(1, s_)
    scale, qs, ks, vs, os_ = case["scales"]
    o, p = oracle_mod.attention_i8(q, k, v, mask, scale, qs, ks, vs, os_, return_weights=True)
    assert p.reshape(-1).tolist() == case["P"]
    assert o.reshape(-1).tolist() == case["O"]


@pytest.mark.parametrize("seed", range(6))
def test_brute_force_tiny(oracle_mod, seed):
    """Scalar loops: scores and weights with math.exp on Python floats, everything after the weights exact."""
    rng = np.random.default_rng(4100 + seed)
    b, h, s_, d = 2, 2, int(rng.integers(1, 7)), int(rng.choice([1, 2, 5]))
    q, k, v = (rng.integers(-128, 128, (b, h, s_, d), dtype=np.int8) for _ in range(3))
    mask = np.where(rng.random((b, s_)) < 0.3, np.float32(-10000.0), np.float32(0.0)).astype(np.float32)
    mask[:, 0] = 0.0
    scale, qs, ks, vs, os_ = 1.0 / math.sqrt(d), 0.031, 0.027, 0.02, 0.011
    o, p = oracle_mod.attention_i8(q, k, v, mask, scale, qs, ks, vs, os_, return_weights=True)
    c = float(np.float32(qs)) * float(np.float32(ks)) * float(np.float32(scale))
    for bi in range(b):
        for hi in range(h):
            for i in range(s_):
                sc = [sum(int(q[bi, hi, i, t]) * int(k[bi, hi, j, t]) for t in range(d)) * c + float(mask[bi, j]) for j in range(s_)]
                m = max(sc)
                x = [127.0 * math.exp(z - m) for z in sc]
                want_p = [int(round_half_even(Fraction(z))) for z in x]
                # a weight within 1e-9 of a tie could legitimately fall either way; none of these seeds has one
                assert all(abs((z % 1.0) - 0.5) > 1e-9 for z in x)
                assert p[bi, hi, i].tolist() == want_p
                assert o[bi, hi, i].tolist() == output_from_weights(want_p, v[bi, hi].tolist(), vs, os_)


def test_invariants(oracle_mod):
    rng = np.random.default_rng(4200)
    b, h, s_, d = 2, 3, 9, 4
    q, k, v = (rng.integers(-100, 101, (b, h, s_, d), dtype=np.int8) for _ in range(3))
    mask = np.zeros((b, s_), np.float32)
    mask[1, 6:] = -10000.0
    args = (1.0 / math.sqrt(d), 0.03, 0.02, 0.05, 0.05)
    o, p = oracle_mod.attention_i8(q, k, v, mask, *args, return_weights=True)
    # every row of weights has its maximum at 127 and masked keys at 0
    assert (p.max(axis=-1) == 127).all() and (p[1, :, :, 6:] == 0).all()
    # a permutation of the keys (with their values and mask entries) changes nothing: integer sums are order-free
    perm = rng.permutation(s_)
    o2 = oracle_mod.attention_i8(q, k[:, :, perm], v[:, :, perm], mask[:, perm], *args)
    assert np.array_equal(o, o2)
    # batch entries and heads are independent
    o3 = oracle_mod.attention_i8(q[1:, 1:2], k[1:, 1:2], v[1:, 1:2], mask[1:], *args)
    assert np.array_equal(o[1:, 1:2], o3)
    # a mask that leaves one key returns that key's value row, rescaled: P = [127] on it alone
    one = np.full((b, s_), -10000.0, np.float32)
    one[:, 2] = 0.0
    o4 = oracle_mod.attention_i8(q, k, v, one, 1.0, 0.03, 0.02, 0.5, 0.25)     # v_scale / o_scale = 2
    want = np.clip(2 * v[:, :, 2:3, :].astype(np.int32), -128, 127).astype(np.int8)
    assert np.array_equal(o4, np.broadcast_to(want, o4.shape))
    # zero queries: uniform weights over the unmasked keys, o = rounded mean of their values
    o5, p5 = oracle_mod.attention_i8(np.zeros_like(q), k, v, None, 1.0, 0.03, 0.02, 1.0, 1.0, return_weights=True)
    assert (p5 == 127).all()
    mean = v.astype(np.float64).sum(axis=2, keepdims=True) / s_
    assert (np.abs(o5.astype(np.float64) - mean) <= 0.5 + 1e-6).all()
    # close to the float attention on the dequantized tensors: quantizing the weights to 7 bits costs about 1/127 each
    ref = oracle_mod.attention(q * np.float64(np.float32(0.03)), k * np.float64(np.float32(0.02)), v * np.float64(np.float32(0.05)),
                               mask, args[0])
    got = o.astype(np.float64) * np.float64(np.float32(0.05))
    # half an output step, plus values up to 100 * 0.05 = 5 times the summed error of S weights, each within 1/127
    assert np.abs(got - ref).max() <= 0.05 * 0.5 + 5.0 * s_ * (1.0 / 127)
