"""Pins for the CPU oracle: everything here checks the oracle against something other than
itself — hand-computed fixtures, exact rational arithmetic, closed forms, invariants, library
GEMMs on special cases — so that a dropped term, a wrong sign or index, or a transposed operand
in the oracle fails at least one test.  No GPU needed."""
import math
import os
from fractions import Fraction

import numpy as np
import pytest

from paper_2301_01333_amd import synth

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
RELU, NONE, GELU, SIGM = synth.ACT_RELU, synth.ACT_NONE, synth.ACT_GELU_TANH, synth.ACT_SIGMOID


# ----------------------------------------------------------------------------------------------
# exact helpers, written without reference to the oracle's code
# ----------------------------------------------------------------------------------------------
def rne_f32(q: Fraction) -> Fraction:
    """Round an exact rational to the nearest IEEE binary32 value, ties to even (normal and
    subnormal range; no overflow handling needed for the magnitudes used here)."""
    if q == 0:
        return Fraction(0)
    sign = -1 if q < 0 else 1
    a = -q if q < 0 else q
    e = a.numerator.bit_length() - a.denominator.bit_length()
    if Fraction(2) ** e > a:
        e -= 1
    elif Fraction(2) ** (e + 1) <= a:
        e += 1
    e = max(e, -126)
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


def F(x) -> Fraction:
    return Fraction(float(np.float32(x)))


def exact_int8_output(xrow, wcol, a_s, a_z, b_s, bias, c_s, c_z, relu=True):
    acc2 = sum((int(x) - a_z) * int(w) for x, w in zip(xrow, wcol))
    f = rne_f32(Fraction(acc2))
    s = rne_f32(F(a_s) * F(b_s))
    y = rne_f32(f * s + F(bias)) if bias is not None else rne_f32(f * s)
    if relu and y < 0:
        y = Fraction(0)
    inv = rne_f32(1 / F(c_s))
    t = rne_f32(y * inv)
    r = round_half_even(t) + c_z
    return min(max(r, 0), 255)


def test_rne_helper_matches_numpy_casts():
    rng = np.random.default_rng(1)
    for v in rng.standard_normal(200) * 10.0 ** rng.integers(-6, 6, 200):
        assert float(rne_f32(Fraction(float(v)))) == float(np.float32(v))
    assert rne_f32(Fraction(2 ** 24 + 1)) == 2 ** 24          # tie -> even
    assert rne_f32(Fraction(2 ** 24 + 3)) == 2 ** 24 + 4      # tie -> even


# ----------------------------------------------------------------------------------------------
# hand-computed fixtures
# ----------------------------------------------------------------------------------------------
def _int8_cases():
    out = []
    for line in open(os.path.join(GOLDEN, "int8_hand_cases.txt")):
        line = line.split("#")[0].strip()
        if line:
            b, q = line.split()
            out.append((float(b), int(q)))
    return out


@pytest.mark.parametrize("bias,expected", _int8_cases())
def test_int8_hand_cases(oracle_mod, bias, expected):
    xq = np.array([[130, 126]], dtype=np.uint8)
    wq = np.array([[3], [-1]], dtype=np.int8)
    y = oracle_mod.layer_i8(xq, wq, np.array([0.25], np.float32), np.array([bias], np.float32), 0.5, 128, RELU, 0.5, 128)
    assert y.dtype == np.uint8 and int(y[0, 0]) == expected
    # the fixture agrees with the exact-arithmetic evaluator as well
    assert exact_int8_output([130, 126], [3, -1], 0.5, 128, 0.25, bias, 0.5, 128) == expected


def _float_fixture():
    d = {"R": []}
    for line in open(os.path.join(GOLDEN, "float_hand_cases.txt")):
        line = line.split("#")[0].strip()
        if not line:
            continue
        tag, *vals = line.split()
        vals = [float(v) for v in vals]
        if tag == "R":
            d["R"].append(vals)
        else:
            d[tag] = vals
    return d


def test_float_hand_case(oracle_mod):
    d = _float_fixture()
    x = np.array(d["X"], np.float32).reshape(2, 2)
    w = np.array(d["W"], np.float32).reshape(2, 2)
    b = np.array(d["B"], np.float32)
    want = np.array(d["Y"], np.float32).reshape(2, 2)
    for dbl in (False, True):
        assert np.array_equal(oracle_mod.layer_f32(x, w, b, RELU, accum_double=dbl), want)
        yb = oracle_mod.layer_bf16(synth.f32_to_bf16_bits(x), synth.f32_to_bf16_bits(w), b, RELU, accum_double=dbl)
        assert np.array_equal(synth.bf16_bits_to_f32(yb), want)


def test_bf16_rounding_fixture(oracle_mod):
    """bf16 output rounding is to nearest even: identity-weight layer so Y = bf16(x)."""
    d = _float_fixture()
    for v, want in d["R"]:
        # split v into bf16-exact pieces (truncate, subtract, repeat): a layer with unit weights sums them
        # back exactly in fp32, so the only rounding is the final one to bf16
        parts, rest = [], np.float32(v)
        while rest != 0:
            p = synth.bf16_bits_to_f32(np.array([np.float32(rest).view(np.uint32) >> 16], np.uint16))[0]
            parts.append(p)
            rest = np.float32(rest - p)
        assert float(sum(float(p) for p in parts)) == v and len(parts) <= 3
        x = synth.f32_to_bf16_bits(np.array([parts], np.float32))
        assert np.array_equal(synth.bf16_bits_to_f32(x)[0], np.array(parts, np.float32))
        w = synth.f32_to_bf16_bits(np.ones((len(parts), 1), np.float32))
        y = oracle_mod.layer_bf16(x, w, None, NONE)
        assert synth.bf16_bits_to_f32(y)[0, 0] == np.float32(want), (v, want)
        # the generator's own conversion follows the same rule
        assert synth.bf16_bits_to_f32(synth.f32_to_bf16_bits(np.array([v], np.float32)))[0] == np.float32(want)


# ----------------------------------------------------------------------------------------------
# exhaustive / brute force against exact rational arithmetic
# ----------------------------------------------------------------------------------------------
def test_int8_exhaustive_k1(oracle_mod):
    """K=1, N=1: every u8 input against every s8 weight (incl. -128), awkward scales."""
    a_s, a_z, b_s, bias, c_s, c_z = 0.05, 128, 0.013, 0.07, 0.11, 128
    xq = np.arange(256, dtype=np.uint8).reshape(256, 1)
    for wv in range(-128, 128):
        y = oracle_mod.layer_i8(xq, np.array([[wv]], np.int8), np.array([b_s], np.float32), np.array([bias], np.float32),
                                a_s, a_z, RELU, c_s, c_z)
        if True:
            want = [exact_int8_output([x], [wv], a_s, a_z, b_s, bias, c_s, c_z) for x in range(256)]
            assert y[:, 0].tolist() == want, wv
        # monotone in x_q for w>0 (scale positive), anti-monotone for w<0: cheap check on all columns
        d = np.diff(y[:, 0].astype(np.int32))
        assert (d >= 0).all() if wv > 0 else (d <= 0).all()


@pytest.mark.parametrize("seed", range(6))
def test_int8_bruteforce_tiny(oracle_mod, seed):
    rng = np.random.default_rng(100 + seed)
    m, k, n = int(rng.integers(1, 5)), int(rng.integers(1, 8)), int(rng.integers(1, 5))
    xq = rng.integers(0, 256, (m, k), dtype=np.uint8)
    wq = rng.integers(-128, 128, (k, n), dtype=np.int8)
    ws = rng.uniform(0.005, 0.02, n).astype(np.float32)
    bias = rng.uniform(-0.5, 0.5, n).astype(np.float32)
    a_s, a_z, c_s, c_z = float(np.float32(0.037)), int(rng.integers(0, 256)), float(np.float32(0.021)), int(rng.integers(0, 256))
    use_bias = seed % 2 == 0
    y = oracle_mod.layer_i8(xq, wq, ws, bias if use_bias else None, a_s, a_z, RELU, c_s, c_z)
    for i in range(m):
        for j in range(n):
            want = exact_int8_output(xq[i], wq[:, j], a_s, a_z, ws[j], bias[j] if use_bias else None, c_s, c_z)
            assert int(y[i, j]) == want, (i, j)


def test_int8_compensation_identity(oracle_mod):
    """acc - a_z*sum_k w_q == sum_k (x_q - a_z) w_q, read back exactly through an fp32 output with
    unit scales (|acc2| < 2^24).  Non-square shapes so a transposed operand cannot pass."""
    rng = np.random.default_rng(7)
    for (m, k, n, a_z) in [(3, 5, 2, 128), (4, 17, 7, 3), (2, 64, 9, 255), (5, 9, 4, 0)]:
        xq = rng.integers(0, 256, (m, k), dtype=np.uint8)
        wq = rng.integers(-128, 128, (k, n), dtype=np.int8)
        y = oracle_mod.layer_i8(xq, wq, np.ones(n, np.float32), None, 1.0, a_z, NONE, out_f32=True)
        want = (xq.astype(np.int64) - a_z) @ wq.astype(np.int64)
        assert np.array_equal(y.astype(np.int64), want)


def test_int8_large_accumulator_rounds_to_nearest_even(oracle_mod):
    """|acc2| above 2^24: the int->float conversion itself rounds (ties to even)."""
    k = 2048
    xq = np.full((1, k), 255, np.uint8)
    wq = np.full((k, 1), 127, np.int8)
    wq[0, 0] = 0                      # acc2 = 255*127*2047 = 66 292 095 (odd, > 2^24 -> spacing 4..8)
    y = oracle_mod.layer_i8(xq, wq, np.ones(1, np.float32), None, 1.0, 0, NONE, out_f32=True)
    acc2 = 255 * 127 * 2047
    assert float(y[0, 0]) == float(rne_f32(Fraction(acc2))) == float(np.float32(acc2))


# ----------------------------------------------------------------------------------------------
# invariants
# ----------------------------------------------------------------------------------------------
def test_zero_weight_invariant(oracle_mod):
    rng = np.random.default_rng(3)
    m, k, n = 5, 11, 6
    bias = rng.uniform(-1, 1, n).astype(np.float32)
    x = rng.standard_normal((m, k)).astype(np.float32)
    y = oracle_mod.layer_f32(x, np.zeros((k, n), np.float32), bias, RELU)
    assert np.array_equal(y, np.broadcast_to(np.maximum(bias, 0), (m, n)))
    yb = oracle_mod.layer_bf16(synth.f32_to_bf16_bits(x), np.zeros((k, n), np.uint16), bias, RELU)
    assert np.array_equal(yb, np.broadcast_to(synth.f32_to_bf16_bits(np.maximum(bias, 0)), (m, n)))
    xq = rng.integers(0, 256, (m, k), dtype=np.uint8)
    c_s, c_z = 0.01, 128
    for a_z in (0, 128, 200):
        q = oracle_mod.layer_i8(xq, np.zeros((k, n), np.int8), np.full(n, 0.01, np.float32), bias, 0.05, a_z, RELU, c_s, c_z)
        want = [min(max(round_half_even(rne_f32(max(F(b), 0) * rne_f32(1 / F(c_s)))) + c_z, 0), 255) for b in bias]
        assert np.array_equal(q, np.broadcast_to(np.array(want, np.uint8), (m, n)))


def test_identity_invariant(oracle_mod):
    rng = np.random.default_rng(4)
    n = 9
    x = np.abs(rng.standard_normal((4, n))).astype(np.float32)
    assert np.array_equal(oracle_mod.layer_f32(x, np.eye(n, dtype=np.float32), None, RELU), x)
    xb = synth.f32_to_bf16_bits(x)
    assert np.array_equal(oracle_mod.layer_bf16(xb, synth.f32_to_bf16_bits(np.eye(n, dtype=np.float32)), None, RELU), xb)
    # int8: W = I, b_s = 1, a_s = c_s (power of two), a_z = c_z: q = x_q above the zero point, a_z below
    xq = rng.integers(0, 256, (6, n), dtype=np.uint8)
    for z in (128, 77):
        q = oracle_mod.layer_i8(xq, np.eye(n, dtype=np.int8), np.ones(n, np.float32), None, 0.25, z, RELU, 0.25, z)
        assert np.array_equal(q, np.maximum(xq, z))
    # non power-of-two scale: f*s*inv lands within rounding distance of the integer, RNE recovers it
    q = oracle_mod.layer_i8(xq, np.eye(n, dtype=np.int8), np.ones(n, np.float32), None, 0.05, 128, RELU, 0.05, 128)
    assert np.array_equal(q, np.maximum(xq, 128))


def test_permutation_invariants(oracle_mod):
    rng = np.random.default_rng(5)
    m, k, n = 7, 33, 10
    xq = rng.integers(0, 256, (m, k), dtype=np.uint8)
    wq = rng.integers(-127, 128, (k, n), dtype=np.int8)
    ws = rng.uniform(0.005, 0.02, n).astype(np.float32)
    bias = rng.uniform(-0.1, 0.1, n).astype(np.float32)
    base = oracle_mod.layer_i8(xq, wq, ws, bias, 0.05, 128, RELU, 0.03, 128)
    pk = rng.permutation(k)
    assert np.array_equal(oracle_mod.layer_i8(np.ascontiguousarray(xq[:, pk]), wq[pk], ws, bias, 0.05, 128, RELU, 0.03, 128), base)
    pn = rng.permutation(n)
    got = oracle_mod.layer_i8(xq, np.ascontiguousarray(wq[:, pn]), ws[pn], bias[pn], 0.05, 128, RELU, 0.03, 128)
    assert np.array_equal(got, base[:, pn])
    # rows are independent
    assert np.array_equal(oracle_mod.layer_i8(xq[2:5], wq, ws, bias, 0.05, 128, RELU, 0.03, 128), base[2:5])


def test_int8_equivalent_to_unrewritten_graph(oracle_mod):
    """Section V: the int8 form is a mathematically equivalent rewrite of DQ -> matmul -> Q.  The two
    can differ only where the pre-rounding value sits within fp32 rounding error of a tie."""
    wl = synth.make_mlp("i8", 64, [479, 256], [RELU], seed=11)
    ly = wl.layers[0]
    a = oracle_mod.layer_i8(wl.x, wl.w[0], wl.w_scale[0], wl.bias[0], ly.in_scale, ly.in_zp, RELU, ly.out_scale, ly.out_zp)
    b = oracle_mod.layer_i8_unfused(wl.x, wl.w[0], wl.w_scale[0], wl.bias[0], ly.in_scale, ly.in_zp, RELU, ly.out_scale, ly.out_zp)
    d = a.astype(np.int32) - b.astype(np.int32)
    assert np.abs(d).max() <= 1
    assert (d != 0).mean() < 1e-3
    # and the outputs are not degenerate: the synthetic scales spread values over the u8 range
    assert a.min() == 128 and a.max() == 255 and 0.3 < (a > 128).mean() < 0.7 and len(np.unique(a)) > 60


# ----------------------------------------------------------------------------------------------
# special cases that reduce to a library routine / closed forms
# ----------------------------------------------------------------------------------------------
def test_float_layer_matches_library_gemm(oracle_mod):
    rng = np.random.default_rng(6)
    m, k, n = 9, 37, 13
    x = rng.standard_normal((m, k)).astype(np.float32)
    w = rng.standard_normal((k, n)).astype(np.float32)
    ref = x.astype(np.float64) @ w.astype(np.float64)
    y32 = oracle_mod.layer_f32(x, w, None, NONE)
    y64 = oracle_mod.layer_f32(x, w, None, NONE, accum_double=True)
    assert np.array_equal(y64, ref.astype(np.float32))
    bound = k * 2.0 ** -24 * (np.abs(x).astype(np.float64) @ np.abs(w).astype(np.float64))  # fp32 summation bound
    assert (np.abs(y32 - ref) <= bound + 1e-30).all()
    # bf16: operands bf16-exact -> fp64 GEMM then one RNE cast
    xb, wb = synth.f32_to_bf16_bits(x), synth.f32_to_bf16_bits(w)
    refb = synth.bf16_bits_to_f32(xb).astype(np.float64) @ synth.bf16_bits_to_f32(wb).astype(np.float64)
    yb = oracle_mod.layer_bf16(xb, wb, None, NONE, accum_double=True)
    assert np.array_equal(yb, synth.f32_to_bf16_bits(refb.astype(np.float32)))
    yb32 = synth.bf16_bits_to_f32(oracle_mod.layer_bf16(xb, wb, None, NONE))
    assert np.allclose(yb32, refb, rtol=2.0 ** -7, atol=1e-6)


def test_residual_and_bias_terms(oracle_mod):
    rng = np.random.default_rng(8)
    m, k = 4, 6
    x = rng.standard_normal((m, k)).astype(np.float32)
    w = rng.standard_normal((k, k)).astype(np.float32)
    b = rng.standard_normal(k).astype(np.float32)
    ref = np.maximum(x.astype(np.float64) @ w + b, 0) + x          # residual is added after the activation
    assert np.allclose(oracle_mod.layer_f32(x, w, b, RELU, residual=x, accum_double=True), ref, rtol=1e-6)
    assert np.allclose(oracle_mod.layer_f32(x, w, b, RELU, residual=x), ref, rtol=1e-4, atol=1e-5)


def test_bf16_residual_is_added_in_fp32_before_the_single_rounding(oracle_mod):
    """Hand case from the fixture: rounding to bf16 before the residual add gives 1.0 where the
    reading taken (fp32 add, one rounding) gives 1.0078125."""
    d = _float_fixture()
    x = synth.f32_to_bf16_bits(np.array([d["RESX"]], np.float32))
    assert np.array_equal(synth.bf16_bits_to_f32(x)[0], np.array(d["RESX"], np.float32))   # operands are bf16-exact
    w = synth.f32_to_bf16_bits(np.array(d["RESW"], np.float32).reshape(2, 2))
    want = np.array([d["RESY"]], np.float32)
    for dbl in (False, True):
        y = oracle_mod.layer_bf16(x, w, None, NONE, residual=x, accum_double=dbl)
        assert np.array_equal(synth.bf16_bits_to_f32(y), want), (dbl, synth.bf16_bits_to_f32(y))
    # without the residual the same layer gives [2^-8, bf16(1 + 2^-8) = 1]
    y0 = synth.bf16_bits_to_f32(oracle_mod.layer_bf16(x, w, None, NONE))
    assert np.array_equal(y0, np.array([[2.0 ** -8, 1.0]], np.float32))


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_chain_residual_is_the_first_input_on_the_last_layer_only(oracle_mod, dtype):
    """Two-layer chain from the fixture: the last layer adds the chain's first input x0 (not its own
    input), and layer 0 adds nothing."""
    d = _float_fixture()
    conv = synth.f32_to_bf16_bits if dtype == "bf16" else (lambda a: np.ascontiguousarray(a, np.float32))
    back = synth.bf16_bits_to_f32 if dtype == "bf16" else (lambda a: a)
    x0 = conv(np.array([d["CHX"]], np.float32))
    ws = [conv(np.array(d[t], np.float32).reshape(2, 2)) for t in ("CHW0", "CHW1")]
    layers = [synth.Layer(2, 2, False, NONE), synth.Layer(2, 2, False, NONE)]
    wl = synth.Workload("hand chain", dtype, 1, layers, True, x0, ws, [None, None], [None, None])
    outs = oracle_mod.mlp(wl, keep=True)
    assert np.array_equal(back(outs[0]), np.array([[2.0, 2.0 ** -7]], np.float32))          # no residual on layer 0
    if dtype == "bf16":
        want = np.array([d["CHY"]], np.float32)
    else:   # the same sums without the bf16 rounding: [2^-7 + 1, 1 + 2^-7 + 2^-8], exact in fp32
        want = np.array([[1.0 + 2.0 ** -7, 1.0 + 2.0 ** -7 + 2.0 ** -8]], np.float32)
    assert np.array_equal(back(outs[1]), want), back(outs[1])
    wl.residual = False
    plain = back(oracle_mod.mlp(wl))
    assert np.array_equal(plain, np.array([[2.0 ** -7, 1.0 + 2.0 ** -7]], np.float32))


def test_activation_closed_forms(oracle_mod):
    from oracle import oracle as o

    for fn, tol in ((o.act_f64, 1e-14), (o.act_f32, 2e-6)):
        assert fn(0.0, GELU) == 0.0
        assert fn(0.0, SIGM) == 0.5
        for v in (0.1, 0.7, 1.3, 2.9, 6.0):
            assert abs(fn(v, GELU) - fn(-v, GELU) - v) < tol * max(1, v)      # gelu(x) - gelu(-x) = x
            assert abs(fn(v, SIGM) + fn(-v, SIGM) - 1.0) < tol
            vv = v if fn is o.act_f64 else float(np.float32(v))
            assert fn(fn(v, RELU), RELU) == fn(v, RELU) == vv and fn(-v, RELU) == 0.0
            assert fn(v, NONE) == vv
    # independent evaluation of the tanh-form GELU and of the logistic function
    for v in (-3.0, -0.5, 0.25, 1.0, 2.5):
        g = 0.5 * v * (1.0 + math.tanh(math.sqrt(2.0 / math.pi) * (v + 0.044715 * v ** 3)))
        assert abs(o.act_f64(v, GELU) - g) < 1e-14
        assert abs(o.act_f32(v, GELU) - g) < 1e-6
        assert abs(o.act_f64(v, SIGM) - 1.0 / (1.0 + math.exp(-v))) < 1e-15
    # large |x|: gelu -> x or 0, sigmoid -> 1 or 0, no NaN
    assert o.act_f32(30.0, GELU) == 30.0 and o.act_f32(-30.0, GELU) == 0.0
    assert o.act_f32(100.0, SIGM) == 1.0 and o.act_f32(-100.0, SIGM) == 0.0


def test_chain_feeds_rounded_outputs_forward(oracle_mod):
    """A chain is the layer definition applied repeatedly: layer l+1 consumes layer l's stored
    (rounded / requantized) output, and the last layer of an int8 chain may emit fp32."""
    wl = synth.make_mlp("i8", 8, [19, 12, 1], [RELU, SIGM], seed=21, last_f32=True)
    outs = oracle_mod.mlp(wl, keep=True)
    assert outs[0].dtype == np.uint8 and outs[1].dtype == np.float32 and outs[1].shape == (8, 1)
    l1 = wl.layers[1]
    assert l1.in_scale == wl.layers[0].out_scale and l1.in_zp == wl.layers[0].out_zp
    real_h = l1.in_scale * (outs[0].astype(np.float64) - l1.in_zp)
    real_w = wl.w_scale[1].astype(np.float64) * wl.w[1].astype(np.float64)
    ref = 1.0 / (1.0 + np.exp(-(real_h @ real_w + wl.bias[1])))
    assert np.allclose(outs[1], ref, rtol=1e-5, atol=1e-7)
    wb = synth.make_mlp("bf16", 8, [13, 24, 5], [RELU, NONE], seed=22)
    ob = oracle_mod.mlp(wb, keep=True)
    h = synth.bf16_bits_to_f32(ob[0]).astype(np.float64)
    ref = h @ synth.bf16_bits_to_f32(wb.w[1]).astype(np.float64) + wb.bias[1]
    assert np.allclose(synth.bf16_bits_to_f32(ob[1]), ref, rtol=2.0 ** -7, atol=1e-6)
    assert np.array_equal(oracle_mod.mlp(wb, rows=slice(2, 6)), ob[1][2:6])


def test_strided_input_rows(oracle_mod):
    wl = synth.make_mlp("i8", 6, [13, 8], [RELU], seed=31, ld_x=20)
    assert wl.x.strides[0] == 20
    ly = wl.layers[0]
    a = oracle_mod.layer_i8(wl.x, wl.w[0], wl.w_scale[0], wl.bias[0], ly.in_scale, ly.in_zp, RELU, ly.out_scale, ly.out_zp)
    b = oracle_mod.layer_i8(np.ascontiguousarray(wl.x), wl.w[0], wl.w_scale[0], wl.bias[0], ly.in_scale, ly.in_zp, RELU,
                            ly.out_scale, ly.out_zp)
    assert np.array_equal(a, b)


def test_int8_dequant_bias_is_one_fused_rounding(oracle_mod):
    """y = fma(f, s, bias): a single rounding.  Read y back through the fp32 output and compare with
    exact arithmetic; separate multiply-then-add rounding differs on a good share of these inputs."""
    rng = np.random.default_rng(12)
    m, k, n = 16, 24, 12
    xq = rng.integers(0, 256, (m, k), dtype=np.uint8)
    wq = rng.integers(-127, 128, (k, n), dtype=np.int8)
    ws = rng.uniform(0.005, 0.02, n).astype(np.float32)
    bias = rng.uniform(-0.1, 0.1, n).astype(np.float32)
    a_s, a_z = float(np.float32(0.05)), 128
    y = oracle_mod.layer_i8(xq, wq, ws, bias, a_s, a_z, NONE, out_f32=True)
    differ = 0
    for i in range(m):
        for j in range(n):
            acc2 = int(((xq[i].astype(np.int64) - a_z) * wq[:, j].astype(np.int64)).sum())
            s = rne_f32(F(a_s) * F(ws[j]))
            fused = rne_f32(Fraction(acc2) * s + F(bias[j]))
            split = rne_f32(rne_f32(Fraction(acc2) * s) + F(bias[j]))
            differ += fused != split
            assert Fraction(float(y[i, j])) == fused, (i, j)
    assert differ > 5   # the case set does distinguish the two
