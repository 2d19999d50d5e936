"""Pins for the attention oracle (oracle/mha.py): hand-computed fixtures, brute force with scalar loops, a
library softmax on the special case that reduces to it, closed forms and invariants, chosen so that a
transposed operand, a mask of the wrong sign or axis, a missing scale or a softmax over the wrong axis each
fail at least one.  No GPU needed."""
import math
import os
from fractions import Fraction

import numpy as np
import pytest

from paper_2301_01333_amd import synth

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


@pytest.fixture(scope="module")
def att():
    import oracle

    return oracle


def _tok(t):
    logs = {"LN2": math.log(2.0), "LN3": math.log(3.0), "LN5": math.log(5.0)}
    return logs[t] if t in logs else float(Fraction(t))


def _cases():
    cases, cur = [], None
    for line in open(os.path.join(GOLDEN, "mha_hand_cases.txt")):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        tag, *rest = line.split()
        if tag == "CASE":
            cur = {"S": int(rest[0]), "d": int(rest[1]), "scale": float(rest[2])}
            cases.append(cur)
        elif tag == "M":
            cur["M"] = None if rest == ["-"] else np.array([_tok(t) for t in rest])
        else:
            cur[tag] = np.array([_tok(t) for t in rest])
    return cases


@pytest.mark.parametrize("case", _cases(), ids=lambda c: "S%d_d%d_scale%g" % (c["S"], c["d"], c["scale"]))
@pytest.mark.parametrize("softmax", [0, 1])
def test_hand_cases(att, case, softmax):
    S, d = case["S"], case["d"]
    q, k, v = (case[t].reshape(1, 1, S, d) for t in "QKV")
    mask = None if case["M"] is None else case["M"].reshape(1, S)
    o = att.attention(q, k, v, mask, case["scale"], softmax)
    np.testing.assert_allclose(o.reshape(-1), case["O"], rtol=1e-14, atol=0)


def _brute(q, k, v, mask, scale, stable):
    """Scalar loops over every index, written from the definition."""
    B, H, S, d = q.shape
    o = np.zeros((B, H, S, d))
    sc = float(np.float32(scale))
    for b in range(B):
        for h in range(H):
            for i in range(S):
                row = []
                for j in range(S):
                    acc = 0.0
                    for c in range(d):
                        acc += float(q[b, h, i, c]) * float(k[b, h, j, c])
                    acc *= sc
                    if mask is not None:
                        acc += float(mask[b, j])
                    row.append(acc)
                top = max(row) if stable else 0.0
                ex = [math.exp(r - top) for r in row]
                tot = math.fsum(ex)
                for c in range(d):
                    o[b, h, i, c] = math.fsum(ex[j] / tot * float(v[b, h, j, c]) for j in range(S))
    return o


@pytest.mark.parametrize("seed", range(6))
def test_brute_force_tiny(att, seed):
    rng = np.random.default_rng(900 + seed)
    B, H, S, d = (int(x) for x in (rng.integers(1, 3), rng.integers(1, 4), rng.integers(1, 8), rng.integers(1, 6)))
    q, k, v = (rng.standard_normal((B, H, S, d)) for _ in range(3))
    mask = rng.uniform(-3, 0, size=(B, S)) if seed % 2 else None
    scale = 1.0 / math.sqrt(d)
    for softmax in (0, 1):
        o = att.attention(q, k, v, mask, scale, softmax)
        np.testing.assert_allclose(o, _brute(q, k, v, mask, scale, softmax == 0), rtol=1e-12, atol=1e-14)


def test_library_softmax_special_case(att):
    """With V the identity (S = d) the output IS the softmax matrix; scipy's softmax is the library routine."""
    from scipy.special import softmax as sp_softmax

    rng = np.random.default_rng(77)
    B, H, S = 2, 3, 9
    q, k = rng.standard_normal((B, H, S, S)), rng.standard_normal((B, H, S, S))
    v = np.broadcast_to(np.eye(S), (B, H, S, S))
    mask = rng.uniform(-2, 0, size=(B, S))
    scale = float(np.float32(0.37))
    want = sp_softmax(np.einsum("bhic,bhjc->bhij", q, k) * scale + mask[:, None, None, :], axis=-1)
    for softmax in (0, 1):
        np.testing.assert_allclose(att.attention(q, k, v, mask, 0.37, softmax), want, rtol=1e-12, atol=1e-15)


def test_zero_queries_give_the_mean_of_v(att):
    rng = np.random.default_rng(5)
    k, v = rng.standard_normal((1, 2, 7, 4)), rng.standard_normal((1, 2, 7, 4))
    o = att.attention(np.zeros((1, 2, 7, 4)), k, v, None, 1.0)
    np.testing.assert_allclose(o, np.broadcast_to(v.mean(axis=2, keepdims=True), o.shape), rtol=1e-13)


def test_mask_selects_a_key_per_batch_entry(att):
    """A padding mask that leaves one key: every query of every head returns that key's value row."""
    rng = np.random.default_rng(6)
    B, H, S, d = 3, 2, 6, 5
    q, k, v = (rng.standard_normal((B, H, S, d)) for _ in range(3))
    keep = [4, 0, 2]
    mask = np.full((B, S), -10000.0)
    for b, j in enumerate(keep):
        mask[b, j] = 0.0
    for softmax in (0, 1):
        o = att.attention(q, k, v, mask, 0.5, softmax)
        for b, j in enumerate(keep):
            np.testing.assert_allclose(o[b], np.broadcast_to(v[b, :, j:j + 1, :], (H, S, d)), rtol=1e-13)


def test_invariants(att):
    rng = np.random.default_rng(8)
    B, H, S, d = 2, 2, 10, 6
    q, k, v = (rng.standard_normal((B, H, S, d)) for _ in range(3))
    mask = rng.uniform(-4, 0, size=(B, S))
    base = att.attention(q, k, v, mask, 0.4)
    # the keys are a set: permuting k, v and the mask together changes nothing
    perm = rng.permutation(S)
    np.testing.assert_allclose(att.attention(q, k[:, :, perm], v[:, :, perm], mask[:, perm], 0.4), base, rtol=1e-12)
    # permuting the queries permutes the output rows
    np.testing.assert_allclose(att.attention(q[:, :, perm], k, v, mask, 0.4), base[:, :, perm], rtol=1e-12)
    # softmax ignores a constant added to every key of a batch entry
    np.testing.assert_allclose(att.attention(q, k, v, mask + 2.5, 0.4), base, rtol=1e-12)
    # the weights of a row sum to one
    np.testing.assert_allclose(att.attention(q, k, np.ones_like(v), mask, 0.4), np.ones_like(v), rtol=1e-13)
    # linear in v
    v2 = rng.standard_normal(v.shape)
    np.testing.assert_allclose(att.attention(q, k, 2 * v - 3 * v2, mask, 0.4),
                               2 * base - 3 * att.attention(q, k, v2, mask, 0.4), rtol=1e-10, atol=1e-12)
    # scaling q by c equals scaling the scalar by c (c and c*scale exact in fp32)
    np.testing.assert_allclose(att.attention(2 * q, k, v, mask, 0.25), att.attention(q, k, v, mask, 0.5), rtol=1e-12)
    # heads and batch entries are independent
    np.testing.assert_allclose(att.attention(q[1:, :1], k[1:, :1], v[1:, :1], mask[1:], 0.4), base[1:, :1], rtol=1e-13)
    # both softmax forms agree where nothing overflows
    np.testing.assert_allclose(att.attention(q, k, v, mask, 0.4, 1), base, rtol=1e-12)


def test_stable_form_survives_huge_scores(att):
    """Scores near 2000: exp overflows without the max subtraction; the stable form picks the top key."""
    q = np.array([[[[1000.0]]]])
    k = np.array([[[[1.0], [2.0]]]])
    v = np.array([[[[5.0], [9.0]]]])
    np.testing.assert_allclose(att.attention(np.broadcast_to(q, (1, 1, 2, 1)), k, v, None, 1.0), [[[[9.0], [9.0]]]])


def test_generator_shapes_and_mask():
    w = synth.make_mha_table1("MHA-1", "bf16", 2)
    assert (w.seq, w.heads, w.head_dim) == (128, 8, 96) and w.q.dtype == np.uint16 and w.q.shape == (2, 128, 768)
    assert w.mask.shape == (2, 128) and set(np.unique(w.mask)) <= {np.float32(0.0), np.float32(-10000.0)}
    assert (w.mask[:, 0] == 0).all() and w.scale == float(np.float32(1 / math.sqrt(96)))
    assert w.ops == 4 * 2 * 8 * 128 * 128 * 96
    w2 = synth.make_mha_table1("MHA-1", "bf16", 2)
    assert (w.q == w2.q).all() and (w.mask == w2.mask).all()
