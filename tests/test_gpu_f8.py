"""GPU parity of the 8-bit-float (E4M3) variant of the quantized chain, through the C ABI, against the CPU oracle.

The gate.  The matrix unit multiplies E4M3 operands exactly but adds the products of one instruction after aligning
them to the largest one and keeping about 13 bits below it (measured on the part: a 16-term instruction is off by up
to 2^-12.8 of its largest product), so the accumulator differs from the oracle's exact sum by more than fp32 rounding
would explain.  The tolerance on the accumulator is therefore  tol_acc = 2^-11 * sum_k |x8 w8|  (several times the
largest error observed at any K from 16 to 1024); everything after the accumulator is the same fp32 sequence on both
sides, so
  * one layer, fp32 output: |gpu - ref| <= 1.2 * tol_acc * scale + 1e-5 |ref|   (1.2 bounds the slope of the activations)
  * one layer, E4M3 output: the GPU's code must be the encoding of SOME value within that tolerance of the oracle's
    pre-rounding value: ordinal(encode(t - tol)) <= ordinal(gpu code) <= ordinal(encode(t + tol)), the encoder being
    the oracle's.  Away from a rounding boundary that pins the code exactly (measured: > 99.9 % of codes are equal).
  * a chain: every layer is also run by itself on the oracle's intermediate (the gate above for each layer's kernel at
    its shape); end to end, a code that moved at a boundary perturbs the next layer, so the final result is held to one
    E4M3 step plus what one moved input code can shift a short dot product by: |gpu - ref| <= 2^-3 |ref| + 6e-2 max|ref|
    on the decoded values (fp32 output: 3e-2 |ref| + 6e-2 max|ref|), and at most 5 % of the codes differ.  (One moved input
    shifts a dot product by up to 2^-3 of its largest term, which over the short reduction axes used here, K >= 48, is up
    to about 5 % of the largest output.)  The per-layer runs are the parity evidence; this one checks the wiring.
"""
import numpy as np
import pytest

from paper_2301_01333_amd import binding, synth

from test_gpu_parity import MODES, assert_close, run_gpu

pytestmark = pytest.mark.gpu

RELU, NONE, GELU, SIGM = synth.ACT_RELU, synth.ACT_NONE, synth.ACT_GELU_TANH, synth.ACT_SIGMOID


def decode(oracle_mod, codes):
    table = np.array([oracle_mod.oracle.e4m3_to_f32(c) for c in range(256)], dtype=np.float64)
    return table[codes]


def single_layer(wl, l, x):
    ly = wl.layers[l]
    return synth.Workload("%s[layer %d]" % (wl.name, l), "f8", wl.m, [ly], False, x, [wl.w[l]], [wl.bias[l]], [wl.w_scale[l]], wl.seed)


def ordinal(codes):
    """Signed position of a code on the number line (-0 and +0 both 0)."""
    c = codes.astype(np.int32)
    return np.where(c & 0x80, -(c & 0x7F), c & 0x7F)


def check_one_layer(oracle_mod, wl, mode, **kw):
    """The gate for a one-layer workload."""
    assert len(wl.layers) == 1
    ly = wl.layers[0]
    got, _ = run_gpu(wl, mode, **kw)
    got = got[:, :ly.n]
    bias = wl.bias[0] if ly.has_bias else None
    y = oracle_mod.oracle.layer_f8(wl.x, wl.w[0], wl.w_scale[0], bias, ly.in_scale, ly.act, out_f32=True).astype(np.float64)
    tol_acc = 2.0 ** -11 * (np.abs(decode(oracle_mod, wl.x)) @ np.abs(decode(oracle_mod, wl.w[0])))
    tol_y = 1.2 * tol_acc * (np.float64(np.float32(ly.in_scale)) * wl.w_scale[0].astype(np.float64))[None, :]
    if ly.out_f32:
        assert np.isfinite(got).all()
        err = np.abs(got.astype(np.float64) - y)
        assert (err <= tol_y + 1e-5 * np.abs(y)).all(), "fp32 output: worst excess %g" % (err - tol_y - 1e-5 * np.abs(y)).max()
        return
    ref = oracle_mod.mlp(wl)
    print("   codes equal: %.4f %%" % (100.0 * (got == ref).mean()), flush=True)
    assert (got == ref).mean() > 0.99
    bad = np.argwhere(got != ref)
    inv = np.float64(np.float32(1.0) / np.float32(ly.out_scale))
    enc = oracle_mod.oracle.f32_to_e4m3
    for i, j in bad:
        t, tol = y[i, j] * inv, tol_y[i, j] * inv * 1.0001 + 1e-30
        lo, hi = ordinal(np.uint8(enc(t - tol))), ordinal(np.uint8(enc(t + tol)))
        assert lo <= ordinal(got[i, j]) <= hi, "code 0x%02x outside the codes 0x%02x..0x%02x reachable from t = %r +- %g at (%d, %d)" % (
            got[i, j], enc(t - tol), enc(t + tol), t, tol, i, j)


def check_chain(oracle_mod, wl, mode, layers_alone=True, **kw):
    print("case:", wl.name, "f8 M=%d" % wl.m, wl.dims, "mode=%s" % mode, kw, flush=True)
    outs = oracle_mod.mlp(wl, keep=True)
    if len(wl.layers) == 1:
        check_one_layer(oracle_mod, wl, mode, **kw)
        return
    if layers_alone:
        x = wl.x
        for l in range(len(wl.layers)):
            check_one_layer(oracle_mod, single_layer(wl, l, np.ascontiguousarray(x)), mode, **({"tile": kw["tile"]} if "tile" in kw else {}))
            x = outs[l]
    got, _ = run_gpu(wl, mode, **kw)
    n = wl.layers[-1].n
    pad, got = got[:, n:], got[:, :n]
    if pad.size:
        assert (pad.view(np.uint8) == 0xCD).all(), "bytes beyond n_last in a strided y were touched"
    ref = outs[-1]
    if wl.layers[-1].out_f32:
        err = np.abs(got.astype(np.float64) - ref)
        assert np.isfinite(got).all() and (err <= 3e-2 * np.abs(ref) + 6e-2 * np.abs(ref).max()).all(), err.max()
        return got
    vg, vr = decode(oracle_mod, got), decode(oracle_mod, ref)
    assert np.isfinite(vg).all()
    err = np.abs(vg - vr)
    bound = 0.125 * np.abs(vr) + 6e-2 * np.abs(vr).max()
    assert (err <= bound).all(), "%d of %d outside one E4M3 step; worst %g" % ((err > bound).sum(), err.size, (err - bound).max())
    assert (got != ref).mean() < 0.05, (got != ref).mean()
    return got


# ---------------------------------------------------------------- the boundary's quantize / dequantize nodes
def test_quantize_and_dequantize_match_the_oracle_encoding(oracle_mod):
    import torch

    table = decode(oracle_mod, np.arange(0x7F, dtype=np.uint8))
    mids = (table[:-1] + table[1:]) / 2
    pts = np.concatenate([table, mids, [464.0, 465.0, 1e30, 2.0 ** -10, 2.0 ** -11, 1e-40, 0.0]]).astype(np.float32)
    pts = np.concatenate([pts, np.nextafter(pts, np.float32(np.inf)), np.nextafter(pts, np.float32(-np.inf))])
    rng = np.random.default_rng(11)
    rnd = np.concatenate([rng.uniform(0, 500, 50000), np.exp(rng.uniform(np.log(2.0 ** -13), np.log(600.0), 50000))]).astype(np.float32)
    a = np.concatenate([pts, rnd, [np.inf]]).astype(np.float32)
    a = np.concatenate([a, -a, [np.nan]]).astype(np.float32)
    a = a[(np.abs(a) >= 2.0 ** -100) | (a == 0) | np.isnan(a)]   # fp32 subnormal inputs are outside the contract (flushed)
    for scale in (1.0, 7.0, 0.013):
        x = torch.from_numpy(a).cuda()
        out = torch.full((a.size + 5,), 0xCD, dtype=torch.uint8, device="cuda")
        binding.ogc_quantize_e4m3(x.data_ptr(), out.data_ptr(), a.size, scale)
        torch.cuda.synchronize()
        got = out.cpu().numpy()
        assert (got[a.size:] == 0xCD).all()
        t = a * (np.float32(1.0) / np.float32(scale))
        want = np.array([oracle_mod.oracle.f32_to_e4m3(float(v)) for v in t], dtype=np.uint8)
        nan = np.isnan(a)
        assert np.array_equal(got[:a.size][~nan], want[~nan]), (a[~nan][got[:a.size][~nan] != want[~nan]][:8], scale)
        assert ((got[:a.size][nan] & 0x7F) == 0x7F).all()    # a NaN stays a NaN (its sign bit is not specified)
    codes = torch.arange(256, dtype=torch.uint8, device="cuda")
    back = torch.empty(256, dtype=torch.float32, device="cuda")
    binding.ogc_dequantize_e4m3(codes.data_ptr(), back.data_ptr(), 256, 0.5)
    torch.cuda.synchronize()
    want = np.array([oracle_mod.oracle.e4m3_to_f32(c) for c in range(256)], dtype=np.float32) * np.float32(0.5)
    got = back.cpu().numpy()
    assert np.array_equal(np.isnan(got), np.isnan(want)) and np.array_equal(got[~np.isnan(want)], want[~np.isnan(want)])
    assert np.array_equal(np.signbit(got[~np.isnan(want)]), np.signbit(want[~np.isnan(want)]))
    with pytest.raises(binding.OgcError):
        binding.ogc_quantize_e4m3(x.data_ptr(), out.data_ptr(), 4, 0.0)
    with pytest.raises(binding.OgcError):
        binding.ogc_quantize_e4m3(x.data_ptr() + 1, out.data_ptr(), 4, 1.0)
    binding.ogc_quantize_e4m3(0, 0, 0, 1.0)   # nothing to do


# ---------------------------------------------------------------- one layer, every kernel
@pytest.mark.parametrize("tile", [0, 1, 2, 3, 4, 5])
def test_one_layer_every_tile(oracle_mod, tile):
    """Of the stream shapes only the eight-wave one (tile 4) is built for E4M3: forced tiles 3 and 5, and tile 4 on a first
    layer whose rows need K padding, fall back to the register-staged 128x128 tile."""
    m = {0: 300, 1: 150, 2: 77, 3: 260, 4: 100, 5: 64}[tile]
    for dims, act, f32 in (([100, 333], RELU, False), ([256, 72], NONE, False), ([479, 33], GELU, False), ([64, 5], SIGM, True)):
        wl = synth.make_mlp("f8", m, dims, [act], seed=1500 + tile, last_f32=f32, name="one-layer")
        print("case:", wl.name, m, dims, act, f32, "tile", tile, flush=True)
        check_one_layer(oracle_mod, wl, "per_layer", tile=tile)


@pytest.mark.parametrize("mode", ["fused", "coop", "auto"])
def test_one_layer_chain_modes(oracle_mod, mode):
    for m, dims in ((77, [37, 130]), (1, [1, 1]), (300, [192, 64])):
        wl = synth.make_mlp("f8", m, dims, [RELU], seed=1600, name="one-layer")
        print("case:", wl.name, m, dims, mode, flush=True)
        check_one_layer(oracle_mod, wl, mode)


def test_saturation_subnormals_and_signed_zero(oracle_mod):
    """Scales chosen so that a large share of the outputs saturate at +-448, and another run so that most land in the
    subnormal range; no activation, so negative results and -0 are stored too."""
    base = synth.make_mlp("f8", 96, [128, 80], [NONE], seed=1700, name="range")
    for factor, what in ((1.0 / 64, "saturating"), (4096.0, "subnormal")):
        ly = base.layers[0]
        ly2 = synth.Layer(ly.k, ly.n, True, NONE, in_scale=ly.in_scale, out_scale=float(np.float32(ly.out_scale * factor)))
        wl = synth.Workload(what, "f8", base.m, [ly2], False, base.x, base.w, base.bias, base.w_scale, base.seed)
        ref = oracle_mod.mlp(wl)
        if what == "saturating":
            assert ((ref & 0x7F) == 0x7E).mean() > 0.3
        else:
            assert ((ref & 0x78) == 0).mean() > 0.3 and ((ref & 0x7F) != 0).any()
        for mode in ("per_layer", "fused"):
            check_one_layer(oracle_mod, wl, mode)
    # all-zero weights and no bias: every output is +0
    wl = synth.make_mlp("f8", 40, [64, 48], [NONE], seed=1701, has_bias=False)
    wl.w[0][:] = 0
    got, _ = run_gpu(wl, "per_layer")
    assert (got == 0).all() and (oracle_mod.mlp(wl) == 0).all()


def test_stream_kernel(oracle_mod):
    """The persistent stream kernel on the full-rate fp8 matrix instruction (K = 64 per instruction): plain and blocked
    input, plain and blocked output, several tiles per workgroup, short (4 steps) and long reduction axes, ragged
    channel counts, every layer also alone against the oracle's intermediate."""
    from paper_2301_01333_amd.harness import DeviceMLP

    wl = synth.make_mlp("f8", 700, [256, 512, 320, 64], [RELU, GELU, NONE], seed=2200, name="stream")
    d = DeviceMLP(wl, binding.OGC_MODE_PER_LAYER, overrides={"tile": 4})
    names = [binding.ogc_mlp_kernel_name(d.mlp.plan, l) for l in range(3)]
    d.close()
    # (the last template argument: the requantizing epilogue with ReLU (1), GELU (4), no activation (3))
    assert names == ["ogc_layer_dma_kernel<3, 1, 1, 0, 1>", "ogc_layer_dma_kernel<3, 1, 0, 0, 4>", "ogc_layer_dma_kernel<3, 1, 0, 1, 3>"], names
    check_chain(oracle_mod, wl, "per_layer", tile=4)
    check_chain(oracle_mod, synth.make_mlp("f8", 16500, [512, 1024, 512], [RELU, RELU], seed=2201, name="stream-260-tiles"), "per_layer", tile=4)
    check_chain(oracle_mod, synth.make_mlp("f8", 300, [4096, 256, 2048], [RELU, NONE], seed=2202, has_bias=False, name="stream-long-k"),
                "per_layer", tile=4)
    check_chain(oracle_mod, synth.make_mlp("f8", 1, [64 * 4, 1], [NONE], seed=2203, name="stream-1x1"), "per_layer", tile=4)
    # ReLU-requantize epilogue into plain rows that are not whole 64-byte segments, and into a ragged last channel block
    check_chain(oracle_mod, synth.make_mlp("f8", 333, [256, 328, 200], [RELU, RELU], seed=2205, name="stream-relu-ragged"), "per_layer", tile=4)
    # the plan's own choice for a large layer is this kernel
    big = synth.make_mlp("f8", 8192, [1024, 1024, 1024], [RELU, RELU], seed=2204, has_bias=False, name="stream-auto")
    d = DeviceMLP(big, binding.OGC_MODE_AUTO)
    assert binding.ogc_mlp_kernel_name(d.mlp.plan, 1).startswith("ogc_layer_dma_kernel<3, 1,")
    d.close()
    check_chain(oracle_mod, big, "auto", layers_alone=False)


# ---------------------------------------------------------------- chains
@pytest.mark.parametrize("mode", ["per_layer", "fused", "coop", "auto"])
def test_chains_ragged(oracle_mod, mode):
    check_chain(oracle_mod, synth.make_mlp("f8", 77, [37, 130, 300, 9], [RELU, RELU, RELU], seed=1800, name="ragged"), mode)
    check_chain(oracle_mod, synth.make_mlp("f8", 700, [100, 333, 72, 33], [RELU, GELU, NONE], seed=1801, name="22-tiles"), mode)
    check_chain(oracle_mod, synth.make_mlp("f8", 256, [479, 1024, 1024, 512, 256, 1], [RELU] * 4 + [SIGM], seed=1802, last_f32=True,
                                           name="table-1 MLP-2 shape"), mode, layers_alone=(mode == "per_layer"))
    check_chain(oracle_mod, synth.make_mlp("f8", 50, [100, 48, 24], [RELU, RELU], seed=1803, ld_x=112), mode, ld_y=64)


@pytest.mark.parametrize("split", [2, 8, -4, -32])
def test_cluster_kernels(oracle_mod, split):
    ksplit, split = split < 0, abs(split)
    ov = {"cluster_split": split, "cluster_ksplit": 1 if ksplit else 0, "cluster_whole": 0}
    check_chain(oracle_mod, synth.make_mlp("f8", 270, [48, 64, 320, 64, 320, 16], [RELU] * 5, seed=1900, name="cluster-uneven-widths"), "coop",
                layers_alone=False, overrides=ov)
    check_chain(oracle_mod, synth.make_mlp("f8", 77, [37, 130, 300, 9], [RELU, GELU, RELU], seed=1901, name="cluster-ragged"), "coop",
                layers_alone=False, overrides=ov)


def test_wide_layers_per_layer_and_sixteen_layers(oracle_mod):
    check_chain(oracle_mod, synth.make_mlp("f8", 1000, [1024, 2048, 1024], [RELU, RELU], seed=2000, name="wide"), "per_layer")
    check_chain(oracle_mod, synth.make_mlp("f8", 70, [32] + [40, 24] * 8, [RELU] * 16, seed=2001, name="16-layers"), "auto", layers_alone=False)


def test_blocked_hand_off_between_two_chains(oracle_mod):
    import torch

    full = synth.make_mlp("f8", 333, [96, 200, 72, 130, 50, 21], [RELU] * 5, seed=2100, name="hand-off")
    ref = oracle_mod.mlp(full)
    to_dev = lambda a: torch.from_numpy(np.ascontiguousarray(a).view(np.uint8).reshape(-1).copy()).cuda()
    a = binding.FusedMLP("f8", full.m, full.layers[:3], mode=binding.OGC_MODE_AUTO, y_layout=binding.OGC_LAYOUT_BLOCKED)
    b = binding.FusedMLP("f8", full.m, full.layers[3:], mode=binding.OGC_MODE_AUTO, x_layout=binding.OGC_LAYOUT_BLOCKED)
    nbytes = binding.ogc_mlp_blocked_bytes(a.plan, 1)
    assert nbytes == binding.ogc_mlp_blocked_bytes(b.plan, 0) > 0
    for part, mlp in ((slice(0, 3), a), (slice(3, 5), b)):
        mlp.prepack([to_dev(w) for w in full.w[part]], [to_dev(v) for v in full.bias[part]], [to_dev(s) for s in full.w_scale[part]])
    x, mid = to_dev(full.x), torch.full((nbytes,), 0xCD, dtype=torch.uint8, device="cuda")
    y = torch.full((ref.nbytes,), 0xCD, dtype=torch.uint8, device="cuda")
    a.run(x, mid)
    b.run(mid, y)
    torch.cuda.synchronize()
    got = y.cpu().numpy().reshape(ref.shape)
    vg, vr = decode(oracle_mod, got), decode(oracle_mod, ref)
    assert (np.abs(vg - vr) <= 0.125 * np.abs(vr) + 6e-2 * np.abs(vr).max()).all() and (got != ref).mean() < 0.05
    a.close()
    b.close()


def test_description_checks():
    lay = lambda **kw: dict(dict(k=64, n=64, has_bias=1, act=1, in_scale=0.05, in_zp=0, out_scale=0.05, out_zp=0), **kw)
    ok = binding.ogc_mlp_plan(binding.OGC_F8, 64, [lay()], 64, 64, 0, binding.OGC_MODE_AUTO)
    binding.ogc_mlp_destroy(ok)
    for bad in (lay(in_zp=128), lay(out_zp=1), lay(in_scale=0.0), lay(out_scale=float("inf"))):
        with pytest.raises(binding.OgcError):
            binding.ogc_mlp_plan(binding.OGC_F8, 64, [bad], 64, 64, 0, binding.OGC_MODE_AUTO)
    with pytest.raises(binding.OgcError):    # the residual add belongs to the float dtypes
        binding.ogc_mlp_plan(binding.OGC_F8, 64, [lay()], 64, 64, 1, binding.OGC_MODE_AUTO)
