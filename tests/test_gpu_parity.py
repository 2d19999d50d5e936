"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on the same seeded
inputs.  int8 results must be bit-exact; bf16 within 1e-2 and fp32 within 1e-5, relative, with the
absolute floor tied to the output magnitude: |gpu-ref| <= tol*|ref| + tol*max|ref|."""
import os

import numpy as np
import pytest

from paper_2301_01333_amd import binding, synth

pytestmark = pytest.mark.gpu

RELU, NONE, GELU, SIGM = synth.ACT_RELU, synth.ACT_NONE, synth.ACT_GELU_TANH, synth.ACT_SIGMOID
TOL = {"f32": 1e-5, "bf16": 1e-2}
MODES = {"fused": binding.OGC_MODE_FUSED, "per_layer": binding.OGC_MODE_PER_LAYER, "auto": binding.OGC_MODE_AUTO,
         "coop": binding.OGC_MODE_COOP}


def as_f32(wl, a):
    return synth.bf16_bits_to_f32(a) if a.dtype == np.uint16 else a.astype(np.float32)


def assert_close(got, ref, tol, what=""):
    got, ref = got.astype(np.float64), ref.astype(np.float64)
    assert np.isfinite(got).all(), what
    bound = tol * np.abs(ref) + tol * np.abs(ref).max()
    err = np.abs(got - ref)
    if not (err <= bound).all():
        i = int((err - bound).argmax())
        raise AssertionError("%s: %d of %d outside tolerance; worst at %s: got %g ref %g bound %g" % (
            what, int((err > bound).sum()), err.size, np.unravel_index(i, err.shape), got.flat[i], ref.flat[i], bound.flat[i]))


def run_gpu(wl, mode, tile=None, ksplit=None, **kw):
    """tile / ksplit: force the plan's tile configuration and the log2 of its split-K factor (plan overrides; both
    are otherwise chosen by the plan's cost model)."""
    from paper_2301_01333_amd.harness import DeviceMLP

    ov = dict(kw.pop("overrides", None) or {})
    if tile is not None:
        ov["tile"] = tile
    if ksplit is not None:
        ov["ksplit_log2"] = ksplit
    d = DeviceMLP(wl, MODES[mode], overrides=ov or None, **kw)
    d.run()
    y = d.result().copy()
    assert d.mlp.check() == binding.OGC_OK, "a barrier wait gave up"
    chosen = d.mlp.mode
    d.close()
    return y, chosen


def check(wl, mode, oracle_mod, tile=None, rows=None, ksplit=None, **kw):
    print("case:", wl.name, wl.dtype, "M=%d" % wl.m, wl.dims, "mode=%s tile=%s ksplit=%s" % (mode, tile, ksplit), kw, flush=True)
    got, _ = run_gpu(wl, mode, tile, ksplit, **kw)
    n = wl.layers[-1].n
    pad = got[:, n:]
    got = got[:, :n]
    if pad.size:
        assert (pad.view(np.uint8) == 0xCD).all(), "bytes beyond n_last in a strided y were touched"
    slices = rows or [slice(0, wl.m)]
    for sl in slices:
        ref = oracle_mod.mlp(wl, rows=sl)
        g = got[sl]
        if ref.dtype == np.uint8:
            if not np.array_equal(g, ref):
                bad = np.argwhere(g != ref)
                raise AssertionError("int8 mismatch: %d of %d differ; first at %s: got %d ref %d" % (
                    len(bad), ref.size, bad[0].tolist(), g[tuple(bad[0])], ref[tuple(bad[0])]))
        elif wl.dtype == "i8":
            assert_close(g, ref, 1e-5, "int8 chain, fp32 output")
        else:
            assert_close(as_f32(wl, g), as_f32(wl, ref), TOL[wl.dtype], "vs fp32-accumulate oracle")
            ref64 = oracle_mod.mlp(wl, rows=sl, accum_double=True)
            assert_close(as_f32(wl, g), as_f32(wl, ref64), TOL[wl.dtype], "vs fp64 oracle")
    return got


# ---------------------------------------------------------------- the five configurations, full size
@pytest.mark.parametrize("mode", ["auto", "per_layer"])
@pytest.mark.parametrize("cfg", [1, 2, 3])
def test_small_configs_full(oracle_mod, cfg, mode):
    check(synth.make_config(cfg), mode, oracle_mod)


@pytest.mark.parametrize("nl", [1, 2, 3, 4])
@pytest.mark.parametrize("mode", ["fused", "per_layer"])
def test_cfg3_u8_intermediates_bit_exact(oracle_mod, nl, mode):
    """The first nl layers of config 3 as a chain of their own: the requantized u8 tensor is the output."""
    full = synth.make_config(3)
    wl = synth.Workload("cfg3[:%d]" % nl, "i8", full.m, full.layers[:nl], False, full.x, full.w[:nl], full.bias[:nl],
                        full.w_scale[:nl], full.seed)
    got = check(wl, mode, oracle_mod)
    assert len(np.unique(got)) > 50   # not degenerate


def test_cfg4_full_size_every_row(oracle_mod):
    """All 4096 x 1024 outputs of the launch configuration the benchmark times (every tile, every k range)."""
    wl = synth.make_config(4)
    check(wl, "auto", oracle_mod)


def test_cfg5_full_size_every_row(oracle_mod):
    """All 32768 x 1024 bytes, bit-exact: every tile of the persistent kernel's walk, all four launches."""
    wl = synth.make_config(5)
    got = check(wl, "auto", oracle_mod)
    assert got.min() == 128 and got.max() == 255 and len(np.unique(got)) > 100


# ---------------------------------------------------------------- reduced sizes: several tiles + ragged tails
@pytest.mark.parametrize("tile", [0, 1, 2, 3, 4, 5])
@pytest.mark.parametrize("dtype", ["i8", "bf16", "f32"])
def test_per_layer_ragged(oracle_mod, dtype, tile):
    m = {0: 300, 1: 150, 2: 77, 3: 600, 4: 700, 5: 333}[tile]
    dims = [100, 333, 72, 33] if dtype == "i8" else [50, 290, 40, 19]
    wl = synth.make_mlp(dtype, m, dims, [RELU, RELU, NONE if dtype != "i8" else RELU], seed=500 + tile, name="ragged")
    check(wl, "per_layer", oracle_mod, tile=tile)


@pytest.mark.parametrize("dtype", ["i8", "bf16", "f32"])
def test_fused_ragged(oracle_mod, dtype):
    wl = synth.make_mlp(dtype, 77, [37, 130, 300, 9], [RELU, GELU if dtype != "i8" else RELU, RELU], seed=600, name="ragged")
    check(wl, "fused", oracle_mod)


@pytest.mark.parametrize("mode", ["fused", "per_layer"])
def test_reduced_cfg4_and_cfg5(oracle_mod, mode):
    check(synth.make_config(4, m=160), "per_layer", oracle_mod, tile=1)   # hidden 4096 does not fit the fused kernel
    check(synth.make_config(5, m=96), mode, oracle_mod)


@pytest.mark.parametrize("tile", [3, 4, 5])
@pytest.mark.parametrize("dtype", ["i8", "bf16", "f32"])
def test_pipelined_kernel_plain_input(oracle_mod, dtype, tile):
    """Tiles 3, 4 and 5 = the three shapes of the persistent global->LDS stream kernel (fp32 falls back to the
    register-staged kernel; tile 5, whose stages hold two k-steps, falls back where a layer has an odd number of them), reading the caller's plain x directly (aligned rows, no K padding), with a ragged
    batch, short and long K, several tiles per workgroup, and a misaligned x that must fall back."""
    k = {"i8": 192, "bf16": 96, "f32": 64}[dtype]
    if tile == 5:
        k *= 2   # an even number of 64-byte k-steps in the first layer: the shape under test really runs it
    wl = synth.make_mlp(dtype, 700, [k, 160, 64, 40], [RELU, RELU, RELU], seed=700, name="dma")
    check(wl, "per_layer", oracle_mod, tile=tile)
    check(synth.make_mlp(dtype, 300, [64, 200], [RELU], seed=701, name="dma-1layer"), "per_layer", oracle_mod, tile=tile)
    check(synth.make_mlp(dtype, 257, [1024, 96], [NONE], seed=702, name="dma-longk", has_bias=False), "per_layer", oracle_mod, tile=tile)
    # more tiles than resident workgroups: every workgroup walks several tiles (stream across tile boundaries)
    check(synth.make_mlp(dtype, 9000, [k, 520, 300], [RELU, GELU if dtype != "i8" else RELU], seed=705, name="dma-many-tiles"),
          "per_layer", oracle_mod, tile=tile)
    esz = {"i8": 1, "bf16": 2, "f32": 4}[dtype]
    check(synth.make_mlp(dtype, 300, [64, 200], [RELU], seed=703, name="dma-misaligned"), "per_layer", oracle_mod, tile=tile,
          x_byte_offset=esz)
    check(synth.make_mlp(dtype, 300, [64, 70], [RELU], seed=704, name="dma-strided", ld_x=80), "per_layer", oracle_mod, tile=tile,
          ld_y=72)


def test_clocked_run(oracle_mod):
    """The diagnostic run that has every workgroup of the stream kernel record the wall clock and the shader cycle
    counter: same result as an ordinary run, one record per workgroup of each stream-kernel launch, none for the other
    kernels, clocks that advance, and a cycle counter rate in the range of this part's shader clock."""
    from paper_2301_01333_amd.harness import DeviceMLP

    wl = synth.make_config(5, m=4096)
    d = DeviceMLP(wl, binding.OGC_MODE_PER_LAYER, overrides={"tile": 4})
    d.run()
    want = d.result().copy()
    c = d.run_clocked()
    got = d.result().copy()
    assert np.array_equal(got, want) and np.array_equal(got[:, :wl.layers[-1].n], oracle_mod.mlp(wl))
    assert c.shape[0] == 4
    for l in range(4):
        assert binding.ogc_mlp_kernel_name(d.mlp.plan, l).startswith("ogc_layer_dma_kernel")
        rec = c[l][c[l][:, 2] != 0]
        assert len(rec) == 64, len(rec)   # 16 x 4 tiles of 256 x 256: one workgroup each
        assert (rec[:, 2] > rec[:, 0]).all() and (rec[:, 3] > rec[:, 1]).all()
        mhz = (rec[:, 3] - rec[:, 1]) / ((rec[:, 2] - rec[:, 0]) / 100.0)
        assert 300.0 < mhz.mean() < 3000.0, mhz.mean()
    d.close()
    # a chain that runs no stream kernel records nothing
    d = DeviceMLP(synth.make_config(5, m=96), binding.OGC_MODE_PER_LAYER, overrides={"tile": 1})
    c = d.run_clocked()
    assert (c == 0).all()
    d.close()
    with pytest.raises(binding.OgcError):
        binding.ogc_mlp_run_clocked(0, 0, 0, 0, 0, 0)


@pytest.mark.parametrize("tile", [3, 4])
def test_stream_kernel_requantizing_epilogues(oracle_mod, tile):
    """Int8 layers without activation and with GELU on the stream kernel, each with an epilogue of its own (last template
    argument 3 / 4; 1 is ReLU's): blocked and plain results, whole 64-byte row segments and ragged ones, several tiles
    per workgroup.  Without activation the result is the oracle's bit for bit.  With GELU the requantized byte is decided
    by a transcendental function that the kernel evaluates with the hardware's exp2 and reciprocal (about an ulp of fp32
    each) and the oracle with libm: a byte may differ by one where y / c_s lies within that error of a rounding boundary,
    which a few values in a million do."""
    from paper_2301_01333_amd.harness import DeviceMLP

    wl = synth.make_mlp("i8", 700, [256, 512, 320, 128], [NONE, RELU, NONE], seed=760, name="stream-none")
    d = DeviceMLP(wl, binding.OGC_MODE_PER_LAYER, overrides={"tile": tile})
    names = [binding.ogc_mlp_kernel_name(d.mlp.plan, l) for l in range(3)]
    d.close()
    shape = tile - 3
    assert names == ["ogc_layer_dma_kernel<2, %d, 1, 0, 3>" % shape, "ogc_layer_dma_kernel<2, %d, 0, 0, 1>" % shape,
                     "ogc_layer_dma_kernel<2, %d, 0, 1, 3>" % shape], names
    check(wl, "per_layer", oracle_mod, tile=tile)
    check(synth.make_mlp("i8", 9000, [192, 520, 300], [NONE, NONE], seed=761, name="stream-none-many-tiles"), "per_layer", oracle_mod, tile=tile)
    check(synth.make_mlp("i8", 333, [256, 328, 200], [NONE, NONE], seed=762, name="stream-none-ragged"), "per_layer", oracle_mod, tile=tile, ld_y=208)
    for dims, seed in (([256, 512, 320, 128], 763), ([192, 520, 300], 764)):
        wl = synth.make_mlp("i8", 2100, dims, [GELU] * (len(dims) - 1), seed=seed, name="stream-gelu")
        d = DeviceMLP(wl, binding.OGC_MODE_PER_LAYER, overrides={"tile": tile})
        assert binding.ogc_mlp_kernel_name(d.mlp.plan, 0) == "ogc_layer_dma_kernel<2, %d, 1, 0, 4>" % shape
        d.close()
        got, _ = run_gpu(wl, "per_layer", tile)
        ref = oracle_mod.mlp(wl)
        diff = np.abs(got[:, :ref.shape[1]].astype(np.int32) - ref.astype(np.int32))
        # (a moved byte of one layer moves the next layer's sums: the chain as a whole is held to one step and a small share)
        assert diff.max() <= 1 and (diff > 0).mean() < 2e-3, (int(diff.max()), float((diff > 0).mean()))
        print("stream-gelu", dims, "bytes that differ by one: %.2e" % (diff > 0).mean(), flush=True)


@pytest.mark.parametrize("tile", [3, 4])
@pytest.mark.parametrize("dtype", ["i8", "bf16"])
def test_split_k(oracle_mod, dtype, tile):
    """The reduction axis cut into 2, 4 and 8 ranges (partial accumulators + the reduction pass that owns the
    epilogue): middle layers (blocked output) and the last layer (plain output, ragged N and M), int8 bit-exact."""
    k = {"i8": 512, "bf16": 256}[dtype]   # 8 k-steps of 64 bytes
    for ls in (1, 2, 3):
        wl = synth.make_mlp(dtype, 300, [k, 2 * k, 72], [RELU, RELU if dtype == "i8" else GELU], seed=720 + ls, name="split-k")
        check(wl, "per_layer", oracle_mod, tile=tile, ksplit=ls)
    wl = synth.make_mlp(dtype, 700, [k, 200], [NONE if dtype != "i8" else RELU], seed=724, name="split-k-1layer", has_bias=False)
    check(wl, "per_layer", oracle_mod, tile=tile, ksplit=2)
    if dtype == "bf16":  # residual + bias in the reduction pass
        check(synth.make_config(4, m=300), "per_layer", oracle_mod, tile=tile, ksplit=2)


@pytest.mark.parametrize("dtype", ["i8", "bf16"])
def test_cost_model_choices(oracle_mod, dtype):
    """Per-layer chains whose tiles and splits the plan's cost model picks by itself: long reduction axes at small
    batch (four-wave stream tile cut along K), mid-size layers (small register-staged tile), a ragged batch that
    fills the chip (eight-wave tile).  int8 bit-exact against the oracle."""
    for m, dims, seed in ((256, [256, 8192, 256, 512], 731), (500, [1024, 4096, 1024], 732), (1536, [768, 3072, 768], 733),
                          (2048, [1024, 1024, 1024], 734), (96, [2048, 2048, 320], 735), (16500, [512, 1024, 512], 736)):
        acts = [RELU] * (len(dims) - 1)
        wl = synth.make_mlp(dtype, m, dims, acts, seed=seed, name="model-chosen", has_bias=(seed % 2 == 0))
        check(wl, "per_layer", oracle_mod)


# ---------------------------------------------------------------- edge cases
@pytest.mark.parametrize("mode", ["fused", "per_layer"])
def test_edges_int8(oracle_mod, mode):
    # single row, single output channel, K = 1
    check(synth.make_mlp("i8", 1, [1, 1], [RELU], seed=1), mode, oracle_mod)
    # zero points away from 128 (compensation path), weights including -128, unpadded K
    check(synth.make_mlp("i8", 33, [479, 65, 31], [RELU, RELU], seed=2, a_z=3, c_z=200, wq_lo=-128), mode, oracle_mod)
    check(synth.make_mlp("i8", 40, [64, 64], [NONE], seed=3, a_z=0, c_z=0, wq_lo=-128), mode, oracle_mod)
    check(synth.make_mlp("i8", 40, [64, 64], [RELU], seed=4, a_z=255, c_z=255), mode, oracle_mod)
    # fp32 result straight from the first layer; sigmoid and no activation
    check(synth.make_mlp("i8", 19, [70, 5], [SIGM], seed=5, last_f32=True), mode, oracle_mod)
    check(synth.make_mlp("i8", 19, [70, 5], [NONE], seed=6, last_f32=True, has_bias=False), mode, oracle_mod)
    # strided x and y, x not 16-byte aligned
    check(synth.make_mlp("i8", 50, [100, 48], [RELU], seed=7, ld_x=112), mode, oracle_mod, ld_y=64)
    check(synth.make_mlp("i8", 50, [96, 48], [RELU], seed=8), mode, oracle_mod, x_byte_offset=3)
    # saturation on both ends: tiny output scale
    wl = synth.make_mlp("i8", 20, [128, 40], [NONE], seed=9)
    wl.layers[0].out_scale = wl.layers[0].out_scale / 50.0
    got = check(wl, mode, oracle_mod)
    assert (got == 0).any() and (got == 255).any()


@pytest.mark.parametrize("mode", ["fused", "per_layer"])
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_edges_float(oracle_mod, dtype, mode):
    check(synth.make_mlp(dtype, 1, [1, 1], [NONE], seed=11), mode, oracle_mod)
    check(synth.make_mlp(dtype, 3, [13, 1], [SIGM], seed=12), mode, oracle_mod)
    check(synth.make_mlp(dtype, 70, [40, 64, 40], [GELU, NONE], seed=13, residual=True), mode, oracle_mod)
    check(synth.make_mlp(dtype, 50, [24, 36], [RELU], seed=14, ld_x=40, has_bias=False), mode, oracle_mod, ld_y=52)
    esz = 4 if dtype == "f32" else 2
    check(synth.make_mlp(dtype, 50, [32, 32], [RELU], seed=15), mode, oracle_mod, x_byte_offset=esz)


def test_zero_and_identity_weights(oracle_mod):
    wl = synth.make_mlp("i8", 64, [64, 64], [RELU], seed=21)
    wl.w[0][:] = 0
    got = check(wl, "per_layer", oracle_mod)
    assert (got == got[0]).all()          # every row equals requant(ReLU(bias)), whatever x is
    wl = synth.make_mlp("i8", 64, [64, 64], [RELU], seed=22, has_bias=False)
    wl.w[0][:] = np.eye(64, dtype=np.int8)
    wl.w_scale[0][:] = 1.0
    wl.layers[0].in_scale = wl.layers[0].out_scale = 0.25
    got = check(wl, "fused", oracle_mod)
    assert np.array_equal(got, np.maximum(wl.x, 128))


def test_run_is_repeatable_and_workspace_is_stateless(oracle_mod):
    from paper_2301_01333_amd.harness import DeviceMLP

    wl = synth.make_config(5, m=512)
    d = DeviceMLP(wl, binding.OGC_MODE_PER_LAYER)
    d.run()
    a = d.result().copy()
    d.mlp.workspace.fill_(0x5A)
    d.y.fill_(0)
    for _ in range(3):
        d.run()
    b = d.result().copy()
    d.close()
    assert np.array_equal(a, b)
    assert np.array_equal(a, oracle_mod.mlp(wl))


def test_run_before_prepack_is_refused():
    import torch

    m = binding.FusedMLP("f32", 4, [dict(k=4, n=4)], mode=binding.OGC_MODE_AUTO)
    x = torch.zeros(16, device="cuda")
    with pytest.raises(binding.OgcError) as e:
        binding.ogc_mlp_run(m.plan, x.data_ptr(), x.data_ptr(), x.data_ptr(), 0, 0)
    assert e.value.status == -6
    m.close()


# ---------------------------------------------------------------- limits and seeded random shapes
def test_int8_longest_reduction_axis_with_extreme_values(oracle_mod):
    """K = 65536, the longest int8 reduction axis the plan accepts, with every activation 255 and every weight
    127 (and -128): the exact sums reach 65536*255*127 = 2 122 383 360, just inside int32."""
    k = 65536
    wl = synth.make_mlp("i8", 40, [k, 33], [RELU], seed=31, has_bias=False, a_z=0, c_z=0)
    wl.x[:] = 255
    wl.w[0][:, :17] = 127
    wl.w[0][:, 17:] = -128
    for ly in wl.layers:
        ly.out_scale = float(np.float32(k * 255 * 127 * ly.in_scale * 0.02 / 200.0))  # keeps part of the range unsaturated
    got = check(wl, "per_layer", oracle_mod)
    assert (got[:, 17:] == 0).all()          # ReLU of the most negative sums
    # the same through the stream kernel (needs zero point 128), whole and cut into eight k ranges
    wl3 = synth.make_mlp("i8", 40, [k, 33], [RELU], seed=31, has_bias=False)
    wl3.x[:] = 255
    wl3.w[0][:, :17] = 127
    wl3.w[0][:, 17:] = -128
    wl3.layers[0].out_scale = float(np.float32(k * 127 * 127 * wl3.layers[0].in_scale * 0.02 / 120.0))
    check(wl3, "per_layer", oracle_mod, tile=4)
    check(wl3, "per_layer", oracle_mod, tile=4, ksplit=3)
    wl2 = synth.make_mlp("i8", 40, [k, 33], [NONE], seed=32, has_bias=False, last_f32=True)
    check(wl2, "per_layer", oracle_mod)


def test_sixteen_layers(oracle_mod):
    """The longest chain the descriptor allows, in both modes (ping-pong slots reused eight times)."""
    for dtype in ("i8", "bf16", "f32"):
        dims = [48, 64, 32, 96, 64, 32, 64, 96, 32, 64, 48, 64, 32, 64, 96, 32, 24]
        wl = synth.make_mlp(dtype, 70, dims, [RELU] * 16, seed=40, name="16-layers")
        check(wl, "fused", oracle_mod)
        check(wl, "per_layer", oracle_mod)


@pytest.mark.parametrize("dtype", ["i8", "bf16", "f32"])
def test_seeded_random_chains(oracle_mod, dtype):
    """Twelve chains per dtype with seeded random depth, widths, batch, activations, bias, strides and mode."""
    rng = np.random.default_rng({"i8": 9001, "bf16": 9002, "f32": 9003}[dtype])
    for case in range(12):
        nl = int(rng.integers(1, 5))
        dims = [int(rng.integers(1, 300)) for _ in range(nl + 1)]
        m = int(rng.integers(1, 400))
        acts = [int(rng.choice([RELU, NONE] if dtype == "i8" else [RELU, NONE, GELU])) for _ in range(nl)]
        if dtype == "i8":
            acts = [RELU if a == NONE and i + 1 < nl else a for i, a in enumerate(acts)]
        kw = dict(has_bias=bool(rng.integers(0, 2)))
        if dtype == "i8":
            kw.update(a_z=int(rng.choice([128, 128, 0, 77])), c_z=int(rng.choice([128, 128, 0, 200])))
        ld_x = dims[0] + int(rng.integers(0, 9)) * int(rng.integers(0, 2))
        wl = synth.make_mlp(dtype, m, dims, acts, seed=9100 + case, name="random-%d" % case, ld_x=ld_x, **kw)
        mode = str(rng.choice(["fused", "per_layer", "auto"]))
        tile = None if mode != "per_layer" else int(rng.integers(0, 5))
        check(wl, mode, oracle_mod, tile=tile, ld_y=dims[-1] + int(rng.integers(0, 5)))


@pytest.mark.parametrize("dtype", ["i8", "bf16", "f32"])
def test_blocked_hand_off_between_two_chains(oracle_mod, dtype):
    """Layout propagation across calls (Section V): chain A emits its y in the blocked operand layout, chain B
    takes that buffer as its x; together they must equal the one five-layer chain the oracle computes.  Ragged
    M, K and N; with the stream kernels (tile 4) and with the heuristic's choice."""
    import torch

    full = synth.make_mlp(dtype, 333, [96, 200, 72, 130, 50, 21], [RELU, RELU, RELU, GELU if dtype != "i8" else RELU, NONE if dtype != "i8" else RELU],
                          seed=800, name="hand-off")
    ref = oracle_mod.mlp(full)
    to_dev = lambda a: torch.from_numpy(np.ascontiguousarray(a).view(np.uint8).reshape(-1).copy()).cuda()
    for tile in (None, 4):
        ov = None if tile is None else {"tile": tile}
        a = binding.FusedMLP(dtype, full.m, full.layers[:3], mode=binding.OGC_MODE_AUTO, y_layout=binding.OGC_LAYOUT_BLOCKED, overrides=ov)
        b = binding.FusedMLP(dtype, full.m, full.layers[3:], mode=binding.OGC_MODE_AUTO, x_layout=binding.OGC_LAYOUT_BLOCKED, overrides=ov)
        assert a.mode == binding.OGC_MODE_PER_LAYER and b.mode == binding.OGC_MODE_PER_LAYER
        nbytes = binding.ogc_mlp_blocked_bytes(a.plan, 1)
        assert nbytes == binding.ogc_mlp_blocked_bytes(b.plan, 0) > 0
        assert binding.ogc_mlp_blocked_bytes(a.plan, 0) == 0 and binding.ogc_mlp_blocked_bytes(b.plan, 1) == 0
        for part, mlp in ((slice(0, 3), a), (slice(3, 5), b)):
            ws = None if dtype != "i8" else [to_dev(s) for s in full.w_scale[part]]
            mlp.prepack([to_dev(w) for w in full.w[part]], [None if v is None else to_dev(v) for v in full.bias[part]], ws)
        x = to_dev(full.x)
        mid = torch.full((nbytes,), 0xCD, dtype=torch.uint8, device="cuda")
        y = torch.full((ref.nbytes,), 0xCD, dtype=torch.uint8, device="cuda")
        a.run(x, mid)
        b.run(mid, y)
        torch.cuda.synchronize()
        got = y.cpu().numpy().view(ref.dtype).reshape(ref.shape)
        if dtype == "i8":
            assert np.array_equal(got, ref)
        else:
            assert_close(as_f32(full, got), as_f32(full, ref), TOL[dtype], "two chains with a blocked hand-off")
        a.close()
        b.close()
    with pytest.raises(binding.OgcError):   # the fused-chain kernel does not take blocked tensors
        binding.FusedMLP(dtype, 64, full.layers[:2], mode=binding.OGC_MODE_FUSED, y_layout=binding.OGC_LAYOUT_BLOCKED)


# ---------------------------------------------------------------- cooperative small-batch kernel
@pytest.mark.parametrize("cfg", [1, 2, 3])
def test_coop_small_configs_full(oracle_mod, cfg):
    check(synth.make_config(cfg), "coop", oracle_mod)


@pytest.mark.parametrize("dtype", ["i8", "bf16", "f32"])
def test_coop_ragged_and_edges(oracle_mod, dtype):
    """One cooperative launch for the chain: output blocks spread over all CUs, the reduction axis split between
    the waves of a workgroup, a device-wide barrier between layers.  Ragged M / K / N, more blocks than CUs,
    a single block, every post-op, strided and misaligned x."""
    act2 = GELU if dtype != "i8" else RELU
    check(synth.make_mlp(dtype, 77, [37, 130, 300, 9], [RELU, act2, RELU], seed=600, name="coop-ragged"), "coop", oracle_mod)
    check(synth.make_mlp(dtype, 700, [100, 333, 72, 33], [RELU, RELU, NONE if dtype != "i8" else RELU], seed=601, name="coop-many-blocks"),
          "coop", oracle_mod)
    check(synth.make_mlp(dtype, 1, [1, 1], [NONE if dtype != "i8" else RELU], seed=602, name="coop-1x1"), "coop", oracle_mod)
    check(synth.make_mlp(dtype, 50, [100, 48], [RELU], seed=603, ld_x=112), "coop", oracle_mod, ld_y=64)
    esz = {"i8": 1, "bf16": 2, "f32": 4}[dtype]
    check(synth.make_mlp(dtype, 50, [96, 48, 40], [RELU, RELU], seed=604), "coop", oracle_mod, x_byte_offset=esz)
    dims = [48, 64, 32, 96, 64, 32, 64, 96, 32, 64, 48, 64, 32, 64, 96, 32, 24]
    check(synth.make_mlp(dtype, 70, dims, [RELU] * 16, seed=40, name="coop-16-layers"), "coop", oracle_mod)
    if dtype == "i8":
        check(synth.make_mlp("i8", 33, [479, 65, 31], [RELU, RELU], seed=2, a_z=3, c_z=200, wq_lo=-128), "coop", oracle_mod)
        check(synth.make_mlp("i8", 19, [70, 64, 5], [RELU, SIGM], seed=5, last_f32=True), "coop", oracle_mod)
    else:
        check(synth.make_mlp(dtype, 70, [40, 64, 40], [GELU, NONE], seed=13, residual=True), "coop", oracle_mod)
        check(synth.make_mlp(dtype, 3, [13, 7, 1], [RELU, SIGM], seed=12), "coop", oracle_mod)


def test_coop_runs_back_to_back(oracle_mod):
    """The barrier counters live in the packed blob and are reset by the last workgroup of each run: many runs
    in a row, on one stream, keep giving the same (correct) result."""
    from paper_2301_01333_amd.harness import DeviceMLP

    wl = synth.make_config(3)
    ref = oracle_mod.mlp(wl)
    d = DeviceMLP(wl, binding.OGC_MODE_COOP)
    assert d.mlp.mode == binding.OGC_MODE_COOP
    for _ in range(25):
        d.run()
    first = d.result().copy()
    assert_close(first[:, :1], ref, 1e-5, "config 3, cooperative kernel")
    for _ in range(3):
        d.y.fill_(0xCD)
        for _ in range(7):
            d.run()
        assert np.array_equal(d.result(), first)
    d.close()


@pytest.mark.parametrize("ov", [{"cluster_split": 0}, {"cluster_split": 4, "cluster_ksplit": 0, "cluster_whole": 0}, {"cluster_split": 8, "cluster_ksplit": 1}])
def test_barrier_that_gives_up_is_reported(oracle_mod, ov):
    """The bounded barrier wait of the cooperative kernels: forced from the host to give up (a tiny poll budget and a
    target one arrival beyond what will ever come, so every workgroup leaves at its first barrier and the kernel ends
    normally), the run must be reported by ogc_mlp_check and by ogc_mlp_run_profiled, once; afterwards the same plan
    and blob run correctly again, and a normal run reports nothing."""
    from paper_2301_01333_amd.harness import DeviceMLP

    wl = synth.make_mlp("i8", 200, [100, 333, 72, 33], [RELU, RELU, RELU], seed=601, name="give-up")
    d = DeviceMLP(wl, binding.OGC_MODE_COOP, overrides=ov)
    ref = oracle_mod.mlp(wl)
    d.run()
    assert d.mlp.check() == binding.OGC_OK and np.array_equal(d.result(), ref)
    binding.ogc_mlp_test_barrier(d.mlp.plan, 50, 1)
    print("forcing the barriers to give up:", binding.ogc_mlp_kernel_name(d.mlp.plan, 0), flush=True)
    d.run()
    assert d.mlp.check() == binding.OGC_ERR_TIMEOUT
    assert d.mlp.check() == binding.OGC_OK            # reported once
    with pytest.raises(binding.OgcError) as e:
        d.run_profiled()
    assert e.value.status == binding.OGC_ERR_TIMEOUT
    binding.ogc_mlp_test_barrier(d.mlp.plan, 1 << 22, 0)
    d.y.fill_(0xCD)
    d.run()
    assert d.mlp.check() == binding.OGC_OK and np.array_equal(d.result(), ref)
    d.close()


# ---------------------------------------------------------------- cluster kernel (a few workgroups per row tile)
@pytest.mark.parametrize("split", [0, 2, 4, 8, -2, -8, -32])
@pytest.mark.parametrize("dtype", ["f32", "bf16", "i8"])
def test_cluster_kernel_ragged_and_edges(oracle_mod, dtype, split):
    """The cooperative mode's second kernel: `split` workgroups share a 32-row tile, each computes every split-th
    group of channel blocks, and the tile travels through the workspace between layers.  The cluster_split override
    forces the split (0: the block-dealing kernel; negative here: the variant whose waves split K inside a member,
    forced with cluster_ksplit), so every variant is checked against the oracle on every dtype.  The exchange is forced
    after every layer too (cluster_whole = 0), and layer widths differ, so that tiles sharing a workspace slot would
    collide if their regions were not private."""
    ksplit, split = split < 0, abs(split)   # negative: the variant whose waves split K inside a member
    ov = {"cluster_split": split, "cluster_ksplit": 1 if ksplit else 0}
    act2 = GELU if dtype != "i8" else RELU
    wl = synth.make_mlp(dtype, 77, [37, 130, 300, 9], [RELU, act2, RELU], seed=600, name="cluster-ragged")
    from paper_2301_01333_amd.harness import DeviceMLP

    d = DeviceMLP(wl, binding.OGC_MODE_COOP, overrides=ov)
    want = "ogc_cluster_ksplit_chain_kernel" if ksplit else "ogc_cluster_chain_kernel" if split else "ogc_coop_chain_kernel"
    assert binding.ogc_mlp_kernel_name(d.mlp.plan, 0).startswith(want)
    d.close()
    check(wl, "coop", oracle_mod, overrides=ov)
    check(synth.make_mlp(dtype, 700, [100, 333, 72, 33], [RELU, RELU, NONE if dtype != "i8" else RELU], seed=601, name="cluster-22-tiles"),
          "coop", oracle_mod, overrides=ov)
    check(synth.make_mlp(dtype, 1, [1, 1], [NONE if dtype != "i8" else RELU], seed=602, name="cluster-1x1"), "coop", oracle_mod, overrides=ov)
    check(synth.make_mlp(dtype, 50, [100, 48, 24], [RELU, RELU], seed=603, ld_x=112), "coop", oracle_mod, ld_y=64, overrides=ov)
    check(synth.make_mlp(dtype, 70, [32] + [40, 24] * 8, [RELU] * 16, seed=40, name="cluster-16-layers"), "coop", oracle_mod, overrides=ov)
    if split:   # every layer exchanged, widths 64 / 320 / 64 / 320 sharing two slots over 9 row tiles
        check(synth.make_mlp(dtype, 270, [48, 64, 320, 64, 320, 16], [RELU] * 5, seed=41, name="cluster-uneven-widths"), "coop", oracle_mod,
              overrides=dict(ov, cluster_whole=0))
    if dtype == "i8":
        check(synth.make_mlp("i8", 33, [479, 65, 31], [RELU, RELU], seed=2, a_z=3, c_z=200, wq_lo=-128), "coop", oracle_mod, overrides=ov)
        check(synth.make_mlp("i8", 19, [70, 64, 5], [RELU, SIGM], seed=5, last_f32=True), "coop", oracle_mod, overrides=ov)
    else:
        check(synth.make_mlp(dtype, 70, [40, 64, 40], [GELU, NONE], seed=13, residual=True), "coop", oracle_mod, overrides=ov)


@pytest.mark.parametrize("dtype,m,split", [("i8", 256, 4), ("i8", 520, 8), ("bf16", 200, 4), ("bf16", 64, 16), ("i8", 2048, 4),
                                           ("f32", 512, -16), ("f32", 200, -32), ("i8", 256, -32), ("bf16", 1024, -8)])
def test_cluster_kernel_table1_mlp2(oracle_mod, dtype, m, split):
    """Table I's MLP-2 through the cluster kernel: int8 weights fit one XCD's L2 (a tile's members share an XCD), the
    bf16 weights do not (members on different XCDs); many runs in a row keep giving the first run's result (each
    tile's members reset their counters at the end of a run)."""
    from paper_2301_01333_amd.harness import DeviceMLP

    ov = {"cluster_split": abs(split), "cluster_ksplit": 1 if split < 0 else 0}   # negative: the k-split variant (fp32 rows of
    dims = [479, 1024, 1024, 512, 256, 1]                                          # 1024 values fit only its single LDS buffer)
    acts = [RELU] * 4 + [SIGM if dtype == "i8" else NONE]
    wl = synth.make_mlp(dtype, m, dims, acts, seed=77, last_f32=(dtype == "i8"), name="cluster-mlp2")
    d = DeviceMLP(wl, binding.OGC_MODE_COOP, overrides=ov)
    assert binding.ogc_mlp_kernel_name(d.mlp.plan, 0).startswith("ogc_cluster_ksplit_chain_kernel" if split < 0 else "ogc_cluster_chain_kernel")
    d.run()
    first = d.result().copy()
    rows = slice(0, m) if m <= 520 else slice(m - 300, m)
    ref = oracle_mod.mlp(wl, rows=rows)
    if dtype == "i8":
        assert_close(first[rows, :1], ref, 1e-5, "MLP-2 int8, cluster kernel")
    else:
        assert_close(as_f32(wl, first[rows, :1]), as_f32(wl, ref), TOL[dtype], "MLP-2 %s, cluster kernel" % dtype)
    for _ in range(3):
        d.y.fill_(0xCD)
        for _ in range(9):
            d.run()
        assert np.array_equal(d.result().view(np.uint8), first.view(np.uint8))
    d.close()


@pytest.mark.parametrize("idx,mode", [(1, "fused"), (3, "fused"), (2, "coop"), (3, "auto"), (5, "per_layer")])
def test_runs_recorded_in_a_hip_graph_replay_correctly(oracle_mod, idx, mode):
    """ogc_mlp_run under stream capture: the graph is replayed several times with eager work and synchronisations
    in between, and every replay must reproduce the eager result (the library records kernels only, no memsets)."""
    import torch

    from paper_2301_01333_amd.harness import DeviceMLP

    wl = synth.make_config(idx, m={1: 32, 2: 128, 3: 256, 5: 512}[idx])
    dev = DeviceMLP(wl, MODES[mode])
    dev.run()
    eager = dev.result().copy()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        dev.run()
        dev.run()
    for rep in range(3):
        dev.y.fill_(0xCD)
        torch.cuda.synchronize()
        graph.replay()
        got = dev.result().copy()
        assert np.array_equal(got.view(np.uint8), eager.view(np.uint8)), "replay %d differs from the eager run" % rep
        dev.run()                       # eager work between the replays
        torch.cuda.synchronize()
    dev.close()
