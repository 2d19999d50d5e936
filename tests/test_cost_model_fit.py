"""The plan's cost-model constants are reproducible from the tree: the committed fitters run on the committed
measurements give the constants the library compiles in (csrc/ogc_cost_layers.inc, csrc/ogc_cost_chains.inc).  CPU only."""
import os
import re

import numpy as np

from paper_2301_01333_amd.calibration import fit_chains, fit_layers


def _tables_in_inc():
    text = open(fit_layers.INC).read()
    out = {}
    for name, tiles_of in (("kCostI8", fit_layers.TILES), ("kCostBf16", fit_layers.TILES), ("kCostF32", fit_layers.TILES_F32)):
        body = text[text.index("const CostTable %s" % name):]
        body = body[:body.index("};") + 2]
        rows = re.findall(r"\{([^{}]*)\}", body)
        assert len(rows) == fit_layers.NUM_TILES, (name, len(rows))
        nums = []
        for t in tiles_of:
            vals = [float(x.rstrip("f")) for x in rows[t].split(",")]
            assert len(vals) == 5
            nums += vals
        for t in range(fit_layers.NUM_TILES):
            if t not in tiles_of:
                assert [float(x.rstrip("f")) for x in rows[t].split(",")] == [0.0] * 5
        tail = body[body.rindex("}},") + 3:body.index("};")]
        nums += [float(x.strip().rstrip("f")) for x in tail.split(",") if x.strip()]
        assert len(nums) == 5 * len(tiles_of) + 5, (name, len(nums))
        out[name] = np.array(nums)
    return out


def test_refit_reproduces_the_compiled_constants():
    rows = fit_layers.read_rows()
    assert len(rows) > 1500 and {r["tile"] for r in rows} == set(fit_layers.TILES) | set(fit_layers.TILES_F32)
    have = _tables_in_inc()
    for dtype, name in (("i8", "kCostI8"), ("bf16", "kCostBf16"), ("f32", "kCostF32")):
        p, rms, geo, worst, n = fit_layers.fit(rows, dtype)
        p = np.where(p > 1e-8, p, 0.0)
        assert rms < 0.13 and geo < 1.02 and worst < 1.4, (dtype, rms, geo, worst)
        # the same constants up to the last printed digits and the optimiser's stopping tolerance
        assert np.allclose(p, have[name], rtol=2e-2, atol=2e-3), (dtype, np.abs(p - have[name]).max())


def test_model_function_matches_the_library(tmp_path):
    """fit_layers.model is the formula of estimate_layer_us: the library's estimate for a forced candidate equals the
    Python model evaluated with the compiled constants."""
    from paper_2301_01333_amd import binding as b

    have = _tables_in_inc()
    cases = [("i8", 32768, 1024, 1024, 4, 0), ("bf16", 4096, 4096, 1024, 5, 0), ("bf16", 4096, 4096, 1024, 3, 1),
             ("i8", 256, 8192, 256, 3, 2), ("i8", 2048, 1024, 1024, 2, 0), ("bf16", 512, 1024, 4096, 1, 0)]
    for dtype, m, k, n, tile, ks in cases:
        esz = 1 if dtype == "i8" else 2
        lay = [dict(k=k, n=k, has_bias=0, act=1, in_scale=0.05, in_zp=128, out_scale=0.05, out_zp=128),
               dict(k=k, n=n, has_bias=0, act=1, in_scale=0.05, in_zp=128, out_scale=0.05, out_zp=128),
               dict(k=n, n=n, has_bias=0, act=1, in_scale=0.05, in_zp=128, out_scale=0.05, out_zp=128)]
        p = b.ogc_mlp_plan_with_overrides(b.DTYPES[dtype], m, lay, k, n, 0, b.OGC_MODE_PER_LAYER, overrides={"tile": tile, "ksplit_log2": ks})
        got = b.ogc_mlp_estimated_us(p, 1)
        b.ogc_mlp_destroy(p)
        # the middle layer's rows are the next layer's padded input width
        gran = 64 if dtype == "i8" else 32
        rows = (n + gran - 1) // gran * gran
        want = fit_layers.model(have["kCostI8" if dtype == "i8" else "kCostBf16"],
                                dict(m=m, n=rows, tile=tile, ks=ks, kt=(k * esz + 63) // 64))
        assert abs(got - want) <= 1e-3 * want, (dtype, m, k, n, tile, ks, got, want)


def _chain_tables_in_inc():
    text = open(fit_chains.INC).read()
    out = {}
    for kind, (_, p0, _, _, struct, name) in fit_chains.MODELS.items():
        body = text[text.index("const %s %s[3]" % (struct, name)):]
        body = body[:body.index("};") + 2]
        rows = re.findall(r"\{([^{}]*)\}", body)
        assert len(rows) == 3
        out[kind] = [np.array([float(x.strip().rstrip("f")) for x in r.split(",")]) for r in rows]
        assert all(len(v) == len(p0) for v in out[kind])
    return out


def test_chain_models_refit_reproduces_the_compiled_constants():
    rows = fit_chains.read_rows()
    assert len(rows) > 2000 and {r["kind"] for r in rows} == set(fit_chains.MODELS)
    have = _chain_tables_in_inc()
    for kind in fit_chains.MODELS:
        for i, dtype in enumerate(fit_chains.DTYPES):
            p, rms, worst, n = fit_chains.fit(rows, kind, dtype)
            assert n >= 30 and rms < 0.15, (kind, dtype, n, rms)
            model = fit_chains.MODELS[kind][0]
            # the compiled constants predict every timed chain as the refit does (the parameters themselves can trade
            # against each other where the data do not separate them, so the predictions are what is compared)
            rs = [r for r in rows if r["kind"] == kind and r["dtype"] == dtype and fit_chains.usable(r)]
            a = np.array([model(p, r) for r in rs])
            b = np.array([model(have[kind][i], r) for r in rs])
            assert np.allclose(a, b, rtol=2e-2), (kind, dtype, np.abs(a / b - 1).max())


def test_chain_model_functions_match_the_library():
    """fit_chains' formulas are the library's: ogc_mlp_mode_estimates on a forced plan equals the Python model evaluated
    with the compiled constants."""
    from paper_2301_01333_amd import binding as b
    from paper_2301_01333_amd import synth

    have = _chain_tables_in_inc()
    for dtype, dims, m in (("i8", [479, 1024, 1024, 512, 256, 1], 256), ("bf16", [13, 512, 256, 128, 64], 128), ("f32", [64, 64, 64, 64], 512),
                           ("bf16", [256, 1024, 256, 1024, 256], 1024)):
        i = fit_chains.DTYPES.index(dtype)
        lay = [dict(k=k, n=n, has_bias=1, act=1, in_scale=0.05, in_zp=128, out_scale=0.05, out_zp=128) for k, n in zip(dims[:-1], dims[1:])]
        base = dict(dtype=dtype, dims=dims, m=m, split=0, whole=0)
        p = b.ogc_mlp_plan_with_overrides(b.DTYPES[dtype], m, lay, dims[0], dims[-1], 0, b.OGC_MODE_AUTO, overrides={"cluster_split": 0})
        est = b.ogc_mlp_mode_estimates(p)      # per-layer, fused, cooperative
        b.ogc_mlp_destroy(p)
        if est[1] >= 0:
            assert abs(est[1] - fit_chains.fused_model(have["fused"][i], base)) <= 1e-3 * est[1]
        assert abs(est[2] - fit_chains.coop_model(have["coop"][i], base)) <= 1e-3 * est[2]
        for kind, ks, model in (("cluster", 0, fit_chains.cluster_model), ("ksplit", 1, fit_chains.ksplit_model)):
            p = b.ogc_mlp_plan_with_overrides(b.DTYPES[dtype], m, lay, dims[0], dims[-1], 0, b.OGC_MODE_COOP,
                                              overrides={"cluster_split": 4, "cluster_ksplit": ks})
            members, is_ks, whole, _ = b.ogc_mlp_cluster_layout(p)
            est = b.ogc_mlp_mode_estimates(p)
            b.ogc_mlp_destroy(p)
            if members != 4 or is_ks != ks:
                continue
            want = model(have[kind][i], dict(base, split=4, whole=whole))
            assert abs(est[2] - want) <= 1e-3 * want, (kind, dtype, dims, est[2], want)
