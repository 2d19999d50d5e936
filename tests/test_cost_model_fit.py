"""The per-layer cost model's constants are reproducible from the tree: the committed fitter run on the committed
measurements gives the constants the library compiles in (csrc/ogc_cost_layers.inc).  CPU only."""
import os
import re

import numpy as np

from paper_2301_01333_amd.calibration import fit_layers


def _tables_in_inc():
    text = open(fit_layers.INC).read()
    out = {}
    for name in ("kCostI8", "kCostBf16"):
        body = text[text.index("const CostTable %s" % name):]
        body = body[:body.index("};") + 2]
        nums = [float(x) for x in re.findall(r"(-?\d+\.\d+)f", body)]
        assert len(nums) == 5 * len(fit_layers.TILES) + 5, (name, len(nums))
        out[name] = np.array(nums)
    return out


def test_refit_reproduces_the_compiled_constants():
    rows = fit_layers.read_rows()
    assert len(rows) > 1500 and {r["tile"] for r in rows} == set(fit_layers.TILES)
    have = _tables_in_inc()
    for dtype, name in (("i8", "kCostI8"), ("bf16", "kCostBf16")):
        p, rms, geo, worst, n = fit_layers.fit(rows, dtype)
        assert rms < 0.10 and geo < 1.02 and worst < 1.4, (dtype, rms, geo, worst)
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
