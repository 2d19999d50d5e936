"""Fits the constants of the plan's per-layer cost model (csrc/ogc_api.cpp, estimate_layer_us) to the launches
timed by sweep_layers.py and writes them as the C++ tables the library compiles in (csrc/ogc_cost_layers.inc).

    python -m paper_2301_01333_amd.calibration.fit_layers            (CPU only; a few seconds)

Model, in microseconds, for a candidate (tile, 2^ks k ranges) on a layer of m rows, n channels, kt k-steps of 64 bytes:

    W      = tiles * 2^ks workgroups, k = kt >> ks steps each
    lone   = (c + d*k) * (1 + g*min(1, W/256))
    stream = l0 + rounds * (a + b*k [+ px if split]),  rounds = (ceil(W/256) + W/256) / 2
    t      = max(lone, stream) [+ r0 + r2*2^ks + r1*(2^ks + 1)*Mp*Np*4 bytes/1e6 if split]

c, d, a, b, g per tile; r0, r1, r2, px, l0 per dtype.  Least squares on log(model / measured); candidates within 25 % of
a shape's fastest weigh double (what matters is which candidate the model ranks first, not the slow ones' times).
"""
from __future__ import annotations

import collections
import csv
import math
import os
import sys

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
CSV = os.path.join(HERE, "data", "layer_times.csv")
INC = os.path.join(os.path.dirname(HERE), "csrc", "ogc_cost_layers.inc")
GEO = {0: (256, 256), 1: (128, 128), 2: (32, 64), 3: (256, 128), 4: (256, 256), 5: (128, 128)}   # tile id -> (rows, channels)
TILES = (1, 2, 3, 4, 5)          # candidates of int8 and bf16 layers
TILES_F32 = (0, 1, 2)            # fp32 runs on the register-staged tiles only, never split
NUM_TILES = 6
NEAR_BEST_WEIGHT = 2.0


def read_rows(path: str = CSV):
    out = []
    with open(path) as f:
        for r in csv.DictReader(f):
            esz = {"i8": 1, "bf16": 2, "f32": 4}[r["dtype"]]
            out.append(dict(dtype=r["dtype"], m=int(r["m"]), k=int(r["k"]), n=int(r["n"]), tile=int(r["tile"]), ks=int(r["ks"]),
                            us=float(r["us"]), kt=(int(r["k"]) * esz + 63) // 64))
    return out


def model(p, r, tiles_of=TILES) -> float:
    i = tiles_of.index(r["tile"])
    c, d, a, b, g = p[5 * i:5 * i + 5]
    r0, r1, r2, px, l0 = p[5 * len(tiles_of):5 * len(tiles_of) + 5]
    bm, bn = GEO[r["tile"]]
    tiles = math.ceil(r["m"] / bm) * math.ceil(r["n"] / bn)
    w, k = tiles << r["ks"], r["kt"] >> r["ks"]
    lone = (c + d * k) * (1.0 + g * min(1.0, w / 256.0))
    rounds = 0.5 * (math.ceil(w / 256.0) + w / 256.0)
    t = max(lone, l0 + rounds * (a + b * k + (px if r["ks"] else 0.0)))
    if r["ks"]:
        mp, np_ = math.ceil(r["m"] / 256) * 256, math.ceil(r["n"] / 256) * 256
        t += r0 + r2 * (1 << r["ks"]) + r1 * ((1 << r["ks"]) + 1) * mp * np_ * 4 / 1e6
    return t


def fit(rows, dtype: str):
    """Returns (parameter vector, rms log error, geometric-mean loss of the model's pick against the fastest measured)."""
    from scipy.optimize import least_squares

    tiles_of = TILES_F32 if dtype == "f32" else TILES
    rs = [r for r in rows if r["dtype"] == dtype and r["tile"] in tiles_of]
    y = np.array([r["us"] for r in rs])
    best = collections.defaultdict(lambda: 1e30)
    for r in rs:
        key = (r["m"], r["k"], r["n"])
        best[key] = min(best[key], r["us"])
    wts = np.array([NEAR_BEST_WEIGHT if r["us"] <= 1.25 * best[(r["m"], r["k"], r["n"])] else 1.0 for r in rs])

    def res(p):
        return wts * np.array([math.log(model(p, r, tiles_of) / yy) for r, yy in zip(rs, y)])

    if dtype == "f32":
        p0 = np.array([10, 2.0, 8, 3.0, 0.2, 7, 1.0, 3, 1.0, 0.2, 5, 0.5, 0.5, 0.2, 0.1, 0, 0, 0, 0, 1.0])
        hi = np.array([np.inf] * 15 + [1e-9, 1e-9, 1e-9, 1e-9, np.inf])   # no split: the pass over the partials has no data
    else:
        p0 = np.array([6.8, 0.45, 2.1, 0.36, 0.18, 5.0, 0.3, 0.3, 0.05, 0.2, 7.5, 0.28, 0.5, 0.6, 0.35, 10.0, 0.46, 8.0, 0.73, 0.3,
                       8.0, 0.3, 3.0, 0.3, 0.3, 1.0, 0.16, 1.0, 2.3, 1.0])
        hi = np.full(p0.shape, np.inf)
    sol = least_squares(res, p0, bounds=(0, hi))
    e = res(sol.x) / wts
    groups = collections.defaultdict(list)
    for r in rs:
        groups[(r["m"], r["k"], r["n"])].append((model(sol.x, r, tiles_of), r["us"]))
    loss = [min(v)[1] / min(u for _, u in v) for v in groups.values()]
    return sol.x, float(np.sqrt((e ** 2).mean())), float(np.exp(np.mean(np.log(loss)))), float(max(loss)), len(rs)


def table_text(name: str, p, tiles_of=TILES) -> str:
    rows = ["{0, 0, 0, 0, 0}"] * NUM_TILES   # a tile that is not a candidate for the dtype keeps a zero row
    for i, t in enumerate(tiles_of):
        rows[t] = "{" + ", ".join("%.4ff" % v for v in p[5 * i:5 * i + 5]) + "}"
    g = [max(v, 0.0) if v > 1e-8 else 0.0 for v in p[5 * len(tiles_of):]]
    return "const CostTable %s = {{%s},\n    %s};\n" % (name, ",\n    ".join(rows), ", ".join("%.4ff" % v for v in g))


def main() -> None:
    rows = read_rows()
    text = ("// Written by paper_2301_01333_amd/calibration/fit_layers.py from calibration/data/layer_times.csv; do not edit.\n"
            "// Per tile {c, d, a, b, g}, indexed by tile id; then r0, r1, r2, px, l0 (see estimate_layer_us).\n")
    for dtype, name in (("i8", "kCostI8"), ("bf16", "kCostBf16"), ("f32", "kCostF32")):
        p, rms, geo, worst, n = fit(rows, dtype)
        print("%s: %d launches, rms log error %.3f, the model's pick is %.3fx the fastest measured (geometric mean), worst %.2fx"
              % (dtype, n, rms, geo, worst))
        text += "// %s: %d launches, rms log error %.3f, pick / fastest %.3f (geometric mean), worst %.2f\n" % (dtype, n, rms, geo, worst)
        text += table_text(name, p, TILES_F32 if dtype == "f32" else TILES)
    if "--check" in sys.argv:
        print(text)
        return
    with open(INC, "w") as f:
        f.write(text)
    print("wrote", INC)


if __name__ == "__main__":
    main()
