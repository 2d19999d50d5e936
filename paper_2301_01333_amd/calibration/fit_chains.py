"""Fits the constants of the plan's chain-mode cost models (csrc/ogc_api.cpp: estimate_fused_us, estimate_coop_us,
estimate_cluster_us, estimate_cluster_ksplit_us) to the chains timed by sweep_chains.py and writes them as the C++
tables the library compiles in (csrc/ogc_cost_chains.inc).

    python -m paper_2301_01333_amd.calibration.fit_chains            (CPU only; about a minute)

Every model is a sum over the chain's layers of a weight-stream term and fixed per-layer / per-barrier terms,
stretched by a fill factor as the chip fills up; the formulas below are the ones in ogc_api.cpp, term for term.
Least squares on log(model / measured), one fit per kernel and dtype.
"""
from __future__ import annotations

import csv
import math
import os
import sys

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
CSV = os.path.join(HERE, "data", "chain_times.csv")
INC = os.path.join(os.path.dirname(HERE), "csrc", "ogc_cost_chains.inc")
ESZ = {"f32": 4, "bf16": 2, "i8": 1}
DTYPES = ("f32", "bf16", "i8")     # the order of ogc_dtype: the tables are indexed by it


def read_rows(path: str = CSV):
    out = []
    with open(path) as f:
        for r in csv.DictReader(f):
            out.append(dict(dtype=r["dtype"], dims=[int(v) for v in r["dims"].split("x")], m=int(r["m"]), kind=r["kind"],
                            split=int(r["split"]), whole=int(r["whole"]), us=float(r["us"])))
    return out


def layers(r):
    """Per layer: (padded input row bytes, 32-channel blocks written, is last), as the plan sizes them."""
    e, g = ESZ[r["dtype"]], (64 if r["dtype"] == "i8" else 32)
    dims, out = r["dims"], []
    for i, (k, n) in enumerate(zip(dims[:-1], dims[1:])):
        kp = -(-k // g) * g
        last = i == len(dims) - 2
        nb = -(-n // 32) if last else (-(-n // g) * g) // 32
        out.append((kp * e, nb, last, n))
    return out


def fused_model(p, r):
    f0, per_mb, per_layer, fill, per_block = p
    rounds = max(1.0, r["m"] / 8192.0)
    s = sum(per_mb * kb * nb * 32 / 1e6 + per_layer + per_block * ((nb + 7) // 8) for kb, nb, _, _ in layers(r))
    return f0 + rounds * s * (1 + fill * min(1.0, r["m"] / 8192.0))


def coop_model(p, r):
    c0, barrier, block, step, fill = p
    ls, mb = layers(r), -(-r["m"] // 32)
    blocks = [mb * (-(-n // 32)) for _, _, _, n in ls]
    g = min(256, max(blocks))
    t = c0
    for (kb, _, _, _), bl in zip(ls, blocks):
        rounds = 0.5 * (math.ceil(bl / g) + bl / g)
        t += barrier + rounds * (block + step * kb / 32.0)
    return t * (1 + fill * min(1.0, max(blocks) / 256.0))


def cluster_layer(p, ls, i, split, whole):
    c0, per_mb, group, per_layer, barrier, copy_mb, fill, all_mb = p
    kb, nb, last, _ = ls[i]
    waves, stride = 8 * (1 if whole else split), (1 if whole else split)
    wg = sum(-(-(nb - w * stride) // waves) for w in range(8) if w * stride < nb)
    per_wave = -(-nb // waves)
    t = per_mb * kb * 32 * wg / 1e6 + group * math.ceil(kb / 128.0) * ((per_wave + 3) // 4) + per_layer
    if not last and not whole:
        t += barrier + copy_mb * ls[i + 1][0] * 32 / 1e6
    return t


def cluster_model(p, r):
    c0, per_mb, group, per_layer, barrier, copy_mb, fill, all_mb = p
    ls, tiles, s = layers(r), -(-r["m"] // 32), r["split"]
    t, wtot = c0, 0.0
    for i, (kb, nb, last, _) in enumerate(ls):
        whole = bool((r["whole"] >> i) & 1)     # the plan's decision when the chain was timed
        t += cluster_layer(p, ls, i, s, whole)
        wtot += kb * nb * 32 / 1e6 * (s if whole else 1)
    return t * (1 + fill * min(1.0, tiles * s / 256.0)) + all_mb * tiles * wtot


def ksplit_model(p, r):
    c0, block, step, barrier, copy_mb, fill, all_mb = p
    ls, tiles, s = layers(r), -(-r["m"] // 32), r["split"]
    t, wtot = c0, 0.0
    for i, (kb, nb, last, _) in enumerate(ls):
        t += -(-nb // s) * (block + step * kb / 256.0)
        if not last:
            t += barrier + copy_mb * ls[i + 1][0] * 32 / 1e6
        wtot += kb * nb * 32 / 1e6
    return t * (1 + fill * min(1.0, tiles * s / 256.0)) + all_mb * tiles * wtot


# kind -> (model, start, lower bounds, upper bounds, C++ struct, table name)
INF = float("inf")
MODELS = {
    "fused": (fused_model, [6, 10, 0.5, 0.1, 0.1], [0] * 5, [INF] * 5, "FusedCost", "kFused"),
    "coop": (coop_model, [8, 3.5, 1.0, 0.05, 0.1], [0] * 5, [INF] * 5, "CoopCost", "kCoop"),
    # the barrier of a tile's members is held between 1 and 3 us: left free, the fit trades it against the copy term
    "cluster": (cluster_model, [6, 10, 0.05, 0.3, 2.0, 20, 0.1, 0.05], [0, 0, 0, 0, 1.0, 0, 0, 0], [INF, INF, INF, INF, 3.0, 80.0, INF, INF],
                "ClusterCost", "kCluster"),
    "ksplit": (ksplit_model, [6, 1, 0.05, 2.3, 20, 0.1, 0.02], [0, 0, 0, 1.0, 0, 0, 0], [INF, INF, INF, 3.5, 60, INF, INF], "KsplitCost", "kKsplit"),
}


def usable(r):
    """The fused kernel's model is fitted where the plan offers it: float chains whose weights fit the L2 share."""
    if r["kind"] != "fused" or r["dtype"] == "i8":
        return True
    return sum(kb * nb * 32 for kb, nb, _, _ in layers(r)) <= 2.6e6


def fit(rows, kind: str, dtype: str):
    """Returns (parameters, rms log error, worst log error, number of chains)."""
    from scipy.optimize import least_squares

    model, p0, lo, hi, _, _ = MODELS[kind]
    rs = [r for r in rows if r["kind"] == kind and r["dtype"] == dtype and usable(r)]
    y = np.array([r["us"] for r in rs])

    def res(p):
        return np.array([math.log(max(model(p, r), 1e-3) / yy) for r, yy in zip(rs, y)])

    sol = least_squares(res, np.array(p0, float), bounds=(lo, hi))
    e = res(sol.x)
    return sol.x, float(np.sqrt((e ** 2).mean())), float(np.abs(e).max()), len(rs)


def main() -> None:
    rows = read_rows()
    text = ("// Written by paper_2301_01333_amd/calibration/fit_chains.py from calibration/data/chain_times.csv; do not edit.\n"
            "// One row per dtype in the order of ogc_dtype (fp32, bf16, int8); fields as in the structs of ogc_api.cpp.\n")
    for kind in ("fused", "coop", "cluster", "ksplit"):
        _, _, _, _, struct, name = MODELS[kind]
        body = []
        for dtype in DTYPES:
            p, rms, worst, n = fit(rows, kind, dtype)
            print("%-7s %-4s %4d chains, rms log error %.3f, worst %.3f" % (kind, dtype, n, rms, worst), np.round(p, 4).tolist(), flush=True)
            text += "// %s %s: %d chains, rms log error %.3f, worst %.3f\n" % (kind, dtype, n, rms, worst)
            body.append("{" + ", ".join("%.4ff" % v for v in p) + "}")
        text += "const %s %s[3] = {%s};\n" % (struct, name, ",\n    ".join(body))
    if "--check" in sys.argv:
        print(text)
        return
    with open(INC, "w") as f:
        f.write(text)
    print("wrote", INC)


if __name__ == "__main__":
    main()
