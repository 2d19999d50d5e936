"""Calibration sweep behind the plan's per-layer cost model (int8, bf16 and fp32): times the MIDDLE layer of three-layer
chains on the GPU for every candidate the plan can choose (tile configuration, number of k ranges), forced through
the plan overrides, and writes one CSV row per launch configuration.

    python -m paper_2301_01333_amd.calibration.sweep_layers [out.csv]      (needs the MI355X; about five minutes)

`fit_layers.py` turns the CSV into the constants compiled into the library.  Columns: dtype, m, k, n (the middle
layer's shape), tile, ks (log2 of the k ranges), us (median of 15 event-timed launches, both launches of a split
layer), kernel (the first kernel's name).  Seeded synthetic tensors; the values do not matter for the timing.
"""
from __future__ import annotations

import csv
import os
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
DEFAULT_OUT = os.path.join(HERE, "data", "layer_times.csv")

CHAINS = {"A": [1024] * 4, "B": [1024, 4096, 1024, 4096], "C": [512] * 4, "D": [2048] * 4, "E": [256, 8192, 256, 8192],
          "F": [768, 3072, 768, 3072], "G": [1536] * 4, "H": [384] * 4, "I": [3072, 768, 3072, 768]}
BATCHES = (32, 64, 128, 256, 512, 1024, 2048, 4096, 8192, 16384, 32768)
CANDIDATES = ((2, 0), (1, 0), (3, 0), (4, 0), (5, 0), (3, 1), (4, 1), (3, 2), (4, 2), (3, 3), (4, 3))
CANDIDATES_F32 = ((2, 0), (1, 0), (0, 0))   # fp32 runs on the register-staged tiles only


def main(out_path: str = DEFAULT_OUT) -> None:
    sys.path.insert(0, os.path.dirname(os.path.dirname(HERE)))
    from paper_2301_01333_amd import binding, synth
    from paper_2301_01333_amd.harness import DeviceMLP

    def median(v):
        v = sorted(v)
        return v[len(v) // 2]

    rows = 0
    with open(out_path, "w", newline="") as f:
        w = csv.writer(f)
        w.writerow(["dtype", "m", "k", "n", "tile", "ks", "us", "kernel"])
        for dtype in ("i8", "bf16", "f32"):
            esz = {"i8": 1, "bf16": 2, "f32": 4}[dtype]
            for cname, dims in CHAINS.items():
                for m in BATCHES:
                    if m * max(dims) * esz > (1 << 28):
                        continue
                    wl = synth.make_mlp(dtype, m, dims, [synth.ACT_RELU] * 3, seed=5, has_bias=False)
                    kt = dims[1] * esz // 64
                    for tile, ks in (CANDIDATES_F32 if dtype == "f32" else CANDIDATES):
                        if tile == 2 and m > 1600:               # thousands of 64 x 32 tiles: never a candidate worth timing
                            continue
                        if ks and (kt % (1 << ks) or (kt >> ks) < 4):
                            continue
                        if tile == 5 and kt % 2:
                            continue
                        try:
                            d = DeviceMLP(wl, binding.OGC_MODE_PER_LAYER, overrides={"tile": tile, "ksplit_log2": ks})
                        except binding.OgcError as e:
                            print("skip", dtype, cname, m, tile, ks, e, flush=True)
                            continue
                        name = binding.ogc_mlp_kernel_name(d.mlp.plan, 1)
                        for _ in range(3):
                            d.run_profiled()
                        us = median([d.run_profiled()[1] for _ in range(15)]) * 1e3
                        d.close()
                        w.writerow([dtype, m, dims[1], dims[2], tile, ks, "%.3f" % us, name])
                        rows += 1
                f.flush()
                print("done", dtype, cname, rows, "rows", flush=True)


if __name__ == "__main__":
    main(sys.argv[1] if len(sys.argv) > 1 else DEFAULT_OUT)
