"""Calibration sweep behind the plan's chain-mode cost models (fused-chain kernel, cooperative kernel, the two cluster
kernels): times whole chains on the GPU in every single-launch mode, each forced through the plan's mode argument and
overrides, and writes one CSV row per (chain, batch, kernel, split).

    python -m paper_2301_01333_amd.calibration.sweep_chains [out.csv]      (needs the MI355X; a few minutes)

`fit_chains.py` turns the CSV into the constants compiled into the library.  Columns: dtype, dims (layer widths joined
by 'x'), m, kind (fused | coop | cluster | ksplit), split (members per row tile, 0 where it does not apply), whole
(bit l set: the cluster kernel computed layer l whole in every member, as the plan decided), us (mean of 50
back-to-back calls, host clock around a synchronize: what a caller sees).  Seeded synthetic tensors; the values do
not matter for the timing.
"""
from __future__ import annotations

import csv
import os
import sys
import time

HERE = os.path.dirname(os.path.abspath(__file__))
DEFAULT_OUT = os.path.join(HERE, "data", "chain_times.csv")

CHAINS = [[13, 512, 256, 128], [479, 1024, 1024, 512, 256, 1], [2048] * 4, [1024, 4096, 1024], [512] * 5, [256] * 4, [1024] * 3,
          [128, 2048, 128], [768, 768, 768], [256, 1024, 256, 1024, 256], [64, 64, 64, 64], [1536, 384, 1536]]
BATCHES = (32, 64, 128, 256, 512, 1024, 2048, 4096, 8192, 16384)


def main(out_path: str = DEFAULT_OUT) -> None:
    sys.path.insert(0, os.path.dirname(os.path.dirname(HERE)))
    import torch

    from paper_2301_01333_amd import binding, synth
    from paper_2301_01333_amd.harness import DeviceMLP

    def timed(wl, mode, overrides, want):
        """Mean microseconds per call, or None if the plan refuses the mode or answers with another kernel."""
        try:
            d = DeviceMLP(wl, mode, overrides=overrides)
        except binding.OgcError:
            return None, 0
        name = binding.ogc_mlp_kernel_name(d.mlp.plan, 0)
        if d.mlp.mode != mode or not name.startswith(want):
            d.close()
            return None, 0
        whole = binding.ogc_mlp_cluster_layout(d.mlp.plan)[2] if mode == binding.OGC_MODE_COOP else 0
        for _ in range(8):
            d.run()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(50):
            d.run()
        torch.cuda.synchronize()
        us = (time.perf_counter() - t0) / 50 * 1e6
        assert d.mlp.check() == binding.OGC_OK
        d.close()
        return us, whole

    rows = 0
    with open(out_path, "w", newline="") as f:
        w = csv.writer(f)
        w.writerow(["dtype", "dims", "m", "kind", "split", "whole", "us"])
        for dtype in ("f32", "bf16", "i8"):
            for dims in CHAINS:
                for m in BATCHES:
                    if m * max(dims) * 4 > (1 << 27):
                        continue
                    nl = len(dims) - 1
                    acts = [synth.ACT_RELU] * nl
                    kw = {}
                    if dims[-1] == 1:
                        acts[-1] = synth.ACT_SIGMOID if dtype == "i8" else synth.ACT_NONE
                        kw = dict(last_f32=True) if dtype == "i8" else {}
                    wl = synth.make_mlp(dtype, m, dims, acts, seed=7, has_bias=True, **kw)
                    cases = [("fused", 0, binding.OGC_MODE_FUSED, None, "ogc_fused_chain_kernel"),
                             ("coop", 0, binding.OGC_MODE_COOP, {"cluster_split": 0}, "ogc_coop_chain_kernel")]
                    if m <= 2048:
                        cases += [("cluster", s, binding.OGC_MODE_COOP, {"cluster_split": s, "cluster_ksplit": 0}, "ogc_cluster_chain_kernel")
                                  for s in (2, 4, 8, 16)]
                        cases += [("ksplit", s, binding.OGC_MODE_COOP, {"cluster_split": s, "cluster_ksplit": 1}, "ogc_cluster_ksplit_chain_kernel")
                                  for s in (2, 4, 8, 16, 32)]
                    for kind, split, mode, ov, want in cases:
                        us, whole = timed(wl, mode, ov, want)
                        if us is not None:
                            w.writerow([dtype, "x".join(str(v) for v in dims), m, kind, split, whole, "%.3f" % us])
                            rows += 1
                f.flush()
                print("done", dtype, dims, rows, "rows", flush=True)


if __name__ == "__main__":
    main(sys.argv[1] if len(sys.argv) > 1 else DEFAULT_OUT)
