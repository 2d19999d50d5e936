#!/usr/bin/env python3
"""Benchmark of the fused-MLP hot path on one MI355X.

`python bench.py --gpus 1 --steps K --warmup W` prints ONE JSON line.  A step is one pass of the whole
hot path (input staging, every layer's MFMA main loop + register epilogue, inter-layer hand-off, final
store: one ogc_mlp_run call) over one batch of seeded synthetic input that is already resident in HBM.
The headline workload is configuration 5 (int8, M=32768, 4 x 1024->1024, ReLU + requantize), the largest
single-GPU configuration; the other four are reported under "per_config".  The roofline object is for the
dominant kernel of the headline workload, timed live with HIP events around every launch; cpu_baseline is
the CPU oracle timed on a bounded sample of the same workload on this machine's host cores.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK = {"i8": (5.0e15, "TOP/s"), "bf16": (2.5e15, "TFLOP/s"), "f32": (157.3e12, "TFLOP/s"), "f8": (5.0e15, "TFLOP/s")}
HBM_PEAK = 8.0e12
METRIC = "fused-MLP TFLOPS/TOPS + fraction of MFMA or HBM roofline, per config"
MODE_NAMES = {1: "per_layer", 2: "fused", 3: "coop"}


def _median(v):
    s = sorted(v)
    return s[len(s) // 2]


def time_steps(dev, steps, warmup):
    """Time of exactly `steps` runs: wall clock synchronised on both sides, and a HIP event pair recorded on
    the launch stream around the same region.  Returns (wall seconds per step, event seconds per step)."""
    import torch

    # The chip's clock comes up from idle over tens of milliseconds of load: whatever `warmup` is,
    # the untimed part lasts at least 50 ms, so that the timed steps run at the clock a loop of such steps settles at.
    t_end = time.perf_counter() + 0.05
    while time.perf_counter() < t_end:
        for _ in range(20):
            dev.run()
        torch.cuda.synchronize()
    for _ in range(warmup):
        dev.run()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    e0.record()
    for _ in range(steps):
        dev.run()
    e1.record()
    torch.cuda.synchronize()
    wall = (time.perf_counter() - t0) / steps
    return wall, e0.elapsed_time(e1) * 1e-3 / steps


def clock_report(dev, launch_idxs, work, peak, reps=20):
    """The clock the chip actually gives the dominant kernel: diagnostic runs in which every workgroup stores the 100 MHz
    wall clock and the shader cycle counter at its start and end (ogc_mlp_run_clocked), repeated back to back after the
    timed region so that the chip is in the same state.  `peak` assumes 2.4 GHz; `mfma_cycles` is the work at the
    matrix pipes' full rate (2048 int8 or 1024 bf16 operations per clock and SIMD), so `matrix_pipe_utilisation` = mfma_cycles /
    cycles_per_launch is the kernel's efficiency in cycles, whatever the clock, and peak_at_clock what 100 % of it
    would give at that clock."""
    import numpy as np

    for _ in range(100):
        dev.run()
    mhz, cycles, alive = [], [], []
    for _ in range(reps):
        c = dev.run_clocked()
        for j in launch_idxs:
            w = c[j][c[j][:, 2] != 0]
            if not len(w):
                continue
            dt_us = (w[:, 2] - w[:, 0]) / 100.0
            dc = (w[:, 3] - w[:, 1]).astype(np.float64)
            mhz.append(float((dc / dt_us).mean()))
            cycles.append(float(dc.mean()))
            alive.append(float(dt_us.mean()))
    if not mhz:
        return None
    # operations per clock of one SIMD's matrix pipe (the published peaks are these x 1024 SIMDs x 2.4 GHz, rounded)
    ops_per_clock_per_simd = {5.0e15: 2048.0, 2.5e15: 1024.0, 157.3e12: 64.0}[peak]
    mfma_cycles = work / 1024.0 / ops_per_clock_per_simd
    m, cyc = sum(mhz) / len(mhz), sum(cycles) / len(cycles)
    return {"shader_mhz": round(m, 1), "cycles_per_launch": round(cyc), "workgroup_alive_us": round(sum(alive) / len(alive), 2),
            "mfma_cycles": round(mfma_cycles), "matrix_pipe_utilisation": round(mfma_cycles / cyc, 4),
            "peak_at_clock": round(peak * m / 2400.0 / 1e12, 1)}


def time_graph_replay(dev, runs_per_graph=50, replays=6):
    """The same runs recorded once into a HIP graph (stream capture of `runs_per_graph` calls) and replayed: what a
    caller whose loop is bound by the launch path of the host gets.  Returns seconds per run."""
    import torch

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        dev.run()                      # plan-time work (kernel attributes) happens outside the capture
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        for _ in range(runs_per_graph):
            dev.run()                  # the launches go to the capturing stream (torch's current stream)
    graph.replay()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(replays):
        graph.replay()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) / (replays * runs_per_graph)


def time_cold(dev, reps=9):
    """One run at a time with the caches flushed before it (a 512 MiB fill goes through L2 and the memory-side
    cache first): median of HIP-event times around the single call.  Returns seconds."""
    import torch

    junk = torch.empty(512 << 20, dtype=torch.uint8, device="cuda")
    times = []
    for i in range(reps):
        junk.fill_(i)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        dev.run()
        e1.record()
        torch.cuda.synchronize()
        times.append(e0.elapsed_time(e1) * 1e-3)
    del junk
    return _median(times)


def profile_launches(dev, reps=30):
    """Per-launch durations (seconds), median over reps, from HIP events recorded around every launch."""
    dev.run_profiled()
    rows = [dev.run_profiled() for _ in range(reps)]
    n = len(rows[0])
    return [_median([r[i] for r in rows]) * 1e-3 for i in range(n)]


def config_report(idx, steps, warmup, with_floor=None):
    from paper_2301_01333_amd import binding, synth
    from paper_2301_01333_amd.harness import DeviceMLP

    wl = synth.make_config(idx)
    dev = DeviceMLP(wl)
    sec, ev_sec = time_steps(dev, steps, warmup)
    launches = profile_launches(dev)
    nl = binding.ogc_mlp_num_launches(dev.mlp.plan)
    peak, unit = PEAK[wl.dtype]
    ops, abytes = wl.ops, wl.algorithmic_bytes
    ridge = peak / HBM_PEAK
    bound = "mfma" if ops / abytes > ridge else "hbm"
    rep = {
        "config": idx, "workload": wl.name, "dtype": wl.dtype, "mode": MODE_NAMES[dev.mlp.mode],
        "kernels": sorted({binding.ogc_mlp_kernel_name(dev.mlp.plan, j) for j in range(nl)}),
        "launches": nl, "ms_per_step": sec * 1e3, "ms_per_step_hip_events": ev_sec * 1e3,
        "ms_sum_of_per_launch_event_pairs": sum(launches) * 1e3,
        "tops_or_tflops": ops / sec / 1e12, "algorithmic_GBps": abytes / sec / 1e9, "bound": bound,
        "frac_of_bound": (ops / sec / peak) if bound == "mfma" else (abytes / sec / HBM_PEAK),
        "ops": ops, "algorithmic_bytes": abytes,
    }
    if bound == "mfma" and rep["mode"] == "per_layer":
        # the clock each launch really ran at, and its efficiency in cycles (see clock_report)
        rep["clock_per_launch"] = [clock_report(dev, [j], 2.0 * wl.m * wl.layers[j].k * wl.layers[j].n, peak, reps=8) for j in range(nl)]
    if with_floor is not None:
        rep["launch_floor_ms"] = with_floor * 1e3
        rep["frac_of_latency_aware_bound"] = (with_floor + abytes / HBM_PEAK) / sec
        # the small configurations are bound by the host's launch path: the same calls replayed from a HIP graph
        g = time_graph_replay(dev)
        rep["ms_per_step_hip_graph_replay"] = g * 1e3
        rep["algorithmic_GBps_hip_graph_replay"] = abytes / g / 1e9
        rep["ms_per_step_cold_caches"] = time_cold(dev) * 1e3   # weights and input come from HBM
    return wl, dev, rep, launches


def launch_floor(steps, warmup):
    """Per-call time of the smallest possible chain (1x1x1): the floor one library call costs on this machine."""
    from paper_2301_01333_amd import synth
    from paper_2301_01333_amd.harness import DeviceMLP

    wl = synth.make_mlp("f32", 1, [1, 1], [0], seed=1)
    dev = DeviceMLP(wl)
    sec, _ = time_steps(dev, steps, warmup)
    dev.close()
    return sec


def cpu_baseline(idx, budget_s=20.0):
    """The CPU oracle, as it stands, timed for about budget_s seconds on a bounded sample of the headline
    workload: a leading slice of its rows if one pass over all rows would take longer, else whole passes."""
    import oracle
    from paper_2301_01333_amd import synth

    full = synth.make_config(idx)
    probe_rows = min(full.m, 256)
    wl = synth.make_config(idx, m=probe_rows)
    t0 = time.perf_counter()
    oracle.mlp(wl)
    t_probe = max(time.perf_counter() - t0, 1e-4)
    rows = int(min(full.m, probe_rows * budget_s / t_probe))
    rows = max(32, rows // 32 * 32)
    wl = synth.make_config(idx, m=rows)
    passes, ops, t0 = 0, 0.0, time.perf_counter()
    while True:
        oracle.mlp(wl)
        passes += 1
        ops += wl.ops
        dt = time.perf_counter() - t0
        if dt >= 0.6 * budget_s or passes >= 64:
            break
    return {"value": ops / dt / 1e12, "unit": "TOP/s" if wl.dtype == "i8" else "TFLOP/s", "cores": oracle.num_threads(),
            "kind": "oracle", "sample": "%d pass(es) over the first %d of %d rows of config %d, all layers, %.1f s of CPU time"
            % (passes, rows, full.m, idx, dt)}


def blocked_io_report(idx, steps, warmup):
    """The same chain with x and y in the blocked hand-off layout (what a chain sees when it sits between two
    other chains of this library): the input is a real activation tensor, produced by running the chain once
    with a blocked y."""
    import numpy as np
    import torch
    from paper_2301_01333_amd import binding, synth

    wl = synth.make_config(idx)
    to_dev = lambda a: torch.from_numpy(np.ascontiguousarray(a).view(np.uint8).reshape(-1).copy()).cuda()
    w = [to_dev(v) for v in wl.w]
    bias = [None if v is None else to_dev(v) for v in wl.bias]
    ws = None if wl.dtype != "i8" else [to_dev(v) for v in wl.w_scale]
    first = binding.FusedMLP(wl.dtype, wl.m, wl.layers, mode=binding.OGC_MODE_PER_LAYER, y_layout=binding.OGC_LAYOUT_BLOCKED)
    chain = binding.FusedMLP(wl.dtype, wl.m, wl.layers, mode=binding.OGC_MODE_PER_LAYER, x_layout=binding.OGC_LAYOUT_BLOCKED,
                             y_layout=binding.OGC_LAYOUT_BLOCKED)
    first.prepack(w, bias, ws)
    chain.prepack(w, bias, ws)
    xb = torch.empty((binding.ogc_mlp_blocked_bytes(chain.plan, 0),), dtype=torch.uint8, device="cuda")
    yb = torch.empty((binding.ogc_mlp_blocked_bytes(chain.plan, 1),), dtype=torch.uint8, device="cuda")
    first.run(to_dev(wl.x), xb)

    class _Dev:
        def run(self_inner):
            chain.run(xb, yb)

    sec, ev_sec = time_steps(_Dev(), steps, warmup)
    peak, _ = PEAK[wl.dtype]
    first.close()
    chain.close()
    return {"workload": wl.name + ", x and y in the blocked hand-off layout", "ms_per_step": sec * 1e3,
            "ms_per_step_hip_events": ev_sec * 1e3, "tops_or_tflops": wl.ops / sec / 1e12, "frac_of_peak": wl.ops / sec / peak}


def fp8_report(steps, warmup):
    """The 8-bit-float (E4M3) variant of the quantized chain on the shapes of configurations 3 and 5 (seeded synthetic
    E4M3 tensors): time per chain with the plan's own choice of kernels, against the dense fp8 matrix peak."""
    from paper_2301_01333_amd import binding, synth
    from paper_2301_01333_amd.harness import DeviceMLP

    rows = []
    cases = [synth.make_mlp("f8", 256, [479, 1024, 1024, 512, 256, 1], [synth.ACT_RELU] * 4 + [synth.ACT_SIGMOID], seed=3001,
                            last_f32=True, name="config 3's shape in E4M3: M=256 479-1024-1024-512-256-1, fp32 sigmoid out"),
             synth.make_mlp("f8", 32768, [1024] * 5, [synth.ACT_RELU] * 4, seed=3002, has_bias=False,
                            name="config 5's shape in E4M3: M=32768 4x(1024-1024) ReLU + requantize")]
    for wl in cases:
        dev = DeviceMLP(wl)
        sec, ev = time_steps(dev, min(steps, 100), min(warmup, 10))
        nl = binding.ogc_mlp_num_launches(dev.mlp.plan)
        rows.append({"workload": wl.name, "mode": MODE_NAMES[dev.mlp.mode],
                     "kernels": sorted({binding.ogc_mlp_kernel_name(dev.mlp.plan, j) for j in range(nl)}),
                     "ms_per_step": sec * 1e3, "ms_per_step_hip_events": ev * 1e3, "tflops": wl.ops / sec / 1e12,
                     "frac_of_fp8_mfma_peak": wl.ops / sec / PEAK["f8"][0]})
        dev.close()
    return rows


def table1_sweep(steps, warmup):
    """The MLP rows of the paper's Table I over its batch range, fp32 and int8 (seeded synthetic tensors of
    those shapes): time per chain with the plan's own choice of kernels."""
    from paper_2301_01333_amd import binding, synth
    from paper_2301_01333_amd.harness import DeviceMLP

    rows = []
    shapes = {"MLP-1": [13, 512, 256, 128], "MLP-2": [479, 1024, 1024, 512, 256, 1]}
    for name, dims in shapes.items():
        for dtype in ("f32", "i8"):
            for m in (32, 64, 128, 256, 512):
                nl = len(dims) - 1
                acts = [synth.ACT_RELU] * nl
                kw = {}
                if name == "MLP-2":
                    acts[-1] = synth.ACT_SIGMOID if dtype == "i8" else synth.ACT_NONE
                    kw = dict(last_f32=True) if dtype == "i8" else {}
                wl = synth.make_mlp(dtype, m, dims, acts, seed=1000 + m, name="%s %s batch %d" % (name, dtype, m), **kw)
                dev = DeviceMLP(wl)
                sec, _ = time_steps(dev, steps, warmup)
                rows.append({"workload": wl.name, "mode": MODE_NAMES[dev.mlp.mode],
                             "kernel": binding.ogc_mlp_kernel_name(dev.mlp.plan, 0).split("<")[0],
                             "us_per_chain": sec * 1e6, "gops": wl.ops / sec / 1e9})
                dev.close()
    return rows


def mha_report(steps, warmup, with_cpu=True, only=None):
    """The attention subgraph on the MHA rows of the paper's Table I (seeded synthetic q, k, v and a padding
    mask of those shapes): one fused launch per run, stable softmax.  The roofline object is for the fp32
    kernel of the largest row (MHA-4, batch 128): both matmuls on the fp32 MFMA path."""
    import dataclasses

    import numpy as np
    import torch

    from paper_2301_01333_amd import binding, synth
    from paper_2301_01333_amd.harness import DeviceMHA

    rows, roof, cpu = [], None, None
    for row in ("MHA-1", "MHA-2", "MHA-3", "MHA-4"):
        if only and only[0] != row:
            continue
        big = synth.make_mha_table1(row, "f32", 128)
        big8 = synth.make_mha_table1(row, "i8", 128)   # the Int8 rows of Table I: int8 q, k, v and output
        for dtype in ("f32", "bf16", "i8"):
            conv = (lambda t: t) if dtype == "f32" else synth.f32_to_bf16_bits
            for batch in (32, 128):
                if only and (only[1] != dtype or int(only[2]) != batch):
                    continue
                if dtype == "i8":
                    wl = dataclasses.replace(big8, batch=batch, q=big8.q[:batch], k=big8.k[:batch], v=big8.v[:batch],
                                             mask=big8.mask[:batch], name="%s %s batch %d" % (row, dtype, batch))
                else:
                    wl = dataclasses.replace(big, dtype=dtype, batch=batch, q=conv(big.q[:batch]), k=conv(big.k[:batch]),
                                             v=conv(big.v[:batch]), mask=big.mask[:batch], name="%s %s batch %d" % (row, dtype, batch))
                dev = DeviceMHA(wl)
                sec, ev = time_steps(dev, max(steps // 3, 10), max(warmup // 3, 3))
                fast_sec = None
                if dtype != "i8":   # the softmax without the max reduction (Section VII); the Int8 form needs the maximum
                    fast_dev = DeviceMHA(wl, binding.OGC_SOFTMAX_FAST)
                    fast_sec, _ = time_steps(fast_dev, max(steps // 6, 10), 3)
                    del fast_dev
                peak = PEAK[dtype][0]
                r = {"workload": wl.name, "seq": wl.seq, "heads": wl.heads, "head_dim": wl.head_dim,
                     "kernel": binding.ogc_mha_i8_kernel_name(dev.desc) if dtype == "i8" else binding.ogc_mha_kernel_name(dev.desc, True),
                     "us_per_run": sec * 1e6, "us_per_run_fast_softmax": None if fast_sec is None else fast_sec * 1e6,
                     "tflops": wl.ops / sec / 1e12, "frac_of_mfma_peak": wl.ops / sec / peak,
                     "gb_per_s_algorithmic": wl.algorithmic_bytes / sec / 1e9}
                rows.append(r)
                if row == "MHA-4" and dtype == "f32" and batch == 128:
                    roof = {"bound": "mfma", "achieved": wl.ops / ev / 1e12, "peak": peak / 1e12, "unit": "TFLOP/s",
                            "frac": wl.ops / ev / peak, "traffic": read_traffic("mha4_f32_kernel_hbm_traffic.txt"), "kernel": r["kernel"],
                            "avg_launch_us": ev * 1e6, "workload": wl.name}
                    if with_cpu:
                        import oracle

                        nb = 2  # batch entries the oracle computes (all heads, all tokens)
                        hv = lambda t: t[:nb].reshape(nb, wl.seq, wl.heads, wl.head_dim).transpose(0, 2, 1, 3)
                        t0 = time.perf_counter()
                        reps = 0
                        while time.perf_counter() - t0 < 5.0:
                            oracle.attention(hv(wl.q), hv(wl.k), hv(wl.v), wl.mask[:nb], wl.scale)
                            reps += 1
                        dt = (time.perf_counter() - t0) / reps
                        cpu = {"value": wl.ops * nb / wl.batch / dt / 1e12, "unit": "TFLOP/s", "cores": os.cpu_count(),
                               "kind": "oracle", "sample": "%d of %d batch entries of %s, float64 numpy, %d passes" % (
                                   nb, wl.batch, wl.name, reps)}
                del dev
        del big, big8
    torch.cuda.synchronize()
    return {"rows": rows, "roofline": roof, "cpu_baseline": cpu}


def copy_calibration(torch):
    """Three plain 256 MiB device-to-device copies: the known-size reference for FETCH_SIZE / WRITE_SIZE runs."""
    src = torch.full((256 << 20,), 7, dtype=torch.uint8, device="cuda")
    dst = torch.empty_like(src)
    for _ in range(3):
        dst.copy_(src)
    torch.cuda.synchronize()


def read_traffic(name="cfg5_layer_kernel_hbm_traffic.txt"):
    """HBM bytes per launch of the dominant kernel from the committed rocprofv3 --pmc summary, if present."""
    path = os.path.join(ROOT, "profiles", name)
    try:
        for line in open(path):
            if line.startswith("traffic_bytes_per_launch:"):
                return float(line.split(":", 1)[1].split()[0])
    except OSError:
        pass
    return None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=300)
    # (the chip's clock takes about 250 steps of the headline workload, 35 ms, to come up from idle: 162 us for the first
    # 50 steps after a pause, 148, 137, 136, 134 for the next blocks of 50, 131-133 from then on)
    ap.add_argument("--warmup", type=int, default=300)
    ap.add_argument("--config", type=int, default=5, help="headline configuration (1..5)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the cpu_baseline leg")
    ap.add_argument("--only-headline", action="store_true", help="skip the per_config table")
    ap.add_argument("--table1", action="store_true",
                    help="instead of the benchmark line, print a JSON list of chain times for the MLP shapes of the paper's "
                         "Table I over batch 32..512 in fp32 and int8")
    ap.add_argument("--mha", action="store_true",
                    help="instead of the benchmark line, print the attention-subgraph report alone (the MHA rows of Table I)")
    ap.add_argument("--no-mha", action="store_true", help="skip the attention-subgraph report")
    ap.add_argument("--mha-workload", default=None, metavar="ROW:DTYPE:BATCH",
                    help="with --mha: only this workload, e.g. MHA-4:f32:128 (the one the report's roofline is for)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run a plain 256 MiB device copy three times (reference reading for rocprofv3 --pmc "
                         "FETCH_SIZE / WRITE_SIZE runs of this same command)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); --gpus %d is not supported" % args.gpus,
              file=sys.stderr)
        return 2
    import torch

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    from paper_2301_01333_amd import binding

    binding.lib()  # fail loudly if the HIP library is missing
    if args.table1:
        print(json.dumps({"table1_mlp_sweep": table1_sweep(args.steps, args.warmup)}))
        return 0
    if args.mha:
        only = args.mha_workload.split(":") if args.mha_workload else None
        print(json.dumps({"mha": mha_report(args.steps, args.warmup, not args.no_cpu, only)}))
        if args.copy_calibration:
            copy_calibration(torch)
        return 0
    floor = launch_floor(args.steps, args.warmup)
    wl, dev, head, launches = config_report(args.config, args.steps, args.warmup)
    peak, unit = PEAK[wl.dtype]
    # dominant kernel = the kernel (name with template arguments) with the largest share of the step; its
    # duration is the mean over its launches in one step, its work the mean of those layers' 2*M*K*N
    # (mfma bound) or the chain's algorithmic bytes (hbm bound, fused single launch)
    if head["mode"] == "per_layer":
        names = [binding.ogc_mlp_kernel_name(dev.mlp.plan, j) for j in range(len(launches))]
        share = {}
        for j, nm in enumerate(names):
            share[nm] = share.get(nm, 0.0) + launches[j]
        kname = max(share, key=share.get)
        idxs = [j for j, nm in enumerate(names) if nm == kname]
        dur = share[kname] / len(idxs)
        work = sum(2.0 * wl.m * wl.layers[j].k * wl.layers[j].n for j in idxs) / len(idxs)
        dom = {"kernel": kname, "launches_of_kernel": idxs, "launch_us": [round(t * 1e6, 2) for t in launches],
               "launch_kernels": names}
    else:
        dur = launches[0]
        work = float(wl.ops)
        dom = {"kernel": binding.ogc_mlp_kernel_name(dev.mlp.plan, 0), "launches_of_kernel": [0],
               "launch_us": [round(launches[0] * 1e6, 2)]}
    # An event pair around a single launch also times the gap to the next command (2-3 us here), while the
    # launches of a step run back to back.  The per-launch pairs therefore give each launch's share, and the
    # event pair around the whole timed region gives the total: duration = share * region time per step.
    dom["avg_launch_us_single_pair"] = round(dur * 1e6, 3)
    dur *= head["ms_per_step_hip_events"] * 1e-3 / sum(launches)
    dom["avg_launch_us"] = round(dur * 1e6, 3)
    if head["bound"] == "mfma":
        roof = {"bound": "mfma", "achieved": work / dur / 1e12, "peak": peak / 1e12, "unit": "TFLOP/s" if wl.dtype != "i8" else "TOP/s"}
    else:
        roof = {"bound": "hbm", "achieved": wl.algorithmic_bytes / dur / 1e9, "peak": HBM_PEAK / 1e9, "unit": "GB/s"}
    roof["frac"] = roof["achieved"] / roof["peak"]
    roof["traffic"] = read_traffic() if args.config == 5 else None
    roof.update(dom)
    if head["mode"] == "per_layer" and head["bound"] == "mfma":
        roof["clock"] = clock_report(dev, idxs, work, peak)
    dev.close()
    if args.copy_calibration:
        copy_calibration(torch)

    per = []
    if not args.only_headline:
        for idx in (1, 2, 3, 4, 5):
            if idx == args.config:
                r = dict(head)
            else:
                _, d, r, _ = config_report(idx, args.steps, args.warmup, with_floor=floor if idx <= 3 else None)
                d.close()
            if idx <= 3 and "launch_floor_ms" not in r:
                r["launch_floor_ms"] = floor * 1e3
            per.append(r)

    blocked = None
    if not args.only_headline and wl.dtype != "f32" and wl.layers[0].k == wl.layers[-1].n and not wl.residual:
        blocked = blocked_io_report(args.config, args.steps, args.warmup)
    out = {
        "metric": METRIC, "value": head["tops_or_tflops"], "unit": "TOPS" if wl.dtype == "i8" else "TFLOPS",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": head["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": {"i8": "u8", "bf16": "bf16", "f32": "f32"}[wl.dtype], "data": "synthetic",
        "config": {"workload": wl.name, "mode": head["mode"], "launches_per_step": head["launches"],
                   "ops_per_step": wl.ops, "algorithmic_bytes_per_step": wl.algorithmic_bytes},
        "frac_of_peak_whole_step": head["frac_of_bound"],
        "roofline": roof,
        "cpu_baseline": None if args.no_cpu else cpu_baseline(args.config),
        "launch_floor_us": floor * 1e6,
        "per_config": per,
        "blocked_io": blocked,
        "mha": None if (args.only_headline or args.no_mha) else mha_report(args.steps, args.warmup, not args.no_cpu),
        "fp8_variant": None if args.only_headline else fp8_report(args.steps, args.warmup),
        # the MLP rows of the paper's Table I over its batch range, each with the plan's own choice of kernel
        "table1_mlp_sweep": None if args.only_headline else table1_sweep(min(args.steps, 200), min(args.warmup, 20)),
    }
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
