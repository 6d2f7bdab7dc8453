#!/usr/bin/env python3
"""Benchmark of the SCC hot path on one MI355X.

A step is one pass of the whole hot path over one batch: scc_forward, scc_backward_input
and scc_backward_weight of the metric layer (N=128, Cin=Cout=256, 16x16, cg=4, co=0.5, fp32),
inputs resident in HBM.  Successive steps rotate through several buffer sets whose total
size exceeds the memory-side cache, so the tensors stream from HBM.

Prints ONE JSON line: whole-job throughput in GB/s of algorithmic bytes (each tensor of each
pass crossing HBM once), the roofline entry of the dominant kernel (timed live with events on
the launch stream) and the CPU oracle's rate on the host cores as a reported baseline.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E bandwidth
# HBM bytes per launch of each pass on the metric layer, from two rocprofv3 --pmc runs (FETCH_SIZE scaled by
# 1.9993, WRITE_SIZE by 1.0; both factors from a plain 64 MiB device copy): profiles/scc_metric_layer_kernels.md
MEASURED_TRAFFIC_BYTES = {"metric": {"fwd": int((16783.3 * 1.9993 + 32782.4) * 1024),
                                     "bwi": int((16785.9 * 1.9993 + 32801.0) * 1024),
                                     "bww": int(((32819.0 + 1038.0) * 1.9993 + 2048.0 + 64.0) * 1024)}}
KERNELS = {"fwd": ["forward_mfma32"], "bwi": ["backward_input_mfma32"],
           "bww": ["backward_weight_mfma32", "backward_weight_reduce"]}
ROTATE_BYTES = 768 << 20       # bytes ONE pass touches between two uses of a buffer (memory-side cache is 256 MB)


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="metric", help="metric | late | late_bf16 | expand | co00 | co25 | co75")
    ap.add_argument("--eager", action="store_true", help="launch from Python every step instead of replaying a HIP graph")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=12.0)
    ap.add_argument("--only", default="", help="time only this pass (fwd|bwi|bww) in the step loop; for profiling")
    ap.add_argument("--sweep", default="", metavar="FILE.json",
                    help="also time every configuration (overlap sweep, 14x14 layer fp32/bf16, expanding layer, "
                         "13-layer stack) pass by pass and write the table to this file")
    return ap.parse_args()


def pick_workload(name):
    import scc_workloads as Wk
    import torch
    table = {"metric": (Wk.METRIC, torch.float32), "late": (Wk.LATE, torch.float32),
             "late_bf16": (Wk.LATE, torch.bfloat16), "expand": (Wk.EXPAND, torch.float32),
             "co00": (Wk.METRIC_SWEEP[0], torch.float32), "co25": (Wk.METRIC_SWEEP[1], torch.float32),
             "co75": (Wk.METRIC_SWEEP[3], torch.float32)}
    return table[name]


def measure(S, Wk, torch, layer, dtype, steps, warmup, eager=False, only="", whole_step=True):
    """Times one layer: the whole step (all passes back to back) and each pass on its own.
    Returns (inputs, dict of figures)."""
    esz = 4 if dtype == torch.float32 else 2
    dev = torch.device("cuda:0")
    x, w, dy = Wk.make_inputs(layer)
    # one set = x, y, dy, dx; a single pass touches only half of it (one input and one output tensor), and the
    # bytes touched between two uses of the same buffer must exceed the memory-side cache for every timed loop
    set_bytes = esz * 2 * layer.N * layer.HW * (layer.Cin + layer.Cout)
    R = max(2, min(256, -(-ROTATE_BYTES // (set_bytes // 2))))
    sets = []
    for r in range(R):
        xs = torch.from_numpy(x).to(dtype).to(dev)
        ds = torch.from_numpy(dy).to(dtype).to(dev)
        if r:  # distinct contents per set, same distribution
            xs = xs.roll(r, 0)
            ds = ds.roll(r, 0)
        sets.append(dict(x=xs.contiguous(), dy=ds.contiguous(), w=torch.from_numpy(w).to(dtype).to(dev),
                         y=torch.empty((layer.N, layer.Cout, layer.H, layer.W), dtype=dtype, device=dev),
                         dx=torch.empty((layer.N, layer.Cin, layer.H, layer.W), dtype=dtype, device=dev),
                         dw=torch.empty((layer.Cout, layer.L), dtype=torch.float32, device=dev)))
    ws_bytes = S.scc_backward_weight_workspace_bytes(layer.N, layer.Cin, layer.Cout, layer.H, layer.W, layer.cg,
                                                     layer.co, dtype)
    workspace = torch.empty(max(ws_bytes, 256), dtype=torch.uint8, device=dev)

    def fwd(b):
        S.scc_forward(b["x"], b["w"], layer.cg, layer.co, out=b["y"])

    def bwi(b):
        S.scc_backward_input(b["dy"], b["w"], layer.Cin, layer.cg, layer.co, out=b["dx"])

    def bww(b):
        S.scc_backward_weight(b["x"], b["dy"], layer.cg, layer.co, out=b["dw"], workspace=workspace)

    passes = {"fwd": fwd, "bwi": bwi, "bww": bww}
    step_passes = [only] if only else ["fwd", "bwi", "bww"]

    def step(b):
        for name in step_passes:
            passes[name](b)

    # ---- one replayable unit = R steps, one per buffer set -------------------------------------
    side = torch.cuda.Stream()

    def make_runner(fn):
        """Returns run(k): enqueue k calls of fn over the rotating buffer sets on `side`."""
        if eager:
            def run(k):
                for i in range(k):
                    fn(sets[i % R])
            return run
        g = torch.cuda.CUDAGraph()
        with torch.cuda.stream(side):
            for b in sets:      # warm every set eagerly before capture
                fn(b)
            side.synchronize()
            with torch.cuda.graph(g, stream=side):
                for b in sets:
                    fn(b)

        def run(k):
            full, rest = divmod(k, R)
            for _ in range(full):
                g.replay()
            for i in range(rest):
                fn(sets[i])
        return run

    def timed(run, k, warm):
        with torch.cuda.stream(side):
            run(warm)
            side.synchronize()
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            t0 = time.perf_counter()
            e0.record(side)
            run(k)
            e1.record(side)
            side.synchronize()
            torch.cuda.synchronize()
            wall = time.perf_counter() - t0
        return e0.elapsed_time(e1) / k, wall * 1e3 / k      # ms per call: device events, host wall

    K = max(R, (steps // R) * R) if not eager else steps
    alg_bytes = {"fwd": Wk.algorithmic_bytes(layer, esz), "bwi": Wk.algorithmic_bytes(layer, esz),
                 "bww": esz * layer.N * layer.HW * (layer.Cin + layer.Cout) + 4 * layer.Cout * layer.L}
    res = {"K": K, "R": R, "alg_bytes": alg_bytes, "step_passes": step_passes,
           "step_bytes": sum(alg_bytes[p] for p in step_passes)}
    if whole_step:
        ms_ev, ms_wall = timed(make_runner(step), K, warmup)
        res.update(ms_ev=ms_ev, ms_wall=ms_wall, ms_step=max(ms_ev, ms_wall))   # the slower clock is the honest one
    # per-pass average durations (events on the launch stream, back-to-back launches)
    res["per_pass_ms"] = {name: timed(make_runner(passes[name]), K, warmup)[0] for name in step_passes}
    return (x, w, dy), res


def sweep(S, Wk, torch, steps, warmup, path):
    """Every configuration of the build, each pass timed on its own; written to `path` and to stderr."""
    cases = [(l, torch.float32) for l in Wk.METRIC_SWEEP] + [(Wk.LATE, torch.float32), (Wk.LATE, torch.bfloat16),
                                                             (Wk.EXPAND, torch.float32)]
    cases += [(l, torch.float32) for l in Wk.STACK]
    cases += [(l, torch.float32) for l in Wk.CG_SWEEP] + [(l, torch.float32) for l in Wk.BATCH_SWEEP]
    cases += [(l, torch.bfloat16) for l in [Wk.METRIC, Wk.EXPAND, Wk.BATCH_SWEEP[0], Wk.BATCH_SWEEP[-1]]]
    rows = []
    for layer, dtype in cases:
        esz = 4 if dtype == torch.float32 else 2
        _, r = measure(S, Wk, torch, layer, dtype, steps, warmup, whole_step=False)
        us = {k: v * 1e3 for k, v in r["per_pass_ms"].items()}
        mb, gf = Wk.algorithmic_bytes(layer, esz) / 1e6, Wk.algorithmic_flops(layer) / 1e9
        # lower bound of one pass: bytes at the HBM peak or flops at the fp32 matrix peak, whichever is longer
        bound_us = max(mb * 1e6 / (HBM_PEAK_GBS * 1e9), gf * 1e9 / 157.3e12) * 1e6
        rows.append({"layer": layer.name, "dtype": "f32" if esz == 4 else "bf16", "MB_per_pass": round(mb, 2),
                     "GFLOP_per_pass": round(gf, 3), "bound_us_per_pass": round(bound_us, 2),
                     "us": {k: round(v, 2) for k, v in us.items()}, "us_sum": round(sum(us.values()), 2),
                     "frac_of_bound": round(3 * bound_us / sum(us.values()), 3)})
        print("%-36s %-4s %7.1f MB %6.2f GF | fwd %7.1f bwi %7.1f bww %7.1f us | bound %5.1f us/pass" %
              (layer.name, rows[-1]["dtype"], mb, gf, us["fwd"], us["bwi"], us["bww"], bound_us), file=sys.stderr,
              flush=True)
    stack = [r for r in rows if r["layer"].startswith("c5_")]
    summary = {"stack_us_sum": round(sum(r["us_sum"] for r in stack), 1),
               "stack_bound_us_sum": round(3 * sum(r["bound_us_per_pass"] for r in stack), 1)}
    os.makedirs(os.path.dirname(path), exist_ok=True)
    with open(path, "w") as f:
        json.dump({"rows": rows, "summary": summary}, f, indent=1)
    print("stack of 13 layers, three passes each: %.1f us (bound %.1f us)" %
          (summary["stack_us_sum"], summary["stack_bound_us_sum"]), file=sys.stderr, flush=True)


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (run with --gpus 1)", file=sys.stderr)
        sys.exit(2)
    import numpy as np
    import torch

    import paper_2101_00745_amd as S
    import scc_workloads as Wk

    if not torch.cuda.is_available():
        print("bench.py needs the GPU: there is no CPU path", file=sys.stderr)
        sys.exit(2)
    S.load()
    if args.sweep:
        sweep(S, Wk, torch, min(args.steps, 64), min(args.warmup, 8), args.sweep)
    layer, dtype = pick_workload(args.workload)
    (x, w, dy), r = measure(S, Wk, torch, layer, dtype, args.steps, args.warmup, args.eager, args.only)
    K, R, W = r["K"], r["R"], args.warmup
    alg_bytes, step_passes, step_bytes = r["alg_bytes"], r["step_passes"], r["step_bytes"]
    ms_ev, ms_wall, ms_step, per_pass = r["ms_ev"], r["ms_wall"], r["ms_step"], r["per_pass_ms"]
    value = step_bytes / (ms_step * 1e-3) / 1e9
    dominant = max(per_pass, key=per_pass.get)
    achieved = alg_bytes[dominant] / (per_pass[dominant] * 1e-3) / 1e9
    traffic = MEASURED_TRAFFIC_BYTES.get(args.workload, {}).get(dominant) if dtype == torch.float32 else None
    roofline = {"bound": "hbm", "kernel": {"fwd": "scc_forward", "bwi": "scc_backward_input",
                                           "bww": "scc_backward_weight"}[dominant],
                "kernels": KERNELS[dominant], "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": traffic,
                "algorithmic_bytes_per_launch": alg_bytes[dominant],
                "avg_us": round(per_pass[dominant] * 1e3, 2),
                "per_pass_us": {k: round(v * 1e3, 2) for k, v in per_pass.items()},
                "per_pass_GBs": {k: round(alg_bytes[k] / (v * 1e-3) / 1e9, 1) for k, v in per_pass.items()},
                "per_pass_TFLOPs": {k: round(Wk.algorithmic_flops(layer) / (v * 1e-3) / 1e12, 2)
                                    for k, v in per_pass.items()}}

    out = {"metric": "SCC fwd+bwd GB/s & fraction of HBM peak, N=128 Cin=Cout=256 16x16 fp32",
           "value": round(value, 1), "unit": "GB/s", "n_gpus": 1, "steps": K, "warmup": W,
           "ms_per_step": round(ms_step, 5), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
           "dtype": "f32" if dtype == torch.float32 else "bf16", "data": "synthetic",
           "config": {"workload": "configs[1]: %s" % layer.name if args.workload == "metric" else layer.name,
                      "N": layer.N, "Cin": layer.Cin, "Cout": layer.Cout, "H": layer.H, "W": layer.W,
                      "cg": layer.cg, "co": layer.co, "passes": "+".join(step_passes),
                      "buffer_sets_rotated": R, "launch": "eager" if args.eager else "hip_graph"},
           "frac_of_hbm_peak": round(value / HBM_PEAK_GBS, 4),
           "ms_per_step_events": round(ms_ev, 5), "ms_per_step_wall": round(ms_wall, 5),
           "roofline": roofline}

    if not args.no_cpu_baseline:
        from oracle import scc_oracle as O
        xr, wr, dyr = (a.astype(np.float64) for a in (x, w, dy))
        t0, reps = time.perf_counter(), 0
        while True:
            if "fwd" in step_passes:
                O.forward(xr, wr, layer.cg, layer.co)
            if "bwi" in step_passes:
                O.backward_input(dyr, wr, layer.Cin, layer.cg, layer.co)
            if "bww" in step_passes:
                O.backward_weight(xr, dyr, layer.cg, layer.co)
            reps += 1
            el = time.perf_counter() - t0
            if el >= args.cpu_seconds or reps >= 200:
                break
        out["cpu_baseline"] = {"value": round(step_bytes * reps / el / 1e9, 3), "unit": "GB/s", "cores": O.threads(),
                               "kind": "oracle", "sample": "%d full steps of the same layer (fp64 oracle, %.1f s)"
                               % (reps, el), "ms_per_step": round(el * 1e3 / reps, 2)}
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
