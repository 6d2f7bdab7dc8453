#!/usr/bin/env python3
"""Benchmark of the SCC hot path on one MI355X.

A step is one pass of the whole hot path over one batch of the metric layer (N=128, Cin=Cout=256, 16x16,
cg=4, co=0.5, fp32), inputs resident in HBM: scc_forward, then scc_backward (grad-input and grad-weight in one
call; for this layer one kernel that reads dy and x once, plus the K-split reduction).  The same step through
the three separate entry points (scc_forward, scc_backward_input, scc_backward_weight) is timed beside it.
Successive steps rotate through buffer sets whose size exceeds the memory-side cache, so tensors stream
from HBM.

Prints ONE JSON line: whole-job throughput in GB/s of the metric's algorithmic bytes (three passes, each tensor
of each pass crossing HBM once: 3 x 67.17 MB), the roofline entry of the dominant pass (timed live with events
on the launch stream), a plain device copy on the same buffers as the ceiling the memory system offers, and the
CPU oracle's rate on the host cores as a reported baseline.
"""
import argparse
import ctypes
import json
import os
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E bandwidth
F32_MATRIX_PEAK = 157.3e12     # dense fp32 matrix peak, flop/s
BF16_MATRIX_PEAK = 2.5e15      # dense bf16 matrix peak, flop/s
# HBM bytes per launch on the metric layer, from two rocprofv3 --pmc runs of the build named below (FETCH_SIZE
# scaled by the factor a plain device copy gives, WRITE_SIZE by 1.0): profiles/scc_metric_layer_kernels.md
TRAFFIC_PROFILED_BUILD = "commit 5274804; profiles/scc_metric_layer_kernels.md"
MEASURED_TRAFFIC_BYTES = {"metric": {"fwd": 67910383, "bwi": 67876558, "bww": 69266705 + 2190045, "bwd": 103423085 + 2190045}}
KERNELS = {"fwd": ["forward_mfma32"], "bwi": ["backward_input_mfma32"],
           "bww": ["backward_weight_mfma32", "backward_weight_reduce"],
           "bwd": ["backward_fused_lds32", "backward_weight_reduce"]}
ENTRY = {"fwd": "scc_forward", "bwi": "scc_backward_input", "bww": "scc_backward_weight", "bwd": "scc_backward"}
ROTATE_BYTES = 768 << 20       # bytes ONE pass touches between two uses of a buffer (memory-side cache is 256 MB)
MIN_REPLAYS = 8
# the paper's own speedups, for context only: another machine, whole CNN training steps, not this metric
PAPER_CONTEXT = {"hardware": "1x NVIDIA Tesla V100 32 GB, Intel Xeon Platinum 8168 (Section 5.1)",
                 "what": "end-to-end CNN training-step speedups of the paper's CUDA kernels over PyTorch operator "
                         "compositions of SCC (Sections 5.3 and 5.4); no per-kernel time or bandwidth is published",
                 "training_step_vs_pytorch_base_mean": 5.68, "training_step_vs_pytorch_opt_mean": 2.34,
                 "backward_only_vs_base_opt_outputcentric_mean": [15.03, 4.55, 1.55]}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="metric", help="metric | late | late_bf16 | expand | co00 | co25 | co75")
    ap.add_argument("--eager", action="store_true", help="launch from Python every step instead of replaying a HIP graph")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=12.0)
    ap.add_argument("--only", default="", help="time only this pass (fwd|bwi|bww|bwd) in the step loop; for profiling")
    ap.add_argument("--sweep", default="", metavar="FILE.json",
                    help="also time every configuration (overlap sweep, 14x14 layer fp32/bf16, expanding layer, "
                         "13-layer stack, group-count and batch sweeps) pass by pass and write the table to this file")
    ap.add_argument("--dispatch-trace", action="store_true",
                    help="run every configuration's entry points once each, a 16-byte membw_read launch before each "
                         "as a separator, and print the order: under `rocprofv3 --kernel-trace` the trace then shows "
                         "which kernels every configuration dispatched")
    ap.add_argument("--block-trace", action="store_true",
                    help="run the forward of the DW + SCC block on the metric layer (fused kernel, then the two stages) "
                         "on rotating buffers and exit: the run a profiler wraps for the block's kernels")
    return ap.parse_args()


def pick_workload(name):
    import scc_workloads as Wk
    import torch
    table = {"metric": (Wk.METRIC, torch.float32), "late": (Wk.LATE, torch.float32),
             "late_bf16": (Wk.LATE, torch.bfloat16), "expand": (Wk.EXPAND, torch.float32),
             "co00": (Wk.METRIC_SWEEP[0], torch.float32), "co25": (Wk.METRIC_SWEEP[1], torch.float32),
             "co75": (Wk.METRIC_SWEEP[3], torch.float32)}
    return table[name]


def load_membw():
    from paper_2101_00745_amd import build as hip_build
    if not os.path.exists(hip_build.MEMBW_LIB):
        raise ImportError("libscc_membw.so is not built: run `python -m paper_2101_00745_amd.build` first")
    lib = ctypes.CDLL(hip_build.MEMBW_LIB)
    for fn in (lib.membw_copy_bytes, lib.membw_read_bytes):
        fn.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_longlong, ctypes.c_void_p]
        fn.restype = ctypes.c_int
    return lib


def pass_bytes(Wk, layer, esz):
    """Algorithmic bytes per call of each entry point: every tensor it must read or write, once."""
    act = esz * layer.N * layer.HW
    wts = layer.Cout * layer.L
    return {"fwd": Wk.algorithmic_bytes(layer, esz), "bwi": Wk.algorithmic_bytes(layer, esz),
            "bww": act * (layer.Cin + layer.Cout) + 4 * wts,
            "bwd": act * (2 * layer.Cin + layer.Cout) + esz * wts + 4 * wts}       # x, dy in; dx out; w in; dw out


class Timer:
    """Replays one unit of work (R calls of fn, one per buffer set) as a HIP graph and times it with events on the
    launch stream and with the host clock."""

    def __init__(self, torch, sets, eager):
        self.torch, self.sets, self.eager, self.R = torch, sets, eager, len(sets)
        self.side = torch.cuda.Stream()

    def runner(self, fn):
        torch, sets = self.torch, self.sets
        if self.eager:
            def replay():
                for b in sets:
                    fn(b)
            return replay
        g = torch.cuda.CUDAGraph()
        with torch.cuda.stream(self.side):
            for b in sets:      # warm every set eagerly before capture
                fn(b)
            self.side.synchronize()
            with torch.cuda.graph(g, stream=self.side):
                for b in sets:
                    fn(b)
        return g.replay

    def time(self, fn, replays, warm_replays):
        """Returns (ms per call from events over all replays, ms per call host wall, median ms per call of the
        per-replay event intervals)."""
        torch, side = self.torch, self.side
        replay = self.runner(fn)
        with torch.cuda.stream(side):
            for _ in range(max(1, warm_replays)):
                replay()
            side.synchronize()
            torch.cuda.synchronize()
            ev = [torch.cuda.Event(enable_timing=True) for _ in range(replays + 1)]
            t0 = time.perf_counter()
            ev[0].record(side)
            for i in range(replays):
                replay()
                ev[i + 1].record(side)
            side.synchronize()
            torch.cuda.synchronize()
            wall = time.perf_counter() - t0
        calls = replays * self.R
        per = [ev[i].elapsed_time(ev[i + 1]) / self.R for i in range(replays)]
        return ev[0].elapsed_time(ev[-1]) / calls, wall * 1e3 / calls, statistics.median(per)


def measure(S, Wk, torch, layer, dtype, steps, warmup, eager=False, only="", whole_step=True, copy_lib=None):
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
    shape = (layer.N, layer.Cin, layer.Cout, layer.H, layer.W, layer.cg, layer.co, dtype)
    ws_bytes = max(S.scc_backward_weight_workspace_bytes(*shape), S.scc_backward_workspace_bytes(*shape))
    workspace = torch.empty(max(ws_bytes, 256), dtype=torch.uint8, device=dev)

    def fwd(b):
        S.scc_forward(b["x"], b["w"], layer.cg, layer.co, out=b["y"])

    def bwi(b):
        S.scc_backward_input(b["dy"], b["w"], layer.Cin, layer.cg, layer.co, out=b["dx"])

    def bww(b):
        S.scc_backward_weight(b["x"], b["dy"], layer.cg, layer.co, out=b["dw"], workspace=workspace)

    def bwd(b):
        S.scc_backward(b["x"], b["dy"], b["w"], layer.cg, layer.co, out_dx=b["dx"], out_dw=b["dw"], workspace=workspace)

    passes = {"fwd": fwd, "bwi": bwi, "bww": bww, "bwd": bwd}
    step_passes = [only] if only else ["fwd", "bwd"]
    three_passes = ["fwd", "bwi", "bww"]

    def step_of(names):
        def step(b):
            for name in names:
                passes[name](b)
        return step

    # whatever --steps says, at least MIN_REPLAYS graph replays are timed (a replay is R steps, one per buffer
    # set), and the warm-up is whole replays: the reported step count is the number actually timed
    replays = max(MIN_REPLAYS, -(-steps // R))
    warm = max(1, -(-warmup // R))
    timer = Timer(torch, sets, eager)
    alg = pass_bytes(Wk, layer, esz)
    res = {"K": replays * R, "W": warm * R, "R": R, "replays": replays, "alg_bytes": alg, "step_passes": step_passes,
           "metric_bytes": 3 * Wk.algorithmic_bytes(layer, esz)}
    if whole_step:
        ev, wall, med = timer.time(step_of(step_passes), replays, warm)
        res.update(ms_ev=ev, ms_wall=wall, ms_median=med, ms_step=max(ev, wall))   # the slower clock is the honest one
        if not only:
            ev3, wall3, med3 = timer.time(step_of(three_passes), replays, warm)
            res["three_pass"] = {"ms_ev": ev3, "ms_wall": wall3, "ms_median": med3, "ms_step": max(ev3, wall3)}
    # per-pass average durations (events on the launch stream, back-to-back launches of one entry point)
    names = step_passes if only else ["fwd", "bwd", "bwi", "bww"]
    res["per_pass_ms"] = {name: timer.time(passes[name], replays, warm)[2] for name in names}
    if copy_lib is not None:
        # what the memory system gives a plain copy of one activation tensor into another, on the same rotating
        # buffers (x -> dx of each set: 32 MiB -> 32 MiB at the metric layer), and a copy too large for any cache
        nbytes = sets[0]["x"].numel() * esz

        def small_copy(b):
            copy_lib.membw_copy_bytes(b["x"].data_ptr(), b["dx"].data_ptr(), nbytes,
                                      ctypes.c_void_p(torch.cuda.current_stream().cuda_stream))
        ms_small = timer.time(small_copy, replays, warm)[2]
        big = 1 << 30
        src = torch.empty(big, dtype=torch.uint8, device=dev).fill_(1)
        dst = torch.empty(big, dtype=torch.uint8, device=dev)
        big_timer = Timer(torch, [dict(a=src, b=dst), dict(a=dst, b=src)], eager)

        def big_copy(b):
            copy_lib.membw_copy_bytes(b["a"].data_ptr(), b["b"].data_ptr(), big,
                                      ctypes.c_void_p(torch.cuda.current_stream().cuda_stream))
        ms_big = big_timer.time(big_copy, 4, 1)[2]
        res["copy"] = {"small_bytes_each_way": nbytes, "small_us": ms_small * 1e3,
                       "small_GBs": 2 * nbytes / (ms_small * 1e-3) / 1e9,
                       "large_bytes_each_way": big, "large_us": ms_big * 1e3, "large_GBs": 2 * big / (ms_big * 1e-3) / 1e9}
        del src, dst
    return (x, w, dy), res


def oracle_step_seconds(Wk, layer, seconds, max_reps=200, sample_n=None):
    """Times the fp64 CPU oracle (forward + grad-input + grad-weight) on the layer, or on its first `sample_n`
    samples.  Returns (seconds per step, steps timed, threads)."""
    import numpy as np
    from oracle import scc_oracle as O
    x, w, dy = Wk.make_inputs(layer)
    if sample_n:
        x, dy = x[:sample_n], dy[:sample_n]
    xr, wr, dyr = (a.astype(np.float64) for a in (x, w, dy))
    t0, reps = time.perf_counter(), 0
    while True:
        O.forward(xr, wr, layer.cg, layer.co)
        O.backward_input(dyr, wr, layer.Cin, layer.cg, layer.co)
        O.backward_weight(xr, dyr, layer.cg, layer.co)
        reps += 1
        el = time.perf_counter() - t0
        if el >= seconds or reps >= max_reps:
            return el / reps, reps, O.threads()


def sweep(S, Wk, torch, steps, warmup, path):
    """Every configuration of the build, each pass timed on its own; written to `path` and to stderr."""
    rows = []
    for layer, dtype in all_cases(Wk, torch):
        esz = 4 if dtype == torch.float32 else 2
        _, r = measure(S, Wk, torch, layer, dtype, steps, warmup, whole_step=False)
        us = {k: v * 1e3 for k, v in r["per_pass_ms"].items()}
        mb, gf = Wk.algorithmic_bytes(layer, esz) / 1e6, Wk.algorithmic_flops(layer) / 1e9
        # lower bound of one pass: bytes at the HBM peak or flops at the matrix peak of the dtype, whichever is longer
        peak = F32_MATRIX_PEAK if esz == 4 else BF16_MATRIX_PEAK
        bound_us = max(mb * 1e6 / (HBM_PEAK_GBS * 1e9), gf * 1e9 / peak) * 1e6
        three = us["fwd"] + us["bwi"] + us["bww"]
        best = us["fwd"] + min(us["bwd"], us["bwi"] + us["bww"])
        # the CPU oracle on the same layer, a bounded sample: a few steps on at most 16 samples, scaled to the layer
        n_or = min(layer.N, 16)
        sec, _, thr = oracle_step_seconds(Wk, layer, 0.5, max_reps=3, sample_n=n_or)
        rows.append({"layer": layer.name, "dtype": "f32" if esz == 4 else "bf16", "MB_per_pass": round(mb, 2),
                     "GFLOP_per_pass": round(gf, 3), "bound_us_per_pass": round(bound_us, 2),
                     "us": {k: round(v, 2) for k, v in us.items()}, "us_three_passes": round(three, 2),
                     "us_fwd_plus_backward": round(best, 2), "frac_of_bound": round(3 * bound_us / best, 3),
                     "oracle_ms_per_step": round(sec * 1e3 * layer.N / n_or, 1), "oracle_threads": thr,
                     "oracle_sample": "%d of %d samples" % (n_or, layer.N)})
        print("%-36s %-4s %7.1f MB %6.2f GF | fwd %7.1f bwi %7.1f bww %7.1f bwd %7.1f us | bound %5.1f us/pass | oracle %8.1f ms" %
              (layer.name, rows[-1]["dtype"], mb, gf, us["fwd"], us["bwi"], us["bww"], us["bwd"], bound_us,
               rows[-1]["oracle_ms_per_step"]), file=sys.stderr, flush=True)
    stack = [r for r in rows if r["layer"].startswith("c5_")]
    summary = {"stack_us_three_passes": round(sum(r["us_three_passes"] for r in stack), 1),
               "stack_us_fwd_plus_backward": round(sum(r["us_fwd_plus_backward"] for r in stack), 1),
               "stack_bound_us_sum": round(3 * sum(r["bound_us_per_pass"] for r in stack), 1)}
    blocks = block_sweep(S, Wk, torch)
    os.makedirs(os.path.dirname(os.path.abspath(path)), exist_ok=True)
    with open(path, "w") as f:
        json.dump({"rows": rows, "summary": summary, "dw_scc_blocks": blocks}, f, indent=1)
    print("stack of 13 layers: %.1f us as three passes, %.1f us as forward + scc_backward (bound %.1f us)" %
          (summary["stack_us_three_passes"], summary["stack_us_fwd_plus_backward"], summary["stack_bound_us_sum"]),
          file=sys.stderr, flush=True)


def block_sweep(S, Wk, torch, replays_floor=MIN_REPLAYS, layers=None):
    """Forward of the DW + SCC block (depthwise 3x3 stage in front of the SCC; stride 2 where the stack's map halves)
    on the metric layer and the 13 stack layers, fp32: the call as the library dispatches it (`auto`), the fused
    kernel forced, and the two stages run one after the other, each on cold rotating buffers."""
    dev = torch.device("cuda:0")
    out = []
    for layer, s in (layers or [(Wk.METRIC, 1)] + list(zip(Wk.STACK, Wk.STACK_DW_STRIDE))):
        xin, kdw, w = Wk.make_block_inputs(layer, s)
        out_bytes = 4 * layer.N * layer.Cout * layer.HW
        R = max(2, min(256, -(-ROTATE_BYTES // max(xin.nbytes, out_bytes))))
        sets = [dict(x=torch.from_numpy(xin).to(dev).roll(r, 0).contiguous(), k=torch.from_numpy(kdw).to(dev),
                     w=torch.from_numpy(w).to(dev),
                     y=torch.empty((layer.N, layer.Cout, layer.H, layer.W), device=dev)) for r in range(R)]
        shape = (layer.N, layer.Cin, layer.Cout, xin.shape[2], xin.shape[3], s, layer.cg, layer.co)
        ws = torch.empty(max(256, S.scc_dw_forward_workspace_bytes(*shape), 4 * layer.N * layer.Cin * layer.HW),
                         dtype=torch.uint8, device=dev)
        z = ws.view(torch.float32)[:layer.N * layer.Cin * layer.HW].view(layer.N, layer.Cin, layer.H, layer.W)

        def auto(b):
            S.scc_dw_forward(b["x"], b["k"], b["w"], layer.cg, layer.co, s, out=b["y"], workspace=ws)

        def fused(b):
            S.scc_dw_forward(b["x"], b["k"], b["w"], layer.cg, layer.co, s, out=b["y"], fused=True)

        def two(b):
            S.scc_depthwise3x3_forward(b["x"], b["k"], s, out=z)
            S.scc_forward(z, b["w"], layer.cg, layer.co, out=b["y"])

        timer = Timer(torch, sets, False)
        reps = max(replays_floor, -(-96 // R))
        us = {name: timer.time(fn, reps, 2)[2] * 1e3 for name, fn in (("auto", auto), ("fused", fused), ("two_stages", two))}
        alg = Wk.block_algorithmic_bytes(layer, s)
        out.append({"layer": layer.name, "dw_stride": s, "MB": round(alg / 1e6, 2), "bound_us": round(alg / (HBM_PEAK_GBS * 1e3), 2),
                    "library_fuses": S.scc_dw_forward_workspace_bytes(*shape) == 0,
                    "us": {k: round(v, 2) for k, v in us.items()}, "GBs_auto": round(alg / us["auto"] / 1e3, 1)})
        print("block %-30s s=%d %6.1f MB | auto %7.1f (%s) fused %7.1f two stages %7.1f us | bound %5.1f us" %
              (layer.name, s, alg / 1e6, us["auto"], "fused" if out[-1]["library_fuses"] else "two stages", us["fused"],
               us["two_stages"], out[-1]["bound_us"]), file=sys.stderr, flush=True)
        del sets, ws, z
    if layers is None:
        print("DW + SCC forward over the 13 stack layers: %.1f us as dispatched, %.1f us in two stages everywhere" %
              (sum(r["us"]["auto"] for r in out[1:]), sum(r["us"]["two_stages"] for r in out[1:])), file=sys.stderr,
              flush=True)
    return out


def all_cases(Wk, torch):
    cases = [(l, torch.float32) for l in Wk.METRIC_SWEEP] + [(Wk.LATE, torch.float32), (Wk.LATE, torch.bfloat16),
                                                             (Wk.EXPAND, torch.float32)]
    cases += [(l, torch.float32) for l in Wk.STACK]
    cases += [(l, torch.float32) for l in Wk.CG_SWEEP] + [(l, torch.float32) for l in Wk.BATCH_SWEEP]
    cases += [(l, torch.bfloat16) for l in [Wk.METRIC, Wk.EXPAND, Wk.BATCH_SWEEP[0], Wk.BATCH_SWEEP[-1]]]
    return cases


def dispatch_trace(S, Wk, torch, copy_lib):
    """One call of every entry point per configuration, separated by a 16-byte membw_read launch."""
    dev = torch.device("cuda:0")
    sink = torch.zeros(64, dtype=torch.float32, device=dev)
    order = []
    for layer, dtype in all_cases(Wk, torch):
        x, w, dy = Wk.make_inputs(layer)
        xd, wd, dyd = (torch.from_numpy(a).to(dtype).to(dev) for a in (x, w, dy))
        for name, fn in (("scc_forward", lambda: S.scc_forward(xd, wd, layer.cg, layer.co)),
                         ("scc_backward_input", lambda: S.scc_backward_input(dyd, wd, layer.Cin, layer.cg, layer.co)),
                         ("scc_backward_weight", lambda: S.scc_backward_weight(xd, dyd, layer.cg, layer.co)),
                         ("scc_backward", lambda: S.scc_backward(xd, dyd, wd, layer.cg, layer.co))):
            copy_lib.membw_read_bytes(sink.data_ptr(), sink.data_ptr() + 64, 16, None)
            fn()
            torch.cuda.synchronize()
            order.append("%s %s %s" % (layer.name, "f32" if dtype == torch.float32 else "bf16", name))
        del xd, wd, dyd
    for layer, s in [(Wk.METRIC, 1)] + list(zip(Wk.STACK, Wk.STACK_DW_STRIDE)):
        xin, kdw, w = Wk.make_block_inputs(layer, s)
        xd, kd, wd = (torch.from_numpy(a).to(dev) for a in (xin, kdw, w))
        copy_lib.membw_read_bytes(sink.data_ptr(), sink.data_ptr() + 64, 16, None)
        S.scc_dw_forward(xd, kd, wd, layer.cg, layer.co, s)
        torch.cuda.synchronize()
        order.append("%s f32 scc_dw_forward(stride=%d)" % (layer.name, s))
        del xd, kd, wd
    print("\n".join(order), flush=True)


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (run with --gpus 1)", file=sys.stderr)
        sys.exit(2)
    import torch

    import paper_2101_00745_amd as S
    import scc_workloads as Wk

    if not torch.cuda.is_available():
        print("bench.py needs the GPU: there is no CPU path", file=sys.stderr)
        sys.exit(2)
    S.load()
    copy_lib = load_membw()
    if args.dispatch_trace:
        dispatch_trace(S, Wk, torch, copy_lib)
        return
    if args.block_trace:
        print(json.dumps(block_sweep(S, Wk, torch, layers=[(Wk.METRIC, 1)])[0]))
        return
    if args.sweep:
        sweep(S, Wk, torch, min(args.steps, 64), min(args.warmup, 8), args.sweep)
    layer, dtype = pick_workload(args.workload)
    _, r = measure(S, Wk, torch, layer, dtype, args.steps, args.warmup, args.eager, args.only, copy_lib=copy_lib)
    K, R, W = r["K"], r["R"], r["W"]
    alg, step_passes = r["alg_bytes"], r["step_passes"]
    # the metric's bytes: three passes, each tensor of each pass once (a single pass when --only is given)
    metric_bytes = r["metric_bytes"] if not args.only else alg[args.only]
    ms_ev, ms_wall, ms_step, per_pass = r["ms_ev"], r["ms_wall"], r["ms_step"], r["per_pass_ms"]
    value = metric_bytes / (ms_step * 1e-3) / 1e9
    in_step = {k: v for k, v in per_pass.items() if k in step_passes}
    dominant = max(in_step, key=in_step.get)
    achieved = alg[dominant] / (per_pass[dominant] * 1e-3) / 1e9
    traffic = MEASURED_TRAFFIC_BYTES.get(args.workload, {}).get(dominant) if dtype == torch.float32 else None
    flops = {"fwd": 1, "bwi": 1, "bww": 1, "bwd": 2}
    roofline = {"bound": "hbm", "kernel": ENTRY[dominant], "kernels": KERNELS[dominant],
                "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": traffic, "traffic_profiled_build": TRAFFIC_PROFILED_BUILD,
                "algorithmic_bytes_per_launch": alg[dominant],
                "avg_us": round(per_pass[dominant] * 1e3, 2),
                "per_pass_us": {k: round(v * 1e3, 2) for k, v in per_pass.items()},
                "per_pass_GBs": {k: round(alg[k] / (v * 1e-3) / 1e9, 1) for k, v in per_pass.items()},
                "per_pass_TFLOPs": {k: round(flops[k] * Wk.algorithmic_flops(layer) / (v * 1e-3) / 1e12, 2)
                                    for k, v in per_pass.items()}}
    if dominant == "bwd":
        # scc_backward performs two passes of the metric in one call and has to read dy only once: `frac` above prices
        # it by the bytes that call must move; by the metric's own accounting (each pass's tensors once per pass, as in
        # `value`) the same time is worth the bytes of grad-input plus grad-weight
        by_pass = alg["bwi"] + alg["bww"]
        roofline["by_the_metrics_per_pass_accounting"] = {
            "algorithmic_bytes": by_pass, "GBs": round(by_pass / (per_pass["bwd"] * 1e-3) / 1e9, 1),
            "frac": round(by_pass / (per_pass["bwd"] * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
            "note": "grad-input + grad-weight counted as two passes (dy once per pass); not the call's real traffic"}

    out = {"metric": "SCC fwd+bwd GB/s & fraction of HBM peak, N=128 Cin=Cout=256 16x16 fp32",
           "value": round(value, 1), "unit": "GB/s", "n_gpus": 1, "steps": K, "warmup": W,
           "ms_per_step": round(ms_step, 5), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
           "dtype": "f32" if dtype == torch.float32 else "bf16", "data": "synthetic",
           "config": {"workload": "configs[1]: %s" % layer.name if args.workload == "metric" else layer.name,
                      "N": layer.N, "Cin": layer.Cin, "Cout": layer.Cout, "H": layer.H, "W": layer.W,
                      "cg": layer.cg, "co": layer.co, "passes": "+".join(ENTRY[p] for p in step_passes),
                      "buffer_sets_rotated": R, "graph_replays_timed": r["replays"],
                      "launch": "eager" if args.eager else "hip_graph"},
           "frac_of_hbm_peak": round(value / HBM_PEAK_GBS, 4),
           "bytes_accounting": {"value_counts": metric_bytes,
                                "note": "the metric's algorithmic bytes: forward, grad-input and grad-weight, each "
                                        "tensor of each pass once (3 x 67.17 MB at the metric layer)",
                                "bytes_the_step_must_move": sum(alg[p] for p in step_passes),
                                "GBs_of_bytes_the_step_must_move": round(sum(alg[p] for p in step_passes) /
                                                                         (ms_step * 1e-3) / 1e9, 1)},
           "ms_per_step_events": round(ms_ev, 5), "ms_per_step_wall": round(ms_wall, 5),
           "ms_per_step_median_replay": round(r["ms_median"], 5),
           "roofline": roofline, "paper_context": PAPER_CONTEXT}
    if "three_pass" in r:
        t3 = r["three_pass"]
        out["three_separate_passes"] = {"passes": "scc_forward+scc_backward_input+scc_backward_weight",
                                        "ms_per_step": round(t3["ms_step"], 5),
                                        "ms_per_step_events": round(t3["ms_ev"], 5),
                                        "ms_per_step_median_replay": round(t3["ms_median"], 5),
                                        "value": round(metric_bytes / (t3["ms_step"] * 1e-3) / 1e9, 1),
                                        "frac_of_hbm_peak": round(metric_bytes / (t3["ms_step"] * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)}
    if "copy" in r:
        c = r["copy"]
        # three passes at the rate of a plain copy of one activation tensor into another (each pass moves that much)
        ceil_ms = 3 * c["small_us"] * 1e-3
        out["copy_ceiling"] = {"what": "plain device copy kernel in the same run: one activation tensor into another on "
                                       "the same rotating buffers, and 1 GiB into 1 GiB",
                               "small_MiB_each_way": round(c["small_bytes_each_way"] / 2 ** 20, 2),
                               "small_us": round(c["small_us"], 2), "small_GBs": round(c["small_GBs"], 1),
                               "large_GiB_each_way": 1, "large_us": round(c["large_us"], 1),
                               "large_GBs": round(c["large_GBs"], 1),
                               "us_for_three_passes_at_small_copy_rate": round(ceil_ms * 1e3, 2)}
        out["frac_of_copy_ceiling"] = round(ceil_ms / ms_step, 4) if not args.only else None

    if not args.no_cpu_baseline:
        sec, reps, threads = oracle_step_seconds(Wk, layer, args.cpu_seconds)
        out["cpu_baseline"] = {"value": round(metric_bytes / sec / 1e9, 3), "unit": "GB/s", "cores": threads,
                               "kind": "oracle", "sample": "%d full steps (forward + grad-input + grad-weight) of the "
                               "same layer, fp64 oracle, %.1f s" % (reps, sec * reps), "ms_per_step": round(sec * 1e3, 2)}
        # one host thread, a bounded sample, in this process: the OpenMP runtime the oracle links is told to use one
        try:
            gomp = ctypes.CDLL("libgomp.so.1")
            gomp.omp_set_num_threads(1)
            ns = min(layer.N, 8)
            s1, n1, t1 = oracle_step_seconds(Wk, layer, 4.0, 50, sample_n=ns)
            gomp.omp_set_num_threads(threads)
            out["cpu_baseline"]["one_thread"] = {"ms_per_step_scaled_to_layer": round(s1 * 1e3 * layer.N / ns, 1),
                                                 "cores": t1, "sample": "%d steps on %d of %d samples" % (n1, ns, layer.N),
                                                 "value": round(metric_bytes / (s1 * layer.N / ns) / 1e9, 3)}
        except OSError as e:   # the baseline is context, never a reason to lose the measurement
            out["cpu_baseline"]["one_thread"] = {"error": repr(e)}
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
