#!/usr/bin/env python3
"""Benchmark of the fp32 convolution hot path on one MI355X.

A step is one pass of the whole hot path over one batch of synthetic input: forward,
backward-data and backward-weight of one layer, enqueued back to back on one stream with
inputs resident in HBM.  The default workload is the ResNet-style down-sampling layer
(N=128, 32x32x64 -> 16x16x128, 3x3, stride 2, pad 1).  Prints ONE JSON line on stdout.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload C2] [--no-cpu-baseline]
  python bench.py --table [cfg2 cfg3 ...] [--with-oracle]   per-layer, per-operator table (stderr + JSON line)
  python bench.py --workload cfg5           a whole configuration back to back (VGG-16: 39 operators per step)
  python bench.py --regret C2,V8            planner pick against an exhaustive tile / order / slice sweep
  python bench.py --streams                 independent operators on separate streams vs one stream
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

import workloads as wl  # noqa: E402

PEAK_FP32_MFMA_TFLOPS = 157.3   # 256 CU x 256 FLOP/clk x 2.4 GHz (published dense fp32 matrix peak)
PEAK_HBM_GBS = 8000.0
OPS = ("fwd", "bwd_data", "bwd_weight")
# HBM bytes per operator launch of the default workload (C2), from FETCH_SIZE + WRITE_SIZE scaled by a
# 256 MiB copy (profiles/bench_C2_kernel_trace.md); bwd_weight = main kernel + slice reduce.
MEASURED_TRAFFIC_BYTES = {"C2": {"fwd": 56.3e6 + 16.8e6, "bwd_data": 43.0e6 + 33.6e6,
                                 "bwd_weight": 84.4e6 + 8.3e6 + 8.3e6 + 0.3e6}}
KERNEL_OF_OP = {"fwd": "gather_gemm_kernel<fwd>", "bwd_data": "gather_gemm_kernel<bwd_data>",
                "bwd_weight": "wgrad_fast_kernel + slice_reduce_kernel"}


def log(*a):
    print(*a, file=sys.stderr, flush=True)


class LayerRunner:
    """Device tensors + workspace for one layer; enqueues operators through the C ABI binding."""

    def __init__(self, layer, mc, torch, random_fill=False):
        self.layer, self.mc, self.torch = layer, mc, torch
        self.desc = mc.make_desc(layer.N, layer.IH, layer.IW, layer.IC, layer.OC, layer.FH, layer.FW,
                                 layer.stride, layer.pad)
        if random_fill:   # timing-only tensors: same distributions, generated on the host once
            rng = np.random.default_rng(wl.stream_key(layer.name) & 0xffffffff)
            host = {"X": rng.standard_normal(layer.x_shape, dtype=np.float32),
                    "W": rng.standard_normal(layer.w_shape, dtype=np.float32) * np.float32(np.sqrt(2.0 / layer.K)),
                    "G": rng.standard_normal(layer.y_shape, dtype=np.float32)}
        else:
            host = wl.make_inputs(layer)
        self.host = host
        self.X = torch.from_numpy(host["X"]).cuda()
        self.W = torch.from_numpy(host["W"]).cuda()
        self.G = torch.from_numpy(host["G"]).cuda()
        self.Y = torch.empty(layer.y_shape, dtype=torch.float32, device="cuda")
        self.dX = torch.empty(layer.x_shape, dtype=torch.float32, device="cuda")
        self.dW = torch.empty(layer.w_shape, dtype=torch.float32, device="cuda")
        opcodes = {"fwd": mc.OP_FWD, "bwd_data": mc.OP_BWD_DATA, "bwd_weight": mc.OP_BWD_WEIGHT}
        self.plans = {op: mc.conv2d_query_plan(opcodes[op], self.desc) for op in OPS}
        need = max(p.workspace_bytes for p in self.plans.values())
        self.ws = torch.empty(max(need, 16), dtype=torch.uint8, device="cuda")

    def run(self, op, stream=None, ws=None):
        mc = self.mc
        ws = self.ws if ws is None else ws
        if op == "fwd":
            mc.conv2d_fwd(self.X, self.W, self.Y, self.desc, ws=ws, stream=stream)
        elif op == "bwd_data":
            mc.conv2d_bwd_data(self.G, self.W, self.dX, self.desc, ws=ws, stream=stream)
        else:
            mc.conv2d_bwd_weight(self.X, self.G, self.dW, self.desc, ws=ws, stream=stream)

    def step(self):
        for op in OPS:
            self.run(op)

    def event_ms(self, fn, launches=100, warm=20, batches=5):
        """Median over `batches` of the average milliseconds per call of fn, each batch `launches`
        calls between two events on the launch stream, after `warm` untimed calls."""
        torch = self.torch
        for _ in range(warm):
            fn()
        out = []
        for _ in range(batches):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            torch.cuda.synchronize()
            e0.record()
            for _ in range(launches):
                fn()
            e1.record()
            torch.cuda.synchronize()
            out.append(e0.elapsed_time(e1) / launches)
        return sorted(out)[len(out) // 2]

    def spin_up(self, seconds=0.2):
        """Keep the GPU busy until its clock governor has settled: the shader clock climbs for
        tens of milliseconds after an idle period, and kernels timed before that run 10-15 % slow."""
        t0 = time.perf_counter()
        while time.perf_counter() - t0 < seconds:
            for _ in range(20):
                self.step()
            self.torch.cuda.synchronize()


def cpu_baseline(layer, host, min_seconds=12.0):
    """The oracle as it stands, timed on the host cores on the same layer (all three operators),
    repeated until about min_seconds of wall time have passed."""
    import oracle
    s, p = layer.stride, layer.pad
    repeats = 0
    t0 = time.perf_counter()
    while True:
        oracle.conv2d_fwd(host["X"], host["W"], s, p)
        oracle.conv2d_bwd_data(host["G"], host["W"], (layer.IH, layer.IW), s, p)
        oracle.conv2d_bwd_weight(host["X"], host["G"], (layer.FH, layer.FW), s, p)
        repeats += 1
        dt = time.perf_counter() - t0
        if dt >= min_seconds or repeats >= 200:
            break
    return {"value": round(3 * layer.flops * repeats / dt / 1e12, 6), "unit": "TFLOP/s",
            "cores": oracle.num_threads(), "kind": "oracle",
            "sample": "%d x (fwd+bwd_data+bwd_weight) of %s at full size, %.1f s wall"
                      % (repeats, layer.name, dt)}


def op_bytes(l, op):
    """Minimum algorithmic HBM bytes of one operator: each operand and the result touched once."""
    x, w, y = l.N * l.IH * l.IW * l.IC, l.OC * l.K, l.M * l.OC
    if l.FH == 1 and l.FW == 1 and l.stride > 1 and op != "bwd_data":
        x = l.M * l.IC            # a strided 1x1 filter reads only every stride-th pixel
    return 4 * (x + w + y)


def oracle_ms(layer, host, op):
    import oracle
    s, p = layer.stride, layer.pad
    t0 = time.perf_counter()
    if op == "fwd":
        oracle.conv2d_fwd(host["X"], host["W"], s, p)
    elif op == "bwd_data":
        oracle.conv2d_bwd_data(host["G"], host["W"], (layer.IH, layer.IW), s, p)
    else:
        oracle.conv2d_bwd_weight(host["X"], host["G"], (layer.FH, layer.FW), s, p)
    return (time.perf_counter() - t0) * 1e3


def table(mc, torch, cfg_names, with_oracle=False, with_epilogue=False):
    """Every layer x operator: warm figure (median of 5 batches of 100 launches on one buffer set)
    and, for the rows that HBM bandwidth bounds, a cold figure that rotates over enough distinct
    buffer sets to exceed the 256 MB Infinity Cache."""
    rows = []
    seen = set()
    ridge = PEAK_FP32_MFMA_TFLOPS * 1e3 / PEAK_HBM_GBS          # FLOP per byte
    log("%-5s %-10s %9s %9s %7s %7s %9s %10s  %s" % ("layer", "op", "ms", "TFLOP/s", "%peak", "GB/s",
                                                     "cold ms", "oracle ms", "plan"))
    for cfg in cfg_names:
        for layer in wl.CONFIGS[cfg]:
            if layer.name in seen:
                continue
            seen.add(layer.name)
            r = LayerRunner(layer, mc, torch, random_fill=True)
            if not rows or with_oracle:
                r.spin_up()      # the oracle's seconds on the host let the clock governor fall back
            hbm_bound = layer.flops / op_bytes(layer, "fwd") < 2.0 * ridge
            sets = [r]
            if hbm_bound:
                per_set = 4 * (layer.N * layer.IH * layer.IW * layer.IC + layer.M * layer.OC)
                sets += [LayerRunner(layer, mc, torch, random_fill=True)
                         for _ in range(min(16, int(320e6 // per_set)))]
            for op in OPS:
                ms = r.event_ms(lambda: r.run(op))
                cold = None
                if hbm_bound:
                    state = {"i": 0}

                    def rotate():
                        state["i"] = (state["i"] + 1) % len(sets)
                        sets[state["i"]].run(op)
                    cold = r.event_ms(rotate)
                tf = layer.flops / ms / 1e9
                pl = r.plans[op]
                plan = "v%d %dx%d s%d pm%d g%d" % (pl.variant, pl.tile_m, pl.tile_n, pl.split,
                                                   pl.pos_major, pl.grid)
                gbs = op_bytes(layer, op) / ms / 1e6
                oms = None
                rows.append({"layer": layer.name, "op": op, "ms": round(ms, 5), "tflops": round(tf, 2),
                             "pct_peak": round(100 * tf / PEAK_FP32_MFMA_TFLOPS, 1),
                             "gbs": round(gbs, 1), "cold_ms": None if cold is None else round(cold, 5),
                             "cold_gbs": None if cold is None else round(op_bytes(layer, op) / cold / 1e6, 1),
                             "oracle_ms": None if oms is None else round(oms, 2), "plan": plan})
                log("%-5s %-10s %9.4f %9.2f %7.1f %7.0f %9s %10s  %s"
                    % (layer.name, op, ms, tf, 100 * tf / PEAK_FP32_MFMA_TFLOPS, gbs,
                       "-" if cold is None else "%.4f" % cold, "-" if oms is None else "%.1f" % oms, plan))
            if with_oracle:      # after the layer's GPU timing, so that it does not cool the clocks in between
                for row in rows[-len(OPS):]:
                    row["oracle_ms"] = round(oracle_ms(layer, r.host, row["op"]), 2)
                    log("%-5s %-10s oracle %.1f ms" % (layer.name, row["op"], row["oracle_ms"]))
            if with_epilogue:   # forward with bias + leaky-ReLU in the epilogue, against the plain forward
                bias = torch.zeros(layer.OC, dtype=torch.float32, device="cuda")
                ms = r.event_ms(lambda: mc.conv2d_fwd_bias_act(r.X, r.W, bias, r.Y, r.desc, 0.01, ws=r.ws))
                tf = layer.flops / ms / 1e9
                rows.append({"layer": layer.name, "op": "fwd_bias_act", "ms": round(ms, 5), "tflops": round(tf, 2),
                             "pct_peak": round(100 * tf / PEAK_FP32_MFMA_TFLOPS, 1)})
                log("%-5s %-10s %9.4f %9.2f %7.1f" % (layer.name, "fwd+b+act", ms, tf, 100 * tf / PEAK_FP32_MFMA_TFLOPS))
            del r, sets
            torch.cuda.empty_cache()
    if with_oracle:
        import oracle
        log("oracle: plain C loop nests, fp64 accumulation, %d OpenMP threads" % oracle.num_threads())
    return rows


def streams_report(mc, torch):
    """Independent operators on separate streams against the same operators on one stream: the three
    inception-style branches of configuration 4 on one shared input (forward), and backward-data
    next to backward-weight for a few layers.  Prints one JSON line."""
    layers = {l.name: l for l in wl.all_layers()}
    out = []

    def timed(fn, launches=100, batches=5):
        for _ in range(20):
            fn()
        ts = []
        for _ in range(batches):
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(launches):
                fn()
            torch.cuda.synchronize()
            ts.append((time.perf_counter() - t0) * 1e3 / launches)
        return sorted(ts)[len(ts) // 2]

    # forward of the 1x1, 3x3, 5x5 branches, one input tensor
    rs = [LayerRunner(layers[n], mc, torch, random_fill=True) for n in ("C4a", "C4b", "C4c")]
    rs[0].spin_up()
    for r in rs[1:]:
        r.X = rs[0].X
    sts = [torch.cuda.Stream() for _ in rs]
    cur = torch.cuda.current_stream()

    def serial():
        for r in rs:
            r.run("fwd")

    def parallel():     # no event between the streams inside the timed loop: each stream is its own queue
        for r, st in zip(rs, sts):
            r.run("fwd", stream=st)
    a, b = timed(serial), timed(parallel)
    out.append({"case": "fwd of C4a | C4b | C4c on one input", "serial_ms": round(a, 5), "streams_ms": round(b, 5),
                "gain": round(a / b, 3)})
    log("%-44s serial %.4f ms   3 streams %.4f ms   x%.3f" % (out[-1]["case"], a, b, a / b))
    del rs
    for name in ("C2", "C3c", "C4a", "V11", "V5"):
        r = LayerRunner(layers[name], mc, torch, random_fill=True)
        # own workspace per operator: they run at the same time
        need = r.plans["bwd_weight"].workspace_bytes
        ws2 = torch.empty(max(need, 16), dtype=torch.uint8, device="cuda")
        s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()

        def serial2():
            r.run("bwd_data")
            r.run("bwd_weight")

        def parallel2():
            r.run("bwd_data", stream=s1)
            r.run("bwd_weight", stream=s2, ws=ws2)
        a, b = timed(serial2), timed(parallel2)
        out.append({"case": "bwd_data | bwd_weight of %s" % name, "serial_ms": round(a, 5),
                    "streams_ms": round(b, 5), "gain": round(a / b, 3)})
        log("%-44s serial %.4f ms   2 streams %.4f ms   x%.3f" % (out[-1]["case"], a, b, a / b))
        del r
        torch.cuda.empty_cache()
    return out


def regret_report(mc, torch, names):
    """Planner pick against an exhaustive sweep of compiled tiles x row orders x slice counts, per
    layer and operator (the overrides conv2d_set_tile / conv2d_set_tuning drive the sweep)."""
    import itertools
    layers = {l.name: l for l in wl.all_layers()}
    gather_tiles = [(128, 128), (128, 64), (64, 64), (128, 32)]
    wgrad_tiles = [(128, 128), (64, 128), (128, 64), (64, 64), (32, 128)]
    splits = (1, 2, 3, 4, 6, 8, 12, 16, 24, 32, 48, 64, 96, 128, 192, 256)
    opcodes = {"fwd": mc.OP_FWD, "bwd_data": mc.OP_BWD_DATA, "bwd_weight": mc.OP_BWD_WEIGHT}
    rows = []
    try:
        for name in names:
            r = LayerRunner(layers[name], mc, torch, random_fill=True)
            r.spin_up()
            for op in OPS:
                mc.conv2d_set_tile(0, 0, -1)
                mc.conv2d_set_tuning(mc.VARIANT_AUTO, 0)
                pl0 = mc.conv2d_query_plan(opcodes[op], r.desc)
                if pl0.workspace_bytes > r.ws.numel():
                    r.ws = torch.empty(pl0.workspace_bytes, dtype=torch.uint8, device="cuda")
                base = r.event_ms(lambda: r.run(op), 50, 10, 3)
                best, best_plan, seen = base, "planner", set()
                for (bm, bn), pm in itertools.product(wgrad_tiles if op == "bwd_weight" else gather_tiles, (0, 1)):
                    for sp in splits:
                        mc.conv2d_set_tile(bm, bn, pm)
                        mc.conv2d_set_tuning(mc.VARIANT_AUTO, sp)
                        pl = mc.conv2d_query_plan(opcodes[op], r.desc)
                        key = (pl.tile_m, pl.tile_n, pl.pos_major, pl.split)
                        if key in seen or pl.variant != mc.VARIANT_MFMA or not 128 <= pl.grid <= 8192:
                            continue
                        seen.add(key)
                        if pl.workspace_bytes > (1 << 29):
                            continue
                        if pl.workspace_bytes > r.ws.numel():
                            r.ws = torch.empty(pl.workspace_bytes, dtype=torch.uint8, device="cuda")
                        ms = r.event_ms(lambda: r.run(op), 30, 5, 3)
                        if ms < best:
                            best, best_plan = ms, "%dx%d pm%d s%d g%d" % (key + (pl.grid,))
                rows.append({"layer": name, "op": op, "planner_ms": round(base, 5), "best_ms": round(best, 5),
                             "best_plan": best_plan, "regret_pct": round(100 * (base / best - 1), 1),
                             "planner_plan": "%dx%d pm%d s%d g%d" % (pl0.tile_m, pl0.tile_n, pl0.pos_major,
                                                                    pl0.split, pl0.grid)})
                log("%-4s %-10s planner %-24s %.4f ms | best %.4f ms %-24s | regret %.1f%%"
                    % (name, op, rows[-1]["planner_plan"], base, best, best_plan, rows[-1]["regret_pct"]))
            del r
            torch.cuda.empty_cache()
    finally:
        mc.conv2d_set_tile(0, 0, -1)
        mc.conv2d_set_tuning(mc.VARIANT_AUTO, 0)
    return rows


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=1000)
    ap.add_argument("--warmup", type=int, default=200)
    ap.add_argument("--workload", default="C2")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--table", nargs="*", default=None, metavar="CFG")
    ap.add_argument("--regret", default=None, metavar="LAYER,LAYER",
                    help="planner pick against an exhaustive sweep of tiles, row orders and slice counts")
    ap.add_argument("--graph", action="store_true",
                    help="with --workload cfgN: capture one step into a HIP graph and time its replay")
    ap.add_argument("--streams", action="store_true",
                    help="independent operators on separate streams vs one stream (inception branches, "
                         "backward-data next to backward-weight)")
    ap.add_argument("--with-epilogue", action="store_true",
                    help="with --table: also time forward with bias + leaky-ReLU in the epilogue")
    ap.add_argument("--with-oracle", action="store_true",
                    help="with --table: also time the CPU oracle once per layer and operator")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="run a plain 256 MiB device copy 5 times (reference for the HBM byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build measures one GPU only (--gpus 1); the hot path has no "
                 "multi-GPU part (it would shard by batch, with one all-reduce of dW per layer)")

    import torch
    import paper_2305_08819_amd as mc
    mc.load()   # fails loudly if the HIP library is not built
    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")

    if args.calibrate_copy:
        # known traffic: 256 MiB read + 256 MiB written per copy; used to scale FETCH_SIZE / WRITE_SIZE
        src = torch.ones(64 * 1024 * 1024, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"calibrate_copy_bytes_each_way": src.numel() * 4, "copies": 5}))
        return

    if args.streams:
        print(json.dumps({"streams": streams_report(mc, torch)}))
        return

    if args.regret:
        print(json.dumps({"regret": regret_report(mc, torch, args.regret.split(","))}))
        return

    if args.table is not None:
        names = args.table or list(wl.CONFIGS)
        rows = table(mc, torch, names, args.with_oracle, args.with_epilogue)
        print(json.dumps({"table": rows}))
        return

    if args.workload in wl.CONFIGS:
        # a whole configuration back to back on one stream (e.g. cfg5: the 39 operators of VGG-16)
        layers = wl.CONFIGS[args.workload]
        rs = [LayerRunner(l, mc, torch, random_fill=True) for l in layers]
        rs[0].spin_up()

        def stack():
            for r in rs:
                r.step()
        for _ in range(max(args.warmup // 10, 5)):
            stack()
        steps = max(args.steps // 10, 10)
        run = stack
        if args.graph:
            # the library only enqueues kernels (no allocation, no memset, no synchronisation), so a
            # whole step can be captured once and replayed with one launch
            side = torch.cuda.Stream()
            side.wait_stream(torch.cuda.current_stream())
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.stream(side):
                stack()                              # first call on this stream outside the capture
                torch.cuda.synchronize()
                with torch.cuda.graph(graph, stream=side):
                    stack()
            torch.cuda.synchronize()
            run = graph.replay
            for _ in range(5):
                run()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            run()
        torch.cuda.synchronize()
        ms = (time.perf_counter() - t0) * 1e3 / steps
        flop = 3 * sum(l.flops for l in layers)
        print(json.dumps({"metric": "TFLOP/s and % FP32 MFMA peak per conv op (fwd/dgrad/wgrad), CIFAR shapes",
                          "value": round(flop / ms / 1e9, 3), "unit": "TFLOP/s", "n_gpus": 1, "steps": steps,
                          "ms_per_step": round(ms, 5), "higher_is_better": True, "dtype": "f32", "data": "synthetic",
                          "config": {"workload": "%s: %d layers x (fwd+bwd_data+bwd_weight) back to back on one stream%s"
                                                 % (args.workload, len(layers), ", replayed as one HIP graph" if args.graph else ""),
                                     "flop_per_step": flop,
                                     "pct_fp32_mfma_peak": round(100 * flop / ms / 1e9 / PEAK_FP32_MFMA_TFLOPS, 2)}}))
        return

    layer = {l.name: l for l in wl.all_layers()}[args.workload]
    r = LayerRunner(layer, mc, torch)

    r.spin_up()          # clock governor settled before anything is timed
    for _ in range(args.warmup):
        r.step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        r.step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_step = dt * 1e3 / args.steps
    value = 3 * layer.flops / (ms_step * 1e-3) / 1e12

    # per-operator event timing (each operator alone on the launch stream); the slowest is the
    # dominant kernel of the step
    per_op = {op: r.event_ms(lambda op=op: r.run(op)) for op in OPS}
    dom = max(per_op, key=per_op.get)
    achieved = layer.flops / per_op[dom] / 1e9
    out = {
        "metric": "TFLOP/s and % FP32 MFMA peak per conv op (fwd/dgrad/wgrad), CIFAR shapes",
        "value": round(value, 3), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_step, 5), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": "%s: N=%d %dx%dx%d -> %dx%dx%d, %dx%d filter, stride %d, pad %d, "
                               "fwd+bwd_data+bwd_weight per step"
                               % (layer.name, layer.N, layer.IH, layer.IW, layer.IC, layer.OH, layer.OW,
                                  layer.OC, layer.FH, layer.FW, layer.stride, layer.pad),
                   "flop_per_step": 3 * layer.flops,
                   "pct_fp32_mfma_peak": round(100 * value / PEAK_FP32_MFMA_TFLOPS, 2)},
        "per_op": {op: {"ms": round(per_op[op], 5),
                        "tflops": round(layer.flops / per_op[op] / 1e9, 2),
                        "pct_peak": round(100 * layer.flops / per_op[op] / 1e9 / PEAK_FP32_MFMA_TFLOPS, 1),
                        "split": r.plans[op].split, "tile": [r.plans[op].tile_m, r.plans[op].tile_n]}
                   for op in OPS},
        # achieved = nominal FLOP of the slowest operator / its event-timed duration; for a sliced
        # operator that duration includes the slice-reduce kernel, so the figure is conservative
        "roofline": {"bound": "mfma", "kernel": KERNEL_OF_OP[dom], "operator": dom,
                     "achieved": round(achieved, 2), "peak": PEAK_FP32_MFMA_TFLOPS, "unit": "TFLOP/s",
                     "frac": round(achieved / PEAK_FP32_MFMA_TFLOPS, 4),
                     "traffic": MEASURED_TRAFFIC_BYTES.get(layer.name, {}).get(dom)},
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(layer, r.host)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
