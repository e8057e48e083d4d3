#!/usr/bin/env python3
"""Benchmark of the fp32 convolution hot path on one MI355X.

A step is one pass of the whole hot path over one batch of synthetic input: forward,
backward-data and backward-weight of every layer of the workload, enqueued back to back on one
stream with inputs resident in HBM.  The default workload is the largest configuration, the
VGG-16-shaped stack (13 layers of 3x3 convolutions, N=128: 39 operators per step).  Prints ONE
JSON line on stdout.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload cfg5|C2|...] [--no-cpu-baseline]
  python bench.py --table [cfg2 cfg3 ...] [--with-oracle]   per-layer, per-operator table (stderr + JSON line)
  python bench.py --workload cfg5 --graph   the step captured once into a HIP graph and replayed
  python bench.py --regret C2,V8            planner pick against an exhaustive tile / order / slice sweep
  python bench.py --streams                 independent operators on separate streams vs one stream
  python bench.py --mfma-peak               register-only fp32 MFMA loop: the matrix rate the chip sustains
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

METRIC = "TFLOP/s and % FP32 MFMA peak per conv op (fwd/dgrad/wgrad), CIFAR shapes"
PEAK_FP32_MFMA_TFLOPS = 157.3   # 256 CU x 256 FLOP/clk x 2.4 GHz (published dense fp32 matrix peak)
PEAK_HBM_GBS = 8000.0
OPS = ("fwd", "bwd_data", "bwd_weight")
# HBM bytes per launch of each kernel, written from rocprofv3 FETCH_SIZE / WRITE_SIZE runs of this
# same command (the summary beside it gives the commands and the copy calibration)
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "bench_cfg5_hbm_traffic.json")


def kernel_name(layer, op, plan, mc):
    """Name of the main kernel a plan launches, spelled as rocprofv3 prints it."""
    b = lambda v: "true" if v else "false"   # noqa: E731
    t = (plan.tile_m, plan.tile_n)
    if plan.kernel == mc.KERNEL_DIRECT:
        return "direct_%s_kernel" % op
    if plan.kernel == mc.KERNEL_FIRST_LAYER:
        return {"fwd": "fwd_small_ic_kernel<false>", "bwd_data": "bwd_data_small_ic_kernel",
                "bwd_weight": "wgrad_small_ic_kernel"}[op]
    if plan.kernel == mc.KERNEL_WGRAD_FAST:
        return "wgrad_fast_kernel<%d, %d, %s, %s>" % (t + (b(plan.pos_major), b(layer.OW > 32)))
    if plan.kernel == mc.KERNEL_WGRAD:
        return "wgrad_kernel<%d, %d, %s>" % (t + (b(layer.IC % 4),))
    bwd = op == "bwd_data"
    waves_m = 4 if plan.tile_n == 32 else 2
    if plan.kernel == mc.KERNEL_GATHER_ELEM:
        return "gather_elem_kernel<%d, %d, %d, %s>" % (t + (waves_m, b(bwd)))
    src, dst = (layer.OC, layer.IC) if bwd else (layer.IC, layer.OC)
    belem = bwd and dst % 4 != 0
    return "gather_gemm_kernel<%d, %d, %d, %s, %s, %s>" % (t + (waves_m, b(bwd), b(belem), b(belem or src % 32 != 0)))


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

    def spin_up(self, seconds=0.2, step=None):
        """Keep the GPU busy until its clock governor has settled: the shader clock climbs for
        tens of milliseconds after an idle period, and kernels timed before that run 10-15 % slow."""
        step = step or self.step
        t0 = time.perf_counter()
        while time.perf_counter() - t0 < seconds:
            for _ in range(5):
                step()
            self.torch.cuda.synchronize()


def cpu_baseline(runners, budget_seconds=25.0):
    """The oracle as it stands, timed on the host cores: one pass of all three operators over the
    workload's layers at full size, in layer order, stopping after the layer during which the
    budget runs out (a bounded sample; what was covered is stated)."""
    import oracle
    flop, done = 0, []
    t0 = time.perf_counter()
    for r in runners:
        l, host = r.layer, r.host
        s, p = l.stride, l.pad
        oracle.conv2d_fwd(host["X"], host["W"], s, p)
        oracle.conv2d_bwd_data(host["G"], host["W"], (l.IH, l.IW), s, p)
        oracle.conv2d_bwd_weight(host["X"], host["G"], (l.FH, l.FW), s, p)
        flop += 3 * l.flops
        done.append(l.name)
        if time.perf_counter() - t0 >= budget_seconds:
            break
    dt = time.perf_counter() - t0
    what = "all %d layers" % len(done) if len(done) == len(runners) else "layers %s..%s" % (done[0], done[-1])
    return {"value": round(flop / dt / 1e12, 6), "unit": "TFLOP/s", "cores": oracle.num_threads(), "kind": "oracle",
            "sample": "one pass of fwd+bwd_data+bwd_weight over %s at full size, %.1f nominal GFLOP in %.1f s wall"
                      % (what, flop / 1e9, dt)}


def op_bytes(l, op):
    """Minimum algorithmic HBM bytes of one operator: each operand and the result touched once."""
    x, w, y = l.N * l.IH * l.IW * l.IC, l.OC * l.K, l.M * l.OC
    if l.FH == 1 and l.FW == 1 and l.stride > 1 and op != "bwd_data":
        x = l.M * l.IC            # a strided 1x1 filter reads only every stride-th pixel
    return 4 * (x + w + y)


def oracle_ms(layer, host, op):
    """(milliseconds, result) of the CPU oracle for one operator at full size."""
    import oracle
    s, p = layer.stride, layer.pad
    t0 = time.perf_counter()
    if op == "fwd":
        ref = oracle.conv2d_fwd(host["X"], host["W"], s, p)
    elif op == "bwd_data":
        ref = oracle.conv2d_bwd_data(host["G"], host["W"], (layer.IH, layer.IW), s, p)
    else:
        ref = oracle.conv2d_bwd_weight(host["X"], host["G"], (layer.FH, layer.FW), s, p)
    return (time.perf_counter() - t0) * 1e3, ref


def table(mc, torch, cfg_names, with_oracle=False, with_epilogue=False):
    """Every layer x operator: warm figure (median of 5 batches of 100 launches on one buffer set)
    and, for the rows that HBM bandwidth bounds, a cold figure that rotates over enough distinct
    buffer sets to exceed the 256 MB Infinity Cache."""
    rows = []
    seen = set()
    ridge = PEAK_FP32_MFMA_TFLOPS * 1e3 / PEAK_HBM_GBS          # FLOP per byte
    log("%-5s %-10s %9s %9s %7s %9s %7s %7s %9s %10s %9s %9s  %s"
        % ("layer", "op", "ms", "TFLOP/s", "%peak", "eff TF/s", "%peak", "GB/s", "cold ms", "oracle ms", "rel-L2", "max-abs", "plan"))
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
                tf, tfe = layer.flops / ms / 1e9, layer.effective_flops / ms / 1e9
                pl = r.plans[op]
                plan = "v%d %dx%d s%d pm%d o%d g%d" % (pl.variant, pl.tile_m, pl.tile_n, pl.split,
                                                       pl.pos_major, pl.order, pl.grid)
                gbs = op_bytes(layer, op) / ms / 1e6
                rows.append({"layer": layer.name, "op": op, "ms": round(ms, 5), "tflops": round(tf, 2),
                             "pct_peak": round(100 * tf / PEAK_FP32_MFMA_TFLOPS, 1),
                             "tflops_effective": round(tfe, 2),
                             "pct_peak_effective": round(100 * tfe / PEAK_FP32_MFMA_TFLOPS, 1),
                             "gbs": round(gbs, 1), "cold_ms": None if cold is None else round(cold, 5),
                             "cold_gbs": None if cold is None else round(op_bytes(layer, op) / cold / 1e6, 1),
                             "oracle_ms": None, "rel_l2": None, "max_abs": None, "plan": plan})
            if with_oracle:      # after the layer's GPU timing, so that it does not cool the clocks in between
                for row in rows[-len(OPS):]:
                    oms, ref = oracle_ms(layer, r.host, row["op"])
                    got = {"fwd": r.Y, "bwd_data": r.dX, "bwd_weight": r.dW}[row["op"]].cpu().numpy().astype(np.float64)
                    diff = got - ref
                    row["oracle_ms"] = round(oms, 2)
                    row["rel_l2"] = float("%.3g" % (np.linalg.norm(diff.ravel()) / np.linalg.norm(ref.ravel())))
                    row["max_abs"] = float("%.3g" % np.abs(diff).max())
            for row in rows[-len(OPS):]:
                log("%-5s %-10s %9.4f %9.2f %7.1f %9.2f %7.1f %7.0f %9s %10s %9s %9s  %s"
                    % (row["layer"], row["op"], row["ms"], row["tflops"], row["pct_peak"], row["tflops_effective"],
                       row["pct_peak_effective"], row["gbs"], "-" if row["cold_ms"] is None else "%.4f" % row["cold_ms"],
                       "-" if row["oracle_ms"] is None else "%.1f" % row["oracle_ms"],
                       "-" if row["rel_l2"] is None else "%.2e" % row["rel_l2"],
                       "-" if row["max_abs"] is None else "%.2e" % row["max_abs"], row["plan"]))
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
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="cfg5", help="a configuration (cfg1..cfg8) or one layer (C2, V9, ...)")
    ap.add_argument("--no-op-events", action="store_true",
                    help="skip the per-operator event timing behind the timed region (no per_op / roofline in the output)")
    ap.add_argument("--op-reps", type=int, default=50, help="launches per event-timed batch of one operator")
    ap.add_argument("--no-two-streams", action="store_true", help="skip the extra two-stream timing of the step")
    ap.add_argument("--mfma-peak", action="store_true",
                    help="register-only fp32 MFMA loop with 0..96 interleaved VALU instructions per 8 MFMAs")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--table", nargs="*", default=None, metavar="CFG")
    ap.add_argument("--regret", default=None, metavar="LAYER,LAYER",
                    help="planner pick against an exhaustive sweep of tiles, row orders and slice counts")
    ap.add_argument("--graph", action="store_true",
                    help="capture one step into a HIP graph and time its replay (no per-operator events)")
    ap.add_argument("--streams", action="store_true",
                    help="independent operators on separate streams vs one stream (inception branches, "
                         "backward-data next to backward-weight)")
    ap.add_argument("--with-epilogue", action="store_true",
                    help="with --table: also time forward with bias + leaky-ReLU in the epilogue")
    ap.add_argument("--with-oracle", action="store_true",
                    help="with --table: also time the CPU oracle once per layer and operator")
    ap.add_argument("--plain-order", action="store_true",
                    help="older workgroup order (longest first over the whole chip) instead of the per-XCD orders")
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

    if args.plain_order:
        mc.conv2d_set_order(0)

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

    if args.mfma_peak:
        print(json.dumps({"mfma_peak": mfma_peak_report(mc, torch)}))
        return

    layers = wl.CONFIGS[args.workload] if args.workload in wl.CONFIGS else \
        [{l.name: l for l in wl.all_layers()}[args.workload]]
    rs = [LayerRunner(l, mc, torch, random_fill=True) for l in layers]
    items = [(r, op) for r in rs for op in OPS]           # the launch order of a step

    def step():
        for r, op in items:
            r.run(op)

    rs[0].spin_up(step=step)     # clock governor settled before anything is timed
    steps, warmup = args.steps, args.warmup
    run = step
    if args.graph:
        # the library only enqueues kernels (no allocation, no memset, no synchronisation), so a
        # whole step can be captured once and replayed with one launch
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.stream(side):
            step()                                   # first call on this stream outside the capture
            torch.cuda.synchronize()
            with torch.cuda.graph(graph, stream=side):
                step()
        torch.cuda.synchronize()
        run = graph.replay
    for _ in range(warmup):
        run()
    torch.cuda.synchronize()

    # ---- the timed region: exactly `steps` steps between two synchronisations ------------------------
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    e0.record()
    for _ in range(steps):
        run()
    e1.record()
    torch.cuda.synchronize()
    ms_step = (time.perf_counter() - t0) * 1e3 / steps
    ms_step_events = e0.elapsed_time(e1) / steps
    flop_step = 3 * sum(l.flops for l in layers)
    eff_step = 3 * sum(l.effective_flops for l in layers)
    value = flop_step / ms_step / 1e9

    # ---- per-operator durations, right behind the timed region (clocks still settled) -----------------
    # Each operator of the step is launched `reps` times back to back between two events on the launch
    # stream, five times over; the median batch gives its average launch duration (main kernel plus,
    # for a sliced reduction, the combine kernel), which is what a kernel trace of this command shows.
    # Events between the operators of a step are not used: each costs about 3.5 us of idle GPU.
    per_op_ms = None
    if not args.no_op_events:
        per_op_ms = [r.event_ms(lambda r=r, op=op: r.run(op), launches=args.op_reps, warm=3, batches=5)
                     for r, op in items]

    out = {
        "metric": METRIC, "value": round(value, 3), "unit": "TFLOP/s", "n_gpus": 1, "steps": steps, "warmup": warmup,
        "ms_per_step": round(ms_step, 5), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": workload_text(args.workload, layers, args.graph),
                   "operators_per_step": len(items), "flop_per_step": flop_step,
                   "effective_flop_per_step": round(eff_step),
                   "pct_fp32_mfma_peak": round(100 * value / PEAK_FP32_MFMA_TFLOPS, 2),
                   "effective_tflops": round(eff_step / ms_step / 1e9, 3),
                   "pct_fp32_mfma_peak_effective": round(100 * eff_step / ms_step / 1e9 / PEAK_FP32_MFMA_TFLOPS, 2)},
    }
    out["ms_per_step_events"] = round(ms_step_events, 5)
    if not args.graph and not args.no_two_streams:
        # The same step with backward-weight on a second stream, next to forward + backward-data (the
        # paper's asynchronous operator submission; dX and dW of a layer do not depend on each other).
        # Reported beside the one-stream figure, which stays the headline value.
        sa, sb = torch.cuda.Stream(), torch.cuda.Stream()
        ws_b = [torch.empty(max(r.plans["bwd_weight"].workspace_bytes, 16), dtype=torch.uint8, device="cuda") for r in rs]

        def step2():
            for r, w in zip(rs, ws_b):
                r.run("fwd", stream=sa)
                r.run("bwd_data", stream=sa)
                r.run("bwd_weight", stream=sb, ws=w)
        torch.cuda.synchronize()
        for _ in range(max(warmup // 2, 3)):
            step2()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            step2()
        torch.cuda.synchronize()
        ms2 = (time.perf_counter() - t0) * 1e3 / steps
        out["two_streams"] = {"schedule": "fwd + bwd_data on one stream, bwd_weight on a second", "ms_per_step": round(ms2, 5),
                              "value": round(flop_step / ms2 / 1e9, 3),
                              "pct_fp32_mfma_peak": round(100 * flop_step / ms2 / 1e9 / PEAK_FP32_MFMA_TFLOPS, 2)}
    if per_op_ms is not None:
        per = []
        for (r, op), ms in zip(items, per_op_ms):
            l, pl = r.layer, r.plans[op]
            tf, tfe = l.flops / ms / 1e9, l.effective_flops / ms / 1e9
            per.append({"layer": l.name, "op": op, "ms": round(ms, 5), "tflops": round(tf, 2),
                        "pct_peak": round(100 * tf / PEAK_FP32_MFMA_TFLOPS, 1),
                        "tflops_effective": round(tfe, 2), "pct_peak_effective": round(100 * tfe / PEAK_FP32_MFMA_TFLOPS, 1),
                        "gbs": round(op_bytes(l, op) / ms / 1e6, 1),
                        "kernel": kernel_name(l, op, pl, mc), "tile": [pl.tile_m, pl.tile_n], "split": pl.split,
                        "pos_major": pl.pos_major, "grid": pl.grid})
        out["per_op"] = per
        out["per_op_sum_ms"] = round(sum(p["ms"] for p in per), 5)
        out["roofline"] = roofline(per, layers)
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(rs)
    print(json.dumps(out))


def workload_text(name, layers, graph):
    if len(layers) == 1:
        l = layers[0]
        return ("%s: N=%d %dx%dx%d -> %dx%dx%d, %dx%d filter, stride %d, pad %d, fwd+bwd_data+bwd_weight per step"
                % (l.name, l.N, l.IH, l.IW, l.IC, l.OH, l.OW, l.OC, l.FH, l.FW, l.stride, l.pad))
    what = {"cfg5": "VGG-16-shaped conv stack, N=128, 32x32x3 input, 13 layers of 3x3 pad-1 convolutions "
                    "(64,64,128,128,256x3,512x3,512x3 channels, maps 32x32 down to 2x2)"}.get(name, name)
    return "%s: %s; %d layers x (fwd+bwd_data+bwd_weight) back to back on one stream%s" % (
        name, what, len(layers), ", replayed as one HIP graph" if graph else "")


def roofline(per, layers):
    """The kernel with the largest share of the step: its launches' effective FLOP (in-range taps
    only; nominal x in-range share) over their event-timed durations, against the fp32 MFMA peak -
    or, where the step is dominated by an HBM-bound kernel, its algorithmic bytes against 8 TB/s."""
    by_layer = {l.name: l for l in layers}
    groups = {}
    for p in per:
        groups.setdefault(p["kernel"], []).append(p)
    kern, rows = max(groups.items(), key=lambda kv: sum(p["ms"] for p in kv[1]))
    ms = sum(p["ms"] for p in rows)
    nominal = sum(by_layer[p["layer"]].flops for p in rows)
    eff = sum(by_layer[p["layer"]].effective_flops for p in rows)
    nbytes = sum(op_bytes(by_layer[p["layer"]], p["op"]) for p in rows)
    ridge = PEAK_FP32_MFMA_TFLOPS * 1e3 / PEAK_HBM_GBS
    traffic = None
    if os.path.exists(TRAFFIC_FILE):
        t = json.load(open(TRAFFIC_FILE)).get("kernels", {}).get(kern)
        traffic = None if t is None else t["hbm_bytes_per_launch"]
    common = {"kernel": kern, "launches_per_step": len(rows), "avg_launch_us": round(1e3 * ms / len(rows), 3),
              "share_of_step": round(ms / sum(p["ms"] for p in per), 4),
              "includes_combine_pass_of_sliced_launches": any(p["split"] > 1 for p in rows),
              "traffic": traffic}
    if nominal / nbytes < ridge:
        a = nbytes / ms / 1e6
        return dict({"bound": "hbm", "achieved": round(a, 1), "peak": PEAK_HBM_GBS, "unit": "GB/s",
                     "frac": round(a / PEAK_HBM_GBS, 4)}, **common)
    a = eff / ms / 1e9
    return dict({"bound": "mfma", "achieved": round(a, 2), "peak": PEAK_FP32_MFMA_TFLOPS, "unit": "TFLOP/s",
                 "frac": round(a / PEAK_FP32_MFMA_TFLOPS, 4),
                 "achieved_nominal": round(nominal / ms / 1e9, 2),
                 "flop_counted": "effective: taps inside the image only (nominal 2*M*OC*K x in-range share)"}, **common)


def mfma_peak_report(mc, torch):
    """Register-only v_mfma_f32_32x32x2_f32 loop with 0 / 16 / 48 / 96 ordinary vector instructions
    per 8 matrix instructions, one and two workgroups per CU."""
    rows = []
    out = torch.empty(512 * 256, dtype=torch.float32, device="cuda")
    iters = 20000
    for wg_per_cu in (1, 2):
        for nv in (0, 16, 48, 96):
            wgs = 256 * wg_per_cu
            for _ in range(3):
                flop = mc.conv2d_probe_mfma_rate(nv, wgs, iters, out)
            torch.cuda.synchronize()
            best = 1e30
            for _ in range(5):
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                mc.conv2d_probe_mfma_rate(nv, wgs, iters, out)
                e1.record()
                torch.cuda.synchronize()
                best = min(best, e0.elapsed_time(e1))
            tf = flop / best / 1e9
            rows.append({"valu_per_8_mfma": nv, "workgroups_per_cu": wg_per_cu, "ms": round(best, 4),
                         "tflops": round(tf, 2), "pct_of_157.3": round(100 * tf / PEAK_FP32_MFMA_TFLOPS, 1)})
            log("MFMA loop, %2d VALU per 8 MFMA, %d workgroup(s) per CU: %8.3f ms  %6.1f TFLOP/s  (%.1f %% of 157.3)"
                % (nv, wg_per_cu, best, tf, 100 * tf / PEAK_FP32_MFMA_TFLOPS))
    return rows


if __name__ == "__main__":
    main()
