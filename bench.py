#!/usr/bin/env python3
"""Throughput of the SFC 3x3 int8 convolution hot path on one MI355X.

A step is one pass of the whole hot path (input-tile transform, transform-domain products,
output transform with dequantization or int8 requantization, NCHW store) over one batch of
synthetic ResNet-shaped input already resident in HBM.  Filter transforms are done once,
outside the timed region, as the paper amortizes them (Sec. 3).

Workloads: the four single ResNet-shaped layers and the 13-layer stack of stride-1 3x3 layers
at batch 64 with int8 activations handed from layer to layer.  The headline is the stack, the
largest of them; every workload gets the same record in `configs`.

Protocol, the same for every workload: one HIP stream; W untimed warm-up steps; the device kept
busy for RAMP_MS (the clocks of an idle GPU take tens of milliseconds of load to come up); then
repeats of exactly K steps each between two HIP events, at least five repeats and at least
MIN_TIMED_MS of timed work; `ms_per_step` is the median repeat.  Buffers rotate over several
sets whose footprint exceeds the 256 MB memory-side cache, so the figures are the cold ones.
Per-kernel durations come from the same protocol with one kernel per launch.  Prints ONE JSON line.
"""
import argparse
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0  # MI355X HBM3E
MFMA_I8_PEAK_TOPS = 5000.0  # dense int8
# Vector ALU, for the side figure `valu_frac`: 256 compute units x 64 lanes x 2.4 GHz, one
# operation per lane and cycle (the path's adds, conversions and scalings are neither fused
# multiply-adds nor packed).  Not a roof of the method: the instruction mix is the kernels' own.
VALU_PEAK_TOPS = 256 * 64 * 2.4e9 / 1e12
# Arithmetic of the add networks per item, counted by tests/host/op_count.cpp:
# algorithm -> (additions per input (tile, channel), operations per output (tile, filter)).
ADD_NETWORK_OPS = {"6x6_p88": (304, 438), "6x6_p100": (300, 422), "7x7_p132": (379, 580),
                   "7x7_p144": (375, 564), "4x4_p46": (110, 158), "4x4_p49": (111, 159)}
ROTATE_BYTES = 320 << 20  # footprint of the rotating buffer sets (> 256 MB memory-side cache)
RAMP_MS = 120.0  # untimed load before every timed region
MIN_TIMED_MS = 50.0  # timed work per figure, whatever --steps says
MIN_REPEATS = 5


def vector_ops(cin, cout, alg, P, tiles):
    """Algorithmic vector-ALU operations of one pass: the add networks, 3 per point for the
    rounding to int8 (convert, scale-and-round, clamp), 2 per point for the int32 products
    (convert, dequantize) and one multiplication per output for the activation scale."""
    if alg not in ADD_NETWORK_OPS:
        return None
    m = int(alg[0])
    in_adds, out_ops = ADD_NETWORK_OPS[alg]
    return tiles * (cin * (in_adds + 3 * P) + cout * (out_ops + 2 * P + m * m))


class Timer:
    """HIP events on the current stream; repeats of exactly `steps` calls of fn(i)."""

    def __init__(self, torch):
        self.torch = torch
        self.e0 = torch.cuda.Event(enable_timing=True)
        self.e1 = torch.cuda.Event(enable_timing=True)

    def ramp(self, fn, ms=RAMP_MS):
        t_end = time.perf_counter() + ms * 1e-3
        i = 0
        while time.perf_counter() < t_end:
            for _ in range(20):
                fn(i)
                i += 1
            self.torch.cuda.synchronize()

    def once(self, fn, steps, first=0):
        self.e0.record()
        for i in range(steps):
            fn(first + i)
        self.e1.record()
        self.torch.cuda.synchronize()
        return self.e0.elapsed_time(self.e1) / steps

    def median(self, fn, steps, warmup=0):
        """ms per call: median over repeats of `steps` calls each (>= MIN_REPEATS repeats and
        >= MIN_TIMED_MS of timed work in total)."""
        for i in range(warmup):
            fn(i)
        self.torch.cuda.synchronize()
        self.ramp(fn)
        first = self.once(fn, steps)
        repeats = max(MIN_REPEATS, min(400, math.ceil(MIN_TIMED_MS / max(first * steps, 1e-6))))
        vals = [self.once(fn, steps, r * steps) for r in range(repeats)]
        vals.sort()
        return vals[len(vals) // 2], repeats


def graph_ms(torch, timer, fn, steps):
    """The same steps captured once into a HIP graph (kernel launches only) and replayed:
    what is left when the host's launch overhead is taken out.  A measurement aid."""
    try:
        side = torch.cuda.Stream()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.stream(side):
            with torch.cuda.graph(graph, stream=side):
                for i in range(steps):
                    fn(i, side)
        for _ in range(2):
            graph.replay()
        torch.cuda.synchronize()
        ms, _ = timer.median(lambda i: graph.replay(), 1)
        del graph
        return ms / steps
    except Exception as exc:
        print(f"graph replay skipped: {exc}", file=sys.stderr)
        return None


def copy_bandwidth(torch, timer):
    """The library's plain copy kernel over rotating 128 MiB buffers: the streaming bandwidth
    (read + write bytes) this device reaches in this run, and a kernel of known traffic for
    scaling the byte counters of a rocprofv3 --pmc run of this command."""
    from paper_2407_02913_amd import binding

    nbytes = 128 << 20
    bufs = [(torch.empty(nbytes, dtype=torch.uint8, device="cuda"),
             torch.empty(nbytes, dtype=torch.uint8, device="cuda")) for _ in range(3)]
    cur = torch.cuda.current_stream()
    for a, b in bufs:
        binding.stream_copy(b, a, stream=cur)
    torch.cuda.synchronize()
    ms = timer.once(lambda i: binding.stream_copy(bufs[i % 3][1], bufs[i % 3][0], stream=cur), 12)
    del bufs
    torch.cuda.empty_cache()
    return 2 * nbytes / (ms * 1e-3) / 1e9


def traffic_from_profiles(kernel, workload, alg):
    """HBM bytes per launch from the committed rocprofv3 --pmc summary of this kernel, if any."""
    tfile = os.path.join(ROOT, "profiles", f"traffic_{kernel}_{workload}_{alg}.txt")
    if os.path.exists(tfile):
        for line in open(tfile):
            if line.startswith("hbm_bytes_per_launch"):
                return float(line.split()[1])
    return None


def roofline(kernel_rows, workload):
    """The roofline object of a workload from its per-kernel rows: the dominant kernel (largest
    share of a step) against the HBM roof -- algorithmic bytes / its average duration / 8 TB/s --
    and the product kernel against the int8 MFMA roof."""
    dom = max(kernel_rows, key=lambda r: r["us_per_step"])
    prod = max((r for r in kernel_rows if r["sfc_ops"]), key=lambda r: r["us_per_step"])
    achieved = dom["algorithmic_bytes"] / (dom["avg_us"] * 1e-6) / 1e9
    out = {"bound": "hbm", "kernel": dom["kernel"], "layer": dom["layer"], "achieved": round(achieved, 1),
           "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4),
           "traffic": traffic_from_profiles(dom["kernel"], dom["layer"], dom["alg"]),
           "algorithmic_bytes": dom["algorithmic_bytes"], "avg_us": round(dom["avg_us"], 2),
           "share_of_step": round(dom["us_per_step"] / sum(r["us_per_step"] for r in kernel_rows), 3),
           "product_kernel": prod["kernel"] + " " + prod["layer"],
           "product_mfma_frac": round(prod["sfc_ops"] / (prod["avg_us"] * 1e-6) / 1e12 / MFMA_I8_PEAK_TOPS, 4)}
    if dom.get("vector_ops"):
        out["valu_frac"] = round(dom["vector_ops"] / (dom["avg_us"] * 1e-6) / 1e12 / VALU_PEAK_TOPS, 4)
    return out


def kernel_rows(timer, layer, name, run_stage, launches, count=1):
    """Per-kernel average durations of one layer: each kernel alone, back to back, over the
    rotating sets (every set already holds valid V / M from full passes)."""
    rows = []
    kernels = layer.kernels()
    for kname, (mask, nbytes, ops) in kernels.items():
        ms, _ = timer.median(lambda i: run_stage(i, mask), launches)
        row = {"kernel": kname, "layer": name, "alg": layer.alg, "avg_us": ms * 1e3,
               "us_per_step": ms * 1e3 * count, "launches_per_step": count,
               "algorithmic_bytes": nbytes, "sfc_ops": ops}
        if len(kernels) == 1:
            row["vector_ops"] = vector_ops(layer.shape.Cin, layer.shape.Cout, layer.alg, layer.P, layer.tiles)
        rows.append(row)
    return rows


def public_rows(rows):
    return [{"kernel": r["kernel"], "layer": r["layer"], "avg_us": round(r["avg_us"], 2),
             "launches_per_step": r["launches_per_step"],
             "hbm_gbs": round(r["algorithmic_bytes"] / (r["avg_us"] * 1e-6) / 1e9, 1),
             "hbm_frac": round(r["algorithmic_bytes"] / (r["avg_us"] * 1e-6) / 1e9 / HBM_PEAK_GBS, 4),
             **({"mfma_frac": round(r["sfc_ops"] / (r["avg_us"] * 1e-6) / 1e12 / MFMA_I8_PEAK_TOPS, 4)}
                if r["sfc_ops"] else {})} for r in rows]


def bench_layer(args, name, torch, timer):
    """One ResNet-shaped layer, float32 output."""
    from paper_2407_02913_amd import binding, layers, synth

    shape = synth.LAYERS[name]
    data = synth.make_layer(shape, kernel=binding.KERNEL_SIZE[args.alg or "auto"])
    layer = layers.Layer(shape, data, out="f32", alg=args.alg or "auto", path=args.path or "auto")
    x_host = torch.from_numpy(data["x"])
    ybytes = 4 * shape.N * shape.Cout * shape.H * shape.W
    per_set = x_host.numel() + layer.workspace_bytes + ybytes
    nsets = args.buffer_sets if args.buffer_sets > 0 else max(2, min(24, -(-ROTATE_BYTES // per_set)))
    sets = [(x_host.cuda(), binding.device_buffer(layer.workspace_bytes), layer.new_output())
            for _ in range(nsets)]

    cur = torch.cuda.current_stream()  # looked up once: the call is slow next to a launch

    def step(i, stream=None, mask=binding.STAGE_ALL):
        xd, ws, y = sets[i % nsets]
        layer.run(xd, y, ws, stream=stream or cur, stages=mask)

    ms, repeats = timer.median(step, args.steps, args.warmup)
    rows = kernel_rows(timer, layer, name, lambda i, mask: step(i, None, mask), max(50, args.steps))
    ksize = layer.plan.kernel_size
    ops = shape.direct_ops * ksize * ksize // 9
    rec = {"workload": f"{name}: N={shape.N} Cin=Cout={shape.Cin} H=W={shape.H} {ksize}x{ksize} s1 p{(ksize - 1) // 2}, float32 out",
           "algorithm": layer.alg, "path": layer.path, "P": layer.P,
           "value": round(ops / (ms * 1e-3) / 1e12, 2), "unit": "TOPS", "ms_per_step": round(ms, 5),
           "repeats": repeats, "buffer_sets": nsets, "direct_gop": round(ops / 1e9, 2),
           "kernels": public_rows(rows), "roofline": roofline(rows, name)}
    if not args.quick:
        rec["graph_replay_ms_per_step"] = graph_ms(torch, timer, lambda i, s: step(i, s), min(nsets, 16))
        if rec["graph_replay_ms_per_step"]:
            rec["graph_replay_ms_per_step"] = round(rec["graph_replay_ms_per_step"], 5)
    layer.close()
    del sets
    torch.cuda.empty_cache()
    return rec


def bench_stack(args, torch, timer):
    """The 13 stride-1 3x3 layers of the ResNet-18-shaped stack at batch 64, int8 activations
    handed from layer to layer inside each resolution stage (the stride-2 layers between stages
    are not part of this path: every stage starts from its own synthetic activations).  One
    step = the 13 layers back to back on one stream."""
    import numpy as np

    from paper_2407_02913_amd import binding, layers, synth

    shapes = synth.stack_layers()
    lay = [layers.Layer(s, synth.make_layer(s, batch=4), out="i8", alg=args.alg or "auto",
                        path=args.path or "auto") for s in shapes]
    ws_bytes = max(l.workspace_bytes for l in lay)
    stages = sorted({(s.Cin, s.H) for s in shapes}, reverse=True, key=lambda t: t[1])
    act_bytes = sum(3 * shapes[0].N * c * h * h for c, h in stages)
    nsets = args.buffer_sets if args.buffer_sets > 0 else max(2, -(-ROTATE_BYTES // (act_bytes + ws_bytes)))
    sets = []
    for k in range(nsets):
        bufs = {}
        for c, h in stages:
            rng = np.random.default_rng(synth.BASE_SEED + c + 1000 * k)
            a = synth.activations((shapes[0].N, c, h, h), "relu", rng)
            bufs[c] = [torch.from_numpy(a).cuda(),
                       torch.empty((shapes[0].N, c, h, h), dtype=torch.int8, device="cuda"),
                       torch.empty((shapes[0].N, c, h, h), dtype=torch.int8, device="cuda")]
        sets.append((bufs, binding.device_buffer(ws_bytes)))

    cur = torch.cuda.current_stream()  # looked up once: the call is slow next to a launch

    def step(i, stream=None):
        stream = stream or cur
        bufs, ws = sets[i % nsets]
        done = {}
        for l in lay:
            c = l.shape.Cin
            k = done.get(c, 0)  # layer k of its stage reads buffer k (0: the stage input) ...
            src = bufs[c][0] if k == 0 else bufs[c][1 + (k - 1) % 2]
            l.run(src, bufs[c][1 + k % 2], ws, stream=stream)  # ... and writes the other one
            done[c] = k + 1

    ms, repeats = timer.median(step, args.steps, args.warmup)
    ops = sum(s.direct_ops for s in shapes)
    rows = []
    for c, h in stages:
        group = [l for l in lay if l.shape.Cin == c]
        l0 = group[0]

        def run_stage(i, mask, l0=l0, c=c):
            bufs, ws = sets[i % nsets]
            l0.run(bufs[c][0], bufs[c][1], ws, stream=cur, stages=mask)

        for i in range(nsets):  # V (and M) of this layer in every set's workspace
            run_stage(i, binding.STAGE_ALL)
        rows += kernel_rows(timer, l0, f"stack_c{c}_s{h}", run_stage, max(50, args.steps), count=len(group))
    rec = {"workload": "resnet18 stack: 13 stride-1 3x3 layers (4x 64@56, 3x 128@28, 3x 256@14, 3x 512@7), "
                       "batch 64, int8 activations between layers",
           "algorithm": sorted({l.alg for l in lay}), "path": [l.path for l in lay],
           "value": round(ops / (ms * 1e-3) / 1e12, 2), "unit": "TOPS", "ms_per_step": round(ms, 5),
           "repeats": repeats, "buffer_sets": nsets, "direct_gop": round(ops / 1e9, 2),
           "kernels": public_rows(rows), "roofline": roofline(rows, "stack")}
    if not args.quick:
        g = graph_ms(torch, timer, lambda i, s: step(i, s), nsets)
        rec["graph_replay_ms_per_step"] = None if g is None else round(g, 5)
    for l in lay:
        l.close()
    return rec


def cpu_baseline(args):
    """The oracle as it stands, on the host cores: whole passes of the headline workload (the
    13-layer stack) at a reduced batch until about 10 s have gone by, then the plain direct
    convolution (the definition of the result) on the same sample."""
    import numpy as np

    from oracle import sfc as oracle  # the cpu_baseline leg is the only user of the oracle here
    from paper_2407_02913_amd import synth

    try:
        from threadpoolctl import threadpool_info

        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = os.cpu_count()
    batch, alg = 4, "4x4_p46"
    shapes = synth.stack_layers(batch=batch)
    data = [synth.make_layer(s) for s in shapes]
    scales = [(oracle.calibrate_act_scales(d["x_calib"], alg), oracle.calibrate_filter_scales(d["w"], alg))
              for d in data]
    ops = sum(s.direct_ops for s in shapes)
    passes, t0 = 0, time.perf_counter()
    while True:
        for d, (sx, sw) in zip(data, scales):
            oracle.conv_requant(d["x"], d["w"], sx, sw, d["x_scale"], d["w_scale"], alg)
        passes += 1
        dt = time.perf_counter() - t0
        if dt >= 10.0 or passes >= 50:
            break
    dpasses, t0 = 0, time.perf_counter()
    while True:
        for d in data:
            oracle.direct_conv(d["x"], d["w"])
        dpasses += 1
        ddt = time.perf_counter() - t0
        if ddt >= 5.0 or dpasses >= 50:
            break
    return {"value": round(passes * ops / dt / 1e12, 5), "unit": "TOPS", "cores": int(cores), "kind": "oracle",
            "sample": f"oracle.conv_requant ({alg}) over the 13 layers of the stack at batch {batch} "
                      f"(filter transforms included), {passes} passes in {dt:.1f} s; numpy: the per-point "
                      "products run in its threaded BLAS, the integer transforms on one thread",
            "direct_conv_value": round(dpasses * ops / ddt / 1e12, 5),
            "direct_conv_sample": f"oracle.direct_conv (nine threaded float64 tensor contractions) on the same "
                                  f"layers, {dpasses} passes in {ddt:.1f} s"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="all",
                    help="all | stack | resnet56 | resnet28 | resnet14 | resnet7 (the headline is the stack; "
                         "a single workload prints its own record as the headline)")
    ap.add_argument("--path", default=None, choices=[None, "staged", "fused", "single"])
    ap.add_argument("--alg", default=None,
                    help="6x6_p88 | 6x6_p100 | 7x7_p132 | 7x7_p144 | 4x4_p46 | 4x4_p49, with 5x5 filters "
                         "6x6_5x5_p184 | 6x6_5x5_p196, with 7x7 filters 4x4_7x7_p184 | 4x4_7x7_p196 "
                         "(default: the library's choice per layer)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--quick", action="store_true", help="skip the graph-replay side figure")
    ap.add_argument("--buffer-sets", type=int, default=0,
                    help="rotating buffer sets (0: enough to exceed the memory-side cache)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (the layer shards over "
              "the batch with no exchange step); run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch

    from paper_2407_02913_amd import binding

    binding.load()
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    timer = Timer(torch)
    names = ["resnet56", "resnet28", "resnet14", "resnet7", "stack"] if args.workload == "all" else [args.workload]
    records = []
    for name in names:
        rec = bench_stack(args, torch, timer) if name == "stack" else bench_layer(args, name, torch, timer)
        records.append(rec)
    head = records[-1]
    head["roofline"]["stream_copy_gbs"] = round(copy_bandwidth(torch, timer), 1)
    out = {
        "metric": "direct-conv-equivalent int8 TOPS per 3x3 layer; % MFMA/HBM roofline",
        "value": head["value"], "unit": "TOPS", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": head["ms_per_step"], "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "int8", "data": "synthetic",
        "config": {"workload": head["workload"], "algorithm": head["algorithm"], "path": head["path"],
                   "mode": "requant-int8 transform domain", "protocol":
                       f"one stream, HIP events, median of {head['repeats']} repeats of {args.steps} steps, "
                       f"{head['buffer_sets']} rotating buffer sets, {RAMP_MS:.0f} ms of untimed load before",
                   "graph_replay_ms_per_step": head.get("graph_replay_ms_per_step")},
        "roofline": head["roofline"],
        "configs": records,
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(args)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
