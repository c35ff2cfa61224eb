#!/usr/bin/env python3
"""Throughput of the SFC 3x3 int8 convolution hot path on one MI355X.

A step is one pass of the whole hot path (input-tile transform, transform-domain
products, output transform with dequantization and NCHW store) over one batch of
synthetic ResNet-shaped input already resident in HBM.  The filter transform is
done once, outside the timed region, as the paper amortizes it (Sec. 3).
Buffers rotate over several sets so that consecutive steps do not re-hit the
memory-side cache.  Prints ONE JSON line.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0  # MI355X HBM3E
MFMA_I8_PEAK_TOPS = 5000.0  # dense int8
# Vector ALU: 256 compute units x 64 lanes x 2.4 GHz, one operation per lane and cycle (the
# path's adds, conversions and scalings are neither fused multiply-adds nor packed).
VALU_PEAK_TOPS = 256 * 64 * 2.4e9 / 1e12
# Arithmetic of the add networks per item, counted by tests/host/op_count.cpp:
# algorithm -> (additions per input (tile, channel), operations per output (tile, filter)).
ADD_NETWORK_OPS = {"6x6_p88": (304, 438), "6x6_p100": (300, 422), "7x7_p132": (379, 580),
                   "7x7_p144": (375, 564), "4x4_p46": (110, 158), "4x4_p49": (111, 159)}


def vector_ops(shape, alg, P, tiles):
    """Algorithmic vector-ALU operations of one pass: the add networks, 3 per point for the
    rounding to int8 (convert, scale-and-round, clamp), 2 per point for the int32 products
    (convert, dequantize) and one multiplication per output for the activation scale."""
    m = int(alg[0])
    in_adds, out_ops = ADD_NETWORK_OPS[alg]
    return tiles * (shape.Cin * (in_adds + 3 * P) + shape.Cout * (out_ops + 2 * P + m * m))
ROTATE_BYTES = 640 << 20  # footprint of the rotating buffer sets (> 256 MB memory-side cache)
RAMP_MS = 120.0  # untimed load before every timed region (see ramp() in main)


def stage_bytes(shape, P, tiles, path):
    """Algorithmic bytes per launch of each kernel (requantized mode)."""
    x = shape.N * shape.Cin * shape.H * shape.W
    v = P * tiles * shape.Cin
    u = P * shape.Cout * shape.Cin
    m = 4 * P * tiles * shape.Cout
    y = 4 * shape.N * shape.Cout * shape.H * shape.W
    if path == "single":
        return {"single_conv": x + u + y}
    if path == "fused":
        return {"input_transform": x + v, "fused_product_output": v + u + y}
    return {"input_transform": x + v, "product": v + u + m, "output_transform": m + y}


def pick_variant(shape, alg=None, path=None):
    """Tile size and path per layer shape, from the per-layer timings on one MI355X: the
    single-kernel path where it exists (Cin <= 64); SFC-4's 4x4 tiles when they divide a
    large feature map (56x56, 28x28: no ragged tiles, two workgroups per compute unit) and
    the channels are few (<= 128: on 28x28 maps its two kernels take 38.0 us back to back
    against 40.4 us for 6x6 and 38.7 us for 7x7 tiles, and 29.7 against 31.4 and 31.9 us per
    step when independent batches overlap on several streams); else 6x6 tiles while the
    feature map is large;
    7x7 tiles on 14x14 and 7x7 maps (no ragged tiles at all), with the products as batched
    GEMMs through HBM once there are too few tiles for the fused kernel's operand stream
    (7x7 maps, 512 channels; with 256 channels on 8x8 maps the fused kernel is still ahead,
    53 against 67 us) or too few (tile block, filter group) pairs to give every compute unit a
    workgroup of the fused kernel (256 channels on 14x14 maps at batch 64: 128 of them, 47 us
    per layer staged against 53 fused); 4x4 tiles on the 16x16 and smaller maps that they cover and 7x7 tiles do not."""
    if alg is None:
        if shape.Cin <= 128 and shape.H >= 28 and shape.H % 4 == 0 and shape.W % 4 == 0:
            alg = "4x4_p46"
        elif shape.H % 7 and shape.W % 7 and shape.H % 4 == 0 and shape.W % 4 == 0 and shape.H <= 16:
            alg = "4x4_p46"  # 16x16, 8x8, 4x4 maps: 4x4 tiles cover them, 7x7 tiles do not
        else:
            alg = "6x6_p88" if shape.H >= 28 else "7x7_p132"
    if path is None:
        if shape.Cin <= 64:
            path = "single"
        else:
            m = int(alg[0])
            tiles = shape.N * -(-shape.H // m) * -(-shape.W // m)
            fused_workgroups = -(-tiles // 16) * -(-shape.Cout // 32)
            if fused_workgroups < 256 or (shape.H < 14 and shape.Cin >= 512):
                path = "staged"
            else:
                path = "fused"
    return alg, path


def run_stack(args):
    """The 13 stride-1 3x3 layers of the ResNet-18-shaped stack at batch 64, filter transforms
    done beforehand, int8 activations handed from layer to layer inside each resolution stage
    (the stride-2 layers between stages are not part of this path: every stage starts from its
    own synthetic activations).  One step = the 13 layers; the layers of a stage run back to back
    on one stream, the four stages (independent chains) on a stream each."""
    import numpy as np
    import torch

    from paper_2407_02913_amd import binding, synth

    binding.load()
    torch.cuda.set_device(0)
    layers = synth.stack_layers()
    plans, bufs, chosen = [], [], []
    for shape in layers:
        d = synth.make_layer(shape, batch=4)  # weights and calibration data; activations below
        alg, path = pick_variant(shape, args.alg, args.path)
        chosen.append(f"{alg}/{path}")
        plan = binding.Plan(shape.N, shape.Cin, shape.Cout, shape.H, shape.W, alg=alg,
                            mode="requant", out="i8", path=path, per_channel_wscale=True)
        w_dev = torch.from_numpy(d["w"]).cuda()
        xc_dev = torch.from_numpy(d["x_calib"]).cuda()
        calib = binding.Plan(4, shape.Cin, shape.Cout, shape.H, shape.W, alg=alg, mode="requant",
                             path="staged", per_channel_wscale=True)
        scratch = binding.device_buffer(calib.workspace_bytes)
        sx = calib.calibrate_act_scales(xc_dev, scratch)
        sw = calib.calibrate_filter_scales(w_dev, scratch)
        calib.close()
        plan.set_point_scales(sx, sw)
        # output scale: spread of a sum of 9*Cin products of the synthetic distributions
        plan.set_output_scale(float(4.0 * 0.02 * 0.0125 * 30.0 * 20.0 * np.sqrt(9.0 * shape.Cin) / 127.0))
        fbuf = binding.device_buffer(plan.filter_bytes)
        plan.transform_filter(w_dev, d["w_scale"], fbuf)
        plans.append(plan)
        bufs.append((fbuf, binding.device_buffer(plan.workspace_bytes),
                     torch.empty((shape.N, shape.Cout, shape.H, shape.W), dtype=torch.int8, device="cuda")))
    stage_in = {}
    for shape in layers:
        if shape.Cin not in stage_in:
            rng = np.random.default_rng(synth.BASE_SEED + shape.Cin)
            a = np.clip(np.rint(np.abs(rng.normal(0.0, 30.0, (shape.N, shape.Cin, shape.H, shape.W)))), 0, 127)
            stage_in[shape.Cin] = torch.from_numpy(a.astype(np.int8)).cuda()

    stage_streams = {cin: torch.cuda.Stream() for cin in stage_in}

    def step(streams=None):
        prev = None
        for shape, plan, (_, ws, y) in zip(layers, plans, bufs):
            x = stage_in[shape.Cin] if prev is None or prev[0].Cin != shape.Cin else prev[1]
            plan.conv2d(x, 0.02, y, ws, stream=None if streams is None else streams[shape.Cin])
            prev = (shape, y)

    def timed(streams):
        for _ in range(args.warmup):
            step(streams)
        torch.cuda.synchronize()
        t_end = time.perf_counter() + RAMP_MS * 1e-3  # untimed load: the clocks of an idle GPU ramp up
        while time.perf_counter() < t_end:
            step(streams)
            torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            step(streams)
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3 / args.steps

    ms_one_stream = timed(None)
    ms = timed(stage_streams)
    ops = sum(sh.direct_ops for sh in layers)
    per_layer = []
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    for shape, plan, (_, ws, y) in zip(layers, plans, bufs):
        x = stage_in[shape.Cin]
        e0.record()
        for _ in range(20):
            plan.conv2d(x, 0.02, y, ws)
        e1.record()
        torch.cuda.synchronize()
        per_layer.append(round(e0.elapsed_time(e1) * 1e3 / 20, 1))
    print(json.dumps({
        "metric": "direct-conv-equivalent int8 TOPS, 13-layer stack", "value": round(ops / (ms * 1e-3) / 1e12, 2),
        "unit": "TOPS", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "int8", "data": "synthetic",
        "config": {"workload": "resnet18 stack: 13 stride-1 3x3 layers, batch 64, int8 activations between layers",
                   "variants": chosen, "direct_gop": round(ops / 1e9, 1), "streams": len(stage_streams),
                   "single_stream_ms_per_step": round(ms_one_stream, 4), "layer_us": per_layer}}))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="resnet56")
    ap.add_argument("--path", default=None, choices=[None, "staged", "fused", "single"])
    ap.add_argument("--alg", default=None,
                    help="6x6_p88 | 6x6_p100 | 7x7_p132 | 7x7_p144 | 4x4_p46 | 4x4_p49, or with 5x5 filters "
                         "6x6_5x5_p184 | 6x6_5x5_p196 (default: 4x4_p46 where Cin <= 64 and 4 divides the "
                         "feature map, else 6x6_p88; per layer for the stack)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--streams", type=int, default=3,
                    help="HIP streams the steps are dealt to round-robin (independent batches overlap)")
    ap.add_argument("--buffer-sets", type=int, default=0,
                    help="rotating input/workspace/output sets (0: enough to exceed the memory-side cache)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (the layer shards over "
              "the batch with no exchange step); run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    if args.workload == "stack":
        return run_stack(args)
    import numpy as np
    import torch

    from paper_2407_02913_amd import binding, synth

    binding.load()
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    shape = synth.LAYERS[args.workload]
    if args.alg is None:  # the fastest form and path measured for this layer shape
        args.alg, default_path = pick_variant(shape, None, args.path)
    else:
        default_path = None
    ksize = binding.KERNEL_SIZE[args.alg]
    data = synth.make_layer(shape, kernel=ksize)
    # one kernel where the layer allows it (3x3 filters, Cin <= 64), else input transform +
    # fused product/output
    path = args.path or default_path or ("single" if shape.Cin <= 64 and ksize == 3 else binding.DEFAULT_PATH)
    direct_ops = shape.direct_ops * ksize * ksize // 9

    plan = binding.Plan(shape.N, shape.Cin, shape.Cout, shape.H, shape.W, alg=args.alg,
                        mode="requant", path=path, per_channel_wscale=shape.per_channel_wscale)
    x_host = torch.from_numpy(data["x"])
    w_dev = torch.from_numpy(data["w"]).cuda()
    xc_dev = torch.from_numpy(data["x_calib"]).cuda()
    fbuf = binding.device_buffer(plan.filter_bytes)
    # scales from the library's own abs-max calibration (no oracle on the product path)
    scratch = binding.device_buffer(plan.workspace_bytes)
    sx = plan.calibrate_act_scales(xc_dev, scratch)
    sw = plan.calibrate_filter_scales(w_dev, scratch)
    plan.set_point_scales(sx, sw)
    plan.transform_filter(w_dev, data["w_scale"], fbuf)
    del scratch

    ybytes = 4 * shape.N * shape.Cout * shape.H * shape.W
    per_set = x_host.numel() + plan.workspace_bytes + ybytes
    nsets = args.buffer_sets if args.buffer_sets > 0 else max(2, min(24, -(-ROTATE_BYTES // per_set)))
    # a whole number of sets per stream: a set is then always used on the same stream
    nsets = -(-nsets // max(1, args.streams)) * max(1, args.streams)
    sets = []
    for _ in range(nsets):
        sets.append((x_host.cuda(), binding.device_buffer(plan.workspace_bytes),
                     torch.empty((shape.N, shape.Cout, shape.H, shape.W), dtype=torch.float32,
                                 device="cuda")))
    xs = float(data["x_scale"])

    def step(i, mask=binding.STAGE_ALL, stream=None):
        xd, ws, y = sets[i % nsets]
        plan.conv2d_stages(xd, xs, y, ws, mask, stream=stream)

    # Whole-job throughput: every step is an independent batch with its own buffers, so
    # consecutive steps are dealt to a few streams and the device overlaps one batch's
    # kernels with another's.  The K timed steps are launched from the host between two
    # device synchronizations and timed with the host clock; beside that figure, the same K
    # steps captured once into a HIP graph with one branch per stream (kernel launches only)
    # and replayed.
    nstreams = max(1, min(args.streams, nsets))
    streams = [torch.cuda.Stream() for _ in range(nstreams)]

    def ramp(mask=binding.STAGE_ALL, on_streams=True):
        """Untimed steps until the device has been busy for RAMP_MS: the clocks of an idle GPU
        take some tens of milliseconds of load to come up (the first 500 steps of this layer run
        at 21 us, the steady state at 16 us), so every timed region starts from a busy device."""
        t_end = time.perf_counter() + RAMP_MS * 1e-3
        i = 0
        while time.perf_counter() < t_end:
            for _ in range(50):
                step(i, mask, stream=streams[i % nstreams] if on_streams else None)
                i += 1
            torch.cuda.synchronize()

    for i in range(args.warmup):
        step(i, stream=streams[i % nstreams])
    torch.cuda.synchronize()
    ramp()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(i, stream=streams[i % nstreams])
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / args.steps
    job_graph_ms = None
    try:
        side = torch.cuda.Stream()
        job = torch.cuda.CUDAGraph()
        with torch.cuda.stream(side):
            with torch.cuda.graph(job, stream=side):
                for b in streams:
                    b.wait_stream(side)
                for i in range(args.steps):
                    step(i, stream=streams[i % nstreams])
                for b in streams:
                    side.wait_stream(b)
        job.replay()  # untimed: the first replay uploads the graph
        torch.cuda.synchronize()
        ramp()  # the capture left the device idle
        t0 = time.perf_counter()
        job.replay()
        torch.cuda.synchronize()
        job_graph_ms = (time.perf_counter() - t0) * 1e3 / args.steps
        del job
    except Exception as exc:  # a measurement aid, never the product path
        print(f"graph of the timed steps not captured: {exc}", file=sys.stderr)

    # latency of one step alone: same steps back to back on one stream, HIP events
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    ramp(on_streams=False)
    e0.record()
    for i in range(args.steps):
        step(i)
    e1.record()
    torch.cuda.synchronize()
    single_stream_ms = e0.elapsed_time(e1) / args.steps

    # The same steps replayed from one HIP graph (launch overhead taken out), and the warm
    # figure: one buffer set, inputs and outputs staying in the memory-side cache.
    graph_ms = warm_ms = None
    try:
        side = torch.cuda.Stream()
        graph = torch.cuda.CUDAGraph()
        nrep = min(nsets, 16)
        with torch.cuda.stream(side):
            with torch.cuda.graph(graph, stream=side):
                for i in range(nrep):
                    step(i, stream=side)
        for _ in range(3):
            graph.replay()
        torch.cuda.synchronize()
        ramp(on_streams=False)
        reps = max(2, args.steps // nrep)
        e0.record()
        for _ in range(reps):
            graph.replay()
        e1.record()
        torch.cuda.synchronize()
        graph_ms = e0.elapsed_time(e1) / (reps * nrep)
    except Exception as exc:  # the capture is a measurement aid, never the product path
        print(f"graph replay skipped: {exc}", file=sys.stderr)
    torch.cuda.synchronize()
    ramp(on_streams=False)
    for _ in range(10):
        step(0)
    torch.cuda.synchronize()
    e0.record()
    for _ in range(args.steps):
        step(0)
    e1.record()
    torch.cuda.synchronize()
    warm_ms = e0.elapsed_time(e1) / args.steps

    # per-kernel durations: each stage alone, back to back, over the rotating sets
    # (every set already holds valid V / M from the full passes above)
    if path == "single":
        stages = {"single_conv": binding.STAGE_ALL}
    elif path == "fused":
        stages = {"input_transform": binding.STAGE_INPUT,
                  "fused_product_output": binding.STAGE_PRODUCT | binding.STAGE_OUTPUT}
    else:
        stages = {"input_transform": binding.STAGE_INPUT, "product": binding.STAGE_PRODUCT,
                  "output_transform": binding.STAGE_OUTPUT}
    launches = max(50, min(args.steps, 400))
    stage_us = {}
    for name, mask in stages.items():
        ramp(mask, on_streams=False)
        e0.record()
        for i in range(launches):
            step(i, mask)
        e1.record()
        torch.cuda.synchronize()
        stage_us[name] = e0.elapsed_time(e1) * 1e3 / launches
    # calibration: the library's plain copy kernel over rotating 128 MiB buffers gives
    # the streaming bandwidth this device reaches in this run (read + write bytes)
    cal_bytes = 128 << 20
    cal = [(torch.empty(cal_bytes, dtype=torch.uint8, device="cuda"),
            torch.empty(cal_bytes, dtype=torch.uint8, device="cuda")) for _ in range(3)]
    for i in range(3):
        binding.stream_copy(cal[i][1], cal[i][0])
    torch.cuda.synchronize()
    e0.record()
    for i in range(12):
        binding.stream_copy(cal[i % 3][1], cal[i % 3][0])
    e1.record()
    torch.cuda.synchronize()
    copy_gbs = 2 * cal_bytes * 12 / (e0.elapsed_time(e1) * 1e-3) / 1e9
    del cal
    bytes_per = stage_bytes(shape, plan.P, plan.tiles, path)
    dominant = max(stage_us, key=stage_us.get)
    achieved = bytes_per[dominant] / (stage_us[dominant] * 1e-6) / 1e9
    traffic = None
    tfile = os.path.join(ROOT, "profiles", f"traffic_{dominant}_{args.workload}_{args.alg}.txt")
    if os.path.exists(tfile):
        for line in open(tfile):
            if line.startswith("hbm_bytes_per_launch"):
                traffic = float(line.split()[1])
    hbm_frac = achieved / HBM_PEAK_GBS
    roofline = {"bound": "hbm", "kernel": dominant, "achieved": round(achieved, 1),
                "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(hbm_frac, 4),
                "traffic": traffic, "algorithmic_bytes": bytes_per[dominant],
                "avg_us": round(stage_us[dominant], 2),
                "stages_us": {k: round(v, 2) for k, v in stage_us.items()},
                "stages_gbs": {k: round(bytes_per[k] / (stage_us[k] * 1e-6) / 1e9, 1) for k in stage_us},
                "stream_copy_gbs": round(copy_gbs, 1)}
    sfc_ops = 2 * plan.P * plan.tiles * shape.Cin * shape.Cout
    prod_key = {"single": "single_conv", "fused": "fused_product_output", "staged": "product"}[path]
    roofline["product_mfma_frac"] = round(sfc_ops / (stage_us[prod_key] * 1e-6) / 1e12 / MFMA_I8_PEAK_TOPS, 4)

    if path == "single":
        # one kernel does all the vector arithmetic of the path: it is nearer to the vector-ALU
        # roof than to the HBM roof, so that is the roof it is reported against
        vops = vector_ops(shape, args.alg, plan.P, plan.tiles)
        valu_tops = vops / (stage_us[dominant] * 1e-6) / 1e12
        roofline.update({"hbm_achieved_gbs": roofline["achieved"], "hbm_frac": roofline["frac"],
                         "algorithmic_vector_ops": vops})
        if valu_tops / VALU_PEAK_TOPS > hbm_frac:
            roofline.update({"bound": "alu", "achieved": round(valu_tops, 2),
                             "peak": round(VALU_PEAK_TOPS, 2), "unit": "TOP/s",
                             "frac": round(valu_tops / VALU_PEAK_TOPS, 4)})
    tops = direct_ops / (ms_per_step * 1e-3) / 1e12
    out = {
        "metric": f"direct-conv-equivalent int8 TOPS per {ksize}x{ksize} layer",
        "value": round(tops, 2), "unit": "TOPS", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 5), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "int8", "data": "synthetic",
        "config": {"workload": f"{args.workload}: N={shape.N} Cin=Cout={shape.Cin} H=W={shape.H} "
                               f"{ksize}x{ksize} s1 p{(ksize - 1) // 2}",
                   "algorithm": f"SFC-{4 if args.alg.startswith('4x4') else 6}({args.alg[:3]},{ksize}x{ksize}) P={plan.P}",
                   "mode": "requant-int8 transform domain",
                   "path": path, "buffer_sets": nsets, "streams": nstreams,
                   "untimed_load_before_each_timed_region_ms": RAMP_MS,
                   "same_steps_as_one_graph_ms_per_step": None if job_graph_ms is None else round(job_graph_ms, 5),
                   "single_stream_ms_per_step": round(single_stream_ms, 5),
                   "graph_replay_ms_per_step": None if graph_ms is None else round(graph_ms, 5),
                   "warm_single_stream_ms_per_step": round(warm_ms, 5)},
        "roofline": roofline,
    }

    if not args.no_cpu_baseline:
        from oracle import sfc as oracle  # the cpu_baseline leg is the only user of the oracle here

        try:
            from threadpoolctl import threadpool_info

            cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
        except Exception:
            cores = os.cpu_count()
        # bounded sample: whole passes over the same batch until about 10 s have gone by
        passes, t0 = 0, time.perf_counter()
        while True:
            oracle.conv_requant(data["x"], data["w"], sx, sw, data["x_scale"], data["w_scale"], args.alg)
            passes += 1
            dt = time.perf_counter() - t0
            if dt >= 10.0 or passes >= 50:
                break
        out["cpu_baseline"] = {"value": round(passes * direct_ops / dt / 1e12, 5), "unit": "TOPS",
                               "cores": int(cores), "kind": "oracle",
                               "sample": f"oracle.conv_requant on the full {args.workload} batch "
                                         f"(N={shape.N}), {passes} passes in {dt:.1f} s"}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
