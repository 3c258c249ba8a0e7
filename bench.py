#!/usr/bin/env python3
"""Benchmark of the fused conv2d / depthwise conv2d hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--skip-extras] [--skip-cpu]

One step = one pass over the 12 ResNet-18 conv2d shapes (TVM paper, Table 2, C1..C12) at
batch 64 with bf16 inputs/outputs, fp32 accumulate and the fused scale/shift + ReLU tail:
12 launches of tvg_conv2d_fused through the C ABI, inputs already resident in HBM.
Prints ONE JSON line.  ``value`` is the whole step's throughput in TFLOP/s (2*MACs of the
direct method over the step time).  ``roofline`` describes ONE kernel, the one with the
largest share of the step (conv3x3_dbuf_kernel: the layers the library plans with it are
launched last and back to back, two HIP events per step bracket exactly them inside the timed
region); ``layers`` lists all twelve.  ``ceilings`` holds what the GPU sustains in this very run
(a plain copy, a register-resident matrix-instruction loop per dtype), so every fraction can be
read against the data-sheet peak and against the achievable rate.  The depthwise layers
(D1..D9), the fp32 batch-1 shapes and the network bodies are measured after the timed region
and reported under their own keys; batch-1 layers are timed three ways (eager on warm
buffers, eager over rotating buffers, and one captured HIP graph of 240 launches over rotating
buffers), kernel-only durations of the same launches are in profiles/.  ``cpu_baseline`` times
the fp64 CPU oracle on the same workload on this machine's host cores.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2516.6      # dense bf16 MFMA, 256 CU x 4096 FLOP/clk x 2.4 GHz
PEAK_FP32_TFLOPS = 157.3       # fp32 MFMA / vector
PEAK_HBM_GBS = 8000.0


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=200,
                    help="untimed steps first: the GPU needs some 50 ms of work to reach its steady "
                         "state (3 steps: 0.273 ms per step, 300 steps: 0.260)")
    ap.add_argument("--skip-extras", action="store_true",
                    help="only the timed region (for profiler runs)")
    ap.add_argument("--skip-cpu", action="store_true", help="do not time the CPU oracle")
    ap.add_argument("--tune", action="store_true",
                    help="before the timed region, time every tile shape of every layer and fix "
                         "the fastest (paper_1802_04799_amd.tune); the choices are reported")
    ap.add_argument("--no-stream-hint", action="store_true",
                    help="operator layers without the TVG_STREAM_OUT store hint")
    ap.add_argument("--only", default="", help="comma-separated layer names (C1..C12): restrict "
                    "the step to these layers (for profiler runs)")
    ap.add_argument("--depthwise-probe", action="store_true",
                    help="only launch the depthwise layers D1..D9 at batch 64 --steps times each "
                         "(for profiler runs)")
    ap.add_argument("--no-arena", action="store_true",
                    help="network bodies with one allocation per tensor instead of the planned arena")
    ap.add_argument("--body-probe", default="", choices=["", "resnet18", "mobilenet"],
                    help="only run this network body at batch 32 --warmup + --steps times "
                         "(for profiler runs)")
    ap.add_argument("--batch1-probe", action="store_true",
                    help="only launch the batch-1 configurations (C1..C12 fp32, D1..D9 fp32) "
                         "--steps times each over rotating buffers (for profiler runs)")
    ap.add_argument("--winograd-probe", action="store_true",
                    help="only launch the pre-transformed-weights path on C2, C6, C9, C12 at batch 64 "
                         "--warmup + --steps times each (for profiler runs)")
    ap.add_argument("--copy-probe", type=int, default=0, metavar="MIB",
                    help="only run a plain device copy of this many MiB --steps times "
                         "(reference for scaling FETCH_SIZE / WRITE_SIZE counters)")
    return ap.parse_args()


def main():
    args = parse()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU only; --gpus must be 1 "
                 "(the path would shard along the batch axis with no exchange)")
    import numpy as np
    import torch
    import tvg_inputs as ti
    import paper_1802_04799_amd as tvg

    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")
    torch.cuda.set_device(0)
    tvg.load()
    dev = torch.device("cuda:0")

    def to_dev(a, bf16):
        t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32))
        return (t.to(torch.bfloat16) if bf16 else t).to(dev)

    # The operator benchmark runs unrelated layers: nothing reads an output again, which is what
    # the library's TVG_STREAM_OUT hint is for.  The ResNet-18 chain below runs without it.
    hint = 0 if args.no_stream_hint else tvg.TVG_STREAM_OUT

    class Layer:
        """One fused conv launch with everything preallocated."""
        def __init__(self, sh, seed, dtype, depthwise=False, copies=1):
            self.sh, self.dtype, self.depthwise = sh, dtype, depthwise
            bf = dtype == "bf16"
            inp = ti.make_inputs(sh, seed, dtype)
            self.host = inp
            self.x = [to_dev(inp["x"], bf)]
            self.w = [to_dev(inp["w"], bf)]
            self.scale = to_dev(inp["scale"], False)
            self.shift = to_dev(inp["shift"], False)
            tdt = torch.bfloat16 if bf else torch.float32
            self.y = [torch.empty(sh.y_shape(), dtype=tdt, device=dev)]
            for _ in range(copies - 1):       # disjoint buffer sets for cold-cache timing
                self.x.append(self.x[0].clone())
                self.w.append(self.w[0].clone())
                self.y.append(torch.empty_like(self.y[0]))
            self.desc = tvg.ConvDesc(sh.n, sh.ic, sh.h, sh.w, sh.oc, sh.r, sh.s, sh.stride,
                                     sh.stride, sh.pad, sh.pad,
                                     tvg.TVG_BF16 if bf else tvg.TVG_F32, tvg.TVG_RELU | hint)
            self.ws_bytes = 0 if depthwise else tvg.tvg_conv2d_workspace_size(self.desc)
            self.ws = torch.empty(max(self.ws_bytes, 1), dtype=torch.uint8, device=dev)
            self.fn = tvg.tvg_dwconv2d_fused if depthwise else tvg.tvg_conv2d_fused
            self.bytes = sh.algorithmic_bytes(2 if bf else 4)

        def launch(self, i=0):
            st = self.fn(self.desc, self.x[i], self.w[i], self.scale, self.shift, None, None,
                         self.y[i], self.ws, self.ws_bytes, None)
            if st != 0:
                raise RuntimeError(f"{self.sh.name}: {tvg.status_string(st)}")

    def time_loop(fn, iters, warmup=3):
        """Mean milliseconds per call of fn over back-to-back calls on the current stream."""
        for _ in range(warmup):
            fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(iters):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / iters

    def time_graph(launch_all, replays=5):
        """Mean milliseconds per replay of one HIP graph that holds whatever launch_all()
        enqueues (the library neither allocates nor synchronises, so its calls record as they
        stand); the capture is warmed up eagerly first and replayed once before timing."""
        launch_all()
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=torch.cuda.Stream()):
            launch_all()
        g.replay()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(replays):
            g.replay()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / replays

    def batch1_three_ways(l, copies, launches=240):
        """One batch-1 layer: eager on the same (warm) buffers, eager over rotating buffer sets
        whose footprint exceeds twice the memory-side cache (cold), and the same rotating
        launches as one captured HIP graph (no host between the launches)."""
        warm = time_loop(lambda: l.launch(0), 200)
        state = {"i": 0}

        def cold_call():
            l.launch(state["i"] % copies)
            state["i"] += 1
        cold = time_loop(cold_call, max(2 * copies, 200), warmup=copies)
        n = max(launches, copies)

        def many():
            for k in range(n):
                l.launch(k % copies)
        graph = time_graph(many) / n
        return warm, cold, graph

    # ---------------------------------------------------------------- the timed region
    if args.copy_probe:
        return copy_probe(torch, args)
    if args.depthwise_probe:
        for i, sh in enumerate(ti.mobilenet_depthwise(64)):
            copies = rotation(sh.algorithmic_bytes(4))
            l = Layer(sh, ti.layer_seed(3, 100 + i), "f32", depthwise=True, copies=copies)
            for k in range(args.warmup + args.steps):
                l.launch(k % copies)
            torch.cuda.synchronize()
            del l
        print(json.dumps({"depthwise_probe": "D1..D9 batch 64 fp32", "launches_each": args.warmup + args.steps}))
        return
    if args.batch1_probe:
        for name, shapes, cfg, dw in (("C", ti.resnet18_convs(1), 2, False),
                                      ("D", ti.mobilenet_depthwise(1), 3, True)):
            for i, sh in enumerate(shapes):
                copies = rotation(sh.algorithmic_bytes(4), cap=400)
                l = Layer(sh, ti.layer_seed(cfg, i), "f32", depthwise=dw, copies=copies)
                for k in range(args.warmup + args.steps):
                    l.launch(k % copies)
                torch.cuda.synchronize()
                del l
        print(json.dumps({"batch1_probe": "C1..C12, D1..D9, fp32, batch 1, rotating buffers",
                          "launches_each": args.warmup + args.steps}))
        return
    if args.winograd_probe:
        for i, sh in enumerate(ti.resnet18_convs(64)):
            if sh.r != 3 or sh.stride != 1:
                continue
            l = Layer(sh, ti.layer_seed(4, i), "bf16")
            pb, wb = tvg.tvg_conv2d_prepack_size(l.desc)
            packed = torch.empty(pb, dtype=torch.uint8, device=dev)
            wws = torch.empty(wb, dtype=torch.uint8, device=dev)
            tvg.tvg_conv2d_prepack(l.desc, l.w[0], packed, pb)
            for k in range(args.warmup + args.steps):
                st = tvg.tvg_conv2d_fused_prepacked(l.desc, l.x[0], packed, l.scale, l.shift, None, None,
                                                    l.y[0], wws, wb, None)
                if st != 0:
                    raise RuntimeError(tvg.status_string(st))
            torch.cuda.synchronize()
            del l, packed, wws
        print(json.dumps({"winograd_probe": "C2, C6, C9, C12 batch 64 bf16", "launches_each": args.warmup + args.steps}))
        return
    if args.body_probe:
        r = bench_body(tvg, ti, torch, np, dev, to_dev, time_loop, args.body_probe,
                       iters=args.steps, warmup=args.warmup, graph=False,
                       use_arena=not args.no_arena)
        print(json.dumps({"body_probe": args.body_probe, **r}))
        return
    shapes = ti.resnet18_convs(64)
    layers = [Layer(sh, ti.layer_seed(4, i), "bf16") for i, sh in enumerate(shapes)]
    if args.only:
        keep = set(args.only.split(","))
        layers = [l for l in layers if l.sh.name in keep]
    # The twelve layers are independent.  The launches of ONE kernel, conv3x3_dbuf_kernel (the
    # software-pipelined bf16 3x3 implicit GEMM, the largest share of the step), come last and
    # back to back, so that two events per step bracket exactly that kernel's launches.
    # Which layers it takes is the library's planning decision, read through tvg_conv2d_get_plan.
    DOM_KERNEL = 2          # TVG_KERNEL_3X3_PIPELINED
    is_dom = lambda l: tvg.tvg_conv2d_get_plan(l.desc)[0] == DOM_KERNEL

    tuning = None
    if args.tune:       # the measured per-shape knob search, outside the timed region
        from paper_1802_04799_amd import tune
        tuning = [dict(tune.tune_conv2d(l.desc, l.x[0], l.w[0], l.scale, l.shift, l.y[0],
                                        workspace=l.ws if l.ws_bytes else None), layer=l.sh.name)
                  for l in layers]

    layers = [l for l in layers if not is_dom(l)] + [l for l in layers if is_dom(l)]
    n_dom = sum(1 for l in layers if is_dom(l))
    first_dom = len(layers) - n_dom
    step_flops = sum(l.sh.flops for l in layers)
    step_bytes = sum(l.bytes for l in layers)

    def step():
        for l in layers:
            l.launch()

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()

    # per-layer durations: a calibration pass with an event before every launch, outside the
    # timed region (the extra events cost about 4 us per launch)
    cal = 5
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(len(layers) + 1)] for _ in range(cal)]
    for k in range(cal):
        for i, l in enumerate(layers):
            ev[k][i].record()
            l.launch()
        ev[k][len(layers)].record()
    torch.cuda.synchronize()
    per_layer_ms = [sum(ev[k][i].elapsed_time(ev[k][i + 1]) for k in range(cal)) / cal
                    for i in range(len(layers))]
    del ev

    K = args.steps
    d0 = [torch.cuda.Event(enable_timing=True) for _ in range(K)]
    d1 = [torch.cuda.Event(enable_timing=True) for _ in range(K)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(K):
        for i, l in enumerate(layers):
            if i == first_dom and n_dom:
                d0[k].record()
            l.launch()
        if n_dom:
            d1[k].record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = wall * 1e3 / K
    value = step_flops / (wall / K) / 1e12

    # ------------------------------------------- what the GPU sustains, in this same run
    ceilings = measure_ceilings(tvg, torch, dev, time_loop)
    ach_bf16, ach_hbm = ceilings["mfma_bf16_tflops"], ceilings["copy_gbs"]

    layer_rows = []
    for l, ms in zip(layers, per_layer_ms):
        tf = l.sh.flops / (ms * 1e-3) / 1e12
        gbs = l.bytes / (ms * 1e-3) / 1e9
        ai = l.sh.flops / l.bytes
        attainable = min(PEAK_BF16_TFLOPS, ai * PEAK_HBM_GBS / 1e3)
        achievable = min(ach_bf16, ai * ach_hbm / 1e3)
        layer_rows.append({"name": l.sh.name, "kernel": tvg.KERNEL_NAMES[tvg.tvg_conv2d_get_plan(l.desc)[0]],
                           "us": round(ms * 1e3, 2), "tflops": round(tf, 1),
                           "gbs": round(gbs, 1), "frac_mfma_peak": round(tf / PEAK_BF16_TFLOPS, 4),
                           "frac_attainable": round(tf / attainable, 4),
                           "frac_achievable": round(tf / achievable, 4),
                           "bound": "mfma" if ai > PEAK_BF16_TFLOPS * 1e3 / PEAK_HBM_GBS else "hbm"})
    roofline = None
    if n_dom:
        dom_ms = sum(d0[k].elapsed_time(d1[k]) for k in range(K)) / K      # all n_dom launches
        dom = [l for l in layers if is_dom(l)]
        dom_flops = sum(l.sh.flops for l in dom)
        dom_bytes = sum(l.bytes for l in dom)
        dom_tf = dom_flops / (dom_ms * 1e-3) / 1e12
        roofline = {"bound": "mfma", "achieved": round(dom_tf, 2), "peak": PEAK_BF16_TFLOPS,
                    "unit": "TFLOP/s", "frac": round(dom_tf / PEAK_BF16_TFLOPS, 4),
                    "traffic": measured_traffic("conv3x3_dbuf_kernel"),
                    "kernel": "conv3x3_dbuf_kernel",
                    "frac_of_achievable_mfma": round(dom_tf / ach_bf16, 4),
                    "launches_per_step": n_dom,
                    "layers": [l.sh.name for l in dom],
                    "flops_per_launch": dom_flops / n_dom,
                    "algorithmic_bytes_per_launch": dom_bytes / n_dom,
                    "avg_launch_us": round(dom_ms * 1e3 / n_dom, 2),
                    "share_of_step_time": round(dom_ms / ms_per_step, 3),
                    "timing": "two HIP events per step around this kernel's back-to-back launches, "
                              "inside the timed region, on the launch stream; per-unit figures: "
                              "2*IC*9 flops per output element, (|x|+|w|+|y|)*2 + 8*OC bytes per launch"}

    r3 = [(l, ms) for l, ms in zip(layers, per_layer_ms) if l.sh.r == 3]
    out = {
        "metric": "fused conv2d TFLOP/s (% MFMA peak); depthwise conv GB/s (% HBM peak)",
        "value": round(value, 2), "unit": "TFLOP/s", "n_gpus": 1, "steps": K,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "configs[3]: the 12 ResNet-18 conv2d shapes of Table 2 (C1..C12), "
                               "batch 64, bf16 in/out, fp32 accumulate, fused scale/shift+ReLU; "
                               "one step = 12 launches" + (f" (restricted to {args.only})" if args.only else ""),
                   "step_gflop": round(step_flops / 1e9, 2), "step_mbytes": round(step_bytes / 1e6, 1),
                   "frac_mfma_peak": round(value / PEAK_BF16_TFLOPS, 4),
                   "frac_achievable_mfma": round(value / ach_bf16, 4),
                   "all_3x3_layers": {"layers": [l.sh.name for l, _ in r3],
                                      "gflop": round(sum(l.sh.flops for l, _ in r3) / 1e9, 2),
                                      "us_calibration_pass": round(sum(ms for _, ms in r3) * 1e3, 1)},
                   "stream_out_hint": not args.no_stream_hint},
        "roofline": roofline,
        "ceilings": ceilings,
        "layers": layer_rows,
        "tuning": tuning,
        "layers_note": "per-launch durations from a calibration pass with an event before every "
                       "launch (adds about 4 us per launch); not part of the timed region",
    }

    # ------------------------------------------------------------ extras (not in `value`)
    if not args.skip_extras:
        # depthwise D1..D9, fp32, batch 1 (configs[2]): three ways
        dw_rows = []
        for i, sh in enumerate(ti.mobilenet_depthwise(1)):
            nbytes = sh.algorithmic_bytes(4)
            copies = rotation(nbytes, cap=1500)
            l = Layer(sh, ti.layer_seed(3, i), "f32", depthwise=True, copies=copies)
            warm, cold, graph = batch1_three_ways(l, copies)
            dw_rows.append({"name": sh.name, "kbytes": round(nbytes / 1e3, 1),
                            "warm_us": round(warm * 1e3, 2), "cold_us": round(cold * 1e3, 2),
                            "graph_cold_us": round(graph * 1e3, 2),
                            "warm_gbs": round(nbytes / (warm * 1e-3) / 1e9, 1),
                            "cold_gbs": round(nbytes / (cold * 1e-3) / 1e9, 1),
                            "graph_cold_gbs": round(nbytes / (graph * 1e-3) / 1e9, 1),
                            "graph_cold_frac_hbm_peak": round(nbytes / (graph * 1e-3) / 1e9 / PEAK_HBM_GBS, 4),
                            "graph_cold_frac_copy": round(nbytes / (graph * 1e-3) / 1e9 / ach_hbm, 4)})
            del l
        # the same kernel at batch 64: HBM-sized traffic, rotating so that a cycle's reads and
        # writes exceed twice the memory-side cache
        dw64_rows = []
        for i, sh in enumerate(ti.mobilenet_depthwise(64)):
            copies = rotation(sh.algorithmic_bytes(4))
            l = Layer(sh, ti.layer_seed(3, 100 + i), "f32", depthwise=True, copies=copies)
            state = {"i": 0}

            def call():
                l.launch(state["i"] % copies)
                state["i"] += 1
            ms = time_loop(call, max(50, 4 * copies), warmup=copies)
            gbs = l.bytes / (ms * 1e-3) / 1e9
            dw64_rows.append({"name": sh.name, "mbytes": round(l.bytes / 1e6, 1), "buffer_sets": copies,
                              "us": round(ms * 1e3, 2), "gbs": round(gbs, 1),
                              "frac_hbm_peak": round(gbs / PEAK_HBM_GBS, 4),
                              "frac_copy": round(gbs / ach_hbm, 4)})
            del l
        tot_b = sum(r["mbytes"] for r in dw64_rows) * 1e6
        tot_t = sum(r["us"] for r in dw64_rows) * 1e-6
        out["depthwise"] = {
            "config3_batch1_fp32": dw_rows,
            "batch64_fp32": dw64_rows,
            "batch64_total_gbs": round(tot_b / tot_t / 1e9, 1),
            "batch64_frac_hbm_peak": round(tot_b / tot_t / 1e9 / PEAK_HBM_GBS, 4),
            "batch64_frac_copy": round(tot_b / tot_t / 1e9 / ach_hbm, 4),
            "note": "algorithmic bytes (x, w, y, scale, shift moved once) / event time.  batch 1: "
                    "warm = same buffers, cold = rotating disjoint buffer sets (> 640 MB in all), "
                    "graph_cold = the rotating launches as one captured HIP graph (no host "
                    "between them); kernel-only durations are in profiles/.  batch 64 "
                    "(supplementary, not a BASELINE.json configuration) rotates buffer sets too.",
        }
        # fp32, batch 1 (configs[0] = C2, configs[1] = C1..C12): three ways
        rows = []
        for i, sh in enumerate(ti.resnet18_convs(1)):
            copies = rotation(sh.algorithmic_bytes(4), cap=400)
            l = Layer(sh, ti.layer_seed(2, i), "f32", copies=copies)
            warm, cold, graph = batch1_three_ways(l, copies)
            rows.append({"name": sh.name, "kernel": tvg.KERNEL_NAMES[tvg.tvg_conv2d_get_plan(l.desc)[0]],
                         "warm_us": round(warm * 1e3, 2), "cold_us": round(cold * 1e3, 2),
                         "graph_cold_us": round(graph * 1e3, 2),
                         "warm_tflops": round(sh.flops / (warm * 1e-3) / 1e12, 2),
                         "graph_cold_tflops": round(sh.flops / (graph * 1e-3) / 1e12, 2),
                         "splits_ws_bytes": l.ws_bytes})
            del l
        fl = sum(s.flops for s in ti.resnet18_convs(1))
        tots = {k: sum(r[k] for r in rows) for k in ("warm_us", "cold_us", "graph_cold_us")}
        out["fp32_batch1"] = {"layers": rows,
                              "total_warm_us": round(tots["warm_us"], 1),
                              "total_cold_us": round(tots["cold_us"], 1),
                              "total_graph_cold_us": round(tots["graph_cold_us"], 1),
                              "tflops_warm": round(fl / tots["warm_us"] / 1e6, 2),
                              "frac_fp32_peak_warm": round(fl / tots["warm_us"] / 1e6 / PEAK_FP32_TFLOPS, 4),
                              "frac_fp32_achievable_warm": round(fl / tots["warm_us"] / 1e6 / ceilings["mfma_fp32_tflops"], 4),
                              "config1_C2": next(r for r in rows if r["name"] == "C2")}
        # The pre-transformed-weights path (Winograd F(2x2,3x3); the paper's "TVM PT") beside the
        # direct kernels on the 3x3 stride-1 layers at batch 64.  FLOPs are counted by the direct
        # method for both (no discount for the multiplications Winograd saves); the weight
        # transform runs once, outside the timed loop, as the paper's pre-transformation does.
        wino_rows = []
        for i, sh in enumerate(ti.resnet18_convs(64)):
            if sh.r != 3 or sh.stride != 1:
                continue
            l = Layer(sh, ti.layer_seed(4, i), "bf16")
            pb, wb = tvg.tvg_conv2d_prepack_size(l.desc)
            packed = torch.empty(pb, dtype=torch.uint8, device=dev)
            wws = torch.empty(wb, dtype=torch.uint8, device=dev)
            if tvg.tvg_conv2d_prepack(l.desc, l.w[0], packed, pb) != 0:
                raise RuntimeError("tvg_conv2d_prepack")
            y2 = torch.empty_like(l.y[0])

            def wino():
                st = tvg.tvg_conv2d_fused_prepacked(l.desc, l.x[0], packed, l.scale, l.shift, None, None,
                                                    y2, wws, wb, None)
                if st != 0:
                    raise RuntimeError(tvg.status_string(st))
            t_direct = time_loop(l.launch, 200, warmup=200)
            t_wino = time_loop(wino, 200, warmup=200)
            diff = (l.y[0].float() - y2.float()).abs()
            rho = l.y[0].float().pow(2).mean().sqrt()
            rel = (diff / torch.maximum(l.y[0].float().abs(), rho)).max().item()
            wino_rows.append({"name": sh.name, "direct_us": round(t_direct * 1e3, 2),
                              "prepacked_us": round(t_wino * 1e3, 2),
                              "direct_tflops": round(sh.flops / (t_direct * 1e-3) / 1e12, 1),
                              "prepacked_tflops_direct_flop_count": round(sh.flops / (t_wino * 1e-3) / 1e12, 1),
                              "packed_weights_mb": round(pb / 1e6, 2), "workspace_mb": round(wb / 1e6, 1),
                              "max_rel_diff_to_direct": round(rel, 5)})
            del l, packed, wws, y2
        out["pretransformed_winograd"] = {
            "layers": wino_rows,
            "note": "tvg_conv2d_fused_prepacked (input transform + contraction with the inverse transform "
                    "and the fused tail in registers) against tvg_conv2d_fused, same buffers back to back, "
                    "warm; FLOPs by the direct count for both"}
        # ResNet-18 body, batch 32, bf16 (configs[4]): 20 convs + 1 max-pool, 21 launches
        out["resnet18_body"] = bench_body(tvg, ti, torch, np, dev, to_dev, time_loop, iters=50,
                                          warmup=20, use_arena=not args.no_arena,
                                          tune_tiles=args.tune)
        if not args.no_arena:      # the same chain with one allocation per tensor, for comparison
            out["resnet18_body"]["ms_separate_tensors"] = bench_body(
                tvg, ti, torch, np, dev, to_dev, time_loop, iters=50, warmup=20, graph=False,
                use_arena=False)["ms"]
        # the same body with every down-sampling block's first conv and projection shortcut as
        # one two-head launch: 18 launches (FLOPs counted as for the 21-launch chain)
        fused = bench_body(tvg, ti, torch, np, dev, to_dev, time_loop, iters=50, warmup=20,
                           use_arena=not args.no_arena, fuse_projection=True)
        out["resnet18_body"]["two_head_blocks"] = {k: fused[k] for k in
                                                   ("launches", "ms", "graph_replay_ms", "images_per_s", "tflops")}
        # MobileNet body, batch 32, bf16: stem + 13 x (depthwise 3x3, 1x1), 27 launches
        out["mobilenet_body"] = bench_body(tvg, ti, torch, np, dev, to_dev, time_loop, "mobilenet",
                                           iters=50, warmup=20, use_arena=not args.no_arena,
                                           tune_tiles=args.tune)
        if not args.no_arena:
            out["mobilenet_body"]["ms_separate_tensors"] = bench_body(
                tvg, ti, torch, np, dev, to_dev, time_loop, "mobilenet", iters=50, warmup=20,
                graph=False, use_arena=False)["ms"]

    if not args.skip_cpu:
        out["cpu_baseline"] = cpu_baseline(ti, np)

    print(json.dumps(out))


def rotation(nbytes, cap=64):
    """Disjoint buffer sets to rotate through so that one cycle touches more than 640 MB, over
    twice the 256 MB memory-side cache: every launch then reads from HBM."""
    return int(min(cap, max(2, 640e6 // nbytes + 1)))


def measure_ceilings(tvg, torch, dev, time_loop):
    """What this GPU sustains, measured in this run: a plain copy (1 GiB each way, far beyond
    the caches) and a register-resident matrix-instruction loop per dtype, two workgroups per
    compute unit."""
    n = 1 << 30
    src = torch.empty(n, dtype=torch.uint8, device=dev)
    dst = torch.empty(n, dtype=torch.uint8, device=dev)
    src.fill_(1)

    def copy():
        assert tvg.tvg_probe_copy(src, dst, n) == 0
    ms = time_loop(copy, 10)
    copy_gbs = 2 * n / (ms * 1e-3) / 1e9
    ms_t = time_loop(lambda: dst.copy_(src), 10)
    del src, dst
    out = torch.empty(512 * 256, dtype=torch.float32, device=dev)
    res = {"copy_gbs": round(copy_gbs, 1), "copy_frac_hbm_peak": round(copy_gbs / PEAK_HBM_GBS, 4),
           "runtime_copy_gbs": round(2 * n / (ms_t * 1e-3) / 1e9, 1)}
    for name, code, iters, peak in (("bf16", tvg.TVG_BF16, 20000, PEAK_BF16_TFLOPS),
                                    ("fp32", tvg.TVG_F32, 4000, PEAK_FP32_TFLOPS)):
        fl = {}

        def run():
            st, fl["v"] = tvg.tvg_probe_mfma(code, iters, 512, out)
            assert st == 0
        ms = time_loop(run, 3, warmup=1)
        tf = fl["v"] / (ms * 1e-3) / 1e12
        res[f"mfma_{name}_tflops"] = round(tf, 1)
        res[f"mfma_{name}_frac_peak"] = round(tf / peak, 4)
    res["note"] = ("copy: 1 GiB read + 1 GiB written by a 16-byte grid-stride copy kernel of the "
                   "library (runtime_copy: the HIP runtime's own copy of the same buffers); mfma: "
                   "512 workgroups x 4 waves x 4 independent accumulator tiles, operands in registers")
    return res


def copy_probe(torch, args):
    n = args.copy_probe * 1024 * 1024 // 4
    x = torch.ones(n, dtype=torch.float32, device="cuda")
    y = torch.empty_like(x)
    torch.cuda.synchronize()
    for _ in range(args.steps):
        y.copy_(x)
    torch.cuda.synchronize()
    print(json.dumps({"copy_probe_mib": args.copy_probe, "copies": args.steps}))


def measured_traffic(kernel):
    """HBM bytes per launch of `kernel` from the committed rocprofv3 counter summary
    (profiles/hbm_traffic.json, written from two --pmc runs), or None when there is none."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    try:
        with open(path) as f:
            return json.load(f).get(kernel, {}).get("bytes_per_launch")
    except (OSError, ValueError):
        return None


def bench_body(tvg, ti, torch, np, dev, to_dev, time_loop, network="resnet18", iters=10, warmup=3,
               graph=True, use_arena=True, tune_tiles=False, fuse_projection=False):
    n = 32
    config = 5 if network == "resnet18" else 6
    steps = ti.resnet18_body(n, fuse_projection) if network == "resnet18" else ti.mobilenet_body(n)
    plain = ti.resnet18_body(n) if network == "resnet18" else steps
    weights = {s.layer_index: ti.make_weights(s.shape, ti.layer_seed(config, s.layer_index), "bf16")
               for s in plain if s.op != "maxpool"}
    dw = {k: {"w": to_dev(p["w"], True), "scale": to_dev(p["scale"], False),
              "shift": to_dev(p["shift"], False)} for k, p in weights.items()}
    images = to_dev(ti.body_images(n, ti.layer_seed(config, 901)), True)
    # Static memory plan (paper Section 3): every intermediate tensor lives in one arena, at the
    # offset tvg_plan_arena gives it; tensors that are never alive together share memory.  The
    # images stay outside (the chain is replayed on them).
    lives = ti.tensor_lives(steps)
    ids = [t for t in lives if t != 0]
    offsets, arena_bytes = tvg.tvg_plan_arena([lives[t] for t in ids])
    arena = torch.empty(arena_bytes, dtype=torch.uint8, device=dev)
    offset_of = dict(zip(ids, offsets))

    def planned(t, shape):
        nbytes = lives[t][0]
        if not use_arena:
            return torch.empty(shape, dtype=torch.bfloat16, device=dev)
        return arena[offset_of[t]:offset_of[t] + nbytes].view(torch.bfloat16).view(shape)

    tensors = {0: images}
    calls = []
    for st in steps:
        src = tensors[st.src]
        if st.op == "dwconv":
            sh = st.shape
            desc = tvg.ConvDesc(sh.n, sh.ic, sh.h, sh.w, sh.oc, 3, 3, sh.stride, sh.stride, 1, 1,
                                tvg.TVG_BF16, tvg.TVG_RELU if st.relu else 0)
            y = planned(st.dst, sh.y_shape())
            p = dw[st.layer_index]
            calls.append((tvg.tvg_dwconv2d_fused, (desc, src, p["w"], p["scale"], p["shift"], None,
                                                   None, y, None, 0, None)))
        elif st.op == "conv_dual":
            # a down-sampling block's first conv and its 1x1 projection (the centre tap of a 3x3
            # filter, weights joined once up front: constant folding) as one two-head launch
            sh, s2 = st.shape, st.shape2
            p1, p2 = weights[st.layer_index], weights[st.layer_index2]
            emb = np.zeros((s2.oc, s2.ic, 3, 3), np.float32)
            emb[:, :, 1, 1] = p2["w"][:, :, 0, 0]
            wj = to_dev(np.concatenate([p1["w"], emb]), True)
            scj = to_dev(np.concatenate([p1["scale"], p2["scale"]]), False)
            sfj = to_dev(np.concatenate([p1["shift"], p2["shift"]]), False)
            desc = tvg.ConvDesc(sh.n, sh.ic, sh.h, sh.w, sh.oc + s2.oc, 3, 3, sh.stride, sh.stride, 1, 1,
                                tvg.TVG_BF16, tvg.TVG_RELU if st.relu else 0)
            y = planned(st.dst, sh.y_shape())
            tensors[st.dst2] = planned(st.dst2, s2.y_shape())
            calls.append((tvg.tvg_conv2d_fused_dual,
                          (desc, sh.oc, (tvg.TVG_RELU if st.relu2 else 0) | tvg.TVG_CENTRE_TAP_ONLY, src,
                           wj, scj, sfj, None, None, y, tensors[st.dst2], None)))
        elif st.op == "conv":
            sh = st.shape
            desc = tvg.ConvDesc(sh.n, sh.ic, sh.h, sh.w, sh.oc, sh.r, sh.s, sh.stride, sh.stride,
                                sh.pad, sh.pad, tvg.TVG_BF16, tvg.TVG_RELU if st.relu else 0)
            y = planned(st.dst, sh.y_shape())
            need = tvg.tvg_conv2d_workspace_size(desc)
            ws = torch.empty(max(need, 1), dtype=torch.uint8, device=dev)
            p = dw[st.layer_index]
            res = None if st.residual is None else tensors[st.residual]
            calls.append((tvg.tvg_conv2d_fused, (desc, src, p["w"], p["scale"], p["shift"], None,
                                                 res, y, ws, need, None)))
        else:
            nn, c, h, w = src.shape
            y = planned(st.dst, (nn, c, (h - 1) // 2 + 1, (w - 1) // 2 + 1))
            calls.append((tvg.tvg_maxpool2d_3x3s2, (nn, c, h, w, tvg.TVG_BF16, src, y, None)))
        tensors[st.dst] = y

    tuned = None
    if tune_tiles:      # the measured tile search over this body's dense layers (batch-32 shapes)
        from paper_1802_04799_amd import tune
        tuned = 0
        for fn, a in calls:
            if fn is tvg.tvg_conv2d_fused:
                desc, x_, w_, sc_, sf_, _, res_, y_ = a[:8]
                tuned += tune.tune_conv2d(desc, x_, w_, sc_, sf_, y_, residual=res_)["chosen"] is not None

    def forward():
        for fn, a in calls:
            st = fn(*a)
            if st != 0:
                raise RuntimeError(tvg.status_string(st))

    ms = time_loop(forward, iters, warmup)
    graph_ms = float("nan")
    if graph:
        # The same launches captured once into a HIP graph and replayed: the library neither
        # allocates nor synchronises, so the chain records as it stands.
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=torch.cuda.Stream()):
            forward()
        graph_ms = time_loop(g.replay, 10)
    flops = sum(s.shape.flops for s in plain if s.op != "maxpool")
    return {"batch": n, "launches": len(calls), "tiles_changed_by_tuning": tuned, "arena": use_arena, "arena_mb": round(arena_bytes / 1e6, 1),
            "unplanned_mb": round(sum(lives[t][0] for t in ids) / 1e6, 1), "ms": round(ms, 4), "graph_replay_ms": round(graph_ms, 4) if graph else None,
            "tflops": round(flops / (ms * 1e-3) / 1e12, 1),
            "images_per_s": round(n / (ms * 1e-3), 1),
            "frac_mfma_peak": round(flops / (ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 4)}


def cpu_baseline(ti, np):
    """The fp64 oracle, as it stands, on a bounded sample of the timed workload."""
    import oracle
    batch = 64
    shapes = ti.resnet18_convs(batch)
    flops, secs = 0, 0.0
    for i, sh in enumerate(shapes):
        inp = ti.make_inputs(sh, ti.layer_seed(4, i), "bf16")
        t = time.perf_counter()
        oracle.conv2d_fused(inp["x"], inp["w"], inp["scale"], inp["shift"],
                            stride=(sh.stride,) * 2, pad=(sh.pad,) * 2, relu=True)
        secs += time.perf_counter() - t
        flops += sh.flops
    return {"value": round(flops / secs / 1e12, 6), "unit": "TFLOP/s",
            "cores": oracle.num_threads(), "kind": "oracle",
            "sample": f"one whole step: the same 12 shapes at batch {batch} ({flops / 1e9:.1f} GFLOP, "
                      f"{secs:.1f} s), fp64 seven-loop direct convolution + fused tail",
            "seconds": round(secs, 2)}


if __name__ == "__main__":
    main()
