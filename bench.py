#!/usr/bin/env python3
"""Benchmark: images/s of the pruned VGG-16 (32x32 inputs) on one MI355X.

A step is one pass of the inference hot path over one batch of synthetic images:
13 pruned conv+BN+ReLU layers (MFMA kernels; the 2x2 max-pools run in their epilogues) and the
FC, through cprune_net_forward.  The one-off pruning stage (L1 ranking, kept-list selection, weight
gather with BN folding) and the per-shape tile selection run before the timed region and
are reported separately (`prune_ms`, `tune_s`).  Inputs and weights are resident in HBM
when timing starts.

Prints ONE JSON line.  `value`: images/s over the timed steps.  `roofline`: the dominant
kernel (the conv instantiation with the most device time per step): useful FLOP of the layers it
runs over the sum of their device times (HIP events around back-to-back launches of each layer),
against the dense fp32 / fp16 MFMA peak; `traffic`: its bytes between L2 and fabric per launch
from hardware counters (fixed figures for the default workload).  `conv_layers`: the same ratio
over all 13 conv layers.
`cpu_baseline`: the CPU oracle's forward on a bounded sample of the same images.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK = {"f32": 157.3, "f16": 2500.0, "bf16": 2500.0}   # dense MFMA TFLOP/s, MI355X
# Bytes between L2 and fabric per launch (FETCH_SIZE + WRITE_SIZE, each scaled by what the counter
# reads for a copy kernel of known size), by (kernel instantiation, batch, layers it ran), for the default
# workload: from the rocprofv3 counter runs summarised in profiles/vgg16_b64_f32_hbm_traffic.md.  The
# timed selection decides which layers a kernel runs; when that differs from the profiled runs the
# figure does not apply and null is reported.
TRAFFIC = {
    ("conv_patch_kernel<float, 1, 8, 8, 1, 1, 1>", 64, ("conv3", "conv5", "conv6")): 8474991,            # algorithmic 5.8e6
    ("conv_patch_kernel<float, 2, 8, 8, 1, 1, 1>", 64, ("conv4",)): 10103478,                            # algorithmic 8.2e6
    ("conv_patch_kernel<float, 1, 8, 8, 1, 2, 2>", 64, ("conv7",)): 12106091,                            # algorithmic 4.7e6
    ("conv_wave_kernel<float, 5, 1, 3>", 64, ("conv8", "conv10")): 10499238,                             # algorithmic 3.7e6
    ("conv_wave_kernel<float, 2, 2, 4>", 64, ("conv9",)): 15049592,                                      # algorithmic 4.8e6
    ("conv_stem2_kernel<float, 2>", 64, ("conv2",)): 3348295,             # conv1 + conv2; algorithmic 2.7e6
}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--batch", type=int, default=64)
    ap.add_argument("--dtype", default="f32", choices=["f32", "f16", "bf16"])
    ap.add_argument("--graph", type=int, default=-1, choices=[-1, 0, 1],
                    help="0 layer-by-layer launches, 1 HIP graph replay, -1 (default) the faster of "
                         "the two by a short untimed trial")
    ap.add_argument("--no-tune", action="store_true")
    ap.add_argument("--variants", default="",
                    help="comma-separated tile variants of the dense layers in network order (the "
                         "`variants` list an earlier run printed): applied instead of timing, so that a run "
                         "under a profiler, which disturbs the timing, executes the same kernels")
    ap.add_argument("--fuse-first", type=int, default=-1, choices=[-1, 0, 1],
                    help="first two layers as one kernel: 1 yes, 0 no, -1 (default) as the timed selection decides "
                         "(no with --no-tune or --variants)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true", help="skip batch-1 and fp16 side figures")
    ap.add_argument("--cpu-images", type=int, default=0, help="oracle sample size (0 = auto)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run a plain 256 MiB channel copy (gather_channels_kernel with the identity "
                         "list) three times, as the known-size reference for HBM traffic counters")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no sharding, no collectives); "
              "use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    from paper_2207_01260_amd import binding as B
    from paper_2207_01260_amd import pipeline, synth

    assert torch.cuda.is_available(), "bench.py needs the GPU"
    torch.cuda.set_device(0)
    dt = {"f32": B.F32, "f16": B.F16, "bf16": B.BF16}[args.dtype]

    net = synth.vgg16(10, 32)
    cid = 2
    params = synth.layer_params(net, cid)
    dparams = pipeline.upload_params(params)

    def build(dtype, batch, tune):
        layers, kept = pipeline.prune_net(net, dparams, dtype)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        handle = pipeline.build_net(net, layers, batch, dtype, tune=tune)
        return handle, layers, kept, time.perf_counter() - t0

    def time_forward(handle, x, steps, warmup, graph):
        logits = torch.empty((x.shape[0], 10), dtype=x.dtype, device="cuda")
        for _ in range(warmup):
            handle.forward(x, logits, use_graph=graph)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            handle.forward(x, logits, use_graph=graph)
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / steps * 1e3

    # ---- prune stage (one-off), timed on its own -------------------------------------
    # the whole network as one plan: scores, kept lists, gathered + folded weights in three launches
    plan = pipeline.prune_plan(net, dparams, dt)
    for _ in range(3):
        plan.run()
    torch.cuda.synchronize()
    reps = 20
    t0 = time.perf_counter()
    for _ in range(reps):
        plan.run()
    torch.cuda.synchronize()
    prune_ms = (time.perf_counter() - t0) / reps * 1e3
    w_read, w_written = plan.traffic()
    prune_bytes = 4 * w_read + (4 if args.dtype == "f32" else 2) * w_written
    plan.close()
    # the same stage as one library call per layer and step (rank, gather + fold)
    pipeline.prune_net(net, dparams, dt)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(5):
        pipeline.prune_net(net, dparams, dt)
    torch.cuda.synchronize()
    prune_calls_ms = (time.perf_counter() - t0) / 5 * 1e3

    # ---- main measurement -------------------------------------------------------------
    pinned = [int(v) for v in args.variants.split(",") if v != ""]
    handle, layers, kept, tune_s = build(dt, args.batch, not (args.no_tune or pinned))
    dense = [i for i, L in enumerate(net.layers) if L.kind in ("conv", "fc")]
    if pinned:
        assert len(pinned) == len(dense), "--variants needs one entry per conv / fc layer"
        for i, v in zip(dense, pinned):
            if v >= 0:                           # -1: a layer without tile variants (first-layer kernel)
                handle.set_layer_variant(i, v)
    if args.fuse_first >= 0:
        handle.fuse_first_layers(bool(args.fuse_first))
    variants = [handle.layer_variant(i) for i in dense]
    kept_counts = {i: int(k.numel()) for i, k in kept.items()}
    x = torch.from_numpy(synth.net_input(net, cid, args.batch)).cuda().to(B.TORCH_DTYPE[dt])
    graph = args.graph
    if graph < 0:
        trial = {g: time_forward(handle, x, 30, 10, g) for g in (0, 1)}
        graph = min(trial, key=trial.get)
    graph = bool(graph)
    ms = time_forward(handle, x, args.steps, args.warmup, graph)
    value = args.batch / (ms * 1e-3)

    # per-layer device time (HIP events on the launch stream around back-to-back launches)
    layer_ms = handle.layer_times(x, iters=20)
    conv_ms = sum(m for m, L in zip(layer_ms, net.layers) if L.kind == "conv")
    n_conv = sum(1 for L in net.layers if L.kind == "conv")
    conv_flops = pipeline.useful_flops(net, kept_counts, args.batch, conv_only=True)
    total_flops = pipeline.useful_flops(net, kept_counts, args.batch)
    per_layer = []
    by_kernel = {}        # kernel instantiation -> [launches, ms, flop]
    shp = synth.shapes(net, kept_counts)
    tname = {"f32": "float", "f16": "_Float16", "bf16": "__bf16"}[args.dtype]
    carried = 0.0          # FLOP of a layer that runs inside its reader's kernel
    fused_first = False
    for i, (L, m) in enumerate(zip(net.layers, layer_ms)):
        if L.kind != "conv":
            continue
        cin, cout, ho, wo = shp[i]
        fl = 2.0 * args.batch * cout * cin * 9 * ho * wo
        if handle.layer_fused(i):                # the first layer inside the second layer's kernel
            carried, fused_first = fl, True
            per_layer.append({"layer": L.name, "c_in": cin, "c_out": cout, "hw": ho, "us": 0.0, "tflops": None,
                              "tile": "-", "kernel": "(inside the next layer's kernel)"})
            continue
        v = handle.layer_variant(i)
        first = L.input < 0 and cin <= 4         # reads the NCHW input itself
        if v < 0 and carried:                    # first two layers in one kernel: no tile variants
            mb = 1 if cout <= 16 else (2 if cout <= 32 else 4)
            tm, tp, sk = 16 * mb, 128, 0
            kern = "conv_stem2_kernel<%s, %d>" % (tname, mb)
        elif v < 0:                              # the first-layer kernel: no tile variants
            tm, tp, sk = 16 * (2 if cout <= 32 else 4), 128, 0
            kern = "conv_stem_kernel<%s, %d, %d, %d>" % (tname, L.k, L.stride, tm // 16)
        else:
            tm, tp, sk = B.cprune_tile_variant_info(v)
            kern = B.cprune_tile_variant_name(v, channels_last=not first, dtype=dt)
        fl, carried = fl + carried, 0.0
        note = (" + fix-up" if sk > 0 else "") + (" (2x2 map as one matrix)" if (ho == 2 and sk >= 0) else "")
        g = by_kernel.setdefault(kern, [0, 0.0, 0.0, []])
        g[0] += 1; g[1] += m; g[2] += fl; g[3].append(L.name)
        per_layer.append({"layer": L.name, "c_in": cin, "c_out": cout, "hw": ho, "us": round(m * 1e3, 2),
                          "tflops": round(fl / (m * 1e-3) / 1e12, 2), "tile": f"{tm}x{tp}/s{sk}",
                          "kernel": kern + note})
    # the dominant kernel: the instantiation with the most device time per step
    dom = max(by_kernel, key=lambda k: by_kernel[k][1])
    d_n, d_ms, d_fl, d_layers = by_kernel[dom]
    achieved = d_fl / (d_ms * 1e-3) / 1e12
    agg = conv_flops / (conv_ms * 1e-3) / 1e12

    out = {
        "metric": "images/sec pruned VGG-16 32x32",
        "value": round(value, 1), "unit": "images/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": args.dtype, "data": "synthetic",
        "config": {"workload": f"pruned VGG-16 (13 conv + FC), 32x32x3 inputs, keep ratios U(0.4,0.9), "
                               f"batch {args.batch}", "batch": args.batch, "hip_graph": graph,
                   "first_two_layers_one_kernel": fused_first,
                   "kept_filters": [kept_counts[i] for i in sorted(kept_counts)]},
        "useful_gflop_per_step": round(total_flops / 1e9, 3),
        "whole_net_tflops": round(total_flops / (ms * 1e-3) / 1e12, 2),
        "prune_ms": round(prune_ms, 4), "prune_per_layer_calls_ms": round(prune_calls_ms, 3),
        "prune": {"bound": "hbm", "launches": 3, "bytes": prune_bytes,
                  "achieved": round(prune_bytes / (prune_ms * 1e-3) / 1e9, 1), "peak": 8000.0, "unit": "GB/s",
                  "frac": round(prune_bytes / (prune_ms * 1e-3) / 8e12, 4),
                  "note": "raw weights read by scoring and by the gather + folded weights written, per run"},
        "tune_s": round(tune_s, 2), "variants": variants,
        "roofline": {"bound": "mfma", "kernel": dom, "launches_per_step": d_n,
                     "achieved": round(achieved, 2), "peak": PEAK[args.dtype], "unit": "TFLOP/s",
                     "frac": round(achieved / PEAK[args.dtype], 4),
                     "layers": d_layers,
                     "traffic": TRAFFIC.get((dom, args.batch, tuple(d_layers))),
                     "traffic_unit": "bytes per launch between L2 and fabric (FETCH_SIZE + WRITE_SIZE, scaled)",
                     "avg_launch_us": round(d_ms / d_n * 1e3, 2),
                     "useful_gflop_per_launch": round(d_fl / d_n / 1e9, 3),
                     "share_of_step": round(d_ms / ms, 3)},
        "conv_layers": {"layers": n_conv, "launches_per_step": n_conv - (1 if fused_first else 0), "tflops": round(agg, 2),
                        "frac_of_peak": round(agg / PEAK[args.dtype], 4),
                        "avg_layer_us": round(conv_ms / n_conv * 1e3, 2),
                        "useful_gflop_per_layer_avg": round(conv_flops / n_conv / 1e9, 3)},
        "layers": per_layer,
    }
    handle.close()

    if args.copy_calibration:
        big = torch.zeros((1, 64, 1024, 1024), dtype=torch.float32, device="cuda")
        ident = torch.arange(64, dtype=torch.int32, device="cuda")
        for _ in range(3):
            B.cprune_gather_channels(big, ident)
        torch.cuda.synchronize()
        out["copy_calibration"] = {"kernel": "gather_channels_kernel", "bytes_read": big.numel() * 4,
                                   "bytes_written": big.numel() * 4, "launches": 3}
        del big

    if not args.no_extras:
        extras = {}
        for name, dtype, batch in [("f32_b1", B.F32, 1), ("f16_b64", B.F16, 64), ("f16_b1", B.F16, 1),
                                   ("f32_b64", B.F32, 64)]:
            if dtype == dt and batch == args.batch:
                continue
            h, _, _, _ = build(dtype, batch, not args.no_tune)
            xb = torch.from_numpy(synth.net_input(net, cid, batch)).cuda().to(B.TORCH_DTYPE[dtype])
            m_graph = time_forward(h, xb, max(50, args.steps // 2), 10, True)
            m_eager = time_forward(h, xb, max(50, args.steps // 2), 10, False)
            extras[name] = {"images_per_s": round(batch / (min(m_graph, m_eager) * 1e-3), 1),
                            "ms_graph": round(m_graph, 4), "ms_eager": round(m_eager, 4)}
            h.close()
        out["extras"] = extras

    if not args.no_cpu_baseline:
        import oracle
        threads = oracle.num_threads()
        ref_layers, _ = oracle.prune_net(net, params)
        oracle.forward(net, ref_layers, synth.net_input(net, cid, 2))          # warm-up
        x8 = synth.net_input(net, cid, 16)
        t0 = time.perf_counter()
        oracle.forward(net, ref_layers, x8)
        per_img = (time.perf_counter() - t0) / 16
        n_img = args.cpu_images or int(min(2048, max(16, 15.0 / max(per_img, 1e-5))))
        xs = synth.net_input(net, cid, n_img)
        t0 = time.perf_counter()
        oracle.forward(net, ref_layers, xs)
        dt_cpu = time.perf_counter() - t0
        out["cpu_baseline"] = {"value": round(n_img / dt_cpu, 2), "unit": "images/s", "cores": threads,
                               "kind": "oracle",
                               "sample": f"{n_img} images of the same pruned VGG-16, fp64-accumulate "
                                         f"direct loops, OpenMP over (image, filter), {dt_cpu:.1f} s"}
        # the same loops on one thread, on a smaller sample
        n1 = max(4, min(64, int(3.0 * n_img / dt_cpu / max(threads, 1))))
        oracle.set_threads(1)
        x1 = synth.net_input(net, cid, n1)
        t0 = time.perf_counter()
        oracle.forward(net, ref_layers, x1)
        dt1 = time.perf_counter() - t0
        oracle.set_threads(threads)
        out["cpu_baseline"]["single_thread"] = {"value": round(n1 / dt1, 2), "unit": "images/s",
                                                "sample": f"{n1} images, {dt1:.1f} s"}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
