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
# reads for a copy kernel of known size), by (kernel instantiation, batch, layer), for the default
# workload: from the rocprofv3 counter runs summarised in profiles/vgg16_b64_f32_hbm_traffic.md (five
# pinned selections, because the timed selection flips between near-equal variants).  The figures belong
# to the kernel sources they were measured on: TRAFFIC_SOURCE_HASH is kernel_source_hash() of that tree,
# and any change to a file under csrc/ since then reports null instead of a stale figure (as does a
# selection that runs a kernel on a layer it was not profiled on).
TRAFFIC_SOURCE_HASH = "44ade6751b488d6a"
TRAFFIC = {
    ("conv_stem2_kernel<float, 2>", 64, "conv2"): 3350342,
    ("conv_patch_kernel<float, 1, 8, 8, 1, 1, 1>", 64, "conv3"): 10522153,
    ("conv_patch_kernel<float, 1, 8, 8, 1, 2, 1>", 64, "conv3"): 10552867,
    ("conv_patch_kernel<float, 1, 8, 8, 1, 2, 2>", 64, "conv3"): 10528295,
    ("conv_patch_kernel<float, 2, 8, 8, 1, 1, 1>", 64, "conv3"): 10578463,
    ("conv_patch32_kernel<float, 1, 1, 4, 8, 16, 1, 1>", 64, "conv4"): 10128045,
    ("conv_patch_kernel<float, 2, 8, 16, 1, 1, 1>", 64, "conv4"): 10117802,
    ("conv_patch_kernel<float, 2, 8, 16, 1, 1, 2>", 64, "conv4"): 10109612,
    ("conv_patch_kernel<float, 2, 8, 8, 1, 1, 1>", 64, "conv4"): 10100399,
    ("conv_patch_kernel<float, 1, 8, 8, 1, 1, 1>", 64, "conv5"): 4493931,
    ("conv_patch_kernel<float, 1, 8, 8, 1, 2, 1>", 64, "conv5"): 4524648,
    ("conv_patch_kernel<float, 1, 8, 8, 1, 2, 2>", 64, "conv5"): 4500075,
    ("conv_patch_kernel<float, 1, 8, 8, 1, 1, 1>", 64, "conv6"): 10399661,
    ("conv_patch_kernel<float, 1, 8, 8, 1, 2, 1>", 64, "conv6"): 10430378,
    ("conv_patch_kernel<float, 1, 8, 8, 1, 2, 2>", 64, "conv6"): 10405808,
    ("conv_patch_kernel<float, 1, 8, 8, 1, 1, 1>", 64, "conv7"): 12095845,
    ("conv_patch_kernel<float, 1, 8, 8, 1, 2, 1>", 64, "conv7"): 12126557,
    ("conv_patch_kernel<float, 1, 8, 8, 1, 2, 2>", 64, "conv7"): 12104034,
    ("conv_wave_kernel<float, 2, 2, 2>", 64, "conv7"): 13495440,
    ("conv_wave_kernel<float, 2, 2, 2>", 64, "conv8"): 9394120,
    ("conv_wave_kernel<float, 2, 2, 4>", 64, "conv8"): 9401286,
    ("conv_wave_kernel<float, 5, 1, 3>", 64, "conv8"): 16851363,
    ("conv_wave_kernel<float, 2, 2, 2>", 64, "conv9"): 15049581,
    ("conv_wave_kernel<float, 2, 2, 4>", 64, "conv9"): 15056750,
    ("conv_wave_kernel<float, 5, 1, 3>", 64, "conv9"): 20934069,
    ("conv_wave_kernel<float, 2, 2, 2>", 64, "conv10"): 11484552,
    ("conv_wave_kernel<float, 2, 2, 4>", 64, "conv10"): 11491715,
    ("conv_wave_kernel<float, 5, 1, 3>", 64, "conv10"): 18686818,
    ("conv_ksplit_kernel<float, 1, 16>", 64, "conv11"): 7694001,
    ("conv_ksplit_kernel<float, 1, 4>", 64, "conv11"): 7678645,
    ("conv_ksplit_kernel<float, 1, 8>", 64, "conv11"): 7689905,
    ("conv_ksplit_kernel<float, 1, 16>", 64, "conv12"): 6407791,
    ("conv_ksplit_kernel<float, 1, 4>", 64, "conv12"): 6392431,
    ("conv_ksplit_kernel<float, 1, 8>", 64, "conv12"): 6403696,
    ("conv_ksplit_kernel<float, 1, 4>", 64, "conv13"): 7768205,
    ("conv_ksplit_kernel<float, 2, 4>", 64, "conv13"): 7537585,
    ("conv_ksplit_kernel<float, 2, 8>", 64, "conv13"): 7537586,
}


def dominant_traffic(kernel, batch, layers):
    """Bytes per launch of `kernel`, averaged over the layers it ran; None unless every one of them was
    profiled with this kernel on this very source tree."""
    if kernel_source_hash() != TRAFFIC_SOURCE_HASH:
        return None
    figures = [TRAFFIC.get((kernel, batch, name)) for name in layers]
    if not figures or any(f is None for f in figures):
        return None
    return int(sum(figures) / len(figures))


def kernel_source_hash():
    """sha256 over the HIP sources the library is built from (names and contents, in name order)."""
    import hashlib
    d = os.path.join(ROOT, "paper_2207_01260_amd", "csrc")
    h = hashlib.sha256()
    for name in sorted(os.listdir(d)):
        if name.endswith((".hip", ".hpp")):
            h.update(name.encode())
            h.update(open(os.path.join(d, name), "rb").read())
    return h.hexdigest()[:16]


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
    ap.add_argument("--no-configs", action="store_true",
                    help="skip the side figures of the other workloads (single layer, ResNet-18, MobileNetV2, "
                         "channel sweep points)")
    ap.add_argument("--print-source-hash", action="store_true",
                    help="print kernel_source_hash() of this tree and exit (what traffic figures are stamped with)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run a plain 256 MiB channel copy (gather_channels_kernel with the identity "
                         "list) three times, as the known-size reference for HBM traffic counters")
    args = ap.parse_args()
    if args.print_source_hash:
        print(kernel_source_hash())
        return
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
                     "traffic": dominant_traffic(dom, args.batch, d_layers),
                     "traffic_unit": "bytes per launch between L2 and fabric (FETCH_SIZE + WRITE_SIZE, scaled); null when "
                                     "the kernel sources differ from the profiled tree or the kernel ran other layers",
                     "kernel_source_hash": kernel_source_hash(),
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
        from paper_2207_01260_amd import report
        # what the device delivers, beside the datasheet peaks every fraction above is taken against
        out["measured_ceilings"] = {
            "mfma_tflops": {"f32": round(B.cprune_probe_mfma(B.F32), 1), "f16": round(B.cprune_probe_mfma(B.F16), 1)},
            "hbm_gbs": {"copy_read_plus_written": round(B.cprune_probe_copy(1 << 32), 1),
                        "read_only": round(B.cprune_probe_read(1 << 32), 1),
                        "write_only": round(B.cprune_probe_write(1 << 32), 1)},
            "datasheet": {"mfma_f32_tflops": 157.3, "mfma_f16_tflops": 2500.0, "hbm_gbs": 8000.0},
            "note": "4 GiB streams (the last-level cache holds 256 MiB); MFMA rate from registers, no memory traffic"}
        extras = {}
        for name, dtype, batch in [("f32_b1", B.F32, 1), ("f16_b64", B.F16, 64), ("f16_b1", B.F16, 1),
                                   ("f32_b64", B.F32, 64)]:
            if dtype == dt and batch == args.batch:
                continue
            h, lay_b, kept_b, _ = build(dtype, batch, not args.no_tune)
            xb = torch.from_numpy(synth.net_input(net, cid, batch)).cuda().to(B.TORCH_DTYPE[dtype])
            m_graph = time_forward(h, xb, max(50, args.steps // 2), 10, True)
            m_eager = time_forward(h, xb, max(50, args.steps // 2), 10, False)
            extras[name] = {"images_per_s": round(batch / (min(m_graph, m_eager) * 1e-3), 1),
                            "ms_graph": round(m_graph, 4), "ms_eager": round(m_eager, 4)}
            if batch == 1:
                # back-to-back replays keep the weights in the last-level cache; this is with the caches
                # scrubbed (a 1 GiB fill) before every forward, timed by events around the forward alone
                extras[name]["ms_cold_caches"] = round(report.time_forward_cold(h, xb, 20), 4)
                lt1 = h.layer_times(xb, iters=20)
                extras[name]["launches"] = sum(1 for t in lt1 if t > 0)
                extras[name]["sum_of_layer_us"] = round(sum(lt1) * 1e3, 2)
            if name == "f16_b64":
                # per layer: which roofline bounds it (arithmetic intensity on input + weights + output once
                # against the ridge 2.5 PFLOP/s / 8 TB/s = 312 FLOP/B) and how close the layer runs to it
                kc = {i: int(k.numel()) for i, k in kept_b.items()}
                shp16 = synth.shapes(net, kc)
                rows, t_bound, t_meas = [], 0.0, 0.0
                for i, (L, t) in enumerate(zip(net.layers, h.layer_times(xb, iters=20))):
                    if L.kind != "conv" or t <= 0:
                        continue
                    cin, cout, ho, wo = shp16[i]
                    hin = net.in_h if L.input < 0 else shp16[L.input][2]
                    fl = 2.0 * batch * cout * cin * 9 * ho * wo
                    if L.input >= 0 and h.layer_fused(L.input):      # carries the first layer's work
                        ci0, co0, h0, w0 = shp16[L.input]
                        fl += 2.0 * batch * co0 * ci0 * 9 * h0 * w0
                    by = 2.0 * (batch * cin * hin * hin + cout * cin * 9 + batch * cout * ho * wo)
                    t_mfma, t_hbm = fl / 2.5e15, by / 8e12
                    bound = "mfma" if t_mfma >= t_hbm else "hbm"
                    floor = max(t_mfma, t_hbm)
                    rows.append({"layer": L.name, "us": round(t * 1e3, 2), "flop_per_byte": round(fl / by, 1),
                                 "bound": bound, "floor_us": round(floor * 1e6, 2),
                                 "frac_of_bound": round(floor / (t * 1e-3), 4)})
                    t_bound += floor; t_meas += t * 1e-3
                extras[name]["roofline"] = {"peak_tflops": 2500.0, "peak_gbs": 8000.0, "ridge_flop_per_byte": 312.5,
                                            "conv_layers_frac_of_bound": round(t_bound / t_meas, 4),
                                            "note": "a layer's floor is the larger of its MFMA time and its HBM time; "
                                                    "launches of 3-10 us each, about 2 us of which is the launch itself",
                                            "layers": rows}
            h.close()
        out["extras"] = extras

        if not args.no_configs:
            cfg = {}
            # the single pruned layer: 64 filters ranked, 45 kept, 32x32, batch 1 (53 MFLOP: latency-bound)
            row = report.single_layer_report(50)[0]
            cfg["single_conv_64to45_32x32_b1_f32"] = {"us_in_handle": row["us_in_handle"],
                                                      "us_entry_point": row["us_entry_point"], "bound": "launch latency"}
            # ResNet-18 224x224, batch 32
            for dtype in (B.F32, B.BF16):
                r = report.net_report("resnet18", synth.resnet18(1000, 224), 3, 32, dtype, 20)
                d = r["by_layer_kind"]["dense_conv"]
                cfg["resnet18_224_b32_" + r["dtype"]] = {
                    "images_per_s": r["images_per_s"], "ms": r["ms_per_forward"], "bound": "mfma",
                    "dense_conv_tflops": d.get("tflops"), "frac": d.get("frac_mfma_peak")}
            # MobileNetV2 224x224, batch 64: bandwidth-bound layers
            r = report.net_report("mobilenetv2", synth.mobilenetv2(1000, 224), 4, 64, B.F32, 20)
            k = r["by_layer_kind"]
            cfg["mobilenetv2_224_b64_f32"] = {
                "images_per_s": r["images_per_s"], "ms": r["ms_per_forward"], "bound": "hbm",
                "dense_conv_gbs": k["dense_conv"].get("gbs"), "frac": k["dense_conv"].get("frac_hbm_peak"),
                "depthwise_gbs": k.get("depthwise", {}).get("gbs"),
                "depthwise_fused_into_reader": k.get("depthwise", {}).get("fused_into_their_1x1_reader", 0)}
            # channel sweep of the 56x56 layer, seven of the 128 counts (tests/test_gpu_fullsize.py runs all)
            from paper_2207_01260_amd import sweep
            counts = [1, 16, 17, 45, 64, 112, 128]
            rows = {r["c_out"]: r for r in sweep.run(step=1, counts=counts)}
            us = [rows[c]["us"] for c in counts]
            cfg["conv3x3_56x56_cin128_b8_f32_sweep"] = {
                "us_by_c_out": {str(c): rows[c]["us"] for c in counts},
                "tflops_at_128": rows[128]["tflops"], "frac_at_128": round(rows[128]["tflops"] / 157.3, 4),
                "bound": "mfma", "inversions_over_3pct": sum(1 for a, b in zip(us, us[1:]) if b < 0.97 * a)}
            extras["configs"] = cfg

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
        # the same loops accumulating in float (the GPU path's own accumulation width), all threads
        oracle.timing_build(True)
        try:
            t0 = time.perf_counter()
            oracle.forward(net, ref_layers, xs[: max(16, n_img // 2)])
            dtf = time.perf_counter() - t0
        finally:
            oracle.timing_build(False)
        out["cpu_baseline"]["f32_accumulate"] = {"value": round(max(16, n_img // 2) / dtf, 2), "unit": "images/s",
                                                 "sample": f"{max(16, n_img // 2)} images, {dtf:.1f} s, same loops with a "
                                                           "float accumulator (timing only, never a reference)"}
        # the GPU result on images of the same sample against the oracle's (the measure of the tests)
        n_par = min(16, n_img)
        hp, _, _, _ = build(dt, n_par, False)
        got = hp.forward(torch.from_numpy(xs[:n_par]).cuda().to(B.TORCH_DTYPE[dt])).float().cpu().numpy().astype(np.float64)
        hp.close()
        want = oracle.forward(net, ref_layers, xs[:n_par]).astype(np.float64)
        rtol = 1e-4 if args.dtype == "f32" else 2e-2
        rms = float(np.sqrt(np.mean(want * want)))
        out["cpu_baseline"]["parity_of_sample"] = {
            "images": n_par, "max_abs_err_over_max_abs_ref": float(np.max(np.abs(got - want)) / np.max(np.abs(want))),
            "rtol": rtol,
            "elementwise_pass_rate": float(np.mean(np.abs(got - want) <= rtol * np.abs(want) + rtol * rms)),
            "definition": "|g - r| <= rtol |r| + rtol rms(r) per logit"}
        if not args.no_configs:
            # the other workloads, one repetition each on a few images
            others = {}
            for label, onet, ocid, nimg in (("resnet18_224", synth.resnet18(1000, 224), 3, 4),
                                            ("mobilenetv2_224", synth.mobilenetv2(1000, 224), 4, 4)):
                op = synth.layer_params(onet, ocid)
                ol, _ = oracle.prune_net(onet, op)
                ox = synth.net_input(onet, ocid, nimg)
                t0 = time.perf_counter()
                oracle.forward(onet, ol, ox)
                dto = time.perf_counter() - t0
                others[label] = {"value": round(nimg / dto, 2), "unit": "images/s", "sample": f"{nimg} images, {dto:.1f} s"}
            snet = synth.single_conv(128, 128, 56)
            sp = synth.layer_params(snet, 5)
            sx = synth.net_input(snet, 5, 8)
            sweep_rows = {}
            for k in (1, 16, 45, 64, 128):
                sp[0]["keep"] = k
                sl, _ = oracle.prune_net(snet, sp)
                t0 = time.perf_counter()
                oracle.forward(snet, sl, sx)
                sweep_rows[str(k)] = round((time.perf_counter() - t0) * 1e3, 1)
            others["conv3x3_56x56_cin128_b8_sweep_ms_by_c_out"] = sweep_rows
            out["cpu_baseline"]["other_workloads"] = others
    print(json.dumps(out))


if __name__ == "__main__":
    main()
