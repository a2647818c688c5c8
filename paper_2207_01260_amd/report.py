"""Per-configuration report: every workload shape of the paper (VGG-16 on CIFAR-sized inputs, the
motivating experiment of Section 3, Fig. 1; ResNet-18, MobileNetV2 and MnasNet1.0 on ImageNet-sized inputs, Section 4.1 and Table 1) as a seeded,
synthetic, channel-pruned network, plus the single pruned layer and the measured ceilings of
the device.  One JSON object per line.

    python -m paper_2207_01260_amd.report [--quick] [--only NAME [--batch N] [--dtype f32|f16|bf16]
                                           [--variants=v0,v1,...] [--first-layer-form F]]

--only keeps the networks whose name contains NAME (and, with --batch / --dtype, that one run) and
skips the device ceilings and the single layer: the form a profiler run of one workload uses.  Every line
carries the tile variant each layer ran (`variants`, -1 for layers without one); --variants pins them (and skips
the timed selection, which a profiler's per-launch overhead would distort), --first-layer-form pins how a 16-bit
7x7 first layer runs, so that a profiled run executes the kernels an undisturbed run chose.

For each network and batch: images/s and ms per forward (at batch 1 also with the caches scrubbed
before every run: back-to-back replays keep the weights in the last-level cache) (HIP graph replay or eager launches,
whichever is faster), useful TFLOP/s on the pruned channel counts, and the device time by
layer kind (dense conv / depthwise / pool / fc) with what bounds it: dense layers against the
MFMA peak of the dtype, depthwise and pools against HBM bandwidth by the bytes they must move
(input once + output once); dense layers also show that byte rate (input, weights and output
once), since 1x1 layers with few channels are bandwidth-bound rather than MFMA-bound.
"""
import argparse
import json
import time

import torch

from . import binding as B
from . import pipeline, synth

PEAK_TFLOPS = {B.F32: 157.3, B.F16: 2500.0, B.BF16: 2500.0}
PEAK_GBS = 8000.0
DT_NAME = {B.F32: "f32", B.F16: "f16", B.BF16: "bf16"}


def time_forward(handle, x, steps, graph):
    out = handle.forward(x, use_graph=graph)
    for _ in range(5):
        handle.forward(x, out, use_graph=graph)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        handle.forward(x, out, use_graph=graph)
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) / steps * 1e3


def time_forward_cold(handle, x, steps):
    """ms per forward with the caches scrubbed before every run (a 1 GiB fill between runs: the
    last-level cache is 256 MiB), timed by events around the forward alone."""
    out = handle.forward(x)
    scrub = torch.empty(1 << 28, dtype=torch.float32, device="cuda")
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    total = 0.0
    for i in range(steps):
        scrub.fill_(float(i))
        e0.record()
        handle.forward(x, out)
        e1.record()
        e1.synchronize()
        total += e0.elapsed_time(e1)
    del scrub
    return total / steps


def net_report(name, net, cid, batch, dtype, steps, ceilings=None, variants=None, first_layer_form=None):
    params = synth.layer_params(net, cid)
    dparams = pipeline.upload_params(params)
    layers, kept = pipeline.prune_net(net, dparams, dtype)
    kept_counts = {i: int(k.numel()) for i, k in kept.items()}
    handle = pipeline.build_net(net, layers, batch, dtype, tune=variants is None)
    if first_layer_form is not None:
        handle.first_layer_form(first_layer_form)
    if variants is not None:
        if len(variants) != len(net.layers):
            raise SystemExit("--variants needs %d entries for %s" % (len(net.layers), name))
        for i, v in enumerate(variants):
            if v >= 0:
                handle.set_layer_variant(i, v)
    chosen = [handle.layer_variant(i) if (L.kind == "fc" or (L.kind == "conv" and L.groups == 1)) else -1
              for i, L in enumerate(net.layers)]
    x = torch.from_numpy(synth.net_input(net, cid, batch)).cuda().to(B.TORCH_DTYPE[dtype])
    ms = min(time_forward(handle, x, steps, g) for g in (False, True))
    ms_cold = time_forward_cold(handle, x, min(steps, 20)) if batch == 1 else None
    lt = handle.layer_times(x, iters=10)
    shp = synth.shapes(net, kept_counts)
    es = 4 if dtype == B.F32 else 2
    groups = {}
    for i, (L, t) in enumerate(zip(net.layers, lt)):
        cin, cout, ho, wo = shp[i]
        hin, win = (net.in_h, net.in_w) if L.input < 0 else shp[L.input][2:4]
        moved = es * batch * (cin * hin * win + cout * ho * wo)   # input once + output once
        if L.kind == "conv" and L.groups == 1:
            kind, fl = "dense_conv", 2.0 * batch * cout * cin * L.k * L.k * ho * wo
            by = moved + es * cout * cin * L.k * L.k
        elif L.kind == "conv":
            # 0 time: the layer runs inside the kernel of the 1x1 conv that reads it
            kind, fl, by = "depthwise", 2.0 * batch * cout * L.k * L.k * ho * wo, (moved if t > 0 else 0.0)
        elif L.kind == "fc":
            kind, fl, by = "fc", 2.0 * batch * cin * hin * win * cout, 0.0
        else:
            kind, fl, by = "pool", 0.0, (moved if t > 0 else 0.0)
        g = groups.setdefault(kind, {"ms": 0.0, "flop": 0.0, "bytes": 0.0, "launches": 0})
        g["ms"] += t; g["flop"] += fl; g["bytes"] += by; g["launches"] += 1 if t > 0 else 0
    by_kind = {}
    for kind, g in groups.items():
        row = {"ms": round(g["ms"], 4), "layers": g["launches"]}
        if g["flop"] and kind in ("dense_conv", "fc") and g["ms"] > 0:
            tf = g["flop"] / (g["ms"] * 1e-3) / 1e12
            row.update(tflops=round(tf, 2), frac_mfma_peak=round(tf / PEAK_TFLOPS[dtype], 4))
        if g["bytes"] and g["ms"] > 0:
            gbs = g["bytes"] / (g["ms"] * 1e-3) / 1e9
            row.update(gbs=round(gbs, 1), frac_hbm_peak=round(gbs / PEAK_GBS, 4))
            if ceilings:     # the same rate against what a plain copy of the same bytes reaches on this device
                row.update(frac_of_measured_copy=round(gbs / ceilings["copy_gbs"], 4))
        by_kind[kind] = row
    total = pipeline.useful_flops(net, kept_counts, batch)
    fused = sum(1 for i, L in enumerate(net.layers) if L.kind == "conv" and L.groups != 1 and handle.layer_fused(i))
    if fused:
        by_kind["depthwise"]["fused_into_their_1x1_reader"] = fused
    handle.close()
    return {"config": name, "batch": batch, "dtype": DT_NAME[dtype], "images_per_s": round(batch / (ms * 1e-3), 1),
            "ms_per_forward": round(ms, 4),
            **({"ms_per_forward_cold_caches": round(ms_cold, 4)} if ms_cold is not None else {}),
            "useful_gflop": round(total / 1e9, 3),
            "useful_tflops": round(total / (ms * 1e-3) / 1e12, 2), "by_layer_kind": by_kind, "variants": chosen}


def single_layer_report(steps):
    """One 3x3 conv + BN + ReLU at 32x32, 64 filters pruned to 45 by L1 rank, batch 1:
    latency-bound (53 MFLOP), so microseconds are the figure."""
    net = synth.single_conv(64, 64, 32)
    params = synth.layer_params(net, 1)
    dparams = pipeline.upload_params(params)
    rows = []
    for keep in (45, 64):
        layers, _ = pipeline.prune_net(net, dparams, B.F32, keep_override={0: keep})
        handle = pipeline.build_net(net, layers, 1, B.F32, tune=True)
        x = torch.from_numpy(synth.net_input(net, 1, 1)).cuda()
        us_handle = min(handle.layer_times(x, iters=50)[0] for _ in range(3)) * 1e3
        handle.close()
        d = B.conv_desc(x.shape, layers[0]["w"].shape, 1, 1)
        _, ms_api, _ = B.cprune_select_tile(d, x, layers[0]["w"], layers[0]["b"], warmup=3, iters=50)
        rows.append({"config": "single conv 64->%d @32x32 b1 f32" % keep, "us_in_handle": round(us_handle, 2),
                     "us_entry_point": round(ms_api * 1e3, 2), "mflop": round(2e-6 * keep * 64 * 9 * 1024, 1)})
    return rows


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--quick", action="store_true", help="fewer timed steps, small batches only")
    ap.add_argument("--only", default="", help="only the networks whose name contains this (case-insensitive)")
    ap.add_argument("--batch", type=int, default=0, help="with --only: only this batch size")
    ap.add_argument("--dtype", default="", choices=["", "f32", "f16", "bf16"], help="with --only: only this dtype")
    ap.add_argument("--variants", default="", help="with --only, --batch and --dtype: pin these tile variants (one per layer, "
                                                   "-1 = leave) instead of selecting by timing")
    ap.add_argument("--first-layer-form", type=int, default=None, choices=[0, 1, 2],
                    help="with --variants: how a 16-bit 7x7 / stride 2 first layer runs (see cprune_net_first_layer_form)")
    args = ap.parse_args()
    steps = 20 if args.quick else 100
    props = torch.cuda.get_device_properties(0)
    print(json.dumps({"device": props.name, "compute_units": props.multi_processor_count,
                      "clock_mhz": getattr(props, "clock_rate", 0) // 1000,
                      "hbm_gib": round(props.total_memory / 2 ** 30, 1)}), flush=True)
    ceilings = None
    if not args.only:
        ceilings = report_device(steps)
    cases = [("pruned VGG-16 32x32", synth.vgg16(10, 32), 2, [(1, B.F32), (64, B.F32), (1, B.F16), (64, B.F16)]),
             ("pruned ResNet-18 224x224", synth.resnet18(1000, 224), 3, [(1, B.F32), (32, B.F32), (1, B.BF16), (32, B.BF16)]),
             ("pruned MobileNetV2 224x224", synth.mobilenetv2(1000, 224), 4, [(1, B.F32), (64, B.F32)]),
             ("pruned MnasNet1.0 224x224", synth.mnasnet(1000, 224), 6, [(1, B.F32), (64, B.F32)])]
    for name, net, cid, runs in cases:
        if args.only and args.only.lower() not in name.lower():
            continue
        for batch, dtype in runs:
            if args.quick and not args.only and batch > 1 and "VGG" not in name:
                continue
            if args.only and ((args.batch and batch != args.batch) or (args.dtype and DT_NAME[dtype] != args.dtype)):
                continue
            pinned = [int(v) for v in args.variants.split(",")] if args.variants else None
            if pinned is not None and not (args.only and args.batch and args.dtype):
                raise SystemExit("--variants needs --only, --batch and --dtype")
            print(json.dumps(net_report(name, net, cid, batch, dtype, steps, ceilings, pinned, args.first_layer_form)), flush=True)


def report_device(steps):
    ceil = {"mfma_f32_tflops": round(B.cprune_probe_mfma(B.F32), 1),
            "mfma_f16_tflops": round(B.cprune_probe_mfma(B.F16), 1),
            "mfma_bf16_tflops": round(B.cprune_probe_mfma(B.BF16), 1),
            "copy_gbs": round(B.cprune_probe_copy(1 << 32), 1),      # 4 GiB each way: well past the 256 MiB last-level cache
            "read_only_gbs": round(B.cprune_probe_read(1 << 32), 1),
            "write_only_gbs": round(B.cprune_probe_write(1 << 32), 1),
            "l2_read_gbs_per_cu": {"consecutive_kib": round(B.cprune_probe_l2_read(0), 1),
                                   "rows_of_64_bytes": round(B.cprune_probe_l2_read(1), 1)},
            "datasheet": {"mfma_f32_tflops": 157.3, "mfma_f16_bf16_tflops": 2500.0, "hbm_gbs": 8000.0}}
    print(json.dumps({"measured_ceilings": ceil}), flush=True)
    for row in single_layer_report(steps):
        print(json.dumps(row), flush=True)
    return ceil


if __name__ == "__main__":
    main()
