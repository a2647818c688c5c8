"""Channel-count sweep of one pruned conv layer: latency, useful TFLOP/s and the tile variant
picked by timing, for every number of surviving filters.

The paper observes that a convolution's execution time grows in steps, not linearly, with
the number of filters (Section 3.5); this measures that staircase on the device for a 3x3
conv + BN + ReLU at 56x56, C_in = 128, batch 8, fp32, with the filters pruned from 128
down to every count 1..128 by L1 rank.

    python -m paper_2207_01260_amd.sweep [--out sweep.json] [--step 1]
"""
import argparse
import json

import torch

from . import binding as B
from . import pipeline, synth


def run(c_in=128, c_full=128, hw=56, batch=8, dtype=B.F32, step=1, iters=20, direct_api=False, counts=None):
    """One row per number of surviving filters.  Default: the layer runs inside a one-layer
    inference handle (channels-last kernels, variant picked by timing at handle creation,
    time = device time of the layer by HIP events).  direct_api=True times the NCHW entry
    point cprune_conv2d_bn_relu with cprune_select_tile instead.  counts: only these filter counts."""
    net = synth.single_conv(c_in, c_full, hw)
    params = synth.layer_params(net, 5)
    dparams = pipeline.upload_params(params)
    x = torch.from_numpy(synth.net_input(net, 5, batch)).cuda().to(B.TORCH_DTYPE[dtype])
    rows = []
    for c_out in (counts if counts is not None else range(1, c_full + 1, step)):
        layers, _ = pipeline.prune_net(net, dparams, dtype, keep_override={0: c_out})
        w, b = layers[0]["w"], layers[0]["b"]
        if direct_api:
            d = B.conv_desc(x.shape, w.shape, 1, 1, 1, dtype)
            v, ms, _ = B.cprune_select_tile(d, x, w, b, warmup=2, iters=iters)
        else:
            handle = pipeline.build_net(net, layers, batch, dtype, tune=True)
            ms = min(handle.layer_times(x, iters=iters)[0] for _ in range(2))
            v = handle.layer_variant(0)
            handle.close()
        tm, tp, sched = B.cprune_tile_variant_info(v)
        flops = 2.0 * batch * hw * hw * c_out * c_in * 9
        rows.append({"c_out": c_out, "us": round(ms * 1e3, 2), "tflops": round(flops / ms / 1e9, 2),
                     "tile_m": tm, "tile_p": tp, "sched": sched})
    return rows


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--out", default="")
    ap.add_argument("--step", type=int, default=1)
    ap.add_argument("--direct-api", action="store_true", help="time the NCHW entry point instead")
    args = ap.parse_args()
    rows = run(step=args.step, direct_api=args.direct_api)
    inversions = sum(1 for a, b in zip(rows, rows[1:]) if b["us"] < a["us"] * 0.97)
    worst_step = max((b["us"] - a["us"] for a, b in zip(rows, rows[1:])), default=0.0)
    summary = {"workload": "3x3 conv+BN+ReLU 56x56 C_in=128 batch 8 fp32, C_out' = 1..128",
               "path": "NCHW entry point" if args.direct_api else "one-layer inference handle",
               "inversions_over_3pct": inversions, "largest_step_us": round(worst_step, 2),
               "rows": rows}
    text = json.dumps(summary)
    if args.out:
        open(args.out, "w").write(text)
    for r in rows:
        print(r)
    print({k: v for k, v in summary.items() if k != "rows"})


if __name__ == "__main__":
    main()
