"""Host-side drivers built on the C-ABI calls: prune a whole network on the
device (rank -> gather -> fold, Section 3.5 of the paper) and wrap the result in
an inference handle (Algorithm 1: the candidate model is run on the device and
timed).  Only sequencing lives here; every tensor operation is a library call.
"""

from __future__ import annotations

from typing import Dict, List, Optional

import numpy as np
import torch

from . import binding as B
from . import synth

BN_EPS = float(np.float32(1e-5))


def upload_params(params: List[dict], device="cuda") -> List[dict]:
    out = []
    for p in params:
        q = {}
        for k, v in p.items():
            q[k] = torch.from_numpy(v).to(device) if isinstance(v, np.ndarray) else v
        out.append(q)
    return out


def prune_net(net: synth.NetSpec, dev_params: List[dict], dtype: int = B.F32,
              keep_override: Optional[Dict[int, int]] = None, stream=None):
    """Rank every 'own'-pruned layer, gather and fold all layers on the device.

    -> (layers, kept): per layer {'w': folded weights in `dtype`, 'b': fp32 bias} (empty
    for pools); kept: layer index -> int32 device tensor of surviving filters (ascending).
    """
    kept: Dict[int, torch.Tensor] = {}
    for i, (L, p) in enumerate(zip(net.layers, dev_params)):
        if L.prune_out == "own":
            k = (keep_override or {}).get(i, p["keep"])
            if L.score_with:     # layers that feed the same shortcut sum lose the same channels
                group = [p["w"]] + [dev_params[j]["w"] for j in L.score_with]
                _, _, kept[i] = B.cprune_rank_filter_group(group, k, want_scores=False, want_order=False,
                                                           stream=stream)
            else:
                _, _, kept[i] = B.cprune_rank_filters(p["w"], k, want_scores=False, want_order=False,
                                                      stream=stream)
    layers = []
    for i, (L, p) in enumerate(zip(net.layers, dev_params)):
        q: dict = {}
        if L.kind == "conv":
            ko = kept.get(i) if L.prune_out == "own" else (
                kept.get(L.prune_out) if isinstance(L.prune_out, int) else None)
            ki = kept.get(L.prune_in) if (L.prune_in is not None and L.groups == 1) else None
            bn = (p["gamma"], p["beta"], p["mean"], p["var"]) if L.bn else None
            q["w"], q["b"] = B.cprune_gather_pruned_weights(p["w"], ko, ki, bn, BN_EPS, None, dtype,
                                                            stream=stream)
        elif L.kind == "fc":
            ki = kept.get(L.prune_in) if L.prune_in is not None else None
            w4 = p["w"].reshape(p["w"].shape[0], p["w"].shape[1], 1, 1)
            w, _ = B.cprune_gather_pruned_weights(w4, None, ki, None, BN_EPS, None, dtype,
                                                  stream=stream)
            q["w"], q["b"] = w.reshape(w.shape[0], w.shape[1]), p["b"]
        layers.append(q)
    return layers, kept


def prune_plan(net: synth.NetSpec, dev_params: List[dict], dtype: int = B.F32,
               keep_override: Optional[Dict[int, int]] = None) -> B.PrunePlan:
    """The same pruning as prune_net, as one plan over the whole network: built once (outputs
    allocated once), every run is three launches.  plan_layers(net, dev_params, plan) gives the
    per-layer dicts prune_net returns."""
    entries = []
    for i, (L, p) in enumerate(zip(net.layers, dev_params)):
        if L.kind == "conv":
            own = L.prune_out == "own"
            entries.append({
                "w": p["w"], "keep": (keep_override or {}).get(i, p["keep"]) if own else 0,
                "rows_from": i if own else (L.prune_out if isinstance(L.prune_out, int) else -1),
                "cols_from": L.prune_in if (L.prune_in is not None and L.groups == 1) else -1,
                "score_with": list(L.score_with or []) if own else [],
                "bn": (p["gamma"], p["beta"], p["mean"], p["var"]) if L.bn else None})
        elif L.kind == "fc":
            w = p["w"]
            entries.append({"w": w.reshape(w.shape[0], w.shape[1], 1, 1), "keep": 0, "rows_from": -1,
                            "cols_from": L.prune_in if L.prune_in is not None else -1})
        else:
            entries.append(None)
    return B.PrunePlan(entries, BN_EPS, dtype)


def plan_layers(net: synth.NetSpec, dev_params: List[dict], plan: B.PrunePlan):
    """(layers, kept) of a plan's outputs, in the form prune_net returns them."""
    layers = []
    for i, (L, p) in enumerate(zip(net.layers, dev_params)):
        q: dict = {}
        if L.kind == "conv":
            q["w"], q["b"] = plan.w_out[i], plan.bias_out.get(i)
        elif L.kind == "fc":
            w = plan.w_out[i]
            q["w"], q["b"] = w.reshape(w.shape[0], w.shape[1]), p["b"]
        layers.append(q)
    return layers, dict(plan.kept)


def layer_descs(net: synth.NetSpec, layers: List[dict]) -> List[B.LayerDesc]:
    """cprune_layer_desc array for a pruned network (channel counts read off the weights)."""
    kind = {"conv": B.LAYER_CONV, "maxpool": B.LAYER_MAXPOOL, "gavgpool": B.LAYER_GAVGPOOL,
            "fc": B.LAYER_FC}
    out, c_out_of = [], []
    for L, q in zip(net.layers, layers):
        c_in = net.in_c if L.input < 0 else c_out_of[L.input]
        if L.kind in ("conv", "fc"):
            c_out = q["w"].shape[0]
            w_ptr, b_ptr = q["w"].data_ptr(), (q["b"].data_ptr() if q.get("b") is not None else None)
        else:
            c_out, w_ptr, b_ptr = c_in, None, None
        groups = c_in if L.groups != 1 else 1
        out.append(B.LayerDesc(kind[L.kind], L.input, -1 if L.residual is None else L.residual,
                               c_in, c_out, L.k, L.stride, L.pad, groups, L.act, w_ptr, b_ptr))
        c_out_of.append(c_out)
    return out


def build_net(net: synth.NetSpec, layers: List[dict], max_batch: int, dtype: int = B.F32,
              tune: bool = True, stream=None) -> B.Net:
    torch.cuda.current_stream().synchronize()
    return B.Net(layer_descs(net, layers), (net.in_c, net.in_h, net.in_w), max_batch, dtype, tune,
                 stream=stream)


def useful_flops(net: synth.NetSpec, kept_counts: Dict[int, int], batch: int, conv_only=False) -> int:
    """2 * multiply-adds on the pruned channel counts (never tile-padded)."""
    if not conv_only:
        return 2 * batch * synth.count_macs_params(net, kept_counts)[0]
    macs = 0
    for L, (cin, cout, ho, wo) in zip(net.layers, synth.shapes(net, kept_counts)):
        if L.kind == "conv" and L.groups == 1:
            macs += cout * cin * L.k * L.k * ho * wo
    return 2 * batch * macs
