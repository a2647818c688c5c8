"""Seeded synthetic workloads: random tensors and network layer lists.

This module holds no arithmetic of the pruning / inference method itself: it
draws random numbers from a counter-based generator and describes network
shapes as plain data.  Both the GPU path and the CPU oracle take their inputs
from here, which is the only thing they have in common.

Generator: splitmix64 (Steele, Lea, Flood 2014) applied to ``key + i``, top 53
bits -> uniform double in [0, 1); normals by Box-Muller in double.  A stream is
named by ``stream_key(base_seed, *tags)`` so tensors are independent of the
order in which they are drawn.

Networks follow the workloads the paper evaluates (VGG-16 on 32x32 inputs in
the motivating experiment that opens Section 3, Fig. 1; ResNet-18 and MobileNetV2 in
Table 1; the CIFAR ResNet-18 of Table 2), as layer lists whose multiply-add and
parameter counts reproduce the figures printed in Tables 1 and 2.
"""

from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import Dict, List, Optional, Tuple

import numpy as np

BASE_SEED = 220701260

_U64 = np.uint64
_MASK = (1 << 64) - 1


# --------------------------------------------------------------------------
# counter-based random numbers
# --------------------------------------------------------------------------

def _splitmix64_scalar(x: int) -> int:
    x = (x + 0x9E3779B97F4A7C15) & _MASK
    z = x
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & _MASK
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & _MASK
    return z ^ (z >> 31)


def _splitmix64(x: np.ndarray) -> np.ndarray:
    with np.errstate(over="ignore"):
        z = x + _U64(0x9E3779B97F4A7C15)
        z = (z ^ (z >> _U64(30))) * _U64(0xBF58476D1CE4E5B9)
        z = (z ^ (z >> _U64(27))) * _U64(0x94D049BB133111EB)
        return z ^ (z >> _U64(31))


def stream_key(base: int, *tags: int) -> int:
    """Mix integer tags into a 64-bit stream key."""
    k = _splitmix64_scalar(base & _MASK)
    for t in tags:
        k = _splitmix64_scalar(k ^ ((int(t) * 0xD6E8FEB86659FD93) & _MASK))
    return k


def uniform01(key: int, n: int) -> np.ndarray:
    """n doubles in [0, 1)."""
    with np.errstate(over="ignore"):
        ctr = _U64(key) + np.arange(n, dtype=np.uint64)
    bits = _splitmix64(ctr)
    return (bits >> _U64(11)).astype(np.float64) * (1.0 / 9007199254740992.0)


def uniform(key: int, n: int, lo: float, hi: float) -> np.ndarray:
    return lo + (hi - lo) * uniform01(key, n)


def normal(key: int, n: int, mean: float = 0.0, std: float = 1.0) -> np.ndarray:
    """n doubles ~ N(mean, std^2), Box-Muller on pairs of uniforms."""
    m = (n + 1) // 2
    u1 = 1.0 - uniform01(stream_key(key, 1), m)          # (0, 1]
    u2 = uniform01(stream_key(key, 2), m)
    r = np.sqrt(-2.0 * np.log(u1))
    z = np.empty(2 * m, dtype=np.float64)
    z[0::2] = r * np.cos(2.0 * math.pi * u2)
    z[1::2] = r * np.sin(2.0 * math.pi * u2)
    return mean + std * z[:n]


# --------------------------------------------------------------------------
# network layer lists
# --------------------------------------------------------------------------

ACT_NONE, ACT_RELU, ACT_RELU6 = 0, 1, 2


@dataclass
class Layer:
    """One node of a network, as plain data.

    kind      'conv' | 'maxpool' | 'gavgpool' | 'fc'
    input     index of the producing layer, -1 = network input
    residual  index of the layer added before the activation, or None
    prune_out None: all filters stay; 'own': filters ranked and pruned by their
              own L1 norm; int i: output channels follow layer i's kept list
              (depthwise conv behind a pruned expansion)
    prune_in  int i: input channels gathered by layer i's kept list; else None
    score_with  for an 'own'-pruned layer: indices of other layers (same c_out) whose filter
              norms are added to its own before ranking; those layers set prune_out to this
              layer's index, so that all of them lose the same channels (layers whose outputs
              a shortcut adds)
    """
    kind: str
    input: int
    c_in: int
    c_out: int
    k: int = 1
    stride: int = 1
    pad: int = 0
    groups: int = 1
    act: int = ACT_NONE
    bn: bool = False
    bias: bool = False
    residual: Optional[int] = None
    score_with: Optional[List[int]] = None
    prune_out: object = None
    prune_in: Optional[int] = None
    name: str = ""


@dataclass
class NetSpec:
    name: str
    in_c: int
    in_h: int
    in_w: int
    layers: List[Layer] = field(default_factory=list)
    keep_lo: float = 1.0
    keep_hi: float = 1.0

    def add(self, layer: Layer) -> int:
        self.layers.append(layer)
        return len(self.layers) - 1


def vgg16(num_classes: int = 10, in_hw: int = 32) -> NetSpec:
    """13 conv3x3+BN+ReLU, five 2x2 max-pools, one FC; every conv pruned."""
    cfg = [64, 64, "M", 128, 128, "M", 256, 256, 256, "M",
           512, 512, 512, "M", 512, 512, 512, "M"]
    net = NetSpec("vgg16", 3, in_hw, in_hw, keep_lo=0.4, keep_hi=0.9)
    prev, c, last_conv, ci = -1, 3, None, 0
    for v in cfg:
        if v == "M":
            prev = net.add(Layer("maxpool", prev, c, c, k=2, stride=2, name="pool"))
        else:
            ci += 1
            prev = net.add(Layer("conv", prev, c, v, k=3, stride=1, pad=1, act=ACT_RELU,
                                 bn=True, prune_out="own", prune_in=last_conv,
                                 name=f"conv{ci}"))
            last_conv, c = prev, v
    net.add(Layer("fc", prev, c, num_classes, bias=True, prune_in=last_conv, name="fc"))
    return net


def resnet18(num_classes: int = 1000, in_hw: int = 224, cifar_stem: bool = False,
             prune_shortcuts: bool = False) -> NetSpec:
    """Basic-block ResNet-18; the first conv of each block is the pruned one.

    prune_shortcuts: also prune the channels that run along the shortcuts.  Every layer that
    writes into one stage's shortcut sum (the stem or the stage's 1x1 downsample conv, and
    the second conv of both blocks) must lose the same channels: the first of them in layer
    order ranks the sum of all their filter norms, the others follow its list, and every
    reader of the sum (the next convs, the next downsample, the FC) drops the matching inputs."""
    net = NetSpec("resnet18_cifar" if cifar_stem else "resnet18", 3, in_hw, in_hw,
                  keep_lo=0.3, keep_hi=0.9)
    lead = None           # layer whose kept list governs the current shortcut stream
    if cifar_stem:
        prev = net.add(Layer("conv", -1, 3, 64, k=3, stride=1, pad=1, act=ACT_RELU, bn=True,
                             name="stem"))
        stem = prev
    else:
        prev = net.add(Layer("conv", -1, 3, 64, k=7, stride=2, pad=3, act=ACT_RELU, bn=True,
                             name="stem"))
        stem = prev
        prev = net.add(Layer("maxpool", prev, 64, 64, k=3, stride=2, pad=1, name="pool"))
    if prune_shortcuts:
        lead = stem
        net.layers[stem].prune_out = "own"
        net.layers[stem].score_with = []
    c = 64
    for si, width in enumerate([64, 128, 256, 512]):
        for bi in range(2):
            stride = 2 if (si > 0 and bi == 0) else 1
            block_in = prev
            stream_in = lead
            if stride != 1 or c != width:
                short = net.add(Layer("conv", block_in, c, width, k=1, stride=stride, pad=0,
                                      act=ACT_NONE, bn=True, prune_in=stream_in, name=f"s{si}b{bi}.down"))
                if prune_shortcuts:
                    lead = short
                    net.layers[short].prune_out = "own"
                    net.layers[short].score_with = []
            else:
                short = block_in
            c1 = net.add(Layer("conv", block_in, c, width, k=3, stride=stride, pad=1,
                               act=ACT_RELU, bn=True, prune_out="own", prune_in=stream_in,
                               name=f"s{si}b{bi}.conv1"))
            prev = net.add(Layer("conv", c1, width, width, k=3, stride=1, pad=1, act=ACT_RELU,
                                 bn=True, residual=short, prune_in=c1, prune_out=lead,
                                 name=f"s{si}b{bi}.conv2"))
            if prune_shortcuts:
                net.layers[lead].score_with.append(prev)
            c = width
    prev = net.add(Layer("gavgpool", prev, c, c, name="gap"))
    net.add(Layer("fc", prev, c, num_classes, bias=True, prune_in=lead, name="fc"))
    return net


def mobilenetv2(num_classes: int = 1000, in_hw: int = 224) -> NetSpec:
    """Width-1.0 MobileNetV2; the expansion channels of every t=6 block are pruned."""
    net = NetSpec("mobilenetv2", 3, in_hw, in_hw, keep_lo=0.4, keep_hi=0.9)
    prev = net.add(Layer("conv", -1, 3, 32, k=3, stride=2, pad=1, act=ACT_RELU6, bn=True,
                         name="stem"))
    c = 32
    table = [(1, 16, 1, 1), (6, 24, 2, 2), (6, 32, 3, 2), (6, 64, 4, 2),
             (6, 96, 3, 1), (6, 160, 3, 2), (6, 320, 1, 1)]
    bidx = 0
    for t, cout, n, s in table:
        for i in range(n):
            stride = s if i == 0 else 1
            block_in = prev
            hidden = c * t
            exp = None
            if t != 1:
                exp = net.add(Layer("conv", prev, c, hidden, k=1, act=ACT_RELU6, bn=True,
                                    prune_out="own", name=f"b{bidx}.expand"))
                prev = exp
            prev = net.add(Layer("conv", prev, hidden, hidden, k=3, stride=stride, pad=1,
                                 groups=hidden, act=ACT_RELU6, bn=True, prune_out=exp,
                                 name=f"b{bidx}.dw"))
            res = block_in if (stride == 1 and c == cout) else None
            prev = net.add(Layer("conv", prev, hidden, cout, k=1, act=ACT_NONE, bn=True,
                                 residual=res, prune_in=exp, name=f"b{bidx}.project"))
            c = cout
            bidx += 1
    prev = net.add(Layer("conv", prev, c, 1280, k=1, act=ACT_RELU6, bn=True, name="last"))
    prev = net.add(Layer("gavgpool", prev, 1280, 1280, name="gap"))
    net.add(Layer("fc", prev, 1280, num_classes, bias=True, name="fc"))
    return net


def mnasnet(num_classes: int = 1000, in_hw: int = 224) -> NetSpec:
    """MnasNet 1.0 (the depth-multiplier-1 network without squeeze-excite stages): inverted
    residual blocks like MobileNetV2's, with 5x5 depthwise convolutions in three of the six
    stages and plain ReLU.  The expansion channels of every block are pruned; depthwise and
    projection follow the expansion's list."""
    net = NetSpec("mnasnet1_0", 3, in_hw, in_hw, keep_lo=0.4, keep_hi=0.9)
    prev = net.add(Layer("conv", -1, 3, 32, k=3, stride=2, pad=1, act=ACT_RELU, bn=True, name="stem"))
    prev = net.add(Layer("conv", prev, 32, 32, k=3, stride=1, pad=1, groups=32, act=ACT_RELU, bn=True,
                         name="stem.dw"))
    prev = net.add(Layer("conv", prev, 32, 16, k=1, act=ACT_NONE, bn=True, name="stem.project"))
    c = 16
    # (expansion, output channels, blocks, stride of the first block, depthwise kernel)
    table = [(3, 24, 3, 2, 3), (3, 40, 3, 2, 5), (6, 80, 3, 2, 5),
             (6, 96, 2, 1, 3), (6, 192, 4, 2, 5), (6, 320, 1, 1, 3)]
    bidx = 0
    for t, cout, n, s, k in table:
        for i in range(n):
            stride = s if i == 0 else 1
            block_in = prev
            hidden = c * t
            exp = net.add(Layer("conv", prev, c, hidden, k=1, act=ACT_RELU, bn=True, prune_out="own",
                                name=f"b{bidx}.expand"))
            prev = net.add(Layer("conv", exp, hidden, hidden, k=k, stride=stride, pad=k // 2, groups=hidden,
                                 act=ACT_RELU, bn=True, prune_out=exp, name=f"b{bidx}.dw"))
            res = block_in if (stride == 1 and c == cout) else None
            prev = net.add(Layer("conv", prev, hidden, cout, k=1, act=ACT_NONE, bn=True, residual=res,
                                 prune_in=exp, name=f"b{bidx}.project"))
            c = cout
            bidx += 1
    prev = net.add(Layer("conv", prev, c, 1280, k=1, act=ACT_RELU, bn=True, name="last"))
    prev = net.add(Layer("gavgpool", prev, 1280, 1280, name="gap"))
    net.add(Layer("fc", prev, 1280, num_classes, bias=True, name="fc"))
    return net


def single_conv(c_in: int, c_out: int, hw: int, k: int = 3, stride: int = 1,
                pad: int = 1) -> NetSpec:
    """One conv+BN+ReLU layer whose filters are pruned (the single-layer workloads)."""
    net = NetSpec(f"conv{k}x{k}_{c_in}to{c_out}_{hw}", c_in, hw, hw)
    net.add(Layer("conv", -1, c_in, c_out, k=k, stride=stride, pad=pad, act=ACT_RELU,
                  bn=True, prune_out="own", name="conv"))
    return net


def out_hw(layer: Layer, h: int, w: int) -> Tuple[int, int]:
    if layer.kind in ("gavgpool", "fc"):
        return 1, 1
    return ((h + 2 * layer.pad - layer.k) // layer.stride + 1,
            (w + 2 * layer.pad - layer.k) // layer.stride + 1)


def shapes(net: NetSpec, kept: Optional[Dict[int, int]] = None) -> List[Tuple[int, int, int, int]]:
    """Per layer (c_in, c_out, h_out, w_out) with channel counts after pruning.

    ``kept`` maps a pruned layer's index to the number of filters it keeps
    (missing = keeps all)."""
    kept = kept or {}
    res = []
    for i, L in enumerate(net.layers):
        if L.input < 0:
            cin, h, w = net.in_c, net.in_h, net.in_w
        else:
            _, cin, h, w = res[L.input]
        ho, wo = out_hw(L, h, w)
        if L.kind in ("maxpool", "gavgpool"):
            cout = cin
        elif L.prune_out == "own":
            cout = kept.get(i, L.c_out)
        elif isinstance(L.prune_out, int):
            cout = kept.get(L.prune_out, L.c_out)
        else:
            cout = L.c_out
        res.append((cin, cout, ho, wo))
    return res


def count_macs_params(net: NetSpec, kept: Optional[Dict[int, int]] = None) -> Tuple[int, int]:
    """Multiply-adds per image and parameter count (conv + FC weights and FC bias,
    batch-norm excluded: the convention of the paper's Tables 1 and 2)."""
    macs = params = 0
    for L, (cin, cout, ho, wo) in zip(net.layers, shapes(net, kept)):
        if L.kind == "conv":
            g = cin if L.groups != 1 else 1
            per = (cin // g) * L.k * L.k
            macs += cout * per * ho * wo
            params += cout * per
        elif L.kind == "fc":
            macs += cin * cout
            params += cin * cout + (cout if L.bias else 0)
    return macs, params


# --------------------------------------------------------------------------
# parameters
# --------------------------------------------------------------------------

TAG_W, TAG_GAMMA, TAG_BETA, TAG_MEAN, TAG_VAR, TAG_BIAS, TAG_RATIO, TAG_X = range(1, 9)


def keep_count(ratio: float, c: int) -> int:
    """Number of filters kept for a keep ratio: round half up, at least one."""
    return int(min(max(math.floor(ratio * c + 0.5), 1), c))


def layer_params(net: NetSpec, config_id: int, base_seed: int = BASE_SEED) -> List[dict]:
    """Raw (unpruned, unfolded) parameters per layer, fp32 arrays.

    conv: 'w' [c_out][c_in/groups][k][k] He-normal on the unpruned fan-in,
    'gamma'~U(0.5,1.5), 'beta'~N(0,0.1), 'mean'~N(0,0.1), 'var'~U(0.5,1.5);
    fc: 'w' [c_out][c_in] He-normal, 'b'~N(0,0.1); 'keep' for 'own'-pruned layers.
    """
    out = []
    for i, L in enumerate(net.layers):
        p: dict = {}
        key = lambda tag: stream_key(base_seed, config_id, i, tag)
        if L.kind == "conv":
            cpg = L.c_in // L.groups
            fan_in = cpg * L.k * L.k
            n = L.c_out * fan_in
            p["w"] = normal(key(TAG_W), n, 0.0, math.sqrt(2.0 / fan_in)) \
                .astype(np.float32).reshape(L.c_out, cpg, L.k, L.k)
            if L.bn:
                p["gamma"] = uniform(key(TAG_GAMMA), L.c_out, 0.5, 1.5).astype(np.float32)
                p["beta"] = normal(key(TAG_BETA), L.c_out, 0.0, 0.1).astype(np.float32)
                p["mean"] = normal(key(TAG_MEAN), L.c_out, 0.0, 0.1).astype(np.float32)
                p["var"] = uniform(key(TAG_VAR), L.c_out, 0.5, 1.5).astype(np.float32)
        elif L.kind == "fc":
            p["w"] = normal(key(TAG_W), L.c_out * L.c_in, 0.0, math.sqrt(2.0 / L.c_in)) \
                .astype(np.float32).reshape(L.c_out, L.c_in)
            p["b"] = normal(key(TAG_BIAS), L.c_out, 0.0, 0.1).astype(np.float32)
        if L.prune_out == "own":
            r = float(uniform(key(TAG_RATIO), 1, net.keep_lo, net.keep_hi)[0])
            p["keep"] = keep_count(r, L.c_out)
        out.append(p)
    return out


def net_input(net: NetSpec, config_id: int, batch: int, base_seed: int = BASE_SEED) -> np.ndarray:
    n = batch * net.in_c * net.in_h * net.in_w
    return normal(stream_key(base_seed, config_id, 9999, TAG_X), n).astype(np.float32) \
        .reshape(batch, net.in_c, net.in_h, net.in_w)


def tensor_normal(shape, *tags, std: float = 1.0, base_seed: int = BASE_SEED) -> np.ndarray:
    n = int(np.prod(shape))
    return normal(stream_key(base_seed, *tags), n, 0.0, std).astype(np.float32).reshape(shape)


def tensor_uniform(shape, lo, hi, *tags, base_seed: int = BASE_SEED) -> np.ndarray:
    n = int(np.prod(shape))
    return uniform(stream_key(base_seed, *tags), n, lo, hi).astype(np.float32).reshape(shape)


def min_relative_gap(scores: np.ndarray) -> float:
    """Smallest relative distance between adjacent sorted values (a check on inputs:
    a ranking is only reproducible under reordered summation if this is not tiny)."""
    s = np.sort(np.asarray(scores, dtype=np.float64))
    if s.size < 2:
        return float("inf")
    d = np.diff(s)
    return float(np.min(d / np.maximum(np.abs(s[1:]), 1e-300)))
