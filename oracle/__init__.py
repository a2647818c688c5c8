"""CPU oracle (test infrastructure only; the product path never imports this).

Thin numpy/ctypes front for ``cprune_oracle.c`` plus the network-level driver
that applies the per-layer definitions in sequence.  See the C file's header for
the passages of the paper each function follows.
"""

from __future__ import annotations

import ctypes as C
import os
from typing import Dict, List, Optional

import numpy as np

from . import build as _build

_lib = None
_lib_f32acc = None
_timing_build = False


def lib():
    """The C oracle: the parity build (fp64 accumulation) unless timing_build(True) is in force."""
    global _lib, _lib_f32acc
    if _timing_build:
        if _lib_f32acc is None:
            _lib_f32acc = C.CDLL(_build.build_f32acc())
            _lib_f32acc.oracle_conv2d_point.restype = C.c_double
            _lib_f32acc.oracle_rank.restype = C.c_int
        return _lib_f32acc
    if _lib is None:
        _lib = C.CDLL(_build.build())
        _lib.oracle_conv2d_point.restype = C.c_double
        _lib.oracle_rank.restype = C.c_int
    return _lib


def timing_build(on: bool) -> None:
    """Switches every later call to the build whose convolution loops accumulate in float (the
    same loops otherwise).  For timing the CPU baseline only: never on while a reference value
    is computed, and the tests never turn it on except to check that it exists."""
    global _timing_build
    _timing_build = bool(on)


def set_threads(n: int) -> None:
    """Threads used by the convolution loops (OpenMP); 0 leaves the default."""
    if n > 0:
        omp = C.CDLL("libgomp.so.1")
        omp.omp_set_num_threads(int(n))


def num_threads() -> int:
    omp = C.CDLL("libgomp.so.1")
    return int(omp.omp_get_max_threads())


def _f32(a):
    return np.ascontiguousarray(a, dtype=np.float32)


def _i32(a):
    return None if a is None else np.ascontiguousarray(a, dtype=np.int32)


def _p(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


# ---- ranking -------------------------------------------------------------

def l1_scores(w: np.ndarray) -> np.ndarray:
    w = _f32(w)
    c_out = w.shape[0]
    s = np.empty(c_out, dtype=np.float64)
    lib().oracle_l1_scores(_p(w), C.c_int(c_out), C.c_long(w.size // c_out), _p(s))
    return s


def rank(scores: np.ndarray, keep: int):
    """-> (order, kept): order by (score desc, index asc); kept ascending."""
    s = np.ascontiguousarray(scores, dtype=np.float64)
    order = np.empty(s.size, dtype=np.int32)
    kept = np.empty(max(keep, 0), dtype=np.int32)
    rc = lib().oracle_rank(_p(s), C.c_int(s.size), C.c_int(keep), _p(order), _p(kept))
    if rc != 0:
        raise ValueError("keep must be in 1..c_out")
    return order, kept


def rank_filters(w: np.ndarray, keep: int):
    s = l1_scores(w)
    order, kept = rank(s, keep)
    return s, order, kept


def group_scores(ws) -> np.ndarray:
    """Per-channel score of a group of layers with the same number of filters: the sum over
    the layers, in the order given, of each layer's filter L1 norm."""
    total = l1_scores(ws[0])
    for w in ws[1:]:
        if w.shape[0] != ws[0].shape[0]:
            raise ValueError("all layers of a group need the same number of filters")
        total = total + l1_scores(w)
    return total


# ---- gather / fold -------------------------------------------------------

def gather_weights(w: np.ndarray, keep_out=None, keep_in=None) -> np.ndarray:
    w = _f32(w)
    c_out, c_in = w.shape[0], w.shape[1]
    khw = int(np.prod(w.shape[2:])) if w.ndim > 2 else 1
    ko, ki = _i32(keep_out), _i32(keep_in)
    n_out = c_out if ko is None else ko.size
    n_in = c_in if ki is None else ki.size
    out = np.empty((n_out, n_in) + tuple(w.shape[2:]), dtype=np.float32)
    lib().oracle_gather_weights(_p(w), C.c_int(c_out), C.c_int(c_in), C.c_int(khw),
                                _p(ko), C.c_int(n_out), _p(ki), C.c_int(n_in), _p(out))
    return out


def gather_vec(v: np.ndarray, keep) -> np.ndarray:
    v = _f32(v)
    k = _i32(keep)
    n = v.size if k is None else k.size
    out = np.empty(n, dtype=np.float32)
    lib().oracle_gather_vec(_p(v), _p(k), C.c_int(n), _p(out))
    return out


def gather_channels(x: np.ndarray, idx) -> np.ndarray:
    x = _f32(x)
    n, c = x.shape[0], x.shape[1]
    hw = int(np.prod(x.shape[2:])) if x.ndim > 2 else 1
    idx = _i32(idx)
    y = np.empty((n, idx.size) + tuple(x.shape[2:]), dtype=np.float32)
    lib().oracle_gather_channels(_p(x), C.c_int(n), C.c_int(c), C.c_long(hw), _p(idx),
                                 C.c_int(idx.size), _p(y))
    return y


def fold_bn(w, gamma=None, beta=None, mean=None, var=None, eps: float = 1e-5, conv_bias=None):
    w = _f32(w)
    c_out = w.shape[0]
    g = None if gamma is None else _f32(gamma)
    b = None if beta is None else _f32(beta)
    m = None if mean is None else _f32(mean)
    v = None if var is None else _f32(var)
    cb = None if conv_bias is None else _f32(conv_bias)
    w_out = np.empty_like(w)
    bias = np.empty(c_out, dtype=np.float32)
    lib().oracle_fold_bn(_p(w), C.c_int(c_out), C.c_long(w.size // c_out), _p(g), _p(b),
                         _p(m), _p(v), C.c_double(eps), _p(cb), _p(w_out), _p(bias))
    return w_out, bias


# ---- layers --------------------------------------------------------------

def conv2d_f64(x, w, stride=1, pad=0, groups=1) -> np.ndarray:
    x, w = _f32(x), _f32(w)
    n, c_in, h, wd = x.shape
    c_out, cpg, kh, kw = w.shape
    assert cpg * groups == c_in and c_out % groups == 0
    ho = (h + 2 * pad - kh) // stride + 1
    wo = (wd + 2 * pad - kw) // stride + 1
    z = np.empty((n, c_out, ho, wo), dtype=np.float64)
    lib().oracle_conv2d_f64(_p(x), _p(w), C.c_int(n), C.c_int(c_in), C.c_int(h), C.c_int(wd),
                            C.c_int(c_out), C.c_int(kh), C.c_int(kw), C.c_int(stride),
                            C.c_int(pad), C.c_int(groups), _p(z))
    return z


def conv2d_point(x, w, b, o, y, xo, stride=1, pad=0, groups=1) -> float:
    """One pre-bias output element z[b][o][y][xo] of conv2d_f64 (x, w must be fp32
    contiguous arrays; not copied)."""
    assert x.dtype == np.float32 and w.dtype == np.float32
    assert x.flags.c_contiguous and w.flags.c_contiguous
    _, c_in, h, wd = x.shape
    c_out, _, kh, kw = w.shape
    return float(lib().oracle_conv2d_point(
        _p(x), _p(w), C.c_int(c_in), C.c_int(h), C.c_int(wd), C.c_int(c_out), C.c_int(kh),
        C.c_int(kw), C.c_int(stride), C.c_int(pad), C.c_int(groups),
        C.c_int(b), C.c_int(o), C.c_int(y), C.c_int(xo)))


def bias_act(z, bias=None, residual=None, act=0) -> np.ndarray:
    z = np.ascontiguousarray(z, dtype=np.float64)
    n, c = z.shape[0], z.shape[1]
    hw = int(np.prod(z.shape[2:])) if z.ndim > 2 else 1
    bias = None if bias is None else _f32(bias)
    residual = None if residual is None else _f32(residual)
    y = np.empty(z.shape, dtype=np.float32)
    lib().oracle_bias_act(_p(z), C.c_int(n), C.c_int(c), C.c_long(hw), _p(bias), _p(residual),
                          C.c_int(act), _p(y))
    return y


def bn_act(z, gamma, beta, mean, var, eps=1e-5, conv_bias=None, residual=None, act=0):
    z = np.ascontiguousarray(z, dtype=np.float64)
    n, c = z.shape[0], z.shape[1]
    hw = int(np.prod(z.shape[2:])) if z.ndim > 2 else 1
    gamma, beta, mean, var = _f32(gamma), _f32(beta), _f32(mean), _f32(var)
    conv_bias = None if conv_bias is None else _f32(conv_bias)
    residual = None if residual is None else _f32(residual)
    y = np.empty(z.shape, dtype=np.float32)
    lib().oracle_bn_act(_p(z), C.c_int(n), C.c_int(c), C.c_long(hw), _p(gamma), _p(beta),
                        _p(mean), _p(var), C.c_double(eps), _p(conv_bias), _p(residual),
                        C.c_int(act), _p(y))
    return y


def conv2d_bias_act(x, w_folded, bias, stride=1, pad=0, groups=1, act=0, residual=None):
    """Folded form: act(conv(x, w'') + b (+ residual))."""
    return bias_act(conv2d_f64(x, w_folded, stride, pad, groups), bias, residual, act)


def conv2d_bn_act(x, w, gamma, beta, mean, var, eps=1e-5, stride=1, pad=0, groups=1, act=0,
                  residual=None, conv_bias=None):
    """Unfolded form: act(BN(conv(x, w)) (+ residual))."""
    return bn_act(conv2d_f64(x, w, stride, pad, groups), gamma, beta, mean, var, eps,
                  conv_bias, residual, act)


def maxpool(x, k, stride, pad=0) -> np.ndarray:
    x = _f32(x)
    n, c, h, w = x.shape
    ho = (h + 2 * pad - k) // stride + 1
    wo = (w + 2 * pad - k) // stride + 1
    y = np.empty((n, c, ho, wo), dtype=np.float32)
    lib().oracle_maxpool(_p(x), C.c_int(n), C.c_int(c), C.c_int(h), C.c_int(w), C.c_int(k),
                         C.c_int(stride), C.c_int(pad), _p(y))
    return y


def gavgpool(x) -> np.ndarray:
    x = _f32(x)
    n, c = x.shape[0], x.shape[1]
    hw = int(np.prod(x.shape[2:]))
    y = np.empty((n, c, 1, 1), dtype=np.float32)
    lib().oracle_gavgpool(_p(x), C.c_int(n), C.c_int(c), C.c_long(hw), _p(y))
    return y


def fc(x, w, bias=None, act=0) -> np.ndarray:
    x, w = _f32(x), _f32(w)
    n = x.shape[0]
    x2 = x.reshape(n, -1)
    c_out, f = w.shape
    assert x2.shape[1] == f
    bias = None if bias is None else _f32(bias)
    y = np.empty((n, c_out), dtype=np.float32)
    lib().oracle_fc(_p(x2), _p(w), _p(bias), C.c_int(n), C.c_int(f), C.c_int(c_out),
                    C.c_int(act), _p(y))
    return y


# ---- network level -------------------------------------------------------

BN_EPS = float(np.float32(1e-5))  # the value as it crosses a float-typed boundary


def prune_net(net, params: List[dict], keep_override: Optional[Dict[int, int]] = None,
              fold: bool = True):
    """Rank, prune and (optionally) fold every layer of a network.

    Section 3.5: each 'own'-pruned layer's filters are ranked on their raw
    weights and the lowest-scoring removed; layers fed by a pruned layer lose the
    matching input channels.  Returns (layers, kept): per layer a dict with the
    pruned 'w' and either folded 'b' or the gathered BN vectors; kept maps layer
    index -> ascending kept-filter indices.
    """
    kept: Dict[int, np.ndarray] = {}
    for i, (L, p) in enumerate(zip(net.layers, params)):
        if L.prune_out == "own":
            k = (keep_override or {}).get(i, p["keep"])
            if getattr(L, "score_with", None):
                # layers whose outputs a shortcut adds lose the same channels (Section 3.5, last
                # paragraph).  Reading: a channel's score is the sum of its filter norms over
                # those layers, added in layer order; the paper only names the mode of the
                # pruning toolkit it uses.
                _, kept[i] = rank(group_scores([p["w"]] + [params[j]["w"] for j in L.score_with]), k)
            else:
                _, _, kept[i] = rank_filters(p["w"], k)
    out = []
    for i, (L, p) in enumerate(zip(net.layers, params)):
        q: dict = {}
        if L.kind == "conv":
            ko = kept.get(i) if L.prune_out == "own" else (
                kept.get(L.prune_out) if isinstance(L.prune_out, int) else None)
            ki = kept.get(L.prune_in) if (L.prune_in is not None and L.groups == 1) else None
            w = gather_weights(p["w"], ko, ki)
            bn = {t: gather_vec(p[t], ko) for t in ("gamma", "beta", "mean", "var")} \
                if L.bn else None
            if fold:
                if bn:
                    q["w"], q["b"] = fold_bn(w, bn["gamma"], bn["beta"], bn["mean"], bn["var"],
                                             BN_EPS)
                else:
                    q["w"], q["b"] = fold_bn(w)
            else:
                q["w"], q["bn"] = w, bn
        elif L.kind == "fc":
            ki = kept.get(L.prune_in) if L.prune_in is not None else None
            q["w"] = gather_weights(p["w"], None, ki)
            q["b"] = p["b"].copy()
        out.append(q)
    return out, kept


def forward(net, layers: List[dict], x: np.ndarray, return_all: bool = False):
    """Run the layer list on x; layers from prune_net (folded or unfolded)."""
    acts: List[np.ndarray] = []
    for L, q in zip(net.layers, layers):
        src = x if L.input < 0 else acts[L.input]
        res = None if L.residual is None else acts[L.residual]
        if L.kind == "conv":
            groups = 1 if L.groups == 1 else src.shape[1]
            if "b" in q:
                y = conv2d_bias_act(src, q["w"], q["b"], L.stride, L.pad, groups, L.act, res)
            else:
                bn = q["bn"]
                y = conv2d_bn_act(src, q["w"], bn["gamma"], bn["beta"], bn["mean"], bn["var"],
                                  BN_EPS, L.stride, L.pad, groups, L.act, res)
        elif L.kind == "maxpool":
            y = maxpool(src, L.k, L.stride, L.pad)
        elif L.kind == "gavgpool":
            y = gavgpool(src)
        elif L.kind == "fc":
            y = fc(src, q["w"], q["b"], L.act)
        else:
            raise ValueError(L.kind)
        acts.append(y)
    return acts if return_all else acts[-1]
