"""ctypes binding of libcprune_hip.so: same names as the C ABI, argument
marshalling only.  Tensors are torch CUDA tensors (device memory and streams are
PyTorch's); every step of the path runs in the library's kernels.  There is no
fallback: a missing library raises.
"""

from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Tuple

import torch

from . import build as _build

F32, F16, BF16 = 0, 1, 2
ACT_NONE, ACT_RELU, ACT_RELU6 = 0, 1, 2
LAYER_CONV, LAYER_MAXPOOL, LAYER_GAVGPOOL, LAYER_FC = 0, 1, 2, 3

OK = 0
ERR_INVALID_ARG, ERR_UNSUPPORTED, ERR_WORKSPACE, ERR_DEVICE, ERR_NOT_TUNED = -1, -2, -3, -4, -5

TORCH_DTYPE = {F32: torch.float32, F16: torch.float16, BF16: torch.bfloat16}
DTYPE_OF_TORCH = {v: k for k, v in TORCH_DTYPE.items()}


class ConvDesc(C.Structure):
    _fields_ = [(n, C.c_int32) for n in
                ("n", "c_in", "h", "w", "c_out", "kh", "kw", "stride", "pad", "groups", "dtype",
                 "act", "has_residual")]


class LayerDesc(C.Structure):
    _fields_ = [(n, C.c_int32) for n in
                ("kind", "input", "residual", "c_in", "c_out", "k", "stride", "pad", "groups",
                 "act")] + [("weight", C.c_void_p), ("bias", C.c_void_p)]


class PruneLayer(C.Structure):
    _fields_ = [("w", C.c_void_p)] + [(n, C.c_int32) for n in
                                      ("c_out", "c_in", "kh", "kw", "keep", "rows_from", "cols_from")] + \
               [("score_with", C.POINTER(C.c_int32)), ("n_score_with", C.c_int32)] + \
               [(n, C.c_void_p) for n in ("gamma", "beta", "mean", "var", "conv_bias", "w_out", "bias_out",
                                          "kept_out")]


EXPORTS = [
    "cprune_status_string", "cprune_last_hip_error",
    "cprune_rank_filters_workspace_bytes", "cprune_rank_filters", "cprune_rank_filter_group",
    "cprune_rank_filters_static", "cprune_rank_filters_static_max",
    "cprune_prune_plan_create", "cprune_prune_plan_run", "cprune_prune_plan_traffic",
    "cprune_prune_plan_destroy",
    "cprune_gather_pruned_weights", "cprune_gather_channels",
    "cprune_num_tile_variants", "cprune_tile_variant_info", "cprune_tile_variant_name",
    "cprune_conv_workspace_bytes",
    "cprune_conv2d_bn_relu", "cprune_select_tile", "cprune_clear_tile_cache",
    "cprune_cached_tile", "cprune_maxpool2d", "cprune_global_avgpool",
    "cprune_fc_workspace_bytes", "cprune_fc",
    "cprune_net_create", "cprune_net_forward", "cprune_net_layer_times",
    "cprune_net_copy_activation", "cprune_net_output_shape", "cprune_net_layer_variant",
    "cprune_net_set_layer_variant", "cprune_net_fuse_depthwise", "cprune_net_fuse_block",
    "cprune_net_fuse_first_layers", "cprune_net_first_layer_form", "cprune_net_layer_fused",
    "cprune_net_destroy",
    "cprune_probe_scratch_bytes", "cprune_probe_mfma", "cprune_probe_copy", "cprune_probe_read",
    "cprune_probe_write",
    "cprune_probe_l2_bytes", "cprune_probe_l2_read",
    "cprune_lcm_step", "cprune_prune_count", "cprune_variant_filter_splits",
    "cprune_variant_prune_step", "cprune_order_tasks", "cprune_net_task_table", "cprune_net_task_key",
    "cprune_search_create", "cprune_search_start", "cprune_search_next_task",
    "cprune_search_report_exhausted", "cprune_search_report_latency", "cprune_search_report_accuracy",
    "cprune_search_log_size", "cprune_search_log_entry", "cprune_search_destroy",
]

_lib = None


class CPruneError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        msg = lib().cprune_status_string(status).decode()
        if status == ERR_DEVICE:
            msg += f" (hipError {lib().cprune_last_hip_error()})"
        super().__init__(f"{where}: {msg} [{status}]")


def lib():
    """The loaded shared library; built on first use if it is not there yet."""
    global _lib
    if _lib is None:
        path = _build.library_path()
        if not os.path.exists(path):
            _build.build()
        L = C.CDLL(path)
        L.cprune_status_string.restype = C.c_char_p
        L.cprune_status_string.argtypes = [C.c_int]
        for name in ("cprune_rank_filters_workspace_bytes", "cprune_conv_workspace_bytes",
                     "cprune_fc_workspace_bytes", "cprune_probe_scratch_bytes", "cprune_probe_l2_bytes"):
            getattr(L, name).restype = C.c_size_t
        L.cprune_clear_tile_cache.restype = None
        _lib = L
    return _lib


def _check(status: int, where: str) -> None:
    if status != OK:
        raise CPruneError(status, where)


def _ptr(t: Optional[torch.Tensor]):
    if t is None:
        return C.c_void_p(None)
    assert t.is_cuda and t.is_contiguous(), "device-resident contiguous tensors only"
    return C.c_void_p(t.data_ptr())


def _stream(stream=None):
    s = stream if stream is not None else torch.cuda.current_stream()
    return C.c_void_p(s.cuda_stream)


def _ws(nbytes: int, device) -> Optional[torch.Tensor]:
    return torch.empty(max(int(nbytes), 16), dtype=torch.uint8, device=device)


# ---- ranking / gather ------------------------------------------------------

def cprune_rank_filters(w: torch.Tensor, keep: int, want_scores=True, want_order=True,
                        stream=None):
    """-> (scores fp64 or None, order int32 or None, kept int32 ascending)."""
    assert w.dtype == torch.float32 and w.dim() == 4
    c_out, cpg, kh, kw = w.shape
    dev = w.device
    scores = torch.empty(c_out, dtype=torch.float64, device=dev) if want_scores else None
    order = torch.empty(c_out, dtype=torch.int32, device=dev) if want_order else None
    kept = torch.empty(max(keep, 1), dtype=torch.int32, device=dev)
    nws = lib().cprune_rank_filters_workspace_bytes(C.c_int(c_out))
    ws = _ws(nws, dev)
    st = lib().cprune_rank_filters(_ptr(w), C.c_int(c_out), C.c_int(cpg), C.c_int(kh), C.c_int(kw),
                                   C.c_int(keep), _ptr(scores), _ptr(order), _ptr(kept), _ptr(ws),
                                   C.c_size_t(ws.numel()), _stream(stream))
    _check(st, "cprune_rank_filters")
    return scores, order, kept


def cprune_rank_filters_static_max() -> int:
    return int(lib().cprune_rank_filters_static_max())


def cprune_rank_filters_static(w: torch.Tensor, keep: int, order: Optional[torch.Tensor],
                               kept: torch.Tensor, stream=None) -> None:
    """The ranking call that allocates nothing: the caller passes the outputs (order int32 [c_out] or
    None, kept int32 [keep]); the scores live in the library's per-device static array."""
    assert w.dtype == torch.float32 and w.dim() == 4
    c_out, cpg, kh, kw = w.shape
    st = lib().cprune_rank_filters_static(_ptr(w), C.c_int(c_out), C.c_int(cpg), C.c_int(kh), C.c_int(kw),
                                          C.c_int(keep), _ptr(order), _ptr(kept), _stream(stream))
    _check(st, "cprune_rank_filters_static")


class PrunePlan:
    """Owner of a cprune_prune_plan: the ranking and gather of a whole network in three launches.
    `entries`: one dict per layer in network order, None for layers without weights; keys w (fp32
    device tensor, 4-d), keep (0 = not ranked), rows_from, cols_from (-1 = all), score_with (list),
    bn (gamma, beta, mean, var) or None, conv_bias or None.  Outputs are allocated here once:
    .w_out[i], .bias_out[i], .kept[i] (ranked layers)."""

    def __init__(self, entries, eps: float, out_dtype: int = F32):
        n = len(entries)
        arr = (PruneLayer * n)()
        self.w_out, self.bias_out, self.kept = {}, {}, {}
        self._keep_alive = []
        dev = None
        keep_of = {i: int(e["keep"]) for i, e in enumerate(entries) if e is not None and e.get("keep", 0) > 0}
        for i, e in enumerate(entries):
            a = arr[i]
            a.rows_from = a.cols_from = -1
            if e is None:
                continue
            w = e["w"]
            assert w.dtype == torch.float32 and w.dim() == 4 and w.is_cuda and w.is_contiguous()
            dev = w.device
            c_out, c_in, kh, kw = w.shape
            a.w = w.data_ptr()
            a.c_out, a.c_in, a.kh, a.kw = c_out, c_in, kh, kw
            a.keep = int(e.get("keep", 0))
            a.rows_from = int(e.get("rows_from", -1))
            a.cols_from = int(e.get("cols_from", -1))
            sw = list(e.get("score_with") or [])
            if sw:
                lst = (C.c_int32 * len(sw))(*sw)
                self._keep_alive.append(lst)
                a.score_with = C.cast(lst, C.POINTER(C.c_int32))
            a.n_score_with = len(sw)
            bn = e.get("bn")
            if bn is not None:
                a.gamma, a.beta, a.mean, a.var = (t.data_ptr() for t in bn)
            cb = e.get("conv_bias")
            if cb is not None:
                a.conv_bias = cb.data_ptr()
            n_out = keep_of.get(a.rows_from, c_out) if a.rows_from >= 0 else c_out
            n_in = keep_of.get(a.cols_from, c_in) if a.cols_from >= 0 else c_in
            self.w_out[i] = torch.empty((n_out, n_in, kh, kw), dtype=TORCH_DTYPE[out_dtype], device=dev)
            a.w_out = self.w_out[i].data_ptr()
            if bn is not None or cb is not None:
                self.bias_out[i] = torch.empty(n_out, dtype=torch.float32, device=dev)
                a.bias_out = self.bias_out[i].data_ptr()
            if a.keep > 0:
                self.kept[i] = torch.empty(a.keep, dtype=torch.int32, device=dev)
                a.kept_out = self.kept[i].data_ptr()
            self._keep_alive.append((w, bn, cb))
        self._h = C.c_void_p(None)
        st = lib().cprune_prune_plan_create(arr, C.c_int(n), C.c_float(eps), C.c_int(out_dtype), C.byref(self._h))
        _check(st, "cprune_prune_plan_create")

    def run(self, stream=None) -> None:
        _check(lib().cprune_prune_plan_run(self._h, _stream(stream)), "cprune_prune_plan_run")

    def traffic(self):
        """-> (weight elements read, weight elements written) per run."""
        r, w = C.c_int64(0), C.c_int64(0)
        _check(lib().cprune_prune_plan_traffic(self._h, C.byref(r), C.byref(w)), "cprune_prune_plan_traffic")
        return int(r.value), int(w.value)

    def close(self):
        if self._h:
            lib().cprune_prune_plan_destroy(self._h)
            self._h = C.c_void_p(None)

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def cprune_rank_filter_group(ws_list, keep: int, want_scores=True, want_order=True, stream=None):
    """Layers that must lose the same channels, ranked on the sum of their filter norms.
    ws_list: fp32 device weight tensors with the same number of filters.
    -> (scores fp64 or None, order int32 or None, kept int32 ascending)."""
    c_out = ws_list[0].shape[0]
    assert all(w.dtype == torch.float32 and w.shape[0] == c_out for w in ws_list)
    dev = ws_list[0].device
    n = len(ws_list)
    ptrs = (C.c_void_p * n)(*[w.data_ptr() for w in ws_list])
    lens = (C.c_int64 * n)(*[w.numel() // c_out for w in ws_list])
    for w in ws_list:
        assert w.is_cuda and w.is_contiguous()
    scores = torch.empty(c_out, dtype=torch.float64, device=dev) if want_scores else None
    order = torch.empty(c_out, dtype=torch.int32, device=dev) if want_order else None
    kept = torch.empty(max(keep, 1), dtype=torch.int32, device=dev)
    ws = _ws(lib().cprune_rank_filters_workspace_bytes(C.c_int(c_out)), dev)
    st = lib().cprune_rank_filter_group(ptrs, lens, C.c_int(n), C.c_int(c_out), C.c_int(keep), _ptr(scores),
                                        _ptr(order), _ptr(kept), _ptr(ws), C.c_size_t(ws.numel()),
                                        _stream(stream))
    _check(st, "cprune_rank_filter_group")
    return scores, order, kept


def cprune_gather_pruned_weights(w: torch.Tensor, keep_out=None, keep_in=None, bn=None,
                                 eps: float = 1e-5, conv_bias=None, out_dtype: int = F32,
                                 stream=None) -> Tuple[torch.Tensor, Optional[torch.Tensor]]:
    """bn = (gamma, beta, mean, var) device fp32 vectors over the unpruned filters, or None.
    -> (w_out [n_out][n_in][kh][kw] in out_dtype, bias_out fp32 [n_out] or None)."""
    assert w.dtype == torch.float32 and w.dim() == 4
    c_out, c_in, kh, kw = w.shape
    n_out = c_out if keep_out is None else keep_out.numel()
    n_in = c_in if keep_in is None else keep_in.numel()
    w_out = torch.empty((n_out, n_in, kh, kw), dtype=TORCH_DTYPE[out_dtype], device=w.device)
    need_bias = bn is not None or conv_bias is not None
    bias_out = torch.empty(n_out, dtype=torch.float32, device=w.device) if need_bias else None
    g, b, m, v = bn if bn is not None else (None, None, None, None)
    st = lib().cprune_gather_pruned_weights(
        _ptr(w), C.c_int(c_out), C.c_int(c_in), C.c_int(kh), C.c_int(kw),
        _ptr(keep_out), C.c_int(n_out), _ptr(keep_in), C.c_int(n_in),
        _ptr(g), _ptr(b), _ptr(m), _ptr(v), C.c_float(eps), _ptr(conv_bias),
        C.c_int(out_dtype), _ptr(w_out), _ptr(bias_out), _stream(stream))
    _check(st, "cprune_gather_pruned_weights")
    return w_out, bias_out


def cprune_gather_channels(x: torch.Tensor, idx: torch.Tensor, stream=None) -> torch.Tensor:
    n, c, h, w = x.shape
    y = torch.empty((n, idx.numel(), h, w), dtype=x.dtype, device=x.device)
    st = lib().cprune_gather_channels(_ptr(x), C.c_int(n), C.c_int(c), C.c_int(h), C.c_int(w),
                                      C.c_int(DTYPE_OF_TORCH[x.dtype]), _ptr(idx),
                                      C.c_int(idx.numel()), _ptr(y), _stream(stream))
    _check(st, "cprune_gather_channels")
    return y


# ---- convolution -------------------------------------------------------------

def conv_desc(x_shape, w_shape, stride=1, pad=0, groups=1, dtype=F32, act=ACT_RELU,
              has_residual=False) -> ConvDesc:
    n, c_in, h, w = x_shape
    c_out, _, kh, kw = w_shape
    return ConvDesc(n, c_in, h, w, c_out, kh, kw, stride, pad, groups, dtype, act,
                    1 if has_residual else 0)


def out_shape(d: ConvDesc):
    ho = (d.h + 2 * d.pad - d.kh) // d.stride + 1
    wo = (d.w + 2 * d.pad - d.kw) // d.stride + 1
    return (d.n, d.c_out, ho, wo)


def cprune_num_tile_variants() -> int:
    return int(lib().cprune_num_tile_variants())


def cprune_tile_variant_name(v: int, channels_last: bool = True, dtype: int = F32) -> str:
    buf = C.create_string_buffer(128)
    _check(lib().cprune_tile_variant_name(C.c_int(v), C.c_int(1 if channels_last else 0), C.c_int(dtype), buf,
                                          C.c_size_t(128)), "cprune_tile_variant_name")
    return buf.value.decode()


def cprune_tile_variant_info(v: int) -> Tuple[int, int, int]:
    tm, tp, sk = C.c_int(), C.c_int(), C.c_int()
    _check(lib().cprune_tile_variant_info(C.c_int(v), C.byref(tm), C.byref(tp), C.byref(sk)),
           "cprune_tile_variant_info")
    return tm.value, tp.value, sk.value


def cprune_conv_workspace_bytes(d: ConvDesc, variant: int = -1) -> int:
    return int(lib().cprune_conv_workspace_bytes(C.byref(d), C.c_int(variant)))


def cprune_conv2d_bn_relu(d: ConvDesc, x, w, bias=None, residual=None, tile_variant: int = -1,
                          ws: Optional[torch.Tensor] = None, y: Optional[torch.Tensor] = None,
                          stream=None) -> torch.Tensor:
    if y is None:
        y = torch.empty(out_shape(d), dtype=TORCH_DTYPE[d.dtype], device=x.device)
    if ws is None:
        ws = _ws(cprune_conv_workspace_bytes(d, tile_variant), x.device)
    st = lib().cprune_conv2d_bn_relu(C.byref(d), _ptr(x), _ptr(w), _ptr(bias), _ptr(residual),
                                     _ptr(y), C.c_int(tile_variant), _ptr(ws),
                                     C.c_size_t(ws.numel()), _stream(stream))
    _check(st, "cprune_conv2d_bn_relu")
    return y


def cprune_select_tile(d: ConvDesc, x, w, bias=None, residual=None, warmup: int = 2,
                       iters: int = 8, stream=None):
    """-> (variant, best_ms, all_ms list)."""
    y = torch.empty(out_shape(d), dtype=TORCH_DTYPE[d.dtype], device=x.device)
    ws = _ws(cprune_conv_workspace_bytes(d, -1), x.device)
    nv = cprune_num_tile_variants()
    all_ms = (C.c_float * nv)()
    v, best = C.c_int(-1), C.c_float(0)
    st = lib().cprune_select_tile(C.byref(d), _ptr(x), _ptr(w), _ptr(bias), _ptr(residual), _ptr(y),
                                  _ptr(ws), C.c_size_t(ws.numel()), C.c_int(warmup), C.c_int(iters),
                                  C.byref(v), C.byref(best), all_ms, _stream(stream))
    _check(st, "cprune_select_tile")
    return v.value, best.value, list(all_ms)


def cprune_clear_tile_cache() -> None:
    lib().cprune_clear_tile_cache()


def cprune_cached_tile(d: ConvDesc) -> Tuple[int, bool]:
    v, timed = C.c_int(), C.c_int()
    _check(lib().cprune_cached_tile(C.byref(d), C.byref(v), C.byref(timed)), "cprune_cached_tile")
    return v.value, bool(timed.value)


# ---- other layers --------------------------------------------------------------

def cprune_maxpool2d(x, k, stride, pad=0, stream=None):
    n, c, h, w = x.shape
    ho, wo = (h + 2 * pad - k) // stride + 1, (w + 2 * pad - k) // stride + 1
    y = torch.empty((n, c, ho, wo), dtype=x.dtype, device=x.device)
    st = lib().cprune_maxpool2d(_ptr(x), C.c_int(n), C.c_int(c), C.c_int(h), C.c_int(w), C.c_int(k),
                                C.c_int(stride), C.c_int(pad), C.c_int(DTYPE_OF_TORCH[x.dtype]),
                                _ptr(y), _stream(stream))
    _check(st, "cprune_maxpool2d")
    return y


def cprune_global_avgpool(x, stream=None):
    n, c, h, w = x.shape
    y = torch.empty((n, c), dtype=x.dtype, device=x.device)
    st = lib().cprune_global_avgpool(_ptr(x), C.c_int(n), C.c_int(c), C.c_int(h), C.c_int(w),
                                     C.c_int(DTYPE_OF_TORCH[x.dtype]), _ptr(y), _stream(stream))
    _check(st, "cprune_global_avgpool")
    return y


def cprune_fc(x, w, bias=None, act=ACT_NONE, stream=None):
    n = x.shape[0]
    f = x.numel() // n
    c_out = w.shape[0]
    dt = DTYPE_OF_TORCH[x.dtype]
    y = torch.empty((n, c_out), dtype=x.dtype, device=x.device)
    ws = _ws(lib().cprune_fc_workspace_bytes(C.c_int(n), C.c_int(f), C.c_int(c_out), C.c_int(dt)),
             x.device)
    st = lib().cprune_fc(_ptr(x), _ptr(w), _ptr(bias), C.c_int(n), C.c_int(f), C.c_int(c_out),
                         C.c_int(act), C.c_int(dt), _ptr(y), _ptr(ws), C.c_size_t(ws.numel()),
                         _stream(stream))
    _check(st, "cprune_fc")
    return y


# ---- search-side rules (host only) ----------------------------------------------

def cprune_lcm_step(l1, l2) -> int:
    a = (C.c_int64 * len(l1))(*l1)
    b = (C.c_int64 * len(l2))(*l2)
    out = C.c_int64(0)
    _check(lib().cprune_lcm_step(a, C.c_int(len(l1)), b, C.c_int(len(l2)), C.byref(out)), "cprune_lcm_step")
    return int(out.value)


def cprune_prune_count(c_out: int, step: int) -> int:
    out = C.c_int(0)
    _check(lib().cprune_prune_count(C.c_int(c_out), C.c_int64(step), C.byref(out)), "cprune_prune_count")
    return int(out.value)


def cprune_variant_filter_splits(variant: int, c_out: int):
    """-> (main-loop split, epilogue split, filters per unit)."""
    ml, ep, unit = (C.c_int64 * 2)(), (C.c_int64 * 2)(), C.c_int(0)
    _check(lib().cprune_variant_filter_splits(C.c_int(variant), C.c_int(c_out), ml, ep, C.byref(unit)),
           "cprune_variant_filter_splits")
    return list(ml), list(ep), int(unit.value)


def cprune_variant_prune_step(variant: int, c_out: int) -> int:
    out = C.c_int64(0)
    _check(lib().cprune_variant_prune_step(C.c_int(variant), C.c_int(c_out), C.byref(out)),
           "cprune_variant_prune_step")
    return int(out.value)


def cprune_order_tasks(exec_time, n_subgraphs):
    """-> (task indices by descending pruning impact, impacts)."""
    n = len(exec_time)
    t = (C.c_double * n)(*[float(v) for v in exec_time])
    c = (C.c_int * n)(*[int(v) for v in n_subgraphs])
    order, impact = (C.c_int * n)(), (C.c_double * n)()
    _check(lib().cprune_order_tasks(t, c, C.c_int(n), order, impact), "cprune_order_tasks")
    return list(order), list(impact)


class Search:
    """Owner of a cprune_search object (the decisions of Algorithm 1); tasks are integers here."""

    def __init__(self, a_goal: float, alpha: float, beta: float, max_passes: int):
        self._h = C.c_void_p(None)
        _check(lib().cprune_search_create(C.c_double(a_goal), C.c_double(alpha), C.c_double(beta),
                                          C.c_int64(min(int(max_passes), (1 << 62))), C.byref(self._h)),
               "cprune_search_create")

    @staticmethod
    def _ids(tasks):
        return (C.c_int64 * max(len(tasks), 1))(*tasks), C.c_int(len(tasks))

    def start(self, tasks_by_impact, l_m: float, a_p: float) -> None:
        arr, n = self._ids(tasks_by_impact)
        _check(lib().cprune_search_start(self._h, arr, n, C.c_double(l_m), C.c_double(a_p)), "cprune_search_start")

    def next_task(self) -> Optional[int]:
        """The task to prune next, or None when the search is over."""
        task, done = C.c_int64(0), C.c_int(0)
        _check(lib().cprune_search_next_task(self._h, C.byref(task), C.byref(done)), "cprune_search_next_task")
        return None if done.value else int(task.value)

    def report_exhausted(self) -> None:
        _check(lib().cprune_search_report_exhausted(self._h), "cprune_search_report_exhausted")

    def report_latency(self, l_m: float) -> bool:
        """-> True when the candidate passed the latency gate and its accuracy is wanted."""
        need = C.c_int(0)
        _check(lib().cprune_search_report_latency(self._h, C.c_double(l_m), C.byref(need)),
               "cprune_search_report_latency")
        return bool(need.value)

    def report_accuracy(self, a_s: float, tasks_by_impact) -> bool:
        """-> True when the candidate was accepted."""
        arr, n = self._ids(tasks_by_impact)
        acc = C.c_int(0)
        _check(lib().cprune_search_report_accuracy(self._h, C.c_double(a_s), arr, n, C.byref(acc)),
               "cprune_search_report_accuracy")
        return bool(acc.value)

    def log(self):
        """-> [(task, l_m or None, l_t, a_s or None, verdict code)]"""
        out = []
        for i in range(int(lib().cprune_search_log_size(self._h))):
            t, v = C.c_int64(0), C.c_int(0)
            l_m, l_t, a_s = C.c_double(0), C.c_double(0), C.c_double(0)
            _check(lib().cprune_search_log_entry(self._h, C.c_int(i), C.byref(t), C.byref(l_m), C.byref(l_t),
                                                 C.byref(a_s), C.byref(v)), "cprune_search_log_entry")
            nn = lambda x: None if x != x else x
            out.append((int(t.value), nn(l_m.value), l_t.value, nn(a_s.value), int(v.value)))
        return out

    def close(self):
        if self._h:
            lib().cprune_search_destroy(self._h)
            self._h = C.c_void_p(None)

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


# ---- measured ceilings ---------------------------------------------------------

def cprune_probe_mfma(dtype: int = F32, stream=None) -> float:
    """TFLOP/s of back-to-back MFMA instructions of `dtype` on register operands."""
    ws = _ws(lib().cprune_probe_scratch_bytes(), "cuda")
    out = C.c_float(0.0)
    st = lib().cprune_probe_mfma(C.c_int(dtype), _ptr(ws), C.c_size_t(ws.numel()), C.byref(out),
                                 _stream(stream))
    _check(st, "cprune_probe_mfma")
    return float(out.value)


def cprune_probe_copy(nbytes: int = 1 << 30, stream=None) -> float:
    """GB/s (read + written) of a plain device copy of `nbytes`."""
    src = torch.zeros(nbytes, dtype=torch.uint8, device="cuda")
    dst = torch.empty_like(src)
    out = C.c_float(0.0)
    st = lib().cprune_probe_copy(_ptr(src), _ptr(dst), C.c_size_t(nbytes), C.byref(out), _stream(stream))
    _check(st, "cprune_probe_copy")
    return float(out.value)


def cprune_probe_read(nbytes: int = 1 << 30, stream=None) -> float:
    """GB/s of a kernel that only reads `nbytes` of device memory."""
    src = torch.zeros(nbytes, dtype=torch.uint8, device="cuda")
    scratch = torch.zeros(16, dtype=torch.uint8, device="cuda")
    out = C.c_float(0.0)
    st = lib().cprune_probe_read(_ptr(src), _ptr(scratch), C.c_size_t(nbytes), C.byref(out), _stream(stream))
    _check(st, "cprune_probe_read")
    return float(out.value)


def cprune_probe_write(nbytes: int = 1 << 30, stream=None) -> float:
    """GB/s of a kernel that only writes `nbytes` of device memory."""
    dst = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    out = C.c_float(0.0)
    st = lib().cprune_probe_write(_ptr(dst), C.c_size_t(nbytes), C.byref(out), _stream(stream))
    _check(st, "cprune_probe_write")
    return float(out.value)


def cprune_probe_l2_read(pattern: int, stream=None) -> float:
    """GB/s one compute unit reads from L2-resident data with 16-byte-per-lane loads; pattern 0: 1 KiB of
    consecutive memory per wavefront-wide load, 1: 16 rows x 64 bytes."""
    buf = torch.zeros(lib().cprune_probe_l2_bytes(), dtype=torch.uint8, device="cuda")
    scratch = torch.zeros(1, dtype=torch.float32, device="cuda")
    out = C.c_float(0.0)
    st = lib().cprune_probe_l2_read(C.c_int(pattern), _ptr(buf), C.c_size_t(buf.numel()), _ptr(scratch),
                                    C.byref(out), _stream(stream))
    _check(st, "cprune_probe_l2_read")
    return float(out.value)


# ---- network handle ------------------------------------------------------------

class Net:
    """Owner of a cprune_net handle."""

    def __init__(self, layer_descs, in_chw, max_batch: int, dtype: int = F32, tune: bool = True,
                 stream=None):
        arr = (LayerDesc * len(layer_descs))(*layer_descs)
        self._h = C.c_void_p(None)
        self._graph_logits = {}
        self.n_layers = len(layer_descs)
        self.dtype = dtype
        self.max_batch = max_batch
        st = lib().cprune_net_create(arr, C.c_int(len(layer_descs)), C.c_int(in_chw[0]),
                                     C.c_int(in_chw[1]), C.c_int(in_chw[2]), C.c_int(max_batch),
                                     C.c_int(dtype), C.c_int(1 if tune else 0), _stream(stream),
                                     C.byref(self._h))
        _check(st, "cprune_net_create")
        c, h, w = C.c_int(0), C.c_int(0), C.c_int(0)
        _check(lib().cprune_net_output_shape(self._h, C.byref(c), C.byref(h), C.byref(w)),
               "cprune_net_output_shape")
        self.out_shape = (c.value,) if h.value * w.value == 1 else (c.value, h.value, w.value)
        self.out_features = c.value * h.value * w.value

    def forward(self, x, logits=None, use_graph=False, stream=None):
        n = x.shape[0]
        if logits is None and use_graph:
            # a recorded graph is keyed by (n, x, logits): without a buffer of the caller's, the same one is
            # handed out for every replay at this batch size (a later call overwrites an earlier result)
            logits = self._graph_logits.get(n)
            if logits is None:
                logits = torch.empty((n,) + self.out_shape, dtype=TORCH_DTYPE[self.dtype], device=x.device)
                self._graph_logits[n] = logits
        if logits is None:
            logits = torch.empty((n,) + self.out_shape, dtype=TORCH_DTYPE[self.dtype], device=x.device)
        elif logits.numel() < n * self.out_features or logits.dtype != TORCH_DTYPE[self.dtype]:
            raise ValueError("logits buffer too small or of the wrong dtype for this net")
        st = lib().cprune_net_forward(self._h, _ptr(x), C.c_int(n), _ptr(logits),
                                      C.c_int(1 if use_graph else 0), _stream(stream))
        _check(st, "cprune_net_forward")
        return logits

    def layer_times(self, x, iters=10, stream=None):
        ms = (C.c_float * self.n_layers)()
        st = lib().cprune_net_layer_times(self._h, _ptr(x), C.c_int(x.shape[0]), C.c_int(iters), ms,
                                          _stream(stream))
        _check(st, "cprune_net_layer_times")
        return list(ms)

    def activation(self, layer: int, n: int, shape, stream=None):
        out = torch.empty((n,) + tuple(shape), dtype=TORCH_DTYPE[self.dtype], device="cuda")
        st = lib().cprune_net_copy_activation(self._h, C.c_int(layer), C.c_int(n), _ptr(out),
                                              C.c_size_t(out.numel() * out.element_size()),
                                              _stream(stream))
        _check(st, "cprune_net_copy_activation")
        return out

    def task_table(self):
        """-> (task of each layer or -1, number of tasks)."""
        tasks = (C.c_int * self.n_layers)()
        n = C.c_int(0)
        _check(lib().cprune_net_task_table(self._h, tasks, C.byref(n)), "cprune_net_task_table")
        return list(tasks), int(n.value)

    def task_key(self, layer: int) -> Tuple[int, ...]:
        """The key the task table groups by, for a dense conv / fully connected layer."""
        key = (C.c_int32 * 18)()
        _check(lib().cprune_net_task_key(self._h, C.c_int(layer), key), "cprune_net_task_key")
        return tuple(key)

    def fuse_depthwise(self, layer: int, enable: bool):
        _check(lib().cprune_net_fuse_depthwise(self._h, C.c_int(layer), C.c_int(1 if enable else 0)),
               "cprune_net_fuse_depthwise")

    def fuse_block(self, layer: int, enable: bool):
        _check(lib().cprune_net_fuse_block(self._h, C.c_int(layer), C.c_int(1 if enable else 0)),
               "cprune_net_fuse_block")

    def first_layer_form(self, form: int):
        """How a 16-bit 7x7 / stride 2 first layer runs: 0 general kernels, 1 its own kernel, 2 with the max-pool."""
        _check(lib().cprune_net_first_layer_form(self._h, C.c_int(form)), "cprune_net_first_layer_form")

    def fuse_first_layers(self, enable: bool):
        _check(lib().cprune_net_fuse_first_layers(self._h, C.c_int(1 if enable else 0)),
               "cprune_net_fuse_first_layers")

    def layer_fused(self, layer: int) -> bool:
        f = C.c_int(0)
        _check(lib().cprune_net_layer_fused(self._h, C.c_int(layer), C.byref(f)), "cprune_net_layer_fused")
        return bool(f.value)

    def set_layer_variant(self, layer: int, variant: int):
        _check(lib().cprune_net_set_layer_variant(self._h, C.c_int(layer), C.c_int(variant)),
               "cprune_net_set_layer_variant")

    def layer_variant(self, layer: int) -> int:
        v = C.c_int()
        _check(lib().cprune_net_layer_variant(self._h, C.c_int(layer), C.byref(v)),
               "cprune_net_layer_variant")
        return v.value

    def close(self):
        if self._h:
            lib().cprune_net_destroy(self._h)
            self._h = C.c_void_p(None)

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
