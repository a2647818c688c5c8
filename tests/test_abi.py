"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every
symbol the header declares, and rejects bad arguments before touching the device."""
import ctypes as C
import os
import re

import pytest

from paper_2207_01260_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "cprune.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(cprune_[a-z0-9_]+)\s*\(", text)))


def test_exports_every_declared_symbol():
    lib = B.lib()
    names = _declared()
    assert len(names) >= 20
    for n in names:
        assert hasattr(lib, n), n
    assert sorted(B.EXPORTS) == names


def test_status_strings():
    lib = B.lib()
    seen = set()
    for code in (0, -1, -2, -3, -4, -5):
        s = lib.cprune_status_string(code)
        assert s and s not in seen
        seen.add(s)
    assert lib.cprune_status_string(-99)


def test_variant_table():
    nv = B.cprune_num_tile_variants()
    assert nv > 8
    seen = set()
    for v in range(nv):
        tm, tp, sk = B.cprune_tile_variant_info(v)
        assert tm % 16 == 0 and tp % 16 == 0 and sk >= -4
        seen.add((tm, tp, sk))
    with pytest.raises(B.CPruneError):
        B.cprune_tile_variant_info(nv)


def _desc(**kw):
    base = dict(n=1, c_in=8, h=8, w=8, c_out=8, kh=3, kw=3, stride=1, pad=1, groups=1,
                dtype=B.F32, act=B.ACT_RELU, has_residual=0)
    base.update(kw)
    return B.ConvDesc(**base)


FAKE = C.c_void_p(0x1000)   # never dereferenced: validation fails first


@pytest.mark.parametrize("kw,code", [
    (dict(n=0), B.ERR_INVALID_ARG), (dict(c_out=0), B.ERR_INVALID_ARG),
    (dict(stride=0), B.ERR_INVALID_ARG), (dict(dtype=7), B.ERR_INVALID_ARG),
    (dict(act=9), B.ERR_INVALID_ARG), (dict(kh=9, kw=9, h=16, w=16), B.ERR_UNSUPPORTED),
    (dict(groups=2), B.ERR_UNSUPPORTED), (dict(h=1, w=1, pad=0), B.ERR_INVALID_ARG),
    (dict(pad=3), B.ERR_UNSUPPORTED),
])
def test_conv_rejects_bad_desc(kw, code):
    d = _desc(**kw)
    st = B.lib().cprune_conv2d_bn_relu(C.byref(d), FAKE, FAKE, None, None, FAKE, C.c_int(-1), None,
                                       C.c_size_t(0), None)
    assert st == code


def test_conv_rejects_null_and_residual_mismatch_and_variant():
    d = _desc()
    L = B.lib()
    assert L.cprune_conv2d_bn_relu(C.byref(d), None, FAKE, None, None, FAKE, C.c_int(-1), None,
                                   C.c_size_t(0), None) == B.ERR_INVALID_ARG
    assert L.cprune_conv2d_bn_relu(C.byref(d), FAKE, FAKE, None, FAKE, FAKE, C.c_int(-1), None,
                                   C.c_size_t(0), None) == B.ERR_INVALID_ARG
    assert L.cprune_conv2d_bn_relu(C.byref(d), FAKE, FAKE, None, None, FAKE, C.c_int(10 ** 6), None,
                                   C.c_size_t(0), None) == B.ERR_INVALID_ARG


def test_cut_tiles_need_workspace():
    d = _desc(c_in=64, c_out=64, h=32, w=32)
    L = B.lib()
    nv = B.cprune_num_tile_variants()
    classic = [v for v in range(nv) if B.cprune_tile_variant_info(v)[2] == 0]
    cut = [v for v in range(nv) if B.cprune_tile_variant_info(v)[2] > 0]
    assert classic and cut
    assert all(B.cprune_conv_workspace_bytes(d, v) == 0 for v in classic)
    needs = {v: B.cprune_conv_workspace_bytes(d, v) for v in cut}
    v = max(needs, key=needs.get)
    assert needs[v] > 0 and B.cprune_conv_workspace_bytes(d, -1) == needs[v]
    tm, tp, _ = B.cprune_tile_variant_info(v)
    assert needs[v] % (2 * tm * tp * 4) == 0
    assert L.cprune_conv2d_bn_relu(C.byref(d), FAKE, FAKE, None, None, FAKE, C.c_int(v), FAKE,
                                   C.c_size_t(needs[v] - 1), None) == B.ERR_WORKSPACE


def test_rank_rejects_bad_args():
    L = B.lib()
    f = lambda c_out, keep, ws_bytes, kept=FAKE, scores=None, ws=FAKE: L.cprune_rank_filters(
        FAKE, C.c_int(c_out), C.c_int(4), C.c_int(3), C.c_int(3), C.c_int(keep), scores, None, kept,
        ws, C.c_size_t(ws_bytes), None)
    assert f(8, 0, 1 << 20) == B.ERR_INVALID_ARG
    assert f(8, 9, 1 << 20) == B.ERR_INVALID_ARG
    assert f(8, 4, 1 << 20, kept=None) == B.ERR_INVALID_ARG
    assert f(8, 4, 8) == B.ERR_WORKSPACE
    assert f(100000, 4, 1 << 30) == B.ERR_UNSUPPORTED
    assert L.cprune_rank_filters_workspace_bytes(C.c_int(8)) == 64


def test_gather_rejects_bad_args():
    L = B.lib()

    def g(n_out=4, n_in=4, gamma=None, bias_out=None, dtype=B.F32, keep_out=FAKE, keep_in=FAKE):
        return L.cprune_gather_pruned_weights(
            FAKE, C.c_int(8), C.c_int(8), C.c_int(3), C.c_int(3), keep_out, C.c_int(n_out), keep_in,
            C.c_int(n_in), gamma, None, None, None, C.c_float(1e-5), None, C.c_int(dtype), FAKE,
            bias_out, None)
    assert g(n_out=0) == B.ERR_INVALID_ARG
    assert g(n_out=9) == B.ERR_INVALID_ARG
    assert g(n_in=9) == B.ERR_INVALID_ARG
    assert g(gamma=FAKE) == B.ERR_INVALID_ARG           # partial BN
    assert g(dtype=5) == B.ERR_INVALID_ARG
    assert L.cprune_gather_channels(FAKE, C.c_int(1), C.c_int(4), C.c_int(2), C.c_int(2), C.c_int(0),
                                    FAKE, C.c_int(5), FAKE, None) == B.ERR_INVALID_ARG


def test_probe_rejects_bad_args():
    L = B.lib()
    out = C.c_float(0.0)
    assert L.cprune_probe_l2_bytes() > 0
    assert L.cprune_probe_l2_read(C.c_int(2), FAKE, C.c_size_t(1 << 30), FAKE, C.byref(out), None) == B.ERR_INVALID_ARG
    assert L.cprune_probe_l2_read(C.c_int(0), None, C.c_size_t(1 << 30), FAKE, C.byref(out), None) == B.ERR_INVALID_ARG
    assert L.cprune_probe_l2_read(C.c_int(0), FAKE, C.c_size_t(16), FAKE, C.byref(out), None) == B.ERR_WORKSPACE


def test_pool_fc_net_reject_bad_args():
    L = B.lib()
    assert L.cprune_maxpool2d(FAKE, C.c_int(1), C.c_int(1), C.c_int(4), C.c_int(4), C.c_int(0),
                              C.c_int(2), C.c_int(0), C.c_int(0), FAKE, None) == B.ERR_INVALID_ARG
    assert L.cprune_global_avgpool(None, C.c_int(1), C.c_int(1), C.c_int(4), C.c_int(4), C.c_int(0),
                                   FAKE, None) == B.ERR_INVALID_ARG
    assert L.cprune_fc(FAKE, FAKE, None, C.c_int(0), C.c_int(4), C.c_int(4), C.c_int(0), C.c_int(0),
                       FAKE, None, C.c_size_t(0), None) == B.ERR_INVALID_ARG
    h = C.c_void_p()
    assert L.cprune_net_create(None, C.c_int(1), C.c_int(3), C.c_int(8), C.c_int(8), C.c_int(1),
                               C.c_int(0), C.c_int(0), None, C.byref(h)) == B.ERR_INVALID_ARG
    # a layer that reads from a later layer is rejected before any allocation
    bad = (B.LayerDesc * 1)(B.LayerDesc(B.LAYER_MAXPOOL, 3, -1, 3, 3, 2, 2, 0, 1, 0, None, None))
    assert L.cprune_net_create(bad, C.c_int(1), C.c_int(3), C.c_int(8), C.c_int(8), C.c_int(1),
                               C.c_int(0), C.c_int(0), None, C.byref(h)) == B.ERR_INVALID_ARG
    assert L.cprune_net_forward(None, FAKE, C.c_int(1), FAKE, C.c_int(0), None) == B.ERR_INVALID_ARG
    assert L.cprune_net_destroy(None) == B.ERR_INVALID_ARG
    assert L.cprune_net_set_layer_variant(None, C.c_int(0), C.c_int(0)) == B.ERR_INVALID_ARG
    assert L.cprune_net_fuse_first_layers(None, C.c_int(1)) == B.ERR_INVALID_ARG
    assert L.cprune_net_first_layer_form(None, C.c_int(1)) == B.ERR_INVALID_ARG
    assert L.cprune_net_fuse_depthwise(None, C.c_int(0), C.c_int(1)) == B.ERR_INVALID_ARG
    assert L.cprune_net_fuse_block(None, C.c_int(0), C.c_int(1)) == B.ERR_INVALID_ARG
    dims = (C.c_int * 3)()
    assert L.cprune_net_output_shape(None, dims, dims, dims) == B.ERR_INVALID_ARG
