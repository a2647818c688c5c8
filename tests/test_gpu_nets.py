"""GPU parity of the whole path (rank -> gather/fold -> inference handle) against the
CPU oracle on the same seeded networks.  Kept lists bit-exact; logits and every layer's
activations within the normalised max error bar (1e-4 fp32, 2e-2 fp16 / bf16 against the
fp32 oracle)."""
import numpy as np
import pytest
import torch

from paper_2207_01260_amd import binding as B
from paper_2207_01260_amd import pipeline, synth

pytestmark = pytest.mark.gpu

TOL = {B.F32: 1e-4, B.F16: 2e-2, B.BF16: 2e-2}


from parity import check, nmax  # noqa: E402


def _run(orc, net, cid, batch, dtype, tune, check_layers=True, use_graph=False):
    params = synth.layer_params(net, cid)
    x = synth.net_input(net, cid, batch)
    ref_layers, ref_kept = orc.prune_net(net, params)
    ref_acts = orc.forward(net, ref_layers, x, return_all=True)

    dparams = pipeline.upload_params(params)
    layers, kept = pipeline.prune_net(net, dparams, dtype)
    assert sorted(kept) == sorted(ref_kept)
    for i in kept:
        assert np.array_equal(kept[i].cpu().numpy(), ref_kept[i]), net.layers[i].name
    if dtype == B.F32:
        for q, r in zip(layers, ref_layers):
            if "w" in q:
                assert np.array_equal(q["w"].cpu().numpy(), r["w"])
                assert np.array_equal(q["b"].cpu().numpy(), r["b"])
    handle = pipeline.build_net(net, layers, batch, dtype, tune=tune)
    xd = torch.from_numpy(x).cuda().to(B.TORCH_DTYPE[dtype])
    logits = handle.forward(xd, use_graph=use_graph)
    torch.cuda.synchronize()
    tol = TOL[dtype]
    if check_layers:
        for i, r in enumerate(ref_acts[:-1]):
            try:
                a = handle.activation(i, batch, r.shape[1:]).float().cpu().numpy()
            except B.CPruneError as e:
                # a conv whose max-pool runs in its epilogue is checked at the pool; a depthwise conv
                # (and the expansion in front of it) computed inside the 1x1 consumer's kernel at
                # that consumer
                assert e.status == B.ERR_UNSUPPORTED
                assert net.layers[i + 1].kind == "maxpool" or handle.layer_fused(i)
                continue
            check(a, r, dtype, net.layers[i].name)
    check(logits.float().cpu().numpy(), ref_acts[-1], dtype, "logits")
    return handle, xd, logits, ref_acts[-1]


def test_single_layer_config(orc):
    """One 3x3 conv+BN+ReLU, 64 filters ranked, top 45 kept, 32x32, batch 1."""
    net = synth.single_conv(64, 64, 32)
    params = synth.layer_params(net, 1)
    params[0]["keep"] = 45
    x = synth.net_input(net, 1, 1)
    ref_layers, ref_kept = orc.prune_net(net, params)
    ref = orc.forward(net, ref_layers, x)
    dparams = pipeline.upload_params(params)
    layers, kept = pipeline.prune_net(net, dparams)
    assert np.array_equal(kept[0].cpu().numpy(), ref_kept[0]) and kept[0].numel() == 45
    d = B.conv_desc(x.shape, layers[0]["w"].shape, 1, 1)
    y = B.cprune_conv2d_bn_relu(d, torch.from_numpy(x).cuda(), layers[0]["w"], layers[0]["b"])
    assert nmax(y.cpu().numpy(), ref) < 1e-4
    # dropping the filters == zeroing those channels of the unpruned layer, then slicing
    full_layers, _ = pipeline.prune_net(net, dparams, keep_override={0: 64})
    dfull = B.conv_desc(x.shape, full_layers[0]["w"].shape, 1, 1)
    yfull = B.cprune_conv2d_bn_relu(dfull, torch.from_numpy(x).cuda(), full_layers[0]["w"],
                                    full_layers[0]["b"])
    sliced = B.cprune_gather_channels(yfull, kept[0])
    assert nmax(sliced.cpu().numpy(), ref) < 1e-4


@pytest.mark.parametrize("batch", [1, 3])
def test_vgg16_fp32(orc, batch):
    print("vgg16 fp32 batch", batch, flush=True)
    handle, xd, logits, _ = _run(orc, synth.vgg16(10, 32), 2, batch, B.F32, tune=(batch == 3))
    # graph replay gives the same bits as the eager run, several times over
    for _ in range(3):
        again = handle.forward(xd, use_graph=True)
        torch.cuda.synchronize()
        assert torch.equal(again, logits)
    handle.close()


@pytest.mark.parametrize("dtype", [B.F16, B.BF16])
def test_vgg16_16bit(orc, dtype):
    print("vgg16 16-bit", dtype, flush=True)
    handle, *_ = _run(orc, synth.vgg16(10, 32), 2, 2, dtype, tune=False)
    handle.close()


def test_two_handles_on_two_streams(orc):
    """The caller owns the stream: two handles of the same net run side by side on two streams of the
    caller's (default priority), eagerly and as recorded graphs, and give the bits of a run on one stream."""
    net = synth.vgg16(10, 32)
    params = synth.layer_params(net, 2)
    layers, _ = pipeline.prune_net(net, pipeline.upload_params(params))
    x = torch.from_numpy(synth.net_input(net, 2, 4)).cuda()
    h0 = pipeline.build_net(net, layers, 4, tune=False)
    h1 = pipeline.build_net(net, layers, 4, tune=False)
    want = h0.forward(x).clone()
    torch.cuda.synchronize()
    s0, s1 = torch.cuda.Stream(), torch.cuda.Stream()
    outs = []
    for rep in range(4):
        with torch.cuda.stream(s0):
            a = h0.forward(x, use_graph=(rep % 2 == 1)).clone()
        with torch.cuda.stream(s1):
            b = h1.forward(x, use_graph=(rep % 2 == 1)).clone()
        outs += [a, b]
    s0.synchronize(); s1.synchronize()
    for o in outs:
        assert torch.equal(o, want)
    h0.close(); h1.close()


def test_vgg16_smaller_batch_than_max(orc):
    net = synth.vgg16(10, 32)
    params = synth.layer_params(net, 2)
    x = synth.net_input(net, 2, 4)
    ref_layers, _ = orc.prune_net(net, params)
    layers, _ = pipeline.prune_net(net, pipeline.upload_params(params))
    handle = pipeline.build_net(net, layers, 4, tune=False)
    xd = torch.from_numpy(x).cuda()
    y4 = handle.forward(xd).cpu().numpy()
    y2 = handle.forward(xd[:2].contiguous()).cpu().numpy()
    ref = orc.forward(net, ref_layers, x)
    assert nmax(y4, ref) < 1e-4 and nmax(y2, ref[:2]) < 1e-4
    with pytest.raises(B.CPruneError):
        handle.forward(torch.zeros((5, 3, 32, 32), device="cuda"))
    handle.close()


@pytest.mark.parametrize("dtype", [B.F32, B.F16, B.BF16])
def test_pinned_variants(orc, dtype):
    """Every variant that accepts a layer's shape can be pinned on it (as a stored tuning result
    would be), also after a graph of the net was recorded; results stay within the bar.  The
    layers cover every kind of tile: 32x32 .. 4x4 maps, with and without a fused pool."""
    net = synth.vgg16(10, 32)
    handle, xd, logits, ref = _run(orc, net, 2, 3, dtype, tune=False, check_layers=False, use_graph=True)
    nv = B.cprune_num_tile_variants()
    # 14, 16: 2x2 maps run as one matrix (16 with the pool in its epilogue); 18: the classifier
    layers = [1, 3, 4, 8, 11, 12, 14, 16, 18] if dtype == B.F32 else [4, 12, 16, 18]
    for layer in layers:
        before = handle.layer_variant(layer)
        pinned = 0
        for v in range(nv):
            try:
                handle.set_layer_variant(layer, v)
            except B.CPruneError as e:
                assert e.status == B.ERR_UNSUPPORTED
                continue
            pinned += 1
            assert handle.layer_variant(layer) == v
            out = handle.forward(xd, use_graph=(v % 2 == 0))
            torch.cuda.synchronize()
            err = nmax(out.float().cpu().numpy(), ref)
            assert err < TOL[dtype], (layer, v, B.cprune_tile_variant_info(v), err)
        print("layer", layer, "variants pinned", pinned, flush=True)
        assert pinned >= 4
        handle.set_layer_variant(layer, before)
    with pytest.raises(B.CPruneError):
        handle.set_layer_variant(2, 0)           # a max-pool has no variants
    with pytest.raises(B.CPruneError):
        handle.set_layer_variant(3, nv)
    handle.close()


def test_resnet18_shortcut_channels_pruned(orc):
    """Dependency-aware pruning: every layer on a stage's shortcut stream follows one kept
    list ranked on the summed filter norms; kept lists bit-exact, activations at the bar."""
    print("resnet18 shortcuts 64x64", flush=True)
    handle, *_ = _run(orc, synth.resnet18(100, 64, prune_shortcuts=True), 7, 2, B.F32, tune=False)
    handle.close()


def test_resnet18_shortcuts_full_size_fp16(orc):
    handle, *_ = _run(orc, synth.resnet18(1000, 224, prune_shortcuts=True), 7, 1, B.F16, tune=False,
                      check_layers=False)
    handle.close()


def test_resnet18_bf16(orc):
    handle, *_ = _run(orc, synth.resnet18(100, 64), 3, 2, B.BF16, tune=False)
    handle.close()


def test_mobilenetv2_reduced_input(orc):
    print("mobilenetv2 64x64", flush=True)
    handle, *_ = _run(orc, synth.mobilenetv2(100, 64), 4, 2, B.F32, tune=False)
    handle.close()


def test_mnasnet_reduced_input(orc):
    """5x5 depthwise stages, plain ReLU; every layer's activation checked."""
    print("mnasnet 64x64", flush=True)
    handle, *_ = _run(orc, synth.mnasnet(100, 64), 6, 2, B.F32, tune=False)
    handle.close()


def test_mnasnet_bf16_full_size_batch1(orc):
    print("mnasnet 224 b1 bf16", flush=True)
    handle, *_ = _run(orc, synth.mnasnet(1000, 224), 6, 1, B.BF16, tune=False, check_layers=False)
    handle.close()


def test_resnet18_full_size_batch1(orc):
    print("resnet18 224 b1", flush=True)
    handle, *_ = _run(orc, synth.resnet18(1000, 224), 3, 1, B.F32, tune=False, check_layers=False)
    handle.close()


def test_mobilenetv2_full_size_batch1(orc):
    print("mobilenetv2 224 b1", flush=True)
    handle, *_ = _run(orc, synth.mobilenetv2(1000, 224), 4, 1, B.F32, tune=False,
                      check_layers=False)
    handle.close()


def _check_forward(handle, net, xd, ref_acts, dtype, batch, use_graph=False):
    logits = handle.forward(xd, use_graph=use_graph)
    torch.cuda.synchronize()
    stored = 0
    for i, r in enumerate(ref_acts[:-1]):
        try:
            a = handle.activation(i, batch, r.shape[1:]).float().cpu().numpy()
        except B.CPruneError as e:
            assert e.status == B.ERR_UNSUPPORTED
            assert net.layers[i + 1].kind == "maxpool" or handle.layer_fused(i)
            continue
        stored += 1
        check(a, r, dtype, net.layers[i].name)
    check(logits.float().cpu().numpy(), ref_acts[-1], dtype, "logits")
    return stored


def _first_layer_probe(c_in, c1, h, w):
    """image -> 7x7 / stride 2 conv -> 3x3 / stride 2 max-pool -> 3x3 conv, on a map of any size"""
    net = synth.NetSpec(f"stemprobe_{c_in}_{c1}_{h}_{w}", c_in, h, w)
    a = net.add(synth.Layer("conv", -1, c_in, c1, k=7, stride=2, pad=3, act=synth.ACT_RELU, bn=True, name="stem"))
    p = net.add(synth.Layer("maxpool", a, c1, c1, k=3, stride=2, pad=1, name="pool"))
    net.add(synth.Layer("conv", p, c1, 24, k=3, stride=1, pad=1, act=synth.ACT_NONE, bn=True, name="b"))
    return net


@pytest.mark.parametrize("case", [
    ("resnet18", 3, B.F16), ("resnet18", 3, B.BF16),
    ((3, 20, 37, 35), 2, B.BF16),     # odd image width (element-wise patch loads), ragged 7x7 pooled blocks, 32-filter tile
    ((1, 40, 30, 50), 3, B.F16),      # one input channel, 64-filter tile with 40 filters
    ((3, 70, 18, 22), 2, B.F16),      # two filter tiles
])
def test_first_layer_forms_16bit(orc, case):
    """The 7x7 / stride 2 first layer in 16-bit data: through the general kernels (form 0), through the kernel
    made for it (1), and with the 3x3 / stride 2 max-pool inside that kernel (2, what an untimed handle takes):
    every stored activation and the output within the bar in each form, graph replay included."""
    which, batch, dtype = case
    print("first layer forms", case, flush=True)
    net = synth.resnet18(100, 64) if which == "resnet18" else _first_layer_probe(*which)
    cid = 70
    params = synth.layer_params(net, cid)
    x = synth.net_input(net, cid, batch)
    ref_layers, _ = orc.prune_net(net, params)
    ref_acts = orc.forward(net, ref_layers, x, return_all=True)
    layers, _ = pipeline.prune_net(net, pipeline.upload_params(params), dtype)
    handle = pipeline.build_net(net, layers, batch, dtype, tune=False)
    xd = torch.from_numpy(x).cuda().to(B.TORCH_DTYPE[dtype])
    fused = _check_forward(handle, net, xd, ref_acts, dtype, batch)
    with pytest.raises(B.CPruneError):          # the conv map is not stored in the form taken by default
        handle.activation(0, batch, ref_acts[0].shape[1:])
    for form in (1, 0, 2):
        handle.first_layer_form(form)
        stored = _check_forward(handle, net, xd, ref_acts, dtype, batch, use_graph=(form == 2))
        assert stored == fused + (1 if form < 2 else 0)
    handle.close()


def test_first_layer_form_needs_16bit_and_a_7x7_opening(orc):
    net = synth.resnet18(100, 64)
    params = synth.layer_params(net, 3)
    layers, _ = pipeline.prune_net(net, pipeline.upload_params(params), B.F32)
    handle = pipeline.build_net(net, layers, 1, B.F32, tune=False)
    with pytest.raises(B.CPruneError) as e:
        handle.first_layer_form(1)
    assert e.value.status == B.ERR_UNSUPPORTED
    handle.close()
    net = synth.vgg16(10, 32)
    params = synth.layer_params(net, 2)
    layers, _ = pipeline.prune_net(net, pipeline.upload_params(params), B.F16)
    handle = pipeline.build_net(net, layers, 1, B.F16, tune=False)
    with pytest.raises(B.CPruneError) as e:
        handle.first_layer_form(1)
    assert e.value.status == B.ERR_UNSUPPORTED
    handle.close()


# ---- the channels-last kernels on arbitrary layer shapes, every variant -----------------

def _two_layer_net(c0, c1, c2, hw, k, stride, pad, act, residual):
    net = synth.NetSpec(f"probe_{c0}_{c1}_{c2}_{hw}_{k}_{stride}", c0, hw, hw)
    a = net.add(synth.Layer("conv", -1, c0, c1, k=3, stride=1, pad=1, act=synth.ACT_RELU, bn=True, name="a"))
    net.add(synth.Layer("conv", a, c1, c2, k=k, stride=stride, pad=pad, act=act, bn=True,
                        residual=(a if residual else None), name="b"))
    return net


@pytest.mark.parametrize("cfg", [
    # c0, c1, c2, hw, k, stride, pad, act, residual, batch, dtype
    (5, 37, 45, 13, 3, 1, 1, synth.ACT_RELU, False, 3, B.F32),       # ragged everything
    (8, 24, 24, 12, 3, 1, 1, synth.ACT_NONE, True, 2, B.F32),        # shortcut add, no activation
    (6, 64, 100, 14, 1, 1, 0, synth.ACT_RELU6, False, 2, B.F32),     # 1x1
    (6, 40, 70, 15, 1, 2, 0, synth.ACT_NONE, False, 2, B.F32),       # strided 1x1 (downsample)
    (7, 19, 33, 17, 3, 2, 1, synth.ACT_RELU, False, 2, B.F32),       # strided 3x3
    (8, 40, 70, 14, 3, 2, 1, synth.ACT_RELU, False, 3, B.BF16),      # strided 3x3, 16-bit, even map, five filter blocks
    (6, 90, 37, 28, 3, 2, 1, synth.ACT_NONE, False, 1, B.F16),       # strided 3x3, three channel chunks, 28 -> 14
    (5, 9, 20, 21, 7, 2, 3, synth.ACT_RELU, False, 1, B.F32),        # 7x7 / 2
    (6, 12, 18, 11, 5, 1, 2, synth.ACT_RELU, False, 2, B.F32),       # 5x5
    (8, 44, 44, 8, 3, 1, 1, synth.ACT_RELU, True, 5, B.BF16),        # 16-bit, shortcut, 8x8 map
    (8, 30, 50, 4, 3, 1, 1, synth.ACT_RELU, False, 9, B.F16),        # 4x4 map: multi-image tiles
    (8, 52, 52, 3, 1, 1, 0, synth.ACT_RELU, True, 5, B.BF16),        # 1x1 with shortcut on a 3x3 map, 16-bit
    (4, 300, 21, 2, 1, 1, 0, synth.ACT_NONE, False, 7, B.F32),       # long reduction, few pixels
])
def test_channels_last_layer_every_variant(orc, cfg):
    c0, c1, c2, hw, k, stride, pad, act, residual, batch, dtype = cfg
    print("probe", cfg, flush=True)
    net = _two_layer_net(c0, c1, c2, hw, k, stride, pad, act, residual)
    cid = 40 + k + stride
    params = synth.layer_params(net, cid)
    x = synth.net_input(net, cid, batch)
    ref_layers, _ = orc.prune_net(net, params)
    ref = orc.forward(net, ref_layers, x)
    layers, _ = pipeline.prune_net(net, pipeline.upload_params(params), dtype)
    handle = pipeline.build_net(net, layers, batch, dtype, tune=False)
    xd = torch.from_numpy(x).cuda().to(B.TORCH_DTYPE[dtype])
    ran, names = 0, set()
    for v in range(B.cprune_num_tile_variants()):
        try:
            handle.set_layer_variant(1, v)
        except B.CPruneError as e:
            assert e.status == B.ERR_UNSUPPORTED
            continue
        ran += 1
        names.add(B.cprune_tile_variant_name(v, True, dtype).split("<")[0])
        out = handle.forward(xd)
        torch.cuda.synchronize()
        err = nmax(out.float().cpu().numpy(), ref)
        assert err < TOL[dtype], (v, B.cprune_tile_variant_name(v, True, dtype), err)
    handle.close()
    assert ran >= 100 or (k == 3 and stride == 1 and ran >= 110)
    if k == 3 and stride == 2:
        assert "conv_patch_s2_kernel" in names, names


@pytest.mark.parametrize("cfg", [
    # c0, c1, c2, hw, batch, dtype: 3x3 conv + 2x2 max-pool (run in the conv's epilogue), every variant
    (6, 40, 52, 6, 5, B.F32),      # 6x6 map: ragged 4x4 blocks, windows never straddle a block
    (5, 33, 21, 10, 3, B.F32),     # 10x10
    (8, 48, 40, 14, 2, B.BF16),    # 14x14, 16-bit
    (7, 150, 70, 4, 11, B.F32),    # 4x4 map, many channels, ragged last group of images
])
def test_pooled_layer_every_variant(orc, cfg):
    c0, c1, c2, hw, batch, dtype = cfg
    print("pooled probe", cfg, flush=True)
    net = synth.NetSpec(f"poolprobe_{c0}_{c1}_{c2}_{hw}", c0, hw, hw)
    a = net.add(synth.Layer("conv", -1, c0, c1, k=3, stride=1, pad=1, act=synth.ACT_RELU, bn=True, name="a"))
    b = net.add(synth.Layer("conv", a, c1, c2, k=3, stride=1, pad=1, act=synth.ACT_RELU, bn=True, name="b"))
    net.add(synth.Layer("maxpool", b, c2, c2, k=2, stride=2, name="pool"))
    cid = 60 + hw
    params = synth.layer_params(net, cid)
    x = synth.net_input(net, cid, batch)
    ref_layers, _ = orc.prune_net(net, params)
    ref = orc.forward(net, ref_layers, x)
    layers, _ = pipeline.prune_net(net, pipeline.upload_params(params), dtype)
    handle = pipeline.build_net(net, layers, batch, dtype, tune=False)
    xd = torch.from_numpy(x).cuda().to(B.TORCH_DTYPE[dtype])
    ran, names = 0, set()
    for v in range(B.cprune_num_tile_variants()):
        try:
            handle.set_layer_variant(1, v)
        except B.CPruneError as e:
            assert e.status == B.ERR_UNSUPPORTED
            continue
        ran += 1
        names.add(B.cprune_tile_variant_name(v, True, dtype).split("<")[0])
        out = handle.forward(xd)
        torch.cuda.synchronize()
        err = nmax(out.float().cpu().numpy(), ref)
        assert err < TOL[dtype], (v, B.cprune_tile_variant_name(v, True, dtype), err)
    handle.close()
    # a fused pool is run by the patch kernels and the independent-wavefront kernel
    assert ran >= 12 and "conv_wave_kernel" in names and "conv_patch_kernel" in names, (ran, names)


def _random_layer_cases():
    rng = np.random.RandomState(220701260)
    cases = []
    for i in range(18):
        k = int(rng.choice([1, 3, 3, 3]))
        stride = int(rng.choice([1, 1, 2]))
        h, w = int(rng.randint(1, 21)), int(rng.randint(1, 21))
        c0, c1, c2 = int(rng.randint(1, 9)), int(rng.randint(1, 91)), int(rng.randint(1, 91))
        residual = bool(k == 3 and stride == 1 and rng.randint(0, 3) == 0)
        if residual:
            c2 = c1
        act = int(rng.choice([synth.ACT_RELU, synth.ACT_NONE, synth.ACT_RELU6]))
        cases.append((c0, c1, c2, h, w, k, stride, act, residual, int(rng.randint(1, 6)), [B.F32, B.F16, B.BF16][i % 3]))
    return cases


@pytest.mark.parametrize("cfg", _random_layer_cases())
def test_random_layer_shapes_every_variant(orc, cfg):
    """Seeded random layer shapes (maps from 1x1 to 20x20, not square, 1-90 channels, 1x1 and 3x3 windows, both
    strides, every activation, with and without a shortcut) through every variant that accepts them."""
    c0, c1, c2, h, w, k, stride, act, residual, batch, dtype = cfg
    print("random probe", cfg, flush=True)
    net = synth.NetSpec(f"rprobe_{c0}_{c1}_{c2}_{h}_{w}_{k}_{stride}", c0, h, w)
    a = net.add(synth.Layer("conv", -1, c0, c1, k=3, stride=1, pad=1, act=synth.ACT_RELU, bn=True, name="a"))
    net.add(synth.Layer("conv", a, c1, c2, k=k, stride=stride, pad=k // 2, act=act, bn=True,
                        residual=(a if residual else None), name="b"))
    cid = 90 + k + stride
    params = synth.layer_params(net, cid)
    x = synth.net_input(net, cid, batch)
    ref_layers, _ = orc.prune_net(net, params)
    ref = orc.forward(net, ref_layers, x)
    layers, _ = pipeline.prune_net(net, pipeline.upload_params(params), dtype)
    handle = pipeline.build_net(net, layers, batch, dtype, tune=False)
    xd = torch.from_numpy(x).cuda().to(B.TORCH_DTYPE[dtype])
    ran = 0
    for v in range(B.cprune_num_tile_variants()):
        try:
            handle.set_layer_variant(1, v)
        except B.CPruneError as e:
            assert e.status == B.ERR_UNSUPPORTED
            continue
        ran += 1
        out = handle.forward(xd)
        torch.cuda.synchronize()
        check(out.float().cpu().numpy(), ref, dtype, f"{cfg} {B.cprune_tile_variant_name(v, True, dtype)}")
    handle.close()
    assert ran >= 50


@pytest.mark.parametrize("cfg", [
    # c0, c1, c2, hw, pool, batch, dtype: image -> 3x3 conv -> 3x3 conv [-> 2x2 pool] as one kernel
    (3, 28, 29, 32, True, 5, B.F32),      # the opening of the benchmark's network
    (3, 19, 45, 13, False, 3, B.F32),     # ragged tiles, two filter tiles of the second layer
    (1, 7, 12, 10, True, 2, B.F32),       # one image channel, one filter block
    (2, 32, 70, 18, True, 2, B.BF16),     # 16-bit, 32 first-layer filters, more than one filter tile
    (3, 30, 33, 24, False, 4, B.F16),
])
def test_first_two_layers_as_one_kernel(orc, cfg):
    c0, c1, c2, hw, pool, batch, dtype = cfg
    print("stem2 probe", cfg, flush=True)
    net = synth.NetSpec(f"stem2probe_{c0}_{c1}_{c2}_{hw}_{int(pool)}", c0, hw, hw)
    a = net.add(synth.Layer("conv", -1, c0, c1, k=3, stride=1, pad=1, act=synth.ACT_RELU, bn=True, name="a"))
    b = net.add(synth.Layer("conv", a, c1, c2, k=3, stride=1, pad=1, act=synth.ACT_RELU, bn=True, name="b"))
    if pool:
        net.add(synth.Layer("maxpool", b, c2, c2, k=2, stride=2, name="pool"))
    cid = 80 + hw
    params = synth.layer_params(net, cid)
    x = synth.net_input(net, cid, batch)
    ref_layers, _ = orc.prune_net(net, params)
    ref = orc.forward(net, ref_layers, x)
    layers, _ = pipeline.prune_net(net, pipeline.upload_params(params), dtype)
    handle = pipeline.build_net(net, layers, batch, dtype, tune=False)
    xd = torch.from_numpy(x).cuda().to(B.TORCH_DTYPE[dtype])
    assert not handle.layer_fused(0)
    apart = handle.forward(xd).float().cpu().numpy()
    handle.fuse_first_layers(True)
    assert handle.layer_fused(0)
    with pytest.raises(B.CPruneError):
        handle.set_layer_variant(1, 0)          # runs inside the fused kernel: no variants
    fused = handle.forward(xd).float().cpu().numpy()
    fused_graph = handle.forward(xd, use_graph=True).float().cpu().numpy()
    small = handle.forward(xd[:1]).float().cpu().numpy()
    handle.fuse_first_layers(False)
    again = handle.forward(xd).float().cpu().numpy()
    handle.close()
    tol = TOL[dtype]
    assert nmax(apart, ref) < tol and nmax(fused, ref) < tol, (nmax(apart, ref), nmax(fused, ref))
    assert np.array_equal(fused, fused_graph) and np.array_equal(apart, again)
    assert nmax(small, ref[:1]) < tol


def test_first_two_layers_fusion_needs_the_shape(orc):
    """A network that opens with a strided first layer has no such form."""
    net = synth.resnet18(10, 32)
    params = synth.layer_params(net, 3)
    layers, _ = pipeline.prune_net(net, pipeline.upload_params(params), B.F32)
    handle = pipeline.build_net(net, layers, 1, B.F32, tune=False)
    with pytest.raises(B.CPruneError) as e:
        handle.fuse_first_layers(True)
    assert e.value.status == B.ERR_UNSUPPORTED
    handle.close()


@pytest.mark.parametrize("which,dtype", [("mobilenetv2", B.F32), ("mnasnet", B.F32), ("mobilenetv2", B.F16),
                                         ("mnasnet", B.F16)])
def test_depthwise_fused_into_projection(orc, which, dtype):
    """Every depthwise + 1x1 pair of the net forced into the fused kernel (3x3 and 5x5 windows,
    stride 1 and 2, shortcut adds, ragged pruned channel counts), then forced apart again:
    logits and every stored activation within the bar both ways."""
    net = synth.mobilenetv2(100, 64) if which == "mobilenetv2" else synth.mnasnet(100, 64)
    cid = 4 if which == "mobilenetv2" else 6
    handle, xd, logits, ref = _run(orc, net, cid, 3, dtype, tune=False, check_layers=False)
    pairs = [i for i, L in enumerate(net.layers) if L.kind == "conv" and L.groups != 1]
    fused = 0
    for i in pairs:
        try:
            handle.fuse_depthwise(i, True)
        except B.CPruneError as e:
            assert e.status == B.ERR_UNSUPPORTED and net.layers[i + 1].k != 1
            continue
        assert handle.layer_fused(i)
        fused += 1
    assert fused >= 16
    params = synth.layer_params(net, cid)
    x = synth.net_input(net, cid, 3)
    ref_layers, _ = orc.prune_net(net, params)
    ref_acts = orc.forward(net, ref_layers, x, return_all=True)
    for graph in (False, True):
        out = handle.forward(xd, use_graph=graph)
        torch.cuda.synchronize()
        assert nmax(out.float().cpu().numpy(), ref) < TOL[dtype]
    for i, r in enumerate(ref_acts[:-1]):
        if net.layers[i].kind == "conv" and net.layers[i].groups != 1:
            with pytest.raises(B.CPruneError):
                handle.activation(i, 3, r.shape[1:])
            continue
        if dtype != B.F32:       # 16-bit: rounding accumulates over ~50 layers; the logits carry the bar
            continue
        a = handle.activation(i, 3, r.shape[1:]).float().cpu().numpy()
        assert nmax(a, r) < TOL[dtype], net.layers[i].name
    for i in pairs:
        handle.fuse_depthwise(i, False)
        assert not handle.layer_fused(i)
    out = handle.forward(xd)
    torch.cuda.synchronize()
    assert nmax(out.float().cpu().numpy(), ref) < TOL[dtype]
    handle.close()


@pytest.mark.parametrize("which,dtype,batch", [("mobilenetv2", B.F32, 3), ("mnasnet", B.F32, 2), ("mobilenetv2", B.F16, 2),
                                               ("mnasnet", B.F16, 3)])
def test_inverted_residual_block_as_one_kernel(orc, which, dtype, batch):
    """Every block whose expansion, depthwise layer and projection can run as one kernel is forced
    into it (3x3 and 5x5 windows, stride 1 and 2, with and without shortcut, ragged pruned
    expansion widths, maps down to 2x2 that a tile covers only partly), then forced apart
    again: logits and every stored activation within the bar both ways; graph replay alike."""
    net = synth.mobilenetv2(100, 64) if which == "mobilenetv2" else synth.mnasnet(100, 64)
    cid = 4 if which == "mobilenetv2" else 6
    handle, xd, logits, ref = _run(orc, net, cid, batch, dtype, tune=False, check_layers=False)
    dws = [i for i, L in enumerate(net.layers) if L.kind == "conv" and L.groups != 1]
    fused = []
    for i in dws:
        try:
            handle.fuse_block(i, True)
        except B.CPruneError as e:
            assert e.status == B.ERR_UNSUPPORTED
            continue
        assert handle.layer_fused(i) and handle.layer_fused(net.layers[i].input)
        fused.append(i)
    print(which, "blocks as one kernel:", len(fused), "of", len(dws), flush=True)
    assert len(fused) >= 4
    params = synth.layer_params(net, cid)
    x = synth.net_input(net, cid, batch)
    ref_layers, _ = orc.prune_net(net, params)
    ref_acts = orc.forward(net, ref_layers, x, return_all=True)
    for graph in (False, True, True):
        out = handle.forward(xd, use_graph=graph)
        torch.cuda.synchronize()
        assert nmax(out.float().cpu().numpy(), ref) < TOL[dtype]
    gone = set(fused) | {net.layers[i].input for i in fused}
    for i, r in enumerate(ref_acts[:-1]):
        if i in gone:
            with pytest.raises(B.CPruneError):
                handle.activation(i, batch, r.shape[1:])
            continue
        if dtype != B.F32 or handle.layer_fused(i):   # 16-bit: rounding accumulates over ~50 layers; the logits carry the bar
            continue
        a = handle.activation(i, batch, r.shape[1:]).float().cpu().numpy()
        assert nmax(a, r) < TOL[dtype], net.layers[i].name
    with pytest.raises(B.CPruneError):
        handle.set_layer_variant(net.layers[fused[0]].input, 0)      # the expansion has no program of its own now
    for i in fused:
        handle.fuse_block(i, False)
        assert handle.layer_fused(i) and not handle.layer_fused(net.layers[i].input)
    out = handle.forward(xd)
    torch.cuda.synchronize()
    assert nmax(out.float().cpu().numpy(), ref) < TOL[dtype]
    for i in fused:
        handle.fuse_depthwise(i, False)
        assert not handle.layer_fused(i)
    out = handle.forward(xd)
    torch.cuda.synchronize()
    assert nmax(out.float().cpu().numpy(), ref) < TOL[dtype]
    handle.close()


@pytest.mark.parametrize("cfg", [
    # c_in, c_exp, c_out, hw, k, stride, shortcut, batch, dtype
    (24, 150, 24, 19, 3, 1, True, 3, B.BF16),      # ragged map (19 = 2 tiles + 3), shortcut, 16-bit
    (20, 90, 37, 17, 3, 2, False, 2, B.BF16),      # stride 2, odd map
    (12, 70, 12, 9, 5, 1, True, 2, B.BF16),        # 5x5 window
    (16, 100, 40, 22, 5, 2, False, 2, B.F16),      # 5x5 / 2
    (64, 100, 48, 7, 3, 1, False, 5, B.F32),       # wide input (several rounds of the expansion's reduction), 7x7 map
    (128, 90, 100, 6, 3, 1, False, 2, B.F16),      # widest projection tile, 16-bit input of 128 channels
    (8, 20, 130, 8, 3, 1, False, 2, B.F32),        # projection too wide for one tile: not eligible
    (96, 400, 96, 7, 3, 1, True, 2, B.F32),        # weights too large to stay in LDS: not eligible
])
def test_inverted_residual_probe_blocks(orc, cfg):
    """One block behind a 3x3 conv, as one kernel and apart, on shapes the networks do not have."""
    c_in, c_exp, c_out, hw, k, stride, shortcut, batch, dtype = cfg
    print("block probe", cfg, flush=True)
    net = synth.NetSpec(f"mbprobe_{c_in}_{c_exp}_{c_out}_{hw}_{k}_{stride}", 3, hw, hw)
    a = net.add(synth.Layer("conv", -1, 3, c_in, k=3, stride=1, pad=1, act=synth.ACT_RELU, bn=True, name="a"))
    e = net.add(synth.Layer("conv", a, c_in, c_exp, k=1, stride=1, pad=0, act=synth.ACT_RELU6, bn=True,
                            prune_out="own", name="e"))
    d = net.add(synth.Layer("conv", e, c_exp, c_exp, k=k, stride=stride, pad=k // 2, groups=c_exp, act=synth.ACT_RELU6,
                            bn=True, prune_out=e, name="d"))
    net.add(synth.Layer("conv", d, c_exp, c_out, k=1, stride=1, pad=0, act=synth.ACT_NONE, bn=True,
                        residual=(a if shortcut else None), prune_in=e, name="p"))
    cid = 60 + k + stride
    params = synth.layer_params(net, cid)
    x = synth.net_input(net, cid, batch)
    ref_layers, _ = orc.prune_net(net, params)
    ref = orc.forward(net, ref_layers, x)
    layers, _ = pipeline.prune_net(net, pipeline.upload_params(params), dtype)
    handle = pipeline.build_net(net, layers, batch, dtype, tune=False)
    xd = torch.from_numpy(x).cuda().to(B.TORCH_DTYPE[dtype])
    if c_out > 128 or c_exp >= 400:
        with pytest.raises(B.CPruneError):
            handle.fuse_block(d, True)
        handle.close()
        return
    for on in (True, False, True):
        handle.fuse_block(d, on)
        assert handle.layer_fused(e) == on
        out = handle.forward(xd, use_graph=on)
        torch.cuda.synchronize()
        err = nmax(out.float().cpu().numpy(), ref)
        assert err < TOL[dtype], (on, err)
    handle.close()
