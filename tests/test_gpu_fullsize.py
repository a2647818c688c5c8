"""GPU parity at the benchmark's own sizes and launch configuration (tuned variants, HIP
graph replay, full batch).  Where the oracle cannot afford the whole batch it computes
whole images sampled from it (images are independent), or sampled output elements."""
import numpy as np
import pytest
import torch

from paper_2207_01260_amd import binding as B
from paper_2207_01260_amd import pipeline, synth

pytestmark = pytest.mark.gpu

TOL = {B.F32: 1e-4, B.F16: 2e-2, B.BF16: 2e-2}


def nmax(g, r):
    g = np.asarray(g, dtype=np.float64)
    r = np.asarray(r, dtype=np.float64)
    assert g.shape == r.shape, (g.shape, r.shape)
    return float(np.max(np.abs(g - r)) / max(np.max(np.abs(r)), 1e-30))


def _net_case(orc, net, cid, batch, dtype, sample):
    params = synth.layer_params(net, cid)
    x = synth.net_input(net, cid, batch)
    ref_layers, ref_kept = orc.prune_net(net, params)
    layers, kept = pipeline.prune_net(net, pipeline.upload_params(params), dtype)
    for i in kept:
        assert np.array_equal(kept[i].cpu().numpy(), ref_kept[i])
    handle = pipeline.build_net(net, layers, batch, dtype, tune=True)
    xd = torch.from_numpy(x).cuda().to(B.TORCH_DTYPE[dtype])
    eager = handle.forward(xd, use_graph=False).float().cpu().numpy()
    for _ in range(3):
        graph = handle.forward(xd, use_graph=True)
        torch.cuda.synchronize()
        assert np.array_equal(graph.float().cpu().numpy(), eager)
    handle.close()
    ref = orc.forward(net, ref_layers, np.ascontiguousarray(x[sample]))
    err = nmax(eager[sample], ref)
    assert err < TOL[dtype], err
    return err


@pytest.mark.parametrize("dtype", [B.F32, B.F16])
def test_vgg16_batch64(orc, dtype):
    print("vgg16 b64", dtype, flush=True)
    _net_case(orc, synth.vgg16(10, 32), 2, 64, dtype, list(range(64)))


def test_vgg16_batch1(orc):
    _net_case(orc, synth.vgg16(10, 32), 2, 1, B.F32, [0])


@pytest.mark.parametrize("dtype", [B.F32, B.BF16])
def test_resnet18_batch32(orc, dtype):
    print("resnet18 b32", dtype, flush=True)
    _net_case(orc, synth.resnet18(1000, 224), 3, 32, dtype, [0, 31])


def test_mobilenetv2_batch64(orc):
    print("mobilenetv2 b64", flush=True)
    _net_case(orc, synth.mobilenetv2(1000, 224), 4, 64, B.F32, [0, 37, 63])


@pytest.mark.parametrize("path", ["entry_point", "handle"])
@pytest.mark.parametrize("c_out", [1, 15, 16, 17, 45, 100, 128])
def test_channel_sweep_points(orc, c_out, path):
    """3x3 conv at 56x56, C_in 128, batch 8, filters pruned from 128 to c_out by L1 rank;
    run through the NCHW entry point with the variant cprune_select_tile picks, and through a
    tuned one-layer inference handle (channels-last kernels); outputs checked at sampled
    positions."""
    print("sweep c_out", c_out, path, flush=True)
    net = synth.single_conv(128, 128, 56)
    params = synth.layer_params(net, 5)
    params[0]["keep"] = c_out
    x = synth.net_input(net, 5, 8)
    ref_layers, ref_kept = orc.prune_net(net, params)
    layers, kept = pipeline.prune_net(net, pipeline.upload_params(params))
    assert np.array_equal(kept[0].cpu().numpy(), ref_kept[0])
    assert np.array_equal(layers[0]["w"].cpu().numpy(), ref_layers[0]["w"])
    xd = torch.from_numpy(x).cuda()
    if path == "handle":
        handle = pipeline.build_net(net, layers, 8, tune=True)
        y = handle.forward(xd, use_graph=True).cpu().numpy()
        assert y.shape == (8, c_out, 56, 56)
        v = handle.layer_variant(0)
        handle.close()
    else:
        d = B.conv_desc(x.shape, layers[0]["w"].shape, 1, 1)
        v, best_ms, _ = B.cprune_select_tile(d, xd, layers[0]["w"], layers[0]["b"], warmup=1, iters=3)
        y = B.cprune_conv2d_bn_relu(d, xd, layers[0]["w"], layers[0]["b"]).cpu().numpy()
    wref, bref = ref_layers[0]["w"], ref_layers[0]["b"]
    rng = np.random.RandomState(c_out)
    pts = [(0, 0, 0, 0), (7, c_out - 1, 55, 55), (3, c_out // 2, 0, 55), (4, 0, 55, 0)]
    pts += [(rng.randint(8), rng.randint(c_out), rng.randint(56), rng.randint(56)) for _ in range(600)]
    scale = float(np.max(np.abs(y)))
    worst = 0.0
    for (b, o, yy, xx) in pts:
        z = orc.conv2d_point(x, wref, b, o, yy, xx, 1, 1, 1) + float(bref[o])
        worst = max(worst, abs(max(z, 0.0) - float(y[b, o, yy, xx])))
    assert worst / scale < 1e-4, (worst, scale, B.cprune_tile_variant_info(v))
