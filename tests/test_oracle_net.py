"""Network-level pins: layer lists against the counts the paper prints, and the
pruning semantics (keep-all == unpruned, pruned == zeroed-and-sliced) on whole nets."""
import os

import numpy as np
import pytest

from paper_2207_01260_amd import synth

GOLD = os.path.join(os.path.dirname(__file__), "golden", "paper_table_counts.txt")


def _golden():
    rows = {}
    for line in open(GOLD):
        if line.startswith("#") or not line.strip():
            continue
        name, macs, params = line.split()[:3]
        rows[name] = (float(macs), float(params))
    return rows


BUILDERS = {
    "resnet18": lambda: synth.resnet18(1000, 224),
    "mobilenetv2": lambda: synth.mobilenetv2(1000, 224),
    "resnet18_cifar": lambda: synth.resnet18(10, 32, cifar_stem=True),
    "mnasnet1_0": lambda: synth.mnasnet(1000, 224),
}


@pytest.mark.parametrize("name", sorted(BUILDERS))
def test_counts_match_paper_tables(name):
    macs, params = synth.count_macs_params(BUILDERS[name]())
    gm, gp = _golden()[name]
    # the paper prints three significant digits
    assert abs(macs - gm) / gm < 5e-3
    assert abs(params - gp) / gp < 5e-3


def test_exact_counts():
    assert synth.count_macs_params(synth.resnet18()) == (1814073344, 11679912)
    assert synth.count_macs_params(synth.mobilenetv2()) == (300774272, 3470760)
    assert synth.count_macs_params(synth.resnet18(10, 32, True)) == (555422720, 11164362)
    assert synth.count_macs_params(synth.vgg16()) == (313201664, 14715594)
    assert synth.count_macs_params(synth.mnasnet()) == (314415872, 4345392)


def test_activations_stay_inside_fp16_range(orc):
    """Self-test of the generators: no activation of the seeded networks comes near the largest fp16 value,
    so a 16-bit run can only differ from the fp32-master oracle by rounding, never by overflow."""
    for net, cid, batch in ((synth.vgg16(10, 32), 2, 2), (synth.resnet18(100, 64), 3, 1), (synth.mobilenetv2(100, 64), 4, 1)):
        params = synth.layer_params(net, cid)
        layers, _ = orc.prune_net(net, params)
        acts = orc.forward(net, layers, synth.net_input(net, cid, batch), return_all=True)
        worst = max(float(np.max(np.abs(a))) for a in acts)
        assert worst < 65504.0 / 16, (net.name, worst)


def test_keep_count_rule():
    assert synth.keep_count(0.7, 64) == 45
    assert synth.keep_count(0.5, 3) == 2          # 1.5 rounds half up
    assert synth.keep_count(0.001, 64) == 1
    assert synth.keep_count(1.0, 64) == 64


def test_generator_is_reproducible_and_sane():
    a = synth.normal(123, 100001)
    b = synth.normal(123, 100001)
    assert np.array_equal(a, b) and a.size == 100001
    assert abs(a.mean()) < 0.02 and abs(a.std() - 1.0) < 0.02
    u = synth.uniform(7, 50000, 0.4, 0.9)
    assert u.min() >= 0.4 and u.max() < 0.9 and abs(u.mean() - 0.65) < 0.01
    assert synth.stream_key(1, 2, 3) != synth.stream_key(1, 3, 2)


def _small_nets():
    return [("vgg16", synth.vgg16(10, 32), 2), ("resnet18", synth.resnet18(20, 64), 3),
            ("mobilenetv2", synth.mobilenetv2(20, 64), 4), ("mnasnet", synth.mnasnet(20, 64), 6),
            ("resnet18_shortcuts", synth.resnet18(20, 64, prune_shortcuts=True), 7)]


@pytest.mark.parametrize("name,net,cid", _small_nets())
def test_keep_all_equals_unpruned(orc, name, net, cid):
    params = synth.layer_params(net, cid)
    x = synth.net_input(net, cid, 1)
    keep_all = {i: L.c_out for i, L in enumerate(net.layers) if L.prune_out == "own"}
    pruned, kept = orc.prune_net(net, params, keep_all, fold=False)
    for i, k in kept.items():
        assert k.tolist() == list(range(net.layers[i].c_out))
    # an unpruned forward built straight from the raw parameters
    raw = []
    for L, p in zip(net.layers, params):
        if L.kind == "conv":
            raw.append({"w": p["w"], "bn": {t: p[t] for t in ("gamma", "beta", "mean", "var")}})
        elif L.kind == "fc":
            raw.append({"w": p["w"], "b": p["b"]})
        else:
            raw.append({})
    y_raw = orc.forward(net, raw, x)
    y_keep = orc.forward(net, pruned, x)
    assert np.array_equal(y_raw, y_keep)
    assert y_raw.shape == (1, net.layers[-1].c_out) and np.all(np.isfinite(y_raw))


@pytest.mark.parametrize("name,net,cid", _small_nets())
def test_pruned_net_equals_masked_full_net(orc, name, net, cid):
    """Pruning == running the unpruned net with every pruned channel forced to zero
    (unfolded BN, so that a removed channel is exactly zero after masking)."""
    params = synth.layer_params(net, cid)
    x = synth.net_input(net, cid, 1)
    pruned, kept = orc.prune_net(net, params, fold=False)
    y_pruned = orc.forward(net, pruned, x)
    # masked full net: zero the filters (and BN shift) of every pruned channel
    masked = []
    for i, (L, p) in enumerate(zip(net.layers, params)):
        if L.kind == "conv":
            src = i if L.prune_out == "own" else (L.prune_out if isinstance(L.prune_out, int)
                                                  else None)
            w = p["w"].copy()
            bn = {t: p[t].copy() for t in ("gamma", "beta", "mean", "var")}
            if src is not None:
                dead = np.setdiff1d(np.arange(L.c_out), kept[src])
                w[dead] = 0.0
                bn["beta"][dead] = 0.0
                bn["mean"][dead] = 0.0
            masked.append({"w": w, "bn": bn})
        elif L.kind == "fc":
            masked.append({"w": p["w"], "b": p["b"]})
        else:
            masked.append({})
    y_masked = orc.forward(net, masked, x)
    assert np.array_equal(y_pruned, y_masked)
    # and the pruned net really is smaller
    macs_full, _ = synth.count_macs_params(net)
    macs_pruned, _ = synth.count_macs_params(net, {i: k.size for i, k in kept.items()})
    assert macs_pruned < 0.9 * macs_full


def test_shortcut_groups_share_one_kept_list(orc):
    """Layers that write into the same shortcut sum follow one kept list, ranked on the sum
    of their filter norms; every reader of the sum drops the matching input channels."""
    net = synth.resnet18(20, 64, prune_shortcuts=True)
    params = synth.layer_params(net, 7)
    layers, kept = orc.prune_net(net, params)
    leads = [i for i, L in enumerate(net.layers) if L.score_with]
    assert len(leads) == 4                      # the stem and three downsample convs
    for lead in leads:
        L = net.layers[lead]
        members = [lead] + L.score_with
        total = sum(np.abs(params[j]["w"].astype(np.float64)).reshape(L.c_out, -1).sum(axis=1) for j in members)
        k = kept[lead].size
        order = sorted(range(L.c_out), key=lambda j: (-total[j], j))
        assert kept[lead].tolist() == sorted(order[:k])
        assert synth.min_relative_gap(total) > 1e-9
        for j in members:
            assert layers[j]["w"].shape[0] == k
            assert net.layers[j].prune_out == (lead if j != lead else "own")
        readers = [i for i, R in enumerate(net.layers) if R.prune_in == lead]
        assert readers
        for r in readers:
            assert layers[r]["w"].shape[1] == k
    assert layers[-1]["w"].shape == (20, kept[leads[-1]].size)


def test_folded_net_close_to_unfolded(orc):
    net = synth.vgg16(10, 32)
    params = synth.layer_params(net, 2)
    x = synth.net_input(net, 2, 2)
    lu, _ = orc.prune_net(net, params, fold=False)
    lf, _ = orc.prune_net(net, params, fold=True)
    yu, yf = orc.forward(net, lu, x), orc.forward(net, lf, x)
    assert np.max(np.abs(yu - yf)) / np.max(np.abs(yu)) < 1e-5


def test_single_layer_config_keeps_45_of_64(orc):
    net = synth.single_conv(64, 64, 32)
    params = synth.layer_params(net, 1)
    s, order, kept = orc.rank_filters(params[0]["w"], 45)
    assert kept.size == 45 and synth.min_relative_gap(s) > 1e-9
    layers, kept2 = orc.prune_net(net, params, {0: 45})
    assert np.array_equal(kept2[0], kept)
    y = orc.forward(net, layers, synth.net_input(net, 1, 1))
    assert y.shape == (1, 45, 32, 32) and np.all(y >= 0)
