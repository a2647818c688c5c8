"""Search-side rows on the device: the handle's task table against the oracle's grouping,
Algorithm 1 driven by measured latencies (the recorded tables and latencies are replayed through
the oracle's loop: same final model, same log), and the predicted prune step against the
measured latency staircase."""
import numpy as np
import pytest
import torch

from oracle import search as osearch
from paper_2207_01260_amd import binding as B
from paper_2207_01260_amd import pipeline, synth
from paper_2207_01260_amd import search as psearch

pytestmark = pytest.mark.gpu


def test_task_table_resnet18_unpruned():
    """Unpruned ResNet-18 has repeated layer shapes; layers with the same shape, stride,
    padding, activation and shortcut are one task (Section 3.4)."""
    net = synth.resnet18(100, 64)
    params = synth.layer_params(net, 3)
    full = {i: L.c_out for i, L in enumerate(net.layers) if L.prune_out == "own"}
    layers, _ = pipeline.prune_net(net, pipeline.upload_params(params), B.F32, keep_override=full)
    handle = pipeline.build_net(net, layers, 2, B.F32, tune=False)
    task_of, n_tasks = handle.task_table()
    handle.close()
    shp = synth.shapes(net, full)
    keys = []
    for i, L in enumerate(net.layers):
        if L.kind == "fc" or (L.kind == "conv" and L.groups == 1):
            cin, cout, ho, wo = shp[i]
            hin, win = (net.in_h, net.in_w) if L.input < 0 else shp[L.input][2:4]
            keys.append((L.kind, cin, cout, hin, win, L.k, L.stride, L.pad, L.act, L.residual is not None))
        else:
            keys.append(None)
    want_of, want_members = osearch.task_table(keys)
    assert task_of == want_of and n_tasks == len(want_members)
    assert max(len(m) for m in want_members) >= 2          # the repeated shapes did merge
    assert n_tasks < sum(k is not None for k in keys)


def test_algorithm1_on_measured_latencies():
    """Algorithm 1 on the device (tune = rank + gather + tuned handle + task table + layer times,
    measure = forward time), then the recorded (model -> table, order, latency) replayed through
    the oracle's loop with the oracle's own prune rule: same final model, same log."""
    print("algorithm 1, vgg16 b8", flush=True)
    net = synth.vgg16(10, 32)
    params = synth.layer_params(net, 2)
    ds = psearch.DeviceSearch(net, params, 2, batch=8, steps=10)
    start = ds.initial_model(params)
    acc = lambda m: 1.0
    final, log = psearch.run_search(start, 0.0, 0.95, 0.999, ds.tune, ds.prune, ds.measure, acc, max_iterations=3)
    assert log, "no candidate was tried"
    for task, l_m, l_t, a_s, verdict in log:
        assert verdict in ("accepted", "slow", "exhausted")
        if verdict == "accepted":
            assert l_m < l_t
        if verdict == "slow":
            assert l_m >= l_t
    assert all(final[i] <= start[i] for i in start)
    n_acc = sum(v == "accepted" for *_, v in log)
    assert sum(start.values()) - sum(final.values()) > 0 if n_acc else final == start

    # replay: the oracle's loop over the latencies and tables the device produced
    recorded = {tuple(sorted(m.items())): (table, order, ms) for m, table, order, ms in ds.trace}

    def tune(model):
        table, order, _ = recorded[tuple(sorted(model.items()))]
        return table, order

    def measure(model):
        return recorded[tuple(sorted(model.items()))][2]

    def prune(model, task, subgraphs, program):
        cand, changed = dict(model), False
        for i in subgraphs:
            if i in cand:
                cut = osearch.prune_count(cand[i], program["step"])
                if cut > 0:
                    cand[i] -= cut
                    changed = True
        return cand if changed else None

    want_final, want_log = osearch.algorithm1(start, 0.0, 0.95, 0.999, tune, prune, measure, acc, max_iterations=3)
    assert final == want_final
    assert log == want_log, (log, want_log)

    # the first candidate is the task with the largest impact, and its cut is the one the step
    # rule gives for the structure of the variant that task runs (the oracle's rule on the
    # variant's split, the oracle's prune count)
    table, order = ds.tune(start)
    first = log[0][0]
    layers_of, program = table[first]
    assert first == order[0]
    if program["variant"] >= 0:
        ml, ep, unit = B.cprune_variant_filter_splits(program["variant"], program["c_out"])
        assert program["step"] == unit * osearch.lcm_step(ml, ep)
    else:
        # a layer that runs inside a fused kernel (the first two layers as one) has no variant of its own: those
        # kernels are built on 16-row blocks with one block loop, so the step is one block
        assert program["step"] == 16
    cand = ds.prune(start, first, layers_of, program)
    for i in layers_of:
        assert start[i] - cand[i] == osearch.prune_count(start[i], program["step"])
    imp = osearch.pruning_impact([table[t][1]["time_ms"] for t in order], [len(table[t][0]) for t in order])
    assert all(a >= b for a, b in zip(imp, imp[1:]))


def test_equal_shapes_with_and_without_pool_are_two_tasks(orc):
    """Two convolutions of the same shape, one of them with a 2x2 pool in its epilogue, run
    different programs: two tasks, two distinct keys, and the 2 x 18 map whose pool no kernel can
    fuse still builds and runs (the pool stays a layer of its own)."""
    for hw, fusable in (((8, 8), True), ((2, 8), True), ((2, 18), False)):
        net = synth.NetSpec("two_convs", 8, hw[0], hw[1])
        a = net.add(synth.Layer("conv", -1, 8, 8, k=3, stride=1, pad=1, act=synth.ACT_RELU, bn=True, name="a"))
        b = net.add(synth.Layer("conv", a, 8, 8, k=3, stride=1, pad=1, act=synth.ACT_RELU, bn=True, name="b"))
        p = net.add(synth.Layer("maxpool", b, 8, 8, k=2, stride=2, name="pool"))
        net.add(synth.Layer("conv", p, 8, 5, k=3, stride=1, pad=1, act=synth.ACT_NONE, bn=True, name="c"))
        params = synth.layer_params(net, 77)
        x = synth.net_input(net, 77, 2)
        ref_layers, _ = orc.prune_net(net, params)
        ref = orc.forward(net, ref_layers, x)
        layers, _ = pipeline.prune_net(net, pipeline.upload_params(params))
        handle = pipeline.build_net(net, layers, 2, B.F32, tune=False)
        task_of, n_tasks = handle.task_table()
        y = handle.forward(torch.from_numpy(x).cuda()).cpu().numpy()
        assert np.max(np.abs(y - ref)) / np.max(np.abs(ref)) < 1e-4
        if fusable:
            assert task_of[:2] == [0, 1] and n_tasks == 3
            assert handle.task_key(0) != handle.task_key(1)
        else:
            assert task_of[:2] == [0, 0] and n_tasks == 2
            assert handle.task_key(0) == handle.task_key(1)
        handle.close()


def test_graph_cache_stays_bounded():
    """Replays with a fresh output buffer per call: the handle keeps a bounded number of recorded
    graphs (the least recently used one makes room), results stay right throughout."""
    net = synth.vgg16(10, 32)
    params = synth.layer_params(net, 2)
    layers, _ = pipeline.prune_net(net, pipeline.upload_params(params))
    handle = pipeline.build_net(net, layers, 2, B.F32, tune=False)
    x = torch.from_numpy(synth.net_input(net, 2, 2)).cuda()
    want = handle.forward(x, use_graph=False).clone()
    torch.cuda.synchronize()
    free0 = torch.cuda.mem_get_info()[0]
    bufs = [torch.empty((2, 10), dtype=torch.float32, device="cuda") for _ in range(40)]
    for rep in range(25):
        for out in bufs:
            handle.forward(x, out, use_graph=True)
        torch.cuda.synchronize()
        assert torch.equal(bufs[rep % 40], want)
    free1 = torch.cuda.mem_get_info()[0]
    assert free0 - free1 < 256 << 20, (free0, free1)      # 1000 replays through 40 buffers leak nothing
    # without a buffer of the caller's, replays share one per batch size
    a = handle.forward(x, use_graph=True)
    b = handle.forward(x, use_graph=True)
    assert a.data_ptr() == b.data_ptr()
    torch.cuda.synchronize()
    assert torch.equal(a, want)
    handle.close()


def test_predicted_step_against_measured_staircase():
    """Config-5 layer (3x3, 56x56, C_in 128, batch 8): inside one predicted step the latency
    stays on its plateau; one step down it drops."""
    net = synth.single_conv(128, 128, 56)
    params = synth.layer_params(net, 5)
    dparams = pipeline.upload_params(params)
    x = torch.from_numpy(synth.net_input(net, 5, 8)).cuda()

    def timed(c_out, variant=None):
        layers, _ = pipeline.prune_net(net, dparams, B.F32, keep_override={0: c_out})
        handle = pipeline.build_net(net, layers, 8, B.F32, tune=(variant is None))
        if variant is not None:
            handle.set_layer_variant(0, variant)
        ms = min(handle.layer_times(x, iters=20)[0] for _ in range(3))
        v = handle.layer_variant(0)
        handle.close()
        return ms, v

    t128, v = timed(128)
    step = B.cprune_variant_prune_step(v, 128)
    assert step in (16, 32, 64, 128)
    t_in, _ = timed(128 - step + 1, v)       # same number of 16-row blocks per tile row
    t_down, _ = timed(128 - step, v)
    print("variant", B.cprune_tile_variant_info(v), "step", step, t128, t_in, t_down, flush=True)
    assert t_in > 0.93 * t128
    assert t_down < 0.97 * t128
