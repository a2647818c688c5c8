"""The search loop of the method on the device: tasks and their pruning impact (Sections 3.3,
3.4), the number of filters to prune from the structure of the chosen program (Section 3.5)
and Algorithm 1's latency-gated iteration (Section 3.2), with every latency measured on the
GPU through the library.

Accuracy is not computed here (no dataset, no training): `accuracy` is a function the caller
supplies; the default accepts every candidate, which leaves the latency gate, the task order
and the step rule as the things that decide.

    python -m paper_2207_01260_amd.search [--net vgg16] [--batch 64] [--iterations 4]
"""
import argparse
import json
import time
from typing import Callable, Dict, List, Optional, Tuple

import torch

from . import binding as B
from . import pipeline, synth


# ---- Algorithm 1: the library decides, the caller measures ------------------------------

VERDICT = {1: "slow", 2: "inaccurate", 3: "accepted", 4: "exhausted"}


def run_search(model, a_goal: float, alpha: float, beta: float, tune: Callable, prune: Callable,
               measure: Callable, accuracy: Callable, max_iterations: int = 1 << 30):
    """Drives the library's search object (cprune_search_*, the decisions of Algorithm 1) with
    measurements made here.  tune(model) -> (table: task -> (subgraphs, program), tasks by
    descending impact); prune(model, task, subgraphs, program) -> candidate or None when nothing
    can be pruned; measure(model) -> time; accuracy(model) -> accuracy.  Tasks are hashable keys
    that mean the same task from model to model; the library sees them as integers.
    -> (final model, log of (task, l_m or None, l_t, a_s or None, verdict))."""
    ids: Dict = {}
    names: List = []

    def as_ids(tasks):
        out = []
        for t in tasks:
            if t not in ids:
                ids[t] = len(names)
                names.append(t)
            out.append(ids[t])
        return out

    table, order = tune(model)
    state = B.Search(a_goal, alpha, beta, max_iterations)
    try:
        state.start(as_ids(order), measure(model), accuracy(model))
        candidate = cand_table = None
        while True:
            task_id = state.next_task()
            if task_id is None:
                break
            task = names[task_id]
            subgraphs, program = table[task]
            candidate = prune(model, task, subgraphs, program)
            if candidate is None:
                state.report_exhausted()
                continue
            cand_table, cand_order = tune(candidate)
            if not state.report_latency(measure(candidate)):
                continue
            if state.report_accuracy(accuracy(candidate), as_ids(cand_order)):
                model, table = candidate, cand_table
        log = [(names[t], l_m, l_t, a_s, VERDICT[v]) for t, l_m, l_t, a_s, v in state.log()]
    finally:
        state.close()
    return model, log


# ---- the pieces, on the device ------------------------------------------------------

class DeviceSearch:
    """tune / prune / measure for a seeded synthetic network on the GPU.  A model is the dict
    {prunable layer index: filters kept}; every other quantity is derived from it by the
    library: kept lists by L1 rank, gathered and folded weights, a tuned handle, its task
    table, per-layer times and the forward time."""

    def __init__(self, net: synth.NetSpec, params: List[dict], config_id: int, batch: int,
                 dtype: int = B.F32, steps: int = 30):
        self.net, self.batch, self.dtype, self.steps = net, batch, dtype, steps
        self.dparams = pipeline.upload_params(params)
        self.x = torch.from_numpy(synth.net_input(net, config_id, batch)).cuda().to(B.TORCH_DTYPE[dtype])
        self.prunable = [i for i, L in enumerate(net.layers) if L.prune_out == "own"]
        self._cache: Dict[Tuple, dict] = {}
        self.trace: List[Tuple] = []      # (model, table, order, ms) of every model tuned, in order

    def initial_model(self, params: List[dict]) -> Dict[int, int]:
        return {i: int(params[i]["keep"]) for i in self.prunable}

    def _state(self, model: Dict[int, int]) -> dict:
        key = tuple(sorted(model.items()))
        st = self._cache.get(key)
        if st is not None:
            return st
        layers, _ = pipeline.prune_net(self.net, self.dparams, self.dtype, keep_override=model)
        handle = pipeline.build_net(self.net, layers, self.batch, self.dtype, tune=True)
        task_of, n_tasks = handle.task_table()
        lt = handle.layer_times(self.x, iters=10)
        shp = synth.shapes(self.net, model)
        members: List[List[int]] = [[] for _ in range(n_tasks)]
        for i, t in enumerate(task_of):
            if t >= 0:
                members[t].append(i)
        # a task's execution time: the mean over its subgraphs' measured times
        times = [sum(lt[i] for i in m) / len(m) for m in members]
        order, impact = B.cprune_order_tasks(times, [len(m) for m in members])
        # a task's identity is the key the library groups by (shape, stride, padding, activation,
        # shortcut, layout): the same from model to model as long as the task's shape is untouched
        keys = [handle.task_key(m[0]) for m in members]
        out = handle.forward(self.x)
        for _ in range(5):
            handle.forward(self.x, out)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(self.steps):
            handle.forward(self.x, out)
        torch.cuda.synchronize()
        ms = (time.perf_counter() - t0) / self.steps * 1e3
        table = {}
        for t, m in enumerate(members):
            v = handle.layer_variant(m[0])
            # kernels without tile variants (first layer, fused depthwise + 1x1) work on 16-filter blocks
            step = B.cprune_variant_prune_step(v, shp[m[0]][1]) if v >= 0 else 16
            table[keys[t]] = (m, {"variant": v, "c_out": shp[m[0]][1], "time_ms": times[t], "impact": impact[t],
                                  "step": step})
        handle.close()
        st = {"table": table, "order": [keys[t] for t in order], "ms": ms}
        self._cache[key] = st
        self.trace.append((dict(model), table, st["order"], ms))
        return st

    def tune(self, model):
        st = self._state(model)
        return st["table"], st["order"]

    def measure(self, model) -> float:
        return self._state(model)["ms"]

    def prune(self, model, task, subgraphs, program) -> Optional[Dict[int, int]]:
        """Every prunable subgraph of the task loses the number of filters the program's
        structure gives (Section 3.5); None when no subgraph of the task can lose any."""
        cand = dict(model)
        changed = False
        for i in subgraphs:
            if i not in cand:
                continue              # not prunable in this workload (stem, block outputs, fc)
            cut = B.cprune_prune_count(cand[i], program["step"])
            if cut > 0:
                cand[i] -= cut
                changed = True
        return cand if changed else None


def run(net_name="vgg16", batch=64, dtype=B.F32, alpha=0.95, beta=0.98, a_goal=0.0, iterations=4,
        accuracy: Optional[Callable] = None):
    net, cid = {"vgg16": (synth.vgg16(10, 32), 2), "resnet18": (synth.resnet18(1000, 224), 3),
                "mobilenetv2": (synth.mobilenetv2(1000, 224), 4),
                "mnasnet": (synth.mnasnet(1000, 224), 6)}[net_name]
    params = synth.layer_params(net, cid)
    ds = DeviceSearch(net, params, cid, batch, dtype)
    model = ds.initial_model(params)
    acc = accuracy or (lambda m: 1.0)
    final, log = run_search(model, a_goal, alpha, beta, ds.tune, ds.prune, ds.measure, acc,
                            max_iterations=iterations)
    return ds, model, final, log


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--net", default="vgg16", choices=["vgg16", "resnet18", "mobilenetv2", "mnasnet"])
    ap.add_argument("--batch", type=int, default=64)
    ap.add_argument("--iterations", type=int, default=4)
    ap.add_argument("--beta", type=float, default=0.98)
    args = ap.parse_args()
    ds, start, final, log = run(args.net, args.batch, iterations=args.iterations, beta=args.beta)
    table, order = ds.tune(start)
    print(json.dumps({"start_ms": round(ds.measure(start), 4), "tasks_by_impact": [
        {"task": list(map(str, t)), "layers": table[t][0], **{k: (round(v, 5) if isinstance(v, float) else v)
                                                             for k, v in table[t][1].items()}} for t in order]}))
    for task, l_m, l_t, a_s, verdict in log:
        print(json.dumps({"task": list(map(str, task)), "l_m": None if l_m is None else round(l_m, 4),
                          "l_t": round(l_t, 4), "verdict": verdict}))
    print(json.dumps({"final_ms": round(ds.measure(final), 4), "kept": [final[i] for i in sorted(final)]}))


if __name__ == "__main__":
    main()
