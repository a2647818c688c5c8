"""Pins of the search-side oracle (oracle/search.py) against what the paper prints and what
the rules mean: the worked step sizes of Section 3.5, the worked impacts and order of
Section 3.3, brute force over box arrangements, and hand-traced runs of Algorithm 1."""
import itertools
import math
import os

import pytest

from oracle import search

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "paper_worked_examples.txt")


def golden_rows(tag):
    rows = []
    for line in open(GOLDEN):
        line = line.split("#")[0].split()
        if line and line[0] == tag:
            rows.append(line[1:])
    return rows


def test_worked_step_sizes():
    rows = golden_rows("lcm_step")
    assert len(rows) == 2
    for l1, l2, want in rows:
        f1 = [int(v) for v in l1.split("x")]
        f2 = [int(v) for v in l2.split("x")]
        assert search.lcm_step(f1, f2) == int(want)
    # the three ways to shrink the 4 x 8 x 16 arrangement remove 8*16, 4*16 or 4*8 filters
    assert sorted(512 // l for l in (4, 8, 16)) == [32, 64, 128]
    assert search.min_prunable([4, 8, 16]) == 32
    assert search.min_prunable([4, 128]) == 4 and search.min_prunable([512, 1]) == 1


def test_min_prunable_is_a_box_slice_by_brute_force():
    """Removing one slice of a box of filters along side d leaves a box again; the smallest
    slice is the smallest count that keeps the structure."""
    for dims in itertools.product([1, 2, 3, 4, 6], repeat=3):
        total = dims[0] * dims[1] * dims[2]
        slices = []
        for d in range(3):
            shrunk = list(dims)
            shrunk[d] -= 1
            slices.append(total - shrunk[0] * shrunk[1] * shrunk[2])
        assert search.min_prunable(dims) == min(slices)
        assert search.min_prunable(dims) == total // max(dims)


def test_lcm_properties():
    for l1 in ([2, 3], [4, 8, 16], [7], [6, 10]):
        for l2 in ([5], [4, 128], [512, 1], [9, 3, 3]):
            s = search.lcm_step(l1, l2)
            a, b = search.min_prunable(l1), search.min_prunable(l2)
            assert s % a == 0 and s % b == 0 and s == math.lcm(a, b)
    assert search.lcm_step([4, 8, 16], [4, 8, 16]) == search.min_prunable([4, 8, 16])
    with pytest.raises(ValueError):
        search.lcm_step([], [4])
    with pytest.raises(ValueError):
        search.lcm_step([4, 0], [4])


def test_prune_count():
    assert search.prune_count(512, 32) == 32          # a multiple: one whole step
    assert search.prune_count(45, 16) == 13           # down to 32
    assert search.prune_count(17, 16) == 1
    assert search.prune_count(16, 16) == 0            # nothing may be left empty
    assert search.prune_count(33, 16) == 1 and search.prune_count(32, 16) == 16
    for c in range(1, 200):
        for s in (1, 4, 16, 32):
            p = search.prune_count(c, s)
            assert 0 <= p <= s and (p == 0 or ((c - p) % s == 0 and c - p >= 1))


def test_worked_task_order():
    rows = golden_rows("impact")
    names = [r[0] for r in rows]
    times = [float(r[1]) for r in rows]
    counts = [int(r[2]) for r in rows]
    imp = search.pruning_impact(times, counts)
    for got, r in zip(imp, rows):
        assert abs(got - float(r[3])) < 5e-4
    order = [names[i] for i in search.order_tasks(times, counts)]
    assert order == golden_rows("order")[0]


def test_order_ties_and_brute_force():
    assert search.order_tasks([1.0, 2.0, 1.0, 0.5], [2, 1, 2, 4]) == [0, 1, 2, 3]
    times = [0.3, 1.7, 0.9, 0.9, 2.0]
    counts = [5, 1, 2, 1, 1]
    order = search.order_tasks(times, counts)
    imp = [t * c for t, c in zip(times, counts)]
    assert all(imp[a] >= imp[b] for a, b in zip(order, order[1:]))
    assert sorted(order) == list(range(5))


def test_task_table():
    keys = [("c", 64, 64), None, ("c", 64, 128), ("c", 64, 64), ("c", 128, 128), ("c", 64, 128), None]
    task_of, members = search.task_table(keys)
    assert task_of == [0, -1, 1, 0, 2, 1, -1]
    assert members == [[0, 3], [2, 5], [4]]


# ---- Algorithm 1 on a toy model: a tuple of per-task filter counts -------------------

def _toy(latency_per_filter, accuracy_of, steps):
    def tune(model):
        table = {t: ([t], steps[t]) for t in range(len(model))}
        times = [latency_per_filter[t] * model[t] for t in range(len(model))]
        return table, search.order_tasks(times, [1] * len(model))

    def prune(model, task, subgraphs, program):
        cut = search.prune_count(model[task], program)
        if cut == 0:
            return None
        m = list(model)
        m[task] -= cut
        return tuple(m)

    def measure(model):
        return sum(latency_per_filter[t] * model[t] for t in range(len(model)))

    return tune, prune, measure, accuracy_of


def test_algorithm1_accepts_in_impact_order_until_accuracy_goal():
    # two tasks; accuracy falls 1 point per 16 filters removed
    acc = lambda m: 90.0 - (64 - m[0]) / 16.0 - (64 - m[1]) / 16.0
    tune, prune, measure, accuracy = _toy([2.0, 1.0], acc, [16, 16])
    final, log = search.algorithm1((64, 64), a_goal=87.5, alpha=0.9, beta=0.99, tune=tune, prune=prune,
                                   measure=measure, accuracy=accuracy)
    verdicts = [(t, v) for t, _, _, _, v in log]
    # task 0 dominates (128 vs 64), then 96 vs 64, then 64 vs 64 (tie -> task 0) ...
    assert verdicts[:3] == [(0, "accepted"), (0, "accepted"), (0, "accepted")]
    assert accuracy(final) <= 87.5 and all(v == "accepted" for _, v in verdicts)
    assert final == (16, 64)


def test_algorithm1_latency_gate_moves_to_next_task():
    # pruning task 0 saves too little to beat beta x previous time; task 1 does
    acc = lambda m: 90.0
    lat = [0.001, 1.0]
    tune, prune, measure, accuracy = _toy(lat, acc, [16, 16])

    def tune_fixed(model):       # list task 0 first regardless, to force the gate
        table, _ = tune(model)
        return table, [0, 1]
    final, log = search.algorithm1((64, 64), a_goal=0.0, alpha=0.9, beta=0.9, tune=tune_fixed, prune=prune,
                                   measure=measure, accuracy=accuracy, max_iterations=1)
    assert [(t, v) for t, _, _, _, v in log] == [(0, "slow"), (1, "accepted")]
    assert final == (64, 48)


def test_algorithm1_drops_inaccurate_task_for_good_and_ends():
    # task 0 is fragile (any cut costs 20 points), task 1 is free
    acc = lambda m: 90.0 - (20.0 if m[0] < 64 else 0.0)
    tune, prune, measure, accuracy = _toy([2.0, 1.0], acc, [16, 16])
    final, log = search.algorithm1((64, 64), a_goal=50.0, alpha=0.95, beta=0.999, tune=tune, prune=prune,
                                   measure=measure, accuracy=accuracy)
    assert log[0][0] == 0 and log[0][4] == "inaccurate"
    assert all(t == 1 for t, *_ in log[1:])                  # never offered again
    assert final[0] == 64 and final[1] == 16                 # task 1 pruned until nothing is left to cut
    assert log[-1][4] == "exhausted"


def test_algorithm1_stops_when_nothing_is_fast_enough():
    acc = lambda m: 90.0
    tune, prune, measure, accuracy = _toy([1.0, 1.0], acc, [16, 16])
    final, log = search.algorithm1((64, 64), a_goal=0.0, alpha=0.9, beta=0.5, tune=tune, prune=prune,
                                   measure=measure, accuracy=accuracy)
    assert final == (64, 64) and [v for *_, v in log] == ["slow", "slow"]
