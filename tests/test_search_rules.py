"""The library's host-side search rules (step size from program structure, prune count, task
ordering) against the oracle and the paper's worked examples.  No GPU needed: these entry
points do no device work."""
import os
import random

import pytest

from oracle import search
from paper_2207_01260_amd import binding as B

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "paper_worked_examples.txt")


def golden_rows(tag):
    rows = []
    for line in open(GOLDEN):
        line = line.split("#")[0].split()
        if line and line[0] == tag:
            rows.append(line[1:])
    return rows


def test_worked_examples_through_the_library():
    for l1, l2, want in golden_rows("lcm_step"):
        f1 = [int(v) for v in l1.split("x")]
        f2 = [int(v) for v in l2.split("x")]
        assert B.cprune_lcm_step(f1, f2) == int(want)
    rows = golden_rows("impact")
    order, impact = B.cprune_order_tasks([float(r[1]) for r in rows], [int(r[2]) for r in rows])
    assert [rows[i][0] for i in order] == golden_rows("order")[0]
    for got, r in zip(impact, rows):
        assert abs(got - float(r[3])) < 5e-4


def test_lcm_step_random_against_oracle():
    rng = random.Random(7)
    for _ in range(500):
        l1 = [rng.choice([1, 2, 3, 4, 5, 7, 8, 16, 32, 128]) for _ in range(rng.randint(1, 4))]
        l2 = [rng.choice([1, 2, 3, 4, 6, 8, 9, 16, 64, 512]) for _ in range(rng.randint(1, 4))]
        assert B.cprune_lcm_step(l1, l2) == search.lcm_step(l1, l2)
    for bad in ([], [0], [4, -1]):
        with pytest.raises(B.CPruneError):
            B.cprune_lcm_step(bad, [4])


def test_prune_count_against_oracle():
    for c in range(1, 300):
        for step in (1, 3, 16, 32, 64, 512):
            assert B.cprune_prune_count(c, step) == search.prune_count(c, step)
    with pytest.raises(B.CPruneError):
        B.cprune_prune_count(0, 16)


def test_order_tasks_random_against_oracle():
    rng = random.Random(11)
    for _ in range(200):
        n = rng.randint(0, 12)
        times = [rng.choice([0.25, 0.5, 1.0, 1.5, 2.0, 0.954, 1.632]) for _ in range(n)]
        counts = [rng.randint(0, 4) for _ in range(n)]
        order, impact = B.cprune_order_tasks(times, counts)
        assert order == search.order_tasks(times, counts)
        assert impact == search.pruning_impact(times, counts)


def test_variant_structure_and_step():
    """Every variant: both filter iterators walk (tile, 16-row block); the step is the rule of
    Section 3.5 applied to that box, in units of 16 filters."""
    nv = B.cprune_num_tile_variants()
    for v in range(nv):
        tile_m, _, _ = B.cprune_tile_variant_info(v)
        for c_out in (1, 16, 45, 64, 128, 247, 512):
            ml, ep, unit = B.cprune_variant_filter_splits(v, c_out)
            assert unit in (16, 32) and ml == ep and tile_m % unit == 0
            tiles, blocks = ml
            assert tiles == -(-c_out // tile_m) and blocks == min(tile_m // unit, -(-c_out // unit))
            assert tiles * blocks * unit >= c_out
            step = B.cprune_variant_prune_step(v, c_out)
            assert step == unit * search.lcm_step(ml, ep)
            assert step % 16 == 0
    # a 16-row tile steps by one MFMA block whatever the filter count
    v16 = next(v for v in range(nv) if B.cprune_tile_variant_info(v)[0] == 16)
    assert all(B.cprune_variant_prune_step(v16, c) == 16 for c in (16, 100, 128, 512))
    # a 64-row tile on 512 filters is an 8 x 4 box of blocks: the smallest slice is 4 blocks
    v64 = next(v for v in range(nv) if B.cprune_tile_variant_info(v)[0] == 64)
    assert B.cprune_variant_prune_step(v64, 512) == 64
    with pytest.raises(B.CPruneError):
        B.cprune_variant_prune_step(nv, 64)


def test_algorithm1_control_flow_against_oracle():
    """The library's search object (driven by run_search) and the oracle's loop take the same
    decisions on seeded toy models (per-task filter counts, linear latency, accuracy that falls
    with every cut)."""
    from paper_2207_01260_amd import search as psearch
    rng = random.Random(3)
    for trial in range(60):
        n = rng.randint(1, 5)
        lat = [rng.choice([0.01, 0.5, 1.0, 2.0]) for _ in range(n)]
        cost = [rng.choice([0.0, 0.5, 3.0, 25.0]) for _ in range(n)]
        steps = [rng.choice([4, 16, 32]) for _ in range(n)]
        start = tuple(rng.choice([48, 64, 100, 128]) for _ in range(n))
        alpha, beta = rng.choice([0.8, 0.95, 0.99]), rng.choice([0.5, 0.9, 0.98, 0.999])
        goal = rng.choice([0.0, 60.0, 85.0])

        def acc(m):
            return 90.0 - sum(cost[t] * (start[t] - m[t]) / 16.0 for t in range(n))

        def tune(model):
            table = {t: ([t], steps[t]) for t in range(n)}
            return table, search.order_tasks([lat[t] * model[t] for t in range(n)], [1] * n)

        def prune(model, task, subgraphs, program):
            cut = search.prune_count(model[task], program)
            if cut == 0:
                return None
            m = list(model)
            m[task] -= cut
            return tuple(m)

        def measure(model):
            return sum(lat[t] * model[t] for t in range(n))

        want = search.algorithm1(start, goal, alpha, beta, tune, prune, measure, acc)
        got = psearch.run_search(start, goal, alpha, beta, tune, prune, measure, acc)
        assert got[0] == want[0], trial
        assert got[1] == want[1], trial


def test_search_object_rejects_calls_out_of_order():
    s = B.Search(0.0, 0.9, 0.9, 10)
    with pytest.raises(B.CPruneError):
        s.next_task()                      # not started
    s.start([7, 3], 1.0, 1.0)
    with pytest.raises(B.CPruneError):
        s.report_exhausted()               # no task handed out
    assert s.next_task() == 7
    with pytest.raises(B.CPruneError):
        s.next_task()                      # a report is due
    with pytest.raises(B.CPruneError):
        s.report_accuracy(1.0, [7, 3])     # latency first
    assert s.report_latency(2.0) is False  # 2.0 >= 0.9: slow, task stays
    assert s.next_task() == 3
    assert s.report_latency(0.5) is True
    with pytest.raises(B.CPruneError):
        s.report_exhausted()               # accuracy is due
    assert s.report_accuracy(0.95, [3, 7]) is True
    assert s.next_task() == 3              # the accepted model's list from its head
    s.report_exhausted()
    assert s.next_task() == 7
    assert s.report_latency(0.44) is True  # target is now 0.9 * 0.5
    assert s.report_accuracy(0.5, [7]) is False   # 0.5 < 0.9 * 0.95: out for good
    assert s.next_task() is None
    assert [e[4] for e in s.log()] == [1, 3, 4, 2]
    s.close()


def test_search_pass_limit():
    s = B.Search(0.0, 0.0, 2.0, 2)       # beta 2: every candidate passes the gate
    s.start([1], 1.0, 1.0)
    for _ in range(2):
        assert s.next_task() == 1
        assert s.report_latency(1.0)
        assert s.report_accuracy(1.0, [1])
    assert s.next_task() is None
    s.close()
