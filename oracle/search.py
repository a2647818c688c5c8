"""CPU oracle of the search-side rules of the method (test infrastructure only; the product
path never imports this): how many filters to prune from the structure of a tuned program
(Section 3.5), the task / subgraph table (Section 3.4), task ordering by pruning impact
(Section 3.3) and the control flow of Algorithm 1 (Section 3.2) over caller-supplied tuning,
latency and accuracy functions.  Plain Python, written from the text; every function says
which passage it follows and which reading it takes where the text leaves a choice.

Pins (tests/test_oracle_search.py): the two worked step sizes of Section 3.5 (32 and 4), the
worked impacts and order of Section 3.3 (1.908, 1.419, 1.632 -> T1, T3, T2), brute force over
box arrangements, and hand-traced runs of the loop.
"""

from __future__ import annotations

from math import gcd
from typing import Callable, Dict, Hashable, List, Optional, Sequence, Tuple


# ---- Section 3.5: number of filters to prune ------------------------------------

def min_prunable(factors: Sequence[int]) -> int:
    """Smallest number of filters whose removal keeps an iterator's split structure.

    The iterator over the filters is split into `factors` (their product is the filter
    count); the filters are arranged as a box with these side lengths.  Shrinking the side
    of length l by one removes product / l filters; the smallest such number over all sides
    is what the section takes per iterator (equivalently product / max side)."""
    if not factors or any(f < 1 for f in factors):
        raise ValueError("factors must be positive")
    prod = 1
    for f in factors:
        prod *= f
    return min(prod // l for l in factors)


def lcm_step(l1: Sequence[int], l2: Sequence[int]) -> int:
    """Minimum number of filters to prune for a program whose two filter iterators (the
    reduction loop's and the output stage's) are split as l1 and l2: the least common
    multiple of the two per-iterator minima (the displayed equation of Section 3.5)."""
    a, b = min_prunable(l1), min_prunable(l2)
    return a // gcd(a, b) * b


def prune_count(c_out: int, step: int) -> int:
    """How many of c_out filters to prune in one iteration for a step size `step`.

    Reading: the section prunes `step` filters from counts the structure divides; pruned
    layers reach counts it does not divide, so the count taken here is the one that brings
    the layer to the next lower multiple of `step` (exactly `step` when c_out is a multiple).
    0 when that would leave no filter."""
    if c_out < 1 or step < 1:
        raise ValueError("positive arguments only")
    keep = (c_out - 1) // step * step
    return c_out - keep if keep >= 1 else 0


# ---- Section 3.4: tasks and their subgraphs -------------------------------------

def task_table(subgraph_keys: Sequence[Optional[Hashable]]) -> Tuple[List[int], List[List[int]]]:
    """Groups subgraphs (conv layers) into tasks: two subgraphs with the same properties
    (shapes, stride, padding, activation, shortcut) are the same task.  `subgraph_keys[i]`
    is layer i's property tuple, or None for a layer that is no tunable subgraph.
    Returns (task of each layer or -1, list of layers per task); tasks are numbered in order
    of first appearance (reading: the text fixes no numbering)."""
    ids: Dict[Hashable, int] = {}
    task_of: List[int] = []
    members: List[List[int]] = []
    for i, key in enumerate(subgraph_keys):
        if key is None:
            task_of.append(-1)
            continue
        if key not in ids:
            ids[key] = len(members)
            members.append([])
        task_of.append(ids[key])
        members[ids[key]].append(i)
    return task_of, members


# ---- Section 3.3: task ordering --------------------------------------------------

def pruning_impact(exec_time: Sequence[float], n_subgraphs: Sequence[int]) -> List[float]:
    """Impact of a task = its execution time x the number of subgraphs that map to it."""
    return [float(t) * int(n) for t, n in zip(exec_time, n_subgraphs)]


def order_tasks(exec_time: Sequence[float], n_subgraphs: Sequence[int]) -> List[int]:
    """Task indices by descending pruning impact (reading: equal impacts keep index order)."""
    imp = pruning_impact(exec_time, n_subgraphs)
    return sorted(range(len(imp)), key=lambda i: (-imp[i], i))


# ---- Section 3.2: Algorithm 1 ----------------------------------------------------

def algorithm1(model, a_goal: float, alpha: float, beta: float,
               tune: Callable, prune: Callable, measure: Callable, accuracy: Callable,
               max_iterations: int = 10 ** 6):
    """Control flow of Algorithm 1 over caller-supplied pieces.

    tune(model) -> (table, order): table maps a task to (its subgraphs, its fastest
        program); order is the tasks by descending pruning impact.
    prune(model, task, subgraphs, program) -> candidate model, or None when the program's
        step leaves nothing to prune from these subgraphs.
    measure(model) -> execution time of the compiled aggregate of tuned tasks.
    accuracy(model) -> (short-term) accuracy.

    Readings: the initial target time is beta x the tuned input model's time and the initial
    a_p its accuracy (the text only says they are initialised); a task whose subgraphs cannot
    be pruned any further is dropped from the list like one that fails the accuracy test;
    the text says a task that failed the accuracy test is not considered again in the rest of
    the search while the listing replaces the list by the candidate's on acceptance: both hold
    here, tasks dropped earlier are filtered out of every later list (tasks are therefore
    identified by their property tuples, which stay the same from one model to the next);
    when a pass over the whole list accepts no candidate and drops no task the search ends
    (the listing would repeat the identical pass forever).

    Returns (final model, log) where log lists per candidate
    (task, l_m, l_t, a_s or None, verdict in {'slow', 'inaccurate', 'accepted', 'exhausted'})."""
    table, order = tune(model)
    remaining = list(order)
    l_t = beta * measure(model)
    a_p = accuracy(model)
    log = []
    banned = set()
    iterations = 0
    while a_p > a_goal and remaining and iterations < max_iterations:
        iterations += 1
        accepted = False
        dropped = False
        for task in list(remaining):
            subgraphs, program = table[task]
            candidate = prune(model, task, subgraphs, program)
            if candidate is None:
                remaining.remove(task)
                banned.add(task)
                dropped = True
                log.append((task, None, l_t, None, "exhausted"))
                continue
            cand_table, cand_order = tune(candidate)
            l_m = measure(candidate)
            if l_m >= l_t:
                log.append((task, l_m, l_t, None, "slow"))
                continue
            a_s = accuracy(candidate)
            if a_s < alpha * a_p:
                remaining.remove(task)
                banned.add(task)
                dropped = True
                log.append((task, l_m, l_t, a_s, "inaccurate"))
                continue
            log.append((task, l_m, l_t, a_s, "accepted"))
            model, table = candidate, cand_table
            remaining = [t for t in cand_order if t not in banned]
            l_t = beta * l_m
            a_p = a_s
            accepted = True
            break
        if not accepted and not dropped:
            break
    return model, log
