"""CPU checker for the adapter placement step (paper Sec. 7: the greedy caching algorithm, Alg. 1, with its
feasibility test, Alg. 2).  TEST INFRASTRUCTURE ONLY: nothing in the product path imports this module, and it
shares no code with the library's own implementation.

The method is a heuristic, so this file takes its steps in the paper's order and names:

* ``priority_sorting``  - adapters by size, largest first; inside a group of equal size by arrival rate in
  zigzag order (highest, lowest, second highest, second lowest, ...).
* ``greedy``  - adapters leave the sorted queue one by one and are provisionally included in the GPU at the head of
  the GPU queue; when that GPU's adapter count reaches a testing point the provisional set is tested: on success
  it is committed, A_max[g] takes the tested configuration and the GPU stays at the head of the queue; on failure
  the provisional set is rolled back into the adapter queue and the GPU leaves the queue.  An adapter with no GPU
  left, or a failing test of what is still provisional when the queue is empty, raises ``Starvation``.
* ``test_allocation``  - predicted throughput under the GPU's current A_max and under the next candidate of the
  same list of counts; the better one is kept; the allocation is rejected if starvation is predicted for it.

The two predictors (the paper's ML models) are inputs: callables (sizes, rates, a_max) -> throughput and
(sizes, rates, a_max) -> bool, given the sizes and rates of every adapter on the GPU (committed first, then
provisional, each in the order it arrived).

Readings where the pseudocode is silent: a GPU that has no configuration yet (A_max = 0) takes the first candidate
without a comparison; the candidate after the last of the list is the last itself; ties in a sort are broken by
adapter index; rolled-back adapters re-enter the queue at their place in the priority order.

Pins (tests, CPU only): a hand-worked sorting example, hand-worked runs with a predictor that allows a fixed number
of adapters per GPU (fill counts, the GPU that closes, the error cases), the A_max walk under a throughput curve with
a known peak, and validity of the result on random inputs.
"""
from __future__ import annotations

from collections import deque
from typing import Callable, List, Sequence, Tuple

TESTING_POINTS = (8, 16, 32, 64, 96, 128, 160, 192, 256, 320, 384)


class Starvation(Exception):
    """No starvation-free allocation was found (paper Sec. 7)."""


def priority_sorting(size: Sequence[int], rate: Sequence[float]) -> List[int]:
    order: List[int] = []
    for s in sorted(set(size), reverse=True):
        group = sorted((a for a in range(len(size)) if size[a] == s), key=lambda a: (-rate[a], a))
        lo, hi, take_high = 0, len(group) - 1, True
        while lo <= hi:
            if take_high:
                order.append(group[lo])
                lo += 1
            else:
                order.append(group[hi])
                hi -= 1
            take_high = not take_high
    return order


def next_gpu_config(p: int) -> int:
    for t in TESTING_POINTS:
        if t > p:
            return t
    return TESTING_POINTS[-1]


def test_allocation(alloc: Sequence[int], prov: Sequence[int], size, rate, p: int,
                    predict_throughput: Callable, predict_starvation: Callable) -> Tuple[bool, List[int], int]:
    p_next = next_gpu_config(p)
    everyone = list(alloc) + list(prov)
    sizes = [size[a] for a in everyone]
    rates = [rate[a] for a in everyone]
    if p == 0:
        p_best = p_next
    else:
        t_now = predict_throughput(sizes, rates, p)
        t_next = predict_throughput(sizes, rates, p_next)
        p_best = p if t_now > t_next else p_next
    if predict_starvation(sizes, rates, p_best):
        return False, [], 0
    return True, list(prov), p_best


def greedy(n_gpus: int, size: Sequence[int], rate: Sequence[float], predict_throughput: Callable,
           predict_starvation: Callable) -> Tuple[List[int], List[int]]:
    """Returns (g[a] for every adapter, A_max[g] for every GPU; 0 for a GPU left empty)."""
    n = len(size)
    g_of = [-1] * n
    a_max = [0] * n_gpus
    order = priority_sorting(size, rate)
    place = {a: k for k, a in enumerate(order)}
    a_q = deque(order)
    g_q = deque(range(n_gpus))
    alloc: List[List[int]] = [[] for _ in range(n_gpus)]
    prov: List[List[int]] = [[] for _ in range(n_gpus)]

    def commit(g: int, alloc_set: List[int], p_new: int) -> None:
        alloc[g] += prov[g]
        prov[g] = []
        for a in alloc_set:
            g_of[a] = g
        a_max[g] = p_new

    while a_q:
        a = a_q.popleft()
        if not g_q:
            raise Starvation("no GPU left for adapter %d" % a)
        g = g_q.popleft()
        prov[g].append(a)
        if len(alloc[g]) + len(prov[g]) in TESTING_POINTS:
            ok, alloc_set, p_new = test_allocation(alloc[g], prov[g], size, rate, a_max[g], predict_throughput,
                                                   predict_starvation)
            if ok:
                commit(g, alloc_set, p_new)
                g_q.appendleft(g)
            else:
                un_alloc = prov[g]
                prov[g] = []
                a_q = deque(sorted(list(a_q) + un_alloc, key=lambda b: place[b]))
        else:
            g_q.appendleft(g)
    for g in range(n_gpus):
        if prov[g]:
            ok, alloc_set, p_new = test_allocation(alloc[g], prov[g], size, rate, a_max[g], predict_throughput,
                                                   predict_starvation)
            if not ok:
                raise Starvation("GPU %d cannot take its last %d adapters" % (g, len(prov[g])))
            commit(g, alloc_set, p_new)
    return g_of, a_max
