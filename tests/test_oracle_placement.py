"""Pins for the placement oracle (paper Sec. 7, Alg. 1 / Alg. 2), CPU only: hand-worked fixtures and properties
that hold whatever the predictors say; the property checker is itself pinned by placements it must reject."""
import os

import numpy as np
import pytest

from conftest import GOLDEN
from oracle import placement as P


def _lines(name):
    return [l.strip() for l in open(os.path.join(GOLDEN, name)) if l.strip() and not l.startswith("#")]


def test_priority_sorting_hand_example():
    kv = dict(l.split(":", 1) for l in _lines("priority_sorting.txt"))
    size = [int(v) for v in kv["size"].split()]
    rate = [float(v) for v in kv["rate"].split()]
    assert P.priority_order(size, rate) == [int(v) for v in kv["order"].split()]


def test_priority_sorting_properties():
    rng = np.random.default_rng(1)
    size = rng.choice([8, 16, 32], size=50).tolist()
    rate = rng.choice([3.2, 1.6, 0.8, 0.4, 0.1, 0.05], size=50).tolist()
    order = P.priority_order(size, rate)
    assert sorted(order) == list(range(50))
    assert [size[a] for a in order] == sorted(size, reverse=True)            # size order kept
    for s in set(size):
        r = [rate[a] for a in order if size[a] == s]
        assert r[0] == max(r) and (len(r) < 2 or r[1] == min(r))             # high, low, ...
        assert r[0::2] == sorted(r[0::2], reverse=True) and r[1::2] == sorted(r[1::2])


def _capacity_predictors(cap):
    return (lambda sizes, rates, p: float(p)), (lambda sizes, rates, p: len(sizes) > cap)


@pytest.mark.parametrize("line", [l for l in _lines("placement_capacity.txt") if l.startswith("case:")])
def test_hand_worked_capacity_cases(line):
    spec, expect = line[len("case:"):].split("->")
    n, g, cap = (int(v) for v in spec.split())
    thr, starve = _capacity_predictors(cap)
    if expect.strip() == "starvation":
        with pytest.raises(P.Starvation):
            P.place(g, [16] * n, [0.1] * n, thr, starve)
        return
    counts, a_max = ([int(v) for v in part.split()] for part in expect.split("|"))
    g_of, got_a_max = P.place(g, [16] * n, [0.1] * n, thr, starve)
    assert [g_of.count(k) for k in range(g)] == counts
    assert got_a_max == a_max
    by_priority = [g_of[a] for a in P.priority_order([16] * n, [0.1] * n)]
    assert by_priority == sorted(by_priority)        # the queue order fills GPU 0 first


def test_a_max_walks_up_to_the_peak_of_the_predicted_throughput():
    # throughput peaks at A_max = 32: the tests at 8, 16, 32 adapters take the next candidate, the one at 64 keeps 32
    thr = lambda sizes, rates, p: -abs(p - 32)
    g_of, a_max = P.place(1, [8] * 70, [0.1] * 70, thr, lambda sizes, rates, p: False)
    assert a_max == [32] and set(g_of) == {0}
    # a GPU that stops at 20 adapters was last configured at the test with 16 adapters (8 against 16: 16), and the
    # final test compares 16 with 32
    g_of, a_max = P.place(1, [8] * 20, [0.1] * 20, thr, lambda sizes, rates, p: False)
    assert a_max == [32]
    thr16 = lambda sizes, rates, p: -abs(p - 16)
    assert P.place(1, [8] * 20, [0.1] * 20, thr16, lambda sizes, rates, p: False)[1] == [16]


def test_predictors_see_committed_then_provisional_adapters():
    seen = []
    def starve(sizes, rates, p):
        seen.append((list(sizes), p))
        return False
    size = [32] * 8 + [16] * 8
    P.place(1, size, [0.1] * 16, lambda s, r, p: 1.0 * p, starve)
    assert seen[0] == ([32] * 8, 8)
    assert seen[1] == ([32] * 8 + [16] * 8, 16)


def _random_case(seed):
    rng = np.random.default_rng(seed)
    n = int(rng.integers(1, 300))
    size = rng.choice([8, 16, 32], size=n).tolist()
    rate = rng.choice([3.2, 1.6, 0.8, 0.4, 0.1, 0.05, 0.025], size=n).tolist()
    load_cap = float(rng.uniform(15.0, 80.0))
    thr = lambda sizes, rates, p: min(sum(rates), load_cap) - 0.001 * abs(p - 64)
    starve = lambda sizes, rates, p: sum(rates) > load_cap
    return n, size, rate, thr, starve


@pytest.mark.parametrize("seed", range(12))
def test_result_is_valid_on_random_inputs(seed):
    n, size, rate, thr, starve = _random_case(seed)
    try:
        g_of, a_max = P.place(24, size, rate, thr, starve)
    except P.Starvation:
        return
    assert all(0 <= g < 24 for g in g_of)
    used = sorted(set(g_of))
    assert used == list(range(len(used)))                                   # GPUs are opened in order
    for g in range(24):
        mine = [a for a in range(n) if g_of[a] == g]
        assert (a_max[g] in P.TESTING_POINTS) if mine else a_max[g] == 0
        if mine:
            assert not starve([size[a] for a in mine], [rate[a] for a in mine], a_max[g])
    P.check(24, size, rate, thr, starve, g_of, a_max)


def test_the_property_checker_rejects_what_the_method_cannot_return():
    rejected = 0
    for seed in range(12):
        n, size, rate, thr, starve = _random_case(seed)
        try:
            g_of, a_max = P.place(24, size, rate, thr, starve)
        except P.Starvation:
            continue
        used = max(g_of) + 1
        if used < 2:
            continue
        order = P.priority_order(size, rate)
        first_of_1 = next(a for a in order if g_of[a] == 1)
        last_of_0 = [a for a in order if g_of[a] == 0][-1]
        variants = []
        v = list(g_of); v[first_of_1] = 0; variants.append((v, a_max))                  # GPU 0 takes one adapter too many
        v = list(g_of); v[last_of_0] = 1; variants.append((v, a_max))                   # GPU 0 stops one adapter early
        v = list(g_of); v[order[0]] = 1; variants.append((v, a_max))                    # not a stretch of the ranking
        w = list(a_max); w[0] = P.candidate_after(w[0]) if w[0] < 384 else 320; variants.append((g_of, w))   # wrong A_max
        for cand_g, cand_a in variants:
            with pytest.raises(AssertionError):
                P.check(24, size, rate, thr, starve, cand_g, cand_a)
            rejected += 1
    assert rejected >= 12
