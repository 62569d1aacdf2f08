"""The library's adapter placement (lora_place_adapters, lora_priority_sorting; paper Sec. 7) against the placement
oracle, through the C ABI.  CPU only: the call touches no device.  Integer results: exact equality."""
import os

import numpy as np
import pytest

from conftest import GOLDEN
from oracle import placement as P
from paper_2602_24044_amd import binding as B


def _workload(rng, n):
    size = rng.choice([8, 16, 32, 64], size=n, p=[0.4, 0.3, 0.2, 0.1]).tolist()
    rate = rng.choice([3.2, 1.6, 0.8, 0.4, 0.1, 0.05, 0.025, 0.0125], size=n).tolist()
    return [int(s) for s in size], [float(r) for r in rate]


def _predictors(rng):
    """A family of deterministic stand-ins for the paper's two ML models: a token-rate budget that shrinks with
    the memory the slots take, a throughput curve with a peak in A_max, and a penalty for swapping."""
    budget = float(rng.uniform(3.0, 60.0))
    peak = int(rng.choice(P.TESTING_POINTS))
    mem = float(rng.uniform(0.0, 0.002))

    def thr(sizes, rates, p):
        cap = budget * (1.0 - mem * p * max(sizes) / 8.0)
        swap = max(0, len(sizes) - p) * 0.01
        return min(sum(rates), cap) - swap - 1e-4 * abs(p - peak)

    def starve(sizes, rates, p):
        return thr(sizes, rates, p) < 0.9 * sum(rates)
    return thr, starve


def _both(size, rate, n_gpus, thr, starve):
    try:
        want = P.place(n_gpus, size, rate, thr, starve)
    except P.Starvation:
        want = None
    try:
        got = B.lora_place_adapters(size, rate, n_gpus, thr, starve)
    except B.LoraError as e:
        assert e.status == B.LORA_ERR_STARVATION
        got = None
    return want, got


@pytest.mark.parametrize("seed", range(40))
def test_placement_matches_the_oracle(seed):
    rng = np.random.default_rng(100 + seed)
    n = int(rng.integers(0, 700))
    size, rate = _workload(rng, n)
    thr, starve = _predictors(rng)
    n_gpus = int(rng.integers(1, 24))
    want, got = _both(size, rate, n_gpus, thr, starve)
    assert (want is None) == (got is None)
    if want is not None:
        assert got[0] == want[0]
        assert got[1] == want[1]
        # and the library's result on its own against the properties the method's result must have
        P.check(n_gpus, size, rate, thr, starve, got[0], got[1])


def test_both_outcomes_occur_in_the_random_cases():
    outcomes = set()
    for seed in range(40):
        rng = np.random.default_rng(100 + seed)
        n = int(rng.integers(0, 700))
        size, rate = _workload(rng, n)
        thr, starve = _predictors(rng)
        outcomes.add(_both(size, rate, int(rng.integers(1, 24)), thr, starve)[0] is None)
    assert outcomes == {True, False}


@pytest.mark.parametrize("seed", range(5))
def test_priority_sorting_matches_the_oracle(seed):
    rng = np.random.default_rng(seed)
    size, rate = _workload(rng, int(rng.integers(0, 400)))
    assert B.lora_priority_sorting(size, rate) == P.priority_order(size, rate)


def test_hand_worked_cases_on_the_library():
    kv = dict(l.strip().split(":", 1) for l in open(os.path.join(GOLDEN, "priority_sorting.txt"))
              if l.strip() and not l.startswith("#"))
    size = [int(v) for v in kv["size"].split()]
    rate = [float(v) for v in kv["rate"].split()]
    assert B.lora_priority_sorting(size, rate) == [int(v) for v in kv["order"].split()]
    for line in open(os.path.join(GOLDEN, "placement_capacity.txt")):
        if not line.startswith("case:"):
            continue
        spec, expect = line[len("case:"):].split("->")
        n, g, cap = (int(v) for v in spec.split())
        thr, starve = (lambda s, r, p: float(p)), (lambda s, r, p: len(s) > cap)
        if expect.strip() == "starvation":
            with pytest.raises(B.LoraError) as e:
                B.lora_place_adapters([16] * n, [0.1] * n, g, thr, starve)
            assert e.value.status == B.LORA_ERR_STARVATION
        else:
            counts, a_max = ([int(v) for v in part.split()] for part in expect.split("|"))
            gpu_of, got = B.lora_place_adapters([16] * n, [0.1] * n, g, thr, starve)
            assert [gpu_of.count(k) for k in range(g)] == counts and got == a_max


def test_argument_errors():
    ok = (lambda s, r, p: 1.0), (lambda s, r, p: False)
    for size, rate in (([0], [0.1]), ([8], [-1.0]), ([8], [float("nan")]), ([-8], [0.1])):
        with pytest.raises(B.LoraError) as e:
            B.lora_place_adapters(size, rate, 2, *ok)
        assert e.value.status == B.LORA_ERR_INVALID_ARG
    with pytest.raises(B.LoraError) as e:
        B.lora_place_adapters([8], [0.1], -1, *ok)
    assert e.value.status == B.LORA_ERR_INVALID_ARG
    assert B.lora_place_adapters([], [], 3, *ok) == ([], [0, 0, 0])          # nothing to place
    with pytest.raises(B.LoraError) as e:                                      # an adapter and no GPU
        B.lora_place_adapters([8], [0.1], 0, *ok)
    assert e.value.status == B.LORA_ERR_STARVATION


def test_placement_under_the_analytic_serving_model():
    # the stand-in predictors built from the measured laws: sanity of the model and validity of what the greedy
    # algorithm returns under it
    from paper_2602_24044_amd.placement_model import ServingModel, place
    m = ServingModel.from_profile()      # constants of the committed measurement (profiles/latency_law.md)
    assert m.max_requests(32, 8) > m.max_requests(32, 384) > 0            # slots take memory from the KV cache
    assert m.step_seconds(256, 32) > m.step_seconds(256, 1) > m.step_seconds(32, 1)
    light, heavy = [0.1] * 16, [40.0] * 16
    assert m.throughput([16] * 16, light, 16) == pytest.approx(m.incoming_token_rate(light))
    assert not m.starvation([16] * 16, light, 16) and m.starvation([16] * 16, heavy, 16)
    # fewer slots than adapters: loads cost step time once the GPU is the bottleneck
    busy = [6.0] * 64
    assert m.throughput([32] * 64, busy, 8) < m.throughput([32] * 64, busy, 64)
    rng = np.random.default_rng(3)
    n = 1500
    size = [int(v) for v in rng.choice([8, 16, 32], size=n)]
    # rates from the upper part of the paper's set: a GPU is then full well before it holds 384 adapters, the last
    # count at which the algorithm tests an allocation (whatever the measured constants of the day are)
    rate = [float(v) for v in rng.choice([3.2, 1.6, 0.8, 0.4], size=n)]
    gpu_of, a_max = place(size, rate, 32, m)
    assert gpu_of == P.place(32, size, rate, m.throughput, m.starvation)[0]
    P.check(32, size, rate, m.throughput, m.starvation, gpu_of, a_max)
    used = max(gpu_of) + 1
    assert 1 < used <= 32
    for g in range(used):
        mine = [a for a in range(n) if gpu_of[a] == g]
        assert not m.starvation([size[a] for a in mine], [rate[a] for a in mine], a_max[g])
    with pytest.raises(B.LoraError) as e:
        place(size, rate, 1, m)
    assert e.value.status == B.LORA_ERR_STARVATION
