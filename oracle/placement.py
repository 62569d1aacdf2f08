"""CPU checker for the adapter placement step (paper Sec. 7: greedy caching over GPUs with a feasibility test at
fixed adapter counts).  TEST INFRASTRUCTURE ONLY: nothing in the product path imports this module, and it shares
no code with the library's own implementation.

The paper gives the method as a queue-driven procedure.  This file does not replay that procedure; it states what
the procedure's result *is* and computes it from that statement, GPU by GPU:

* Adapters are ranked once (``priority_order``): by size, largest first; adapters of one size by arrival rate,
  alternating between the high end and the low end of what is left (highest, lowest, second highest, ...).
* Rolled-back adapters return to the front of the ranked sequence and a GPU only ever takes from its front, so the
  adapters of one GPU are a contiguous stretch of the ranking and the GPUs are used in index order.  What one GPU
  ends up with therefore depends only on the part of the ranking that is still unplaced (``fill_gpu``): it grows
  through the checkpoint counts 8, 16, ..., 384; at each checkpoint the first `count` unplaced adapters are judged
  as a set; the GPU keeps the largest checkpoint that was judged free of starvation before the first one that was
  not, and after a failed judgement takes nothing more.  If every checkpoint up to the number of unplaced adapters
  passes, the GPU also takes the remainder, which is judged once as a whole; failing that judgement, or running
  out of GPUs, means no starvation-free placement exists under this method (``Starvation``).
* Each judgement also moves the GPU's configuration A_max (``choose_config``): the candidate is the next count of
  the checkpoint list above the current A_max; the GPU keeps whichever of the two the throughput predictor rates
  higher for the judged set (the candidate on a tie or when there is no current one), and the starvation predictor
  is asked about the set under that choice.

``check`` is the converse: given any placement it verifies those properties one by one, without building the
placement itself.  The tests run it on this file's own results and on the library's.

The two predictors (the paper trains ML models for them) are inputs: callables (sizes, rates, a_max) -> throughput
and (sizes, rates, a_max) -> bool, given the sizes and rates of the judged set in ranking order.

Readings where the paper is silent: a GPU without a configuration takes the first candidate without a comparison;
the candidate above the last checkpoint is the last checkpoint; ties in a ranking go to the lower adapter index.

Pins (tests, CPU only): a hand-worked ranking example, hand-worked runs with a predictor that allows a fixed number
of adapters per GPU (fill counts, the GPU that closes, the error cases), the A_max walk under a throughput curve with
a known peak, the order in which the predictors see the adapters, and ``check`` on random inputs (including that it
rejects perturbed placements).
"""
from __future__ import annotations

from typing import Callable, List, Sequence, Tuple

TESTING_POINTS = (8, 16, 32, 64, 96, 128, 160, 192, 256, 320, 384)


class Starvation(Exception):
    """No starvation-free allocation was found (paper Sec. 7)."""


def priority_order(size: Sequence[int], rate: Sequence[float]) -> List[int]:
    """Ranking of the adapters: position k of a size group of m adapters, sorted by falling rate, holds the
    (k/2)-th from the top when k is even and the (k/2)-th from the bottom when k is odd."""
    ranking: List[int] = []
    for s in sorted(set(size), reverse=True):
        falling = sorted((a for a in range(len(size)) if size[a] == s), key=lambda a: (-rate[a], a))
        m = len(falling)
        ranking += [falling[k // 2] if k % 2 == 0 else falling[m - 1 - k // 2] for k in range(m)]
    return ranking


def candidate_after(a_max: int) -> int:
    higher = [c for c in TESTING_POINTS if c > a_max]
    return higher[0] if higher else TESTING_POINTS[-1]


def choose_config(sizes, rates, a_max: int, predict_throughput: Callable) -> int:
    cand = candidate_after(a_max)
    if a_max == 0:
        return cand
    return a_max if predict_throughput(sizes, rates, a_max) > predict_throughput(sizes, rates, cand) else cand


def fill_gpu(sizes: Sequence[int], rates: Sequence[float], predict_throughput: Callable,
             predict_starvation: Callable) -> Tuple[int, int, bool]:
    """One GPU facing the unplaced adapters (sizes / rates in ranking order).  Returns (how many of them it keeps,
    its A_max, whether it is closed).  Raises Starvation when the judgement of the remainder fails."""
    kept, a_max = 0, 0
    stops = [c for c in TESTING_POINTS if c <= len(sizes)]
    if len(sizes) not in stops:
        stops.append(len(sizes))                      # the remainder, judged once everything else is placed
    for count in stops:
        choice = choose_config(sizes[:count], rates[:count], a_max, predict_throughput)
        if predict_starvation(sizes[:count], rates[:count], choice):
            if count not in TESTING_POINTS:
                raise Starvation("the last %d adapters do not fit their GPU" % (count - kept))
            return kept, a_max, True
        kept, a_max = count, choice
    return kept, a_max, False


def place(n_gpus: int, size: Sequence[int], rate: Sequence[float], predict_throughput: Callable,
          predict_starvation: Callable) -> Tuple[List[int], List[int]]:
    """Returns (GPU of every adapter, A_max of every GPU; 0 for a GPU that holds nothing)."""
    ranking = priority_order(size, rate)
    gpu_of = [-1] * len(size)
    a_max = [0] * n_gpus
    first = 0                                         # ranking[first:] is unplaced
    for g in range(n_gpus):
        if first == len(ranking):
            break
        rest = ranking[first:]
        kept, a_max[g], _ = fill_gpu([size[a] for a in rest], [rate[a] for a in rest], predict_throughput,
                                     predict_starvation)
        for a in rest[:kept]:
            gpu_of[a] = g
        first += kept
    if first < len(ranking):
        raise Starvation("no GPU left for adapter %d" % ranking[first])
    return gpu_of, a_max


def check(n_gpus: int, size: Sequence[int], rate: Sequence[float], predict_throughput: Callable,
          predict_starvation: Callable, gpu_of: Sequence[int], a_max: Sequence[int]) -> None:
    """Asserts that (gpu_of, a_max) has the properties the method's result must have; builds nothing."""
    n = len(size)
    ranking = priority_order(size, rate)
    assert len(gpu_of) == n and len(a_max) == n_gpus
    assert all(0 <= g < n_gpus for g in gpu_of)
    along = [gpu_of[a] for a in ranking]
    assert along == sorted(along), "a GPU's adapters must be one stretch of the ranking, GPUs in index order"
    first = 0
    for g in range(n_gpus):
        count = along.count(g)
        rest = ranking[first:]
        sz, rt = [size[a] for a in rest], [rate[a] for a in rest]
        last_gpu_with_work = first + count == n
        # the walk of A_max over the checkpoints this GPU passed, and that each of them was free of starvation
        walk = 0
        passed = [c for c in TESTING_POINTS if c <= count]
        if count and count not in TESTING_POINTS:
            assert last_gpu_with_work, "only the GPU that takes the end of the ranking holds an off-checkpoint count"
            assert passed == [c for c in TESTING_POINTS if c <= len(rest)]
            passed.append(count)
        for c in passed:
            walk = choose_config(sz[:c], rt[:c], walk, predict_throughput)
            assert not predict_starvation(sz[:c], rt[:c], walk), (g, c)
        assert a_max[g] == walk, (g, a_max[g], walk)
        # a GPU that stopped short of the unplaced adapters did so because its next checkpoint was judged to starve
        if not last_gpu_with_work and first < n:
            nxt = [c for c in TESTING_POINTS if c > count]
            assert nxt and nxt[0] <= len(rest), (g, count)
            choice = choose_config(sz[:nxt[0]], rt[:nxt[0]], walk, predict_throughput)
            assert predict_starvation(sz[:nxt[0]], rt[:nxt[0]], choice), (g, count)
        first += count
    assert first == n
