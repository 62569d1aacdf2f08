"""Pins for the slot-table oracle (CPU only): a hand-traced sequence and an independent
ordered-list model of least-recently-used replacement."""
import os

import numpy as np
import pytest

import oracle
from conftest import GOLDEN


def parse_trace(path):
    n_slots = None
    calls = []
    with open(path) as f:
        for line in f:
            line = line.split("#", 1)[0].strip()
            if not line:
                continue
            if line.startswith("n_slots:"):
                n_slots = int(line.split(":")[1])
                continue
            assert line.startswith("call:")
            body, rest = line[5:].split("->")
            in_use, reqs = body.split("|")
            expect, state = rest.split("state:")
            in_use = [int(v) for v in in_use.split()]
            reqs = [tuple(int(v) for v in r.split(":")) for r in reqs.split()]
            expect = expect.strip()
            exp = None if expect == "X" else [(int(e.split(":")[0]), bool(int(e.split(":")[1]))) for e in expect.split()]
            calls.append((in_use, reqs, exp, [int(v) for v in state.split()]))
    return n_slots, calls


def test_hand_traced_sequence():
    n_slots, calls = parse_trace(os.path.join(GOLDEN, "slot_trace.txt"))
    tab = oracle.SlotTable(n_slots)
    for in_use, reqs, exp, state in calls:
        if exp is None:
            with pytest.raises(oracle.SlotsExhausted):
                tab.load(reqs, in_use)
        else:
            assert tab.load(reqs, in_use) == exp
        assert tab.adapter == state


class _RecencyList:
    """Independent model: a recency-ordered list of resident adapters (front = oldest);
    one adapter per call, so ties between equal ages never arise."""

    def __init__(self, n):
        self.n = n
        self.order = []
        self.slot = {}

    def touch(self, a):
        self.order.remove(a)
        self.order.append(a)

    def load(self, a):
        if a in self.slot:
            self.touch(a)
            return self.slot[a], False
        if len(self.order) < self.n:
            s = min(set(range(self.n)) - set(self.slot.values()))
        else:
            victim = self.order.pop(0)
            s = self.slot.pop(victim)
        self.slot[a] = s
        self.order.append(a)
        return s, True


def test_against_recency_list_model():
    rng = np.random.default_rng(0)
    n = 5
    tab = oracle.SlotTable(n)
    ref = _RecencyList(n)
    for _ in range(400):
        a = int(rng.integers(0, 12))
        got = tab.load([(a, 8, -1)])
        assert got == [ref.load(a)]
    m = tab.id2slot(12)
    for a, s in ref.slot.items():
        assert m[a] == s
    assert (m >= 0).sum() == n
