"""Pins for the slot-table oracle (CPU only): a hand-traced sequence and an independent
ordered-list model of least-recently-used replacement."""
import os

import numpy as np
import pytest

import oracle
from conftest import GOLDEN


def parse_trace(path):
    n_slots = n_pages = None
    calls = []
    with open(path) as f:
        for line in f:
            line = line.split("#", 1)[0].strip()
            if not line:
                continue
            if line.startswith("n_slots:"):
                n_slots = int(line.split(":")[1])
                continue
            if line.startswith("n_pages:"):
                n_pages = int(line.split(":")[1])
                continue
            assert line.startswith("call:")
            body, rest = line[5:].split("->")
            in_use, reqs = body.split("|")
            expect, state = rest.split("state:")
            pages = None
            if "pages:" in state:
                state, pages = state.split("pages:")
                pages = [int(v) for v in pages.split()]
            in_use = [int(v) for v in in_use.split()]
            reqs = [tuple(int(v) for v in r.split(":")) for r in reqs.split()]
            expect = expect.strip()
            exp = None if expect == "X" else [(int(e.split(":")[0]), bool(int(e.split(":")[1]))) for e in expect.split()]
            state = [int(v) for v in state.split()]
            calls.append((in_use, reqs, exp, state) if pages is None else (in_use, reqs, exp, state, pages))
    return (n_slots, calls) if n_pages is None else (n_slots, n_pages, calls)


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


# ---- the slot table over a pool of pages ----
def test_hand_traced_sequence_with_pages():
    n_slots, n_pages, calls = parse_trace(os.path.join(GOLDEN, "page_trace.txt"))
    tab = oracle.PagedSlotTable(n_slots, n_pages)
    for in_use, reqs, exp, state, pages in calls:
        if exp is None:
            with pytest.raises(oracle.SlotsExhausted):
                tab.load(reqs, in_use)
        else:
            assert tab.load(reqs, in_use) == exp
        assert tab.adapter == state
        assert tab.first_page == pages


def _check_pool(tab):
    used = 0
    for s in range(tab.n_slots):
        k = tab.rank[s] // 8 if tab.adapter[s] >= 0 else 0
        if k == 0:
            assert tab.first_page[s] == -1
            continue
        p = tab.first_page[s]
        assert 0 <= p and p + k <= tab.n_pages
        assert tab.owner[p:p + k] == [s] * k                 # its run, whole and its own
        used += k
    assert sum(o >= 0 for o in tab.owner) == used            # nobody else holds a page


@pytest.mark.parametrize("seed", range(6))
def test_pool_invariants_on_random_sequences(seed):
    rng = np.random.default_rng(seed)
    n_slots, n_pages, n_ids = 6, int(rng.integers(6, 20)), 24
    tab = oracle.PagedSlotTable(n_slots, n_pages)
    for _ in range(400):
        ads = rng.choice(n_ids, size=int(rng.integers(1, 4)), replace=False)
        reqs = [(int(a), int(rng.choice([0, 8, 16, 32])), int(rng.integers(0, n_slots)) if rng.random() < 0.1 else -1)
                for a in ads]
        in_use = [int(v) for v in rng.choice(n_ids, size=int(rng.integers(0, 5)), replace=False)]
        before = (list(tab.adapter), list(tab.first_page), list(tab.owner), tab.tick)
        try:
            res = tab.load(reqs, in_use)
        except oracle.SlotsExhausted:
            assert (tab.adapter, tab.first_page, tab.owner, tab.tick) == before     # undone as a whole
            continue
        _check_pool(tab)
        for (aid, rank, want), (s, copied) in zip(reqs, res):
            assert want < 0 or s == want
        # an adapter of in_use that was resident before the call and is not named by it is still where it was
        named = {r[0] for r in reqs}
        for a in in_use:
            if a in before[0] and a not in named:
                s = before[0].index(a)
                forced = any(w == s for (_, _, w) in reqs)
                assert forced or (tab.adapter[s] == a and tab.first_page[s] == before[1][s])


@pytest.mark.parametrize("seed", range(4))
def test_a_pool_that_never_fills_is_the_plain_slot_table(seed):
    # A pool so large that a free run of the largest size (4 pages) always exists: the other n_slots - 1 adapters hold
    # at most 16 of the 40 pages and cut the rest into at most 5 gaps, one of which has more than 3 pages.  Pages then
    # never force anyone out, so slots, copies and residency are those of the slot table that the hand trace and the
    # recency-list model pin.
    rng = np.random.default_rng(100 + seed)
    n_slots, n_ids = 5, 18
    paged, plain = oracle.PagedSlotTable(n_slots, n_slots * 8), oracle.SlotTable(n_slots)
    for _ in range(400):
        ads = rng.choice(n_ids, size=int(rng.integers(1, 4)), replace=False)
        reqs = [(int(a), int(rng.choice([0, 8, 16, 32])), int(rng.integers(0, n_slots)) if rng.random() < 0.1 else -1)
                for a in ads]
        in_use = [int(v) for v in rng.choice(n_ids, size=int(rng.integers(0, 6)), replace=False)]
        try:
            want = plain.load(reqs, in_use)
        except oracle.SlotsExhausted:
            with pytest.raises(oracle.SlotsExhausted):
                paged.load(reqs, in_use)
        else:
            assert paged.load(reqs, in_use) == want
        assert paged.adapter == plain.adapter and paged.last_used == plain.last_used
        _check_pool(paged)
