"""Pins for the segment-map oracle (CPU only)."""
import itertools

import numpy as np
import pytest

import oracle


def _brute_sorted_perm(slot):
    # position of token t = #{u : slot[u] < slot[t]} + #{u < t : slot[u] == slot[t]}
    T = len(slot)
    perm = [0] * T
    for t in range(T):
        pos = sum(1 for u in range(T) if slot[u] < slot[t]) + sum(1 for u in range(t) if slot[u] == slot[t])
        perm[pos] = t
    return perm


def _check_segments(ordered, seg_start, seg_slot, n_seg):
    T = len(ordered)
    assert len(seg_start) == n_seg + 1 and len(seg_slot) == n_seg
    assert seg_start[0] == 0 and seg_start[n_seg] == T
    for g in range(n_seg):
        a, b = seg_start[g], seg_start[g + 1]
        assert b > a
        assert all(ordered[m] == seg_slot[g] for m in range(a, b))
        if g + 1 < n_seg:
            assert seg_slot[g + 1] != seg_slot[g]


def test_hand_example_sorted():
    # ids:   5  2 -1  5  7  2  5      id2slot: 2->0, 5->3, 7->1
    ids = np.array([5, 2, -1, 5, 7, 2, 5], dtype=np.int32)
    id2slot = np.full(8, -1, dtype=np.int32)
    id2slot[2], id2slot[5], id2slot[7] = 0, 3, 1
    perm, seg_start, seg_slot, n_seg, flags = oracle.bucket(ids, id2slot, oracle.SORTED)
    assert perm.tolist() == [2, 1, 5, 4, 0, 3, 6]
    assert seg_start.tolist() == [0, 1, 3, 4, 7]
    assert seg_slot.tolist() == [-1, 0, 1, 3]
    assert n_seg == 4 and flags == 0


def test_hand_example_runs():
    ids = np.array([5, 5, 2, 2, 2, -1, 5, 7], dtype=np.int32)
    id2slot = np.full(8, -1, dtype=np.int32)
    id2slot[2], id2slot[5], id2slot[7] = 0, 3, 1
    perm, seg_start, seg_slot, n_seg, flags = oracle.bucket(ids, id2slot, oracle.RUNS)
    assert perm.tolist() == list(range(8))
    assert seg_start.tolist() == [0, 2, 5, 6, 7, 8]
    assert seg_slot.tolist() == [3, 0, -1, 3, 1]
    assert n_seg == 5 and flags == 0


def test_exhaustive_small_strings():
    id2slot = np.array([2, 0, 1], dtype=np.int32)          # adapter id -> slot, a non-trivial map
    for T in range(0, 7):
        for ids in itertools.product([-1, 0, 1, 2], repeat=T):
            ids = np.array(ids, dtype=np.int32)
            slot = [(-1 if i < 0 else int(id2slot[i])) for i in ids]
            perm, seg_start, seg_slot, n_seg, flags = oracle.bucket(ids, id2slot, oracle.SORTED)
            assert flags == 0
            assert perm.tolist() == _brute_sorted_perm(slot)
            ordered = [slot[m] for m in perm]
            assert ordered == sorted(ordered)
            _check_segments(ordered, seg_start.tolist(), seg_slot.tolist(), n_seg)
            assert seg_slot.tolist() == sorted(set(slot))
            perm, seg_start, seg_slot, n_seg, flags = oracle.bucket(ids, id2slot, oracle.RUNS)
            assert perm.tolist() == list(range(T))
            _check_segments(slot, seg_start.tolist(), seg_slot.tolist(), n_seg)
            assert n_seg == sum(1 for m in range(T) if m == 0 or slot[m] != slot[m - 1])


@pytest.mark.parametrize("T,n_slots,seed", [(1, 1, 0), (64, 4, 1), (65, 33, 2), (1000, 384, 3), (4097, 7, 4)])
def test_random_properties(T, n_slots, seed):
    rng = np.random.default_rng(seed)
    n_ids = n_slots + 5
    id2slot = np.full(n_ids, -1, dtype=np.int32)
    chosen = rng.permutation(n_ids)[:n_slots]
    id2slot[chosen] = rng.permutation(n_slots)
    ids = rng.choice(np.concatenate([chosen, [-1]]), size=T).astype(np.int32)
    perm, seg_start, seg_slot, n_seg, flags = oracle.bucket(ids, id2slot, oracle.SORTED)
    assert flags == 0
    assert sorted(perm.tolist()) == list(range(T))
    slot = np.where(ids < 0, -1, id2slot[np.maximum(ids, 0)])
    ordered = slot[perm]
    assert np.all(np.diff(ordered) >= 0)
    same = ordered[1:] == ordered[:-1]
    assert np.all(perm[1:][same] > perm[:-1][same])        # stability
    assert (np.diff(seg_start) > 0).all() and seg_start[-1] == T
    assert np.all(np.diff(seg_slot) > 0)


def test_non_resident_token_is_flagged_and_served_backbone_only():
    id2slot = np.array([0, -1, 1], dtype=np.int32)
    ids = np.array([0, 1, 2, 7], dtype=np.int32)            # 1: not resident, 7: unknown id
    perm, seg_start, seg_slot, n_seg, flags = oracle.bucket(ids, id2slot, oracle.SORTED)
    assert flags == oracle.FLAG_NOT_RESIDENT
    assert perm.tolist() == [1, 3, 0, 2]
    assert seg_slot.tolist() == [-1, 0, 1]
