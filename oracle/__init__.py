"""CPU checker ("oracle") for the multi-adapter LoRA serving step.

TEST INFRASTRUCTURE ONLY.  Nothing in the product path imports this package; it
shares no code with the GPU library and never falls back to it or from it.

Three independent definitions live here:

* ``project`` / ``project_at``  - the projection y = x W^T + s_i (x A_i^T) B_i^T in
  IEEE double, plain loops in C (``lora_oracle.c``), tokens indexed directly by
  their adapter id (paper Sec. 2.2, LoRA as two low-rank matrices whose activations
  are added to the backbone layer's output; Sec. 1, adapters kept unmerged).
* ``bucket``  - the token->adapter segment map: the unique stable ascending sort of
  token indices by slot (NumPy's stable argsort is the sorting step) followed by
  run-length encoding; or run-length encoding in token order.
* ``SlotTable``  - the bounded adapter-slot region (paper Sec. 2.2: at most A_max
  adapters resident, uniform slot size S_max, adapters swapped in from CPU memory)
  with least-recently-used replacement, written as an ordered list.

Every function is pinned by CPU-only tests to facts that do not depend on this
code: float64 library matmul for backbone-only batches, the merged-weight
identity, bitwise base-only special cases, hand-computed integer fixtures,
brute-force enumeration for the bucket map, hand-traced slot sequences.
Nothing here is "parity unpinned".
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "lora_oracle.c")
_LIB = os.path.join(_HERE, "_lora_oracle.so")
_lib = None

SORTED = 0
RUNS = 1
FLAG_NOT_RESIDENT = 1


def build(force: bool = False) -> str:
    """Compile the C checker with gcc (-O2, OpenMP, strict IEEE: no fast-math)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-fopenmp", "-fno-fast-math", "-ffp-contract=off", "-shared", "-fPIC",
               "-o", _LIB, _SRC]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        P = ctypes.c_void_p
        lib.lora_oracle_project.restype = ctypes.c_int
        lib.lora_oracle_project.argtypes = [ctypes.c_int32] * 3 + [P, P, P, ctypes.c_int32, P, P, P, P, P, P]
        lib.lora_oracle_project_at.restype = ctypes.c_int
        lib.lora_oracle_project_at.argtypes = ([ctypes.c_int32] * 3 + [P, P, P, ctypes.c_int32, P, P, P, P, P]
                                               + [ctypes.c_int64, P, P, P])
        lib.lora_oracle_threads.restype = ctypes.c_int
        _lib = lib
    return _lib


def threads() -> int:
    return int(_load().lora_oracle_threads())


def _adapter_tables(adapters: Dict[int, Tuple[int, float, Optional[np.ndarray], Optional[np.ndarray]]],
                    d_in: int, d_out: int):
    """adapters: id -> (rank, scale, A uint16 [rank,d_in] or None, B uint16 [d_out,rank] or None)."""
    n = (max(adapters) + 1) if adapters else 0
    rank = np.zeros(max(n, 1), dtype=np.int32)
    scale = np.zeros(max(n, 1), dtype=np.float64)
    A_ptr = (ctypes.c_void_p * max(n, 1))()
    B_ptr = (ctypes.c_void_p * max(n, 1))()
    keep = []
    for i, (r, s, A, B) in adapters.items():
        rank[i] = r
        scale[i] = float(np.float32(s))          # the scale is an fp32 quantity, widened exactly
        if r > 0 and A is not None and B is not None:
            A = np.ascontiguousarray(A, dtype=np.uint16)
            B = np.ascontiguousarray(B, dtype=np.uint16)
            assert A.shape == (r, d_in), (A.shape, r, d_in)
            assert B.shape == (d_out, r), (B.shape, d_out, r)
            keep += [A, B]
            A_ptr[i] = A.ctypes.data
            B_ptr[i] = B.ctypes.data
    return n, rank, scale, A_ptr, B_ptr, keep


def _bias_arg(bias, d_out: int):
    if bias is None:
        return None, None
    bias = np.ascontiguousarray(bias, dtype=np.uint16)
    assert bias.shape == (d_out,), (bias.shape, d_out)
    return bias, bias.ctypes.data


def project(x: np.ndarray, W: np.ndarray, ids: np.ndarray, adapters, bias=None) -> np.ndarray:
    """y_ref [T, d_out] float64 for bf16-bit inputs x [T,d_in], W [d_out,d_in]; bias: bf16 bits [d_out] of the
    backbone layer's bias, or None."""
    x = np.ascontiguousarray(x, dtype=np.uint16)
    W = np.ascontiguousarray(W, dtype=np.uint16)
    ids = np.ascontiguousarray(ids, dtype=np.int32)
    T, d_in = x.shape
    d_out = W.shape[0]
    assert W.shape[1] == d_in and ids.shape == (T,)
    n, rank, scale, A_ptr, B_ptr, keep = _adapter_tables(adapters, d_in, d_out)
    y = np.empty((T, d_out), dtype=np.float64)
    bias, bias_p = _bias_arg(bias, d_out)
    rc = _load().lora_oracle_project(T, d_in, d_out, x.ctypes.data, W.ctypes.data, ids.ctypes.data, n,
                                     rank.ctypes.data, scale.ctypes.data,
                                     ctypes.cast(A_ptr, ctypes.c_void_p), ctypes.cast(B_ptr, ctypes.c_void_p),
                                     bias_p, y.ctypes.data)
    if rc != 0:
        raise ValueError(f"oracle: token names an unknown adapter (rc={rc})")
    del keep
    return y


def project_at(x, W, ids, adapters, ts: np.ndarray, ns: np.ndarray, bias=None) -> np.ndarray:
    """y_ref at the sampled (token, column) pairs only, each evaluated on its own."""
    x = np.ascontiguousarray(x, dtype=np.uint16)
    W = np.ascontiguousarray(W, dtype=np.uint16)
    ids = np.ascontiguousarray(ids, dtype=np.int32)
    ts = np.ascontiguousarray(ts, dtype=np.int32)
    ns = np.ascontiguousarray(ns, dtype=np.int32)
    T, d_in = x.shape
    d_out = W.shape[0]
    n, rank, scale, A_ptr, B_ptr, keep = _adapter_tables(adapters, d_in, d_out)
    y = np.empty(ts.shape[0], dtype=np.float64)
    bias, bias_p = _bias_arg(bias, d_out)
    rc = _load().lora_oracle_project_at(T, d_in, d_out, x.ctypes.data, W.ctypes.data, ids.ctypes.data, n,
                                        rank.ctypes.data, scale.ctypes.data,
                                        ctypes.cast(A_ptr, ctypes.c_void_p), ctypes.cast(B_ptr, ctypes.c_void_p),
                                        bias_p, ts.shape[0], ts.ctypes.data, ns.ctypes.data, y.ctypes.data)
    if rc != 0:
        raise ValueError(f"oracle: bad sample or unknown adapter (rc={rc})")
    del keep
    return y


def adapters_of(workload, p: int):
    """Adapter table of projection p in the form ``project`` takes (duck-typed workload)."""
    return {aid: (a.rank, a.scale, a.A[p] if a.rank > 0 else None, a.B[p] if a.rank > 0 else None)
            for aid, a in workload.adapters.items()}


# ---------------------------------------------------------------------------
# token -> adapter segment map
# ---------------------------------------------------------------------------
def token_slots(ids: np.ndarray, id2slot: np.ndarray) -> Tuple[np.ndarray, int]:
    """slot[t] for every token; -1 for backbone-only tokens.  A token whose adapter is
    unknown or not resident (paper Sec. 2.2: a request runs only with its adapter in GPU
    memory) is a caller error: it is reported in the flag word and served backbone-only."""
    ids = np.asarray(ids, dtype=np.int64)
    id2slot = np.asarray(id2slot, dtype=np.int64)
    slot = np.full(ids.shape, -1, dtype=np.int64)
    flags = 0
    for t, i in enumerate(ids):
        if i < 0:
            continue
        if i >= id2slot.shape[0] or id2slot[i] < 0:
            flags |= FLAG_NOT_RESIDENT
            continue
        slot[t] = id2slot[i]
    return slot.astype(np.int32), flags


def bucket(ids: np.ndarray, id2slot: np.ndarray, mode: int):
    """Returns (perm, seg_start, seg_slot, n_seg, flags), all int32.

    SORTED: perm is the stable ascending sort of 0..T-1 by slot[t]; segments are the runs of
    equal slot in that order (so seg_slot is strictly ascending, a -1 segment comes first).
    RUNS:   perm is the identity; segments are the runs of equal slot in token order.
    seg_start has n_seg+1 entries: seg_start[0] = 0, seg_start[n_seg] = T."""
    slot, flags = token_slots(ids, id2slot)
    T = slot.shape[0]
    if mode == SORTED:
        perm = np.argsort(slot, kind="stable").astype(np.int32)
    elif mode == RUNS:
        perm = np.arange(T, dtype=np.int32)
    else:
        raise ValueError("mode")
    ordered = slot[perm]
    starts: List[int] = []
    seg_slot: List[int] = []
    for m in range(T):
        if m == 0 or ordered[m] != ordered[m - 1]:
            starts.append(m)
            seg_slot.append(int(ordered[m]))
    n_seg = len(starts)
    starts.append(T)
    return (perm, np.array(starts, dtype=np.int32), np.array(seg_slot, dtype=np.int32), n_seg, flags)


# ---------------------------------------------------------------------------
# adapter slot region with LRU replacement
# ---------------------------------------------------------------------------
class SlotsExhausted(Exception):
    pass


class SlotTable:
    """A_max slots; each holds one adapter id (or is empty).  ``load(requests, in_use)``
    is one load call: a global tick advances once per call; every adapter in ``in_use`` that
    is resident and every adapter the call loads or re-touches gets last_used = tick.
    Victim for a request without an explicit slot: the lowest-index empty slot; else, among
    slots whose adapter is not in ``in_use`` (and was not placed by this same call), the one
    with the smallest last_used, ties to the lowest index; none -> SlotsExhausted."""

    def __init__(self, n_slots: int):
        self.n_slots = n_slots
        self.adapter = [-1] * n_slots
        self.rank = [0] * n_slots
        self.last_used = [0] * n_slots
        self.tick = 0

    def slot_of(self, adapter_id: int) -> int:
        for s, a in enumerate(self.adapter):
            if a == adapter_id:
                return s
        return -1

    def id2slot(self, n_ids: int) -> np.ndarray:
        m = np.full(n_ids, -1, dtype=np.int32)
        for s, a in enumerate(self.adapter):
            if 0 <= a < n_ids:
                m[a] = s
        return m

    def load(self, requests: Sequence[Tuple[int, int, int]], in_use: Sequence[int] = ()):
        """requests: (adapter_id, rank, slot) with slot >= 0 explicit or -1 = pick by LRU.
        Returns a list of (slot, copied) per request, copied = False for a touch.
        A call that cannot place every request changes nothing (state and tick are restored)."""
        saved = (list(self.adapter), list(self.rank), list(self.last_used), self.tick)
        try:
            return self._load(requests, in_use)
        except SlotsExhausted:
            self.adapter, self.rank, self.last_used, self.tick = saved
            raise

    def _load(self, requests, in_use):
        self.tick += 1
        protected = set(int(a) for a in in_use)
        for a in protected:
            s = self.slot_of(a)
            if s >= 0:
                self.last_used[s] = self.tick
        placed_now = set()
        out = []
        for (aid, rank, want) in requests:
            cur = self.slot_of(aid)
            if cur >= 0 and (want < 0 or want == cur):
                self.last_used[cur] = self.tick
                placed_now.add(cur)
                out.append((cur, False))
                continue
            if want >= 0:
                s = want
            else:
                empties = [k for k in range(self.n_slots) if self.adapter[k] < 0]
                if empties:
                    s = empties[0]
                else:
                    cands = [k for k in range(self.n_slots)
                             if self.adapter[k] not in protected and k not in placed_now]
                    if not cands:
                        raise SlotsExhausted()
                    s = min(cands, key=lambda k: (self.last_used[k], k))
            if cur >= 0:                      # moving an adapter to an explicit other slot
                self.adapter[cur] = -1
                self.rank[cur] = 0
            self.adapter[s] = aid
            self.rank[s] = rank
            self.last_used[s] = self.tick
            placed_now.add(s)
            out.append((s, True))
        return out


# ---------------------------------------------------------------------------
# the same slot table over a pool of pages (unified paging of the adapter region)
# ---------------------------------------------------------------------------
class PagedSlotTable(SlotTable):
    """The slot table with the adapters' weights in a pool of ``n_pages`` pages instead of one region of the
    largest rank per slot (paper Sec. 2.2: memory management that pages adapters of different sizes into one
    pool, against the uniform per-adapter footprint the paper's setting uses).  One page holds 8 rank units; an
    adapter of rank r occupies r / 8 consecutive pages (none for rank 0), found first-fit: the lowest first page
    whose run is free.

    A request that needs a copy first gets its slot by the rules of ``SlotTable`` (whoever sat there leaves and
    frees its pages, as does the adapter's own old slot when it moves).  While the pool then has no free run of
    the needed length, further adapters leave, chosen like a slot victim: not in ``in_use``, not placed by this
    call, smallest last_used, ties to the lowest slot; their slots become empty.  No such adapter left ->
    SlotsExhausted, and the whole call is undone.  ``first_page[s]``: first page of slot s, -1 for an empty slot
    or a rank-0 adapter."""

    PAGE_RANKS = 8

    def __init__(self, n_slots: int, n_pages: int):
        super().__init__(n_slots)
        self.n_pages = n_pages
        self.first_page = [-1] * n_slots
        self.owner = [-1] * n_pages          # slot that holds each page, -1 = free

    def load(self, requests, in_use=()):
        saved = (list(self.adapter), list(self.rank), list(self.last_used), self.tick, list(self.first_page),
                 list(self.owner))
        try:
            return self._load(requests, in_use)
        except SlotsExhausted:
            self.adapter, self.rank, self.last_used, self.tick, self.first_page, self.owner = saved
            raise

    def _release(self, s: int) -> None:
        self.adapter[s] = -1
        self.rank[s] = 0
        self.first_page[s] = -1
        self.owner = [-1 if o == s else o for o in self.owner]

    def _first_fit(self, k: int) -> int:
        for p in range(self.n_pages - k + 1):
            if all(o < 0 for o in self.owner[p:p + k]):
                return p
        return -1

    def _load(self, requests, in_use):
        self.tick += 1
        protected = set(int(a) for a in in_use)
        for a in protected:
            s = self.slot_of(a)
            if s >= 0:
                self.last_used[s] = self.tick
        placed_now = set()
        out = []
        for (aid, rank, want) in requests:
            cur = self.slot_of(aid)
            if cur >= 0 and (want < 0 or want == cur):
                self.last_used[cur] = self.tick
                placed_now.add(cur)
                out.append((cur, False))
                continue
            if want >= 0:
                s = want
            else:
                empties = [k for k in range(self.n_slots) if self.adapter[k] < 0]
                if empties:
                    s = empties[0]
                else:
                    cands = [k for k in range(self.n_slots)
                             if self.adapter[k] not in protected and k not in placed_now]
                    if not cands:
                        raise SlotsExhausted()
                    s = min(cands, key=lambda k: (self.last_used[k], k))
            if cur >= 0:
                self._release(cur)
            if self.adapter[s] >= 0:
                self._release(s)
            placed_now.add(s)
            need = rank // self.PAGE_RANKS
            first = -1
            if need > 0:
                if need > self.n_pages:
                    raise SlotsExhausted()
                first = self._first_fit(need)
                while first < 0:
                    cands = [k for k in range(self.n_slots) if self.adapter[k] >= 0
                             and self.adapter[k] not in protected and k not in placed_now]
                    if not cands:
                        raise SlotsExhausted()
                    self._release(min(cands, key=lambda k: (self.last_used[k], k)))
                    first = self._first_fit(need)
                for p in range(first, first + need):
                    self.owner[p] = s
            self.adapter[s] = aid
            self.rank[s] = rank
            self.first_page[s] = first
            self.last_used[s] = self.tick
            out.append((s, True))
        return out


# ---------------------------------------------------------------------------
# gated MLP input: silu(gate) * up on two projections of the same tokens
# ---------------------------------------------------------------------------
def silu(z: np.ndarray) -> np.ndarray:
    """z * sigmoid(z) = z / (1 + exp(-z)), float64, written so that neither branch overflows."""
    z = np.asarray(z, dtype=np.float64)
    out = np.empty_like(z)
    pos = z >= 0
    out[pos] = z[pos] / (1.0 + np.exp(-z[pos]))
    ez = np.exp(z[~pos])
    out[~pos] = z[~pos] * ez / (1.0 + ez)
    return out


def gated(x, W_gate, W_up, ids, adapters_gate, adapters_up) -> np.ndarray:
    """h[t, n] = silu(gate[t, n]) * up[t, n] with gate and up the two LoRA projections of the same x (the input
    of the `down` projection in the gated MLP of the Llama and Qwen2.5 model families the paper evaluates on,
    Sec. 8.1): each projection by the definition above, unrounded, then the activation and the product in float64."""
    g = project(x, W_gate, ids, adapters_gate)
    u = project(x, W_up, ids, adapters_up)
    return silu(g) * u
