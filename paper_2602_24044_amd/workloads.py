"""Seeded synthetic inputs for multi-adapter LoRA serving steps.

This module only *draws inputs*: shapes, adapter ranks, token->adapter ids and
bf16 bit patterns.  It holds none of the projection, bucketing or slot-table
arithmetic, so both the CPU checker and the GPU library can be fed from it
without sharing any of the method's code.

Shapes follow the paper's evaluation setup (Sec. 8.1: Llama-3.1-8B-class
backbone, LoRA ranks {8,16,32}; Sec. 7: up to 384 simultaneously loaded
adapters; Sec. 2.1: a step mixes prefill tokens and one-token decode requests).
All tensors are drawn once on the host with NumPy's PCG64, rounded to bf16
(round-to-nearest-even) and handed to every consumer as the same uint16 bits.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np

BUCKET_SORTED = 0
BUCKET_RUNS = 1

ALPHA = 16.0  # LoRA alpha shared by all synthetic adapters: scale = ALPHA / rank


# --------------------------------------------------------------------------
# bf16 bit helpers (storage format only)
# --------------------------------------------------------------------------
def to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """float32 array -> uint16 bf16 bit patterns, round-to-nearest-even."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32)
    r = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + r) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """uint16 bf16 bit patterns -> float32 (exact)."""
    b = np.ascontiguousarray(b, dtype=np.uint16)
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def bf16_bits_to_f64(b: np.ndarray) -> np.ndarray:
    """uint16 bf16 bit patterns -> float64 (exact)."""
    return bf16_bits_to_f32(b).astype(np.float64)


def _normal_bf16(rng: np.random.Generator, shape: Tuple[int, ...], std: float) -> np.ndarray:
    """bf16 bits of N(0, std) samples; drawn in row chunks to bound host memory."""
    n_rows = int(shape[0]) if len(shape) else 1
    out = np.empty(shape, dtype=np.uint16)
    if out.size == 0:
        return out
    row_elems = max(1, out.size // max(1, n_rows))
    step = max(1, (1 << 24) // row_elems)
    flat = out.reshape(n_rows, -1)
    for r0 in range(0, n_rows, step):
        r1 = min(n_rows, r0 + step)
        blk = rng.standard_normal((r1 - r0, flat.shape[1]), dtype=np.float32)
        blk *= np.float32(std)
        flat[r0:r1] = to_bf16_bits(blk)
    return out


# --------------------------------------------------------------------------
# containers
# --------------------------------------------------------------------------
@dataclass
class Adapter:
    adapter_id: int
    rank: int
    scale: float                      # fp32-representable alpha / rank
    A: List[np.ndarray]               # per projection: uint16 [rank, d_in]
    B: List[np.ndarray]               # per projection: uint16 [d_out, rank]


@dataclass
class Workload:
    name: str
    seed: int
    proj: List[Tuple[int, int]]       # (d_in, d_out) per targeted projection
    proj_names: List[str]
    n_slots: int                      # A_max
    max_rank: int                     # S_max
    mode: int                         # BUCKET_SORTED or BUCKET_RUNS
    token_ids: np.ndarray             # int32 [T], adapter id per token, -1 = backbone only
    adapters: Dict[int, Adapter]
    W: List[np.ndarray]               # per projection: uint16 [d_out, d_in]
    x: List[np.ndarray]               # per projection: uint16 [T, d_in]
    resident: List[int] = field(default_factory=list)   # adapter ids preloaded before the step
    missing: List[int] = field(default_factory=list)    # adapter ids the step must load first
    request_lens: Optional[np.ndarray] = None
    bias: List[Optional[np.ndarray]] = field(default_factory=list)   # per projection: uint16 [d_out] or None

    def bias_of(self, p: int) -> Optional[np.ndarray]:
        return self.bias[p] if p < len(self.bias) else None

    @property
    def T(self) -> int:
        return int(self.token_ids.shape[0])

    @property
    def max_adapter_id(self) -> int:
        return max(self.adapters.keys()) if self.adapters else 0

    def distinct_adapters(self) -> List[int]:
        ids = np.unique(self.token_ids)
        return [int(i) for i in ids if i >= 0]


# --------------------------------------------------------------------------
# shapes
# --------------------------------------------------------------------------
def llama_proj_shapes(hidden: int, intermediate: int, kv: int) -> Tuple[List[Tuple[int, int]], List[str]]:
    """The seven LoRA-targeted projections of one decoder layer: (d_in, d_out)."""
    names = ["q", "k", "v", "o", "gate", "up", "down"]
    shapes = [(hidden, hidden), (hidden, kv), (hidden, kv), (hidden, hidden),
              (hidden, intermediate), (hidden, intermediate), (intermediate, hidden)]
    return shapes, names


def shapes_8b(shrink: int = 1):
    return llama_proj_shapes(4096 // shrink, 14336 // shrink, 1024 // shrink)


def shapes_70b(shrink: int = 1):
    return llama_proj_shapes(8192 // shrink, 28672 // shrink, 1024 // shrink)


def shapes_qwen_7b(shrink: int = 1):
    """Qwen2.5-7B, the paper's second backbone (Sec. 8.1): no dimension is a power of two."""
    return llama_proj_shapes(3584 // shrink, 18944 // shrink, 512 // shrink)


# --------------------------------------------------------------------------
# building blocks
# --------------------------------------------------------------------------
def make_adapter(rng: np.random.Generator, adapter_id: int, rank: int,
                 proj: Sequence[Tuple[int, int]], scale: Optional[float] = None) -> Adapter:
    A, B = [], []
    for (d_in, d_out) in proj:
        A.append(_normal_bf16(rng, (rank, d_in), 1.0 / np.sqrt(d_in)))
        B.append(_normal_bf16(rng, (d_out, rank), 0.02))
    if scale is None:
        scale = float(np.float32(ALPHA / rank)) if rank > 0 else 0.0
    return Adapter(adapter_id, rank, float(np.float32(scale)), A, B)


def make_backbone(rng: np.random.Generator, proj: Sequence[Tuple[int, int]]) -> List[np.ndarray]:
    return [_normal_bf16(rng, (d_out, d_in), 0.02) for (d_in, d_out) in proj]


def make_activations(rng: np.random.Generator, T: int, proj: Sequence[Tuple[int, int]]) -> List[np.ndarray]:
    return [_normal_bf16(rng, (T, d_in), 1.0) for (d_in, _) in proj]


def zipf_probs(n: int, s: float = 1.0) -> np.ndarray:
    p = 1.0 / np.arange(1, n + 1, dtype=np.float64) ** s
    return p / p.sum()


def zipf_ids(rng: np.random.Generator, n_tokens: int, population: Sequence[int], s: float = 1.0) -> np.ndarray:
    """Token ids drawn Zipf(s) over `population`; popularity order is a seeded shuffle."""
    pop = np.array(population, dtype=np.int32)
    order = rng.permutation(len(pop))
    draws = rng.choice(len(pop), size=n_tokens, p=zipf_probs(len(pop), s))
    return pop[order[draws]].astype(np.int32)


def lognormal_lengths(rng: np.random.Generator, n_req: int, median: float = 512.0, sigma: float = 1.0,
                      lo: int = 16, hi: int = 4096) -> np.ndarray:
    z = rng.standard_normal(n_req)
    ln = np.rint(np.exp(np.log(median) + sigma * z))
    return np.clip(ln, lo, hi).astype(np.int64)


# --------------------------------------------------------------------------
# generic workload + the five named configurations
# --------------------------------------------------------------------------
def custom(name: str, seed: int, proj, proj_names, n_slots: int, max_rank: int, mode: int,
           token_ids: np.ndarray, adapter_ranks: Dict[int, int], resident=None, missing=None,
           scales: Optional[Dict[int, float]] = None, request_lens=None) -> Workload:
    """Draw W, x and every adapter in `adapter_ranks` for a given token->adapter map."""
    rng = np.random.default_rng(seed)
    W = make_backbone(rng, proj)
    adapters = {}
    for aid in sorted(adapter_ranks):
        sc = None if scales is None else scales.get(aid)
        adapters[aid] = make_adapter(rng, aid, adapter_ranks[aid], proj, sc)
    token_ids = np.ascontiguousarray(token_ids, dtype=np.int32)
    x = make_activations(rng, int(token_ids.shape[0]), proj)
    if resident is None:
        resident = sorted(adapter_ranks)[:n_slots]
    return Workload(name, seed, list(proj), list(proj_names), n_slots, max_rank, mode, token_ids,
                    adapters, W, x, list(resident), list(missing or []), request_lens)


def config1() -> Workload:
    """Tiny single projection, 4 rank-8 adapters, 16 decode tokens, seed 0."""
    seed = 0
    rng = np.random.default_rng(1000 + seed)
    ids = rng.integers(0, 4, size=16).astype(np.int32)
    return custom("cfg1_tiny", seed, [(512, 512)], ["p"], 4, 8, BUCKET_SORTED, ids,
                  {i: 8 for i in range(4)}, scales={i: 2.0 for i in range(4)})


def config2(shrink: int = 1, n_tokens: int = 256) -> Workload:
    """8B-shape decode: 256 one-token requests, 32 resident adapters, ranks {8,16,32}, Zipf(1) ids."""
    seed = 1
    rng = np.random.default_rng(1000 + seed)
    proj, names = shapes_8b(shrink)
    ranks = {i: int(r) for i, r in enumerate(rng.choice([8, 16, 32], size=32))}
    ids = zipf_ids(rng, n_tokens, list(range(32)), 1.0)
    return custom(f"cfg2_8b_decode_s{shrink}", seed, proj, names, 32, 32, BUCKET_SORTED, ids, ranks)


def config3(shrink: int = 1, n_req: int = 32, len_div: int = 1) -> Workload:
    """8B-shape prefill: 32 requests, lognormal lengths, 64 rank-16 adapters, contiguous segments."""
    seed = 2
    rng = np.random.default_rng(1000 + seed)
    proj, names = shapes_8b(shrink)
    lens = lognormal_lengths(rng, n_req)
    if len_div > 1:
        lens = np.maximum(1, lens // len_div)
    req_adapter = rng.integers(0, 64, size=n_req).astype(np.int32)
    ids = np.repeat(req_adapter, lens).astype(np.int32)
    ranks = {i: 16 for i in range(64)}
    return custom(f"cfg3_8b_prefill_s{shrink}", seed, proj, names, 64, 16, BUCKET_RUNS, ids, ranks,
                  request_lens=lens)


def config4(shrink: int = 1, n_tokens: int = 512, n_adapters: int = 384) -> Workload:
    """Many-adapter decode: 384 resident adapters, ranks {8,16,32,64}, ids uniform."""
    seed = 3
    rng = np.random.default_rng(1000 + seed)
    proj, names = shapes_8b(shrink)
    ranks = {i: int(r) for i, r in enumerate(rng.choice([8, 16, 32, 64], size=n_adapters))}
    ids = rng.integers(0, n_adapters, size=n_tokens).astype(np.int32)
    return custom(f"cfg4_many_adapter_s{shrink}", seed, proj, names, n_adapters, 64, BUCKET_SORTED, ids, ranks)


def config5(shrink: int = 1, prefill_len: int = 2048, n_decode: int = 384, population: int = 256,
            n_slots: int = 128, n_missing: int = 8) -> Workload:
    """70B-shape mixed step: one prefill chunk + decode tokens; exactly `n_missing` distinct
    adapters of the batch are not resident and must be loaded first."""
    seed = 4
    rng = np.random.default_rng(1000 + seed)
    proj, names = shapes_70b(shrink)
    ranks_all = {i: int(r) for i, r in enumerate(rng.choice([8, 16, 32], size=population))}
    resident = [int(i) for i in rng.permutation(population)[:n_slots]]
    res_set = set(resident)
    cold = [i for i in range(population) if i not in res_set]
    missing = [int(i) for i in rng.choice(cold, size=n_missing, replace=False)]
    prefill_adapter = missing[0]
    # decode tokens: Zipf over resident adapters, plus at least one token for each other cold adapter
    dec = zipf_ids(rng, n_decode, resident, 1.0)
    slots_for_cold = rng.choice(n_decode, size=n_missing - 1, replace=False)
    for pos, aid in zip(slots_for_cold, missing[1:]):
        dec[pos] = aid
    dec = dec[rng.permutation(n_decode)]
    ids = np.concatenate([np.full(prefill_len, prefill_adapter, dtype=np.int32), dec.astype(np.int32)])
    used = set(int(i) for i in np.unique(ids)) | res_set
    ranks = {i: ranks_all[i] for i in sorted(used)}
    return custom(f"cfg5_70b_mixed_s{shrink}", seed, proj, names, n_slots, 32, BUCKET_SORTED, ids, ranks,
                  resident=resident, missing=missing)


def qwen_decode(shrink: int = 1, n_tokens: int = 256, mode: int = BUCKET_SORTED) -> Workload:
    """Config-2-like decode step at Qwen2.5-7B shapes: 32 adapters of ranks {8,16,32}, Zipf(1) ids."""
    seed = 7
    rng = np.random.default_rng(1000 + seed)
    proj, names = shapes_qwen_7b(shrink)
    ranks = {i: int(r) for i, r in enumerate(rng.choice([8, 16, 32], size=32))}
    ids = zipf_ids(rng, n_tokens, list(range(32)), 1.0)
    if mode != BUCKET_SORTED:
        ids = np.sort(ids)[::-1].copy()          # runs of equal adapters, as contiguous prefill requests would be
    w = custom(f"qwen7b_decode_s{shrink}", seed, proj, names, 32, 32, mode, ids, ranks)
    # the q, k, v projections of this model family have a bias; drawn from a generator of its own, of the
    # size of the projections' outputs so that dropping it is far outside the parity tolerance
    brng = np.random.default_rng(2000 + seed)
    w.bias = [to_bf16_bits(brng.standard_normal(d_out).astype(np.float32)) if nm in ("q", "k", "v") else None
              for nm, (_, d_out) in zip(names, proj)]
    return w


def model_layers(base: Workload, n_layers: int) -> List[Workload]:
    """The step of `base` seen by n_layers decoder layers of one model: the same tokens, adapter ids, ranks, scales,
    resident / missing sets and bias pattern in every layer; each layer draws its own W, x, adapter matrices
    (and bias values) from a seed of its own.  Layer 0 is `base` itself."""
    layers = [base]
    ranks = {aid: a.rank for aid, a in base.adapters.items()}
    scales = {aid: a.scale for aid, a in base.adapters.items()}
    for l in range(1, n_layers):
        w = custom(f"{base.name}_layer{l}", base.seed + 7919 * l, base.proj, base.proj_names, base.n_slots,
                   base.max_rank, base.mode, base.token_ids, ranks, base.resident, base.missing, scales,
                   base.request_lens)
        if base.bias:
            brng = np.random.default_rng(2000 + base.seed + 7919 * l)
            w.bias = [None if b is None else to_bf16_bits(brng.standard_normal(b.shape[0]).astype(np.float32))
                      for b in base.bias]
        layers.append(w)
    return layers


def by_index(i: int, **kw) -> Workload:
    return {1: config1, 2: config2, 3: config3, 4: config4, 5: config5, 6: qwen_decode}[i](**kw)


# --------------------------------------------------------------------------
# algorithmic work of one layer-step (what must be moved / computed, nothing padded)
# --------------------------------------------------------------------------
def algorithmic_bytes(w: Workload, proj_index: Optional[int] = None) -> int:
    """HBM bytes a layer-step must touch: W once, each used adapter's A and B once at its
    true rank, x once, out once, plus the token id / permutation arrays."""
    projs = list(enumerate(w.proj)) if proj_index is None else [(proj_index, w.proj[proj_index])]
    used = w.distinct_adapters()
    T = w.T
    total = 0
    for _, (d_in, d_out) in projs:
        total += 2 * d_in * d_out
        total += sum(2 * w.adapters[a].rank * (d_in + d_out) for a in used)
        total += 2 * T * d_in + 2 * T * d_out
    if proj_index is None:
        total += 4 * T * 3
    return int(total)


def algorithmic_flops(w: Workload, proj_index: Optional[int] = None) -> int:
    projs = list(enumerate(w.proj)) if proj_index is None else [(proj_index, w.proj[proj_index])]
    T = w.T
    rank_sum = int(sum(w.adapters[int(a)].rank for a in w.token_ids if a >= 0))
    total = 0
    for _, (d_in, d_out) in projs:
        total += 2 * T * d_in * d_out + 2 * rank_sum * (d_in + d_out)
    return int(total)
