"""Whole-model measurements of the adapter slot table on one GPU (run: python -m paper_2602_24044_amd.model_step).

The paper's Digital Twin needs, besides the forward latency law, two facts about adapter residency that depend on
the hardware (Sec. 5.2, Eq. 1): the time `Lat_load(S)` to bring an adapter of size S from CPU memory into the GPU's
adapter region (a table over S; Sec. 5.1.3: it grows with the adapter size and matters for short requests), and the
memory the region takes from everything else (Sec. 5.1.1; Sec. 2.2 and 8.1: A_max slots of the uniform size
S_max, the largest adapter's).  This module measures the first on the library (one context holding every decoder
layer, a slot = one adapter's matrices of all layers) and computes the second:

* `slot_region_bytes` - bytes of the region with uniform S_max slots against a region packed at the adapters' own
  ranks (what a unified paging scheme, the alternative the paper discusses in Sec. 2.2, would hold).  Arithmetic on
  shapes only.
* `measure` - per-rank load time of whole adapters, the time of a decode step over all layers, and the same step
  when it follows a load: after waiting for it, or enqueued straight behind it on another stream (the copies
  travel layer after layer and each layer's forward waits only for its own); each with the copy engine and
  with the copy kernel carrying the adapters (every adapter is one pinned buffer: one run per layer).

Weights and adapter values are random bits of the right shape, generated on the device / in pinned memory: only
sizes and residency matter for these timings.
"""
from __future__ import annotations

import json
import sys
import time
from typing import Dict, List, Sequence, Tuple

import numpy as np


def slot_region_bytes(proj: Sequence[Tuple[int, int]], n_layers: int, ranks: Sequence[int], s_max: int,
                      a_max: int) -> Dict[str, int]:
    """Bytes (bf16) of the adapter region for `a_max` slots of rank `s_max`, and of the same adapters (`ranks`,
    at most a_max of them) stored at their own ranks."""
    per_rank = 2 * n_layers * sum(d_in + d_out for d_in, d_out in proj)       # bytes one rank unit takes
    held = list(ranks)[:a_max]
    return {"uniform": int(a_max * s_max * per_rank), "packed": int(sum(held) * per_rank),
            "per_rank_unit": int(per_rank)}


def measure(n_layers: int = 32, n_tokens: int = 256, n_slots: int = 32, n_swap: int = 8, reps: int = 3,
            ranks: Sequence[int] = (8, 16, 32)) -> Dict[str, object]:
    import torch

    from . import binding as B
    from . import workloads as wl
    from .runtime import packed_groups

    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    proj, names = wl.shapes_8b()
    small = wl.config2(shrink=16, n_tokens=n_tokens)            # token ids and ranks of the decode workload
    ids0 = small.token_ids.copy()
    base_rank = {a: small.adapters[a].rank for a in range(n_slots)}
    s_max = max(max(ranks), max(base_rank.values()))
    # adapter ids: 0 .. n_slots-1 the resident set; then one set of n_swap adapters per measured rank
    swap_sets = {r: list(range(n_slots + k * n_swap, n_slots + (k + 1) * n_swap)) for k, r in enumerate(ranks)}
    rank_of = dict(base_rank)
    for r, ids in swap_sets.items():
        rank_of.update({a: r for a in ids})
    n_flat = n_layers * len(proj)

    cfg = B.make_config(proj, n_slots, s_max, n_tokens, max(rank_of), n_layers=n_layers)
    nbytes = B.lora_slab_bytes(cfg)
    slab = torch.empty(nbytes, dtype=torch.uint8, device=dev)
    cfg.slab, cfg.slab_bytes = slab.data_ptr(), nbytes
    ctx = B.lora_create(cfg)
    try:
        gen = torch.Generator(device=dev).manual_seed(5)
        W = [[torch.empty((d_out, d_in), dtype=torch.bfloat16, device=dev).normal_(0, 0.02, generator=gen)
              for d_in, d_out in proj] for _ in range(n_layers)]
        x = [torch.empty((n_tokens, d_in), dtype=torch.bfloat16, device=dev).normal_(0, 1, generator=gen)
             for d_in, _ in proj]
        out = [torch.empty((n_tokens, d_out), dtype=torch.bfloat16, device=dev) for _, d_out in proj]
        groups = packed_groups(small)

        # pinned host copy of every adapter: one page-locked buffer per adapter holding [layer][projection] A then
        # B matrices back to back (every matrix a multiple of 16 bytes); values from one random block per rank
        blocks: Dict[int, torch.Tensor] = {}
        unit = sum(d_in + d_out for d_in, d_out in proj)

        adapters = {}
        for a, r in rank_of.items():
            n_el = r * n_layers * unit
            if r not in blocks:
                blocks[r] = torch.empty(n_el, dtype=torch.bfloat16).normal_(0, 0.02)
            buf = torch.empty(n_el, dtype=torch.bfloat16, pin_memory=True)
            buf.copy_(blocks[r])
            A_ptrs, B_ptrs, off = [], [], 0
            for _ in range(n_layers):
                for d_in, d_out in proj:
                    A_ptrs.append(buf.data_ptr() + 2 * off)
                    off += r * d_in
                    B_ptrs.append(buf.data_ptr() + 2 * off)
                    off += r * d_out
            assert off == n_el
            adapters[a] = {"adapter_id": a, "rank": r, "scale": 2.0, "slot": -1, "buf": buf,
                           "A_ptrs": A_ptrs, "B_ptrs": B_ptrs}
        assert all(len(d["A_ptrs"]) == n_flat for d in adapters.values())
        adapter_bytes = {r: 2 * r * n_layers * sum(a + b for a, b in proj) for r in ranks}

        compute, copy = torch.cuda.Stream(), torch.cuda.Stream()

        def load(ids, slots, stream):
            descs = [dict(adapters[a], slot=sl) for a, sl in zip(ids, slots)]
            res = B.lora_slots_load(ctx, descs, (), stream.cuda_stream)
            assert all(c for _, c in res)

        def step(d_ids, stream, after_layer0=None):
            seg = B.lora_bucket(ctx, d_ids.data_ptr(), n_tokens, wl.BUCKET_SORTED, stream.cuda_stream)
            for l in range(n_layers):
                for g in groups:
                    B.lora_model_forward_group(ctx, l, g, [x[p].data_ptr() for p in g], [W[l][p].data_ptr() for p in g],
                                               seg, [out[p].data_ptr() for p in g], stream.cuda_stream)
                if l == 0 and after_layer0 is not None:
                    after_layer0.record(stream)

        def ids_with(swap):      # the step's tokens once adapters 0 .. n_swap-1 have been replaced by `swap`
            ids = ids0.copy()
            for k, a in enumerate(swap):
                ids[ids0 == k] = a
            return torch.from_numpy(ids).to(dev)

        d_ids0 = torch.from_numpy(ids0).to(dev)
        home = list(range(n_swap))
        load(list(range(n_slots)), list(range(n_slots)), copy)
        torch.cuda.synchronize()
        for _ in range(2):
            step(d_ids0, compute)
        torch.cuda.synchronize()

        def timed_wall(fn):
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            fn()
            torch.cuda.synchronize()
            return (time.perf_counter() - t0) * 1e3

        res: Dict[str, object] = {"n_layers": n_layers, "tokens": n_tokens, "n_slots": n_slots, "s_max": s_max,
                                  "slab_bytes": int(nbytes), "adapters_per_load": n_swap}
        res["step_ms"] = min(timed_wall(lambda: step(d_ids0, compute)) for _ in range(reps + 2))

        per_rank = {}
        engines = {"copy_engine": B.LORA_COPY_ENGINE, "copy_kernel": B.LORA_COPY_KERNEL}
        for r, (ename, evalue) in [(r, e) for r in ranks for e in engines.items()]:
            B.lora_set_tuning(ctx, B.LORA_TUNE_COPY_ENGINE, evalue)
            swap = swap_sets[r]
            d_ids1 = ids_with(swap)
            t_load, t_serial, t_overlap, t_first = [], [], [], []
            for _ in range(reps):
                # load alone (device time on the copy stream), then back home
                torch.cuda.synchronize()
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record(copy)
                load(swap, home, copy)
                e1.record(copy)
                torch.cuda.synchronize()
                t_load.append(e0.elapsed_time(e1))
                load(home, home, copy)
                # load, wait, step
                def serial():
                    load(swap, home, copy)
                    copy.synchronize()
                    step(d_ids1, compute)
                t_serial.append(timed_wall(serial))
                load(home, home, copy)
                # step enqueued behind the load
                torch.cuda.synchronize()
                s0, s1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                def overlapped():
                    s0.record(compute)
                    load(swap, home, copy)
                    step(d_ids1, compute, after_layer0=s1)
                t_overlap.append(timed_wall(overlapped))
                t_first.append(s0.elapsed_time(s1))
                load(home, home, copy)
                torch.cuda.synchronize()
            st, word = B.lora_poll_device_flags(ctx)
            if st != B.LORA_OK or word != 0:
                raise RuntimeError("device flags set during the measurement")
            per_rank[f"{r}/{ename}"] = {"adapter_bytes": int(adapter_bytes[r]),
                                "load_ms_per_adapter": min(t_load) / n_swap,
                                "load_GBps": adapter_bytes[r] * n_swap / (min(t_load) * 1e-3) / 1e9,
                                "load_then_step_ms": min(t_serial), "step_behind_load_ms": min(t_overlap),
                                "first_layer_done_ms": min(t_first)}
        res["per_rank"] = per_rank
        a_maxes = [8, 32, 128, 384]
        mix = [int(v) for v in np.random.default_rng(0).choice(list(ranks), size=max(a_maxes))]
        res["slot_region"] = {str(a): slot_region_bytes(proj, n_layers, mix, s_max, a) for a in a_maxes}
        return res
    finally:
        B.lora_destroy(ctx)


def main() -> None:
    json.dump(measure(), sys.stdout)
    sys.stdout.write("\n")


if __name__ == "__main__":
    main()
