"""Analytic stand-ins for the two predictors the placement step needs (paper Sec. 6: a throughput regressor and a
starvation classifier, trained on Digital-Twin runs), built from the laws the Digital Twin itself uses (Sec. 5.2,
Eq. 1) with the constants measured on this library, so that `lora_place_adapters` can be driven end to end on one
machine without the paper's training data.  (run: python -m paper_2602_24044_amd.placement_model)

This is a steady-state estimate, not the paper's models:

* memory (Mem_max): the adapter region takes a_max slots of the largest adapter's size (Sec. 2.2, 8.1); what is left
  of HBM after the backbone holds the KV cache, which bounds the number of requests in flight;
* latency (Lat_model): a step over B requests with A distinct adapters costs n_layers (K4 B + K5)(K6 A + K7) plus a
  per-step constant for everything that is not a LoRA projection; the requests in flight follow from Little's law,
  B = arrival rate x output length x step latency, capped by the memory bound;
* loading (Lat_load): with more adapters than slots, a request whose adapter is not among the a_max most requested
  ones pays one load of its size; that time is taken from the steps;
* starvation: predicted throughput below 90 % of the incoming token rate (the paper's definition, Sec. 6).
"""
from __future__ import annotations

import json
import os
import sys
from dataclasses import dataclass, field
from typing import Dict, List, Optional, Sequence, Tuple

# the measured laws: written by `python -m paper_2602_24044_amd.latency_model --write profiles/latency_law.md`
LATENCY_LAW = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "profiles", "latency_law.md")


@dataclass
class ServingModel:
    # Eq. 1 constants of one layer-step on this library (us), Llama-3.1-8B shapes: no defaults, they are measured
    # (from_profile reads them from the committed measurement)
    k4: float
    k5: float
    k6: float
    k7: float
    # Lat_load: ms per adapter (whole model, host link): a table over the measured sizes, else the fitted line
    load_ms_fixed: float
    load_ms_per_rank: float
    load_table_ms: Dict[int, float] = field(default_factory=dict)
    n_layers: int = 32
    other_us_per_step: float = 4000.0         # attention, norms, sampling: not part of this library
    # memory
    hbm_bytes: float = 288e9
    backbone_bytes: float = 16.1e9
    rank_unit_bytes: float = 5.0 * 2 ** 20     # one unit of rank of one slot, all layers
    kv_bytes_per_token: float = 131072.0       # 32 layers x 2 x 8 kv heads x 128 x bf16
    # workload: global mean lengths (the paper approximates traces this way, Sec. 6)
    mean_input: float = 250.0
    mean_output: float = 230.0

    @classmethod
    def from_profile(cls, path: Optional[str] = None, **overrides) -> "ServingModel":
        """The model with the constants of the committed measurement (profiles/latency_law.md)."""
        from .latency_model import read_profile
        kv = read_profile(path or LATENCY_LAW)
        need = ("K4_us_per_token", "K5_us", "K6_per_adapter", "K7", "load_fixed_ms", "load_per_rank_ms")
        missing = [k for k in need if k not in kv]
        if missing:
            raise ValueError(f"{path or LATENCY_LAW}: no value for {missing}")
        args = dict(k4=kv["K4_us_per_token"], k5=kv["K5_us"], k6=kv["K6_per_adapter"], k7=kv["K7"],
                    load_ms_fixed=kv["load_fixed_ms"], load_ms_per_rank=kv["load_per_rank_ms"],
                    load_table_ms=dict(kv.get("load_table_ms", {})), n_layers=int(kv.get("load_layers", 32)))
        args.update(overrides)
        return cls(**args)

    def load_ms(self, size: int) -> float:
        if int(size) in self.load_table_ms:
            return self.load_table_ms[int(size)]
        return self.load_ms_fixed + self.load_ms_per_rank * size

    def max_requests(self, s_max: int, a_max: int) -> float:
        free = self.hbm_bytes - self.backbone_bytes - a_max * s_max * self.rank_unit_bytes
        return max(0.0, free / (self.kv_bytes_per_token * (self.mean_input + self.mean_output)))

    def step_seconds(self, batch: float, adapters_in_batch: float) -> float:
        lora = self.n_layers * (self.k4 * batch + self.k5) * (self.k6 * adapters_in_batch + self.k7)
        return (lora + self.other_us_per_step) * 1e-6

    def incoming_token_rate(self, rates: Sequence[float]) -> float:
        return sum(rates) * (self.mean_input + self.mean_output)

    def throughput(self, sizes: Sequence[int], rates: Sequence[float], a_max: int) -> float:
        """Tokens per second one GPU sustains for these adapters under `a_max` slots."""
        lam = sum(rates)
        if not sizes or lam <= 0.0:
            return 0.0
        b_max = self.max_requests(max(sizes), a_max)
        if b_max < 1.0:
            return 0.0
        # share of the step time lost to loads: requests of adapters outside the a_max most requested ones
        by_rate = sorted(zip(rates, sizes), reverse=True)
        miss = by_rate[a_max:]
        load_s_per_s = sum(r * self.load_ms(s) * 1e-3 for r, s in miss)
        busy = max(0.05, 1.0 - load_s_per_s)
        # requests in flight by Little's law: B = lam * mean_output * step(B) / busy, by fixed-point iteration
        b = 1.0
        for _ in range(200):
            a_b = min(float(a_max), float(len(sizes)), b)
            b_new = max(1.0, lam * self.mean_output * self.step_seconds(b, a_b) / busy)
            if abs(b_new - b) < 1e-9 * b or b_new > 4.0 * b_max:
                b = b_new
                break
            b = b_new
        total = self.mean_input + self.mean_output
        if b <= b_max:
            return lam * total                     # every request is served as it arrives
        a_b = min(float(a_max), float(len(sizes)), b_max)
        return busy * b_max / (self.mean_output * self.step_seconds(b_max, a_b)) * total

    def starvation(self, sizes: Sequence[int], rates: Sequence[float], a_max: int) -> bool:
        return self.throughput(sizes, rates, a_max) < 0.9 * self.incoming_token_rate(rates)


def place(size: Sequence[int], rate: Sequence[float], n_gpus: int, model: ServingModel) -> Tuple[List[int], List[int]]:
    """Placement by the library's greedy algorithm under this model's predictions."""
    from . import binding as B
    return B.lora_place_adapters(size, rate, n_gpus, model.throughput, model.starvation)


def main() -> None:
    import numpy as np
    rng = np.random.default_rng(0)
    model = ServingModel.from_profile()
    out = []
    # workloads in the style of the paper's evaluation (Sec. 8.1, 8.3): sizes from {8, 16, 32}, Poisson rates from the
    # upper part of its rate set (a GPU of this size is then full before it holds 384 adapters, the last count
    # at which the algorithm tests an allocation)
    for n in (64, 256, 1024):
        size = [int(v) for v in rng.choice([8, 16, 32], size=n)]
        rate = [float(v) for v in rng.choice([3.2, 1.6, 0.8, 0.4, 0.1], size=n)]
        rec = {"adapters": n, "requests_per_s": round(sum(rate), 2)}
        try:
            gpu_of, a_max = place(size, rate, 16, model)
            used = max(gpu_of) + 1
            rec.update({"gpus_used": used, "adapters_per_gpu": [gpu_of.count(g) for g in range(used)],
                        "a_max": a_max[:used],
                        "predicted_tokens_per_s": [round(model.throughput([size[a] for a in range(n) if gpu_of[a] == g],
                                                                          [rate[a] for a in range(n) if gpu_of[a] == g],
                                                                          a_max[g])) for g in range(used)]})
        except Exception as e:       # LoraError: starvation on 16 GPUs
            rec["error"] = str(e)
        out.append(rec)
    json.dump(out, sys.stdout, indent=1)
    sys.stdout.write("\n")


if __name__ == "__main__":
    main()
