"""Latency model of one multi-adapter layer-step, fitted on measurements of this library.

The paper models the latency of a serving step as the product of a term linear in the batch size B and a term
linear in the number A of distinct adapters in the batch (Sec. 5.2, Eq. 1):

    Lat_model(B, A) = (K4 * B + K5) * (K6 * A + K7)

and observes on its own system that the adapter overhead grows about linearly with A, with a sharp step from
no adapter to one (Sec. 5.1.2).  `fit` finds the constants for a table of measured (B, A, latency) points;
`sweep` measures such a table with the library on the current GPU (one decoder layer at 8B shapes: bucket + the
seven projections, q|k|v and gate|up as packed calls); running the module prints both as JSON.
The model is scale-ambiguous (K4, K5 can be traded against K6, K7), so K7 is fixed to 1: K4 * B + K5 is then the
latency without adapters and K6 the relative overhead per adapter in the batch.
"""
from __future__ import annotations

import json
import sys
from typing import Dict, List, Sequence

import numpy as np


def predict(k: Sequence[float], B, A):
    k4, k5, k6, k7 = k
    return (k4 * np.asarray(B, dtype=np.float64) + k5) * (k6 * np.asarray(A, dtype=np.float64) + k7)


def fit(B: Sequence[float], A: Sequence[float], lat: Sequence[float], iters: int = 200) -> Dict[str, object]:
    """Least-squares fit of Eq. 1 with K7 = 1 by alternating linear solves (each half of the product is linear in
    its own constants once the other half is fixed).  Returns the constants, the symmetric mean absolute
    percentage error and the largest relative error of the fit."""
    B = np.asarray(B, dtype=np.float64)
    A = np.asarray(A, dtype=np.float64)
    y = np.asarray(lat, dtype=np.float64)
    if not (B.shape == A.shape == y.shape) or B.size < 3:
        raise ValueError("need at least three (B, A, latency) points of equal length")
    k6 = 0.0
    k4 = k5 = 0.0
    for _ in range(iters):
        v = k6 * A + 1.0
        # y ~ (k4 B + k5) v : linear in (k4, k5)
        F = np.stack([B * v, v], axis=1)
        (k4, k5), *_ = np.linalg.lstsq(F, y, rcond=None)
        u = k4 * B + k5
        # y - u ~ k6 (u A)
        ua = u * A
        den = float(np.dot(ua, ua))
        k6 = float(np.dot(y - u, ua) / den) if den > 0 else 0.0
    k = (float(k4), float(k5), float(k6), 1.0)
    pred = predict(k, B, A)
    smape = float(np.mean(2.0 * np.abs(pred - y) / (np.abs(pred) + np.abs(y))) * 100.0)
    worst = float(np.max(np.abs(pred - y) / np.abs(y)))
    return {"K4": k[0], "K5": k[1], "K6": k[2], "K7": k[3], "smape_percent": smape, "max_rel_err": worst}


def fit_additive(B: Sequence[float], A: Sequence[float], lat: Sequence[float]) -> Dict[str, float]:
    """Plain linear least squares of Lat = c_B * B + c_0 + c_A * A + c_step * [A >= 1]: a term linear in A plus the
    step from no adapter to one that the paper observes (Sec. 5.1.2), added to the backbone term instead of
    multiplying it."""
    B = np.asarray(B, dtype=np.float64)
    A = np.asarray(A, dtype=np.float64)
    y = np.asarray(lat, dtype=np.float64)
    if not (B.shape == A.shape == y.shape) or B.size < 4:
        raise ValueError("need at least four (B, A, latency) points of equal length")
    F = np.stack([B, np.ones_like(B), A, (A >= 1).astype(np.float64)], axis=1)
    c, *_ = np.linalg.lstsq(F, y, rcond=None)
    pred = F @ c
    return {"c_B": float(c[0]), "c_0": float(c[1]), "c_A": float(c[2]), "c_step": float(c[3]),
            "smape_percent": float(np.mean(2.0 * np.abs(pred - y) / (np.abs(pred) + np.abs(y))) * 100.0),
            "max_rel_err": float(np.max(np.abs(pred - y) / np.abs(y)))}


def sweep(batch_sizes: Sequence[int] = (32, 64, 128, 256, 512), adapters_in_batch: Sequence[int] = (0, 1, 2, 4, 8, 16, 32),
          rank: int = 16, steps: int = 40, warmup: int = 8) -> List[Dict[str, float]]:
    """Measures the layer-step latency (us) for every (B, A): B one-token requests spread round-robin over A
    resident adapters of the given rank (A = 0: backbone only).  Two copies of the weights alternate so that a
    step streams them from HBM."""
    import torch

    from . import binding as Bd
    from . import workloads as wl
    from .runtime import Session

    n_adapters = max(max(adapters_in_batch), 1)
    t_max = max(batch_sizes)
    proj, names = wl.shapes_8b()
    ids0 = (np.arange(t_max) % n_adapters).astype(np.int32)
    w = wl.custom("latency_model", 3, proj, names, n_adapters, max(rank, 8), wl.BUCKET_SORTED, ids0,
                  {i: rank for i in range(n_adapters)})
    s = Session(w)
    try:
        s.load(w.resident)
        weights = [s.W, [t.clone() for t in s.W]]
        rows = []
        for Bsz in batch_sizes:
            for A in adapters_in_batch:
                if A > Bsz:
                    continue
                ids = np.full(Bsz, -1, dtype=np.int32) if A == 0 else (np.arange(Bsz) % A).astype(np.int32)
                d_ids = torch.from_numpy(ids).to(s.device)

                def step(i):
                    s.W = weights[i % 2]
                    s.bucket(ids=d_ids)
                    for g in s.packed_groups():
                        if len(g) > 1:
                            s.forward_group(g)
                        else:
                            s.forward(g[0])

                for i in range(warmup):
                    step(i)
                torch.cuda.synchronize()
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                for i in range(steps):
                    step(i)
                e1.record()
                torch.cuda.synchronize()
                st, word = Bd.lora_poll_device_flags(s.ctx)
                if st != Bd.LORA_OK or word != 0:
                    raise RuntimeError("device flags set during the sweep")
                rows.append({"B": int(Bsz), "A": int(A), "latency_us": e0.elapsed_time(e1) / steps * 1e3})
        s.W = weights[0]
        return rows
    finally:
        s.close()


def main() -> None:
    rows = sweep()
    with_ad = [r for r in rows if r["A"] > 0]
    out = {"points": rows,
           "fit_all": fit([r["B"] for r in rows], [r["A"] for r in rows], [r["latency_us"] for r in rows]),
           # the step from no adapter to one is not part of a law linear in A: fitted apart as well
           "fit_A_ge_1": fit([r["B"] for r in with_ad], [r["A"] for r in with_ad], [r["latency_us"] for r in with_ad]),
           "fit_additive": fit_additive([r["B"] for r in rows], [r["A"] for r in rows], [r["latency_us"] for r in rows])}
    json.dump(out, sys.stdout)
    sys.stdout.write("\n")


if __name__ == "__main__":
    main()
