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


def fit_load(sizes: Sequence[float], ms: Sequence[float]) -> Dict[str, object]:
    """Lat_load(S) of Eq. 1 (Sec. 5.2: the time to bring an adapter of size S from CPU memory into the GPU's adapter
    region, kept as a table over the sizes that occur; Sec. 5.1.3: it grows with the adapter size).  From measured
    (size, milliseconds) points: the table (mean per distinct size) and the straight line ms = fixed + per_rank * S
    through the points by least squares, with the line's error against the points."""
    S = np.asarray(sizes, dtype=np.float64)
    y = np.asarray(ms, dtype=np.float64)
    if S.shape != y.shape or S.size < 2 or np.unique(S).size < 2:
        raise ValueError("need (size, ms) points of equal length over at least two distinct sizes")
    table = {int(v): float(np.mean(y[S == v])) for v in np.unique(S)}
    F = np.stack([np.ones_like(S), S], axis=1)
    (fixed, per_rank), *_ = np.linalg.lstsq(F, y, rcond=None)
    pred = F @ np.array([fixed, per_rank])
    return {"table_ms": table, "fixed_ms": float(fixed), "per_rank_ms": float(per_rank),
            "smape_percent": float(np.mean(2.0 * np.abs(pred - y) / (np.abs(pred) + np.abs(y))) * 100.0),
            "max_rel_err": float(np.max(np.abs(pred - y) / np.abs(y)))}


def predict_load(law: Dict[str, object], size: int) -> float:
    """Milliseconds to load an adapter of `size`: the table entry where the size was measured, else the line."""
    table = law.get("table_ms", {})
    if int(size) in table:
        return float(table[int(size)])
    return float(law["fixed_ms"]) + float(law["per_rank_ms"]) * float(size)


def sweep(batch_sizes: Sequence[int] = (32, 64, 128, 256, 512), adapters_in_batch: Sequence[int] = (0, 1, 2, 4, 8, 16, 32),
          rank: int = 16, steps: int = 40, warmup: int = 8, shrink: int = 1) -> List[Dict[str, float]]:
    """Measures the layer-step latency (us) for every (B, A): B one-token requests spread round-robin over A
    resident adapters of the given rank (A = 0: backbone only).  Two copies of the weights alternate so that a
    step streams them from HBM."""
    import torch

    from . import binding as Bd
    from . import workloads as wl
    from .runtime import Session

    n_adapters = max(max(adapters_in_batch), 1)
    t_max = max(batch_sizes)
    proj, names = wl.shapes_8b(shrink)            # shrink > 1: the model dimensions divided (tests)
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


def measure_all(load_layers: int = 32) -> Dict[str, object]:
    """The sweep, its fits, and the load table of whole adapters (model_step.measure) with its fit."""
    from . import model_step

    rows = sweep()
    with_ad = [r for r in rows if r["A"] > 0]
    out: Dict[str, object] = {
        "points": rows,
        "fit_all": fit([r["B"] for r in rows], [r["A"] for r in rows], [r["latency_us"] for r in rows]),
        # the step from no adapter to one is not part of a law linear in A: fitted apart as well
        "fit_A_ge_1": fit([r["B"] for r in with_ad], [r["A"] for r in with_ad], [r["latency_us"] for r in with_ad]),
        "fit_additive": fit_additive([r["B"] for r in rows], [r["A"] for r in rows], [r["latency_us"] for r in rows])}
    m = model_step.measure(n_layers=load_layers)
    pts = [(int(k.split("/")[0]), v["load_ms_per_adapter"]) for k, v in m["per_rank"].items() if k.endswith("/copy_engine")]
    out["load_points"] = [{"rank": r, "ms": ms} for r, ms in pts]
    out["load_layers"] = load_layers
    out["fit_load"] = fit_load([r for r, _ in pts], [ms for _, ms in pts])
    out["step_ms_all_layers"] = m["step_ms"]
    return out


def write_profile(res: Dict[str, object], path: str) -> None:
    """profiles/latency_law.md: the tables, the fits and a machine-readable block (read by placement_model)."""
    rows = res["points"]
    Bs = sorted({r["B"] for r in rows})
    As = sorted({r["A"] for r in rows})
    lat = {(r["B"], r["A"]): r["latency_us"] for r in rows}
    fa, fg, fd, fl = res["fit_all"], res["fit_A_ge_1"], res["fit_additive"], res["fit_load"]
    L = ["# The paper's latency law (Sec. 5.2, Eq. 1) measured on this library, one MI355X", "",
         "Written by `python -m paper_2602_24044_amd.latency_model --write profiles/latency_law.md` (on the GPU box, from the",
         "repository root).  One 8B-shape layer-step (lora_bucket + the seven projections, q|k|v and gate|up packed, two",
         "alternating copies of the weights) for B one-token requests spread over A resident rank-16 adapters; microseconds per step:", "",
         "| B \\ A | " + " | ".join(str(a) for a in As) + " |", "|---|" + "---|" * len(As)]
    for b in Bs:
        L.append(f"| {b} | " + " | ".join(f"{lat[(b, a)]:.0f}" if (b, a) in lat else "-" for a in As) + " |")
    L += ["", f"Eq. 1, `Lat(B, A) = (K4 B + K5)(K6 A + K7)` with K7 = 1, all points: K4 = {fa['K4']:.4f} us per token, K5 = {fa['K5']:.1f} us, "
          f"K6 = {fa['K6']:.5f} per adapter; SMAPE {fa['smape_percent']:.2f} %, worst point {fa['max_rel_err'] * 100:.1f} %.",
          f"Points with A >= 1 only: K4 = {fg['K4']:.4f}, K5 = {fg['K5']:.1f}, K6 = {fg['K6']:.5f}; SMAPE {fg['smape_percent']:.2f} %.",
          f"As a sum, `c_B B + c_0 + c_A A + c_step [A >= 1]`: c_B = {fd['c_B']:.4f}, c_0 = {fd['c_0']:.1f}, c_A = {fd['c_A']:.3f} us per adapter, "
          f"c_step = {fd['c_step']:.1f} us; SMAPE {fd['smape_percent']:.2f} %.", "",
          f"`Lat_load(S)` (Sec. 5.2; whole adapters of {res['load_layers']} layers of 8B shapes, one pinned host buffer each, copy engine, idle GPU), "
          "milliseconds per adapter:", "", "| rank | ms |", "|---|---|"]
    for r in sorted(res["load_points"], key=lambda q: q["rank"]):
        L.append(f"| {r['rank']} | {r['ms']:.3f} |")
    L += ["", f"Line through the points: {fl['fixed_ms']:.3f} ms + {fl['per_rank_ms']:.4f} ms per rank unit; SMAPE {fl['smape_percent']:.2f} %.",
          f"The step over all {res['load_layers']} layers alone: {res['step_ms_all_layers']:.2f} ms.", "",
          "Machine-readable (read by `paper_2602_24044_amd/placement_model.py`):", ""]
    kv = {"K4_us_per_token": fa["K4"], "K5_us": fa["K5"], "K6_per_adapter": fa["K6"], "K7": 1.0,
          "eq1_smape_percent": fa["smape_percent"], "load_fixed_ms": fl["fixed_ms"], "load_per_rank_ms": fl["per_rank_ms"],
          "load_smape_percent": fl["smape_percent"], "load_layers": res["load_layers"]}
    L += [f"{k}: {v:.6g}" for k, v in kv.items()]
    L += ["load_table_ms: " + " ".join(f"{r}={ms:.4f}" for r, ms in sorted(fl["table_ms"].items())), ""]
    with open(path, "w") as f:
        f.write("\n".join(L))


def read_profile(path: str) -> Dict[str, object]:
    """The machine-readable block of a file written by write_profile."""
    out: Dict[str, object] = {}
    with open(path) as f:
        for line in f:
            key, sep, val = line.partition(":")
            key, val = key.strip(), val.strip()
            if not sep or not key or " " in key or key.startswith(("|", "#", "`")):
                continue
            if key == "load_table_ms":
                out[key] = {int(a): float(b) for a, b in (item.split("=") for item in val.split())}
            else:
                try:
                    out[key] = float(val)
                except ValueError:
                    pass
    return out


def main() -> None:
    res = measure_all()
    if len(sys.argv) >= 3 and sys.argv[1] == "--write":
        write_profile(res, sys.argv[2])
    json.dump(res, sys.stdout)
    sys.stdout.write("\n")


if __name__ == "__main__":
    main()
