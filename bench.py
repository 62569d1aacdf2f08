#!/usr/bin/env python3
"""Benchmark of one multi-adapter LoRA layer-step on one MI355X.

A step = lora_bucket + the seven projections of one decoder layer (q, k, v, o, gate, up, down; q|k|v and
gate|up as packed lora_layer_forward_group calls, o and down as lora_layer_forward calls), each projection
with its own synthetic input, already resident in HBM.  The default workload is
the 8B-shape decode step: 256 one-token requests, 32 resident adapters of ranks {8,16,32}, adapter
ids Zipf(1.0).  Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0        # MI355X HBM3E, vendor figure
MFMA_BF16_PEAK_TFLOPS = 2500.0


def kernel_algorithmic_bytes(w, kernel: str, projections, shrink_inside: bool = False) -> float:
    """Bytes one layer-step's launches of `kernel` must move (over the projections that launch it): each
    array counted once, in the kernel that has to touch it; split-K partials and re-reads are not counted.
    shrink_inside: the fused GEMM launch also does the shrink (no separate shrink launch for these projections)."""
    used = w.distinct_adapters()
    rank_sum = sum(w.adapters[a].rank for a in used)
    T = w.T
    tot = 0.0
    for p in projections:
        d_in, d_out = w.proj[p]
        if kernel.startswith("gemm_splitk"):
            # W once, x once, and (the shrink shares this launch) every used adapter's A once
            tot += 2.0 * d_in * d_out + 2.0 * T * d_in + 2.0 * rank_sum * d_in
        elif kernel.startswith("gemm_fused"):
            tot += 2.0 * d_in * d_out + 2.0 * T * d_in + 2.0 * T * d_out + 2.0 * rank_sum * d_out
            if shrink_inside:
                tot += 2.0 * rank_sum * d_in
        elif kernel == "reduce_expand":
            tot += 2.0 * T * d_out + 2.0 * rank_sum * d_out
        elif kernel == "shrink":
            tot += 2.0 * rank_sum * d_in
    return tot


def kernel_flops(w, kernel: str, projections) -> float:
    T = w.T
    if kernel.startswith("gemm"):
        return float(sum(2.0 * T * w.proj[p][0] * w.proj[p][1] for p in projections))
    return 0.0


def kernel_sources_sha256() -> str:
    """Hash of the HIP sources: a stored counter measurement only counts while the kernels are unchanged."""
    import glob
    import hashlib
    h = hashlib.sha256()
    for f in sorted(glob.glob(os.path.join(ROOT, "paper_2602_24044_amd", "csrc", "*.h*"))):
        h.update(os.path.basename(f).encode())
        h.update(open(f, "rb").read())
    return h.hexdigest()


def stored_traffic(kernel: str, workload: str):
    """HBM bytes per launch of `kernel` from the committed rocprofv3 counter summary (FETCH_SIZE + WRITE_SIZE,
    each scaled by what the same counter reads for a plain copy kernel of known size), or None when there
    is no summary for this kernel and workload or the kernel sources have changed since it was taken."""
    path = os.path.join(ROOT, "profiles", f"{workload}_{kernel}_hbm_traffic.md")
    if not os.path.exists(path):
        return None
    kv = {}
    for line in open(path):
        if ":" in line and not line.startswith("#"):
            k, _, v = line.partition(":")
            kv[k.strip().strip("`")] = v.strip().strip("`")
    if kv.get("sources_sha256") != kernel_sources_sha256():
        return None
    try:
        return float(kv["traffic_bytes_per_launch"])
    except (KeyError, ValueError):
        return None


def calibrate_copy():
    """A plain device copy kernel of known size (256 MiB read + 256 MiB written per launch), ten launches:
    run under `rocprofv3 --pmc FETCH_SIZE` / `WRITE_SIZE` to get the factor between what the counter
    reads and the bytes actually moved."""
    import torch
    n = 256 << 20
    src = torch.empty(n // 4, dtype=torch.int32, device="cuda").fill_(1)
    dst = torch.empty_like(src)
    # evict the source from the last-level cache between launches with a second, larger pair
    big_a = torch.empty(n, dtype=torch.int32, device="cuda").fill_(2)
    big_b = torch.empty_like(big_a)
    torch.cuda.synchronize()
    for _ in range(10):
        big_b.copy_(big_a)
        dst.copy_(src)
    torch.cuda.synchronize()
    print(json.dumps({"copy_bytes_read_per_launch": n, "copy_bytes_written_per_launch": n,
                      "big_copy_bytes_per_launch": 4 * n, "launches": 10}))


def calibrate_stream():
    """Read rate of a plain stream (lora_calibrate_stream): 16 bytes per lane and load, one launch per figure,
    over a buffer far larger than the last-level cache, for a few workgroup counts."""
    import torch
    from paper_2602_24044_amd import binding as B
    n = 2 << 30
    buf = torch.empty(n, dtype=torch.uint8, device="cuda").fill_(1)
    sink = torch.zeros(65536, dtype=torch.int32, device="cuda")
    s = torch.cuda.current_stream().cuda_stream
    out = {}
    for wgs in (224, 256, 512, 1024, 2048, 4096):
        per = 256 << 20
        for i in range(3):
            B.lora_calibrate_stream(buf.data_ptr() + (i % 8) * per, per, wgs, sink.data_ptr(), s)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for i in range(16):
            B.lora_calibrate_stream(buf.data_ptr() + (i % 8) * per, per, wgs, sink.data_ptr(), s)
        e1.record()
        torch.cuda.synchronize()
        us = e0.elapsed_time(e1) / 16 * 1e3
        out[str(wgs)] = {"us_per_launch": us, "gbs": per / us / 1e3}
    best = max(v["gbs"] for v in out.values())
    print(json.dumps({"probe": "stream", "bytes_per_launch": 256 << 20, "by_workgroups": out, "best_gbs": best,
                      "frac_of_peak": best / HBM_PEAK_GBS}))


def calibrate_gemm(sample_clocks: bool = True):
    """Context for the MFMA fraction of the prefill GEMM: the library's backbone GEMM (no adapter rows) and the
    vendor library's bf16 GEMM (torch.matmul) on one prefill-sized problem, first on normally distributed data, then
    on zeros, with the shader clock that rocm-smi shows under each.  Operands of zeros toggle almost no bits in
    the MFMA data path, so the difference between the two data sets is what the power limit costs; the vendor's
    figure on the same data is what a tuned kernel reaches on this chip."""
    import numpy as np
    import torch
    from paper_2602_24044_amd import binding as B
    from paper_2602_24044_amd import workloads as wl
    from paper_2602_24044_amd.runtime import Session
    T, N, K = 8192, 14336, 4096
    flops = 2.0 * T * N * K
    ids = np.full(T, -1, dtype=np.int32)
    w = wl.custom("calibrate_gemm", 0, [(K, N)], ["p"], 8, 16, wl.BUCKET_SORTED, ids, {0: 16}, resident=[])
    sess = Session(w, path=B.LORA_PATH_FUSED)
    sess.bucket()
    x, W = sess.x[0], sess.W[0]
    out = {}

    def timed(fn, iters=12):
        for _ in range(3):
            fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(iters):
            fn()
        e1.record()
        torch.cuda.synchronize()
        clocks = {}
        if sample_clocks:                                    # (starts rocm-smi as a child: not under a counter run)
            with ClockSampler() as cs:                       # keep the load up while the clocks are read
                t_end = time.time() + 1.5
                while time.time() < t_end:
                    for _ in range(iters):
                        fn()
                    torch.cuda.synchronize()
            clocks = cs.summary() or {}
        us = e0.elapsed_time(e1) / iters * 1e3
        return {"us": us, "tflops": flops / us / 1e6, "frac_of_peak": flops / us / 1e6 / MFMA_BF16_PEAK_TFLOPS,
                "sclk_mhz": [clocks.get("sclk_mhz_min"), clocks.get("sclk_mhz_max")]}

    for data in ("normal", "zeros"):
        if data == "zeros":
            x.zero_()
            W.zero_()
        out[data] = {"library": timed(lambda: sess.forward(0)),
                     "library_kernel": B.lora_last_launches(sess.ctx),
                     "vendor_matmul": timed(lambda: torch.matmul(x, W.t()))}
    sess.close()
    print(json.dumps({"probe": "gemm", "shape": {"T": T, "N": N, "K": K}, "dtype": "bf16", "results": out}))


def calibrate_mfma():
    """Sustained bf16 MFMA rate and the shader clock under that load (lora_calibrate_mfma)."""
    import torch
    from paper_2602_24044_amd import binding as B
    out = {}
    for wgs in (256, 512):
        sink = torch.zeros(wgs * 256, dtype=torch.float32, device="cuda")
        ticks = torch.zeros(wgs * 2, dtype=torch.int64, device="cuda")
        s = torch.cuda.current_stream().cuda_stream
        iters = 8192
        B.lora_calibrate_mfma(wgs, iters, sink.data_ptr(), ticks.data_ptr(), s)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(5):
            B.lora_calibrate_mfma(wgs, iters, sink.data_ptr(), ticks.data_ptr(), s)
        e1.record()
        torch.cuda.synchronize()
        us = e0.elapsed_time(e1) / 5 * 1e3
        flops = wgs * 4 * iters * 16 * 32768.0
        t = ticks.cpu().numpy().reshape(-1, 2).astype("float64")
        mhz = float((t[:, 0] / t[:, 1]).mean() * 100.0)        # wall clock ticks are 10 ns
        out[str(wgs)] = {"us_per_launch": us, "tflops": flops / us / 1e6, "shader_clock_mhz": mhz}
    best = max(v["tflops"] for v in out.values())
    print(json.dumps({"probe": "mfma", "by_workgroups": out, "best_tflops": best,
                      "frac_of_peak": best / MFMA_BF16_PEAK_TFLOPS}))


class ClockSampler:
    """Samples `rocm-smi --showclocks` in a thread while the GPU is kept busy (the clocks of an idle GPU say nothing)."""

    def __init__(self):
        import threading
        self.samples = []
        self._stop = False
        self._t = threading.Thread(target=self._run, daemon=True)

    def _run(self):
        import re
        import subprocess
        while not self._stop:
            try:
                txt = subprocess.run(["rocm-smi", "--showclocks"], capture_output=True, text=True, timeout=10).stdout
            except Exception:
                return
            m = {k: int(v) for k, v in re.findall(r"(sclk|mclk) clock level: \S+ \((\d+)Mhz\)", txt)}
            if m:
                self.samples.append(m)

    def __enter__(self):
        self._t.start()
        return self

    def __exit__(self, *a):
        self._stop = True
        self._t.join(timeout=15)

    def summary(self):
        if not self.samples:
            return None
        sclk = [x.get("sclk", 0) for x in self.samples]
        mclk = [x.get("mclk", 0) for x in self.samples]
        return {"source": "rocm-smi --showclocks while steps run", "samples": len(self.samples),
                "sclk_mhz_max": max(sclk), "sclk_mhz_min": min(sclk), "mclk_mhz_max": max(mclk)}


def cpu_baseline(w, budget_s: float = 15.0):
    """The fp64 oracle, as it stands, on a bounded sample of the same workload: the first n tokens of
    the step through all seven projections."""
    import numpy as np
    import oracle
    n = 1
    t_used = 0.0
    done = 0
    while done < w.T and t_used < budget_s:
        take = min(n, w.T - done)
        sl = slice(done, done + take)
        t0 = time.perf_counter()
        oracle.bucket(w.token_ids[sl], np.arange(w.max_adapter_id + 1, dtype=np.int32), w.mode)
        for p in range(len(w.proj)):
            oracle.project(w.x[p][sl], w.W[p], w.token_ids[sl], oracle.adapters_of(w, p), bias=w.bias_of(p))
        t_used += time.perf_counter() - t0
        done += take
        n *= 2
    return {"value": done / t_used, "unit": "tokens/s", "cores": oracle.threads(), "kind": "oracle",
            "sample": f"first {done} of {w.T} tokens of the step, all 7 projections, fp64"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", type=int, default=2, help="workload 2 (8B decode, the headline), 3, 4, 5, or 6 (config 2's recipe at Qwen2.5-7B shapes)")
    ap.add_argument("--copies", type=int, default=0,
                    help="distinct weight/slot copies rotated through (0 = 4 for configs 2 and 4, else 2)")
    ap.add_argument("--shrink", type=int, default=1, help="divide the model dimensions (debugging only)")
    ap.add_argument("--path", type=int, default=0)
    ap.add_argument("--tune", action="append", default=[], metavar="KEY=VALUE",
                    help="lora_set_tuning on every context (kernel variants; repeatable)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-clocks", action="store_true", help="skip the rocm-smi clock samples (about a second of extra steps)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="run plain device copy kernels of known size and exit (reference for the HBM byte counters)")
    ap.add_argument("--calibrate-stream", action="store_true",
                    help="measure the read rate of a plain stream (the roof a weight stream can reach) and exit")
    ap.add_argument("--calibrate-gemm", action="store_true",
                    help="backbone GEMM of the library and the vendor library's GEMM on normal data and on zeros")
    ap.add_argument("--calibrate-mfma", action="store_true",
                    help="measure the sustained bf16 MFMA rate and the clock under it and exit")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: the library runs on one GPU; the path shards by adapter with no exchange, "
              "so --gpus must be 1", file=sys.stderr)
        sys.exit(2)

    if args.calibrate_copy:
        calibrate_copy()
        return
    if args.calibrate_stream:
        calibrate_stream()
        return
    if args.calibrate_gemm:
        calibrate_gemm(sample_clocks=not args.no_clocks)
        return
    if args.calibrate_mfma:
        calibrate_mfma()
        return

    import torch
    from paper_2602_24044_amd import binding as B
    from paper_2602_24044_amd import workloads as wl
    from paper_2602_24044_amd.runtime import Session

    kw = {"shrink": args.shrink} if args.shrink != 1 else {}
    w = wl.by_index(args.config, **kw)
    names = {2: "8B-shape decode, 256 requests x 1 token, 32 adapters ranks {8,16,32}, Zipf(1.0) ids",
             3: "8B-shape prefill, 32 requests lognormal lengths, 64 adapters rank 16",
             4: "8B-shape many-adapter decode, 512 tokens uniform over 384 adapters ranks {8,16,32,64}",
             5: "70B-shape mixed step, 2048-token prefill chunk + 384 decode tokens, 128 slots",
             6: "Qwen2.5-7B-shape decode, 256 requests x 1 token, 32 adapters ranks {8,16,32}, Zipf(1.0) ids, q/k/v bias"}
    metrics = {2: "LoRA-layer tokens/s at 8B-shape decode B=256; % MFMA peak & HBM GB/s",
               3: "LoRA-layer tokens/s at 8B-shape prefill, 32 lognormal-length requests; % MFMA peak & HBM GB/s",
               4: "LoRA-layer tokens/s at 8B-shape many-adapter decode B=512 over 384 adapters; % MFMA peak & HBM GB/s",
               5: "LoRA-layer tokens/s at 70B-shape mixed step (2048 prefill + 384 decode) with 8 adapter loads per step; % MFMA peak & HBM GB/s",
               6: "LoRA-layer tokens/s at Qwen2.5-7B-shape decode B=256; % MFMA peak & HBM GB/s"}
    tune = {}
    for kv in args.tune:
        k, _, v = kv.partition("=")
        tune[int(k)] = int(v)

    copies = args.copies if args.copies > 0 else (4 if args.config in (2, 4, 6) else 2)
    # Config 5: every step loads the batch's cold adapters again (H2D copies inside the timed region).
    # Rank-0 placeholder adapters are put into their slots first (metadata only), so the next load of the
    # real adapters finds them non-resident and copies their weights from pinned host memory.
    reload_each_step = bool(w.missing)
    placeholders = []
    if reload_each_step:
        base_id = w.max_adapter_id + 1
        for i in range(len(w.missing)):
            w.adapters[base_id + i] = wl.Adapter(base_id + i, 0, 0.0, [], [])
            placeholders.append(base_id + i)
    in_use = w.distinct_adapters()
    sessions = []
    for _ in range(copies):
        # adapters that travel inside the timed region are kept as one pinned buffer each (A and B of a projection
        # back to back, as inside a slot): the load then moves one run per projection
        s = Session(w, path=args.path, packed_host=reload_each_step)
        for k, v in tune.items():
            B.lora_set_tuning(s.ctx, k, v)
        s.load(w.resident)
        if w.missing:
            s.load(w.missing, in_use=in_use)
            s.cold_slots = [B.lora_slot_of(s.ctx, a) for a in w.missing]
            s.copy_stream = torch.cuda.Stream()
        sessions.append(s)
    torch.cuda.synchronize()

    def one_step(i, reload=reload_each_step, bucket=True):
        s = sessions[i % copies]
        if reload:
            s.load(placeholders, slots=s.cold_slots, stream=s.copy_stream)
            s.load(w.missing, in_use=in_use, slots=s.cold_slots, stream=s.copy_stream)
        if bucket:
            s.step()
        else:
            s.forward_all()

    def run(n, **kwargs):
        for i in range(n):
            one_step(i, **kwargs)

    def timed(n, **kwargs):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        run(n, **kwargs)
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / n

    # ---- the headline figure: K steps between two synchronisations, inputs resident in HBM ----
    run(args.warmup)
    per_step_s = timed(args.steps)
    ms_per_step = per_step_s * 1e3
    tokens_per_s = w.T / per_step_s

    # ---- the same steps one by one between HIP events on the stream: median and min ----
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
    torch.cuda.synchronize()
    for i, (e0, e1) in enumerate(evs):
        e0.record()
        one_step(i)
        e1.record()
    torch.cuda.synchronize()
    ev_us = sorted(e0.elapsed_time(e1) * 1e3 for e0, e1 in evs)
    step_events = {"median_us": ev_us[len(ev_us) // 2], "min_us": ev_us[0], "max_us": ev_us[-1],
                   "note": "one event pair per step on the stream; a pair adds about 2 us to what it brackets"}

    # ---- without lora_bucket (in a model one segment map serves every layer of the step) ----
    for s in sessions:
        s.bucket()
    run(min(args.warmup, 5), bucket=False)
    no_bucket_s = timed(args.steps, bucket=False)

    # ---- config 5: the same step with every adapter already resident (no copies over the host link) ----
    compute_only = None
    if reload_each_step:
        run(2, reload=False)
        co_s = timed(args.steps, reload=False)
        compute_only = {"ms_per_step": co_s * 1e3, "tokens_per_s": w.T / co_s,
                        "note": "all adapters resident; `value` includes the step's adapter copies over the host link"}

    # ---- second pass of the same steps with every kernel bracketed by HIP events on its stream ----
    for s in sessions:
        B.lora_profile_reset(s.ctx)
        B.lora_profile_enable(s.ctx, True)
    done = 0
    while done < args.steps:
        n = min(args.steps - done, 64 * copies)
        run(n)
        torch.cuda.synchronize()
        done += n
        for s in sessions:
            B.lora_profile_collect(s.ctx)      # drains the event pool into the context's running totals
    prof = {}
    for s in sessions:
        for k, (ms, cnt) in B.lora_profile_collect(s.ctx).items():
            a, b = prof.get(k, (0.0, 0))
            prof[k] = (a + ms, b + cnt)
        B.lora_profile_enable(s.ctx, False)
    kernels = {k: {"avg_us": ms / cnt * 1e3, "launches_per_step": cnt / args.steps,
                   "us_per_step": ms / args.steps * 1e3} for k, (ms, cnt) in prof.items() if cnt}
    dominant = max(kernels, key=lambda k: kernels[k]["us_per_step"])
    # which projections launch the dominant kernel
    launched_by = []
    shrink_inside = False
    s0 = sessions[0]
    s0.bucket()
    for g in s0.packed_groups():
        if len(g) > 1:
            s0.forward_group(g)
        else:
            s0.forward(g[0])
        if dominant in B.lora_last_launches(s0.ctx):
            launched_by += g
            shrink_inside = shrink_inside or "shrink" not in B.lora_last_launches(s0.ctx)
    torch.cuda.synchronize()
    dom_t = kernels[dominant]["us_per_step"] * 1e-6
    dom_bytes = kernel_algorithmic_bytes(w, dominant, launched_by, shrink_inside and dominant.startswith("gemm_fused"))
    dom_flops = kernel_flops(w, dominant, launched_by)
    achieved_gbs = dom_bytes / dom_t / 1e9
    roofline = {"bound": "hbm", "kernel": dominant, "achieved": achieved_gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": achieved_gbs / HBM_PEAK_GBS, "traffic": stored_traffic(dominant, w.name),
                "projections": [w.proj_names[p] for p in launched_by] if hasattr(w, "proj_names") else launched_by,
                "algorithmic_bytes_per_launch": dom_bytes / max(1.0, kernels[dominant]["launches_per_step"]),
                "launch_avg_us": kernels[dominant]["avg_us"],
                "mfma_tflops": dom_flops / dom_t / 1e12, "mfma_frac": dom_flops / dom_t / 1e12 / MFMA_BF16_PEAK_TFLOPS}
    if args.config in (3, 5):
        tf = dom_flops / dom_t / 1e12
        roofline.update({"bound": "mfma", "achieved": tf, "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                         "frac": tf / MFMA_BF16_PEAK_TFLOPS, "hbm_gbs": achieved_gbs})

    # ---- the LoRA part alone (HBM-bound workloads): the same step without adapters, and what the difference
    #      moves: every used adapter's A and B once ----
    lora_leg = None
    if args.config in (2, 4, 6):
        import numpy as np
        w0 = wl.by_index(args.config, **kw)
        w0.token_ids = np.full_like(w0.token_ids, -1)
        w0.resident, w0.missing = [], []
        base_sessions = []
        for _ in range(copies):
            s = Session(w0, path=args.path)
            for k, v in tune.items():
                B.lora_set_tuning(s.ctx, k, v)
            base_sessions.append(s)
        for i in range(args.warmup):
            base_sessions[i % copies].step()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(args.steps):
            base_sessions[i % copies].step()
        torch.cuda.synchronize()
        base_s = (time.perf_counter() - t0) / args.steps
        for s in base_sessions:
            s.close()
        ab_bytes = sum(2.0 * w.adapters[a].rank * sum(di + do for di, do in w.proj) for a in w.distinct_adapters())
        d_us = (per_step_s - base_s) * 1e6
        lora_leg = {"backbone_only_ms_per_step": base_s * 1e3, "added_us_per_step": d_us, "adapter_bytes": ab_bytes,
                    "gbs": (ab_bytes / (d_us * 1e-6) / 1e9) if d_us > 0 else None,
                    "frac": (ab_bytes / (d_us * 1e-6) / 1e9 / HBM_PEAK_GBS) if d_us > 0 else None,
                    "note": "A and B of every adapter in the batch, once, over the time the adapters add to the step"}

    # ---- clocks under this load ----
    clocks = None
    if not args.no_clocks:
        with ClockSampler() as cs:
            t_end = time.perf_counter() + 1.5
            i = 0
            while time.perf_counter() < t_end:
                one_step(i, reload=False)
                i += 1
                if i % 64 == 0:
                    torch.cuda.synchronize()
            torch.cuda.synchronize()
        clocks = cs.summary()

    step_bytes = wl.algorithmic_bytes(w)
    out = {
        "metric": metrics.get(args.config, metrics[2]),
        "value": tokens_per_s, "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": names.get(args.config, w.name), "name": w.name, "tokens": w.T,
                   "h2d_adapter_bytes_per_step": (sum(2 * w.adapters[a].rank * sum(di + do for di, do in w.proj)
                                                      for a in w.missing) if reload_each_step else 0),
                   "projections": len(w.proj), "distinct_adapters": len(w.distinct_adapters()),
                   "weight_copies_rotated": copies, "path": args.path, "tuning": tune},
        "layer_step": {"algorithmic_bytes": step_bytes, "hbm_gbs": step_bytes / (ms_per_step * 1e-3) / 1e9,
                       "hbm_frac": step_bytes / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS,
                       "flops": wl.algorithmic_flops(w),
                       "tflops": wl.algorithmic_flops(w) / (ms_per_step * 1e-3) / 1e12},
        "step_events": step_events,
        "without_bucket": {"ms_per_step": no_bucket_s * 1e3, "tokens_per_s": w.T / no_bucket_s},
        "kernels": kernels,
        "roofline": roofline,
    }
    if compute_only is not None:
        out["compute_only"] = compute_only
    if lora_leg is not None:
        out["lora_leg"] = lora_leg
    if clocks is not None:
        out["clocks"] = clocks
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w)
    for s in sessions:
        s.close()
    print(json.dumps(out))


if __name__ == "__main__":
    main()
