"""Shared helpers for the GPU parity tests (not collected by pytest)."""
import numpy as np
import torch

import oracle
from paper_2602_24044_amd import binding as B
from paper_2602_24044_amd import workloads as wl
from paper_2602_24044_amd.runtime import Session, bf16_tensor_to_bits

TOL = 5e-3   # max|y - y_ref| / max|y_ref|, bf16 in, fp32 accumulate, bf16 out


def announce(msg):
    print(f"[gpu-case] {msg}", flush=True)


def check_segments(sess, w, mode=None):
    """Segment map of the last bucket call against the oracle, bit for bit."""
    mode = w.mode if mode is None else mode
    perm, seg_start, seg_slot, n_seg = sess.read_segments()
    o_perm, o_start, o_slot, o_n, o_flags = oracle.bucket(w.token_ids, sess.id2slot(), mode)
    assert n_seg == o_n
    assert np.array_equal(perm, o_perm)
    assert np.array_equal(seg_start, o_start)
    assert np.array_equal(seg_slot, o_slot)
    return o_flags


def rel_err(out_bits, y_ref):
    got = wl.bf16_bits_to_f64(out_bits)
    denom = np.max(np.abs(y_ref))
    return float(np.max(np.abs(got - y_ref)) / (denom if denom > 0 else 1.0))


def run_and_check(w, path=B.LORA_PATH_AUTO, split_k=0, preload=None, check_maps=True, tol=TOL, packed=False, tuning=None,
                  n_pages=0):
    """Loads the resident adapters, runs one step, compares every projection with the oracle.  packed: q|k|v
    and gate|up go through lora_layer_forward_group (each projection still has its own x).  tuning: {key: value}
    passed to lora_set_tuning (kernel variants).  n_pages > 0: the adapters share a pool of that many pages."""
    announce(f"{w.name} T={w.T} path={path} split_k={split_k} packed={packed} tuning={tuning} n_pages={n_pages} proj={w.proj}")
    sess = Session(w, path=path, split_k=split_k, n_pages=n_pages)
    try:
        for key, value in (tuning or {}).items():
            B.lora_set_tuning(sess.ctx, key, value)
        resident = w.resident if preload is None else preload
        sess.load(resident)
        if w.missing:
            sess.load(w.missing, in_use=w.distinct_adapters())
        sess.bucket()
        if check_maps:
            flags = check_segments(sess, w)
            assert flags == 0
        errs = []
        group_launches = {}
        if packed:
            for g in sess.packed_groups():
                if len(g) > 1:
                    sess.forward_group(g)
                else:
                    sess.forward(g[0])
                for p in g:
                    group_launches[p] = B.lora_last_launches(sess.ctx)
            torch.cuda.synchronize()
        for p in range(len(w.proj)):
            out = sess.out[p] if packed else sess.forward(p)
            torch.cuda.synchronize()
            y_ref = oracle.project(w.x[p], w.W[p], w.token_ids, oracle.adapters_of(w, p), bias=w.bias_of(p))
            e = rel_err(bf16_tensor_to_bits(out), y_ref)
            launches = group_launches[p] if packed else B.lora_last_launches(sess.ctx)
            announce(f"  proj {p} {w.proj[p]} launches={launches} rel_err={e:.3e}")
            errs.append(e)
        st, word = B.lora_poll_device_flags(sess.ctx)
        assert st == B.LORA_OK and word == 0
        assert max(errs) <= tol, errs
        return errs
    finally:
        sess.close()


N_UNIFORM = 400
BLOCK = 128        # the smallest output tile any GEMM variant here owns is 128 x 128 (the largest 256 x 256)
TAIL_ROWS = 1024   # at least the rows the library may hand to the split-K path behind the full rounds


def stratified_samples(rng, perm, seg_start, n_seg, T, d_out, n_uniform=N_UNIFORM):
    """(token, column) pairs: one per BLOCK x BLOCK block of (position, column), two per segment, one per position
    of the last TAIL_ROWS, n_uniform uniform ones, the corners.  Positions index the segment map's order; a
    position becomes a token through perm."""
    pos, col = [], []
    for r0 in range(0, T, BLOCK):
        for c0 in range(0, d_out, BLOCK):
            pos.append(r0 + rng.integers(0, min(BLOCK, T - r0)))
            col.append(c0 + rng.integers(0, min(BLOCK, d_out - c0)))
    for s in range(n_seg):
        for _ in range(2):
            pos.append(rng.integers(seg_start[s], seg_start[s + 1]))
            col.append(rng.integers(0, d_out))
    for m in range(max(0, T - TAIL_ROWS), T):
        pos.append(m)
        col.append(rng.integers(0, d_out))
    pos += list(rng.integers(0, T, size=n_uniform)) + [0, 0, T - 1, T - 1]
    col += list(rng.integers(0, d_out, size=n_uniform)) + [0, d_out - 1, 0, d_out - 1]
    pos = np.asarray(pos, dtype=np.int64)
    return perm[pos].astype(np.int32), np.asarray(col, dtype=np.int32)
