"""GPU parity of the integer segment-map kernel alone: bit-exact against the oracle."""
import numpy as np
import pytest
import torch

import oracle
from gpu_util import announce, check_segments
from paper_2602_24044_amd import binding as B
from paper_2602_24044_amd import workloads as wl
from paper_2602_24044_amd.runtime import Session

pytestmark = pytest.mark.gpu


def _bucket_only_workload(T, n_slots, seed, mode, frac_none=0.1, zipf=False):
    """Token ids only (rank-0 adapters: nothing to copy).  RUNS mode gets request-like runs."""
    rng = np.random.default_rng(seed)
    n_ids = n_slots + 9
    if mode == wl.BUCKET_RUNS:
        ids = np.zeros(0, dtype=np.int32)
        while ids.size < T:
            run = int(rng.integers(1, 90))
            ids = np.concatenate([ids, np.full(run, rng.integers(-1, n_slots), dtype=np.int32)])
        ids = ids[:T]
    else:
        if zipf:
            ids = wl.zipf_ids(rng, T, list(range(n_slots)), 1.0)
        else:
            ids = rng.integers(0, n_slots, size=T).astype(np.int32)
        ids[rng.random(T) < frac_none] = -1
    return wl.custom("bucket_only", seed, [(64, 8)], ["p"], n_slots, 8, mode, ids.astype(np.int32),
                     {i: 0 for i in range(n_ids)}, resident=[])


@pytest.mark.parametrize("mode", [wl.BUCKET_SORTED, wl.BUCKET_RUNS])
@pytest.mark.parametrize("T,n_slots,seed", [(1, 1, 0), (63, 3, 1), (64, 4, 2), (65, 33, 3), (256, 32, 4), (512, 384, 5),
                                            (1023, 100, 6), (1024, 17, 7), (1025, 1000, 8), (2432, 128, 9),
                                            (26000, 64, 10), (5000, 4095, 11),
                                            # around the limit up to which the kernel keeps its intermediates on chip
                                            (4095, 300, 12), (4096, 4095, 13), (4097, 37, 14)])
def test_segment_map_bit_exact(mode, T, n_slots, seed):
    w = _bucket_only_workload(T, n_slots, seed, mode, zipf=(seed % 2 == 0))
    announce(f"bucket T={T} n_slots={n_slots} mode={mode} seed={seed}")
    sess = Session(w, upload_inputs=False)
    try:
        # scatter the adapters over slots in a shuffled order so that slot != adapter id
        rng = np.random.default_rng(seed + 100)
        order = rng.permutation(n_slots)
        sess.load([int(a) for a in order], slots=[int(s) for s in rng.permutation(n_slots)])
        ids = torch.from_numpy(w.token_ids).to(sess.device)
        sess.bucket(ids)
        assert check_segments(sess, w) == 0
        # a second call with different ids on the same context
        ids2 = w.token_ids[::-1].copy()
        sess.bucket(torch.from_numpy(ids2).to(sess.device))
        w2 = w
        w2.token_ids = ids2
        assert check_segments(sess, w2) == 0
    finally:
        sess.close()


def test_runs_map_over_several_workgroups_with_runs_across_their_boundaries():
    # above 4096 tokens the RUNS map is built by one workgroup per 1024 tokens: runs that end exactly at, one
    # before, one after and far across those boundaries, a run of one token on each side of a boundary, tokens of an
    # adapter that is not resident (flag, served backbone-only), and a ragged last chunk; the projection on top reads
    # the per-row tables and the piece records of the same call
    from gpu_util import TOL, rel_err
    from paper_2602_24044_amd.runtime import bf16_tensor_to_bits
    T = 5 * 1024 + 77
    ids = np.full(T, -1, dtype=np.int32)
    cuts = [0, 5, 1023, 1024, 1025, 2047, 2049, 3072, 3073, 3500, 4096 + 31, 4096 + 32, 4096 + 33, 5120, 5121, T]
    for k, (b, e) in enumerate(zip(cuts[:-1], cuts[1:])):
        ids[b:e] = [0, 1, 2, -1, 3, 7][k % 6]            # adapter 7 is never loaded
    ranks = {0: 8, 1: 16, 2: 32, 3: 8, 7: 8}
    w = wl.custom("runs_chunks", 31, [(128, 96)], ["p"], 6, 32, wl.BUCKET_RUNS, ids, ranks, resident=[0, 1, 2, 3])
    announce(f"bucket runs over several workgroups T={T}")
    sess = Session(w)
    try:
        sess.load(w.resident, slots=[4, 0, 5, 2])
        sess.bucket()
        assert check_segments(sess, w) == oracle.FLAG_NOT_RESIDENT
        out = sess.forward(0)
        torch.cuda.synchronize()
        st, word = B.lora_poll_device_flags(sess.ctx)
        assert st == B.LORA_ERR_NOT_RESIDENT and word == B.LORA_FLAG_NOT_RESIDENT
        served = np.where(ids == 7, -1, ids).astype(np.int32)
        y_ref = oracle.project(w.x[0], w.W[0], served, oracle.adapters_of(w, 0))
        assert rel_err(bf16_tensor_to_bits(out), y_ref) <= TOL
        # the same context, a shorter step through the single-workgroup kernel, then the long one again
        short = torch.from_numpy(ids[:700].copy()).to(sess.device)
        sess.bucket(short)
        w_short = wl.custom("runs_short", 31, [(128, 96)], ["p"], 6, 32, wl.BUCKET_RUNS, ids[:700].copy(), ranks, resident=[])
        assert check_segments(sess, w_short) == 0
        sess.bucket()
        assert check_segments(sess, w) == oracle.FLAG_NOT_RESIDENT
    finally:
        sess.close()
