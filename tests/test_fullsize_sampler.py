"""The sampler of the full-size GPU parity tests must reach every unit a kernel could get wrong as a whole."""
import numpy as np

from gpu_util import BLOCK, TAIL_ROWS, stratified_samples


def test_the_sampler_reaches_every_block_segment_and_tail_row():
    rng = np.random.default_rng(0)
    T, d_out = 1500, 700
    perm = rng.permutation(T).astype(np.int32)
    seg_start = np.array([0, 3, 4, 900, T])
    ts, ns = stratified_samples(rng, perm, seg_start, 4, T, d_out, n_uniform=0)
    inv = np.empty(T, np.int64)
    inv[perm] = np.arange(T)
    ps = inv[ts]
    blocks = {(int(p) // BLOCK, int(c) // BLOCK) for p, c in zip(ps, ns)}
    assert blocks == {(r, c) for r in range(-(-T // BLOCK)) for c in range(-(-d_out // BLOCK))}
    for s in range(4):
        assert np.any((ps >= seg_start[s]) & (ps < seg_start[s + 1]))
    assert set(range(T - TAIL_ROWS, T)) <= set(int(p) for p in ps)
    assert ns.min() >= 0 and ns.max() < d_out
