"""GPU parity of a context whose adapters share a pool of pages (lora_config.n_pages; paper Sec. 2.2: adapters of
different sizes paged into one pool instead of a uniform footprint each): the same projection oracle, the paged slot
oracle for where things sit, and steps across evictions that leave the pool fragmented."""
import numpy as np
import pytest
import torch

import oracle
from gpu_util import TOL, announce, check_segments, rel_err, run_and_check
from paper_2602_24044_amd import binding as B
from paper_2602_24044_amd import workloads as wl
from paper_2602_24044_amd.runtime import Session, bf16_tensor_to_bits

pytestmark = pytest.mark.gpu


def _pages_needed(w, ids=None):
    ids = w.resident if ids is None else ids
    return sum(w.adapters[a].rank // 8 for a in ids)


@pytest.mark.parametrize("path", [B.LORA_PATH_AUTO, B.LORA_PATH_FUSED, B.LORA_PATH_SPLITK])
@pytest.mark.parametrize("packed", [False, True])
def test_decode_step_from_a_pool_that_fits_exactly(path, packed):
    w = wl.config2(shrink=8, n_tokens=300)
    run_and_check(w, path=path, packed=packed, n_pages=_pages_needed(w))


def test_many_adapter_step_and_prefill_step_from_a_pool():
    w = wl.config4(shrink=8, n_tokens=400, n_adapters=96)          # ranks 8 .. 64, sorted map
    run_and_check(w, packed=True, n_pages=_pages_needed(w))
    w = wl.config3(shrink=8, n_req=6, len_div=4)                   # runs map, fused path above 1024 tokens
    run_and_check(w, packed=True, n_pages=_pages_needed(w) + 3)


def test_steps_across_evictions_that_fragment_the_pool():
    # 6 slots over 10 pages; adapters of ranks 8 .. 32 come and go so that free pages end up apart and a load has to
    # send further adapters away; after every load the step must see each token's current adapter, wherever its pages
    # are, and the table must be where the paged slot oracle says
    ranks = {0: 8, 1: 16, 2: 32, 3: 8, 4: 16, 5: 32, 6: 8, 7: 24, 8: 16, 9: 8}
    rng = np.random.default_rng(5)
    T = 200
    w = wl.custom("paged_steps", 77, [(128, 96), (128, 192)], ["p", "q"], 6, 32, wl.BUCKET_SORTED,
                  rng.integers(-1, 10, size=T).astype(np.int32), ranks, resident=[])
    sess = Session(w, n_pages=10)
    tab = oracle.PagedSlotTable(6, 10)
    plan = [[0, 1, 2], [3, 4], [5], [6, 7], [2, 8, 9], [0, 5], [1, 3, 4, 6]]
    try:
        for step, batch in enumerate(plan):
            reqs = [(a, ranks[a], -1) for a in batch]
            want = tab.load(reqs, in_use=batch)
            got = sess.load(batch, in_use=batch)
            assert got == want, (step, got, want)
            assert [B.lora_slot_first_page(sess.ctx, s) for s in range(6)] == tab.first_page
            resident = [a for a in tab.adapter if a >= 0]
            ids = rng.choice(resident + [-1], size=T).astype(np.int32)
            w.token_ids = ids
            sess.bucket(torch.from_numpy(ids).to(sess.device))
            assert check_segments(sess, w) == 0
            for p in range(2):
                out = sess.forward(p)
                torch.cuda.synchronize()
                y_ref = oracle.project(w.x[p], w.W[p], ids, oracle.adapters_of(w, p))
                e = rel_err(bf16_tensor_to_bits(out), y_ref)
                announce(f"paged step {step} batch={batch} pages={tab.first_page} proj {p} rel_err={e:.3e}")
                assert e <= TOL, (step, p, e)
        assert B.lora_poll_device_flags(sess.ctx) == (B.LORA_OK, 0)
    finally:
        sess.close()


def test_the_pool_is_smaller_than_uniform_slots():
    w = wl.config4(shrink=8, n_tokens=64, n_adapters=96)
    uniform = B.lora_slab_bytes(B.make_config(w.proj, w.n_slots, w.max_rank, w.T, w.max_adapter_id))
    pooled = B.lora_slab_bytes(B.make_config(w.proj, w.n_slots, w.max_rank, w.T, w.max_adapter_id,
                                             n_pages=_pages_needed(w)))
    unit = 2 * sum(a + b for a, b in w.proj)
    saved = (w.n_slots * w.max_rank - sum(w.adapters[a].rank for a in w.resident)) * unit
    announce(f"slab bytes uniform={uniform} pooled={pooled} saved={uniform - pooled} expected about {saved}")
    assert 0.9 * saved <= uniform - pooled <= 1.1 * saved


def test_whole_model_context_over_a_pool():
    # several layers: a page holds 8 rank units of every layer's matrices, so an adapter is still one run
    from paper_2602_24044_amd.runtime import ModelSession
    layers = wl.model_layers(wl.qwen_decode(shrink=8, n_tokens=150), 3)
    lw0 = layers[0]
    ms = ModelSession(layers, n_pages=_pages_needed(lw0))
    announce(f"paged model step {lw0.name} layers=3 T={lw0.T} pages={_pages_needed(lw0)}")
    try:
        ms.load(lw0.resident)
        ms.step()
        torch.cuda.synchronize()
        for l, lw in enumerate(ms.layers):
            for p in range(len(lw.proj)):
                y_ref = oracle.project(lw.x[p], lw.W[p], lw.token_ids, oracle.adapters_of(lw, p), bias=lw.bias_of(p))
                assert rel_err(bf16_tensor_to_bits(ms.out[l][p]), y_ref) <= TOL, (l, p)
        assert B.lora_poll_device_flags(ms.ctx) == (B.LORA_OK, 0)
    finally:
        ms.close()
