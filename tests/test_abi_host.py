"""CPU-only checks of the C-ABI library: it loads, exports what the header declares, validates
arguments, and its host-side slot table follows the slot-table oracle."""
import os
import re

import numpy as np
import pytest

import oracle
from conftest import GOLDEN, ROOT
from paper_2602_24044_amd import binding as B
from test_oracle_slots import parse_trace


def _host_ctx(n_slots=3, max_rank=32, proj=((64, 64),), max_adapter_id=63, n_pages=0):
    cfg = B.make_config(proj, n_slots, max_rank, 16, max_adapter_id, flags=B.LORA_CREATE_HOST_ONLY, n_pages=n_pages)
    return B.lora_create(cfg)


def test_library_exports_every_declared_symbol():
    import ctypes
    hdr = open(os.path.join(ROOT, "include", "lora_mi355.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    declared = set(re.findall(r"\b(lora_[a-z0-9_]+)\s*\(", hdr))
    assert declared == set(B.EXPORTS)
    lib = ctypes.CDLL(B.LIB_PATH)
    for name in declared:
        assert hasattr(lib, name), name


def test_status_strings():
    assert B.lora_status_string(B.LORA_OK) == "ok"
    assert "slot" in B.lora_status_string(B.LORA_ERR_SLOTS_EXHAUSTED)


def test_config_validation():
    bad = [
        dict(proj=((60, 64),)),            # d_in not a multiple of 64
        dict(proj=((64, 12),)),            # d_out not a multiple of 8
        dict(max_rank=12),                 # S_max not a multiple of 8
        dict(max_rank=128),
    ]
    for kw in bad:
        args = dict(proj=((64, 64),), n_slots=2, max_rank=8, max_tokens=4, max_adapter_id=3)
        args.update(kw)
        cfg = B.make_config(args["proj"], args["n_slots"], args["max_rank"], args["max_tokens"],
                            args["max_adapter_id"], flags=B.LORA_CREATE_HOST_ONLY)
        assert B.lora_slab_bytes(cfg) == 0
        with pytest.raises(B.LoraError) as e:
            B.lora_create(cfg)
        assert e.value.status == B.LORA_ERR_SHAPE
    cfg = B.make_config(((64, 64),), 0, 8, 4, 3, flags=B.LORA_CREATE_HOST_ONLY)
    with pytest.raises(B.LoraError) as e:
        B.lora_create(cfg)
    assert e.value.status == B.LORA_ERR_INVALID_ARG


def test_slab_bytes_covers_the_slot_region():
    proj = ((4096, 4096), (4096, 1024))
    cfg = B.make_config(proj, 32, 32, 256, 31)
    slot_region = 32 * 32 * sum(a + b for a, b in proj) * 2   # A_max x S_max x sum(d_in + d_out) x 2 bytes
    assert B.lora_slab_bytes(cfg) >= slot_region
    # without device memory a real context cannot be created
    with pytest.raises(B.LoraError) as e:
        B.lora_create(cfg)
    assert e.value.status == B.LORA_ERR_INVALID_ARG


def test_hand_traced_sequence_on_the_library():
    n_slots, calls = parse_trace(os.path.join(GOLDEN, "slot_trace.txt"))
    ctx = _host_ctx(n_slots)
    try:
        for in_use, reqs, exp, state in calls:
            descs = [dict(adapter_id=a, rank=r, scale=1.0, slot=s) for (a, r, s) in reqs]
            if exp is None:
                with pytest.raises(B.LoraError) as e:
                    B.lora_slots_load(ctx, descs, in_use)
                assert e.value.status == B.LORA_ERR_SLOTS_EXHAUSTED
            else:
                assert B.lora_slots_load(ctx, descs, in_use) == exp
            assert [B.lora_slot_adapter(ctx, s) for s in range(n_slots)] == state
    finally:
        B.lora_destroy(ctx)


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_random_sequences_match_the_slot_oracle(seed):
    rng = np.random.default_rng(seed)
    n_slots, n_ids = 6, 20
    ctx = _host_ctx(n_slots)
    tab = oracle.SlotTable(n_slots)
    try:
        for _ in range(300):
            k = int(rng.integers(1, 4))
            ads = rng.choice(n_ids, size=k, replace=False)
            reqs = []
            for a in ads:
                slot = int(rng.integers(0, n_slots)) if rng.random() < 0.1 else -1
                reqs.append((int(a), int(rng.choice([0, 8, 16, 32])), slot))
            in_use = [int(v) for v in rng.choice(n_ids, size=int(rng.integers(0, 7)), replace=False)]
            descs = [dict(adapter_id=a, rank=r, scale=1.0, slot=s) for (a, r, s) in reqs]
            try:
                want = tab.load(reqs, in_use)
            except oracle.SlotsExhausted:
                with pytest.raises(B.LoraError) as e:
                    B.lora_slots_load(ctx, descs, in_use)
                assert e.value.status == B.LORA_ERR_SLOTS_EXHAUSTED
            else:
                assert B.lora_slots_load(ctx, descs, in_use) == want
            assert [B.lora_slot_adapter(ctx, s) for s in range(n_slots)] == tab.adapter
            m = tab.id2slot(n_ids)
            assert [B.lora_slot_of(ctx, i) for i in range(n_ids)] == m.tolist()
    finally:
        B.lora_destroy(ctx)


def test_load_argument_errors():
    ctx = _host_ctx(n_slots=2, max_rank=16, max_adapter_id=7)
    try:
        cases = [
            (dict(adapter_id=9, rank=8, scale=1.0), B.LORA_ERR_ID_RANGE),
            (dict(adapter_id=1, rank=32, scale=1.0), B.LORA_ERR_RANK_EXCEEDS_SMAX),
            (dict(adapter_id=1, rank=12, scale=1.0), B.LORA_ERR_SHAPE),
            (dict(adapter_id=1, rank=8, scale=1.0, slot=2), B.LORA_ERR_SLOT_RANGE),
            (dict(adapter_id=1, rank=-8, scale=1.0), B.LORA_ERR_INVALID_ARG),
        ]
        for d, status in cases:
            with pytest.raises(B.LoraError) as e:
                B.lora_slots_load(ctx, [d])
            assert e.value.status == status
            assert [B.lora_slot_adapter(ctx, s) for s in range(2)] == [-1, -1]
        with pytest.raises(B.LoraError) as e:
            B.lora_slots_load(ctx, [dict(adapter_id=1, rank=8, scale=1.0)], in_use=[99])
        assert e.value.status == B.LORA_ERR_ID_RANGE
    finally:
        B.lora_destroy(ctx)


def test_host_only_context_refuses_device_work():
    ctx = _host_ctx()
    try:
        with pytest.raises(B.LoraError) as e:
            B.lora_bucket(ctx, 0, 0, B.LORA_BUCKET_SORTED)
        assert e.value.status == B.LORA_ERR_HIP
    finally:
        B.lora_destroy(ctx)


def test_group_argument_errors():
    ctx = _host_ctx(proj=((64, 64), (64, 128), (128, 64)))
    seg = B.lora_segments()
    try:
        def status(projs):
            n = len(projs)
            with pytest.raises(B.LoraError) as e:
                B.lora_layer_forward_group(ctx, projs, [16] * n, [16] * n, seg, [16] * n)
            return e.value.status
        assert status([]) == B.LORA_ERR_INVALID_ARG                   # at least one projection
        assert status([0, 1, 0, 1, 0]) == B.LORA_ERR_INVALID_ARG      # at most four
        assert status([0, 0]) == B.LORA_ERR_INVALID_ARG               # distinct
        assert status([0, 3]) == B.LORA_ERR_INVALID_ARG               # in range
        assert status([0, 2]) == B.LORA_ERR_SHAPE                     # d_in 64 vs 128
        assert status([0, 1]) == B.LORA_ERR_INVALID_ARG               # no segment map yet
    finally:
        B.lora_destroy(ctx)


def test_gated_pair_argument_errors():
    cfg = B.make_config(((64, 128), (64, 128), (64, 96), (128, 64)), 3, 32, 16, 63, flags=B.LORA_CREATE_HOST_ONLY, n_layers=2)
    ctx = B.lora_create(cfg)
    seg = B.lora_segments()
    try:
        def status(layer, pg, pu):
            with pytest.raises(B.LoraError) as e:
                B.lora_model_forward_glu(ctx, layer, pg, pu, 16, 16, 16, seg, 16)
            return e.value.status
        assert status(2, 0, 1) == B.LORA_ERR_INVALID_ARG              # layers 0 and 1 only
        assert status(-1, 0, 1) == B.LORA_ERR_INVALID_ARG
        assert status(0, 0, 0) == B.LORA_ERR_INVALID_ARG              # two different projections
        assert status(0, 0, 4) == B.LORA_ERR_INVALID_ARG              # in range
        assert status(1, 0, 2) == B.LORA_ERR_SHAPE                    # d_out 128 vs 96
        assert status(1, 0, 3) == B.LORA_ERR_SHAPE                    # d_in 64 vs 128
        assert status(1, 0, 1) == B.LORA_ERR_INVALID_ARG              # no segment map yet
        B.lora_set_bias(ctx, 1, 256, layer=1)                         # a bias on the second projection of layer 1 only
        with pytest.raises(B.LoraError) as e:
            B.lora_layer_forward_glu(ctx, 0, 1, 16, 16, 16, seg, 16)  # layer 0: past the bias rule, stopped by the missing map
        assert e.value.status == B.LORA_ERR_INVALID_ARG
        assert status(1, 0, 1) == B.LORA_ERR_INVALID_ARG
    finally:
        B.lora_destroy(ctx)


def test_bias_argument_errors():
    ctx = _host_ctx(proj=((64, 64), (64, 128)))
    try:
        B.lora_set_bias(ctx, 1, 0)                       # removing a bias that is not set is fine
        B.lora_set_bias(ctx, 0, 4096)                    # host state only: the address is not touched here
        for proj, addr in ((-1, 4096), (2, 4096), (0, 4096 + 8)):
            with pytest.raises(B.LoraError) as e:
                B.lora_set_bias(ctx, proj, addr)
            assert e.value.status == B.LORA_ERR_INVALID_ARG
    finally:
        B.lora_destroy(ctx)


def test_layers_in_the_config():
    proj = ((4096, 4096), (4096, 1024))
    per_layer = 32 * 32 * sum(a + b for a, b in proj) * 2           # one layer's share of the slot region
    one = B.lora_slab_bytes(B.make_config(proj, 32, 32, 256, 31, n_layers=1))
    assert B.lora_slab_bytes(B.make_config(proj, 32, 32, 256, 31, n_layers=0)) == one     # 0 is read as 1
    four = B.lora_slab_bytes(B.make_config(proj, 32, 32, 256, 31, n_layers=4))
    assert abs((four - one) - 3 * per_layer) <= 4096                  # scratch does not grow with the layers
    assert B.lora_slab_bytes(B.make_config(proj, 32, 32, 256, 31, n_layers=257)) == 0
    assert B.lora_slab_bytes(B.make_config(proj, 32, 32, 256, 31, n_layers=-1)) == 0
    # layer arguments of the calls that take one
    cfg = B.make_config(((64, 64),), 3, 32, 16, 63, flags=B.LORA_CREATE_HOST_ONLY, n_layers=2)
    ctx = B.lora_create(cfg)
    try:
        B.lora_set_bias(ctx, 0, 4096, layer=1)
        for layer in (-1, 2):
            with pytest.raises(B.LoraError) as e:
                B.lora_set_bias(ctx, 0, 4096, layer=layer)
            assert e.value.status == B.LORA_ERR_INVALID_ARG
            with pytest.raises(B.LoraError) as e:
                B.lora_model_forward_group(ctx, layer, [0], [16], [16], B.lora_segments(), [16])
            assert e.value.status == B.LORA_ERR_INVALID_ARG
        # the slot table is one for all layers: a load names the adapter once
        assert B.lora_slots_load(ctx, [dict(adapter_id=5, rank=8, scale=1.0)]) == [(0, True)]
        assert B.lora_slot_of(ctx, 5) == 0
    finally:
        B.lora_destroy(ctx)


# ---- slots over a pool of pages (lora_config.n_pages) ----
def test_hand_traced_page_sequence_on_the_library():
    n_slots, n_pages, calls = parse_trace(os.path.join(GOLDEN, "page_trace.txt"))
    ctx = _host_ctx(n_slots, n_pages=n_pages)
    try:
        for in_use, reqs, exp, state, pages in calls:
            descs = [dict(adapter_id=a, rank=r, scale=1.0, slot=s) for (a, r, s) in reqs]
            if exp is None:
                with pytest.raises(B.LoraError) as e:
                    B.lora_slots_load(ctx, descs, in_use)
                assert e.value.status == B.LORA_ERR_SLOTS_EXHAUSTED
            else:
                assert B.lora_slots_load(ctx, descs, in_use) == exp
            assert [B.lora_slot_adapter(ctx, s) for s in range(n_slots)] == state
            assert [B.lora_slot_first_page(ctx, s) for s in range(n_slots)] == pages
    finally:
        B.lora_destroy(ctx)


@pytest.mark.parametrize("seed,n_pages", [(0, 4), (1, 7), (2, 12), (3, 24), (4, 5)])
def test_random_sequences_match_the_paged_slot_oracle(seed, n_pages):
    rng = np.random.default_rng(seed)
    n_slots, n_ids = 6, 20
    ctx = _host_ctx(n_slots, n_pages=n_pages)
    tab = oracle.PagedSlotTable(n_slots, n_pages)
    try:
        for _ in range(400):
            ads = rng.choice(n_ids, size=int(rng.integers(1, 4)), replace=False)
            reqs = [(int(a), int(rng.choice([0, 8, 16, 32])), int(rng.integers(0, n_slots)) if rng.random() < 0.1 else -1)
                    for a in ads]
            in_use = [int(v) for v in rng.choice(n_ids, size=int(rng.integers(0, 7)), replace=False)]
            descs = [dict(adapter_id=a, rank=r, scale=1.0, slot=s) for (a, r, s) in reqs]
            try:
                want = tab.load(reqs, in_use)
            except oracle.SlotsExhausted:
                with pytest.raises(B.LoraError) as e:
                    B.lora_slots_load(ctx, descs, in_use)
                assert e.value.status == B.LORA_ERR_SLOTS_EXHAUSTED
            else:
                assert B.lora_slots_load(ctx, descs, in_use) == want
            assert [B.lora_slot_adapter(ctx, s) for s in range(n_slots)] == tab.adapter
            assert [B.lora_slot_first_page(ctx, s) for s in range(n_slots)] == tab.first_page
            assert [B.lora_slot_of(ctx, i) for i in range(n_ids)] == tab.id2slot(n_ids).tolist()
    finally:
        B.lora_destroy(ctx)


def test_page_pool_in_the_config():
    proj = [(4096, 4096), (4096, 14336)]
    uniform = B.lora_slab_bytes(B.make_config(proj, 384, 64, 512, 400))
    # 384 slots over a pool that holds their adapters at an average rank of 32 instead of 64 each
    pooled = B.lora_slab_bytes(B.make_config(proj, 384, 64, 512, 400, n_pages=384 * 4))
    unit = sum(a + b for a, b in proj) * 2                   # bytes per rank unit
    assert uniform - pooled >= 384 * 32 * unit - 4096 * 384  # the other half of the region, up to alignment
    assert pooled >= 384 * 4 * 8 * unit
    # a pool that cannot hold one adapter of the largest rank is refused; without pages the query says -1
    with pytest.raises(B.LoraError):
        B.lora_create(B.make_config([(64, 64)], 4, 32, 16, 9, flags=B.LORA_CREATE_HOST_ONLY, n_pages=3))
    ctx = _host_ctx()
    try:
        B.lora_slots_load(ctx, [dict(adapter_id=1, rank=8, scale=1.0)])
        assert B.lora_slot_first_page(ctx, 0) == -1
    finally:
        B.lora_destroy(ctx)
