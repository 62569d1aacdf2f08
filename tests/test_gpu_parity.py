"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on the same seeded
inputs.  Segment maps bit-exact; outputs max|y - y_ref| / max|y_ref| <= 5e-3 per projection."""
import numpy as np
import pytest
import torch

import oracle
from gpu_util import TOL, announce, check_segments, rel_err, run_and_check
from paper_2602_24044_amd import binding as B
from paper_2602_24044_amd import workloads as wl
from paper_2602_24044_amd.runtime import Session, bf16_tensor_to_bits

pytestmark = pytest.mark.gpu

PATHS = [B.LORA_PATH_AUTO, B.LORA_PATH_FUSED, B.LORA_PATH_SPLITK]


@pytest.mark.parametrize("path", PATHS)
def test_config1_tiny(path):
    run_and_check(wl.config1(), path=path)


@pytest.mark.parametrize("path", PATHS)
@pytest.mark.parametrize("n_tokens", [256, 300])
def test_config2_decode_reduced(path, n_tokens):
    run_and_check(wl.config2(shrink=8, n_tokens=n_tokens), path=path)


@pytest.mark.parametrize("path", [B.LORA_PATH_AUTO, B.LORA_PATH_FUSED])
def test_config3_prefill_reduced(path):
    w = wl.config3(shrink=8, n_req=12, len_div=4)
    assert w.T > 1024
    run_and_check(w, path=path)


def test_config3_prefill_short_splitk():
    w = wl.config3(shrink=8, n_req=6, len_div=8)
    assert w.T <= 1024
    run_and_check(w, path=B.LORA_PATH_SPLITK)


@pytest.mark.parametrize("path", PATHS)
def test_config4_many_adapters_reduced(path):
    run_and_check(wl.config4(shrink=8), path=path)


@pytest.mark.parametrize("path", PATHS)
def test_config5_mixed_with_loads_reduced(path):
    w = wl.config5(shrink=8, prefill_len=700, n_decode=200, population=96, n_slots=48, n_missing=8)
    run_and_check(w, path=path)


@pytest.mark.parametrize("path", PATHS)
@pytest.mark.parametrize("packed", [False, True])
def test_qwen_shapes_decode_reduced(path, packed):
    # hidden 896, intermediate 4736, kv 128: ragged last tiles along N for every tile width, K not a power of two
    run_and_check(wl.qwen_decode(shrink=4, n_tokens=200), path=path, packed=packed)


def test_qwen_shapes_prefill_runs_reduced():
    w = wl.qwen_decode(shrink=4, n_tokens=1300, mode=wl.BUCKET_RUNS)
    run_and_check(w, path=B.LORA_PATH_AUTO, packed=True)


@pytest.mark.parametrize("engine", [B.LORA_COPY_AUTO, B.LORA_COPY_KERNEL, B.LORA_COPY_ENGINE])
@pytest.mark.parametrize("packed_host", [False, True])
def test_adapter_copies_by_engine_kernel_and_host_layout(engine, packed_host):
    # mixed ranks below S_max: the adapters sit packed at their own rank in their slots; loads with evictions
    w = wl.config5(shrink=8, prefill_len=300, n_decode=100, population=40, n_slots=32, n_missing=6)
    announce(f"copies {w.name} engine={engine} packed_host={packed_host}")
    s = Session(w, packed_host=packed_host)
    try:
        B.lora_set_tuning(s.ctx, B.LORA_TUNE_COPY_ENGINE, engine)
        s.load(w.resident)
        s.load(w.missing, in_use=w.distinct_adapters())
        s.bucket()
        assert check_segments(s, w) == 0
        for g in s.packed_groups():
            s.forward_group(g) if len(g) > 1 else s.forward(g[0])
        torch.cuda.synchronize()
        for p in range(len(w.proj)):
            y_ref = oracle.project(w.x[p], w.W[p], w.token_ids, oracle.adapters_of(w, p))
            assert rel_err(bf16_tensor_to_bits(s.out[p]), y_ref) <= TOL
    finally:
        s.close()


@pytest.mark.parametrize("path", PATHS)
def test_bias_is_added_and_can_be_removed(path):
    # the q, k, v projections of the Qwen2.5 family have a bias: added before the rounding, for rows with and
    # without an adapter; removing it restores the bias-free result
    w = wl.qwen_decode(shrink=4, n_tokens=300)
    w.token_ids[::5] = -1
    announce(f"bias on/off {w.name} T={w.T} path={path}")
    s = Session(w, path=path)
    try:
        s.load(w.resident)
        s.bucket()
        g = [w.proj_names.index(nm) for nm in ("q", "k", "v")]
        assert all(w.bias_of(p) is not None for p in g)
        for packed in (True, False):
            if packed:
                s.forward_group(g)
            else:
                for p in g:
                    s.forward(p)
            torch.cuda.synchronize()
            for p in g:
                ad = oracle.adapters_of(w, p)
                with_b = oracle.project(w.x[p], w.W[p], w.token_ids, ad, bias=w.bias_of(p))
                without = oracle.project(w.x[p], w.W[p], w.token_ids, ad)
                got = bf16_tensor_to_bits(s.out[p])
                assert rel_err(got, with_b) <= TOL
                assert rel_err(got, without) > 10 * TOL          # the bias is far outside the tolerance
        for p in g:
            B.lora_set_bias(s.ctx, p, 0)
        s.forward_group(g)
        torch.cuda.synchronize()
        for p in g:
            without = oracle.project(w.x[p], w.W[p], w.token_ids, oracle.adapters_of(w, p))
            assert rel_err(bf16_tensor_to_bits(s.out[p]), without) <= TOL
    finally:
        s.close()


@pytest.mark.parametrize("mode", [wl.BUCKET_SORTED, wl.BUCKET_RUNS])
def test_poorly_filled_last_round_takes_the_split_path(mode):
    # 18 x 16 tiles of 256 x 256: one full round of 256 and 32 more.  The fused launch stops after 16 row tiles and
    # the last 356 rows go through split-K + reduce; both parts must agree with the oracle.
    rng = np.random.default_rng(11)
    T = 17 * 256 + 100
    ids = rng.integers(-1, 6, size=T).astype(np.int32)
    if mode == wl.BUCKET_RUNS:
        ids = np.sort(ids)
    w = wl.custom("tail_rows", 11, [(512, 4096)], ["p"], 8, 32, mode, ids, {i: [8, 16, 32][i % 3] for i in range(6)})
    sess = Session(w)
    try:
        sess.load(w.resident)
        sess.bucket()
        assert check_segments(sess, w) == 0
        out = sess.forward(0)
        torch.cuda.synchronize()
        launches = B.lora_last_launches(sess.ctx)
        announce(f"tail rows mode={mode} launches={launches}")
        assert "gemm_fused_staged_256x256x64_w8" in launches and "reduce_expand" in launches, launches
        y_ref = oracle.project(w.x[0], w.W[0], w.token_ids, oracle.adapters_of(w, 0))
        e = rel_err(bf16_tensor_to_bits(out), y_ref)
        announce(f"  rel_err={e:.3e}")
        assert e <= TOL
    finally:
        sess.close()


@pytest.mark.parametrize("split_k", [1, 2, 3, 16])
def test_split_k_values(split_k):
    run_and_check(wl.config2(shrink=8, n_tokens=130), path=B.LORA_PATH_SPLITK, split_k=split_k)


def _int_workload(seed, T, d_in, d_out, ranks, n_slots):
    """Small-integer inputs: every partial sum is exact in fp32 and v is exact in bf16, so the GPU must
    reproduce the rounded oracle bit for bit whatever its summation order."""
    rng = np.random.default_rng(seed)
    ids = rng.integers(-1, len(ranks), size=T).astype(np.int32)
    w = wl.custom("int_exact", seed, [(d_in, d_out)], ["p"], n_slots, max(max(ranks), 8), wl.BUCKET_SORTED, ids,
                  {i: r for i, r in enumerate(ranks)}, scales={i: 2.0 ** (i % 3 - 1) for i in range(len(ranks))})
    w.W[0] = wl.to_bf16_bits(rng.integers(-2, 3, size=(d_out, d_in)).astype(np.float32))
    w.x[0] = wl.to_bf16_bits(rng.integers(-1, 2, size=(T, d_in)).astype(np.float32))
    for a in w.adapters.values():
        if a.rank > 0:
            a.A[0] = wl.to_bf16_bits(rng.integers(-1, 2, size=(a.rank, d_in)).astype(np.float32))
            a.B[0] = wl.to_bf16_bits(rng.integers(-2, 3, size=(d_out, a.rank)).astype(np.float32) * 0.25)
    return w


@pytest.mark.parametrize("path", PATHS)
def test_small_integer_inputs_are_bit_exact(path):
    w = _int_workload(5, T=77, d_in=128, d_out=264, ranks=[8, 16, 0, 32, 8], n_slots=5)
    announce(f"int exact path={path}")
    sess = Session(w, path=path)
    try:
        sess.load(w.resident)
        sess.bucket()
        out = sess.forward(0)
        torch.cuda.synchronize()
        y_ref = oracle.project(w.x[0], w.W[0], w.token_ids, oracle.adapters_of(w, 0))
        assert np.max(np.abs(y_ref)) < 2.0 ** 20
        want = wl.to_bf16_bits(y_ref.astype(np.float32))
        got = bf16_tensor_to_bits(out)
        # +0 and -0 are the same value
        assert np.array_equal(wl.bf16_bits_to_f32(got), wl.bf16_bits_to_f32(want))
    finally:
        sess.close()


@pytest.mark.parametrize("path", PATHS)
def test_lora_term_alone(path):
    # W = 0: the tolerance is then relative to the LoRA term itself
    w = wl.config2(shrink=8, n_tokens=200)
    for p in range(len(w.W)):
        w.W[p] = np.zeros_like(w.W[p])
    run_and_check(w, path=path)


@pytest.mark.parametrize("path", PATHS)
def test_zero_adapters_equal_the_gpu_base_run(path):
    w = wl.config2(shrink=8, n_tokens=96)
    sess = Session(w, path=path)
    try:
        sess.load(w.resident)
        # base-only reference run on the GPU: every token without adapter
        ids_none = torch.full((w.T,), -1, dtype=torch.int32, device=sess.device)
        sess.bucket(ids_none)
        base = [bf16_tensor_to_bits(sess.forward(p)).copy() for p in range(len(w.proj))]
        # B = 0 for every adapter
        wz = wl.config2(shrink=8, n_tokens=96)
        for a in wz.adapters.values():
            a.B = [np.zeros_like(b) for b in a.B]
        sz = Session(wz, path=path)
        try:
            sz.load(wz.resident)
            sz.bucket()
            for p in range(len(w.proj)):
                got = bf16_tensor_to_bits(sz.forward(p))
                assert np.array_equal(wl.bf16_bits_to_f32(got), wl.bf16_bits_to_f32(base[p]))
        finally:
            sz.close()
    finally:
        sess.close()


def test_rank0_and_backbone_only_tokens():
    rng = np.random.default_rng(3)
    ids = rng.integers(-1, 4, size=150).astype(np.int32)
    w = wl.custom("rank0", 13, [(256, 136)], ["p"], 4, 16, wl.BUCKET_SORTED, ids, {0: 8, 1: 0, 2: 16, 3: 0})
    for path in PATHS:
        run_and_check(w, path=path)


EDGE_IDS = {
    "one_token": np.array([2], dtype=np.int32),
    "all_same": np.full(100, 3, dtype=np.int32),
    "all_distinct": np.arange(40, dtype=np.int32),
    "all_backbone": np.full(70, -1, dtype=np.int32),
    "ragged_65": (np.arange(65) % 7).astype(np.int32),
    "alternating": (np.arange(257) % 2).astype(np.int32),
}


@pytest.mark.parametrize("name", sorted(EDGE_IDS))
@pytest.mark.parametrize("mode", [wl.BUCKET_SORTED, wl.BUCKET_RUNS])
def test_edge_batches(name, mode):
    ids = EDGE_IDS[name]
    w = wl.custom(f"edge_{name}", 17, [(128, 72)], ["p"], 40, 16, mode, ids, {i: (8 if i % 2 else 16) for i in range(40)})
    for path in (B.LORA_PATH_FUSED, B.LORA_PATH_SPLITK):
        run_and_check(w, path=path)


def test_empty_batch():
    w = wl.custom("empty", 1, [(64, 64)], ["p"], 2, 8, wl.BUCKET_SORTED, np.zeros(0, np.int32), {0: 8, 1: 8})
    sess = Session(w, max_tokens=8)
    try:
        sess.load(w.resident)
        sess.bucket()
        perm, seg_start, seg_slot, n_seg = sess.read_segments()
        assert n_seg == 0 and seg_start.tolist() == [0] and perm.size == 0
        sess.forward(0)      # no-op
        torch.cuda.synchronize()
    finally:
        sess.close()


def test_non_resident_token_sets_flag_and_runs_backbone_only():
    ids = np.array([0, 1, 2, 1, 0, 5], dtype=np.int32)
    w = wl.custom("nonres", 19, [(128, 64)], ["p"], 2, 8, wl.BUCKET_SORTED, ids, {i: 8 for i in range(6)})
    sess = Session(w)
    try:
        sess.load([0, 2])                      # adapters 1 and 5 are not resident
        sess.bucket()
        flags = check_segments(sess, w)
        assert flags == oracle.FLAG_NOT_RESIDENT
        out = sess.forward(0)
        torch.cuda.synchronize()
        st, word = B.lora_poll_device_flags(sess.ctx)
        assert st == B.LORA_ERR_NOT_RESIDENT and word & B.LORA_FLAG_NOT_RESIDENT
        st, word = B.lora_poll_device_flags(sess.ctx)
        assert st == B.LORA_OK and word == 0   # read-and-clear
        served = np.where(np.isin(ids, [0, 2]), ids, -1).astype(np.int32)
        y_ref = oracle.project(w.x[0], w.W[0], served, oracle.adapters_of(w, 0))
        assert rel_err(bf16_tensor_to_bits(out), y_ref) <= TOL
    finally:
        sess.close()


def test_eviction_reloads_slot_contents():
    # two slots, three adapters used in turn: each step must see the adapter loaded last into its slot
    ids_all = {a: np.full(33, a, dtype=np.int32) for a in range(3)}
    w = wl.custom("evict", 23, [(128, 80)], ["p"], 2, 16, wl.BUCKET_SORTED, ids_all[0], {0: 8, 1: 16, 2: 8})
    sess = Session(w)
    tab = oracle.SlotTable(2)
    try:
        for a in [0, 1, 2, 0, 1, 1, 2]:
            got = sess.load([a], in_use=[a])
            want = tab.load([(a, w.adapters[a].rank, -1)], [a])
            assert got == want
            ids = ids_all[a]
            sess.bucket(torch.from_numpy(ids).to(sess.device))
            out = sess.forward(0)
            torch.cuda.synchronize()
            y_ref = oracle.project(w.x[0], w.W[0], ids, oracle.adapters_of(w, 0))
            assert rel_err(bf16_tensor_to_bits(out), y_ref) <= TOL
    finally:
        sess.close()


def test_results_are_deterministic_run_to_run():
    w = wl.config4(shrink=8, n_tokens=200, n_adapters=64)
    for path in (B.LORA_PATH_FUSED, B.LORA_PATH_SPLITK):
        sess = Session(w, path=path)
        try:
            sess.load(w.resident)
            sess.bucket()
            first = [bf16_tensor_to_bits(sess.forward(p)).copy() for p in range(len(w.proj))]
            for _ in range(3):
                sess.bucket()
                for p in range(len(w.proj)):
                    assert np.array_equal(bf16_tensor_to_bits(sess.forward(p)), first[p])
        finally:
            sess.close()


def test_stale_segment_map_is_rejected():
    w = wl.config1()
    sess = Session(w)
    try:
        sess.load(w.resident)
        old = sess.bucket()
        sess.bucket()
        with pytest.raises(B.LoraError) as e:
            B.lora_layer_forward(sess.ctx, 0, sess.x[0].data_ptr(), sess.W[0].data_ptr(), old, sess.out[0].data_ptr())
        assert e.value.status == B.LORA_ERR_INVALID_ARG
        with pytest.raises(B.LoraError):
            B.lora_layer_forward(sess.ctx, 3, sess.x[0].data_ptr(), sess.W[0].data_ptr(), sess.seg, sess.out[0].data_ptr())
    finally:
        sess.close()


# ---- packed projections (q|k|v and gate|up through lora_layer_forward_group) ----

@pytest.mark.parametrize("path", PATHS)
@pytest.mark.parametrize("n_tokens", [256, 300])
def test_packed_config2_decode_reduced(path, n_tokens):
    run_and_check(wl.config2(shrink=8, n_tokens=n_tokens), path=path, packed=True)


@pytest.mark.parametrize("path", [B.LORA_PATH_AUTO, B.LORA_PATH_FUSED])
def test_packed_config3_prefill_reduced(path):
    run_and_check(wl.config3(shrink=8), path=path, packed=True)


@pytest.mark.parametrize("path", PATHS)
def test_packed_config4_many_adapters_reduced(path):
    run_and_check(wl.config4(shrink=8), path=path, packed=True)


@pytest.mark.parametrize("path", PATHS)
def test_packed_config5_mixed_with_loads_reduced(path):
    run_and_check(wl.config5(shrink=8), path=path, packed=True)


def test_packed_equals_separate_calls_bit_for_bit_on_the_fused_path():
    # the fused path has no split-K: a projection's result may not depend on what it is packed with
    w = wl.config2(shrink=8, n_tokens=300)
    a = Session(w, path=B.LORA_PATH_FUSED)
    b = Session(w, path=B.LORA_PATH_FUSED)
    try:
        for s in (a, b):
            s.load(w.resident)
            s.bucket()
        for g in a.packed_groups():
            if len(g) > 1:
                a.forward_group(g)
            else:
                a.forward(g[0])
        for p in range(len(w.proj)):
            b.forward(p)
        torch.cuda.synchronize()
        for p in range(len(w.proj)):
            assert torch.equal(a.out[p].view(torch.int16), b.out[p].view(torch.int16)), w.proj_names[p]
    finally:
        a.close()
        b.close()


def test_group_with_one_shared_input_tensor():
    # q, k, v reading the very same x tensor
    w = wl.config2(shrink=8, n_tokens=256)
    s = Session(w)
    try:
        s.load(w.resident)
        s.bucket()
        g = [w.proj_names.index(nm) for nm in ("q", "k", "v")]
        x = s.x[g[0]]
        B.lora_layer_forward_group(s.ctx, g, [x.data_ptr()] * 3, [s.W[p].data_ptr() for p in g], s.seg,
                                   [s.out[p].data_ptr() for p in g], torch.cuda.current_stream().cuda_stream)
        torch.cuda.synchronize()
        for p in g:
            y_ref = oracle.project(w.x[g[0]], w.W[p], w.token_ids, oracle.adapters_of(w, p))
            assert rel_err(bf16_tensor_to_bits(s.out[p]), y_ref) <= TOL
    finally:
        s.close()


def test_launches_do_not_depend_on_the_context_size():
    # a context sized for more tokens has more scratch; the same step must take the same kernels (a cost model that
    # priced a single K range like a split once sent gate|up down the split path as soon as scratch allowed two)
    w = wl.config2(shrink=2, n_tokens=256)
    seen = []
    for max_tokens in (None, 4096):
        s = Session(w, max_tokens=max_tokens)
        try:
            s.load(w.resident)
            s.bucket()
            per_group = []
            for g in s.packed_groups():
                s.forward_group(g) if len(g) > 1 else s.forward(g[0])
                per_group.append(tuple(B.lora_last_launches(s.ctx)))
            torch.cuda.synchronize()
            seen.append(per_group)
        finally:
            s.close()
    announce(f"launches per call: {seen[0]}")
    assert seen[0] == seen[1]
