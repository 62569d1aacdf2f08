"""GPU parity of the whole-model form: one context with several layers (one slot table, one segment map per step, a
slot holds an adapter's matrices of every layer), every (layer, projection) against the oracle."""
import numpy as np
import pytest
import torch

import oracle
from gpu_util import TOL, announce, rel_err
from paper_2602_24044_amd import binding as B
from paper_2602_24044_amd import workloads as wl
from paper_2602_24044_amd.runtime import ModelSession, bf16_tensor_to_bits

pytestmark = pytest.mark.gpu


def _check_all(ms, outs=None, ids=None):
    worst = 0.0
    for l, lw in enumerate(ms.layers):
        for p in range(len(lw.proj)):
            out = ms.out[l][p] if outs is None else outs[l][p]
            y_ref = oracle.project(lw.x[p], lw.W[p], lw.token_ids if ids is None else ids, oracle.adapters_of(lw, p),
                                   bias=lw.bias_of(p))
            e = rel_err(bf16_tensor_to_bits(out), y_ref)
            assert e <= TOL, (l, p, e)
            worst = max(worst, e)
    return worst


@pytest.mark.parametrize("path,engine,packed_host", [
    (B.LORA_PATH_AUTO, B.LORA_COPY_AUTO, True), (B.LORA_PATH_FUSED, B.LORA_COPY_KERNEL, True),
    (B.LORA_PATH_SPLITK, B.LORA_COPY_ENGINE, True), (B.LORA_PATH_AUTO, B.LORA_COPY_AUTO, False),
    (B.LORA_PATH_AUTO, B.LORA_COPY_ENGINE, False)])
def test_every_layer_reads_its_own_part_of_the_slots(path, engine, packed_host):
    # an adapter kept as one host buffer travels as one run per layer, one kept matrix by matrix as many; by the
    # copy engine, by the copy kernel, or by whichever the run lengths select
    layers = wl.model_layers(wl.qwen_decode(shrink=8, n_tokens=150), 3)      # with the q, k, v bias of that family
    announce(f"model step {layers[0].name} layers={len(layers)} T={layers[0].T} path={path} engine={engine} "
             f"packed_host={packed_host}")
    ms = ModelSession(layers, path=path, packed_host=packed_host)
    try:
        B.lora_set_tuning(ms.ctx, B.LORA_TUNE_COPY_ENGINE, engine)
        ms.load(layers[0].resident)
        ms.step()
        torch.cuda.synchronize()
        announce(f"  worst rel_err {_check_all(ms):.3e}")
        st, word = B.lora_poll_device_flags(ms.ctx)
        assert st == B.LORA_OK and word == 0
    finally:
        ms.close()


def test_step_behind_a_load_on_another_stream():
    # step 1 runs with the resident set; the load that follows on a copy stream evicts adapters step 1 still reads
    # and brings in the ones step 2 needs; step 2 is enqueued on the compute stream straight away.  Layer l of
    # step 2 may only start once layer l's copies have landed, and no copy may land before step 1 has finished.
    base = wl.config5(shrink=8, prefill_len=300, n_decode=100, population=40, n_slots=32, n_missing=6)
    layers = wl.model_layers(base, 4)
    announce(f"model load behind compute {base.name} layers=4 T={base.T} missing={base.missing}")
    ms = ModelSession(layers)
    compute, copy = torch.cuda.Stream(), torch.cuda.Stream()
    try:
        ms.load(base.resident, stream=copy)
        # step 1: the tokens of the adapters that are not resident yet use the resident adapters that step 2 does
        # not need instead, i.e. the ones the load is going to evict
        idle = sorted(set(base.resident) - set(base.distinct_adapters()))
        assert len(idle) >= len(base.missing)
        ids1 = base.token_ids.copy()
        pos = np.flatnonzero(np.isin(ids1, base.missing))
        ids1[pos] = np.array(idle, dtype=np.int32)[np.arange(pos.size) % len(idle)]
        ms.ids = torch.from_numpy(ids1).to(ms.device)
        with torch.cuda.stream(compute):
            ms.step(stream=compute)
            outs1 = [[t.clone() for t in row] for row in ms.out]
        res = ms.load(base.missing, in_use=base.distinct_adapters(), stream=copy)
        assert all(copied for _, copied in res)
        assert sum(B.lora_slot_of(ms.ctx, a) < 0 for a in idle) == len(base.missing)     # step 1's adapters left
        ms.ids = torch.from_numpy(base.token_ids).to(ms.device)
        with torch.cuda.stream(compute):
            ms.step(stream=compute)
        torch.cuda.synchronize()
        announce(f"  step 1 worst rel_err {_check_all(ms, outs=outs1, ids=ids1):.3e}")
        announce(f"  step 2 worst rel_err {_check_all(ms):.3e}")
        st, word = B.lora_poll_device_flags(ms.ctx)
        assert st == B.LORA_OK and word == 0
    finally:
        ms.close()


def test_many_layers():
    # 40 layers of small shapes: the last layers sit far into every slot; only the first, a middle and the last
    # layer are compared (every layer is computed)
    layers = wl.model_layers(wl.config2(shrink=16, n_tokens=96), 40)
    announce(f"model step {layers[0].name} layers={len(layers)} T={layers[0].T}")
    ms = ModelSession(layers)
    try:
        ms.load(layers[0].resident)
        ms.step()
        torch.cuda.synchronize()
        for l in (0, 17, 39):
            lw = layers[l]
            for p in range(len(lw.proj)):
                y_ref = oracle.project(lw.x[p], lw.W[p], lw.token_ids, oracle.adapters_of(lw, p))
                assert rel_err(bf16_tensor_to_bits(ms.out[l][p]), y_ref) <= TOL, (l, p)
        st, word = B.lora_poll_device_flags(ms.ctx)
        assert st == B.LORA_OK and word == 0
    finally:
        ms.close()


def test_gated_mlp_of_every_layer_reads_that_layers_part_of_the_slots():
    # silu(gate) * up of each layer in one call per layer (lora_model_forward_glu): layer l's W, x and the layer-l
    # matrices of the adapters; a wrong layer offset would pick another layer's A and B
    layers = wl.model_layers(wl.config2(shrink=8, n_tokens=300), 3)
    g, u = layers[0].proj_names.index("gate"), layers[0].proj_names.index("up")
    announce(f"model glu {layers[0].name} layers={len(layers)} T={layers[0].T}")
    ms = ModelSession(layers)
    try:
        ms.load(layers[0].resident)
        ms.bucket()
        for l, lw in enumerate(layers):
            out = ms.forward_glu(l, g, u)
            torch.cuda.synchronize()
            h_ref = oracle.gated(lw.x[g], lw.W[g], lw.W[u], lw.token_ids, oracle.adapters_of(lw, g), oracle.adapters_of(lw, u))
            e = rel_err(bf16_tensor_to_bits(out), h_ref)
            announce(f"  layer {l} launches={B.lora_last_launches(ms.ctx)} rel_err={e:.3e}")
            assert e <= TOL, (l, e)
        with pytest.raises(B.LoraError) as err:
            B.lora_model_forward_glu(ms.ctx, len(layers), g, u, ms.x[0][g].data_ptr(), ms.W[0][g].data_ptr(),
                                     ms.W[0][u].data_ptr(), ms.seg, out.data_ptr())
        assert err.value.status == B.LORA_ERR_INVALID_ARG
        assert B.lora_poll_device_flags(ms.ctx) == (B.LORA_OK, 0)
    finally:
        ms.close()
