"""GPU parity at the full workload sizes, in the launch configuration bench.py times (automatic path,
q|k|v and gate|up as packed calls) and with one call per projection: segment maps bit-exact against the
oracle, outputs checked on sampled (token, column) pairs that the oracle evaluates one by one.  The samples are
stratified over what a kernel could get wrong as a unit: every 128 x 128 block of the output (so every output tile of every GEMM variant, 128 x 128 to 256 x 256) in the order the
kernels walk the rows (the segment map's order), every segment, and every row of the last 1024 positions (the
range that may leave the fused launch for the split-K path), plus uniform draws and the four corners."""
import numpy as np
import pytest
import torch

import oracle
from gpu_util import TOL, announce, check_segments, stratified_samples
from paper_2602_24044_amd import binding as B
from paper_2602_24044_amd import workloads as wl
from paper_2602_24044_amd.runtime import Session, bf16_tensor_to_bits

pytestmark = pytest.mark.gpu


def _run_full(w, packed=True, n_pages=0):
    announce(f"full-size {w.name} T={w.T} packed={packed} n_pages={n_pages} proj={w.proj}")
    sess = Session(w, n_pages=n_pages)
    try:
        sess.load(w.resident)
        if w.missing:
            sess.load(w.missing, in_use=w.distinct_adapters())
        sess.bucket()
        assert check_segments(sess, w) == 0
        # the segment map the kernels walk, from the oracle (check_segments has just shown the two agree)
        perm, seg_start, _, n_seg, _ = oracle.bucket(w.token_ids, sess.id2slot(), w.mode)
        rng = np.random.default_rng(12345)
        launches = {}
        if packed:
            for g in sess.packed_groups():
                if len(g) > 1:
                    sess.forward_group(g)
                else:
                    sess.forward(g[0])
                for p in g:
                    launches[p] = B.lora_last_launches(sess.ctx)
        for p, (d_in, d_out) in enumerate(w.proj):
            out = sess.out[p]
            if not packed:
                out = sess.forward(p)
                launches[p] = B.lora_last_launches(sess.ctx)
            torch.cuda.synchronize()
            got_all = bf16_tensor_to_bits(out)
            ts, ns = stratified_samples(rng, perm, seg_start, n_seg, w.T, d_out)
            y_ref = oracle.project_at(w.x[p], w.W[p], w.token_ids, oracle.adapters_of(w, p), ts, ns, bias=w.bias_of(p))
            got = wl.bf16_bits_to_f64(got_all[ts, ns])
            # scale of the projection: the largest sampled reference magnitude (a lower bound of max|y_ref|)
            err = float(np.max(np.abs(got - y_ref)) / np.max(np.abs(y_ref)))
            announce(f"  proj {p} {w.proj[p]} launches={launches[p]} samples={ts.shape[0]} rel_err={err:.3e}")
            assert err <= TOL, (p, err)
            assert np.isfinite(wl.bf16_bits_to_f32(got_all)).all()
        st, word = B.lora_poll_device_flags(sess.ctx)
        assert st == B.LORA_OK and word == 0
    finally:
        sess.close()


def test_config2_full():
    _run_full(wl.config2())


def test_config2_full_one_call_per_projection():
    _run_full(wl.config2(), packed=False)


def test_config4_full():
    _run_full(wl.config4())


def test_config4_full_lora_term_alone():
    # W = 0 at the full many-adapter shape: the output is the adapter term alone, which is a few percent of |y|
    # with the backbone in and would hide in the tolerance there
    w = wl.config4()
    for p in range(len(w.proj)):
        w.W[p] = np.zeros_like(w.W[p])
    _run_full(w)


def test_config4_full_from_a_pool_of_pages():
    # the 384 adapters at their own ranks in a pool that fits them exactly (against 384 regions of rank 64)
    w = wl.config4()
    pages = sum(w.adapters[a].rank // 8 for a in w.resident)
    uniform = B.lora_slab_bytes(B.make_config(w.proj, w.n_slots, w.max_rank, w.T, w.max_adapter_id))
    pooled = B.lora_slab_bytes(B.make_config(w.proj, w.n_slots, w.max_rank, w.T, w.max_adapter_id, n_pages=pages))
    announce(f"  slab bytes: uniform slots {uniform / 2**30:.2f} GiB, pool of {pages} pages {pooled / 2**30:.2f} GiB")
    assert pooled < 0.6 * uniform
    _run_full(w, n_pages=pages)


def test_config3_full():
    _run_full(wl.config3())


def test_config5_full():
    _run_full(wl.config5())


def test_qwen_7b_decode_full():
    _run_full(wl.qwen_decode())


def test_whole_model_two_layers_full_size():
    # two layers of 8B shapes in one context: the second layer sits 5 MB x rank into every slot; sampled outputs of
    # both layers
    from paper_2602_24044_amd.runtime import ModelSession
    layers = wl.model_layers(wl.config2(), 2)
    announce(f"model step {layers[0].name} layers=2 T={layers[0].T} (full size)")
    ms = ModelSession(layers)
    rng = np.random.default_rng(5)
    try:
        ms.load(layers[0].resident)
        ms.step()
        torch.cuda.synchronize()
        for l, lw in enumerate(layers):
            for p, (d_in, d_out) in enumerate(lw.proj):
                ts = rng.integers(0, lw.T, size=200).astype(np.int32)
                ns = rng.integers(0, d_out, size=200).astype(np.int32)
                ts[:2], ns[:2] = [0, lw.T - 1], [0, d_out - 1]
                y_ref = oracle.project_at(lw.x[p], lw.W[p], lw.token_ids, oracle.adapters_of(lw, p), ts, ns)
                got = wl.bf16_bits_to_f64(bf16_tensor_to_bits(ms.out[l][p])[ts, ns])
                err = float(np.max(np.abs(got - y_ref)) / np.max(np.abs(y_ref)))
                assert err <= TOL, (l, p, err)
        st, word = B.lora_poll_device_flags(ms.ctx)
        assert st == B.LORA_OK and word == 0
    finally:
        ms.close()


@pytest.mark.parametrize("make", [wl.config2, wl.config3, wl.config5])
def test_gated_gate_up_full(make):
    # silu(gate) * up in one call at full size: stratified samples, each factor evaluated by the oracle on its own
    w = make()
    g, u = w.proj_names.index("gate"), w.proj_names.index("up")
    announce(f"full-size glu {w.name} T={w.T} proj={w.proj[g]}")
    sess = Session(w)
    try:
        sess.load(w.resident)
        if w.missing:
            sess.load(w.missing, in_use=w.distinct_adapters())
        sess.bucket()
        assert check_segments(sess, w) == 0
        perm, seg_start, _, n_seg, _ = oracle.bucket(w.token_ids, sess.id2slot(), w.mode)
        out = sess.forward_glu(g, u)
        torch.cuda.synchronize()
        launches = B.lora_last_launches(sess.ctx)
        got_all = bf16_tensor_to_bits(out)
        ts, ns = stratified_samples(np.random.default_rng(99), perm, seg_start, n_seg, w.T, w.proj[g][1])
        gate = oracle.project_at(w.x[g], w.W[g], w.token_ids, oracle.adapters_of(w, g), ts, ns)
        up = oracle.project_at(w.x[g], w.W[u], w.token_ids, oracle.adapters_of(w, u), ts, ns)
        h_ref = oracle.silu(gate) * up
        got = wl.bf16_bits_to_f64(got_all[ts, ns])
        err = float(np.max(np.abs(got - h_ref)) / np.max(np.abs(h_ref)))
        announce(f"  launches={launches} samples={ts.shape[0]} rel_err={err:.3e}")
        assert err <= TOL
        assert np.isfinite(wl.bf16_bits_to_f32(got_all)).all()
        assert B.lora_poll_device_flags(sess.ctx) == (B.LORA_OK, 0)
    finally:
        sess.close()
