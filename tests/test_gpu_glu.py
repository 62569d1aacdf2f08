"""GPU parity of gate and up in one call with their product (lora_layer_forward_glu): silu(gate) * up against the
oracle's float64 definition, on the three kernels that serve it (128-row and 256-row small-batch tiles, the
register-staged prefill tile), with many adapters, without any, and from a pool of pages."""
import numpy as np
import pytest
import torch

import oracle
from gpu_util import TOL, announce, check_segments, rel_err
from paper_2602_24044_amd import binding as B
from paper_2602_24044_amd import workloads as wl
from paper_2602_24044_amd.runtime import Session, bf16_tensor_to_bits

pytestmark = pytest.mark.gpu


def _gate_up(w):
    return w.proj_names.index("gate"), w.proj_names.index("up")


def _run(w, expect_kernel, n_pages=0, ids=None):
    g, u = _gate_up(w)
    if ids is not None:
        w.token_ids = ids
    announce(f"glu {w.name} T={w.T} proj={w.proj[g]} n_pages={n_pages}")
    sess = Session(w, n_pages=n_pages)
    try:
        sess.load(w.resident)
        sess.bucket(torch.from_numpy(w.token_ids).to(sess.device))
        assert check_segments(sess, w) == 0
        out = sess.forward_glu(g, u)
        torch.cuda.synchronize()
        launches = B.lora_last_launches(sess.ctx)
        h_ref = oracle.gated(w.x[g], w.W[g], w.W[u], w.token_ids, oracle.adapters_of(w, g), oracle.adapters_of(w, u))
        e = rel_err(bf16_tensor_to_bits(out), h_ref)
        announce(f"  launches={launches} rel_err={e:.3e}")
        assert expect_kernel in launches, launches
        assert e <= TOL
        # and the separate projections still come out as before on the same context
        for p in (g, u):
            y = sess.forward(p)
            torch.cuda.synchronize()
            y_ref = oracle.project(w.x[p], w.W[p], w.token_ids, oracle.adapters_of(w, p))
            assert rel_err(bf16_tensor_to_bits(y), y_ref) <= TOL
        assert B.lora_poll_device_flags(sess.ctx) == (B.LORA_OK, 0)
    finally:
        sess.close()


def test_small_batch_tiles():
    _run(wl.config2(shrink=8, n_tokens=100), "gemm_glu_128x128x64_w4")
    _run(wl.config2(shrink=8, n_tokens=300), "gemm_glu_256x128x64_w8")
    _run(wl.config2(shrink=4, n_tokens=777), "gemm_glu_256x128x64_w8")


def test_prefill_tile_and_ragged_sizes():
    _run(wl.config3(shrink=8, n_req=6, len_div=4), "gemm_glu_staged_256x256x64_w8")
    _run(wl.qwen_decode(shrink=8, n_tokens=150), "gemm_glu_256x128x64_w8")          # 18944 / 8 = 2368 columns: ragged last tile


def test_many_adapters_none_and_a_pool_of_pages():
    w = wl.config4(shrink=8, n_tokens=400, n_adapters=96)
    _run(w, "gemm_glu_256x128x64_w8")
    _run(wl.config4(shrink=8, n_tokens=400, n_adapters=96), "gemm_glu_256x128x64_w8",
         n_pages=sum(w.adapters[a].rank // 8 for a in w.resident))
    w = wl.config2(shrink=8, n_tokens=300)
    _run(w, "gemm_glu_256x128x64_w8", ids=np.full(w.T, -1, dtype=np.int32))


def test_argument_errors():
    w = wl.qwen_decode(shrink=8, n_tokens=40)
    sess = Session(w)
    try:
        sess.load(w.resident)
        sess.bucket()
        g, u = _gate_up(w)
        q, k = w.proj_names.index("q"), w.proj_names.index("k")
        out = torch.empty((w.T, w.proj[g][1]), dtype=torch.bfloat16, device=sess.device)
        for pa, pb, status in ((g, g, B.LORA_ERR_INVALID_ARG), (g, 99, B.LORA_ERR_INVALID_ARG), (q, k, B.LORA_ERR_SHAPE)):
            with pytest.raises(B.LoraError) as e:
                B.lora_layer_forward_glu(sess.ctx, pa, pb, sess.x[g].data_ptr(), sess.W[g].data_ptr(), sess.W[u].data_ptr(),
                                         sess.seg, out.data_ptr())
            assert e.value.status == status
        # projections with a bias (q and v of this family have one and the same shape only if kv = hidden; use k, v)
        kk, v = w.proj_names.index("k"), w.proj_names.index("v")
        with pytest.raises(B.LoraError) as e:
            B.lora_layer_forward_glu(sess.ctx, kk, v, sess.x[kk].data_ptr(), sess.W[kk].data_ptr(), sess.W[v].data_ptr(),
                                     sess.seg, out.data_ptr())
        assert e.value.status == B.LORA_ERR_INVALID_ARG
    finally:
        sess.close()
