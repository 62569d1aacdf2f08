"""lora_layer_forward_static (the entry point for callers that cannot allocate: its scratch is the library's static
device array) against lora_layer_forward, through the C ABI: two calls in a row, the second on a smaller batch, so
that what the first call left in the shared scratch is there when the second runs."""
import numpy as np
import pytest
import torch

import oracle
from gpu_util import TOL, announce, rel_err
from paper_2602_24044_amd import binding as B
from paper_2602_24044_amd import workloads as wl
from paper_2602_24044_amd.runtime import Session, bf16_tensor_to_bits

pytestmark = pytest.mark.gpu


def _both(w, path):
    """Every projection through both entry points; returns [(bits by lora_layer_forward, bits by the static one)]."""
    sess = Session(w, path=path)
    try:
        sess.load(w.resident)
        sess.bucket()
        s = torch.cuda.current_stream().cuda_stream
        res = []
        for p in range(len(w.proj)):
            sess.out[p].fill_(float("nan"))
            sess.forward(p)
            torch.cuda.synchronize()
            ref = bf16_tensor_to_bits(sess.out[p]).copy()
            sess.out[p].fill_(float("nan"))
            B.lora_layer_forward_static(sess.ctx, p, sess.x[p].data_ptr(), sess.W[p].data_ptr(), sess.seg,
                                        sess.out[p].data_ptr(), s)
            torch.cuda.synchronize()
            res.append((ref, bf16_tensor_to_bits(sess.out[p]).copy()))
        assert B.lora_poll_device_flags(sess.ctx) == (B.LORA_OK, 0)
        return res
    finally:
        sess.close()


@pytest.mark.parametrize("path", [B.LORA_PATH_AUTO, B.LORA_PATH_SPLITK, B.LORA_PATH_FUSED])
def test_static_scratch_entry_point_two_calls(path):
    assert B.lora_static_scratch_bytes() == 40 << 20
    big = wl.config2(shrink=8, n_tokens=200)
    small = wl.config2(shrink=8, n_tokens=37)
    for w in (big, small):                     # the second batch is smaller: the scratch still holds the first one's
        announce(f"static scratch: {w.name} T={w.T} path={path}")
        for p, (ref, got) in enumerate(_both(w, path)):
            # same kernels, same plan (the scratch is large enough for the same K split): the same bits
            assert np.array_equal(ref, got), (w.T, p)
            y_ref = oracle.project(w.x[p], w.W[p], w.token_ids, oracle.adapters_of(w, p))
            assert rel_err(got, y_ref) <= TOL, (w.T, p)


def test_static_scratch_limit_is_an_error():
    # shrink results of 4 chunks x 1024 tokens x rank 64 x 14 chunks of K: beyond the 2 Mi values of the buffer
    w = wl.config2(shrink=8, n_tokens=16)
    proj = [(16384, 512)]
    cfg = B.make_config(proj, 4, 64, 40000, 7)
    nbytes = B.lora_slab_bytes(cfg)
    slab = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    cfg.slab, cfg.slab_bytes = slab.data_ptr(), nbytes
    ctx = B.lora_create(cfg)
    try:
        T = 40000
        ids = torch.full((T,), -1, dtype=torch.int32, device="cuda")
        seg = B.lora_bucket(ctx, ids.data_ptr(), T, B.LORA_BUCKET_RUNS)
        x = torch.zeros((8, 8), dtype=torch.bfloat16, device="cuda")     # never read: the call must fail first
        with pytest.raises(B.LoraError) as e:
            B.lora_layer_forward_static(ctx, 0, x.data_ptr(), x.data_ptr(), seg, x.data_ptr())
        assert e.value.status == B.LORA_ERR_SCRATCH_LIMIT
        torch.cuda.synchronize()
    finally:
        B.lora_destroy(ctx)
    del w
