"""GPU tests of boundary rules that are not plain parity: forwards of one context on several streams, and the
handling of an expired bounded wait inside a launch (forced from the host; every kernel ends normally)."""
import numpy as np
import pytest
import torch

import oracle
from gpu_util import TOL, announce, rel_err
from paper_2602_24044_amd import binding as B
from paper_2602_24044_amd import workloads as wl
from paper_2602_24044_amd.runtime import Session, bf16_tensor_to_bits

pytestmark = pytest.mark.gpu


def _check_all(sess, w):
    for p in range(len(w.proj)):
        y_ref = oracle.project(w.x[p], w.W[p], w.token_ids, oracle.adapters_of(w, p), bias=w.bias_of(p))
        assert rel_err(bf16_tensor_to_bits(sess.out[p]), y_ref) <= TOL, p


def test_forwards_of_one_context_on_two_streams():
    """The calls share the context's scratch; the library orders a call behind the previous one when the stream
    changes, so a caller that alternates streams without events of its own still gets every projection right."""
    w = wl.config2(shrink=8, n_tokens=300)
    announce(f"two streams: {w.name} T={w.T}")
    sess = Session(w)
    try:
        sess.load(w.resident)
        s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
        torch.cuda.synchronize()
        for rep in range(3):
            for p in range(len(w.proj)):
                sess.out[p].fill_(float("nan"))
            torch.cuda.synchronize()
            sess.bucket(stream=s1 if rep % 2 == 0 else s2)
            for k, g in enumerate(sess.packed_groups()):
                st = s2 if (k + rep) % 2 == 0 else s1
                if len(g) > 1:
                    sess.forward_group(g, stream=st)
                else:
                    sess.forward(g[0], stream=st)
            torch.cuda.synchronize()
            _check_all(sess, w)
        assert B.lora_poll_device_flags(sess.ctx) == (B.LORA_OK, 0)
    finally:
        sess.close()


def test_expired_wait_inside_a_launch_is_flagged_and_the_context_recovers():
    """Shrink inside the fused launch: the tile workgroups wait, bounded, for the launch's shrink workgroups.  The
    test knob makes them expect one report too many and give up after one poll.  The flag must be raised, the poll
    must set the counters back and switch the context to a shrink launch of its own, and the next step must be right."""
    w = wl.config2(shrink=8, n_tokens=300)
    announce(f"expired wait: {w.name} T={w.T}")
    sess = Session(w, path=B.LORA_PATH_FUSED)
    try:
        B.lora_set_tuning(sess.ctx, B.LORA_TUNE_FUSED_VARIANT, 8)
        B.lora_set_tuning(sess.ctx, B.LORA_TUNE_INLINE_SHRINK, B.LORA_INLINE_SHRINK_ON)
        sess.load(w.resident)
        # a normal step first: shrink inside the launch, nothing flagged
        sess.step()
        torch.cuda.synchronize()
        g = [g for g in sess.packed_groups() if len(g) > 1][-1]
        sess.forward_group(g)
        assert "shrink" not in B.lora_last_launches(sess.ctx)
        torch.cuda.synchronize()
        assert B.lora_poll_device_flags(sess.ctx) == (B.LORA_OK, 0)
        # the forced give-up
        B.lora_set_tuning(sess.ctx, B.LORA_TUNE_SHRINK_WAIT_TEST, 1)
        sess.forward_group(g)
        torch.cuda.synchronize()
        with pytest.raises(B.LoraError) as e:
            B.lora_poll_device_flags(sess.ctx)
        assert e.value.status == B.LORA_ERR_HIP
        B.lora_set_tuning(sess.ctx, B.LORA_TUNE_SHRINK_WAIT_TEST, 0)
        # the flag is cleared, the context shrinks in a launch of its own from now on, results are right again
        assert B.lora_poll_device_flags(sess.ctx) == (B.LORA_OK, 0)
        for rep in range(2):
            for p in range(len(w.proj)):
                sess.out[p].fill_(float("nan"))
            sess.step()
            torch.cuda.synchronize()
            _check_all(sess, w)
        sess.forward_group(g)
        assert "shrink" in B.lora_last_launches(sess.ctx)
        torch.cuda.synchronize()
        assert B.lora_poll_device_flags(sess.ctx) == (B.LORA_OK, 0)
    finally:
        sess.close()


def test_loads_on_a_copy_stream_between_steps_wait_for_this_contexts_forwards_only():
    """Two contexts share the compute stream; context A reloads two slots before each of its steps on a copy stream
    of its own.  The load must wait for A's previous forwards (they read the slots it overwrites) and may run while
    B's step, enqueued in between, is still computing: A's outputs are checked after every step against the adapters
    that were in the slots for that step."""
    wa = wl.config2(shrink=8, n_tokens=300)
    wb = wl.config2(shrink=4, n_tokens=512)
    announce(f"loads between steps: A={wa.name} B={wb.name}")
    A, Bs = Session(wa), Session(wb)
    copy = torch.cuda.Stream()
    try:
        A.load(wa.resident)
        Bs.load(wb.resident)
        ids = sorted(wa.distinct_adapters())
        a0, a1 = ids[0], ids[1]
        slot0, slot1 = B.lora_slot_of(A.ctx, a0), B.lora_slot_of(A.ctx, a1)
        torch.cuda.synchronize()
        outs = []
        for step in range(6):
            # swap the two adapters' slots before every step: tokens of a0 must still get a0's weights
            tgt = (slot1, slot0) if step % 2 == 0 else (slot0, slot1)
            A.load([a0, a1], in_use=ids, slots=list(tgt), stream=copy)
            A.step()
            outs.append([o.clone() for o in A.out])
            Bs.step()                                  # long work of another context behind A's step
        torch.cuda.synchronize()
        for step, out in enumerate(outs):
            for p in range(len(wa.proj)):
                y_ref = oracle.project(wa.x[p], wa.W[p], wa.token_ids, oracle.adapters_of(wa, p), bias=wa.bias_of(p))
                assert rel_err(bf16_tensor_to_bits(out[p]), y_ref) <= TOL, (step, p)
        assert B.lora_poll_device_flags(A.ctx) == (B.LORA_OK, 0)
    finally:
        A.close()
        Bs.close()
