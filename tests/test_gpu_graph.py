"""A step captured into a HIP graph (bucket + every projection) and replayed: serving loops replay the same launch
sequence on new token ids.  Each replay is checked, with eager work and synchronisations between the replays."""
import numpy as np
import pytest
import torch

import oracle
from gpu_util import TOL, announce, rel_err
from paper_2602_24044_amd import binding as B
from paper_2602_24044_amd import workloads as wl
from paper_2602_24044_amd.runtime import Session, bf16_tensor_to_bits

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("path", [B.LORA_PATH_AUTO, B.LORA_PATH_FUSED, B.LORA_PATH_SPLITK])
def test_captured_step_replays_on_new_token_ids(path):
    w = wl.config2(shrink=8, n_tokens=256)
    announce(f"graph capture {w.name} T={w.T} path={path}")
    s = Session(w, path=path)
    other = Session(wl.config4(shrink=8))            # eager work between the replays
    try:
        s.load(w.resident)
        other.load(other.w.resident)
        torch.cuda.synchronize()
        s.step()                                     # eager result for the first ids
        torch.cuda.synchronize()
        eager = [bf16_tensor_to_bits(o).copy() for o in s.out]
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            s.step(packed=True)                      # warm-up on the capture stream
        side.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=side):
            s.step(packed=True)
        torch.cuda.synchronize()
        rng = np.random.default_rng(4)
        resident = np.array(w.resident, dtype=np.int32)
        for rep in range(4):
            if rep == 0:
                ids = w.token_ids
            else:                                    # a new batch of the same size: other adapters, some tokens without
                ids = resident[rng.integers(0, len(resident), size=w.T)].astype(np.int32)
                ids[rng.random(w.T) < 0.1] = -1
            s.ids.copy_(torch.from_numpy(ids).to(s.device))
            for o in s.out:
                o.zero_()
            other.step()                             # unrelated eager launches in between
            torch.cuda.synchronize()
            g.replay()
            torch.cuda.synchronize()
            for p in range(len(w.proj)):
                got = bf16_tensor_to_bits(s.out[p])
                if rep == 0:
                    assert np.array_equal(got, eager[p]), (rep, p)
                y_ref = oracle.project(w.x[p], w.W[p], ids, oracle.adapters_of(w, p))
                assert rel_err(got, y_ref) <= TOL, (rep, p)
        st, word = B.lora_poll_device_flags(s.ctx)
        assert st == B.LORA_OK and word == 0
    finally:
        s.close()
        other.close()
