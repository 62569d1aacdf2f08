"""Harness helper around the C ABI: owns the torch tensors (device slab, pinned host adapters, device
inputs/outputs) that one synthetic workload needs and forwards every operation to liblora_mi355.
No arithmetic of the method happens here."""
from __future__ import annotations

from typing import Dict, List, Optional, Sequence

import numpy as np
import torch

from . import binding as B
from .workloads import Workload


def _bf16_tensor(bits: np.ndarray, device=None, pin: bool = False) -> torch.Tensor:
    t = torch.from_numpy(np.ascontiguousarray(bits).view(np.int16))
    if pin:
        t = t.pin_memory()
    if device is not None:
        t = t.to(device, non_blocking=False)
    return t.view(torch.bfloat16)


def pin_matrices(A: Sequence[np.ndarray], B: Sequence[np.ndarray], packed: bool) -> dict:
    """Page-locked host copies of an adapter's matrices (bf16 bits), A[k] / B[k] in the order the library takes them.
    packed: one buffer holding A[0], B[0], A[1], B[1], ... back to back (the order inside a slot: the load then
    moves whole runs); otherwise one buffer per matrix."""
    if not packed:
        A_t = [_bf16_tensor(m, pin=True) for m in A]
        B_t = [_bf16_tensor(m, pin=True) for m in B]
        return {"keep": A_t + B_t, "A_ptrs": [t.data_ptr() for t in A_t], "B_ptrs": [t.data_ptr() for t in B_t]}
    n_el = sum(a.size + b.size for a, b in zip(A, B))
    buf = torch.empty(n_el, dtype=torch.int16, pin_memory=True)
    view = buf.numpy()
    A_ptrs, B_ptrs, off = [], [], 0
    for a, b in zip(A, B):
        for m, ptrs in ((a, A_ptrs), (b, B_ptrs)):
            view[off:off + m.size] = np.ascontiguousarray(m).view(np.int16).reshape(-1)
            ptrs.append(buf.data_ptr() + 2 * off)
            off += m.size
    return {"keep": [buf], "A_ptrs": A_ptrs, "B_ptrs": B_ptrs}


def bf16_tensor_to_bits(t: torch.Tensor) -> np.ndarray:
    return t.detach().contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


def packed_groups(w: Workload) -> List[List[int]]:
    """Projections a decoder layer computes from one input side by side: q|k|v and gate|up."""
    names = list(w.proj_names)
    groups, used = [], set()
    for fam in (("q", "k", "v"), ("gate", "up")):
        g = [names.index(nm) for nm in fam if nm in names]
        if len(g) > 1 and len({w.proj[p][0] for p in g}) == 1:
            groups.append(g)
            used.update(g)
    out = []
    for p in range(len(names)):
        if p in used:
            g = next(g for g in groups if p in g)
            if g[0] == p:
                out.append(g)
        else:
            out.append([p])
    return out


class Session:
    def __init__(self, w: Workload, path: int = B.LORA_PATH_AUTO, split_k: int = 0, device: str = "cuda:0",
                 max_tokens: Optional[int] = None, upload_inputs: bool = True, packed_host: bool = False,
                 n_pages: int = 0):
        if not torch.cuda.is_available():
            raise RuntimeError("liblora_mi355 needs a GPU; there is no CPU path")
        self.w = w
        self.packed_host = packed_host
        self.device = torch.device(device)
        torch.cuda.set_device(self.device)
        self.max_tokens = int(max_tokens or max(w.T, 1))
        cfg = B.make_config(w.proj, w.n_slots, w.max_rank, self.max_tokens, w.max_adapter_id, path=path,
                            split_k=split_k, n_pages=n_pages)
        nbytes = B.lora_slab_bytes(cfg)
        if nbytes == 0:
            raise B.LoraError(B.LORA_ERR_SHAPE, "lora_slab_bytes")
        self.slab = torch.empty(nbytes, dtype=torch.uint8, device=self.device)
        cfg.slab = self.slab.data_ptr()
        cfg.slab_bytes = nbytes
        self.cfg = cfg
        self.ctx = B.lora_create(cfg)
        self.pinned: Dict[int, dict] = {}
        self.seg: Optional[B.lora_segments] = None
        self.W: List[torch.Tensor] = []
        self.x: List[torch.Tensor] = []
        self.out: List[torch.Tensor] = []
        self.ids: Optional[torch.Tensor] = None
        self.bias: List[Optional[torch.Tensor]] = []
        if upload_inputs:
            self.upload_inputs()

    # ---- inputs ----
    def upload_inputs(self):
        w = self.w
        self.W = [_bf16_tensor(m, self.device) for m in w.W]
        self.x = [_bf16_tensor(m, self.device) for m in w.x]
        self.out = [torch.empty((w.T, d_out), dtype=torch.bfloat16, device=self.device) for (_, d_out) in w.proj]
        self.ids = torch.from_numpy(w.token_ids).to(self.device)
        self.bias = [None if w.bias_of(p) is None else _bf16_tensor(w.bias_of(p), self.device)
                     for p in range(len(w.proj))]
        for p, b in enumerate(self.bias):
            B.lora_set_bias(self.ctx, p, 0 if b is None else b.data_ptr())

    def pin_adapter(self, aid: int) -> dict:
        if aid not in self.pinned:
            a = self.w.adapters[aid]
            ent = {"adapter_id": aid, "rank": a.rank, "scale": a.scale, "slot": -1}
            if a.rank > 0:
                ent.update(pin_matrices(a.A, a.B, self.packed_host))
            self.pinned[aid] = ent
        return self.pinned[aid]

    # ---- the three hot calls ----
    def load(self, adapter_ids: Sequence[int], in_use: Sequence[int] = (), stream: Optional[torch.cuda.Stream] = None,
             slots: Optional[Sequence[int]] = None, chunk: int = 64):
        res = []
        ids = list(adapter_ids)
        s = (stream or torch.cuda.current_stream()).cuda_stream
        for i in range(0, len(ids), chunk):
            descs = []
            for k, aid in enumerate(ids[i:i + chunk]):
                d = dict(self.pin_adapter(aid))
                if slots is not None:
                    d["slot"] = int(slots[i + k])
                descs.append(d)
            res += B.lora_slots_load(self.ctx, descs, in_use, s)
        return res

    def bucket(self, ids: Optional[torch.Tensor] = None, mode: Optional[int] = None,
               stream: Optional[torch.cuda.Stream] = None) -> B.lora_segments:
        ids = self.ids if ids is None else ids
        mode = self.w.mode if mode is None else mode
        s = (stream or torch.cuda.current_stream()).cuda_stream
        self.seg = B.lora_bucket(self.ctx, ids.data_ptr() if ids.numel() else 0, int(ids.numel()), mode, s)
        return self.seg

    def forward(self, p: int, x: Optional[torch.Tensor] = None, W: Optional[torch.Tensor] = None,
                out: Optional[torch.Tensor] = None, stream: Optional[torch.cuda.Stream] = None) -> torch.Tensor:
        x = self.x[p] if x is None else x
        W = self.W[p] if W is None else W
        out = self.out[p] if out is None else out
        s = (stream or torch.cuda.current_stream()).cuda_stream
        B.lora_layer_forward(self.ctx, p, x.data_ptr(), W.data_ptr(), self.seg, out.data_ptr(), s)
        return out

    def forward_group(self, ps: Sequence[int], stream: Optional[torch.cuda.Stream] = None) -> List[torch.Tensor]:
        s = (stream or torch.cuda.current_stream()).cuda_stream
        B.lora_layer_forward_group(self.ctx, list(ps), [self.x[p].data_ptr() for p in ps],
                                   [self.W[p].data_ptr() for p in ps], self.seg,
                                   [self.out[p].data_ptr() for p in ps], s)
        return [self.out[p] for p in ps]

    def forward_glu(self, p_gate: int, p_up: int, out: Optional[torch.Tensor] = None,
                    stream: Optional[torch.cuda.Stream] = None) -> torch.Tensor:
        """silu(gate) * up of the two projections on the input of p_gate (lora_layer_forward_glu)."""
        if out is None:
            out = torch.empty((self.w.T, self.w.proj[p_gate][1]), dtype=torch.bfloat16, device=self.device)
        s = (stream or torch.cuda.current_stream()).cuda_stream
        B.lora_layer_forward_glu(self.ctx, p_gate, p_up, self.x[p_gate].data_ptr(), self.W[p_gate].data_ptr(),
                                 self.W[p_up].data_ptr(), self.seg, out.data_ptr(), s)
        return out

    def packed_groups(self) -> List[List[int]]:
        return packed_groups(self.w)

    def forward_all(self, packed: bool = True) -> None:
        """Every projection of the layer on the current segment map (q|k|v and gate|up as packed calls)."""
        if packed:
            for g in self.packed_groups():
                if len(g) == 1:
                    self.forward(g[0])
                else:
                    self.forward_group(g)
        else:
            for p in range(len(self.w.proj)):
                self.forward(p)

    def step(self, packed: bool = True) -> None:
        """One pass of the whole path: segment map + every projection."""
        self.bucket()
        self.forward_all(packed)

    # ---- read-back helpers ----
    def _i32_at(self, ptr: int, n: int) -> np.ndarray:
        off = ptr - self.slab.data_ptr()
        assert 0 <= off and off + 4 * n <= self.slab.numel()
        return self.slab[off:off + 4 * n].view(torch.int32).cpu().numpy()

    def read_segments(self):
        torch.cuda.synchronize()
        seg = self.seg
        n_seg = int(self._i32_at(seg.n_seg, 1)[0])
        perm = self._i32_at(seg.perm, seg.T) if seg.T else np.zeros(0, np.int32)
        return (perm, self._i32_at(seg.seg_start, n_seg + 1), self._i32_at(seg.seg_slot, n_seg) if n_seg else
                np.zeros(0, np.int32), n_seg)

    def id2slot(self) -> np.ndarray:
        return np.array([B.lora_slot_of(self.ctx, i) for i in range(self.w.max_adapter_id + 1)], dtype=np.int32)

    def close(self):
        if self.ctx:
            B.lora_destroy(self.ctx)
            self.ctx = 0

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class ModelSession:
    """Whole-model harness: `layers` are the per-layer workloads of one step (workloads.model_layers), served by
    one context with n_layers layers: one slot table, one segment map per step, a slot holds an adapter's matrices
    of every layer.  Owns tensors and forwards to the C ABI; no arithmetic of the method happens here."""

    def __init__(self, layers: Sequence[Workload], path: int = B.LORA_PATH_AUTO, split_k: int = 0,
                 device: str = "cuda:0", n_slots: Optional[int] = None, packed_host: bool = True, n_pages: int = 0):
        if not torch.cuda.is_available():
            raise RuntimeError("liblora_mi355 needs a GPU; there is no CPU path")
        self.layers = list(layers)
        self.packed_host = packed_host
        w = self.w = self.layers[0]
        for lw in self.layers:
            assert lw.proj == w.proj and np.array_equal(lw.token_ids, w.token_ids)
        self.device = torch.device(device)
        torch.cuda.set_device(self.device)
        cfg = B.make_config(w.proj, n_slots or w.n_slots, w.max_rank, max(w.T, 1), w.max_adapter_id, path=path,
                            split_k=split_k, n_layers=len(self.layers), n_pages=n_pages)
        nbytes = B.lora_slab_bytes(cfg)
        if nbytes == 0:
            raise B.LoraError(B.LORA_ERR_SHAPE, "lora_slab_bytes")
        self.slab_bytes = nbytes
        self.slab = torch.empty(nbytes, dtype=torch.uint8, device=self.device)
        cfg.slab = self.slab.data_ptr()
        cfg.slab_bytes = nbytes
        self.cfg = cfg
        self.ctx = B.lora_create(cfg)
        self.W = [[_bf16_tensor(m, self.device) for m in lw.W] for lw in self.layers]
        self.x = [[_bf16_tensor(m, self.device) for m in lw.x] for lw in self.layers]
        self.out = [[torch.empty((w.T, d_out), dtype=torch.bfloat16, device=self.device) for (_, d_out) in w.proj]
                    for _ in self.layers]
        self.bias = [[None if lw.bias_of(p) is None else _bf16_tensor(lw.bias_of(p), self.device)
                      for p in range(len(w.proj))] for lw in self.layers]
        for l, row in enumerate(self.bias):
            for p, b in enumerate(row):
                if b is not None:
                    B.lora_set_bias(self.ctx, p, b.data_ptr(), layer=l)
        self.ids = torch.from_numpy(w.token_ids).to(self.device)
        self.groups = packed_groups(w)
        self.pinned: Dict[int, dict] = {}
        self.seg: Optional[B.lora_segments] = None

    def pin_adapter(self, aid: int) -> dict:
        if aid not in self.pinned:
            a0 = self.w.adapters[aid]
            ent = {"adapter_id": aid, "rank": a0.rank, "scale": a0.scale, "slot": -1}
            if a0.rank > 0:
                # layer-major: every projection of layer 0, then of layer 1, ...
                ent.update(pin_matrices([m for lw in self.layers for m in lw.adapters[aid].A],
                                        [m for lw in self.layers for m in lw.adapters[aid].B], self.packed_host))
            self.pinned[aid] = ent
        return self.pinned[aid]

    def load(self, adapter_ids: Sequence[int], in_use: Sequence[int] = (), stream: Optional[torch.cuda.Stream] = None,
             chunk: int = 64):
        s = (stream or torch.cuda.current_stream()).cuda_stream
        ids, res = list(adapter_ids), []
        for i in range(0, len(ids), chunk):
            res += B.lora_slots_load(self.ctx, [dict(self.pin_adapter(a)) for a in ids[i:i + chunk]], in_use, s)
        return res

    def bucket(self, stream: Optional[torch.cuda.Stream] = None) -> B.lora_segments:
        s = (stream or torch.cuda.current_stream()).cuda_stream
        self.seg = B.lora_bucket(self.ctx, self.ids.data_ptr() if self.ids.numel() else 0, int(self.ids.numel()),
                                 self.w.mode, s)
        return self.seg

    def forward_layer(self, l: int, stream: Optional[torch.cuda.Stream] = None) -> None:
        s = (stream or torch.cuda.current_stream()).cuda_stream
        for g in self.groups:
            B.lora_model_forward_group(self.ctx, l, g, [self.x[l][p].data_ptr() for p in g],
                                       [self.W[l][p].data_ptr() for p in g], self.seg,
                                       [self.out[l][p].data_ptr() for p in g], s)

    def forward_glu(self, l: int, p_gate: int, p_up: int, out: Optional[torch.Tensor] = None,
                    stream: Optional[torch.cuda.Stream] = None) -> torch.Tensor:
        """silu(gate) * up of layer l's two projections on the input of p_gate (lora_model_forward_glu)."""
        w = self.layers[l]
        if out is None:
            out = torch.empty((w.T, w.proj[p_gate][1]), dtype=torch.bfloat16, device=self.device)
        s = (stream or torch.cuda.current_stream()).cuda_stream
        B.lora_model_forward_glu(self.ctx, l, p_gate, p_up, self.x[l][p_gate].data_ptr(), self.W[l][p_gate].data_ptr(),
                                 self.W[l][p_up].data_ptr(), self.seg, out.data_ptr(), s)
        return out

    def step(self, stream: Optional[torch.cuda.Stream] = None) -> None:
        """One step of the whole model: one segment map, then every layer's projections."""
        self.bucket(stream)
        for l in range(len(self.layers)):
            self.forward_layer(l, stream)

    def close(self):
        if self.ctx:
            B.lora_destroy(self.ctx)
            self.ctx = 0

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
