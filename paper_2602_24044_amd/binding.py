"""Thin ctypes binding of liblora_mi355: same names as the C ABI, argument marshalling only.

Every step of the serving path runs inside the library's HIP kernels; PyTorch is used by callers
for device memory, pinned host memory and streams only.  There is no CPU fallback: if the shared
library is missing, importing this module raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Dict, List, Optional, Sequence, Tuple

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "liblora_mi355.so")

if not os.path.exists(LIB_PATH):
    raise ImportError(
        f"{LIB_PATH} is not built; run `python -m paper_2602_24044_amd.build` (needs hipcc). "
        "There is no fallback path.")



def _preload_hip_runtime() -> None:
    """One process must hold one HIP runtime.  PyTorch ships its own libamdhip64 (same soname as the
    system one) and resolves it by file name, so load that copy first when PyTorch is installed: this
    library's dependency on the soname then binds to the same runtime that owns torch's memory and
    streams, whichever of the two modules is imported first."""
    import importlib.util
    try:
        spec = importlib.util.find_spec("torch")
    except (ImportError, ValueError):
        spec = None
    if spec is None or not spec.submodule_search_locations:
        return
    cand = os.path.join(list(spec.submodule_search_locations)[0], "lib", "libamdhip64.so")
    if os.path.exists(cand):
        ctypes.CDLL(cand, mode=ctypes.RTLD_GLOBAL)


_preload_hip_runtime()
_lib = ctypes.CDLL(LIB_PATH)

# ---- status / enums (mirror include/lora_mi355.h) ----
LORA_OK = 0
LORA_ERR_INVALID_ARG = 1
LORA_ERR_SHAPE = 2
LORA_ERR_OOM = 3
LORA_ERR_SLOT_RANGE = 4
LORA_ERR_RANK_EXCEEDS_SMAX = 5
LORA_ERR_SLOTS_EXHAUSTED = 6
LORA_ERR_NOT_RESIDENT = 7
LORA_ERR_HIP = 8
LORA_ERR_ID_RANGE = 9
LORA_ERR_STARVATION = 10
LORA_ERR_SCRATCH_LIMIT = 11
LORA_BUCKET_SORTED = 0
LORA_BUCKET_RUNS = 1
LORA_PATH_AUTO = 0
LORA_PATH_FUSED = 1
LORA_PATH_SPLITK = 2
LORA_FLAG_NOT_RESIDENT = 1
LORA_FLAG_INTERNAL = 2
LORA_CREATE_HOST_ONLY = 1

EXPORTS = [
    "lora_slab_bytes", "lora_create", "lora_destroy", "lora_slots_load", "lora_bucket", "lora_layer_forward",
    "lora_layer_forward_group",
    "lora_layer_forward_glu", "lora_model_forward_glu", "lora_poll_device_flags", "lora_slot_of", "lora_slot_adapter", "lora_slot_first_page", "lora_last_launches",
    "lora_profile_enable", "lora_profile_collect", "lora_profile_reset", "lora_status_string",
    "lora_last_hip_error", "lora_calibrate_stream", "lora_calibrate_mfma", "lora_layer_forward_static", "lora_static_scratch_bytes", "lora_set_tuning", "lora_set_bias", "lora_model_forward_group", "lora_place_adapters", "lora_priority_sorting",
]
LORA_TUNE_FUSED_VARIANT = 0
LORA_TUNE_SPLIT_VARIANT = 1
LORA_TUNE_COPY_ENGINE = 2
LORA_COPY_AUTO, LORA_COPY_KERNEL, LORA_COPY_ENGINE = 0, 1, 2
LORA_TUNE_INLINE_SHRINK = 3
LORA_TUNE_SHRINK_WAIT_TEST = 4
LORA_INLINE_SHRINK_AUTO, LORA_INLINE_SHRINK_OFF, LORA_INLINE_SHRINK_ON = 0, 1, 2
# values of LORA_TUNE_FUSED_VARIANT / LORA_TUNE_SPLIT_VARIANT (tile rows x columns x K tile, wavefronts)
FUSED_VARIANTS = {"256x256x32_w4": 1, "256x256x32_w4_3stages": 2, "128x128x32_w4": 3, "256x128x32_w8": 4,
                  "256x128x32_w8_allcopy": 5, "256x128x64_w8": 8, "128x128x64_w4": 9, "256x256x64_w8": 10, "256x192x64_w8": 11,
                  "256x256x32_w8": 12, "256x128x64_w4": 13, "256x256x64_w4": 14,
                  "staged_256x256x64_w8": 15, "staged_256x256x64_w4": 16}
SPLIT_VARIANTS = {"256x128x32_w4": 1, "256x64x32_w4": 2, "128x128x32_w4": 3, "128x128x32_w4_8stages": 4,
                  "256x128x64_w8": 6, "128x128x64_w4": 7, "256x128x32_w8": 8, "256x128x64_w4": 9}


class lora_proj_shape(ctypes.Structure):
    _fields_ = [("d_in", ctypes.c_int32), ("d_out", ctypes.c_int32)]


class lora_config(ctypes.Structure):
    _fields_ = [("n_slots", ctypes.c_int32), ("max_rank", ctypes.c_int32), ("n_proj", ctypes.c_int32),
                ("proj", ctypes.POINTER(lora_proj_shape)), ("max_tokens", ctypes.c_int32),
                ("max_adapter_id", ctypes.c_int32), ("slab", ctypes.c_void_p), ("slab_bytes", ctypes.c_size_t),
                ("path", ctypes.c_int32), ("split_k", ctypes.c_int32), ("flags", ctypes.c_uint32),
                ("n_layers", ctypes.c_int32), ("n_pages", ctypes.c_int32)]


class lora_adapter_desc(ctypes.Structure):
    _fields_ = [("adapter_id", ctypes.c_int32), ("rank", ctypes.c_int32), ("scale", ctypes.c_float),
                ("slot", ctypes.c_int32), ("copied", ctypes.c_int32),
                ("A", ctypes.POINTER(ctypes.c_void_p)), ("B", ctypes.POINTER(ctypes.c_void_p))]


class lora_segments(ctypes.Structure):
    _fields_ = [("perm", ctypes.c_void_p), ("seg_start", ctypes.c_void_p), ("seg_slot", ctypes.c_void_p),
                ("n_seg", ctypes.c_void_p), ("T", ctypes.c_int32), ("mode", ctypes.c_int32),
                ("epoch", ctypes.c_uint64)]


_P = ctypes.c_void_p
_lib.lora_slab_bytes.restype = ctypes.c_size_t
_lib.lora_slab_bytes.argtypes = [ctypes.POINTER(lora_config)]
_lib.lora_create.restype = ctypes.c_int
_lib.lora_create.argtypes = [ctypes.POINTER(lora_config), ctypes.POINTER(_P)]
_lib.lora_destroy.restype = ctypes.c_int
_lib.lora_destroy.argtypes = [_P]
_lib.lora_slots_load.restype = ctypes.c_int
_lib.lora_slots_load.argtypes = [_P, ctypes.c_int32, ctypes.POINTER(lora_adapter_desc),
                                 ctypes.POINTER(ctypes.c_int32), ctypes.c_int32, _P]
_lib.lora_bucket.restype = ctypes.c_int
_lib.lora_bucket.argtypes = [_P, _P, ctypes.c_int32, ctypes.c_int32, ctypes.POINTER(lora_segments), _P]
_lib.lora_layer_forward.restype = ctypes.c_int
_lib.lora_layer_forward.argtypes = [_P, ctypes.c_int32, _P, _P, ctypes.POINTER(lora_segments), _P, _P]
_lib.lora_layer_forward_static.restype = ctypes.c_int
_lib.lora_layer_forward_static.argtypes = [_P, ctypes.c_int32, _P, _P, ctypes.POINTER(lora_segments), _P, _P]
_lib.lora_static_scratch_bytes.restype = ctypes.c_size_t
_lib.lora_static_scratch_bytes.argtypes = []
_lib.lora_layer_forward_group.restype = ctypes.c_int
_lib.lora_layer_forward_group.argtypes = [_P, ctypes.c_int32, ctypes.POINTER(ctypes.c_int32), ctypes.POINTER(_P),
                                          ctypes.POINTER(_P), ctypes.POINTER(lora_segments), ctypes.POINTER(_P), _P]
_lib.lora_model_forward_group.restype = ctypes.c_int
_lib.lora_model_forward_group.argtypes = [_P, ctypes.c_int32, ctypes.c_int32, ctypes.POINTER(ctypes.c_int32),
                                          ctypes.POINTER(_P), ctypes.POINTER(_P), ctypes.POINTER(lora_segments),
                                          ctypes.POINTER(_P), _P]
_lib.lora_poll_device_flags.restype = ctypes.c_int
_lib.lora_poll_device_flags.argtypes = [_P, ctypes.POINTER(ctypes.c_uint32), _P]
_lib.lora_slot_of.restype = ctypes.c_int32
_lib.lora_slot_of.argtypes = [_P, ctypes.c_int32]
_lib.lora_slot_adapter.restype = ctypes.c_int32
_lib.lora_slot_adapter.argtypes = [_P, ctypes.c_int32]
_lib.lora_slot_first_page.restype = ctypes.c_int32
_lib.lora_slot_first_page.argtypes = [_P, ctypes.c_int32]
_lib.lora_last_launches.restype = ctypes.c_int32
_lib.lora_last_launches.argtypes = [_P, ctypes.POINTER(ctypes.c_char_p), ctypes.c_int32]
_lib.lora_profile_enable.restype = ctypes.c_int
_lib.lora_profile_enable.argtypes = [_P, ctypes.c_int32]
_lib.lora_profile_collect.restype = ctypes.c_int32
_lib.lora_profile_collect.argtypes = [_P, ctypes.POINTER(ctypes.c_char_p), ctypes.POINTER(ctypes.c_double),
                                      ctypes.POINTER(ctypes.c_int64), ctypes.c_int32]
_lib.lora_profile_reset.restype = ctypes.c_int
_lib.lora_profile_reset.argtypes = [_P]
_lib.lora_status_string.restype = ctypes.c_char_p
_lib.lora_status_string.argtypes = [ctypes.c_int]
_lib.lora_set_bias.restype = ctypes.c_int
_lib.lora_set_bias.argtypes = [_P, ctypes.c_int32, ctypes.c_int32, _P]
_lib.lora_set_tuning.restype = ctypes.c_int
_lib.lora_set_tuning.argtypes = [_P, ctypes.c_int32, ctypes.c_int32]
_lib.lora_calibrate_stream.restype = ctypes.c_int
_lib.lora_calibrate_stream.argtypes = [_P, ctypes.c_size_t, ctypes.c_int32, _P, _P]
_lib.lora_calibrate_mfma.restype = ctypes.c_int
_lib.lora_calibrate_mfma.argtypes = [ctypes.c_int32, ctypes.c_int32, _P, _P, _P]
_lib.lora_last_hip_error.restype = ctypes.c_char_p
_lib.lora_last_hip_error.argtypes = []


class LoraError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        detail = f" [{lora_last_hip_error()}]" if status == LORA_ERR_HIP else ""
        super().__init__(f"{where}: {lora_status_string(status)} (status {status}){detail}")


def lora_status_string(status: int) -> str:
    return _lib.lora_status_string(int(status)).decode()


def lora_last_hip_error() -> str:
    return _lib.lora_last_hip_error().decode()


def make_config(proj: Sequence[Tuple[int, int]], n_slots: int, max_rank: int, max_tokens: int,
                max_adapter_id: int, slab_ptr: int = 0, slab_bytes: int = 0, path: int = LORA_PATH_AUTO,
                split_k: int = 0, flags: int = 0, n_layers: int = 1, n_pages: int = 0):
    arr = (lora_proj_shape * len(proj))(*[lora_proj_shape(int(a), int(b)) for a, b in proj])
    cfg = lora_config(int(n_slots), int(max_rank), len(proj), arr, int(max_tokens), int(max_adapter_id),
                      ctypes.c_void_p(slab_ptr or None), int(slab_bytes), int(path), int(split_k), int(flags),
                      int(n_layers), int(n_pages))
    cfg._keep = arr
    return cfg


def lora_slab_bytes(cfg: lora_config) -> int:
    return int(_lib.lora_slab_bytes(ctypes.byref(cfg)))


def lora_create(cfg: lora_config) -> int:
    """Returns the context handle (an integer address); raises LoraError."""
    h = _P()
    st = _lib.lora_create(ctypes.byref(cfg), ctypes.byref(h))
    if st != LORA_OK:
        raise LoraError(st, "lora_create")
    return h.value


def lora_destroy(ctx: int) -> None:
    st = _lib.lora_destroy(_P(ctx))
    if st != LORA_OK:
        raise LoraError(st, "lora_destroy")


def lora_slots_load(ctx: int, adapters: Sequence[dict], in_use: Sequence[int] = (), copy_stream: int = 0):
    """adapters: dicts with adapter_id, rank, scale, slot (default -1), A_ptrs / B_ptrs (lists of pinned
    host addresses, one per projection; may be omitted for rank 0 or host-only contexts).
    Returns [(slot, copied)] per adapter."""
    n = len(adapters)
    descs = (lora_adapter_desc * max(n, 1))()
    keep = []
    for i, a in enumerate(adapters):
        d = descs[i]
        d.adapter_id = int(a["adapter_id"])
        d.rank = int(a["rank"])
        d.scale = float(a["scale"])
        d.slot = int(a.get("slot", -1))
        d.copied = 0
        ap, bp = a.get("A_ptrs"), a.get("B_ptrs")
        if ap is not None and bp is not None:
            A = (ctypes.c_void_p * len(ap))(*[ctypes.c_void_p(int(v)) for v in ap])
            B = (ctypes.c_void_p * len(bp))(*[ctypes.c_void_p(int(v)) for v in bp])
            keep += [A, B]
            d.A = ctypes.cast(A, ctypes.POINTER(ctypes.c_void_p))
            d.B = ctypes.cast(B, ctypes.POINTER(ctypes.c_void_p))
    iu = (ctypes.c_int32 * max(len(in_use), 1))(*[int(v) for v in in_use])
    st = _lib.lora_slots_load(_P(ctx), n, descs, iu, len(in_use), _P(copy_stream or None))
    if st != LORA_OK:
        raise LoraError(st, "lora_slots_load")
    return [(int(descs[i].slot), bool(descs[i].copied)) for i in range(n)]


def lora_bucket(ctx: int, d_token_adapter: int, T: int, mode: int, stream: int = 0) -> lora_segments:
    seg = lora_segments()
    st = _lib.lora_bucket(_P(ctx), _P(d_token_adapter or None), int(T), int(mode), ctypes.byref(seg),
                          _P(stream or None))
    if st != LORA_OK:
        raise LoraError(st, "lora_bucket")
    return seg


def lora_layer_forward(ctx: int, proj: int, d_x: int, d_W: int, seg: lora_segments, d_out: int,
                       stream: int = 0) -> None:
    st = _lib.lora_layer_forward(_P(ctx), int(proj), _P(d_x or None), _P(d_W or None), ctypes.byref(seg),
                                 _P(d_out or None), _P(stream or None))
    if st != LORA_OK:
        raise LoraError(st, "lora_layer_forward")


def lora_layer_forward_static(ctx: int, proj: int, d_x: int, d_W: int, seg: lora_segments, d_out: int,
                              stream: int = 0) -> None:
    st = _lib.lora_layer_forward_static(_P(ctx), int(proj), _P(d_x or None), _P(d_W or None), ctypes.byref(seg),
                                        _P(d_out or None), _P(stream or None))
    if st != LORA_OK:
        raise LoraError(st, "lora_layer_forward_static")


def lora_static_scratch_bytes() -> int:
    return int(_lib.lora_static_scratch_bytes())


def lora_layer_forward_group(ctx: int, projs: Sequence[int], d_x: Sequence[int], d_W: Sequence[int],
                             seg: lora_segments, d_out: Sequence[int], stream: int = 0) -> None:
    n = len(projs)
    pa = (ctypes.c_int32 * n)(*[int(p) for p in projs])
    xa = (_P * n)(*[_P(v or None) for v in d_x])
    wa = (_P * n)(*[_P(v or None) for v in d_W])
    oa = (_P * n)(*[_P(v or None) for v in d_out])
    st = _lib.lora_layer_forward_group(_P(ctx), n, pa, xa, wa, ctypes.byref(seg), oa, _P(stream or None))
    if st != LORA_OK:
        raise LoraError(st, "lora_layer_forward_group")


def lora_model_forward_group(ctx: int, layer: int, projs: Sequence[int], d_x: Sequence[int], d_W: Sequence[int],
                             seg: lora_segments, d_out: Sequence[int], stream: int = 0) -> None:
    n = len(projs)
    pa = (ctypes.c_int32 * n)(*[int(p) for p in projs])
    xa = (_P * n)(*[_P(v or None) for v in d_x])
    wa = (_P * n)(*[_P(v or None) for v in d_W])
    oa = (_P * n)(*[_P(v or None) for v in d_out])
    st = _lib.lora_model_forward_group(_P(ctx), int(layer), n, pa, xa, wa, ctypes.byref(seg), oa, _P(stream or None))
    if st != LORA_OK:
        raise LoraError(st, "lora_model_forward_group")


THROUGHPUT_FN = ctypes.CFUNCTYPE(ctypes.c_double, _P, ctypes.c_int32, ctypes.POINTER(ctypes.c_int32),
                                 ctypes.POINTER(ctypes.c_double), ctypes.c_int32)
STARVATION_FN = ctypes.CFUNCTYPE(ctypes.c_int32, _P, ctypes.c_int32, ctypes.POINTER(ctypes.c_int32),
                                 ctypes.POINTER(ctypes.c_double), ctypes.c_int32)
_lib.lora_place_adapters.restype = ctypes.c_int
_lib.lora_place_adapters.argtypes = [ctypes.c_int32, ctypes.POINTER(ctypes.c_int32), ctypes.POINTER(ctypes.c_double),
                                     ctypes.c_int32, THROUGHPUT_FN, STARVATION_FN, _P,
                                     ctypes.POINTER(ctypes.c_int32), ctypes.POINTER(ctypes.c_int32)]
_lib.lora_priority_sorting.restype = ctypes.c_int
_lib.lora_priority_sorting.argtypes = [ctypes.c_int32, ctypes.POINTER(ctypes.c_int32), ctypes.POINTER(ctypes.c_double),
                                       ctypes.POINTER(ctypes.c_int32)]


def lora_priority_sorting(size: Sequence[int], rate: Sequence[float]) -> List[int]:
    n = len(size)
    sz = (ctypes.c_int32 * max(n, 1))(*[int(v) for v in size])
    rt = (ctypes.c_double * max(n, 1))(*[float(v) for v in rate])
    out = (ctypes.c_int32 * max(n, 1))()
    st = _lib.lora_priority_sorting(n, sz, rt, out)
    if st != LORA_OK:
        raise LoraError(st, "lora_priority_sorting")
    return [int(out[i]) for i in range(n)]


def lora_place_adapters(size: Sequence[int], rate: Sequence[float], n_gpus: int, predict_throughput,
                        predict_starvation) -> Tuple[List[int], List[int]]:
    """predict_throughput(sizes, rates, a_max) -> float, predict_starvation(sizes, rates, a_max) -> bool, called
    with the lists of one GPU's adapters.  Returns (gpu_of, a_max_of); raises LoraError (LORA_ERR_STARVATION)."""
    n = len(size)
    sz = (ctypes.c_int32 * max(n, 1))(*[int(v) for v in size])
    rt = (ctypes.c_double * max(n, 1))(*[float(v) for v in rate])
    gpu_of = (ctypes.c_int32 * max(n, 1))()
    a_max_of = (ctypes.c_int32 * max(n_gpus, 1))()
    thr = THROUGHPUT_FN(lambda user, k, s, r, p: float(predict_throughput([s[i] for i in range(k)],
                                                                            [r[i] for i in range(k)], p)))
    stv = STARVATION_FN(lambda user, k, s, r, p: int(bool(predict_starvation([s[i] for i in range(k)],
                                                                              [r[i] for i in range(k)], p))))
    st = _lib.lora_place_adapters(n, sz, rt, int(n_gpus), thr, stv, None, gpu_of, a_max_of)
    if st != LORA_OK:
        raise LoraError(st, "lora_place_adapters")
    return [int(gpu_of[i]) for i in range(n)], [int(a_max_of[g]) for g in range(n_gpus)]


_lib.lora_layer_forward_glu.restype = ctypes.c_int
_lib.lora_layer_forward_glu.argtypes = [_P, ctypes.c_int32, ctypes.c_int32, _P, _P, _P, ctypes.POINTER(lora_segments), _P, _P]
_lib.lora_model_forward_glu.restype = ctypes.c_int
_lib.lora_model_forward_glu.argtypes = [_P, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, _P, _P, _P,
                                        ctypes.POINTER(lora_segments), _P, _P]


def lora_layer_forward_glu(ctx: int, proj_gate: int, proj_up: int, d_x: int, d_W_gate: int, d_W_up: int,
                           seg: lora_segments, d_out: int, stream: int = 0) -> None:
    st = _lib.lora_layer_forward_glu(_P(ctx), int(proj_gate), int(proj_up), _P(d_x), _P(d_W_gate), _P(d_W_up),
                                     ctypes.byref(seg), _P(d_out), _P(stream or None))
    if st != LORA_OK:
        raise LoraError(st, "lora_layer_forward_glu")


def lora_model_forward_glu(ctx: int, layer: int, proj_gate: int, proj_up: int, d_x: int, d_W_gate: int, d_W_up: int,
                           seg: lora_segments, d_out: int, stream: int = 0) -> None:
    st = _lib.lora_model_forward_glu(_P(ctx), int(layer), int(proj_gate), int(proj_up), _P(d_x), _P(d_W_gate),
                                     _P(d_W_up), ctypes.byref(seg), _P(d_out), _P(stream or None))
    if st != LORA_OK:
        raise LoraError(st, "lora_model_forward_glu")


def lora_poll_device_flags(ctx: int, stream: int = 0) -> Tuple[int, int]:
    """Returns (status, raw flag word); status is LORA_OK or LORA_ERR_NOT_RESIDENT."""
    w = ctypes.c_uint32(0)
    st = _lib.lora_poll_device_flags(_P(ctx), ctypes.byref(w), _P(stream or None))
    if st not in (LORA_OK, LORA_ERR_NOT_RESIDENT):
        raise LoraError(st, "lora_poll_device_flags")
    return st, int(w.value)


def lora_slot_of(ctx: int, adapter_id: int) -> int:
    return int(_lib.lora_slot_of(_P(ctx), int(adapter_id)))


def lora_slot_adapter(ctx: int, slot: int) -> int:
    return int(_lib.lora_slot_adapter(_P(ctx), int(slot)))


def lora_slot_first_page(ctx: int, slot: int) -> int:
    return int(_lib.lora_slot_first_page(_P(ctx), int(slot)))


def lora_set_bias(ctx: int, proj: int, d_bias: int, layer: int = 0) -> None:
    """d_bias: device address of bf16 [d_out] (0 removes the bias); the memory stays the caller's."""
    st = _lib.lora_set_bias(_P(ctx), int(layer), int(proj), _P(int(d_bias) or None))
    if st != LORA_OK:
        raise LoraError(st, "lora_set_bias")


def lora_set_tuning(ctx: int, key: int, value: int) -> None:
    st = _lib.lora_set_tuning(_P(ctx), int(key), int(value))
    if st != LORA_OK:
        raise LoraError(st, "lora_set_tuning")


def lora_last_launches(ctx: int) -> List[str]:
    buf = (ctypes.c_char_p * 16)()
    n = _lib.lora_last_launches(_P(ctx), buf, 16)
    return [buf[i].decode() for i in range(min(n, 16))]


def lora_profile_enable(ctx: int, on: bool) -> None:
    st = _lib.lora_profile_enable(_P(ctx), 1 if on else 0)
    if st != LORA_OK:
        raise LoraError(st, "lora_profile_enable")


def lora_profile_collect(ctx: int) -> Dict[str, Tuple[float, int]]:
    """kernel name -> (total milliseconds, launches) since the last reset."""
    cap = 32
    names = (ctypes.c_char_p * cap)()
    ms = (ctypes.c_double * cap)()
    cnt = (ctypes.c_int64 * cap)()
    n = _lib.lora_profile_collect(_P(ctx), names, ms, cnt, cap)
    return {names[i].decode(): (float(ms[i]), int(cnt[i])) for i in range(min(n, cap))}


def lora_calibrate_stream(d_src: int, nbytes: int, workgroups: int, d_sink: int, stream: int = 0) -> None:
    st = _lib.lora_calibrate_stream(_P(d_src), int(nbytes), int(workgroups), _P(d_sink), _P(stream or None))
    if st != LORA_OK:
        raise LoraError(st, "lora_calibrate_stream")


def lora_calibrate_mfma(workgroups: int, iters: int, d_sink: int, d_ticks: int, stream: int = 0) -> None:
    st = _lib.lora_calibrate_mfma(int(workgroups), int(iters), _P(d_sink), _P(d_ticks), _P(stream or None))
    if st != LORA_OK:
        raise LoraError(st, "lora_calibrate_mfma")


def lora_profile_reset(ctx: int) -> None:
    _lib.lora_profile_reset(_P(ctx))
