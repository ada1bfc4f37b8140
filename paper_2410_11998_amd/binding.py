"""ctypes binding of libdadam.so - argument marshalling only.

Every function below has the name and the arguments of the C entry point it wraps (see
include/dadam.h); nothing of the method is computed in Python.  Device memory comes from
PyTorch tensors (their ``data_ptr()``), streams from ``torch.cuda.current_stream()``.

The library must have been built (``python -m paper_2410_11998_amd.build`` or
``__graft_entry__.build()``); importing this module without it raises, there is no
fallback path.
"""

from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libdadam.so")

DADAM_ABI_VERSION = 2
DADAM_MAX_ROWS = 160
DADAM_MAX_SLOTS = 16
DADAM_STATIC_SCRATCH_BYTES = 8192
DADAM_DEVICE_NONE = -1
DADAM_F32, DADAM_BF16 = 0, 1
DADAM_OK, DADAM_EINVAL, DADAM_EALIGN, DADAM_ETOPO, DADAM_EALIAS, DADAM_ESTATE, DADAM_EHIP = 0, -1, -2, -3, -4, -5, -6
DADAM_FUSE_ACCUM, DADAM_FORCE_DIRECT, DADAM_FORCE_TILE = 1, 2, 4
DADAM_WARN_NOT_COLUMN_STOCHASTIC = 1
DADAM_PLACE_TWO_REGIONS, DADAM_PLACE_ARENA_ELSEWHERE, DADAM_PLACE_TOO_LARGE = 1, 2, 4

EXPORTS = [
    "dadam_init", "dadam_set_topology", "dadam_bind", "dadam_swap_x", "dadam_gossip_step",
    "dadam_gossip_step_range", "dadam_accumulate", "dadam_mix", "dadam_mix_consensus", "dadam_mix_consensus_static", "dadam_set_lr", "dadam_get_plan_info",
    "dadam_slot_uses_tile_mode", "dadam_get_row_order", "dadam_pack_offsets", "dadam_spread_offsets", "dadam_place_offsets", "dadam_deal_offsets", "dadam_find_stretches", "dadam_regions_from_stretches",
    "dadam_place_by_timing",
    "dadam_last_error",
    "dadam_destroy",
]


class dadam_tensor_desc(C.Structure):
    _fields_ = [("offset_elems", C.c_uint64), ("numel", C.c_uint64), ("weight_decay", C.c_float), ("flags", C.c_uint32)]


class dadam_config(C.Structure):
    _fields_ = [
        ("abi_version", C.c_uint32), ("n_rows", C.c_uint32), ("n_cols", C.c_uint32), ("d", C.c_uint64),
        ("n_tensors", C.c_uint32), ("tensors", C.POINTER(dadam_tensor_desc)),
        ("param_dtype", C.c_uint32), ("grad_dtype", C.c_uint32),
        ("lr", C.c_float), ("beta1", C.c_float), ("beta2", C.c_float), ("eps", C.c_float),
        ("accum_s", C.c_uint32), ("beta_vhat", C.c_float), ("device", C.c_int32),
        ("lds_limit_bytes", C.c_uint32), ("n_xcds", C.c_uint32),
    ]


class dadam_buffers(C.Structure):
    _fields_ = [("x_src", C.POINTER(C.c_void_p)), ("x_dst", C.POINTER(C.c_void_p)), ("m_hat", C.POINTER(C.c_void_p)),
                ("v_hat", C.POINTER(C.c_void_p)), ("acc", C.POINTER(C.c_void_p))]


class dadam_plan_info(C.Structure):
    _fields_ = [("n_segments", C.c_uint32), ("tile_elems", C.c_uint32), ("direct_elems", C.c_uint32),
                ("n_tiles_tile", C.c_uint64), ("n_tiles_direct", C.c_uint64), ("lds_bytes_tile", C.c_uint32),
                ("tile_mode_possible", C.c_uint32), ("lds_limit_bytes", C.c_uint32), ("n_xcds", C.c_uint32),
                ("mix_tile_elems", C.c_uint32), ("lds_bytes_mix", C.c_uint32), ("n_tiles_mix", C.c_uint64),
                ("tile_waves", C.c_uint32), ("tile_vectors", C.c_uint32), ("mix_waves", C.c_uint32),
                ("mix_vectors", C.c_uint32), ("streaming", C.c_uint32)]


PROBE_CHUNK_BYTES, PROBE_STEP_BYTES, MAX_STRETCHES = 1 << 30, 4 << 30, 6
DADAM_POLICY_TIMED_REGIONS, DADAM_POLICY_RULE_REGIONS, DADAM_POLICY_EQUAL_DISTANCES = 1, 2, 3
DADAM_NOTE_NO_PROBE, DADAM_NOTE_NO_PICTURE, DADAM_NOTE_NO_ROOM, DADAM_NOTE_NOT_CONFIRMED = 1, 2, 3, 4
PAIR_RATE_FN = C.CFUNCTYPE(C.c_double, C.c_uint64, C.c_uint64, C.c_void_p)


class dadam_stretch(C.Structure):
    _fields_ = [("third", C.c_uint32), ("reserved", C.c_uint32), ("lo", C.c_uint64), ("hi", C.c_uint64)]


class dadam_placement(C.Structure):
    _fields_ = [("policy", C.c_uint32), ("advice", C.c_uint32), ("every", C.c_uint32), ("note", C.c_uint32),
                ("n_stretches", C.c_uint32), ("probe_launches", C.c_uint32), ("stretches", dadam_stretch * MAX_STRETCHES),
                ("regions", C.c_uint64 * 4), ("rate_across", C.c_float), ("rate_inside", C.c_float * 2), ("reserved", C.c_uint32)]


def _load() -> C.CDLL:
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: build it first (python -m paper_2410_11998_amd.build); "
                          "there is no fallback implementation")
    lib = C.CDLL(LIB_PATH)
    H = C.c_void_p
    lib.dadam_init.argtypes = [C.POINTER(dadam_config), C.POINTER(H)]
    lib.dadam_set_topology.argtypes = [H, C.c_uint32, C.POINTER(C.c_int32), C.POINTER(C.c_int32), C.POINTER(C.c_float), C.POINTER(C.c_uint32)]
    lib.dadam_bind.argtypes = [H, C.POINTER(dadam_buffers)]
    lib.dadam_swap_x.argtypes = [H]
    lib.dadam_gossip_step.argtypes = [H, C.c_uint32, C.POINTER(C.c_void_p), C.c_uint64, C.c_uint32, C.c_void_p]
    lib.dadam_gossip_step_range.argtypes = [H, C.c_uint32, C.POINTER(C.c_void_p), C.c_uint64, C.c_uint32, C.c_uint32, C.c_uint32, C.c_void_p]
    lib.dadam_accumulate.argtypes = [H, C.POINTER(C.c_void_p), C.c_uint64, C.c_void_p]
    lib.dadam_mix.argtypes = [H, C.c_uint32, C.c_uint32, C.c_void_p]
    lib.dadam_mix_consensus.argtypes = [H, C.c_uint32, C.c_uint32, C.c_void_p, C.c_void_p]
    lib.dadam_mix_consensus_static.argtypes = [H, C.c_uint32, C.c_uint32, C.c_void_p, C.c_void_p]
    lib.dadam_set_lr.argtypes = [H, C.c_float]
    lib.dadam_get_plan_info.argtypes = [H, C.POINTER(dadam_plan_info)]
    lib.dadam_slot_uses_tile_mode.argtypes = [H, C.c_uint32]
    lib.dadam_pack_offsets.argtypes = [C.POINTER(C.c_uint64), C.c_uint32, C.c_uint32, C.POINTER(C.c_uint64), C.POINTER(C.c_uint64)]
    lib.dadam_spread_offsets.argtypes = [C.POINTER(C.c_uint64), C.c_uint32, C.c_uint64, C.POINTER(C.c_uint64)]
    lib.dadam_place_offsets.argtypes = [C.POINTER(C.c_uint64), C.c_uint32, C.c_uint64, C.c_uint64,
                                        C.POINTER(C.c_uint64), C.POINTER(C.c_uint64), C.POINTER(C.c_uint32)]
    lib.dadam_find_stretches.argtypes = [C.c_uint64, PAIR_RATE_FN, C.c_void_p, C.POINTER(dadam_stretch), C.POINTER(C.c_uint32)]
    lib.dadam_regions_from_stretches.argtypes = [C.POINTER(dadam_stretch), C.c_uint32, C.POINTER(C.c_uint64), C.c_uint32,
                                                 C.POINTER(C.c_uint64), C.POINTER(C.c_uint32)]
    lib.dadam_place_by_timing.argtypes = [C.c_void_p, C.c_uint64, C.c_int32, C.POINTER(C.c_uint64), C.c_uint32, C.c_uint64,
                                          C.POINTER(C.c_uint64), C.POINTER(dadam_placement)]
    lib.dadam_get_row_order.argtypes = [H, C.c_uint32, C.POINTER(C.c_int32)]
    lib.dadam_deal_offsets.argtypes = [C.POINTER(C.c_uint64), C.c_uint32, C.c_uint64, C.c_uint64, C.c_uint64, C.c_uint64,
                                       C.c_uint32, C.POINTER(C.c_uint64)]
    lib.dadam_last_error.argtypes = [H]
    lib.dadam_last_error.restype = C.c_char_p
    lib.dadam_destroy.argtypes = [H]
    lib.dadam_destroy.restype = None
    for name in EXPORTS:
        if name not in ("dadam_last_error", "dadam_destroy"):
            getattr(lib, name).restype = C.c_int
    return lib


lib = _load()


class DadamError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"dadam error {code}: {msg}")
        self.code = code


def _ptr_array(ptrs: Sequence[int]):
    arr = (C.c_void_p * len(ptrs))(*[C.c_void_p(int(p)) for p in ptrs])
    return arr


_SHAPE_OF_HANDLE = {}   # handle value -> (d, bytes per parameter, bytes per gradient): host-side size checks only


def _ptrs_of(tensors, h=None, elem_bytes: int = 0, what: str = "") -> Sequence[int]:
    """Device addresses of tensors (or integers taken as addresses).  When tensors are given, their
    size is checked against the handle's d before the address is handed to the library: a buffer
    shorter than d would be overrun by the kernels, which no later check can catch."""
    out = []
    info = _SHAPE_OF_HANDLE.get(getattr(h, "value", None)) if h is not None else None
    for k, t in enumerate(tensors):
        if isinstance(t, int):
            out.append(t)
            continue
        if info is not None and elem_bytes:
            if not t.is_contiguous():
                raise ValueError(f"{what}[{k}] is not contiguous")
            if t.element_size() != elem_bytes:
                raise ValueError(f"{what}[{k}] has {t.element_size()}-byte elements, the handle expects {elem_bytes}")
            if t.numel() < info[0]:
                raise ValueError(f"{what}[{k}] holds {t.numel()} elements, the handle needs {info[0]}")
        out.append(t.data_ptr())
    return out


def _check(h, rc: int) -> int:
    if rc < 0:
        raise DadamError(rc, (lib.dadam_last_error(h) or b"").decode())
    return rc


def dadam_last_error(h) -> str:
    return (lib.dadam_last_error(h) or b"").decode()


def dadam_pack_offsets(numel: Sequence[int], align_elems: int):
    n = len(numel)
    a = (C.c_uint64 * n)(*[int(x) for x in numel])
    o = (C.c_uint64 * n)()
    d = C.c_uint64(0)
    rc = lib.dadam_pack_offsets(a, n, align_elems, o, C.byref(d))
    if rc < 0:
        raise DadamError(rc, "dadam_pack_offsets")
    return np.asarray(list(o), dtype=np.uint64), int(d.value)


def dadam_spread_offsets(nbytes: Sequence[int], arena_bytes: int):
    n = len(nbytes)
    a = (C.c_uint64 * n)(*[int(x) for x in nbytes])
    o = (C.c_uint64 * n)()
    rc = lib.dadam_spread_offsets(a, n, int(arena_bytes), o)
    if rc < 0:
        raise DadamError(rc, f"dadam_spread_offsets: {n} buffers of {sum(int(x) for x in nbytes)} bytes do not fit in {arena_bytes}")
    return [int(x) for x in o]


def dadam_place_offsets(nbytes: Sequence[int], arena_bytes: int, device_total_bytes: int):
    """Returns (offsets, regions, advice) with regions = [(lo0, hi0), (lo1, hi1)], or [(0, arena_bytes)] for the
    fall-back, and advice the DADAM_PLACE_* flag the library reports."""
    n = len(nbytes)
    a = (C.c_uint64 * n)(*[int(x) for x in nbytes])
    o = (C.c_uint64 * n)()
    r = (C.c_uint64 * 4)()
    adv = C.c_uint32(0)
    rc = lib.dadam_place_offsets(a, n, int(arena_bytes), int(device_total_bytes), o, r, C.byref(adv))
    if rc < 0:
        raise DadamError(rc, f"dadam_place_offsets: {n} buffers of {sum(int(x) for x in nbytes)} bytes do not fit in {arena_bytes}")
    regions = [(int(r[0]), int(r[1]))] + ([(int(r[2]), int(r[3]))] if r[3] else [])
    return [int(x) for x in o], regions, int(adv.value)


def dadam_find_stretches(arena_bytes: int, rate):
    """Stretches [(third id, lo, hi)] of an arena from pair timings; rate(off_a, off_b) -> fraction of peak."""
    out = (dadam_stretch * MAX_STRETCHES)()
    n = C.c_uint32(0)
    cb = PAIR_RATE_FN(lambda a, b, _ctx: float(rate(int(a), int(b))))
    rc = lib.dadam_find_stretches(int(arena_bytes), cb, None, out, C.byref(n))
    if rc < 0:
        raise DadamError(rc, "dadam_find_stretches failed")
    return [(int(out[k].third), int(out[k].lo), int(out[k].hi)) for k in range(n.value)]


def dadam_regions_from_stretches(stretches, nbytes: Sequence[int]):
    """((lo0, hi0), (lo1, hi1), every) for dadam_deal_offsets, or None."""
    st = (dadam_stretch * max(1, len(stretches)))()
    for k, (t, lo, hi) in enumerate(stretches):
        st[k].third, st[k].lo, st[k].hi = int(t), int(lo), int(hi)
    a = (C.c_uint64 * len(nbytes))(*[int(x) for x in nbytes])
    reg, every = (C.c_uint64 * 4)(), C.c_uint32(0)
    rc = lib.dadam_regions_from_stretches(st, len(stretches), a, len(nbytes), reg, C.byref(every))
    if rc < 0:
        raise DadamError(rc, "dadam_regions_from_stretches failed")
    return ((int(reg[0]), int(reg[1])), (int(reg[2]), int(reg[3])), int(every.value)) if rc == 1 else None


def dadam_place_by_timing(arena_ptr: int, arena_bytes: int, device: int, nbytes: Sequence[int], device_total_bytes: int):
    """(offsets, report): the buffers placed in a device arena by the library's timing probe (see include/dadam.h)."""
    n = len(nbytes)
    a = (C.c_uint64 * n)(*[int(x) for x in nbytes])
    o = (C.c_uint64 * n)()
    rep = dadam_placement()
    rc = lib.dadam_place_by_timing(C.c_void_p(int(arena_ptr)), int(arena_bytes), int(device), a, n, int(device_total_bytes), o, C.byref(rep))
    if rc < 0:
        raise DadamError(rc, f"dadam_place_by_timing failed for {n} buffers in an arena of {arena_bytes} bytes")
    return [int(x) for x in o], rep


def dadam_get_row_order(h, slot: int, n_rows: int):
    """(order, in_use): the order in which direct mode takes the n_rows rows of a slot."""
    out = (C.c_int32 * int(n_rows))()
    rc = lib.dadam_get_row_order(h, slot, out)
    if rc < 0:
        _check(h, rc)
    return [int(x) for x in out], bool(rc)


def dadam_deal_offsets(nbytes: Sequence[int], region0, region1, every: int = 2):
    """Offsets of the buffers dealt over the regions (lo, hi) of one arena: every `every`-th one in region1."""
    n = len(nbytes)
    a = (C.c_uint64 * n)(*[int(x) for x in nbytes])
    o = (C.c_uint64 * n)()
    rc = lib.dadam_deal_offsets(a, n, int(region0[0]), int(region0[1]), int(region1[0]), int(region1[1]), int(every), o)
    if rc < 0:
        raise DadamError(rc, f"dadam_deal_offsets: {n} buffers do not fit the regions {region0}, {region1} (or bad bounds)")
    return [int(x) for x in o]


def dadam_init(n_rows: int, n_cols: int, d: int, offsets: Sequence[int], numels: Sequence[int],
               param_dtype: int = DADAM_F32, grad_dtype: int = DADAM_F32, lr: float = 1e-3, beta1: float = 0.9,
               beta2: float = 0.999, eps: float = 1e-8, accum_s: int = 1, beta_vhat: float = -1.0,
               device: int = 0, abi_version: int = DADAM_ABI_VERSION, weight_decay=None, tensor_flags=None,
               lds_limit_bytes: int = 0, n_xcds: int = 0):
    n = len(offsets)
    descs = (dadam_tensor_desc * max(n, 1))()
    for k in range(n):
        descs[k].offset_elems = int(offsets[k])
        descs[k].numel = int(numels[k])
        descs[k].weight_decay = float(weight_decay[k]) if weight_decay is not None else 0.0
        descs[k].flags = int(tensor_flags[k]) if tensor_flags is not None else 0
    cfg = dadam_config(abi_version, n_rows, n_cols, d, n, descs, param_dtype, grad_dtype, lr, beta1, beta2, eps,
                       accum_s, beta_vhat, device, lds_limit_bytes, n_xcds)
    h = C.c_void_p()
    rc = lib.dadam_init(C.byref(cfg), C.byref(h))
    if rc < 0:
        raise DadamError(rc, (lib.dadam_last_error(None) or b"").decode())
    _SHAPE_OF_HANDLE[h.value] = (int(d), 2 if param_dtype == DADAM_BF16 else 4, 2 if grad_dtype == DADAM_BF16 else 4)
    return h


def dadam_set_topology(h, slot: int, row_ptr, col_idx, w) -> int:
    rp = np.ascontiguousarray(row_ptr, dtype=np.int32)
    ci = np.ascontiguousarray(col_idx, dtype=np.int32)
    ww = np.ascontiguousarray(w, dtype=np.float32)
    warn = C.c_uint32(0)
    _check(h, lib.dadam_set_topology(h, slot, rp.ctypes.data_as(C.POINTER(C.c_int32)), ci.ctypes.data_as(C.POINTER(C.c_int32)),
                                     ww.ctypes.data_as(C.POINTER(C.c_float)), C.byref(warn)))
    return int(warn.value)


def dadam_bind(h, x_src, x_dst, m_hat, v_hat, acc=None) -> None:
    px = _SHAPE_OF_HANDLE.get(h.value, (0, 0, 0))[1]
    keep = [_ptr_array(_ptrs_of(x_src, h, px, "x_src")), _ptr_array(_ptrs_of(x_dst, h, px, "x_dst")),
            _ptr_array(_ptrs_of(m_hat, h, 4, "m_hat")), _ptr_array(_ptrs_of(v_hat, h, 4, "v_hat")),
            _ptr_array(_ptrs_of(acc, h, 4, "acc")) if acc is not None else None]
    b = dadam_buffers(keep[0], keep[1], keep[2], keep[3], keep[4] if keep[4] is not None else C.POINTER(C.c_void_p)())
    _check(h, lib.dadam_bind(h, C.byref(b)))


def dadam_swap_x(h) -> None:
    _check(h, lib.dadam_swap_x(h))


def _grad_ptrs(h, grads):
    if isinstance(grads, C.Array):          # a table made by grad_table(): already marshalled and checked
        return grads
    return _ptr_array(_ptrs_of(grads, h, _SHAPE_OF_HANDLE.get(h.value, (0, 0, 0))[2], "grads"))


def grad_table(h, grads):
    """The host array of device pointers that the step calls take, marshalled (and size-checked) once; callers
    that reuse a gradient set pass this instead of the list of tensors.  The tensors must stay alive."""
    return _grad_ptrs(h, grads)


def dadam_gossip_step(h, slot: int, grads, t: int, flags: int = DADAM_FUSE_ACCUM, stream: int = 0) -> None:
    _check(h, lib.dadam_gossip_step(h, slot, _grad_ptrs(h, grads), t, flags, C.c_void_p(stream)))


def dadam_gossip_step_range(h, slot: int, grads, t: int, flags: int, tensor_begin: int, tensor_end: int, stream: int = 0) -> None:
    _check(h, lib.dadam_gossip_step_range(h, slot, _grad_ptrs(h, grads), t, flags, tensor_begin, tensor_end, C.c_void_p(stream)))


def dadam_accumulate(h, grads, t: int, stream: int = 0) -> None:
    _check(h, lib.dadam_accumulate(h, _grad_ptrs(h, grads), t, C.c_void_p(stream)))


def dadam_mix(h, slot: int, flags: int = 0, stream: int = 0) -> None:
    _check(h, lib.dadam_mix(h, slot, flags, C.c_void_p(stream)))


def dadam_mix_consensus(h, slot: int, out, flags: int = 0, stream: int = 0) -> None:
    """out: a device tensor holding one float64 (or an integer device address)."""
    if not isinstance(out, int):
        if out.numel() < 1 or out.element_size() != 8:
            raise ValueError("consensus output must hold one float64")
        out = out.data_ptr()
    _check(h, lib.dadam_mix_consensus(h, slot, flags, C.c_void_p(out), C.c_void_p(stream)))


def dadam_mix_consensus_static(h, slot: int, out, flags: int = 0, stream: int = 0) -> None:
    """out: a device tensor holding one float64 (or an integer device address)."""
    if not isinstance(out, int):
        if out.numel() < 1 or out.element_size() != 8:
            raise ValueError("consensus output must hold one float64")
        out = out.data_ptr()
    _check(h, lib.dadam_mix_consensus_static(h, slot, flags, C.c_void_p(out), C.c_void_p(stream)))


def dadam_set_lr(h, lr: float) -> None:
    _check(h, lib.dadam_set_lr(h, lr))


def dadam_get_plan_info(h) -> dadam_plan_info:
    info = dadam_plan_info()
    _check(h, lib.dadam_get_plan_info(h, C.byref(info)))
    return info


def dadam_slot_uses_tile_mode(h, slot: int) -> bool:
    return _check(h, lib.dadam_slot_uses_tile_mode(h, slot)) == 1


def dadam_destroy(h) -> None:
    _SHAPE_OF_HANDLE.pop(getattr(h, "value", None), None)
    lib.dadam_destroy(h)


def current_stream() -> int:
    """The HIP stream PyTorch is launching on, as an integer handle."""
    import torch
    return int(torch.cuda.current_stream().cuda_stream)
