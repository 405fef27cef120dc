"""Thin binding over the host-side dispatching ABI of libsp_mi355x.so (include/sp_dispatch.h): the length-aware
buffer, the student-number controller and the dispatcher loop in virtual time.

Argument marshalling only; the data structures and the loop are the library's C++.  Apart from serve_replay no call
here touches the GPU (they produce the packed batch and k_active that sp_forward consumes).
"""
from __future__ import annotations

import ctypes as C
from dataclasses import dataclass

import numpy as np

SP_EFULL, SP_EEMPTY = -6, -7


class sp_sim_config(C.Structure):
    _fields_ = [("total_students", C.c_int32), ("slots", C.c_int32), ("k_min", C.c_int32), ("k_start", C.c_int32),
                ("window_us", C.c_int64), ("bin_width", C.c_int32), ("max_len", C.c_int32), ("max_elem", C.c_int32),
                ("capacity", C.c_int32), ("padded", C.c_int32), ("base_us", C.c_void_p), ("per_token_ns", C.c_void_p)]


def _load() -> C.CDLL:
    # The library is taken from the sp module, which imports torch before loading it: the process must end up with one
    # HIP runtime (torch's), also when this module is imported first and only the host-side calls are used.
    from . import sp as _sp
    lib = _sp.raw_lib()
    vp, i32, i64 = C.c_void_p, C.c_int32, C.c_int64
    pi32 = C.POINTER(C.c_int32)
    lib.sp_lab_create.restype = C.c_int; lib.sp_lab_create.argtypes = [i32, i32, i32, i32, C.POINTER(vp)]
    lib.sp_lab_free.restype = None; lib.sp_lab_free.argtypes = [vp]
    lib.sp_lab_bin_of.restype = C.c_int; lib.sp_lab_bin_of.argtypes = [vp, i32]
    lib.sp_lab_bin_len.restype = C.c_int; lib.sp_lab_bin_len.argtypes = [vp, i32]
    lib.sp_lab_push.restype = C.c_int; lib.sp_lab_push.argtypes = [vp, i64, i32, pi32]
    lib.sp_lab_pop.restype = C.c_int; lib.sp_lab_pop.argtypes = [vp, pi32, pi32, vp, vp, pi32]
    lib.sp_lab_elements.restype = C.c_int; lib.sp_lab_elements.argtypes = [vp]
    lib.sp_lab_samples.restype = C.c_int; lib.sp_lab_samples.argtypes = [vp]
    lib.sp_ctl_create.restype = C.c_int; lib.sp_ctl_create.argtypes = [i32, i32, i32, i64, i32, C.POINTER(vp)]
    lib.sp_ctl_free.restype = None; lib.sp_ctl_free.argtypes = [vp]
    lib.sp_ctl_k.restype = C.c_int; lib.sp_ctl_k.argtypes = [vp]
    lib.sp_ctl_groups.restype = C.c_int; lib.sp_ctl_groups.argtypes = [vp]
    lib.sp_ctl_on_buffered.restype = C.c_int; lib.sp_ctl_on_buffered.argtypes = [vp, i32]
    lib.sp_ctl_on_tick.restype = C.c_int; lib.sp_ctl_on_tick.argtypes = [vp, i64, i32, i32]
    lib.sp_dispatch_simulate.restype = C.c_int
    lib.sp_dispatch_simulate.argtypes = [C.POINTER(sp_sim_config), vp, vp, i64, vp, vp, vp, vp, vp, vp, C.POINTER(i64),
                                         vp, vp, i64, C.POINTER(i64), C.POINTER(i64)]
    lib.sp_strerror.restype = C.c_char_p; lib.sp_strerror.argtypes = [C.c_int]
    return lib


_lib = _load()


class DispatchError(RuntimeError):
    def __init__(self, code: int):
        self.code = code
        super().__init__(f"sp error {code}: {_lib.sp_strerror(code).decode()}")


def _check(rc: int) -> int:
    if rc < 0:
        raise DispatchError(rc)
    return rc


class LengthAwareBuffer:
    """sp_lab_* of the library."""

    def __init__(self, bin_width=8, max_len=128, max_elem=4, capacity=64):
        self._h = C.c_void_p()
        _check(_lib.sp_lab_create(bin_width, max_len, max_elem, capacity, C.byref(self._h)))
        self.max_elem = max_elem
        self._ids = np.zeros(max_elem, np.int64)
        self._lens = np.zeros(max_elem, np.int32)

    def __del__(self):
        if getattr(self, "_h", None):
            _lib.sp_lab_free(self._h)
            self._h = None

    def bin_of(self, length: int) -> int:
        return _check(_lib.sp_lab_bin_of(self._h, length))

    def bin_len(self, b: int) -> int:
        return _check(_lib.sp_lab_bin_len(self._h, b))

    def push(self, sample_id: int, length: int) -> bool:
        joined = C.c_int32()
        _check(_lib.sp_lab_push(self._h, sample_id, length, C.byref(joined)))
        return bool(joined.value)

    def pop(self):
        b, bl, n = C.c_int32(), C.c_int32(), C.c_int32()
        _check(_lib.sp_lab_pop(self._h, C.byref(b), C.byref(bl), self._ids.ctypes.data, self._lens.ctypes.data, C.byref(n)))
        return b.value, bl.value, self._ids[:n.value].tolist(), self._lens[:n.value].tolist()

    def __len__(self) -> int:
        return _check(_lib.sp_lab_elements(self._h))

    def samples(self) -> int:
        return _check(_lib.sp_lab_samples(self._h))


class StudentNumberController:
    """sp_ctl_* of the library."""

    def __init__(self, total_students, slots, k_min=1, window_us=120_000_000, k_start=None):
        self._h = C.c_void_p()
        _check(_lib.sp_ctl_create(total_students, slots, k_min, window_us, k_start or 0, C.byref(self._h)))

    def __del__(self):
        if getattr(self, "_h", None):
            _lib.sp_ctl_free(self._h)
            self._h = None

    @property
    def k(self) -> int:
        return _check(_lib.sp_ctl_k(self._h))

    def groups(self) -> int:
        return _check(_lib.sp_ctl_groups(self._h))

    def on_buffered(self, buffer_elements: int) -> bool:
        return bool(_check(_lib.sp_ctl_on_buffered(self._h, buffer_elements)))

    def on_tick(self, now_us: int, buffer_elements: int, busy_groups: int) -> bool:
        return bool(_check(_lib.sp_ctl_on_tick(self._h, now_us, buffer_elements, busy_groups)))


@dataclass
class SimResult:
    dispatch_us: np.ndarray
    done_us: np.ndarray
    k_used: np.ndarray
    element: np.ndarray
    elem_tokens: np.ndarray
    elem_size: np.ndarray
    k_trace: list
    refused: int


def simulate(arrival_us, lengths, *, total_students, slots, k_min, window_us, base_us, per_token_ns, padded,
             bin_width=8, max_len=128, max_elem=4, capacity=64, k_start=None, trace_cap=1 << 16) -> SimResult:
    """sp_dispatch_simulate of the library (same arguments as the oracle's function of this name)."""
    arr = np.ascontiguousarray(arrival_us, np.int64)
    lens = np.ascontiguousarray(lengths, np.int32)
    n = len(arr)
    base = np.ascontiguousarray(base_us, np.int64)
    per = np.ascontiguousarray(per_token_ns, np.int64)
    assert len(lens) == n and len(base) == total_students + 1 == len(per)
    cfg = sp_sim_config(total_students, slots, k_min, k_start or 0, window_us, bin_width, max_len, max_elem, capacity,
                        1 if padded else 0, base.ctypes.data, per.ctypes.data)
    disp, done = np.empty(n, np.int64), np.empty(n, np.int64)
    k_used, element = np.empty(n, np.int32), np.empty(n, np.int64)
    etok, esize = np.empty(max(n, 1), np.int64), np.empty(max(n, 1), np.int32)
    tus, tk = np.empty(trace_cap, np.int64), np.empty(trace_cap, np.int32)
    ne, nt, nref = C.c_int64(), C.c_int64(), C.c_int64()
    _check(_lib.sp_dispatch_simulate(C.byref(cfg), arr.ctypes.data, lens.ctypes.data, n, disp.ctypes.data, done.ctypes.data,
                                     k_used.ctypes.data, element.ctypes.data, etok.ctypes.data, esize.ctypes.data,
                                     C.byref(ne), tus.ctypes.data, tk.ctypes.data, trace_cap, C.byref(nt), C.byref(nref)))
    m = min(nt.value, trace_cap)
    return SimResult(disp, done, k_used, element, etok[:ne.value].copy(), esize[:ne.value].copy(),
                     list(zip(tus[:m].tolist(), tk[:m].tolist())), nref.value)


class sp_serve_config(C.Structure):
    _fields_ = [("slots", C.c_int32), ("k_min", C.c_int32), ("k_start", C.c_int32), ("window_us", C.c_int64),
                ("bin_width", C.c_int32), ("max_len", C.c_int32), ("max_elem", C.c_int32), ("capacity", C.c_int32),
                ("padded", C.c_int32), ("pad_id", C.c_int32)]


_lib.sp_serve_replay.restype = C.c_int
_lib.sp_serve_replay.argtypes = [C.c_void_p, C.POINTER(sp_serve_config)] + [C.c_void_p] * 3 + [C.c_int64] + \
    [C.c_void_p] * 5 + [C.POINTER(C.c_int64), C.c_void_p, C.POINTER(C.c_int64), C.POINTER(C.c_int32)]


@dataclass
class ReplayResult:
    dispatch_us: np.ndarray
    done_us: np.ndarray
    k_used: np.ndarray
    element: np.ndarray
    elem_size: np.ndarray
    logits: np.ndarray
    refused: int
    k_final: int


def serve_replay(model_handle, classes: int, arrival_us, token_ids, id_offsets, *, slots, k_min, window_us, padded=False,
                 pad_id=0, bin_width=8, max_len=128, max_elem=4, capacity=4096, k_start=None) -> ReplayResult:
    """sp_serve_replay of the library: real-time replay on the GPU.  model_handle: the sp_model* of a loaded group
    (Students.handle of the sp module); token_ids int32 host array, sample i owns [id_offsets[i], id_offsets[i+1])."""
    arr = np.ascontiguousarray(arrival_us, np.int64)
    ids = np.ascontiguousarray(token_ids, np.int32)
    off = np.ascontiguousarray(id_offsets, np.int64)
    n = len(arr)
    assert len(off) == n + 1 and off[-1] <= len(ids)
    cfg = sp_serve_config(slots, k_min, k_start or 0, window_us, bin_width, max_len, max_elem, capacity,
                          1 if padded else 0, pad_id)
    disp, done = np.full(n, -1, np.int64), np.full(n, -1, np.int64)
    k_used, element = np.zeros(n, np.int32), np.full(n, -1, np.int64)
    esize = np.zeros(max(n, 1), np.int32)
    logits = np.zeros((n, classes), np.float32)
    ne, nref, kf = C.c_int64(), C.c_int64(), C.c_int32()
    _check(_lib.sp_serve_replay(model_handle, C.byref(cfg), arr.ctypes.data, ids.ctypes.data, off.ctypes.data, n,
                                disp.ctypes.data, done.ctypes.data, k_used.ctypes.data, element.ctypes.data,
                                esize.ctypes.data, C.byref(ne), logits.ctypes.data, C.byref(nref), C.byref(kf)))
    return ReplayResult(disp, done, k_used, element, esize[:ne.value].copy(), logits, nref.value, kf.value)
